// MVUE(dY^T) written out as a packed 2:4 operand (paper Sec. 5.1): the same device sparsifier that the
// weight-gradient GEMM applies while loading its operand, used here to check it bit for bit.
// One lane handles eight consecutive tokens (two groups) of one output channel: it reads eight
// elements down a column of dY (lanes run along the channel axis, so each row access is contiguous
// across the wave) and writes four values and one metadata byte of row o of the packed operand.
#include "common.h"
#include "mvue_device.h"

namespace sste {

template <bool FP8>
__global__ void __launch_bounds__(256)
k_mvue_materialize(const void* __restrict__ dY, int64_t T, int64_t O, int64_t lddy, RngKey key,
                   void* __restrict__ vals, uint8_t* __restrict__ meta) {
  int64_t o = (int64_t)blockIdx.x * 256 + threadIdx.x;
  int64_t kp = blockIdx.y;                       // pair of token groups: tokens 8kp .. 8kp+7
  if (o >= O) return;
  uint32_t nib[2], packed[2];
#pragma unroll
  for (int g = 0; g < 2; g++) {
    int64_t k = 2 * kp + g;
    int64_t t0 = 4 * k;
    uint64_t gid = (uint64_t)k * (uint64_t)O + (uint64_t)o;
    uint32_t x = draw_u32(key.k0, key.k1, (uint32_t)gid, (uint32_t)(gid >> 32));
    if (FP8) {
      const uint8_t* p = (const uint8_t*)dY + t0 * lddy + o;
      uint32_t gw = (uint32_t)p[0] | ((uint32_t)p[lddy] << 8) | ((uint32_t)p[2 * lddy] << 16) | ((uint32_t)p[3 * lddy] << 24);
      packed[g] = mvue_group_e4m3(gw, x, nib[g]);
    } else {
      const uint16_t* p = (const uint16_t*)dY + t0 * lddy + o;
      uint32_t lo = (uint32_t)p[0] | ((uint32_t)p[lddy] << 16);
      uint32_t hi = (uint32_t)p[2 * lddy] | ((uint32_t)p[3 * lddy] << 16);
      packed[g] = mvue_group_bf16(lo, hi, x, nib[g]);
    }
  }
  // blocked layout of include/sste.h: block (rb, s) of 16 channels x one k-step; slot 16 q + j
  constexpr int KS = FP8 ? 128 : 64;             // tokens per k-step
  const int64_t steps = T / KS, t0 = 8 * kp;
  const int64_t blk = (o / 16) * steps + t0 / KS;
  const int to = (int)(t0 % KS), q = to / (KS / 4), pi = (to % (KS / 4)) / 8;
  const int64_t slot = blk * 64 + 16 * q + (o & 15);
  if (FP8) {
    ((uint32_t*)vals)[slot * 4 + pi] = packed[0] | (packed[1] << 16);
    meta[slot * 4 + pi] = (uint8_t)(nib[0] | (nib[1] << 4));
  } else {
    uint2 v;
    v.x = packed[0];
    v.y = packed[1];
    ((uint2*)vals)[slot * 2 + pi] = v;
    meta[slot * 2 + pi] = (uint8_t)(nib[0] | (nib[1] << 4));
  }
}

hipError_t launch_mvue_materialize(const void* dY, int64_t T, int64_t O, int64_t lddy, int dtype, RngKey key,
                                   void* vals, void* meta, hipStream_t s) {
  if (T == 0 || O == 0) return hipSuccess;
  dim3 grid((unsigned)((O + 255) / 256), (unsigned)(T / 8)), block(256);
  if (dtype == SSTE_F8E4M3)
    hipLaunchKernelGGL((k_mvue_materialize<true>), grid, block, 0, s, dY, T, O, lddy, key, vals, (uint8_t*)meta);
  else
    hipLaunchKernelGGL((k_mvue_materialize<false>), grid, block, 0, s, dY, T, O, lddy, key, vals, (uint8_t*)meta);
  return hipGetLastError();
}

}  // namespace sste
