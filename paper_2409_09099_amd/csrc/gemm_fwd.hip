// Forward GEMM of the S-STE linear layer (paper Sec. 5.1): Z = X S(W)^T with S(W) 2:4 sparse.
//
// MFMA mapping: Z^T = S(W) X^T, so the sparse matrix is MFMA operand A (rows = output channels o,
// contraction k = input features, 2:4 along k) and X supplies operand B with k contiguous in memory.
// One sparse MFMA (v_smfmac_f32_16x16x64_bf16 / v_smfmac_f32_16x16x128_fp8_fp8) consumes, per lane,
// 16 bytes of packed values, their position bits, and two 16-byte pieces of an X row:
//   A: lane (row i = lane % 16, qa = lane / 16) holds compressed values [8 qa, 8 qa + 8) of the 32
//      (64 for fp8) that make up the k-step, and their 2-bit positions, 2 bits per value;
//   B: lane (col j = lane % 16, qb = lane / 16) holds dense k in [8 qb, 8 qb + 8) and [32 + 8 qb, 32 + 8 qb + 8)
//      (bf16; for fp8 16-element pieces at 16 qb and 64 + 16 qb): byte offsets 16 qb and 64 + 16 qb.
//   D: lane (j, q) register r holds element (row 4 q + r, col j).
// In bytes a k-step is the same for both types: 64 B of values + 128 B of X per row.
//
// Tiling: 128 (o) x 128 (t) per workgroup of 4 waves (2 x 2, 64 x 64 each = 4 x 4 MFMA tiles),
// operands staged through LDS with register prefetch of the next k-step.  LDS rows are padded
// (80 B for values, 144 B for X) so that the 16-byte fragment reads of 8 consecutive rows fall in
// distinct banks.
#include "common.h"

namespace sste {

namespace {
constexpr int BM = 128, BN = 128;
constexpr int A_STRIDE = 80;    // 64 B of packed values + 16 B pad
constexpr int B_STRIDE = 144;   // 128 B of X + 16 B pad
constexpr int M_STRIDE = 16;    // metadata bytes per row and k-step: 8 (bf16) or 16 (fp8)
}  // namespace

template <bool FP8>
__global__ void __launch_bounds__(256)
k_linear_fwd(const uint8_t* __restrict__ X, int64_t T, int64_t k_bytes, int64_t ldx_bytes,
             const uint8_t* __restrict__ vals, const uint8_t* __restrict__ meta, int64_t meta_row_bytes,
             int64_t O, float scale, uint16_t* __restrict__ Z, int64_t ldz) {
  __shared__ __align__(16) uint8_t sA[BM * A_STRIDE];
  __shared__ __align__(16) uint8_t sM[BM * M_STRIDE];
  __shared__ __align__(16) uint8_t sB[BN * B_STRIDE];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int j = lane & 15, q = lane >> 4;
  const int64_t o0 = (int64_t)blockIdx.x * BM, t0 = (int64_t)blockIdx.y * BN;
  const int nsteps = (int)(k_bytes / 128);
  const int64_t vals_row_bytes = k_bytes / 2;
  constexpr int MB = FP8 ? 16 : 8;

  f32x4 acc[4][4];
#pragma unroll
  for (int a = 0; a < 4; a++)
#pragma unroll
    for (int b = 0; b < 4; b++) acc[a][b] = (f32x4){0.f, 0.f, 0.f, 0.f};

  uint4 ra[2], rb[4], rm;

  // Rows past the end of the matrix are read from the last valid row (always mapped memory) and then
  // zeroed, so the loads need no branch.
  const uint8_t* pa[2];
  bool oka[2];
#pragma unroll
  for (int r = 0; r < 2; r++) {
    int c = tid + 256 * r, row = c >> 2, part = c & 3;
    oka[r] = (o0 + row) < O;
    int64_t rr = oka[r] ? (o0 + row) : (O - 1);
    pa[r] = vals + rr * vals_row_bytes + part * 16;
  }
  const bool okm = (tid < BM) && (o0 + tid < O);
  const uint8_t* pm = meta + (okm ? (o0 + tid) : (O - 1)) * meta_row_bytes;
  const uint8_t* pb[4];
  bool okb[4];
#pragma unroll
  for (int r = 0; r < 4; r++) {
    int c = tid + 256 * r, row = c >> 3, part = c & 7;
    okb[r] = (t0 + row) < T;
    int64_t rr = okb[r] ? (t0 + row) : (T - 1);
    pb[r] = X + rr * ldx_bytes + part * 16;
  }

#define FWD_LOAD_GLOBAL(step)                                                        \
  do {                                                                               \
    _Pragma("unroll") for (int r = 0; r < 2; r++) {                                  \
      uint4 v = *(const uint4*)(pa[r] + (int64_t)(step) * 64);                       \
      ra[r] = oka[r] ? v : make_uint4(0, 0, 0, 0);                                   \
    }                                                                                \
    if (FP8) {                                                                       \
      uint4 v = *(const uint4*)(pm + (int64_t)(step) * 16);                          \
      rm = okm ? v : make_uint4(0, 0, 0, 0);                                         \
    } else {                                                                         \
      uint2 v = *(const uint2*)(pm + (int64_t)(step) * 8);                           \
      rm = okm ? make_uint4(v.x, v.y, 0, 0) : make_uint4(0, 0, 0, 0);                \
    }                                                                                \
    _Pragma("unroll") for (int r = 0; r < 4; r++) {                                  \
      uint4 v = *(const uint4*)(pb[r] + (int64_t)(step) * 128);                      \
      rb[r] = okb[r] ? v : make_uint4(0, 0, 0, 0);                                   \
    }                                                                                \
  } while (0)

#define FWD_STORE_LDS()                                                              \
  do {                                                                               \
    _Pragma("unroll") for (int r = 0; r < 2; r++) {                                  \
      int c = tid + 256 * r, row = c >> 2, part = c & 3;                             \
      *(uint4*)(sA + row * A_STRIDE + part * 16) = ra[r];                            \
    }                                                                                \
    if (tid < BM) *(uint4*)(sM + tid * M_STRIDE) = rm;                               \
    _Pragma("unroll") for (int r = 0; r < 4; r++) {                                  \
      int c = tid + 256 * r, row = c >> 3, part = c & 7;                             \
      *(uint4*)(sB + row * B_STRIDE + part * 16) = rb[r];                            \
    }                                                                                \
  } while (0)

  if (nsteps > 0) FWD_LOAD_GLOBAL(0);
  for (int step = 0; step < nsteps; step++) {
    FWD_STORE_LDS();
    __syncthreads();
    if (step + 1 < nsteps) FWD_LOAD_GLOBAL(step + 1);

    uint4 fa[4];
    int fidx[4];
    uint4 fb[4][2];
#pragma unroll
    for (int mi = 0; mi < 4; mi++) {
      int row = 64 * wm + 16 * mi + j;
      fa[mi] = *(const uint4*)(sA + row * A_STRIDE + 16 * q);
      if (FP8) fidx[mi] = *(const int*)(sM + row * M_STRIDE + 4 * q);
      else fidx[mi] = *(const uint16_t*)(sM + row * M_STRIDE + 2 * q);
    }
#pragma unroll
    for (int ni = 0; ni < 4; ni++) {
      int row = 64 * wn + 16 * ni + j;
      fb[ni][0] = *(const uint4*)(sB + row * B_STRIDE + 16 * q);
      fb[ni][1] = *(const uint4*)(sB + row * B_STRIDE + 64 + 16 * q);
    }
#pragma unroll
    for (int mi = 0; mi < 4; mi++)
#pragma unroll
      for (int ni = 0; ni < 4; ni++) {
        if (FP8) {
          i32x4 av;
          i32x8 bv;
          __builtin_memcpy(&av, &fa[mi], 16);
          __builtin_memcpy(&bv, &fb[ni][0], 32);
          acc[mi][ni] = __builtin_amdgcn_smfmac_f32_16x16x128_fp8_fp8(av, bv, acc[mi][ni], fidx[mi], 0, 0);
        } else {
          bf16x8 av;
          bf16x16 bv;
          __builtin_memcpy(&av, &fa[mi], 16);
          __builtin_memcpy(&bv, &fb[ni][0], 32);
          acc[mi][ni] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(av, bv, acc[mi][ni], fidx[mi], 0, 0);
        }
      }
    __syncthreads();
  }

#undef FWD_LOAD_GLOBAL
#undef FWD_STORE_LDS

  // epilogue: lane (j, q) register r of tile (mi, ni) is Z[t][o + r], four consecutive channels
#pragma unroll
  for (int mi = 0; mi < 4; mi++)
#pragma unroll
    for (int ni = 0; ni < 4; ni++) {
      int64_t o = o0 + 64 * wm + 16 * mi + 4 * q;
      int64_t t = t0 + 64 * wn + 16 * ni + j;
      if (t < T && o < O) {
        uint2 v;
        v.x = bf16_rne_pack(acc[mi][ni][0] * scale, acc[mi][ni][1] * scale);
        v.y = bf16_rne_pack(acc[mi][ni][2] * scale, acc[mi][ni][3] * scale);
        *(uint2*)(Z + t * ldz + o) = v;
      }
    }
}

hipError_t launch_linear_fwd(const void* X, int64_t T, int64_t I, int64_t ldx, int dtype, float scale,
                             const void* vals, const void* meta, int64_t O, void* Z, int64_t ldz, hipStream_t s) {
  if (T == 0 || O == 0) return hipSuccess;
  dim3 grid((unsigned)((O + BM - 1) / BM), (unsigned)((T + BN - 1) / BN)), block(256);
  if (dtype == SSTE_F8E4M3)
    SSTE_LAUNCH(SSTE_K_FWD, (k_linear_fwd<true>), grid, block, s, (const uint8_t*)X, T, I, ldx, (const uint8_t*)vals,
                       (const uint8_t*)meta, I / 8, O, scale, (uint16_t*)Z, ldz);
  else
    SSTE_LAUNCH(SSTE_K_FWD, (k_linear_fwd<false>), grid, block, s, (const uint8_t*)X, T, I * 2, ldx * 2,
                       (const uint8_t*)vals, (const uint8_t*)meta, I / 8, O, scale, (uint16_t*)Z, ldz);
  return hipGetLastError();
}

}  // namespace sste
