// Weight-gradient GEMM of the S-STE linear layer (paper Sec. 5.1): grad_W = MVUE(grad_Z^T) X --
// the variant with the estimator fused into the operand load, used for small problems.
//
// MFMA mapping: rows = output channels o, columns = input features i, contraction = tokens t.
// The sparse operand A = MVUE(dY^T) is never materialised in HBM: every k-step the workgroup loads a
// [tokens x channels] tile of dY, runs the estimator on groups of four consecutive tokens in
// registers, and writes packed values + position bits straight into the LDS layout the sparse MFMA
// reads (row o: 16 bytes per lane quarter).  The random number of a group depends only on
// (key, group id), so any tiling or split of the token axis gives the same sparsified operand.
// Operand B = X arrives with the contraction index strided (X is [t][i]); its fragments are read
// with the transposing LDS load (ds_read_b64_tr_b16 / _b8), which hands each lane 4 (8) consecutive
// k of one column.
//
// Tiling: 128 (o) x 128 (i) per workgroup of 4 waves (2 x 2), k-step of 64 tokens (bf16) / 128 (fp8),
// token axis split over gridDim.z with partial sums reduced in a fixed order by a second kernel.
#include "common.h"
#include "mvue_device.h"

namespace sste {

namespace {
constexpr int BM = 128, BN = 128;
constexpr int A_STRIDE = 80;     // 64 B of packed values per row + pad
constexpr int MB_STRIDE = 32;    // one metadata byte per group: 16 (bf16) / 32 (fp8) groups per k-step

// component c (compile-time after unrolling) of a uint4
__device__ __forceinline__ uint32_t comp(const uint4& v, int c) { return c == 0 ? v.x : (c == 1 ? v.y : (c == 2 ? v.z : v.w)); }

typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;
typedef __attribute__((address_space(3))) i32x2 lds_i32x2;
}  // namespace

template <bool FP8, bool BF8>
__global__ void __launch_bounds__(256)
k_linear_wgrad_fused(const uint8_t* __restrict__ dY, int64_t T, int64_t O, int64_t lddy_bytes,
               const uint8_t* __restrict__ X, int64_t I, int64_t ldx_bytes, RngKey key,
               int steps_per_split, float scale, int accumulate,
               float* __restrict__ out, int64_t ld_out, int64_t split_stride) {
  constexpr int EB = FP8 ? 1 : 2;               // bytes per element
  constexpr int BK = FP8 ? 128 : 64;            // tokens per k-step
  constexpr int B_STRIDE = BN * EB + 32;        // X tile row (one token) + pad
  constexpr int GROUPS = BK / 4;                // token groups per k-step
  __shared__ __align__(16) uint8_t sA[BM * A_STRIDE];
  __shared__ __align__(16) uint8_t sM[BM * MB_STRIDE];
  __shared__ __align__(16) uint8_t sB[BK * B_STRIDE];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int j = lane & 15, q = lane >> 4;
  const int64_t o0 = (int64_t)blockIdx.x * BM, i0 = (int64_t)blockIdx.y * BN;
  const int64_t total_steps = T / BK;
  const int64_t step_begin = (int64_t)blockIdx.z * steps_per_split;
  int64_t step_end = step_begin + steps_per_split;
  if (step_end > total_steps) step_end = total_steps;

  f32x4 acc[4][4];
#pragma unroll
  for (int a = 0; a < 4; a++)
#pragma unroll
    for (int b = 0; b < 4; b++) acc[a][b] = (f32x4){0.f, 0.f, 0.f, 0.f};

  // dY tile: a lane owns 4 tokens (one group) x 16 bytes of channels (8 bf16 / 16 fp8 channels)
  constexpr int OC = BM * EB / 16;              // 16-byte channel chunks per tile row: 16 (bf16) / 8 (fp8)
  const int kg = tid / OC, oc = tid % OC;       // kg in [0, GROUPS): 256 / OC == GROUPS for both types
  constexpr int CH = 16 / EB;                   // channels per chunk
  // X tile: BK rows of BN * EB bytes
  constexpr int XCHUNKS = BK * BN * EB / 16 / 256;   // 16-byte chunks per lane: 4 (bf16) / 4 (fp8)
  constexpr int XPR = BN * EB / 16;                  // chunks per row: 16 / 8

  uint4 rdy[4], rx[XCHUNKS];

  // Columns past the end of the matrix are read from column chunk 0 (always mapped) and then zeroed,
  // so the loads need no branch.
  const bool okdy = (o0 + (int64_t)oc * CH) < O;
  const uint8_t* pdy = dY + (int64_t)(4 * kg) * lddy_bytes + (okdy ? (o0 + (int64_t)oc * CH) : 0) * EB;
  const uint8_t* px[XCHUNKS];
  bool okx[XCHUNKS];
#pragma unroll
  for (int r = 0; r < XCHUNKS; r++) {
    int c = tid + 256 * r, row = c / XPR, part = c % XPR;
    okx[r] = (i0 + (int64_t)part * CH) < I;
    px[r] = X + (int64_t)row * ldx_bytes + (okx[r] ? (i0 + (int64_t)part * CH) : 0) * EB;
  }

#define WG_LOAD_GLOBAL(step)                                                                  \
  do {                                                                                        \
    int64_t tb_ = (int64_t)(step) * BK;                                                       \
    _Pragma("unroll") for (int r = 0; r < 4; r++) {                                           \
      uint4 v = *(const uint4*)(pdy + (tb_ + r) * lddy_bytes);                                \
      rdy[r] = okdy ? v : make_uint4(0, 0, 0, 0);                                             \
    }                                                                                         \
    _Pragma("unroll") for (int r = 0; r < XCHUNKS; r++) {                                     \
      uint4 v = *(const uint4*)(px[r] + tb_ * ldx_bytes);                                     \
      rx[r] = okx[r] ? v : make_uint4(0, 0, 0, 0);                                            \
    }                                                                                         \
  } while (0)

  // The estimator on the lane's CH groups (tokens 4 kg .. 4 kg + 3 of CH channels), written to LDS in
  // the layout the sparse MFMA reads, then the X tile.
#define WG_SPARSIFY_AND_STORE(step)                                                           \
  do {                                                                                        \
    uint64_t gid_base = (key.first_group + (uint64_t)((int64_t)(step) * GROUPS + kg)) * (uint64_t)O + (uint64_t)(o0 + (int64_t)oc * CH); \
    _Pragma("unroll") for (int e = 0; e < CH; e++) {                                          \
      uint64_t gid = gid_base + e;                                                            \
      uint32_t x = draw_u32(key.k0, key.k1, (uint32_t)gid, (uint32_t)(gid >> 32));            \
      uint32_t nib, v;                                                                        \
      int row = oc * CH + e;                                                                  \
      if (FP8) {                                                                              \
        uint32_t w0 = comp(rdy[0], e >> 2), w1 = comp(rdy[1], e >> 2);                        \
        uint32_t w2 = comp(rdy[2], e >> 2), w3 = comp(rdy[3], e >> 2);                        \
        int sh = 8 * (e & 3);                                                                 \
        uint32_t g = ((w0 >> sh) & 0xFFu) | (((w1 >> sh) & 0xFFu) << 8) | (((w2 >> sh) & 0xFFu) << 16) | (((w3 >> sh) & 0xFFu) << 24); \
        v = mvue_group_f8<BF8>(g, x, nib);                                                      \
        *(uint16_t*)(sA + row * A_STRIDE + 2 * kg) = (uint16_t)v;                             \
      } else {                                                                                \
        uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;                                   \
        uint32_t lo = __builtin_amdgcn_perm(comp(rdy[1], e >> 1), comp(rdy[0], e >> 1), sel); \
        uint32_t hi = __builtin_amdgcn_perm(comp(rdy[3], e >> 1), comp(rdy[2], e >> 1), sel); \
        v = mvue_group_bf16(lo, hi, x, nib);                                                  \
        *(uint32_t*)(sA + row * A_STRIDE + 4 * kg) = v;                                       \
      }                                                                                       \
      /* nibble pre-shifted to its place inside the byte pair: consumers OR neighbouring bytes */ \
      sM[row * MB_STRIDE + kg] = (uint8_t)(nib << (4 * (kg & 1)));                            \
    }                                                                                         \
    _Pragma("unroll") for (int r = 0; r < XCHUNKS; r++) {                                     \
      int c = tid + 256 * r, row = c / XPR, part = c % XPR;                                   \
      *(uint4*)(sB + row * B_STRIDE + part * 16) = rx[r];                                     \
    }                                                                                         \
  } while (0)

  if (step_begin < step_end) WG_LOAD_GLOBAL(step_begin);
  for (int64_t step = step_begin; step < step_end; step++) {
    WG_SPARSIFY_AND_STORE(step);
    __syncthreads();
    if (step + 1 < step_end) WG_LOAD_GLOBAL(step + 1);

    uint4 fa[4];
    int fidx[4];
#pragma unroll
    for (int mi = 0; mi < 4; mi++) {
      int row = 64 * wm + 16 * mi + j;
      fa[mi] = *(const uint4*)(sA + row * A_STRIDE + 16 * q);
      if (FP8) {
        // 8 groups per lane: bytes b0..b7, odd ones pre-shifted by 4
        uint2 w = *(const uint2*)(sM + row * MB_STRIDE + 8 * q);
        uint32_t a = w.x | (w.x >> 8), b = w.y | (w.y >> 8);
        fidx[mi] = (int)((a & 0xFFu) | ((a >> 8) & 0xFF00u) | ((b & 0xFFu) << 16) | ((b << 8) & 0xFF000000u));
      } else {
        uint32_t w = *(const uint32_t*)(sM + row * MB_STRIDE + 4 * q);
        uint32_t a = w | (w >> 8);
        fidx[mi] = (int)((a & 0xFFu) | ((a >> 8) & 0xFF00u));
      }
    }
#pragma unroll
    for (int ni = 0; ni < 4; ni++) {
      int n0 = 64 * wn + 16 * ni;
      uint2 piece[4];
#pragma unroll
      for (int r = 0; r < 4; r++) {
        if (FP8) {
          // piece r holds 8 consecutive tokens: k0 = 16 q + 8 (r & 1) + 64 (r >> 1);
          // source lane s of the 16-lane block addresses row k0 + s / 2, columns n0 + 8 (s % 2) ..
          int k0 = 16 * q + 8 * (r & 1) + 64 * (r >> 1);
          const uint8_t* p = sB + (k0 + (j >> 1)) * B_STRIDE + (n0 + 8 * (j & 1));
          i32x2 t = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_i32x2*)p);
          piece[r].x = (uint32_t)t[0];
          piece[r].y = (uint32_t)t[1];
        } else {
          // piece r holds 4 consecutive tokens: k0 = 8 q + 4 (r & 1) + 32 (r >> 1);
          // source lane s addresses row k0 + s / 4, columns n0 + 4 (s % 4) ..
          int k0 = 8 * q + 4 * (r & 1) + 32 * (r >> 1);
          const uint8_t* p = sB + (k0 + (j >> 2)) * B_STRIDE + (n0 + 4 * (j & 3)) * 2;
          bf16x4 t = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)p);
          __builtin_memcpy(&piece[r], &t, 8);
        }
      }
#pragma unroll
      for (int mi = 0; mi < 4; mi++) {
        if (FP8) {
          i32x4 av;
          i32x8 bv;
          __builtin_memcpy(&av, &fa[mi], 16);
          __builtin_memcpy(&bv, &piece[0], 32);
          if (BF8) acc[mi][ni] = __builtin_amdgcn_smfmac_f32_16x16x128_bf8_fp8(av, bv, acc[mi][ni], fidx[mi], 0, 0);
          else acc[mi][ni] = __builtin_amdgcn_smfmac_f32_16x16x128_fp8_fp8(av, bv, acc[mi][ni], fidx[mi], 0, 0);
        } else {
          bf16x8 av;
          bf16x16 bv;
          __builtin_memcpy(&av, &fa[mi], 16);
          __builtin_memcpy(&bv, &piece[0], 32);
          acc[mi][ni] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(av, bv, acc[mi][ni], fidx[mi], 0, 0);
        }
      }
    }
    __syncthreads();
  }

#undef WG_LOAD_GLOBAL
#undef WG_SPARSIFY_AND_STORE

  // epilogue: lane (j, q) register r of tile (mi, ni) is element (o + r, i)
  float* dst = out + (int64_t)blockIdx.z * split_stride;
#pragma unroll
  for (int mi = 0; mi < 4; mi++)
#pragma unroll
    for (int ni = 0; ni < 4; ni++) {
      int64_t o = o0 + 64 * wm + 16 * mi + 4 * q;
      int64_t i = i0 + 64 * wn + 16 * ni + j;
      if (i < I) {
#pragma unroll
        for (int r = 0; r < 4; r++) {
          if (o + r < O) {
            float v = acc[mi][ni][r] * scale;
            float* p = dst + (o + r) * ld_out + i;
            *p = accumulate ? (*p + v) : v;
          }
        }
      }
    }
}

// Launch of the fused kernel on one split range; `out` is dW (single split) or the partial-sum buffer.
hipError_t launch_wgrad_fused(const void* dY, int64_t T, int64_t O, int64_t lddy, int dtype, const void* X, int64_t I,
                              int64_t ldx, RngKey key, int splits, int steps_per_split, float scale, int accumulate,
                              float* out, int64_t ld_out, int64_t split_stride, hipStream_t s) {
  bool fp8 = dtype != SSTE_BF16, bf8 = dtype == SSTE_F8E5M2;
  int eb = fp8 ? 1 : 2;
  dim3 grid((unsigned)((O + BM - 1) / BM), (unsigned)((I + BN - 1) / BN), (unsigned)splits), block(256);
  if (bf8)
    SSTE_LAUNCH(SSTE_K_WGRAD, (k_linear_wgrad_fused<true, true>), grid, block, s, (const uint8_t*)dY, T, O, lddy * eb, (const uint8_t*)X, I,
                ldx * eb, key, steps_per_split, scale, accumulate, out, ld_out, split_stride);
  else if (fp8)
    SSTE_LAUNCH(SSTE_K_WGRAD, (k_linear_wgrad_fused<true, false>), grid, block, s, (const uint8_t*)dY, T, O, lddy * eb, (const uint8_t*)X, I,
                ldx * eb, key, steps_per_split, scale, accumulate, out, ld_out, split_stride);
  else
    SSTE_LAUNCH(SSTE_K_WGRAD, (k_linear_wgrad_fused<false, false>), grid, block, s, (const uint8_t*)dY, T, O, lddy * eb, (const uint8_t*)X, I,
                ldx * eb, key, steps_per_split, scale, accumulate, out, ld_out, split_stride);
  return hipGetLastError();
}

}  // namespace sste
