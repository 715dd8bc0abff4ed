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
// Tiling: a workgroup of 4 waves (2 x 2) computes BM (o) x BN (t); each wave owns MI x NI MFMA tiles.
// The large shape is 256 x 128 (wave 128 x 64): per sparse MFMA the wave then reads about 540 B from
// LDS, which keeps the four SIMDs inside the measured LDS read rate (about 220 B/clk per CU for
// 16-byte reads).  Operands are staged through LDS with a register prefetch of the next k-step.
// LDS rows are padded to an odd multiple of 32 bytes (96 B for values, 160 B for X): measured
// conflict-free for the fragment reads (16 rows x 4 adjacent 16-byte pieces per instruction).
// Workgroups are numbered so that each XCD (the chip routes consecutive workgroup ids to its 8 XCDs
// in turn) works on a contiguous range of tiles, o-tiles fastest: the packed weight stays in that
// XCD's L2 and an X tile is fetched from HBM once per XCD.
#include "common.h"

namespace sste {

namespace {
constexpr int A_STRIDE = 96;    // 64 B of packed values + 32 B pad
constexpr int B_STRIDE = 160;   // 128 B of X + 32 B pad
constexpr int M_STRIDE = 16;    // metadata bytes per row and k-step: 8 (bf16) or 16 (fp8)
constexpr int NUM_XCD = 8;
}  // namespace

template <bool FP8, int MI, int NI>
__global__ void __launch_bounds__(256, 2)
k_linear_fwd(const uint8_t* __restrict__ X, int64_t T, int64_t k_bytes, int64_t ldx_bytes,
             const uint8_t* __restrict__ vals, const uint8_t* __restrict__ meta, int64_t meta_row_bytes,
             int64_t O, float scale, uint16_t* __restrict__ Z, int64_t ldz, int m_tiles) {
  constexpr int BM = 32 * MI, BN = 32 * NI;      // 2 x 2 waves of MI x NI tiles of 16 x 16
  constexpr int ACH = BM * 4 / 256;              // 16-byte chunks of packed values per lane and k-step
  constexpr int BCH = BN * 8 / 256;              // 16-byte chunks of X per lane and k-step
  __shared__ __align__(16) uint8_t sA[BM * A_STRIDE];
  __shared__ __align__(16) uint8_t sM[BM * M_STRIDE];
  __shared__ __align__(16) uint8_t sB[BN * B_STRIDE];

  // XCD-aware tile order: XCD x owns a contiguous range of logical tiles
  const int bid = blockIdx.x, nblk = gridDim.x;
  const int per_xcd = (nblk + NUM_XCD - 1) / NUM_XCD, rem = nblk % NUM_XCD;
  const int xcd = bid % NUM_XCD, slot = bid / NUM_XCD;
  const int logical = (rem == 0 || xcd < rem) ? xcd * per_xcd + slot
                                              : rem * per_xcd + (xcd - rem) * (per_xcd - 1) + slot;
  const int tm = logical % m_tiles, tn = logical / m_tiles;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int j = lane & 15, q = lane >> 4;
  const int64_t o0 = (int64_t)tm * BM, t0 = (int64_t)tn * BN;
  const int nsteps = (int)(k_bytes / 128);
  const int64_t vals_row_bytes = k_bytes / 2;

  f32x4 acc[MI][NI];
#pragma unroll
  for (int a = 0; a < MI; a++)
#pragma unroll
    for (int b = 0; b < NI; b++) acc[a][b] = (f32x4){0.f, 0.f, 0.f, 0.f};

  uint4 ra[ACH], rb[BCH], rm;

  // Operand tiles are read through buffer descriptors that cover exactly the valid rows of this
  // tile: rows past the end of the matrix come back as zeros without a branch.
  const int rows_a = (int)((O - o0) < BM ? (O - o0) : BM), rows_b = (int)((T - t0) < BN ? (T - t0) : BN);
  const BufferRsrc ba = make_rsrc(vals + o0 * vals_row_bytes, (uint32_t)(rows_a * vals_row_bytes));
  const BufferRsrc bm = make_rsrc(meta + o0 * meta_row_bytes, (uint32_t)(rows_a * meta_row_bytes));
  const BufferRsrc bb = make_rsrc(X + t0 * ldx_bytes, (uint32_t)((rows_b - 1) * ldx_bytes + k_bytes));
  uint32_t offa[ACH], offb[BCH];
#pragma unroll
  for (int r = 0; r < ACH; r++) {
    int c = tid + 256 * r, row = c >> 2, part = c & 3;
    offa[r] = (uint32_t)(row * vals_row_bytes + part * 16);
  }
  // lanes that own no metadata row point past the end of the descriptor
  const uint32_t offm = (tid < BM) ? (uint32_t)(tid * meta_row_bytes) : 0x7FFFFF00u;
#pragma unroll
  for (int r = 0; r < BCH; r++) {
    int c = tid + 256 * r, row = c >> 3, part = c & 7;
    offb[r] = (uint32_t)(row * ldx_bytes + part * 16);
  }

#define FWD_LOAD_GLOBAL(step)                                                        \
  do {                                                                               \
    _Pragma("unroll") for (int r = 0; r < ACH; r++) ra[r] = buffer_load_b128(ba, offa[r], (step) * 64); \
    if (FP8) rm = buffer_load_b128(bm, offm, (step) * 16);                           \
    else { uint2 v = buffer_load_b64(bm, offm, (step) * 8); rm = make_uint4(v.x, v.y, 0, 0); } \
    _Pragma("unroll") for (int r = 0; r < BCH; r++) rb[r] = buffer_load_b128(bb, offb[r], (step) * 128); \
  } while (0)

#define FWD_STORE_LDS()                                                              \
  do {                                                                               \
    _Pragma("unroll") for (int r = 0; r < ACH; r++) {                                \
      int c = tid + 256 * r, row = c >> 2, part = c & 3;                             \
      *(uint4*)(sA + row * A_STRIDE + part * 16) = ra[r];                            \
    }                                                                                \
    if (tid < BM) *(uint4*)(sM + tid * M_STRIDE) = rm;                               \
    _Pragma("unroll") for (int r = 0; r < BCH; r++) {                                \
      int c = tid + 256 * r, row = c >> 3, part = c & 7;                             \
      *(uint4*)(sB + row * B_STRIDE + part * 16) = rb[r];                            \
    }                                                                                \
  } while (0)

  if (nsteps > 0) FWD_LOAD_GLOBAL(0);
  for (int step = 0; step < nsteps; step++) {
    FWD_STORE_LDS();
    __syncthreads();
    if (step + 1 < nsteps) FWD_LOAD_GLOBAL(step + 1);

    uint4 fb[NI][2];
#pragma unroll
    for (int ni = 0; ni < NI; ni++) {
      int row = (16 * NI) * wn + 16 * ni + j;
      fb[ni][0] = *(const uint4*)(sB + row * B_STRIDE + 16 * q);
      fb[ni][1] = *(const uint4*)(sB + row * B_STRIDE + 64 + 16 * q);
    }
#pragma unroll
    for (int mi = 0; mi < MI; mi++) {
      int row = (16 * MI) * wm + 16 * mi + j;
      uint4 fa = *(const uint4*)(sA + row * A_STRIDE + 16 * q);
      int fidx;
      if (FP8) fidx = *(const int*)(sM + row * M_STRIDE + 4 * q);
      else fidx = *(const uint16_t*)(sM + row * M_STRIDE + 2 * q);
#pragma unroll
      for (int ni = 0; ni < NI; ni++) {
        if (FP8) {
          i32x4 av;
          i32x8 bv;
          __builtin_memcpy(&av, &fa, 16);
          __builtin_memcpy(&bv, &fb[ni][0], 32);
          acc[mi][ni] = __builtin_amdgcn_smfmac_f32_16x16x128_fp8_fp8(av, bv, acc[mi][ni], fidx, 0, 0);
        } else {
          bf16x8 av;
          bf16x16 bv;
          __builtin_memcpy(&av, &fa, 16);
          __builtin_memcpy(&bv, &fb[ni][0], 32);
          acc[mi][ni] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(av, bv, acc[mi][ni], fidx, 0, 0);
        }
      }
    }
    __syncthreads();
  }
#undef FWD_LOAD_GLOBAL
#undef FWD_STORE_LDS

  // epilogue: lane (j, q) register r of tile (mi, ni) is Z[t][o + r], four consecutive channels
#pragma unroll
  for (int mi = 0; mi < MI; mi++)
#pragma unroll
    for (int ni = 0; ni < NI; ni++) {
      int64_t o = o0 + (16 * MI) * wm + 16 * mi + 4 * q;
      int64_t t = t0 + (16 * NI) * wn + 16 * ni + j;
      if (t < T && o < O) {
        uint2 v;
        v.x = bf16_rne_pack(acc[mi][ni][0] * scale, acc[mi][ni][1] * scale);
        v.y = bf16_rne_pack(acc[mi][ni][2] * scale, acc[mi][ni][3] * scale);
        *(uint2*)(Z + t * ldz + o) = v;
      }
    }
}

template <bool FP8, int MI, int NI>
static void launch_fwd_cfg(const void* X, int64_t T, int64_t I, int64_t ldx, float scale, const void* vals,
                           const void* meta, int64_t O, void* Z, int64_t ldz, hipStream_t s) {
  constexpr int BM = 32 * MI, BN = 32 * NI;
  int m_tiles = (int)((O + BM - 1) / BM), n_tiles = (int)((T + BN - 1) / BN);
  dim3 grid((unsigned)(m_tiles * n_tiles)), block(256);
  int64_t eb = FP8 ? 1 : 2;
  SSTE_LAUNCH(SSTE_K_FWD, (k_linear_fwd<FP8, MI, NI>), grid, block, s, (const uint8_t*)X, T, I * eb, ldx * eb,
              (const uint8_t*)vals, (const uint8_t*)meta, I / 8, O, scale, (uint16_t*)Z, ldz, m_tiles);
}

hipError_t launch_linear_fwd(const void* X, int64_t T, int64_t I, int64_t ldx, int dtype, float scale,
                             const void* vals, const void* meta, int64_t O, void* Z, int64_t ldz, hipStream_t s) {
  if (T == 0 || O == 0) return hipSuccess;
  if (((O + 127) / 128) * ((T + 127) / 128) > 0x7FFFFFFFll) return hipErrorInvalidValue;
  // large problems use the 256 x 128 tile; small ones keep 128 x 128 so that more workgroups exist
  bool big = ((O + 255) / 256) * ((T + 127) / 128) >= 512;
  bool fp8 = dtype == SSTE_F8E4M3;
  if (big) {
    if (fp8) launch_fwd_cfg<true, 8, 4>(X, T, I, ldx, scale, vals, meta, O, Z, ldz, s);
    else launch_fwd_cfg<false, 8, 4>(X, T, I, ldx, scale, vals, meta, O, Z, ldz, s);
  } else {
    if (fp8) launch_fwd_cfg<true, 4, 4>(X, T, I, ldx, scale, vals, meta, O, Z, ldz, s);
    else launch_fwd_cfg<false, 4, 4>(X, T, I, ldx, scale, vals, meta, O, Z, ldz, s);
  }
  return hipGetLastError();
}

}  // namespace sste
