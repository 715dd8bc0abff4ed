// Weight-gradient path of the S-STE linear layer (paper Sec. 5.1): grad_W = MVUE(grad_Z^T) X.
//
// Large problems run in three kernels on the caller's stream:
//   1. k_mvue_pack: the estimator is applied once per group of four tokens and the result is written
//      to the workspace as a packed 2:4 operand in sparse-MFMA fragment order (the format of
//      include/sste.h with rows = output channels, columns = tokens).  It streams dY once: at about
//      90 vector instructions per group (three of them half-rate 32-bit multiplies of the hash) the
//      bf16 kernel runs at the rate of a plain copy, the e4m3 kernel (twice the groups per byte) is
//      bound by the vector pipe.
//   2. k_wgrad_gemm: sparse MFMA GEMM, rows = channels o, columns = input features i, contraction =
//      tokens, split over the token axis.  The packed operand is loaded like the packed weight of the
//      forward GEMM; X arrives with the contraction index strided (X is [t][i]) and its fragments are
//      read with the transposing LDS load (ds_read_b64_tr_b16 / _b8).  Tile shape and split count are
//      chosen per problem (wgrad_plan).
//   3. k_wgrad_reduce: sums the splits in a fixed order (bitwise reproducible) and applies the scale.
// Why not fuse the estimator into the GEMM's operand load everywhere: a GEMM tile that is N columns
// wide re-derives every group I / N times.  With a 128-wide tile that is 6 to 40 times per group and
// the vector pipe, not the matrix pipe or HBM, sets the time (measured: 176 us fused against 55 us
// here for the 3072 x 768 layer at 8192 tokens; on the 5120 x 1280 layer a 256-wide tile would issue
// five times the pre-pass's vector work, about 280 us against the 110 us of the whole GEMM).  The fused kernel (gemm_wgrad_fused.hip) is kept for
// small problems, where one launch and no workspace matter more.
#include "common.h"
#include "mvue_device.h"

#include <atomic>
#include <mutex>

namespace sste {

hipError_t launch_wgrad_fused(const void* dY, int64_t T, int64_t O, int64_t lddy, int dtype, const void* X, int64_t I,
                              int64_t ldx, RngKey key, int splits, int steps_per_split, float scale, int accumulate,
                              float* out, int64_t ld_out, int64_t split_stride, hipStream_t s);

namespace {
constexpr int NUM_CU = 256;
typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;
typedef __attribute__((address_space(3))) i32x2 lds_i32x2;

__device__ __forceinline__ uint32_t comp4(const uint4& v, int c) { return c == 0 ? v.x : (c == 1 ? v.y : (c == 2 ? v.z : v.w)); }
}  // namespace

// ---------------------------------------------------------------------------------------------------------
// 1. estimator -> packed operand.  One workgroup: one k-step (64 / 128 tokens) x 128 channels.
template <bool FP8, bool BF8>
__global__ void __launch_bounds__(256)
k_mvue_pack(const uint8_t* __restrict__ dY, int64_t T, int64_t O, int64_t lddy_bytes, RngKey key,
            uint8_t* __restrict__ vals, uint8_t* __restrict__ meta) {
  constexpr int EB = FP8 ? 1 : 2;
  constexpr int KS = FP8 ? 128 : 64;              // tokens per k-step
  constexpr int GROUPS = KS / 4;                  // 16 / 32 token groups per k-step
  constexpr int CH = 16 / EB;                     // channels per 16-byte chunk: 8 / 16
  constexpr int OC = 128 / CH;                    // chunks across the 128 channels: 16 / 8
  constexpr int GPQ = GROUPS / 4;                 // groups per lane quarter: 4 / 8
  constexpr int MBLK = FP8 ? 256 : 128;           // metadata bytes per block
  // LDS staging, padded against bank conflicts: the lanes of a wave write the same slot of 8 different
  // blocks (1040-byte block pitch puts them 4 banks apart) and the same group of 8 or 16 different
  // channels (a pitch of GROUPS + 4 bytes spreads those over the banks).
  constexpr int VPITCH = 1024 + 16, NPITCH = GROUPS + 4;
  __shared__ __align__(16) uint8_t sV[8 * VPITCH];
  __shared__ __align__(16) uint8_t sN[128 * NPITCH];

  const int tid = threadIdx.x;
  const int kg = tid / OC, oc = tid % OC;
  const int64_t s = blockIdx.y, steps = T / KS;
  const int64_t o0 = (int64_t)blockIdx.x * 128;
  const int64_t och = o0 + (int64_t)oc * CH;

  uint4 rdy[4];
  if (och < O) {
    const uint8_t* p = dY + (s * KS + 4 * kg) * lddy_bytes + och * EB;
#pragma unroll
    for (int r = 0; r < 4; r++) {
      i32x4 t = __builtin_nontemporal_load((const i32x4*)(p + r * lddy_bytes));
      rdy[r] = make_uint4((uint32_t)t[0], (uint32_t)t[1], (uint32_t)t[2], (uint32_t)t[3]);
    }
  } else {
#pragma unroll
    for (int r = 0; r < 4; r++) rdy[r] = make_uint4(0, 0, 0, 0);
  }
  // Group ids of this lane: gid_base + e.  O and och are multiples of CH, so gid_base is one too and the
  // CH consecutive ids share their high word (no carry out of the low word inside the piece).
  const uint64_t gid_base = (key.first_group + (uint64_t)(s * GROUPS + kg)) * (uint64_t)O + (uint64_t)och;
  const uint32_t gid_lo0 = (uint32_t)gid_base;
  const uint32_t hi_term = (uint32_t)(gid_base >> 32) * 0x9E3779B9u;
  const int q = kg / GPQ, g = kg % GPQ;
  // 8-bit: the four token rows' dwords of four channels, transposed 4 x 4 bytes at a time (eight byte permutes
  // for four groups): grp[k] holds channel 4 (e / 4) + k with token 0 in byte 0
  uint32_t grp[4] = {0, 0, 0, 0};
#pragma unroll
  for (int e = 0; e < CH; e++) {
    uint32_t x = draw_u32_pre(key.k0, key.k1, gid_lo0 + (uint32_t)e, hi_term);
    uint32_t nib, v;
    int c = oc * CH + e;                           // channel inside the tile
    uint8_t* slot = sV + (c >> 4) * VPITCH + (16 * q + (c & 15)) * 16;
    if (FP8) {
      if ((e & 3) == 0) {
        uint32_t w0 = comp4(rdy[0], e >> 2), w1 = comp4(rdy[1], e >> 2), w2 = comp4(rdy[2], e >> 2), w3 = comp4(rdy[3], e >> 2);
        uint32_t a01 = __builtin_amdgcn_perm(w1, w0, 0x05010400u), b01 = __builtin_amdgcn_perm(w1, w0, 0x07030602u);
        uint32_t a23 = __builtin_amdgcn_perm(w3, w2, 0x05010400u), b23 = __builtin_amdgcn_perm(w3, w2, 0x07030602u);
        grp[0] = __builtin_amdgcn_perm(a23, a01, 0x05040100u);
        grp[1] = __builtin_amdgcn_perm(a23, a01, 0x07060302u);
        grp[2] = __builtin_amdgcn_perm(b23, b01, 0x05040100u);
        grp[3] = __builtin_amdgcn_perm(b23, b01, 0x07060302u);
      }
      v = mvue_group_f8<BF8>(grp[e & 3], x, nib);
      *(uint16_t*)(slot + 2 * g) = (uint16_t)v;
    } else {
      uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;
      uint32_t lo = __builtin_amdgcn_perm(comp4(rdy[1], e >> 1), comp4(rdy[0], e >> 1), sel);
      uint32_t hi = __builtin_amdgcn_perm(comp4(rdy[3], e >> 1), comp4(rdy[2], e >> 1), sel);
      v = mvue_group_bf16(lo, hi, x, nib);
      *(uint32_t*)(slot + 4 * g) = v;
    }
    sN[c * NPITCH + kg] = (uint8_t)(nib << (4 * (kg & 1)));   // pre-shifted: neighbours are OR-ed below
  }
  __syncthreads();

  const int64_t rb0 = o0 / 16, rbn = (O + 15) / 16;
#pragma unroll
  for (int it = 0; it < 2; it++) {
    int ci = tid + 256 * it, rb = ci >> 6, sl = ci & 63;     // block and slot inside the tile
    if (rb0 + rb < rbn) {
      int64_t blk = (rb0 + rb) * steps + s;
      *(uint4*)(vals + blk * 1024 + sl * 16) = *(const uint4*)(sV + rb * VPITCH + sl * 16);
      int c = rb * 16 + (sl & 15), qq = sl >> 4;
      if (FP8) {
        uint32_t wx = *(const uint32_t*)(sN + c * NPITCH + 8 * qq), wy = *(const uint32_t*)(sN + c * NPITCH + 8 * qq + 4);
        uint32_t a = wx | (wx >> 8), b = wy | (wy >> 8);
        uint32_t idx = (a & 0xFFu) | ((a >> 8) & 0xFF00u) | ((b & 0xFFu) << 16) | ((b << 8) & 0xFF000000u);
        *(uint32_t*)(meta + blk * MBLK + sl * 4) = idx;
      } else {
        uint32_t w = *(const uint32_t*)(sN + c * NPITCH + 4 * qq);
        uint32_t a = w | (w >> 8);
        *(uint16_t*)(meta + blk * MBLK + sl * 2) = (uint16_t)((a & 0xFFu) | ((a >> 8) & 0xFF00u));
      }
    }
  }
}

static void launch_mvue_pack(const void* dY, int64_t T, int64_t O, int64_t lddy, int dtype, RngKey key, void* vals,
                             void* meta, hipStream_t s, int timed_kind) {
  bool fp8 = dtype != SSTE_BF16;
  int ks = fp8 ? 128 : 64;
  dim3 grid((unsigned)((O + 127) / 128), (unsigned)(T / ks)), block(256);
#define MP_CASE(F8, B8)                                                                                                  \
  do {                                                                                                                   \
    if (timed_kind >= 0)                                                                                                 \
      SSTE_LAUNCH(timed_kind, (k_mvue_pack<F8, B8>), grid, block, s, (const uint8_t*)dY, T, O, lddy*(F8 ? 1 : 2), key,   \
                  (uint8_t*)vals, (uint8_t*)meta);                                                                       \
    else                                                                                                                 \
      hipLaunchKernelGGL((k_mvue_pack<F8, B8>), grid, block, 0, s, (const uint8_t*)dY, T, O, lddy*(F8 ? 1 : 2), key,     \
                         (uint8_t*)vals, (uint8_t*)meta);                                                                \
  } while (0)
  if (dtype == SSTE_F8E5M2) MP_CASE(true, true);
  else if (fp8) MP_CASE(true, false);
  else MP_CASE(false, false);
#undef MP_CASE
}

hipError_t launch_mvue_materialize(const void* dY, int64_t T, int64_t O, int64_t lddy, int dtype, RngKey key,
                                   void* vals, void* meta, hipStream_t s) {
  if (T == 0 || O == 0) return hipSuccess;
  launch_mvue_pack(dY, T, O, lddy, dtype, key, vals, meta, s, -1);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------------------
// 2. sparse GEMM on the packed operand.  8 waves (2 x 4), each owning MI_ x NI_ MFMA tiles: a workgroup
// covers 32 MI_ channels x 64 NI_ features (256 x 256, 192 x 192, ...) over one split of the token axis.
// Same software pipeline as the forward GEMM: X fragments double-buffered in registers and read one
// k-step ahead, packed fragments rolling one row block ahead, direct-to-LDS loads spread over the MFMA
// groups, separate three-slot rings for the two operands, one barrier per k-step.
// X tile in LDS: one row per token, 512 B (bf16: 256 features) or 256 B (fp8) whatever the tile width;
// narrower tiles leave the tail of each row unused.  32-byte feature pair p (bf16) / 16-byte chunk c
// (fp8) of token row r is stored at position p ^ x_swizzle(r) (common.h), which keeps the transposing
// reads below -- 4 (8) consecutive token rows x 16 features per 16 lanes, the four lane quarters 8 (16)
// rows apart -- off each other's banks.

template <bool FP8, int MI_, int NI_, bool BF8>
__global__ void __launch_bounds__(512, 1)
k_wgrad_gemm(const uint8_t* __restrict__ vals, const uint8_t* __restrict__ meta, int64_t O, int64_t total_steps,
             const uint8_t* __restrict__ X, int64_t I, int64_t ldx_bytes, int steps_per_split, float scale,
             int accumulate, float* __restrict__ out, int64_t ld_out, int64_t split_stride, int m_tiles, int n_tiles,
             int features_fastest) {
  constexpr int WN = 4, NW = 8, NR = 3;
  constexpr int BM = 32 * MI_, BN = 64 * NI_;
  constexpr int EB = FP8 ? 1 : 2;
  constexpr int KS = FP8 ? 128 : 64;              // tokens per k-step
  constexpr int MB = FP8 ? 16 : 8, MBLK = 16 * MB;
  constexpr int ROWB = 256 * EB;                  // LDS bytes per token row: 512 / 256
  constexpr int LA = (BM / 16 + NW - 1) / NW;     // packed blocks (1 KiB) per wave and k-step
  constexpr int LM = (BM * MB / 256 + NW - 1) / NW;
  constexpr int BSTAGE = KS * ROWB;               // 32 KiB
  constexpr int LB = BSTAGE / 1024 / NW;          // 4
  constexpr int A_BYTES = NW * LA * 1024, M_BYTES = NW * LM * 256, ASTAGE = A_BYTES + M_BYTES;
  constexpr int NLOAD = LA + LM + LB;             // issue order inside a k-step: A.., M.., B..
  constexpr int NPIECE = 4 * NI_;                 // 8-byte pieces of the next X fragments
  constexpr int RPL = 1024 / ROWB;                // token rows per 1 KiB load: 2 / 4
  constexpr int CPR = ROWB / 16;                  // 16-byte chunks per row: 32 / 16
  __shared__ __align__(1024) uint8_t smem[NR * (ASTAGE + BSTAGE)];
  uint8_t* const smemA = smem;
  uint8_t* const smemB = smem + NR * ASTAGE;

  // tile order: XCD x owns a contiguous range of (tile, split) units; inside a split either the channel
  // tiles or the feature tiles run fastest (the host picks what costs the XCD's L2 fewer operand bytes)
  const int logical = xcd_contiguous(blockIdx.x, gridDim.x);
  const int tiles = m_tiles * n_tiles;
  const int z = logical / tiles, tile = logical % tiles;
  const int tm = features_fastest ? tile / n_tiles : tile % m_tiles;
  const int tn = features_fastest ? tile % n_tiles : tile / m_tiles;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN, wn = wave % WN;
  const int j = lane & 15, q = lane >> 4;
  const int64_t o0 = (int64_t)tm * BM, i0 = (int64_t)tn * BN;
  const int64_t step_begin = (int64_t)z * steps_per_split;
  int64_t step_end = step_begin + steps_per_split;
  if (step_end > total_steps) step_end = total_steps;
  const int nsteps = (int)(step_end - step_begin);

  const int64_t rblk0 = o0 / 16, rbn = (O + 15) / 16;
  const int blks_a = (int)((rbn - rblk0) < BM / 16 ? (rbn - rblk0) : BM / 16);
  const i32x4 ba = rsrc_words(vals + (rblk0 * total_steps + step_begin) * 1024, (uint32_t)((blks_a * total_steps - step_begin) * 1024));
  const i32x4 bm = rsrc_words(meta + (rblk0 * total_steps + step_begin) * MBLK, (uint32_t)((blks_a * total_steps - step_begin) * MBLK));
  const int cols_b = (int)((I - i0) < BN ? (I - i0) : BN);
  const i32x4 bb = rsrc_words(X + step_begin * KS * ldx_bytes + i0 * EB, (uint32_t)(((int64_t)nsteps * KS - 1) * ldx_bytes + cols_b * EB));

  // Packed blocks past the tile's last one must fetch nothing although the descriptor (which runs to
  // the end of the tile's last block row) may still cover their offsets: push them out of range.
  uint32_t offa[LA], offb[LB], offm[LM];
#pragma unroll
  for (int i = 0; i < LA; i++)
    offa[i] = (LA * wave + i) < blks_a ? (uint32_t)((LA * wave + i) * total_steps * 1024 + lane * 16) : 0x80000000u;
#pragma unroll
  for (int i = 0; i < LB; i++) {
    int wl = LB * wave + i;
    int r = RPL * wl + lane / CPR, cs = lane % CPR;          // token row inside the k-step, stored chunk
    int c = FP8 ? (cs ^ x_swizzle<true>(r)) : ((((cs >> 1) ^ x_swizzle<false>(r)) << 1) | (cs & 1));   // source chunk
    // chunks past the last feature column of the tile must read as zeros
    offb[i] = (c * 16 < cols_b * EB) ? (uint32_t)(r * ldx_bytes + c * 16) : 0x80000000u;
  }
#pragma unroll
  for (int i = 0; i < LM; i++) {
    int d = 64 * (LM * wave + i) + lane;
    int blk = d / (MBLK / 4);
    offm[i] = blk < blks_a ? (uint32_t)(blk * total_steps * MBLK + 4 * (d % (MBLK / 4))) : 0x80000000u;
  }
  const uint32_t ldsA = (uint32_t)(uintptr_t)(lds_u8*)smemA;
  const uint32_t ldsB = (uint32_t)(uintptr_t)(lds_u8*)smemB;
  constexpr uint32_t DEAD = 0x40000000u;

#define WG_LOAD(n, sa, slot_a, sb, slot_b)                                                                \
  do {                                                                                                    \
    if ((n) < LA)                                                                                         \
      dma_b128(ba, ldsA + (uint32_t)(slot_a) * ASTAGE + (LA * wave + (n)) * 1024, offa[(n) < LA ? (n) : 0], \
               (sa) < nsteps ? (uint32_t)(sa) * 1024u : DEAD);                                            \
    else if ((n) < LA + LM)                                                                               \
      dma_b32(bm, ldsA + (uint32_t)(slot_a) * ASTAGE + A_BYTES + (LM * wave + ((n) - LA)) * 256,          \
              offm[((n) >= LA && (n) < LA + LM) ? (n) - LA : 0],                                          \
              (sa) < nsteps ? (uint32_t)(sa) * (uint32_t)MBLK : DEAD);                                    \
    else                                                                                                  \
      dma_b128(bb, ldsB + (uint32_t)(slot_b) * BSTAGE + (LB * wave + ((n) - LA - LM)) * 1024,             \
               offb[(n) >= LA + LM ? (n) - LA - LM : 0],                                                  \
               (sb) < nsteps ? (uint32_t)((sb) * KS * ldx_bytes) : DEAD);                                 \
  } while (0)

  f32x4 acc[MI_][NI_];
#pragma unroll
  for (int a = 0; a < MI_; a++)
#pragma unroll
    for (int b = 0; b < NI_; b++) acc[a][b] = (f32x4){0.f, 0.f, 0.f, 0.f};

  const uint32_t fa_off = (uint32_t)(MI_ * wm * 1024 + lane * 16);
  const uint32_t fm_off = (uint32_t)(A_BYTES + MI_ * wm * MBLK + lane * (MB / 4));
  // transposing reads of X: piece r of tile ni covers tokens k0 .. k0 + 3 (bf16) / k0 .. k0 + 7 (fp8)
  uint32_t fb_off[NI_][4];
#pragma unroll
  for (int ni = 0; ni < NI_; ni++)
#pragma unroll
    for (int r = 0; r < 4; r++) {
      int p = NI_ * wn + ni;                                      // feature pair (bf16) / chunk (fp8) of the tile
      if (FP8) {
        int row = 16 * q + 8 * (r & 1) + 64 * (r >> 1) + (j >> 1);
        fb_off[ni][r] = (uint32_t)(row * ROWB + ((p ^ x_swizzle<true>(row)) * 16) + 8 * (j & 1));
      } else {
        int row = 8 * q + 4 * (r & 1) + 32 * (r >> 1) + (j >> 2);
        fb_off[ni][r] = (uint32_t)(row * ROWB + ((p ^ x_swizzle<false>(row)) * 32) + ((j & 3) >> 1) * 16 + 8 * (j & 1));
      }
    }

#define WG_READ_B(dst, base, pc)                                                                          \
  do {                                                                                                    \
    const uint8_t* p_ = (base) + fb_off[(pc) >> 2][(pc) & 3];                                             \
    if (FP8) {                                                                                            \
      i32x2 t_ = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_i32x2*)p_);                                  \
      dst[(pc) >> 2][(pc) & 3] = make_uint2((uint32_t)t_[0], (uint32_t)t_[1]);                            \
    } else {                                                                                              \
      bf16x4 t_ = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)p_);                              \
      __builtin_memcpy(&dst[(pc) >> 2][(pc) & 3], &t_, 8);                                                \
    }                                                                                                     \
  } while (0)

  // prologue: packed tiles 0, 1 and X tiles 0, 1, 2 in flight, in the order the barriers expect
#pragma unroll
  for (int n = 0; n < NLOAD; n++) WG_LOAD(n, 0, 0, 0, 0);
#pragma unroll
  for (int n = 0; n < NLOAD; n++) WG_LOAD(n, 1, 1, 1, 1);
#pragma unroll
  for (int n = LA + LM; n < NLOAD; n++) WG_LOAD(n, 0, 0, 2, 2);

  uint2 fb0[NI_][4], fb1[NI_][4];     // X fragments: current / next k-step, roles swap every k-step
  uint4 fa[2];                        // packed fragment of row block mi in fa[mi % 2]
  int fidx[2];
  wait_vmcnt<LA + LM + 2 * LB>();     // tiles of k-step 0 have landed
  __syncthreads();
#pragma unroll
  for (int pc = 0; pc < NPIECE; pc++) WG_READ_B(fb0, smemB, pc);
  fa[0] = *(const uint4*)(smemA + fa_off);
  if (FP8) fidx[0] = *(const int*)(smemA + fm_off);
  else fidx[0] = *(const uint16_t*)(smemA + fm_off);

  int s0 = 0, s1 = 1, s2 = 2;         // ring slots of k-steps step, step + 1, step + 2 (both rings)

#define WG_STEP(BC, BX)                                                                                   \
  do {                                                                                                    \
    wait_vmcnt<LB>();                 /* all but the newest X tile: k-step step + 1 has landed */          \
    __syncthreads();                  /* ... for every wave; slots of step - 1 (packed) and step (X) are free */ \
    const uint8_t* pa = smemA + s0 * ASTAGE;                                                              \
    const uint8_t* pa1 = smemA + s1 * ASTAGE;                                                             \
    const uint8_t* pb1 = smemB + s1 * BSTAGE;                                                             \
    _Pragma("unroll") for (int mi = 0; mi < MI_; mi++) {                                                  \
      const uint8_t* an = mi < MI_ - 1 ? pa + (mi + 1) * 1024 : pa1;                                      \
      const uint8_t* mn = mi < MI_ - 1 ? pa + (mi + 1) * MBLK : pa1;                                      \
      fa[(mi + 1) & 1] = *(const uint4*)(an + fa_off);                                                    \
      if (FP8) fidx[(mi + 1) & 1] = *(const int*)(mn + fm_off);                                           \
      else fidx[(mi + 1) & 1] = *(const uint16_t*)(mn + fm_off);                                          \
      _Pragma("unroll") for (int pc = 0; pc < NPIECE; pc++)                                               \
        if (spread(pc, NPIECE, MI_) == mi) WG_READ_B(BX, pb1, pc);                                        \
      _Pragma("unroll") for (int n = 0; n < NLOAD; n++)                                                   \
        if (spread(n, NLOAD, MI_) == mi) WG_LOAD(n, step + 2, s2, step + 3, s0);                          \
      _Pragma("unroll") for (int ni = 0; ni < NI_; ni++) {                                                \
        if (FP8) {                                                                                        \
          i32x4 av;                                                                                       \
          i32x8 bv;                                                                                       \
          __builtin_memcpy(&av, &fa[mi & 1], 16);                                                         \
          __builtin_memcpy(&bv, &BC[ni][0], 32);                                                          \
          /* e5m2 sparsified gradient (packed operand) against e4m3 activations, or both e4m3 */          \
          if (BF8) acc[mi][ni] = __builtin_amdgcn_smfmac_f32_16x16x128_bf8_fp8(av, bv, acc[mi][ni], fidx[mi & 1], 0, 0); \
          else acc[mi][ni] = __builtin_amdgcn_smfmac_f32_16x16x128_fp8_fp8(av, bv, acc[mi][ni], fidx[mi & 1], 0, 0); \
        } else {                                                                                          \
          bf16x8 av;                                                                                      \
          bf16x16 bv;                                                                                     \
          __builtin_memcpy(&av, &fa[mi & 1], 16);                                                         \
          __builtin_memcpy(&bv, &BC[ni][0], 32);                                                          \
          acc[mi][ni] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(av, bv, acc[mi][ni], fidx[mi & 1], 0, 0); \
        }                                                                                                 \
      }                                                                                                   \
      __builtin_amdgcn_sched_barrier(0);                                                                  \
    }                                                                                                     \
    const int t_ = s0;                                                                                    \
    s0 = s1;                                                                                              \
    s1 = s2;                                                                                              \
    s2 = t_;                                                                                              \
  } while (0)

  int step = 0;
  for (; step + 1 < nsteps; step += 2) {
    WG_STEP(fb0, fb1);
    step++;
    WG_STEP(fb1, fb0);
    step--;
  }
  if (step < nsteps) WG_STEP(fb0, fb1);
#undef WG_STEP
#undef WG_READ_B
#undef WG_LOAD
  wait_vmcnt<0>();

  // epilogue: lane (j, q) register r of tile (mi, ni) is element (o + r, i)
  float* dst = out + (int64_t)z * split_stride;
#pragma unroll
  for (int mi = 0; mi < MI_; mi++)
#pragma unroll
    for (int ni = 0; ni < NI_; ni++) {
      int64_t o = o0 + 16 * MI_ * wm + 16 * mi + 4 * q;
      int64_t i = i0 + 16 * NI_ * wn + 16 * ni + j;
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

// ---------------------------------------------------------------------------------------------------------
// 3. out[o][i] = scale * sum_z ws[z][o][i]  (+ out[o][i]); z ascending: a fixed order.
__global__ void __launch_bounds__(256)
k_wgrad_reduce(const float* __restrict__ ws, int splits, int64_t O, int64_t I, float scale, int accumulate,
               float* __restrict__ dW, int64_t lddw) {
  int64_t n4 = O * (I / 4);
  for (int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x; c < n4; c += (int64_t)gridDim.x * 256) {
    int64_t row = c / (I / 4), col = (c - row * (I / 4)) * 4;
    f32x4 s0 = __builtin_nontemporal_load((const f32x4*)(ws + row * I + col));
    float4 s = make_float4(s0[0], s0[1], s0[2], s0[3]);
    for (int z = 1; z < splits; z++) {
      f32x4 v0 = __builtin_nontemporal_load((const f32x4*)(ws + (int64_t)z * O * I + row * I + col));
      float4 v = make_float4(v0[0], v0[1], v0[2], v0[3]);
      s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
    }
    float4* p = (float4*)(dW + row * lddw + col);
    float4 r = make_float4(s.x * scale, s.y * scale, s.z * scale, s.w * scale);
    if (accumulate) { float4 d = *p; r.x += d.x; r.y += d.y; r.z += d.z; r.w += d.w; }
    store_stream_b128(p, r);
  }
}

__global__ void __launch_bounds__(256)
k_zero_rows(float* __restrict__ dW, int64_t O, int64_t I, int64_t lddw) {
  int64_t n = O * I;
  for (int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x; c < n; c += (int64_t)gridDim.x * 256) {
    int64_t row = c / I, col = c - row * I;
    dW[row * lddw + col] = 0.0f;
  }
}

// ---------------------------------------------------------------------------------------------------------
// host: path choice, tile and split choice, workspace layout
struct WgradPlan {
  bool packed;          // true: estimator pre-pass + GEMM on the packed operand; false: fused kernel
  int mi, ni;           // MFMA tiles per wave of the packed GEMM (workgroup tile 32 mi x 64 ni)
  int splits;           // token-axis splits
  int steps_per_split;
  size_t vals_bytes, meta_bytes, partial_bytes;   // workspace sections (each a multiple of 256)
};

static size_t round256(size_t x) { return (x + 255) / 256 * 256; }

// Time model (microseconds) behind the tile / split choice of the packed GEMM, fitted to timings of the
// 3072 x 768 (8192 tokens) and 5120 x 1280 (16384 tokens) layers.  One workgroup per CU; a k-step costs
// about 0.34 + 0.0175 per MFMA tile of the wave (0.90 for 8 x 4, 0.66 for 6 x 3), a workgroup about 4 us
// of ramp-up and drain, and the split partials are written once and read once at 5.5 TB/s.  The model
// only has to rank a handful of candidates; it is within 10 % of the measurements it was fitted to.
static double wgrad_model_us(int64_t O, int64_t I, int64_t steps, int mi, int ni, int64_t s, int64_t* sps_out) {
  int64_t bm = 32 * mi, bn = 64 * ni;
  int64_t tiles = ((O + bm - 1) / bm) * ((I + bn - 1) / bn);
  int64_t sps = (steps + s - 1) / s;
  int64_t splits = (steps + sps - 1) / sps;
  int64_t rounds = (tiles * splits + NUM_CU - 1) / NUM_CU;
  double t_step = 0.34 + 0.0175 * mi * ni;
  double t = (double)rounds * ((double)sps * t_step + 4.0);
  double out_bytes = (double)O * (double)I * 4.0;
  if (splits > 1) t += 2.0 + (double)(2 * splits + 1) * out_bytes / 5.5e6;
  *sps_out = sps;
  return t;
}

// Tile shape / split count forced by sste_wgrad_plan_override (0 = automatic choice).
static std::atomic<int> g_force_mi{0}, g_force_ni{0}, g_force_splits{0};

bool wgrad_plan_override(int mi, int ni, int splits) {
  const bool shape_ok = (mi == 0 && ni == 0) || (mi == 8 && ni == 4) || (mi == 6 && ni == 3) || (mi == 8 && ni == 3);
  if (!shape_ok || splits < 0 || splits > 32) return false;
  g_force_mi = mi;
  g_force_ni = ni;
  g_force_splits = splits;
  return true;
}

static WgradPlan wgrad_plan(int64_t T, int64_t O, int64_t I, int dtype) {
  WgradPlan p{};
  bool fp8 = dtype != SSTE_BF16;
  int ks = fp8 ? 128 : 64;
  int64_t steps = T / ks;
  // the pre-pass pays off once the GEMM tiles would re-derive each group several times and the problem
  // is large enough to fill the chip; everything else runs the fused kernel
  p.packed = (T >= 2048) && (O >= 256) && (I >= 256) && !product_reaches(T, O / 16 * 16 + 16, 1ll << 40);
  p.mi = 8;
  p.ni = 4;
  if (steps <= 0) {
    p.splits = 1;
    p.steps_per_split = 1;
    return p;
  }
  if (p.packed) {
    static const int shapes[3][2] = {{8, 4}, {6, 3}, {8, 3}};
    const int fmi = g_force_mi, fni = g_force_ni, fs = g_force_splits;
    double best = 1e30;
    for (int k = 0; k < 3; k++) {
      if (fmi && (shapes[k][0] != fmi || shapes[k][1] != fni)) continue;
      int64_t smax = steps / 8 < 32 ? steps / 8 : 32;
      if (smax < 1) smax = 1;
      for (int64_t s = 1; s <= smax; s++) {
        if (fs && s != (fs < smax ? fs : smax)) continue;
        int64_t sps;
        double t = wgrad_model_us(O, I, steps, shapes[k][0], shapes[k][1], s, &sps);
        if (t < best) {
          best = t;
          p.mi = shapes[k][0];
          p.ni = shapes[k][1];
          p.steps_per_split = (int)sps;
          p.splits = (int)((steps + sps - 1) / sps);
        }
      }
    }
    int64_t rows = (O + 15) / 16 * 16;
    p.vals_bytes = round256((size_t)rows * (size_t)(T / 2) * (fp8 ? 1 : 2));
    p.meta_bytes = round256((size_t)rows * (size_t)(T / 8));
  } else {
    int64_t tiles = ((O + 127) / 128) * ((I + 127) / 128);
    int64_t s = (2 * NUM_CU + tiles - 1) / tiles;
    if (s > steps / 8) s = steps / 8;
    if (s > 32) s = 32;
    if (s < 1) s = 1;
    int64_t sps = (steps + s - 1) / s;
    p.splits = (int)((steps + sps - 1) / sps);                // no empty split
    p.steps_per_split = (int)sps;
  }
  p.partial_bytes = p.splits > 1 ? round256((size_t)p.splits * (size_t)O * (size_t)I * sizeof(float)) : 0;
  return p;
}

template <bool FP8, int MI_, int NI_, bool BF8>
static void launch_wgrad_gemm_cfg(const void* vals, const void* meta, int64_t O, int64_t steps, const void* X, int64_t I,
                                  int64_t ldx_bytes, int splits, int steps_per_split, float scale, int accumulate,
                                  float* out, int64_t ld_out, int64_t split_stride, hipStream_t s) {
  int m_tiles = (int)((O + 32 * MI_ - 1) / (32 * MI_)), n_tiles = (int)((I + 64 * NI_ - 1) / (64 * NI_));
  dim3 grid((unsigned)(m_tiles * n_tiles * splits)), block(512);
  // Tile order inside a split.  The workgroups of one XCD (an eighth of the grid, consecutive logical numbers)
  // share an L2: with channel tiles fastest they cover many channel tiles of few feature tiles, with feature
  // tiles fastest the other way round.  Each channel tile costs the XCD a slice of the packed operand
  // (0.5625 bytes per element), each feature tile a slice of X (1 byte per element): take the cheaper order
  // (measured 1...4 % on the layers where the choice differs from channel tiles fastest).
  const int per_xcd = (m_tiles * n_tiles * splits + 7) / 8;
  auto xcd_cost = [&](int fast, int slow, double fast_bytes, double slow_bytes) {
    const int nfast = per_xcd < fast ? per_xcd : fast;
    int nslow = (per_xcd + fast - 1) / fast;
    if (nslow > slow) nslow = slow;
    return nfast * fast_bytes + nslow * slow_bytes;
  };
  const double a_bytes = 32.0 * MI_ * 0.5625, x_bytes = 64.0 * NI_;
  int features_fastest = xcd_cost(n_tiles, m_tiles, x_bytes, a_bytes) < xcd_cost(m_tiles, n_tiles, a_bytes, x_bytes) ? 1 : 0;
  SSTE_LAUNCH(SSTE_K_WGRAD, (k_wgrad_gemm<FP8, MI_, NI_, BF8>), grid, block, s, (const uint8_t*)vals, (const uint8_t*)meta, O, steps,
              (const uint8_t*)X, I, ldx_bytes, steps_per_split, scale, accumulate, out, ld_out, split_stride, m_tiles, n_tiles,
              features_fastest);
}

static void launch_wgrad_gemm(bool fp8, bool bf8, int mi, int ni, const void* vals, const void* meta, int64_t O, int64_t steps,
                              const void* X, int64_t I, int64_t ldx_bytes, int splits, int steps_per_split, float scale,
                              int accumulate, float* out, int64_t ld_out, int64_t split_stride, hipStream_t s) {
#define WG_CASE(F, M, N, B)                                                                                    \
  if (fp8 == F && bf8 == B && mi == M && ni == N)                                                              \
    return launch_wgrad_gemm_cfg<F, M, N, B>(vals, meta, O, steps, X, I, ldx_bytes, splits, steps_per_split, scale, \
                                             accumulate, out, ld_out, split_stride, s)
  WG_CASE(false, 8, 4, false);
  WG_CASE(false, 6, 3, false);
  WG_CASE(false, 8, 3, false);
  WG_CASE(true, 8, 4, false);
  WG_CASE(true, 6, 3, false);
  WG_CASE(true, 8, 3, false);
  WG_CASE(true, 8, 4, true);
  WG_CASE(true, 6, 3, true);
  WG_CASE(true, 8, 3, true);
#undef WG_CASE
}

size_t wgrad_workspace_bytes(int64_t T, int64_t O, int64_t I, int dtype) {
  WgradPlan p = wgrad_plan(T, O, I, dtype);
  return p.vals_bytes + p.meta_bytes + p.partial_bytes;
}

bool linear_wgrad_supported(int64_t T, int64_t O, int64_t I, int64_t ldx, int dtype) {
  int64_t eb = dtype != SSTE_BF16 ? 1 : 2;
  if (product_reaches(O / 128 + 1, I / 128 + 1, 0x80000000ll / 32)) return false;
  if (product_reaches(T, O / 16 * 16 + 16, 1ll << 40)) return false;                            // the packed operand's size
  if (product_reaches(T, ldx, (1ll << 31) / eb)) return wgrad_plan(T, O, I, dtype).packed ? false : true;   // 32-bit offsets in the GEMM
  return true;
}

hipError_t launch_linear_wgrad(const void* dY, int64_t T, int64_t O, int64_t lddy, int dtype, const void* X,
                               int64_t I, int64_t ldx, float scale, RngKey key, float* dW, int64_t lddw,
                               int accumulate, void* ws, hipStream_t s) {
  if (O == 0 || I == 0) return hipSuccess;
  bool fp8 = dtype != SSTE_BF16;
  int ks = fp8 ? 128 : 64, eb = fp8 ? 1 : 2;
  int64_t steps = T / ks;
  if (steps == 0) {
    if (!accumulate) {
      int64_t blocks = (O * I + 255) / 256;
      if (blocks > 4096) blocks = 4096;
      hipLaunchKernelGGL(k_zero_rows, dim3((unsigned)blocks), dim3(256), 0, s, dW, O, I, lddw);
    }
    return hipGetLastError();
  }
  WgradPlan p = wgrad_plan(T, O, I, dtype);
  uint8_t* wsb = (uint8_t*)ws;
  float* partial = (float*)(wsb + p.vals_bytes + p.meta_bytes);
  float* out = p.splits > 1 ? partial : dW;
  int64_t ld_out = p.splits > 1 ? I : lddw;
  int64_t split_stride = p.splits > 1 ? O * I : 0;
  float k_scale = p.splits > 1 ? 1.0f : scale;
  int k_acc = p.splits > 1 ? 0 : accumulate;
  if (p.packed) {
    uint8_t* vals = wsb;
    uint8_t* meta = wsb + p.vals_bytes;
    launch_mvue_pack(dY, T, O, lddy, dtype, key, vals, meta, s, SSTE_K_MVUE_PACK);
    launch_wgrad_gemm(fp8, dtype == SSTE_F8E5M2, p.mi, p.ni, vals, meta, O, steps, X, I, ldx * eb, p.splits, p.steps_per_split, k_scale, k_acc, out,
                      ld_out, split_stride, s);
  } else {
    hipError_t e = launch_wgrad_fused(dY, T, O, lddy, dtype, X, I, ldx, key, p.splits, p.steps_per_split, k_scale, k_acc,
                                      out, ld_out, split_stride, s);
    if (e != hipSuccess) return e;
  }
  if (p.splits > 1) {
    int64_t blocks = (O * (I / 4) + 255) / 256;
    if (blocks > 2048) blocks = 2048;
    SSTE_LAUNCH(SSTE_K_WGRAD_REDUCE, k_wgrad_reduce, dim3((unsigned)blocks), dim3(256), s, (const float*)partial, p.splits, O, I,
                scale, accumulate, dW, lddw);
  }
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------------------
// Scratch for callers that cannot allocate: the workspace of launch_linear_wgrad inside the library's own
// device image.  Every GPU the library runs on holds its own copy of the array until the process ends.  In
// host code the array's name is only a handle for the runtime; the device address is asked for once per
// device (with that device current) and used from then on.
static __device__ __align__(256) unsigned char scratch[SSTE_NOALLOC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};
}  // namespace

// Device address of this GPU's scratch array (nullptr + *err on failure).  No allocation takes place.
void* noalloc_scratch(hipError_t* err) {
  int dev = -1;
  *err = hipGetDevice(&dev);
  if (*err != hipSuccess) return nullptr;
  if (dev < 0 || dev >= kMaxDevices) {
    *err = hipErrorInvalidDevice;
    return nullptr;
  }
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    *err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (*err != hipSuccess) return nullptr;
    g_scratch_ptr[dev] = p;
  }
  return g_scratch_ptr[dev];
}

}  // namespace sste
