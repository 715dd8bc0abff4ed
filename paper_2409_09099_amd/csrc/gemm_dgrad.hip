// Input gradient of the S-STE linear layer (paper Sec. 5.1): grad_X = grad_Z S(W).  The paper keeps this
// product dense (only grad_Z is sparsified, and only for the weight gradient), so it runs on the dense
// matrix instruction; what it shares with the forward pass is the packed weight, which is decoded to
// dense-with-zeros on its way into LDS instead of being kept a second time in memory.
//
// MFMA mapping: grad_X^T = S(W)^T grad_Z^T.  Rows = input features i, columns = tokens t, contraction
// k = output channels o.  v_mfma_f32_16x16x32_bf16: A lane (row i = lane % 16, q = lane / 16) holds
// k = 8q .. 8q+7, B lane (col j, q) the same k range of its column, D lane (j, q) register r is
// element (4q + r, j).  A 64-channel k-step takes two instructions per tile (k 0..31 and 32..63).
//   B operand = grad_Z tile: token rows with 64 channels (128 B) contiguous -- the same tile, swizzle
//     and 16-byte fragment reads as X in the forward GEMM; direct-to-LDS loads into a two-slot ring.
//   A operand = S(W) tile: 64 channels x 256 features.  Each wave loads two 1 KiB blocks of packed
//     values plus their position bits into registers, expands every group of four (two values, two
//     2-bit positions -> four bf16) and writes dense rows [channel][feature] into a three-slot LDS
//     ring, in the layout and swizzle the weight-gradient GEMM uses for X (512-byte rows, 32-byte
//     feature pair p of row r at position p ^ x_swizzle(r), see common.h; here the two 16-byte halves
//     of a pair also swap places in rows with bit 2 set, which spreads the expansion's 16-byte writes
//     over all banks).  The contraction index is strided there, so the fragments are read with the
//     transposing LDS load (ds_read_b64_tr_b16).
// Pipeline per k-step s: wait for everything issued during s - 1 (grad_Z tile s + 1 in LDS, packed
// blocks s + 2 in registers), barrier, decode blocks s + 2 into LDS, then eight groups of MFMAs during
// which the grad_Z fragments of s + 1 are read (register double buffer), the S(W) fragments roll one
// row block ahead, the grad_Z tile s + 2 is requested and, last, the packed blocks s + 3 are loaded.
// Loads get one k-step (about 2000 clocks here) to complete; that keeps the LDS at exactly 160 KiB.
// Epilogue as in the forward GEMM: transposed through LDS, 16-byte streaming stores of bf16 rows.
//
// e4m3 operands (per-tensor scales, Sec. 5.2): the same kernel with 128 channels per k-step, so that a
// grad_Z row of the tile is again 128 bytes and both LDS rings keep their size.  One
// v_mfma_f32_16x16x128_f8f6f4 per tile and k-step; the only layout requirement of that instruction
// used here is that byte e of lane (., q) of both operands is the same channel.  The decoded tile has
// 256-byte channel rows of 16-byte feature chunks (chunk c of row r at position c ^ x_swizzle(r)), read
// with ds_read_b64_tr_b8; a group expands with one byte permute.
#include "common.h"

namespace sste {

namespace {
typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;
typedef __attribute__((address_space(3))) i32x2 lds_i32x2;

// One group of a packed 2:4 operand -> its four dense bf16: w = value0 | value1 << 16 (ascending
// positions), nib = pos0 | pos1 << 2 with pos0 < pos1.  lo holds positions 0, 1; hi positions 2, 3.
__device__ __forceinline__ void expand_group(uint32_t w, uint32_t nib, uint32_t& lo, uint32_t& hi) {
  // each value shifted to its 16-bit position inside the 64-bit group: two 64-bit shifts and an OR
  // (a third of the instructions of per-position selects)
  const uint64_t d = ((uint64_t)(w & 0xFFFFu) << ((nib & 3u) << 4)) | ((uint64_t)(w >> 16) << ((nib & 12u) << 2));
  lo = (uint32_t)d;
  hi = (uint32_t)(d >> 32);
}

// The same for e4m3 values: w holds value0 at byte b0 and value1 at byte b0 + 1; the result is the four
// dense bytes of the group.  A byte permute with a computed selector: selector bytes 0..3 pick from the
// zero operand, 4..7 from w.
__device__ __forceinline__ uint32_t expand_group8(uint32_t w, uint32_t b0, uint32_t nib) {
  const uint32_t sel = ((4u + b0) << (((nib & 3u) << 3) & 31u)) | ((5u + b0) << (((nib & 12u) << 1) & 31u));
  return __builtin_amdgcn_perm(w, 0u, sel);
}
}  // namespace

template <bool FP8, int NI_>
constexpr int dgrad_smem() {
  return 3 * (FP8 ? 128 : 64) * 256 * (FP8 ? 1 : 2) + 2 * 64 * NI_ * 128;
}

// One tile: features [256 tm, 256 tm + 256) x tokens [t0, t0 + 64 NI_), by a 512-thread workgroup.
template <bool FP8, int NI_, bool BF8>
__device__ __forceinline__ void dgrad_tile(uint8_t* smem, const uint8_t* __restrict__ dY, int64_t T, int64_t O,
                                           int64_t lddy_bytes, const uint8_t* __restrict__ vals,
                                           const uint8_t* __restrict__ meta, int64_t I, int isteps, float scale,
                                           uint16_t* __restrict__ dX, int64_t lddx, int tm, int64_t t0,
                                           const uint16_t* __restrict__ H, int64_t ldh) {
  constexpr int WN = 4, NW = 8, MI_ = 8;
  constexpr int EB = FP8 ? 1 : 2;
  constexpr int KC = FP8 ? 128 : 64;                // channels per k-step (128 bytes of a grad_Z row)
  constexpr int RBK = KC / 16;                      // packed row blocks per k-step
  constexpr int CST = FP8 ? 2 : 4;                  // packed column steps per 256 features
  constexpr int MBLK = FP8 ? 256 : 128;             // metadata bytes per packed block
  constexpr int BM = 256, BN = 64 * NI_;            // features x tokens per workgroup (256 x 256 or 256 x 128)
  constexpr int AROW = BM * EB;                     // bytes of one channel row of the decoded tile
  constexpr int ASLOT = KC * AROW;                  // decoded S(W): KC channels x 256 features
  constexpr int BSLOT = BN * 128;                   // grad_Z: BN tokens x KC channels
  constexpr int NRA = 3, NRB = 2;
  constexpr int LB = BSLOT / 1024 / NW;             // direct-to-LDS loads per wave and k-step: 4 / 2
  constexpr int EROW = 32 * MI_ + 16;
  constexpr int NPIECE = 2 * NI_;
  static_assert(NRA * ASLOT + NRB * BSLOT == dgrad_smem<FP8, NI_>(), "LDS size");
  static_assert(NRA * ASLOT + NRB * BSLOT <= 160 * 1024 && NW * 16 * NI_ * EROW <= NRA * ASLOT + NRB * BSLOT, "LDS budget");
  uint8_t* const smemA = smem;
  uint8_t* const smemB = smem + NRA * ASLOT;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN, wn = wave % WN;
  const int j = lane & 15, q = lane >> 4;
  const int64_t i0 = (int64_t)tm * BM;
  const int nsteps = (int)((O + KC - 1) / KC);
  const int64_t rbn = (O + 15) / 16;

  // grad_Z tile: exactly the valid rows and channels; what lies outside reads as zeros
  const int rows_b = (int)((T - t0) < BN ? (T - t0) : BN);
  const i32x4 bb = rsrc_words(dY + t0 * lddy_bytes, (uint32_t)((rows_b - 1) * lddy_bytes + O * EB));
  uint32_t offb[LB];
#pragma unroll
  for (int i = 0; i < LB; i++) {
    int wl = LB * wave + i;
    int r = 8 * wl + (lane >> 3), c = (lane & 7) ^ ((r >> 1) & 7);
    offb[i] = (uint32_t)(r * lddy_bytes + c * 16);
  }
  const uint32_t ldsB = (uint32_t)(uintptr_t)(lds_u8*)smemB;
  constexpr uint32_t DEAD = 0x40000000u;

  // packed S(W): this wave's two blocks of a k-step are (row block RBK s + rbl, column step CST tm + csl)
  const BufferRsrc rv = make_rsrc(vals, (uint32_t)(rbn * isteps * 1024));
  const BufferRsrc rm = make_rsrc(meta, (uint32_t)(rbn * isteps * MBLK));
  uint32_t pv_off[2], pm_off[2], dec_off[2];
#pragma unroll
  for (int e = 0; e < 2; e++) {
    const int blkid = 2 * wave + e, rbl = blkid / CST, csl = blkid % CST;
    const int cs = CST * tm + csl;
    const bool live = cs < isteps;                  // column steps past the last feature: nothing to fetch
    pv_off[e] = live ? (uint32_t)((rbl * isteps + cs) * 1024 + lane * 16) : 0x80000000u;
    pm_off[e] = live ? (uint32_t)((rbl * isteps + cs) * MBLK + lane * (MBLK / 64)) : 0x80000000u;
    // the lane's 32 dense bytes: bf16 one 32-byte feature pair, e4m3 two 16-byte chunks (second at ^ 16)
    const int row = 16 * rbl + j, p = FP8 ? 8 * csl + 2 * q : 4 * csl + q;
    // bf16: the two 16-byte halves of the pair swap places in rows with bit 2 set, so that the 16 lanes
    // (16 consecutive rows) of one write cover all sixteen 16-byte bank groups
    dec_off[e] = FP8 ? (uint32_t)(row * AROW + ((p ^ x_swizzle<true>(row)) * 16))
                     : (uint32_t)(row * AROW + ((p ^ x_swizzle<false>(row)) * 32) + 16 * ((row >> 2) & 1));
  }
  uint4 pk[2], pk2[2];                // packed blocks in flight / being expanded (second set: 256 x 128 tile only)
  uint32_t pmeta[2], pmeta2[2];
  uint32_t dec[8];                    // one block row being expanded: 16 dense bf16
#define DG_LOAD_PACKED(step, PK, PM)                                                                            \
  do {                                                                                                    \
    const uint32_t sv_ = (uint32_t)(step) * (uint32_t)RBK * (uint32_t)isteps * 1024u;                     \
    const uint32_t sm_ = (uint32_t)(step) * (uint32_t)RBK * (uint32_t)isteps * (uint32_t)MBLK;            \
    _Pragma("unroll") for (int e = 0; e < 2; e++) {                                                       \
      /* row blocks past the last one (tail of the channel axis, k-steps past the end) fetch nothing */    \
      const bool live_ = RBK * (int64_t)(step) + ((2 * wave + e) / CST) < rbn;                            \
      PK[e] = buffer_load_b128(rv, live_ ? pv_off[e] : 0x80000000u, live_ ? sv_ : 0u);                    \
      if (FP8)                                                                                            \
        PM[e] = (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(rm, (int)(live_ ? pm_off[e] : 0x80000000u), \
                                                               (int)(live_ ? sm_ : 0u), 0);               \
      else                                                                                                \
        PM[e] = (uint32_t)(uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rm, (int)(live_ ? pm_off[e] : 0x80000000u), \
                                                                           (int)(live_ ? sm_ : 0u), 0);  \
    }                                                                                                     \
  } while (0)
// expansion of quarter g of block e (one bf16 group / two e4m3 groups: eight dense bytes) into the
// staging registers; after the fourth quarter the 32 bytes are written
#define DG_DECODE_PIECE(slot_, e, g, PK, PM)                                                                    \
  do {                                                                                                    \
    const uint32_t w_ = (g) == 0 ? PK[e].x : (g) == 1 ? PK[e].y : (g) == 2 ? PK[e].z : PK[e].w;           \
    if (FP8) {                                                                                            \
      dec[2 * (g)] = expand_group8(w_, 0u, (PM[e] >> (8 * (g))) & 15u);                                   \
      dec[2 * (g) + 1] = expand_group8(w_, 2u, (PM[e] >> (8 * (g) + 4)) & 15u);                           \
    } else {                                                                                              \
      expand_group(w_, (PM[e] >> (4 * (g))) & 15u, dec[2 * (g)], dec[2 * (g) + 1]);                       \
    }                                                                                                     \
    if ((g) == 3) {                                                                                       \
      uint8_t* dst_ = smemA + (slot_) * ASLOT + dec_off[e];                                               \
      uint8_t* dst2_ = smemA + (slot_) * ASLOT + (dec_off[e] ^ 16u);                                      \
      *(uint4*)dst_ = make_uint4(dec[0], dec[1], dec[2], dec[3]);                                         \
      *(uint4*)dst2_ = make_uint4(dec[4], dec[5], dec[6], dec[7]);                                        \
    }                                                                                                     \
  } while (0)
#define DG_DECODE(slot_, PK, PM)                                                                             \
  do {                                                                                                    \
    _Pragma("unroll") for (int d_ = 0; d_ < 8; d_++) DG_DECODE_PIECE(slot_, d_ >> 2, d_ & 3, PK, PM);     \
  } while (0)
#define DG_DMA_B(i, step, slot_)                                                                          \
  dma_b128(bb, ldsB + (uint32_t)(slot_) * BSLOT + (LB * wave + (i)) * 1024, offb[i],                      \
           (step) < nsteps ? (uint32_t)(step) * 128u : DEAD)

  f32x4 acc[MI_][NI_];
#pragma unroll
  for (int a = 0; a < MI_; a++)
#pragma unroll
    for (int b = 0; b < NI_; b++) acc[a][b] = (f32x4){0.f, 0.f, 0.f, 0.f};

  // fragment addresses.  S(W): transposing reads, piece r covers channels 8q + 4 (r & 1) + 32 (r >> 1) .. + 3
  // of the 16 features of row block mi; the feature pair index 8 wm + mi enters through the XOR below
  // (mi only touches the low three bits of the pair position).
  // e4m3: piece r covers channels 16q + 8 (r & 1) + 64 (r >> 1) .. + 7 of the 16 features of chunk 8 wm + mi.
  uint32_t fa_off[4];
#pragma unroll
  for (int r = 0; r < 4; r++) {
    if (FP8) {
      int row = 16 * q + 8 * (r & 1) + 64 * (r >> 1) + (j >> 1);
      fa_off[r] = (uint32_t)(row * AROW + (((8 * wm) ^ x_swizzle<true>(row)) * 16) + 8 * (j & 1));
    } else {
      int row = 8 * q + 4 * (r & 1) + 32 * (r >> 1) + (j >> 2);
      fa_off[r] = (uint32_t)(row * AROW + (((8 * wm) ^ x_swizzle<false>(row)) * 32) + ((((j & 3) >> 1) ^ ((row >> 2) & 1)) * 16) + 8 * (j & 1));
    }
  }
  const int rb0 = 16 * NI_ * wn + j;
  const int cb0 = q ^ ((j >> 1) & 7);
  const uint32_t fb_off0 = (uint32_t)(rb0 * 128 + cb0 * 16);
  const uint32_t fb_off1 = (uint32_t)(rb0 * 128 + (cb0 ^ 4) * 16);

#define DG_READ_A(dst, base, mi_)                                                                         \
  do {                                                                                                    \
    _Pragma("unroll") for (int r = 0; r < 4; r++) {                                                       \
      /* e4m3 256 x 256 tile: the offset is made opaque so that the 32 swizzled addresses of a k-step   */ \
      /* are formed where they are used (one XOR each); kept in registers across the loop they spill    */ \
      uint32_t o_ = fa_off[r];                                                                            \
      if (FP8 && NI_ == 4) asm volatile("" : "+v"(o_));                                                   \
      if (FP8) {                                                                                          \
        i32x2 t_ = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_i32x2*)((base) + (o_ ^ (uint32_t)((mi_) * 16)))); \
        dst[r] = make_uint2((uint32_t)t_[0], (uint32_t)t_[1]);                                            \
      } else {                                                                                            \
        bf16x4 t_ = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)((base) + (o_ ^ (uint32_t)((mi_) * 32)))); \
        __builtin_memcpy(&dst[r], &t_, 8);                                                                \
      }                                                                                                   \
    }                                                                                                     \
  } while (0)

  // prologue: grad_Z tiles 0 and 1 requested, S(W) tiles 0 and 1 decoded, packed blocks of k-step 2 in registers
#pragma unroll
  for (int i = 0; i < LB; i++) DG_DMA_B(i, 0, 0);
#pragma unroll
  for (int i = 0; i < LB; i++) DG_DMA_B(i, 1, 1);
  DG_LOAD_PACKED(0, pk, pmeta);
  DG_DECODE(0, pk, pmeta);
  DG_LOAD_PACKED(1, pk, pmeta);
  DG_DECODE(1, pk, pmeta);
  DG_LOAD_PACKED(2, pk, pmeta);

  uint4 fb0[NI_][2], fb1[NI_][2];     // grad_Z fragments: current / next k-step
  // S(W) fragments roll AD row blocks ahead of their use (two where registers allow: the 256 x 128 tile
  // issues only four MFMAs per group, too few to cover an LDS round trip); block mi lives in fa[mi % AB]
  constexpr int AD = NI_ == 2 ? 2 : 1, AB = 2 * AD;
  uint2 fa[AB][4];
  wait_vmcnt<0>();
  __syncthreads();
#pragma unroll
  for (int ni = 0; ni < NI_; ni++) {
    fb0[ni][0] = *(const uint4*)(smemB + fb_off0 + ni * 2048);
    fb0[ni][1] = *(const uint4*)(smemB + fb_off1 + ni * 2048);
  }
#pragma unroll
  for (int b = 0; b < AD; b++) DG_READ_A(fa[b], smemA, b);

  int a0 = 0, a1 = 1, a2 = 2;         // S(W) ring slots of k-steps step, step + 1, step + 2
  int b1 = 1;                         // grad_Z ring slot of k-step step + 1 (step + 2 goes to the other one)

#define DG_STEP(BC, BX, PKC, PMC, PKN, PMN)                                                                                 \
  do {                                                                                                    \
    wait_vmcnt<0>();                  /* everything issued during the previous k-step has arrived */      \
    __syncthreads();                  /* ... for every wave; S(W) slot a2 and grad_Z slot 1 - b1 are free */ \
    /* the 256 x 256 tile has no registers to spare for an expansion in flight across the MFMA groups */ \
    if (NI_ == 4) DG_DECODE(a2, PKC, PMC);                                                                \
    const uint8_t* pa = smemA + a0 * ASLOT;                                                               \
    const uint8_t* pa1 = smemA + a1 * ASLOT;                                                              \
    const uint8_t* pb1 = smemB + b1 * BSLOT;                                                              \
    _Pragma("unroll") for (int mi = 0; mi < MI_; mi++) {                                                  \
      if (NI_ != 4) DG_DECODE_PIECE(a2, mi >> 2, mi & 3, PKC, PMC);   /* blocks of k-step step + 2 -> dense, a group per MFMA group */ \
      /* next packed blocks: into the second register set at once (256 x 128), or into the same one    */ \
      /* at the end of the k-step (256 x 256: a load in flight across the groups would spill)           */ \
      if (NI_ != 4 && mi == 0) DG_LOAD_PACKED(step + 3, PKN, PMN);                                        \
      if (NI_ == 4 && mi == MI_ - 1) DG_LOAD_PACKED(step + 3, PKC, PMC);                                  \
      if (mi + AD < MI_) DG_READ_A(fa[(mi + AD) & (AB - 1)], pa, mi + AD);                                \
      else DG_READ_A(fa[(mi + AD) & (AB - 1)], pa1, mi + AD - MI_);                                       \
      _Pragma("unroll") for (int pc = 0; pc < NPIECE; pc++)                                               \
        if (spread(pc, NPIECE, MI_) == mi)                                                                \
          BX[pc >> 1][pc & 1] = *(const uint4*)(pb1 + ((pc & 1) ? fb_off1 : fb_off0) + (pc >> 1) * 2048); \
      _Pragma("unroll") for (int n = 0; n < LB; n++)                                                      \
        if (n == mi) DG_DMA_B(n, step + 2, 1 - b1);                                                       \
      _Pragma("unroll") for (int ni = 0; ni < NI_; ni++) {                                                \
        if (FP8) {                                                                                        \
          /* one 128-channel instruction; byte e of both operands is the same channel (16q + e, then    */ \
          /* 64 + 16q + e - 16), zero scale arguments select the unscaled form                          */ \
          i32x8 av, bv;                                                                                   \
          __builtin_memcpy(&av, &fa[mi & (AB - 1)][0], 32);                                               \
          __builtin_memcpy(&bv, &BC[ni][0], 32);                                                          \
          /* format arguments: A (expanded weight) e4m3; B (grad_Z) e4m3, or e5m2 when BF8              */ \
          acc[mi][ni] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(av, bv, acc[mi][ni], 0, BF8 ? 1 : 0, 0, 0, 0, 0); \
        } else {                                                                                          \
          bf16x8 av0, av1, bv0, bv1;                                                                      \
          __builtin_memcpy(&av0, &fa[mi & (AB - 1)][0], 16);                                              \
          __builtin_memcpy(&av1, &fa[mi & (AB - 1)][2], 16);                                              \
          __builtin_memcpy(&bv0, &BC[ni][0], 16);                                                         \
          __builtin_memcpy(&bv1, &BC[ni][1], 16);                                                         \
          acc[mi][ni] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av0, bv0, acc[mi][ni], 0, 0, 0);          \
          acc[mi][ni] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av1, bv1, acc[mi][ni], 0, 0, 0);          \
        }                                                                                                 \
      }                                                                                                   \
      __builtin_amdgcn_sched_barrier(0);                                                                  \
    }                                                                                                     \
    const int t_ = a0;                                                                                    \
    a0 = a1;                                                                                              \
    a1 = a2;                                                                                              \
    a2 = t_;                                                                                              \
    b1 = 1 - b1;                                                                                          \
  } while (0)

  int step = 0;
  for (; step + 1 < nsteps; step += 2) {
    if (NI_ == 4) {
      DG_STEP(fb0, fb1, pk, pmeta, pk, pmeta);
      step++;
      DG_STEP(fb1, fb0, pk, pmeta, pk, pmeta);
      step--;
    } else {
      DG_STEP(fb0, fb1, pk, pmeta, pk2, pmeta2);
      step++;
      DG_STEP(fb1, fb0, pk2, pmeta2, pk, pmeta);
      step--;
    }
  }
  if (step < nsteps) {
    if (NI_ == 4) DG_STEP(fb0, fb1, pk, pmeta, pk, pmeta);
    else DG_STEP(fb0, fb1, pk, pmeta, pk2, pmeta2);
  }
#undef DG_STEP
#undef DG_READ_A
#undef DG_DMA_B
#undef DG_DECODE
#undef DG_DECODE_PIECE
#undef DG_LOAD_PACKED

  // epilogue: accumulators -> LDS (row = token, the wave's 128 features contiguous) -> 16-byte stores
  wait_vmcnt<0>();
  __syncthreads();
  uint8_t* eb = smem + wave * (16 * NI_ * EROW);
#pragma unroll
  for (int mi = 0; mi < MI_; mi++)
#pragma unroll
    for (int ni = 0; ni < NI_; ni++) {
      uint2 v;
      v.x = bf16_rne_pack(acc[mi][ni][0] * scale, acc[mi][ni][1] * scale);
      v.y = bf16_rne_pack(acc[mi][ni][2] * scale, acc[mi][ni][3] * scale);
      *(uint2*)(eb + (16 * ni + j) * EROW + (16 * mi + 4 * q) * 2) = v;
    }
  constexpr int CHUNKS = 2 * MI_, NCH = 16 * NI_ * CHUNKS;
#pragma unroll
  for (int it = 0; it < (NCH + 63) / 64; it++) {
    int c = 64 * it + lane;
    if (c < NCH) {
      int row = c / CHUNKS, chunk = c % CHUNKS;
      uint4 v = *(const uint4*)(eb + row * EROW + chunk * 16);
      int64_t t = t0 + 16 * NI_ * wn + row, i = i0 + 16 * MI_ * wm + 8 * chunk;
      if (t < T && i < I) {
        if (H) {
          // backward of the activation that produced this layer's input: grad_H = grad_A * GELU'(H), on the
          // bf16 gradient just formed and the stored pre-activation (read once: streaming load)
          const i32x4 hv = __builtin_nontemporal_load((const i32x4*)(H + t * ldh + i));
          const uint32_t g[4] = {v.x, v.y, v.z, v.w};
          uint32_t r[4];
#pragma unroll
          for (int e = 0; e < 4; e++) {
            const uint32_t hw = (uint32_t)hv[e];
            r[e] = bf16_rne_pack(bf16lo_f32(g[e]) * gelu_tanh_grad(bf16lo_f32(hw)), bf16hi_f32(g[e]) * gelu_tanh_grad(bf16hi_f32(hw)));
          }
          v = make_uint4(r[0], r[1], r[2], r[3]);
        }
        store_stream_b128(dX + t * lddx + i, v);
      }
    }
  }
}

template <bool FP8, int NI_, bool BF8>
__global__ void __launch_bounds__(512, 1)
k_linear_dgrad(const uint8_t* __restrict__ dY, int64_t T, int64_t O, int64_t lddy_bytes,
               const uint8_t* __restrict__ vals, const uint8_t* __restrict__ meta, int64_t I, int isteps,
               float scale, uint16_t* __restrict__ dX, int64_t lddx, int m_tiles, const uint16_t* __restrict__ H, int64_t ldh) {
  __shared__ __align__(1024) uint8_t smem[dgrad_smem<FP8, NI_>()];
  const int logical = xcd_contiguous(blockIdx.x, gridDim.x);
  const int tm = logical % m_tiles, tn = logical / m_tiles;
  dgrad_tile<FP8, NI_, BF8>(smem, dY, T, O, lddy_bytes, vals, meta, I, isteps, scale, dX, lddx, tm, (int64_t)tn * (64 * NI_), H, ldh);
}

// Whole rounds of 256 x 256 tiles (workgroups 0 .. n_big - 1), then the tiles of the last, partial round
// as twice as many 256 x 128 tiles, so that the round takes half a tile time on twice the CUs.
template <bool FP8, bool BF8>
__global__ void __launch_bounds__(512, 1)
k_linear_dgrad_dual(const uint8_t* __restrict__ dY, int64_t T, int64_t O, int64_t lddy_bytes,
                    const uint8_t* __restrict__ vals, const uint8_t* __restrict__ meta, int64_t I, int isteps,
                    float scale, uint16_t* __restrict__ dX, int64_t lddx, int m_tiles, int n_big, const uint16_t* __restrict__ H,
                    int64_t ldh) {
  __shared__ __align__(1024) uint8_t smem[dgrad_smem<FP8, 4>()];
  const int bid = blockIdx.x;
  if (bid < n_big) {
    const int logical = xcd_contiguous(bid, n_big);
    dgrad_tile<FP8, 4, BF8>(smem, dY, T, O, lddy_bytes, vals, meta, I, isteps, scale, dX, lddx, logical % m_tiles,
                       (int64_t)(logical / m_tiles) * 256, H, ldh);
  } else {
    const int h = xcd_contiguous(bid - n_big, (int)gridDim.x - n_big);      // half-tile number
    const int tile = n_big + (h >> 1);
    const int64_t t0 = (int64_t)(tile / m_tiles) * 256 + 128 * (h & 1);
    if (t0 >= T) return;                       // second half of a ragged last token tile: nothing to do
    dgrad_tile<FP8, 2, BF8>(smem, dY, T, O, lddy_bytes, vals, meta, I, isteps, scale, dX, lddx, tile % m_tiles, t0, H, ldh);
  }
}

bool linear_dgrad_supported(int64_t T, int64_t O, int64_t lddy, int64_t I, int dtype) {
  const int eb = dtype != SSTE_BF16 ? 1 : 2;
  if (product_reaches(lddy, 256 * eb, 1ll << 30)) return false;           // 32-bit offsets inside a grad_Z tile
  if (product_reaches(O / 16 * 16 + 16, I, 1ll << 31)) return false;      // packed operand addressed with 32-bit offsets
  if (product_reaches(I / 256 + 1, T / 128 + 1, 0x80000000ll)) return false;
  return true;
}

hipError_t launch_linear_dgrad(const void* dY, int64_t T, int64_t O, int64_t lddy, int dtype, float scale, const void* vals,
                               const void* meta, int64_t I, void* dX, int64_t lddx, const void* H, int64_t ldh, hipStream_t s) {
  if (T == 0 || I == 0) return hipSuccess;
  const uint16_t* hp = (const uint16_t*)H;
  const bool fp8 = dtype != SSTE_BF16, bf8 = dtype == SSTE_F8E5M2;
  int m_tiles = (int)((I + 255) / 256);
  // 256 x 256 tiles unless they leave a quarter or more of the CUs without work in the only round
  int64_t big = (int64_t)m_tiles * ((T + 255) / 256);
  int64_t rem = big % 256;
  const uint8_t* dy = (const uint8_t*)dY;
  const uint8_t* pv = (const uint8_t*)vals;
  const uint8_t* pm = (const uint8_t*)meta;
  const int isteps = (int)(I / (fp8 ? 128 : 64));
  const int64_t lddy_bytes = lddy * (fp8 ? 1 : 2);
  if (big > 256 && rem > 0 && rem <= 128) {
    int n_big = (int)(big - rem);
    dim3 grid((unsigned)(n_big + 2 * rem)), block(512);
#define DG_DUAL(F8, B8)                                                                                                \
  SSTE_LAUNCH(SSTE_K_DGRAD, (k_linear_dgrad_dual<F8, B8>), grid, block, s, dy, T, O, lddy_bytes, pv, pm, I, isteps, scale, \
              (uint16_t*)dX, lddx, m_tiles, n_big, hp, ldh)
    if (bf8) DG_DUAL(true, true);
    else if (fp8) DG_DUAL(true, false);
    else DG_DUAL(false, false);
#undef DG_DUAL
    return hipGetLastError();
  }
  bool half = big < 192;
  int n_tiles = (int)((T + (half ? 127 : 255)) / (half ? 128 : 256));
  dim3 grid((unsigned)(m_tiles * n_tiles)), block(512);
#define DG_CASE(F8, NI, B8)                                                                                            \
  SSTE_LAUNCH(SSTE_K_DGRAD, (k_linear_dgrad<F8, NI, B8>), grid, block, s, dy, T, O, lddy_bytes, pv, pm, I, isteps, scale, \
              (uint16_t*)dX, lddx, m_tiles, hp, ldh)
  if (bf8 && half) DG_CASE(true, 2, true);
  else if (bf8) DG_CASE(true, 4, true);
  else if (fp8 && half) DG_CASE(true, 2, false);
  else if (fp8) DG_CASE(true, 4, false);
  else if (half) DG_CASE(false, 2, false);
  else DG_CASE(false, 4, false);
#undef DG_CASE
  return hipGetLastError();
}

}  // namespace sste
