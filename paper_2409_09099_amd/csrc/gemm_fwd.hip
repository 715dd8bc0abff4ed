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
// Tiling: every wave owns a grid of 16 x 16 MFMA tiles (8 x 4 = 128 channels x 64 tokens in the main
// shape): per sparse MFMA it reads about 540 B of fragments from LDS, inside the LDS read rate of the CU.
// Three kernels share the operand layouts:
//   k_linear_fwd        the first, phase-structured kernel (fragment reads, then loads, then MFMAs);
//                       kept as 256 x 128 / 4 waves / 2-stage ring, two workgroups per CU, for layers
//                       with fewer than 128 tiles of 256 x 256, and as 128 x 64 / 1 wave for tiny ones;
//   k_linear_fwd_pipe   software-pipelined 256 x 256 tiles, 8 waves, one workgroup per CU (below);
//   k_linear_fwd_dual   the same tile code for 256 x 256 and 256 x 128 tiles in one grid, for layers
//                       whose last round of 256 x 256 tiles would fill at most half of the CUs.
// Operand tiles travel L2 -> LDS directly (buffer_load ... lds, no staging registers) into rings of
// LDS slots.  What limits all of them is the L1 of the CU: it keeps 64 line requests in flight, and a
// request takes 400 - 500 clocks under load, so a CU receives about 20 B/clk (measured; a 256 x 256
// k-step needs 50 KiB per 1024 MFMA clocks).
// The packed weight is stored in memory in the order the sparse MFMA consumes it (1 KiB blocks of
// 16 rows x one k-step, one 16-byte slot per lane), so its loads are contiguous and its fragment
// reads are lane-contiguous.  For X, whose 64 lanes of a load land on consecutive LDS addresses, bank
// conflicts are avoided by choosing WHICH 16-byte piece each lane fetches: piece c of row r is stored
// at position c ^ ((r / 2) % 8), which makes every fragment read (16 rows x one piece) hit 16
// different 16-byte bank groups.
// The loads are written in inline assembly: the compiler otherwise orders every later LDS read
// behind ALL outstanding LDS-writing loads, which would drain the ring each k-step.  Their
// completion is tracked by hand with s_waitcnt vmcnt(n) + a workgroup barrier.
// The epilogue transposes the accumulators through LDS so that each lane stores 16 contiguous bytes
// and each wave writes whole 256-byte rows of Z.
// Workgroups are numbered so that each XCD (the chip routes consecutive workgroup ids to its 8 XCDs
// in turn) works on a contiguous range of tiles, o-tiles fastest: the packed weight stays in that
// XCD's L2 and an X tile is fetched from HBM once per XCD.
#include "common.h"

namespace sste {

namespace {
constexpr int MI = 8, NI = 4;                     // MFMA tiles per wave: 128 channels x 64 tokens
constexpr int EPI_ROW = 272;                      // 128 channels x 2 B + 16 B pad
constexpr int NUM_CU = 256;

}  // namespace

// Output side of the forward GEMMs.  z8 == nullptr: Z is bf16, value = acc * scale.  Otherwise Z is e4m3
// with its own per-tensor scale folded into `scale` by the host (Sec. 5.2: the output of an FP8 layer is
// rescaled per tensor and cast; the consumer multiplies by z_scale again).  amax_bits, if given,
// receives max |acc| * amax_scale over the whole tensor (float32 bits; non-negative floats order like
// their patterns): one atomic per workgroup, skipped when it cannot raise the value.
struct FwdOut {
  uint16_t* z16;          // bf16 output (ZF8 = false); with `act`: the pre-activation H, may then be null
  uint8_t* z8;            // e4m3 output (ZF8 = true)
  int64_t ldz;            // leading dimension in elements
  float scale;            // acc -> stored value (before rounding)
  float amax_scale;       // acc -> the tensor's real units
  uint32_t* amax_bits;    // nullable
  // activation fused into the bf16 epilogue (kernels instantiated with ZF8 = false, AMAX = false):
  // H = RNE_bf16(acc * scale) goes to z16 (if given), A = GELU(H) to a16 (bf16) or a8 (e4m3 of A * a_inv_scale);
  // with a8 the largest |A| goes to amax_bits.
  int act;                // 0: none
  uint16_t* a16;
  uint8_t* a8;
  int64_t lda;
  float a_inv_scale;
};

// Activation stage of the epilogue on one 16-byte piece (8 consecutive channels of one token): stores A in
// the requested format and returns max |A| of the piece (float32 bits).
__device__ __forceinline__ uint32_t fwd_act_piece(const uint4& h, const FwdOut& out, int64_t t, int64_t o) {
  const uint32_t w[4] = {h.x, h.y, h.z, h.w};
  float a[8];
  uint32_t m = 0;
#pragma unroll
  for (int e = 0; e < 4; e++) {
    a[2 * e] = gelu_tanh(bf16lo_f32(w[e]));
    a[2 * e + 1] = gelu_tanh(bf16hi_f32(w[e]));
    m = max(m, max(f2u(a[2 * e]) & 0x7FFFFFFFu, f2u(a[2 * e + 1]) & 0x7FFFFFFFu));
  }
  if (out.a8) {
    const float r = out.a_inv_scale;
    int lo = __builtin_amdgcn_cvt_pk_fp8_f32(clamp448(a[0] * r), clamp448(a[1] * r), 0, false);
    lo = __builtin_amdgcn_cvt_pk_fp8_f32(clamp448(a[2] * r), clamp448(a[3] * r), lo, true);
    int hi = __builtin_amdgcn_cvt_pk_fp8_f32(clamp448(a[4] * r), clamp448(a[5] * r), 0, false);
    hi = __builtin_amdgcn_cvt_pk_fp8_f32(clamp448(a[6] * r), clamp448(a[7] * r), hi, true);
    i32x2 v = {lo, hi};
    __builtin_nontemporal_store(v, (i32x2*)(out.a8 + t * out.lda + o));
  } else {
    uint4 v = make_uint4(bf16_rne_pack(a[0], a[1]), bf16_rne_pack(a[2], a[3]), bf16_rne_pack(a[4], a[5]), bf16_rne_pack(a[6], a[7]));
    store_stream_b128(out.a16 + t * out.lda + o, v);
  }
  return m;
}

// max |acc| of the calling workgroup (NW waves) -> *amax_bits.  `red` is NW dwords of LDS nobody else uses
// between the two barriers.
template <int NW>
__device__ __forceinline__ void publish_tile_amax(uint32_t m, float amax_scale, uint32_t* __restrict__ amax_bits, uint32_t* red) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) m = max(m, (uint32_t)__shfl_xor((int)m, off, 64));
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
#pragma unroll
    for (int w = 1; w < NW; w++) m = max(m, red[w]);
    const uint32_t v = f2u(u2f(m) * amax_scale);
    if (v > __hip_atomic_load(amax_bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(amax_bits, v);
  }
  __syncthreads();
}

__global__ void k_fill_u32_fwd(uint32_t* p, uint32_t v) { *p = v; }

template <bool FP8, int WM, int WN, int NS, bool ZF8, bool AMAX>
__global__ void __launch_bounds__(64 * WM * WN, (WM * WN <= 4 && NS <= 2) ? 2 : 1)
k_linear_fwd(const uint8_t* __restrict__ X, int64_t T, int64_t k_bytes, int64_t ldx_bytes,
             const uint8_t* __restrict__ vals, const uint8_t* __restrict__ meta,
             int64_t O, FwdOut out, int m_tiles) {
  const float scale = out.scale;
  uint16_t* __restrict__ Z = out.z16;
  const int64_t ldz = out.ldz;
  constexpr int NW = WM * WN;
  constexpr int BM = 128 * WM, BN = 64 * WN;
  constexpr int MB = FP8 ? 16 : 8;                // position bytes per row and k-step
  constexpr int MBLK = 16 * MB;                   // ... per 16-row block
  constexpr int A_BYTES = BM * 64, B_BYTES = BN * 128, M_BYTES = BM * MB;
  constexpr int STAGE = A_BYTES + B_BYTES + M_BYTES;
  constexpr int EPI_BYTES = NW * 64 * EPI_ROW;
  constexpr int SMEM = NS * STAGE > EPI_BYTES ? NS * STAGE : EPI_BYTES;
  constexpr int LA = BM / 16 / NW, LB = BN / 8 / NW, LM = M_BYTES / 256 / NW;   // loads per wave and stage
  constexpr int LPW = LA + LB + LM;
  static_assert(LA >= 1 && LB >= 1 && LM >= 1, "tile too small for this many waves");
  __shared__ __align__(1024) uint8_t smem[SMEM];

  // XCD-aware tile order: XCD x owns a contiguous range of logical tiles
  const int logical = xcd_contiguous(blockIdx.x, gridDim.x);
  const int tm = logical % m_tiles, tn = logical / m_tiles;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN, wn = wave % WN;
  const int j = lane & 15, q = lane >> 4;
  const int64_t o0 = (int64_t)tm * BM, t0 = (int64_t)tn * BN;
  const int nsteps = (int)(k_bytes / 128);

  // buffer descriptors over exactly the valid part of this tile: what lies past the end reads as zeros
  const int64_t rblk0 = o0 / 16, rbn = (O + 15) / 16;
  const int blks_a = (int)((rbn - rblk0) < BM / 16 ? (rbn - rblk0) : BM / 16);
  const int rows_b = (int)((T - t0) < BN ? (T - t0) : BN);
  const i32x4 ba = rsrc_words(vals + rblk0 * nsteps * 1024, (uint32_t)(blks_a * nsteps * 1024));
  const i32x4 bm = rsrc_words(meta + rblk0 * nsteps * MBLK, (uint32_t)(blks_a * nsteps * MBLK));
  const i32x4 bb = rsrc_words(X + t0 * ldx_bytes, (uint32_t)((rows_b - 1) * ldx_bytes + k_bytes));

  // per-lane source offsets of the direct-to-LDS loads (destination = stage base + load index * 1 KiB
  // (256 B for the position bits) + lane * 16 (4), fixed by the hardware)
  uint32_t offa[LA], offb[LB], offm[LM];
#pragma unroll
  for (int i = 0; i < LA; i++) offa[i] = (uint32_t)((LA * wave + i) * nsteps * 1024 + lane * 16);
#pragma unroll
  for (int i = 0; i < LB; i++) {
    int wl = LB * wave + i;
    int r = 8 * wl + (lane >> 3), c = (lane & 7) ^ ((r >> 1) & 7);
    offb[i] = (uint32_t)(r * ldx_bytes + c * 16);
  }
#pragma unroll
  for (int i = 0; i < LM; i++) {
    int d = 64 * (LM * wave + i) + lane;          // dword index inside the stage's position bits
    offm[i] = (uint32_t)((d / (MBLK / 4)) * nsteps * MBLK + 4 * (d % (MBLK / 4)));
  }
  const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_u8*)smem;

  // loads of k-step `step` into ring slot `stg`; past the last k-step the scalar offset is pushed out
  // of range so that the same number of loads is always in flight (they fetch nothing)
#define FWD_ISSUE(step, stg)                                                                           \
  do {                                                                                                 \
    const bool live_ = (step) < nsteps;                                                                \
    const uint32_t sa_ = live_ ? (uint32_t)(step) * 1024u : 0x40000000u;                                 \
    const uint32_t sb_ = live_ ? (uint32_t)(step) * 128u : 0x40000000u;                                \
    const uint32_t sm_ = live_ ? (uint32_t)(step) * (uint32_t)MBLK : 0x40000000u;                        \
    const uint32_t base_ = lds0 + (uint32_t)(stg) * STAGE;                                             \
    _Pragma("unroll") for (int i = 0; i < LA; i++) dma_b128(ba, base_ + (LA * wave + i) * 1024, offa[i], sa_); \
    _Pragma("unroll") for (int i = 0; i < LB; i++) dma_b128(bb, base_ + A_BYTES + (LB * wave + i) * 1024, offb[i], sb_); \
    _Pragma("unroll") for (int i = 0; i < LM; i++) dma_b32(bm, base_ + A_BYTES + B_BYTES + (LM * wave + i) * 256, offm[i], sm_); \
  } while (0)

  f32x4 acc[MI][NI];
#pragma unroll
  for (int a = 0; a < MI; a++)
#pragma unroll
    for (int b = 0; b < NI; b++) acc[a][b] = (f32x4){0.f, 0.f, 0.f, 0.f};

  // per-lane fragment addresses inside a stage
  const uint32_t fa_off = (uint32_t)(8 * wm * 1024 + lane * 16);          // + 1024 mi
  const uint32_t fm_off = (uint32_t)(A_BYTES + B_BYTES + 8 * wm * MBLK + lane * (MB / 4));   // + MBLK mi
  const int rb0 = 64 * wn + j;                                           // + 16 ni
  const int cb0 = q ^ ((j >> 1) & 7);
  const uint32_t fb_off0 = (uint32_t)(A_BYTES + rb0 * 128 + cb0 * 16);
  const uint32_t fb_off1 = (uint32_t)(A_BYTES + rb0 * 128 + (cb0 ^ 4) * 16);

#pragma unroll
  for (int s = 0; s < NS - 1; s++) FWD_ISSUE(s, s);

  int stg = 0;
  for (int step = 0; step < nsteps; step++) {
    wait_vmcnt<(NS - 2) * LPW>();        // this wave's share of k-step `step` has landed in LDS
    __syncthreads();                     // ... and everybody else's; slot (step - 1) % NS is free again
    const uint8_t* sb = smem + stg * STAGE;
    uint4 fb[NI][2];
#pragma unroll
    for (int ni = 0; ni < NI; ni++) {
      fb[ni][0] = *(const uint4*)(sb + fb_off0 + ni * 2048);
      fb[ni][1] = *(const uint4*)(sb + fb_off1 + ni * 2048);
    }
    uint4 fa[MI];
    int fidx[MI];
#pragma unroll
    for (int mi = 0; mi < MI; mi++) {
      fa[mi] = *(const uint4*)(sb + fa_off + mi * 1024);
      if (FP8) fidx[mi] = *(const int*)(sb + fm_off + mi * MBLK);
      else fidx[mi] = *(const uint16_t*)(sb + fm_off + mi * MBLK);
    }
    {
      int nstg = stg + NS - 1;
      if (nstg >= NS) nstg -= NS;
      FWD_ISSUE(step + NS - 1, nstg);
    }
#pragma unroll
    for (int mi = 0; mi < MI; mi++) {
#pragma unroll
      for (int ni = 0; ni < NI; ni++) {
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
    }
    stg = (stg + 1 == NS) ? 0 : stg + 1;
  }
#undef FWD_ISSUE

  // epilogue: accumulators -> LDS (row = token, the wave's 128 channels contiguous) -> 16-byte stores
  wait_vmcnt<0>();
  __syncthreads();
  if (AMAX) {
    // float maxima of magnitudes: the absolute value is a free source modifier and two values go into one
    // three-operand maximum (the accumulators are finite)
    float mf = 0.0f;
#pragma unroll
    for (int mi = 0; mi < MI; mi++)
#pragma unroll
      for (int ni = 0; ni < NI; ni++)
#pragma unroll
        for (int r = 0; r < 4; r++) mf = __builtin_fmaxf(mf, __builtin_fabsf(acc[mi][ni][r]));
    publish_tile_amax<NW>(f2u(mf), out.amax_scale, out.amax_bits, (uint32_t*)smem);
  }
  uint8_t* eb = smem + wave * (64 * EPI_ROW);
  if (ZF8) {
    // e4m3 output: a lane's four values of a tile are four consecutive channels = one dword
#pragma unroll
    for (int mi = 0; mi < MI; mi++)
#pragma unroll
      for (int ni = 0; ni < NI; ni++) {
        int w = __builtin_amdgcn_cvt_pk_fp8_f32(clamp448(acc[mi][ni][0] * scale), clamp448(acc[mi][ni][1] * scale), 0, false);
        w = __builtin_amdgcn_cvt_pk_fp8_f32(clamp448(acc[mi][ni][2] * scale), clamp448(acc[mi][ni][3] * scale), w, true);
        *(int*)(eb + (16 * ni + j) * EPI_ROW + 16 * mi + 4 * q) = w;
      }
#pragma unroll
    for (int it = 0; it < 8; it++) {
      int row = 8 * it + (lane >> 3), chunk = lane & 7;
      uint4 v = *(const uint4*)(eb + row * EPI_ROW + chunk * 16);
      int64_t t = t0 + 64 * wn + row, o = o0 + 128 * wm + 16 * chunk;
      if (t < T && o < O) store_stream_b128(out.z8 + t * ldz + o, v);
    }
    return;
  }
#pragma unroll
  for (int mi = 0; mi < MI; mi++)
#pragma unroll
    for (int ni = 0; ni < NI; ni++) {
      uint2 v;
      v.x = bf16_rne_pack(acc[mi][ni][0] * scale, acc[mi][ni][1] * scale);
      v.y = bf16_rne_pack(acc[mi][ni][2] * scale, acc[mi][ni][3] * scale);
      *(uint2*)(eb + (16 * ni + j) * EPI_ROW + (16 * mi + 4 * q) * 2) = v;
    }
  // same-wave LDS accesses are ordered; no barrier needed for a wave-private region
  uint32_t act_max = 0;
#pragma unroll
  for (int it = 0; it < 16; it++) {
    int row = 4 * it + (lane >> 4), chunk = lane & 15;
    uint4 v = *(const uint4*)(eb + row * EPI_ROW + chunk * 16);
    int64_t t = t0 + 64 * wn + row, o = o0 + 128 * wm + 8 * chunk;
    if (t < T && o < O) {
      if (Z) store_stream_b128(Z + t * ldz + o, v);
      if (out.act) act_max = max(act_max, fwd_act_piece(v, out, t, o));
    }
  }
  if (out.act && out.amax_bits) {           // uniform over the workgroup
    __syncthreads();                        // every wave is done with its part of the LDS
    publish_tile_amax<NW>(act_max, 1.0f, out.amax_bits, (uint32_t*)smem);
  }
}

// ---------------------------------------------------------------------------------------------------------
// Software-pipelined variant: 8 waves (2 x 4), each owning MI_ x NI_ MFMA tiles, so a workgroup covers
// 32 MI_ channels x 64 NI_ tokens (256 x 256, 192 x 256, ...).  The kernel above alternates,
// workgroup-wide, between a phase that reads fragments from LDS and a phase that issues MFMAs; here the
// three pipes (vector memory, LDS, matrix) run side by side within a k-step:
//   * X fragments are double-buffered in registers: while the MFMAs of k-step s run on one set, the
//     set for k-step s + 1 is read from LDS, spread over the groups of NI_ MFMAs;
//   * packed-weight fragments roll through a two-deep register buffer, one row block ahead of its use;
//   * the direct-to-LDS loads of a k-step are spread over the groups instead of issued in one burst.
// Weight and X tiles live in separate three-slot rings because their LDS lifetimes differ: X of
// k-step s is consumed during k-step s - 1, the weight tile of k-step s during s - 1 (row block 0)
// and s.  At the single barrier of k-step s the tiles of s + 1 must have landed; the loads issued
// during s are the weight tile of s + 2 and the X tile of s + 3.
// Every wave issues the same number of loads per k-step (the counts in s_waitcnt are compile-time
// constants); where the tile has fewer 1 KiB blocks than 8 waves x loads, the surplus loads address
// blocks past the end of the tile's buffer descriptor and fetch nothing.

// LDS bytes one tile of the pipelined kernel needs (rings, reused by the epilogue)
template <bool FP8, int MI_, int NI_>
constexpr int fwd_pipe_smem() {
  constexpr int NW = 8, NR = 3, MB = FP8 ? 16 : 8;
  constexpr int LA = (32 * MI_ / 16 + NW - 1) / NW, LM = (32 * MI_ * MB / 256 + NW - 1) / NW;
  constexpr int RING = NR * (NW * LA * 1024 + NW * LM * 256 + 64 * NI_ * 128);
  constexpr int EPI = NW * 16 * NI_ * (32 * MI_ + 16);
  return RING > EPI ? RING : EPI;
}

// One output tile: channels [o0, o0 + 32 MI_) x tokens [t0, t0 + 64 NI_).  `smem` is the workgroup's LDS.
template <bool FP8, int MI_, int NI_, bool ZF8, bool AMAX>
__device__ __forceinline__ void fwd_pipe_tile(uint8_t* smem, const uint8_t* __restrict__ X, int64_t T, int64_t k_bytes,
                                              int64_t ldx_bytes, const uint8_t* __restrict__ vals,
                                              const uint8_t* __restrict__ meta, int64_t O, const FwdOut& out,
                                              int64_t o0, int64_t t0) {
  const float scale = out.scale;
  uint16_t* __restrict__ Z = out.z16;
  const int64_t ldz = out.ldz;
  constexpr int WN = 4, NW = 8, BM = 32 * MI_, BN = 64 * NI_, NR = 3;
  constexpr int MB = FP8 ? 16 : 8, MBLK = 16 * MB;
  constexpr int LA = (BM / 16 + NW - 1) / NW;                    // weight blocks (1 KiB) per wave and k-step
  constexpr int LM = (BM * MB / 256 + NW - 1) / NW;              // 256-byte pieces of position bits
  constexpr int LB = NI_;                                        // 8-token slabs (1 KiB) of X
  constexpr int A_BYTES = NW * LA * 1024, M_BYTES = NW * LM * 256;
  constexpr int ASTAGE = A_BYTES + M_BYTES, BSTAGE = BN * 128;
  // epilogue row: the wave's channels + pad; bf16 rows of the 256-channel tile are XOR-swizzled instead of padded
  constexpr int EROW = (MI_ == 8 && !ZF8) ? 256 : 32 * MI_ + 16;
  constexpr int NLOAD = LA + LM + LB;                            // issue order inside a k-step: A.., M.., B..
  constexpr int NPIECE = 2 * NI_;                                // 16-byte pieces of the next X fragments
  static_assert(NR * (ASTAGE + BSTAGE) <= fwd_pipe_smem<FP8, MI_, NI_>() && NW * 16 * NI_ * EROW <= fwd_pipe_smem<FP8, MI_, NI_>(),
                "LDS size helper out of step with the tile layout");
  uint8_t* const smemA = smem;
  uint8_t* const smemB = smem + NR * ASTAGE;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN, wn = wave % WN;
  const int j = lane & 15, q = lane >> 4;
  const int nsteps = (int)(k_bytes / 128);

  const int64_t rblk0 = o0 / 16, rbn = (O + 15) / 16;
  const int blks_a = (int)((rbn - rblk0) < BM / 16 ? (rbn - rblk0) : BM / 16);
  const int rows_b = (int)((T - t0) < BN ? (T - t0) : BN);
  const i32x4 ba = rsrc_words(vals + rblk0 * nsteps * 1024, (uint32_t)(blks_a * nsteps * 1024));
  const i32x4 bm = rsrc_words(meta + rblk0 * nsteps * MBLK, (uint32_t)(blks_a * nsteps * MBLK));
  const i32x4 bb = rsrc_words(X + t0 * ldx_bytes, (uint32_t)((rows_b - 1) * ldx_bytes + k_bytes));

  uint32_t offa[LA], offb[LB], offm[LM];
#pragma unroll
  for (int i = 0; i < LA; i++) offa[i] = (uint32_t)((LA * wave + i) * nsteps * 1024 + lane * 16);
#pragma unroll
  for (int i = 0; i < LB; i++) {
    int wl = LB * wave + i;
    int r = 8 * wl + (lane >> 3), c = (lane & 7) ^ ((r >> 1) & 7);
    offb[i] = (uint32_t)(r * ldx_bytes + c * 16);
  }
#pragma unroll
  for (int i = 0; i < LM; i++) {
    int d = 64 * (LM * wave + i) + lane;
    offm[i] = (uint32_t)((d / (MBLK / 4)) * nsteps * MBLK + 4 * (d % (MBLK / 4)));
  }
  const uint32_t ldsA = (uint32_t)(uintptr_t)(lds_u8*)smemA;
  const uint32_t ldsB = (uint32_t)(uintptr_t)(lds_u8*)smemB;
  constexpr uint32_t DEAD = 0x40000000u;            // scalar offset past every descriptor: the load fetches nothing

  // load number n (0 .. NLOAD-1) of this wave for weight k-step sa -> slot slot_a, X k-step sb -> slot slot_b
#define PIPE_LOAD(n, sa, slot_a, sb, slot_b)                                                              \
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
               offb[(n) >= LA + LM ? (n) - LA - LM : 0], (sb) < nsteps ? (uint32_t)(sb) * 128u : DEAD);   \
  } while (0)

  f32x4 acc[MI_][NI_];
#pragma unroll
  for (int a = 0; a < MI_; a++)
#pragma unroll
    for (int b = 0; b < NI_; b++) acc[a][b] = (f32x4){0.f, 0.f, 0.f, 0.f};

  const uint32_t fa_off = (uint32_t)(MI_ * wm * 1024 + lane * 16);                  // + 1024 mi
  const uint32_t fm_off = (uint32_t)(A_BYTES + MI_ * wm * MBLK + lane * (MB / 4));  // + MBLK mi
  const int rb0 = 16 * NI_ * wn + j;                                                // + 16 ni
  const int cb0 = q ^ ((j >> 1) & 7);
  const uint32_t fb_off0 = (uint32_t)(rb0 * 128 + cb0 * 16);
  const uint32_t fb_off1 = (uint32_t)(rb0 * 128 + (cb0 ^ 4) * 16);

  // prologue: weight tiles 0, 1 and X tiles 0, 1, 2 in flight, in the order the barriers expect
#pragma unroll
  for (int n = 0; n < NLOAD; n++) PIPE_LOAD(n, 0, 0, 0, 0);
#pragma unroll
  for (int n = 0; n < NLOAD; n++) PIPE_LOAD(n, 1, 1, 1, 1);
#pragma unroll
  for (int n = LA + LM; n < NLOAD; n++) PIPE_LOAD(n, 0, 0, 2, 2);

  uint4 fb0[NI_][2], fb1[NI_][2];     // X fragments: current / next k-step, roles swap every k-step
  uint4 fa[2];                        // packed-weight fragment of row block mi in fa[mi % 2]
  int fidx[2];
  wait_vmcnt<LA + LM + 2 * LB>();     // tiles of k-step 0 have landed
  __syncthreads();
#pragma unroll
  for (int ni = 0; ni < NI_; ni++) {
    fb0[ni][0] = *(const uint4*)(smemB + fb_off0 + ni * 2048);
    fb0[ni][1] = *(const uint4*)(smemB + fb_off1 + ni * 2048);
  }
  fa[0] = *(const uint4*)(smemA + fa_off);
  if (FP8) fidx[0] = *(const int*)(smemA + fm_off);
  else fidx[0] = *(const uint16_t*)(smemA + fm_off);

  int s0 = 0, s1 = 1, s2 = 2;         // ring slots of k-steps step, step + 1, step + 2 (both rings)

  // one k-step: MFMAs on BC, next X fragments into BX
#define PIPE_STEP(BC, BX)                                                                                 \
  do {                                                                                                    \
    wait_vmcnt<LB>();                 /* all but the newest X tile: k-step step + 1 has landed */          \
    __syncthreads();                  /* ... for every wave; slots of step - 1 (weights) and step (X) are free */ \
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
        if (spread(pc, NPIECE, MI_) == mi)                                                                \
          BX[pc >> 1][pc & 1] = *(const uint4*)(pb1 + ((pc & 1) ? fb_off1 : fb_off0) + (pc >> 1) * 2048); \
      _Pragma("unroll") for (int n = 0; n < NLOAD; n++)                                                   \
        if (spread(n, NLOAD, MI_) == mi) PIPE_LOAD(n, step + 2, s2, step + 3, s0);                        \
      _Pragma("unroll") for (int ni = 0; ni < NI_; ni++) {                                                \
        if (FP8) {                                                                                        \
          i32x4 av;                                                                                       \
          i32x8 bv;                                                                                       \
          __builtin_memcpy(&av, &fa[mi & 1], 16);                                                         \
          __builtin_memcpy(&bv, &BC[ni][0], 32);                                                          \
          acc[mi][ni] = __builtin_amdgcn_smfmac_f32_16x16x128_fp8_fp8(av, bv, acc[mi][ni], fidx[mi & 1], 0, 0); \
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
    PIPE_STEP(fb0, fb1);
    step++;
    PIPE_STEP(fb1, fb0);
    step--;
  }
  if (step < nsteps) PIPE_STEP(fb0, fb1);
#undef PIPE_STEP
#undef PIPE_LOAD

  // epilogue: accumulators -> LDS (row = token, the wave's 16 MI_ channels contiguous) -> 16-byte stores
  wait_vmcnt<0>();
  __syncthreads();
  if (AMAX) {
    // float maxima of magnitudes: the absolute value is a free source modifier and two values go into one
    // three-operand maximum (the accumulators are finite)
    float mf = 0.0f;
#pragma unroll
    for (int mi = 0; mi < MI_; mi++)
#pragma unroll
      for (int ni = 0; ni < NI_; ni++)
#pragma unroll
        for (int r = 0; r < 4; r++) mf = __builtin_fmaxf(mf, __builtin_fabsf(acc[mi][ni][r]));
    publish_tile_amax<NW>(f2u(mf), out.amax_scale, out.amax_bits, (uint32_t*)smem);
  }
  uint8_t* eb = smem + wave * (16 * NI_ * EROW);
  if (ZF8) {
    // e4m3 output: a lane's four values of a tile are four consecutive channels = one dword; a token row of
    // the wave is 16 MI_ bytes
#pragma unroll
    for (int mi = 0; mi < MI_; mi++)
#pragma unroll
      for (int ni = 0; ni < NI_; ni++) {
        int w = __builtin_amdgcn_cvt_pk_fp8_f32(clamp448(acc[mi][ni][0] * scale), clamp448(acc[mi][ni][1] * scale), 0, false);
        w = __builtin_amdgcn_cvt_pk_fp8_f32(clamp448(acc[mi][ni][2] * scale), clamp448(acc[mi][ni][3] * scale), w, true);
        *(int*)(eb + (16 * ni + j) * EROW + 16 * mi + 4 * q) = w;
      }
    constexpr int CHUNKS8 = MI_;                                 // 16-byte chunks (16 channels) per token row
    constexpr int NCH8 = 16 * NI_ * CHUNKS8;
#pragma unroll
    for (int it = 0; it < (NCH8 + 63) / 64; it++) {
      int c = 64 * it + lane;
      if (c < NCH8) {
        int row = c / CHUNKS8, chunk = c % CHUNKS8;
        uint4 v = *(const uint4*)(eb + row * EROW + chunk * 16);
        int64_t t = t0 + 16 * NI_ * wn + row, o = o0 + 16 * MI_ * wm + 16 * chunk;
        if (t < T && o < O) store_stream_b128(out.z8 + t * ldz + o, v);
      }
    }
    return;
  }
#pragma unroll
  for (int mi = 0; mi < MI_; mi++)
#pragma unroll
    for (int ni = 0; ni < NI_; ni++) {
      uint2 v;
      v.x = bf16_rne_pack(acc[mi][ni][0] * scale, acc[mi][ni][1] * scale);
      v.y = bf16_rne_pack(acc[mi][ni][2] * scale, acc[mi][ni][3] * scale);
      // 16-byte chunk c of token row t sits at position c ^ (t % 16) (MI_ == 8: a row is 256 B = every bank once,
      // and the padding is not needed): the four-row reads below then run at the full LDS rate, where rows
      // shifted by the 16-byte pad cost half as much again (measured 567 vs 860 clocks per 128 KiB)
      if (MI_ == 8) *(uint2*)(eb + (16 * ni + j) * EROW + (((2 * mi + (q >> 1)) ^ j) * 16) + 8 * (q & 1)) = v;
      else *(uint2*)(eb + (16 * ni + j) * EROW + (16 * mi + 4 * q) * 2) = v;
    }
  // same-wave LDS accesses are ordered; no barrier needed for a wave-private region
  constexpr int CHUNKS = 2 * MI_;                                // 16-byte chunks per token row
  constexpr int NCH = 16 * NI_ * CHUNKS;
  uint32_t act_max = 0;
#pragma unroll
  for (int it = 0; it < (NCH + 63) / 64; it++) {
    int c = 64 * it + lane;
    if (c < NCH) {
      int row = c / CHUNKS, chunk = c % CHUNKS;
      uint4 v = *(const uint4*)(eb + row * EROW + (MI_ == 8 ? (chunk ^ (row & 15)) : chunk) * 16);
      int64_t t = t0 + 16 * NI_ * wn + row, o = o0 + 16 * MI_ * wm + 8 * chunk;
      if (t < T && o < O) {
        if (Z) store_stream_b128(Z + t * ldz + o, v);
        if (out.act) act_max = max(act_max, fwd_act_piece(v, out, t, o));
      }
    }
  }
  if (out.act && out.amax_bits) {           // uniform over the workgroup
    __syncthreads();                        // every wave is done with its part of the LDS
    publish_tile_amax<NW>(act_max, 1.0f, out.amax_bits, (uint32_t*)smem);
  }
}

// One tile shape for the whole grid.  Workgroups are numbered so that each XCD works on a contiguous
// range of tiles, o-tiles fastest.
template <bool FP8, int MI_, int NI_, bool ZF8, bool AMAX>
__global__ void __launch_bounds__(512, 1)
k_linear_fwd_pipe(const uint8_t* __restrict__ X, int64_t T, int64_t k_bytes, int64_t ldx_bytes,
                  const uint8_t* __restrict__ vals, const uint8_t* __restrict__ meta,
                  int64_t O, FwdOut out, int m_tiles) {
  __shared__ __align__(1024) uint8_t smem[fwd_pipe_smem<FP8, MI_, NI_>()];
  const int logical = xcd_contiguous(blockIdx.x, gridDim.x);
  const int tm = logical % m_tiles, tn = logical / m_tiles;
  fwd_pipe_tile<FP8, MI_, NI_, ZF8, AMAX>(smem, X, T, k_bytes, ldx_bytes, vals, meta, O, out, (int64_t)tm * (32 * MI_),
                                          (int64_t)tn * (64 * NI_));
}

// Two tile shapes in one grid, for layers whose 256 x 256 tiles fill the CUs a whole number of times plus
// a remainder of at most half a round: the first n_big workgroups take 256 x 256 tiles, the rest take
// the remaining tiles as 256 x 128 halves.  The last round then has twice as many, half as long
// workgroups instead of leaving more than half of the CUs idle for a full tile time.
template <bool FP8, bool ZF8, bool AMAX>
__global__ void __launch_bounds__(512, 1)
k_linear_fwd_dual(const uint8_t* __restrict__ X, int64_t T, int64_t k_bytes, int64_t ldx_bytes,
                  const uint8_t* __restrict__ vals, const uint8_t* __restrict__ meta,
                  int64_t O, FwdOut out, int m_tiles, int n_big) {
  __shared__ __align__(1024) uint8_t smem[fwd_pipe_smem<FP8, 8, 4>()];
  static_assert(fwd_pipe_smem<FP8, 8, 2>() <= fwd_pipe_smem<FP8, 8, 4>(), "the half tile fits in the full tile's LDS");
  const int bid = blockIdx.x;
  if (bid < n_big) {
    const int logical = xcd_contiguous(bid, n_big);
    const int tm = logical % m_tiles, tn = logical / m_tiles;
    fwd_pipe_tile<FP8, 8, 4, ZF8, AMAX>(smem, X, T, k_bytes, ldx_bytes, vals, meta, O, out, (int64_t)tm * 256, (int64_t)tn * 256);
  } else {
    const int h = xcd_contiguous(bid - n_big, (int)gridDim.x - n_big);      // half-tile number
    const int tile = n_big + (h >> 1);
    const int tm = tile % m_tiles, tn = tile / m_tiles;
    const int64_t t0 = (int64_t)tn * 256 + 128 * (h & 1);
    if (t0 >= T) return;                       // second half of a ragged last token tile: nothing to do
    fwd_pipe_tile<FP8, 8, 2, ZF8, AMAX>(smem, X, T, k_bytes, ldx_bytes, vals, meta, O, out, (int64_t)tm * 256, t0);
  }
}

template <bool FP8, int MI_, int NI_, bool ZF8, bool AMAX>
static void launch_fwd_pipe(const void* X, int64_t T, int64_t I, int64_t ldx, const FwdOut& out, const void* vals,
                            const void* meta, int64_t O, hipStream_t s) {
  constexpr int BM = 32 * MI_, BN = 64 * NI_;
  int m_tiles = (int)((O + BM - 1) / BM), n_tiles = (int)((T + BN - 1) / BN);
  dim3 grid((unsigned)(m_tiles * n_tiles)), block(512);
  int64_t eb = FP8 ? 1 : 2;
  SSTE_LAUNCH(SSTE_K_FWD, (k_linear_fwd_pipe<FP8, MI_, NI_, ZF8, AMAX>), grid, block, s, (const uint8_t*)X, T, I * eb, ldx * eb,
              (const uint8_t*)vals, (const uint8_t*)meta, O, out, m_tiles);
}

template <bool FP8, bool ZF8, bool AMAX>
static void launch_fwd_dual(const void* X, int64_t T, int64_t I, int64_t ldx, const FwdOut& out, const void* vals,
                            const void* meta, int64_t O, int n_big, hipStream_t s) {
  int m_tiles = (int)((O + 255) / 256), n_tiles = (int)((T + 255) / 256);
  int n_small = 2 * (m_tiles * n_tiles - n_big);
  dim3 grid((unsigned)(n_big + n_small)), block(512);
  int64_t eb = FP8 ? 1 : 2;
  SSTE_LAUNCH(SSTE_K_FWD, (k_linear_fwd_dual<FP8, ZF8, AMAX>), grid, block, s, (const uint8_t*)X, T, I * eb, ldx * eb,
              (const uint8_t*)vals, (const uint8_t*)meta, O, out, m_tiles, n_big);
}

template <bool FP8, int WM, int WN, int NS, bool ZF8, bool AMAX>
static void launch_fwd_cfg(const void* X, int64_t T, int64_t I, int64_t ldx, const FwdOut& out, const void* vals,
                           const void* meta, int64_t O, hipStream_t s) {
  constexpr int BM = 128 * WM, BN = 64 * WN;
  int m_tiles = (int)((O + BM - 1) / BM), n_tiles = (int)((T + BN - 1) / BN);
  dim3 grid((unsigned)(m_tiles * n_tiles)), block(64 * WM * WN);
  int64_t eb = FP8 ? 1 : 2;
  SSTE_LAUNCH(SSTE_K_FWD, (k_linear_fwd<FP8, WM, WN, NS, ZF8, AMAX>), grid, block, s, (const uint8_t*)X, T, I * eb, ldx * eb,
              (const uint8_t*)vals, (const uint8_t*)meta, O, out, m_tiles);
}

bool linear_fwd_supported(int64_t T, int64_t I, int64_t ldx, int64_t O, int dtype) {
  int64_t eb = dtype == SSTE_F8E4M3 ? 1 : 2;
  // 32-bit offsets inside a tile, 32-bit tile count
  if (product_reaches(ldx, 256 * eb, 1ll << 30) || product_reaches(I, 256 * eb, 1ll << 30)) return false;
  if (product_reaches(O / 256 + 1, T / 128 + 1, 0x80000000ll)) return false;
  return true;
}

// Kernel choice for one combination of operand type, output type and amax.
template <bool FP8, bool ZF8, bool AMAX>
static void launch_fwd_variant(const void* X, int64_t T, int64_t I, int64_t ldx, const FwdOut& out, const void* vals,
                               const void* meta, int64_t O, hipStream_t s) {
  // 256 x 256 tiles (8 waves, 3-stage ring) unless the problem has too few of them to occupy the chip;
  // measured faster than 256 x 128 even at 1.5 rounds of tiles (3072 x 8192 outputs: 33.6 vs 36.4 us)
  int64_t big_tiles = ((O + 255) / 256) * ((T + 255) / 256);
  int64_t rem = big_tiles % NUM_CU;
  if (big_tiles > NUM_CU && rem > 0 && rem <= NUM_CU / 2) {
    // whole rounds of 256 x 256 tiles, then the remainder as twice as many 256 x 128 tiles
    launch_fwd_dual<FP8, ZF8, AMAX>(X, T, I, ldx, out, vals, meta, O, (int)(big_tiles - rem), s);
  } else if (big_tiles >= 128) {
    launch_fwd_pipe<FP8, 8, 4, ZF8, AMAX>(X, T, I, ldx, out, vals, meta, O, s);
  } else if (((O + 255) / 256) * ((T + 127) / 128) < 32) {
    // tiny problems: 128 x 64 tiles by one wave each, eight times as many workgroups (512 x 256 outputs: 14.1 vs 17.3 us)
    launch_fwd_cfg<FP8, 1, 1, 2, ZF8, AMAX>(X, T, I, ldx, out, vals, meta, O, s);
  } else {
    launch_fwd_cfg<FP8, 2, 2, 2, ZF8, AMAX>(X, T, I, ldx, out, vals, meta, O, s);
  }
}

hipError_t launch_linear_fwd(const void* X, int64_t T, int64_t I, int64_t ldx, int dtype, float scale,
                             const void* vals, const void* meta, int64_t O, void* Z, int64_t ldz, int z_dtype,
                             float amax_scale, float* amax_out, hipStream_t s) {
  if (amax_out) hipLaunchKernelGGL(k_fill_u32_fwd, dim3(1), dim3(1), 0, s, (uint32_t*)amax_out, 0u);
  if (T == 0 || O == 0) return hipGetLastError();
  const bool fp8 = dtype == SSTE_F8E4M3, zf8 = z_dtype == SSTE_F8E4M3;
  FwdOut out;
  out.z16 = zf8 ? nullptr : (uint16_t*)Z;
  out.z8 = zf8 ? (uint8_t*)Z : nullptr;
  out.ldz = ldz;
  out.scale = scale;
  out.amax_scale = amax_scale;
  out.amax_bits = (uint32_t*)amax_out;
  out.act = 0;
  out.a16 = nullptr;
  out.a8 = nullptr;
  out.lda = 0;
  out.a_inv_scale = 1.0f;
  const bool amax = amax_out != nullptr;
#define FWD_CASE(F, Z8, A)                                                                \
  if (fp8 == F && zf8 == Z8 && amax == A) launch_fwd_variant<F, Z8, A>(X, T, I, ldx, out, vals, meta, O, s)
  FWD_CASE(false, false, false);
  FWD_CASE(false, false, true);
  FWD_CASE(false, true, true);          // an e4m3 output always comes with its largest magnitude (the API insists)
  FWD_CASE(true, false, false);
  FWD_CASE(true, false, true);
  FWD_CASE(true, true, true);
#undef FWD_CASE
  return hipGetLastError();
}

// Forward product with the activation in the epilogue: H = RNE_bf16(acc * scale) (stored if H != null),
// A = GELU(H) stored as bf16 or as e4m3 of A * a_inv_scale (then with the largest |A| in amax_out).
hipError_t launch_linear_fwd_act(const void* X, int64_t T, int64_t I, int64_t ldx, int dtype, float scale,
                                 const void* vals, const void* meta, int64_t O, void* H, int64_t ldh, void* A, int64_t lda,
                                 int a_dtype, float a_inv_scale, float* amax_out, hipStream_t s) {
  if (amax_out) hipLaunchKernelGGL(k_fill_u32_fwd, dim3(1), dim3(1), 0, s, (uint32_t*)amax_out, 0u);
  if (T == 0 || O == 0) return hipGetLastError();
  FwdOut out;
  out.z16 = (uint16_t*)H;
  out.z8 = nullptr;
  out.ldz = ldh;
  out.scale = scale;
  out.amax_scale = 1.0f;
  out.amax_bits = (uint32_t*)amax_out;
  out.act = 1;
  out.a16 = a_dtype == SSTE_F8E4M3 ? nullptr : (uint16_t*)A;
  out.a8 = a_dtype == SSTE_F8E4M3 ? (uint8_t*)A : nullptr;
  out.lda = lda;
  out.a_inv_scale = a_inv_scale;
  if (dtype == SSTE_F8E4M3) launch_fwd_variant<true, false, false>(X, T, I, ldx, out, vals, meta, O, s);
  else launch_fwd_variant<false, false, false>(X, T, I, ldx, out, vals, meta, O, s);
  return hipGetLastError();
}

}  // namespace sste
