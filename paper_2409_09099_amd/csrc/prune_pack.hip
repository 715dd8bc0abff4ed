// S(W) = beta * S_soft(W): 2:4 soft-threshold projection (paper Sec. 4.1), frozen scale (Sec. 4.2)
// and packing into values + 2-bit position metadata, in one streaming pass over W.
// Also: the same pass fused with the dense-weight step of Eq. (7), the MSE-optimal beta reduction of
// Sec. 4.2 and the flip count of Sec. 3.3.
//
// Data movement per weight: 2 B read, 1 B (bf16 values) or 0.5 B (e4m3 values) + 0.125 B written.
// The kernel is bound by HBM bandwidth.
#include "common.h"

namespace sste {

struct Proj {
  float p0, p1;   // beta * (a -/+ t) of the two recorded elements, ascending position order
  uint32_t nib;   // pos0 | pos1 << 2
};

// One group {hi:lo} of four bf16.  Order: magnitude field descending, then index ascending.
// GAMMA: the threshold interpolated between the third-largest magnitude m3 (gamma = 0, the method) and the
// second-largest m2 (gamma = 1), the ablation of Sec. 4.1 "Choosing optimal threshold":
// t = m3 + gamma * (m2 - m3), three float32 operations.
template <bool GAMMA = false>
__device__ __forceinline__ Proj project_group(uint32_t lo, uint32_t hi, float beta, float gamma = 0.0f) {
  // key = magnitude << 2 | (3 - index): a larger key ranks first, keys are distinct
  uint32_t k0 = ((lo & 0x7FFFu) << 2) | 3u;
  uint32_t k1 = ((lo >> 14) & 0x1FFFCu) | 2u;
  uint32_t k2 = ((hi & 0x7FFFu) << 2) | 1u;
  uint32_t k3 = ((hi >> 14) & 0x1FFFCu);
  // partial sorting network on four distinct keys.  {first, x} partition {a, c} and {y, w} partition
  // {b, d}; the runner-up is the better of x (loser of the two pair winners) and y (best pair loser),
  // and the third is the better of the two keys that are left.
  uint32_t a = max(k0, k1), b = min(k0, k1), c = max(k2, k3), d = min(k2, k3);
  uint32_t first = max(a, c), x = min(a, c);
  uint32_t y = max(b, d), w = min(b, d);
  uint32_t second = max(x, y), z = min(x, y);
  uint32_t third = max(z, w);
  uint32_t pa = 3u - (first & 3u), pb = 3u - (second & 3u);
  uint32_t pos0 = min(pa, pb), pos1 = max(pa, pb);
  uint32_t tbits = (third >> 2) << 16;              // float32 pattern of t (>= 0)
  if (GAMMA) {
    const float m3 = u2f(tbits), m2 = u2f((second >> 2) << 16);
    const float span = m2 - m3;
    const float part = gamma * span;
    tbits = f2u(m3 + part) & 0x7FFFFFFFu;
  }
  Proj r;
  uint32_t g0 = pick16_as_f32bits(lo, hi, pos0), g1 = pick16_as_f32bits(lo, hi, pos1);
  float sd0 = u2f(g0) - u2f(tbits | (g0 & 0x80000000u));    // a - t  or  a + t
  float sd1 = u2f(g1) - u2f(tbits | (g1 & 0x80000000u));
  r.p0 = sd0 * beta;
  r.p1 = sd1 * beta;
  r.nib = pos0 | (pos1 << 2);
  return r;
}

// One wave produces one 16-row x one-column-step block of the packed operand in the blocked layout
// described in include/sste.h: lane (j = lane % 16, q = lane / 16) reads the 16 (bf16 values) or 32
// (e4m3 values) weights of row 16 rb + j that feed slot q of the sparse matrix instruction, and
// writes its 16 bytes of values to position lane of the 1 KiB block and its position bits to
// position lane of the metadata block.  A wave therefore writes 1 KiB + 128 (256) B contiguously
// and reads whole 128-byte (256-byte) row segments.
//
// Block `blk` (row block rb = blk / steps, column step s = blk % steps) of one tensor, by one wave.
// Returns the largest |p| this lane recorded (only computed when AMAX).
// The lane's weights (bf16 pairs, w[2g] and w[2g+1] = group g) -> its slot of block `blk`.
// STREAM: the packed values are written with the streaming hint.  Right for the whole-model launches, whose
// output (hundreds of MB) is not read back before it has left the caches anyway (measured 0.394 -> 0.380 ms
// for the 144 tensors of the 774M model); wrong for a single layer, whose GEMM reads the operand next.
template <bool FP8, bool AMAX, bool GAMMA = false, bool STREAM = false>
__device__ __forceinline__ float project_store(const uint32_t (&w)[FP8 ? 16 : 8], int64_t blk, float beta,
                                               float val_scale, uint4* __restrict__ vals, void* __restrict__ meta,
                                               int lane, float gamma = 0.0f) {
  constexpr int NG = FP8 ? 8 : 4;                       // groups per lane
  float amax = 0.0f;
  float p[2 * NG];
  uint32_t nibs = 0;
#pragma unroll
  for (int g = 0; g < NG; g++) {
    Proj r = project_group<GAMMA>(w[2 * g], w[2 * g + 1], beta, gamma);
    p[2 * g] = r.p0;
    p[2 * g + 1] = r.p1;
    nibs |= r.nib << (4 * g);
    if (AMAX) amax = fmaxf(amax, fmaxf(fabsf(r.p0), fabsf(r.p1)));
  }
  uint4 out;
  if (FP8) {
    uint32_t o[4];
#pragma unroll
    for (int c = 0; c < 4; c++) {
      uint32_t lo = e4m3_rne_pack(clamp448(p[4 * c] / val_scale), clamp448(p[4 * c + 1] / val_scale));
      uint32_t hi = e4m3_rne_pack(clamp448(p[4 * c + 2] / val_scale), clamp448(p[4 * c + 3] / val_scale));
      o[c] = lo | (hi << 16);
    }
    out = make_uint4(o[0], o[1], o[2], o[3]);
    ((uint32_t*)meta)[blk * 64 + lane] = nibs;
  } else {
    out = make_uint4(bf16_rne_pack(p[0], p[1]), bf16_rne_pack(p[2], p[3]), bf16_rne_pack(p[4], p[5]),
                     bf16_rne_pack(p[6], p[7]));
    ((uint16_t*)meta)[blk * 64 + lane] = (uint16_t)nibs;
  }
  if (STREAM) store_stream_b128(&vals[blk * 64 + lane], out);
  else vals[blk * 64 + lane] = out;
  return amax;
}

template <bool FP8, bool AMAX, bool GAMMA = false, bool STREAM = false>
__device__ __forceinline__ float project_block(const uint8_t* __restrict__ W, int64_t O, int32_t steps, int64_t blk,
                                               int64_t ldw_bytes, float beta, float val_scale,
                                               uint4* __restrict__ vals, void* __restrict__ meta, int lane,
                                               float gamma = 0.0f) {
  constexpr int NG = FP8 ? 8 : 4;
  const int64_t rb = blk / steps;
  const int32_t s = (int32_t)(blk - rb * steps);
  const int j = lane & 15, q = lane >> 4;
  const int64_t row = rb * 16 + j;
  uint32_t w[2 * NG];
  if (row < O) {
    const uint4* src = (const uint4*)(W + row * ldw_bytes + ((int64_t)s * 4 + q) * (NG * 8));
#pragma unroll
    for (int c = 0; c < NG / 2; c++) {
      uint4 v = src[c];
      w[4 * c] = v.x; w[4 * c + 1] = v.y; w[4 * c + 2] = v.z; w[4 * c + 3] = v.w;
    }
  } else {
#pragma unroll
    for (int c = 0; c < 2 * NG; c++) w[c] = 0;
  }
  return project_store<FP8, AMAX, GAMMA, STREAM>(w, blk, beta, val_scale, vals, meta, lane, gamma);
}

// Dense-weight step of Eq. (7) fused with the projection of the new weight (Sec. 2: update the dense
// weight with the gradient taken at the sparse weight, then prune it again): one pass reads W and the
// gradient, writes W back and writes the packed S(W).  step = alpha * g and w' = w - step are single
// float32 operations.  A bf16 dense weight stores RNE_bf16(w') and is projected from it; a float32
// dense weight stores w' and is projected from RNE_bf16(w').  Same block-per-wave mapping as above.
// Per weight: 2 + 4 B read, 2 B written (bf16 weight; 4 + 4, 4 for float32) + the packed bytes.
template <bool FP8, bool F32, bool STREAM = false>
__device__ __forceinline__ void sgd_block(uint8_t* W, const float* __restrict__ G, int64_t O, int32_t steps, int64_t blk,
                                          int64_t ldw_bytes, int64_t ldg, float alpha, float beta, float val_scale,
                                          uint4* __restrict__ vals, void* __restrict__ meta, int lane) {
  constexpr int NG = FP8 ? 8 : 4;
  const int64_t rb = blk / steps;
  const int32_t s = (int32_t)(blk - rb * steps);
  const int j = lane & 15, q = lane >> 4;
  const int64_t row = rb * 16 + j;
  uint32_t w[2 * NG];
  if (row < O) {
    const int64_t col = ((int64_t)s * 4 + q) * (NG * 4);
    const f32x4* gp = (const f32x4*)(G + row * ldg + col);
    f32x4 g[NG];
#pragma unroll
    for (int c = 0; c < NG; c++) g[c] = gp[c];
    if (F32) {
      float4* wp = (float4*)(W + row * ldw_bytes + col * 4);
      float4 v[NG];
#pragma unroll
      for (int c = 0; c < NG; c++) v[c] = wp[c];
#pragma unroll
      for (int c = 0; c < NG; c++) {
        v[c].x = v[c].x - alpha * g[c][0];
        v[c].y = v[c].y - alpha * g[c][1];
        v[c].z = v[c].z - alpha * g[c][2];
        v[c].w = v[c].w - alpha * g[c][3];
        wp[c] = v[c];
        w[2 * c] = bf16_rne_pack(v[c].x, v[c].y);
        w[2 * c + 1] = bf16_rne_pack(v[c].z, v[c].w);
      }
    } else {
      uint4* wp = (uint4*)(W + row * ldw_bytes + col * 2);
      uint4 v[NG / 2];
#pragma unroll
      for (int c = 0; c < NG / 2; c++) v[c] = wp[c];
#pragma unroll
      for (int c = 0; c < NG / 2; c++) {
        const uint32_t in[4] = {v[c].x, v[c].y, v[c].z, v[c].w};
        const float gg[8] = {g[2 * c][0], g[2 * c][1], g[2 * c][2], g[2 * c][3],
                             g[2 * c + 1][0], g[2 * c + 1][1], g[2 * c + 1][2], g[2 * c + 1][3]};
#pragma unroll
        for (int e = 0; e < 4; e++) {
          float a = u2f(in[e] << 16) - alpha * gg[2 * e];
          float b = u2f(in[e] & 0xFFFF0000u) - alpha * gg[2 * e + 1];
          w[4 * c + e] = bf16_rne_pack(a, b);
        }
        wp[c] = make_uint4(w[4 * c], w[4 * c + 1], w[4 * c + 2], w[4 * c + 3]);
      }
    }
  } else {
#pragma unroll
    for (int c = 0; c < 2 * NG; c++) w[c] = 0;
  }
  project_store<FP8, false, false, STREAM>(w, blk, beta, val_scale, vals, meta, lane);
}

template <bool FP8, bool F32>
__global__ void __launch_bounds__(256)
k_sgd_project_pack(uint8_t* W, const float* __restrict__ G, int64_t O, int32_t steps, int64_t n_blocks,
                   int64_t ldw_bytes, int64_t ldg, float alpha, float beta, float val_scale,
                   uint4* __restrict__ vals, void* __restrict__ meta) {
  const int lane = threadIdx.x & 63;
  const int64_t blk = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (blk >= n_blocks) return;
  sgd_block<FP8, F32>(W, G, O, steps, blk, ldw_bytes, ldg, alpha, beta, val_scale, vals, meta, lane);
}

// Many tensors in one grid, like k_project_pack_batch.  80 bytes per item, layout shared with api.hip.
// The learning rate is a launch argument: it changes every iteration, the table does not.
struct UpdateTableItem {
  uint8_t* W;
  const float* G;
  uint4* vals;
  void* meta;
  int64_t O;
  int64_t ldw_bytes;
  int64_t ldg;
  int64_t first_block;
  int32_t steps;
  float beta;
  float val_scale;
  int32_t pad;
};
static_assert(sizeof(UpdateTableItem) == 80, "table item size is part of the C ABI (SSTE_UPDATE_TABLE_ITEM_BYTES)");

// A wave of the multi-tensor kernels takes kBatchRun consecutive global blocks: one table search, then
// it walks on through the table (items are sorted by first_block; empty items own no block and are
// stepped over).
constexpr int kBatchRun = 2;

template <bool FP8, bool F32, bool STREAM>
__global__ void __launch_bounds__(256)
k_sgd_project_pack_batch(const UpdateTableItem* __restrict__ table, int n_items, int64_t total_blocks, float alpha) {
  const int lane = threadIdx.x & 63;
  const int64_t blk0 = ((int64_t)blockIdx.x * 4 + __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6))) * kBatchRun;
  if (blk0 >= total_blocks) return;
  int lo = 0, hi = n_items - 1;                          // last item whose first_block <= blk0
  while (lo < hi) {
    int mid = (lo + hi + 1) >> 1;
    if (table[mid].first_block <= blk0) lo = mid;
    else hi = mid - 1;
  }
  UpdateTableItem it = table[lo];
  int64_t next_first = lo + 1 < n_items ? table[lo + 1].first_block : total_blocks;
  for (int b = 0; b < kBatchRun; b++) {
    const int64_t blk = blk0 + b;
    if (blk >= total_blocks) break;
    while (blk >= next_first) {
      lo++;
      it = table[lo];
      next_first = lo + 1 < n_items ? table[lo + 1].first_block : total_blocks;
    }
    sgd_block<FP8, F32, STREAM>(it.W, it.G, it.O, it.steps, blk - it.first_block, it.ldw_bytes, it.ldg, alpha, it.beta, it.val_scale,
                              it.vals, it.meta, lane);
  }
}

template <bool FP8, bool AMAX, bool GAMMA>
__global__ void __launch_bounds__(256)
k_project_pack(const uint8_t* __restrict__ W, int64_t O, int32_t steps, int64_t n_blocks, int64_t ldw_bytes,
               float beta, float val_scale, uint4* __restrict__ vals, void* __restrict__ meta,
               uint32_t* __restrict__ amax_bits, float gamma) {
  const int lane = threadIdx.x & 63;
  const int64_t blk = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  float amax = 0.0f;
  if (blk < n_blocks) amax = project_block<FP8, AMAX, GAMMA>(W, O, steps, blk, ldw_bytes, beta, val_scale, vals, meta, lane, gamma);
  if (AMAX) {
    // non-negative floats order like their bit patterns: reduce as unsigned integers
    uint32_t m = f2u(amax);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) m = max(m, (uint32_t)__shfl_xor((int)m, off, 64));
    __shared__ uint32_t wave_max[4];
    if ((threadIdx.x & 63) == 0) wave_max[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
      m = max(max(wave_max[0], wave_max[1]), max(wave_max[2], wave_max[3]));
      // atomics on one address serialise: only a workgroup that can raise the value issues one
      if (m > __hip_atomic_load(amax_bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(amax_bits, m);
    }
  }
}

// Many tensors in one grid: wave w of the grid takes global block w; the table (sorted by first_block)
// says which tensor that block belongs to.  64 bytes per item, layout shared with api.hip.
struct PackTableItem {
  const uint8_t* W;
  uint4* vals;
  void* meta;
  int64_t O;
  int64_t ldw_bytes;
  int64_t first_block;
  int32_t steps;
  float beta;
  float val_scale;
  int32_t pad;
};
static_assert(sizeof(PackTableItem) == 64, "table item size is part of the C ABI (SSTE_PACK_TABLE_ITEM_BYTES)");

template <bool FP8, bool STREAM>
__global__ void __launch_bounds__(256)
k_project_pack_batch(const PackTableItem* __restrict__ table, int n_items, int64_t total_blocks) {
  const int lane = threadIdx.x & 63;
  const int64_t blk0 = ((int64_t)blockIdx.x * 4 + __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6))) * kBatchRun;
  if (blk0 >= total_blocks) return;
  int lo = 0, hi = n_items - 1;                          // last item whose first_block <= blk0
  while (lo < hi) {
    int mid = (lo + hi + 1) >> 1;
    if (table[mid].first_block <= blk0) lo = mid;
    else hi = mid - 1;
  }
  PackTableItem it = table[lo];
  int64_t next_first = lo + 1 < n_items ? table[lo + 1].first_block : total_blocks;
  for (int b = 0; b < kBatchRun; b++) {
    const int64_t blk = blk0 + b;
    if (blk >= total_blocks) break;
    while (blk >= next_first) {
      lo++;
      it = table[lo];
      next_first = lo + 1 < n_items ? table[lo + 1].first_block : total_blocks;
    }
    project_block<FP8, false, false, STREAM>(it.W, it.O, it.steps, blk - it.first_block, it.ldw_bytes, it.beta, it.val_scale, it.vals, it.meta, lane);
  }
}

__global__ void k_fill_u32(uint32_t* p, uint32_t v) { *p = v; }
__global__ void k_fill_u64(unsigned long long* p, unsigned long long v) { *p = v; }

hipError_t launch_project_pack(const void* W, int64_t O, int64_t I, int64_t ldw, float beta, float gamma, int val_dtype,
                               float val_scale, void* vals, void* meta, float* amax_out, hipStream_t s) {
  if (amax_out) hipLaunchKernelGGL(k_fill_u32, dim3(1), dim3(1), 0, s, (uint32_t*)amax_out, 0u);
  bool fp8 = val_dtype == SSTE_F8E4M3;
  int64_t steps = I / (fp8 ? 128 : 64), n = ((O + 15) / 16) * steps;
  if (n == 0) return hipGetLastError();
  dim3 grid((unsigned)((n + 3) / 4)), block(256);
  const uint8_t* w = (const uint8_t*)W;
  uint32_t* ab = (uint32_t*)amax_out;
  const bool am = amax_out != nullptr, gm = gamma != 0.0f;
#define PP_CASE(F, A, G)                                                                                                   \
  if (fp8 == F && am == A && gm == G)                                                                                      \
    SSTE_LAUNCH(SSTE_K_PROJECT_PACK, (k_project_pack<F, A, G>), grid, block, s, w, O, (int32_t)steps, n, ldw * 2, beta, val_scale, \
                (uint4*)vals, meta, ab, gamma)
  PP_CASE(false, false, false);
  PP_CASE(false, true, false);
  PP_CASE(true, false, false);
  PP_CASE(true, true, false);
  PP_CASE(false, false, true);
  PP_CASE(false, true, true);
  PP_CASE(true, false, true);
  PP_CASE(true, true, true);
#undef PP_CASE
  return hipGetLastError();
}

hipError_t launch_sgd_project_pack(void* W, bool w_f32, int64_t O, int64_t I, int64_t ldw, const float* G, int64_t ldg,
                                   float alpha, float beta, int val_dtype, float val_scale, void* vals, void* meta,
                                   hipStream_t s) {
  bool fp8 = val_dtype == SSTE_F8E4M3;
  int64_t steps = I / (fp8 ? 128 : 64), n = ((O + 15) / 16) * steps;
  if (n == 0) return hipSuccess;
  dim3 grid((unsigned)((n + 3) / 4)), block(256);
  uint8_t* w = (uint8_t*)W;
  int64_t ldw_bytes = ldw * (w_f32 ? 4 : 2);
#define SGD_CASE(F8, F32)                                                                                      \
  SSTE_LAUNCH(SSTE_K_SGD_PROJECT_PACK, (k_sgd_project_pack<F8, F32>), grid, block, s, w, G, O, (int32_t)steps, n, \
              ldw_bytes, ldg, alpha, beta, val_scale, (uint4*)vals, meta)
  if (fp8 && w_f32) SGD_CASE(true, true);
  else if (fp8) SGD_CASE(true, false);
  else if (w_f32) SGD_CASE(false, true);
  else SGD_CASE(false, false);
#undef SGD_CASE
  return hipGetLastError();
}

hipError_t launch_sgd_project_pack_batch(const void* table, int n_items, int64_t total_blocks, bool w_f32, int val_dtype,
                                         float alpha, hipStream_t s) {
  if (n_items == 0 || total_blocks == 0) return hipSuccess;
  dim3 grid((unsigned)((total_blocks + 4 * kBatchRun - 1) / (4 * kBatchRun))), block(256);
  const UpdateTableItem* t = (const UpdateTableItem*)table;
  bool fp8 = val_dtype == SSTE_F8E4M3;
  // packed output larger than the 256 MB cache: nobody reads it back from the cache, write it with the streaming hint
  const bool stream = total_blocks > (int64_t)(256 << 10);
#define SGD_CASE(F8, F32)                                                                                                          \
  do {                                                                                                                             \
    if (stream) SSTE_LAUNCH(SSTE_K_SGD_PROJECT_PACK, (k_sgd_project_pack_batch<F8, F32, true>), grid, block, s, t, n_items, total_blocks, alpha); \
    else SSTE_LAUNCH(SSTE_K_SGD_PROJECT_PACK, (k_sgd_project_pack_batch<F8, F32, false>), grid, block, s, t, n_items, total_blocks, alpha);       \
  } while (0)
  if (fp8 && w_f32) SGD_CASE(true, true);
  else if (fp8) SGD_CASE(true, false);
  else if (w_f32) SGD_CASE(false, true);
  else SGD_CASE(false, false);
#undef SGD_CASE
  return hipGetLastError();
}

hipError_t launch_project_pack_batch(const void* table, int n_items, int64_t total_blocks, int val_dtype, hipStream_t s) {
  if (n_items == 0 || total_blocks == 0) return hipSuccess;
  dim3 grid((unsigned)((total_blocks + 4 * kBatchRun - 1) / (4 * kBatchRun))), block(256);
  // packed output (1 KiB of values per block) larger than the 256 MB cache: nobody reads it back from the cache, so it is
  // written with the streaming hint; a few layers' worth is read by the GEMMs that follow and is written normally
  const bool stream = total_blocks > (int64_t)(256 << 10);
  const PackTableItem* t = (const PackTableItem*)table;
#define PB_CASE(F8, ST) SSTE_LAUNCH(SSTE_K_PROJECT_PACK, (k_project_pack_batch<F8, ST>), grid, block, s, t, n_items, total_blocks)
  if (val_dtype == SSTE_F8E4M3 && stream) PB_CASE(true, true);
  else if (val_dtype == SSTE_F8E4M3) PB_CASE(true, false);
  else if (stream) PB_CASE(false, true);
  else PB_CASE(false, false);
#undef PB_CASE
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// beta = <w, S_soft(w)> / ||S_soft(w)||^2  (Sec. 4.2).  Exact products in float64, fixed-order sums.
constexpr int kBetaBlocks = 1024;

__global__ void __launch_bounds__(256)
k_beta_partial(const uint4* __restrict__ W, int64_t n_chunks, int32_t chunks_per_row, int64_t ldw_chunks,
               double* __restrict__ partial, int l1, float gamma) {
  double num = 0.0, den = 0.0;
  for (int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x; c < n_chunks; c += (int64_t)gridDim.x * 256) {
    int64_t row = c / chunks_per_row;
    int64_t col = c - row * chunks_per_row;
    uint4 w = W[row * ldw_chunks + col];
#pragma unroll
    for (int g = 0; g < 2; g++) {
      uint32_t lo = g ? w.z : w.x, hi = g ? w.w : w.y;
      Proj p = project_group<true>(lo, hi, 1.0f, gamma);   // p = a -/+ t as float32 (gamma = 0: t is the third magnitude)
      uint32_t pos0 = p.nib & 3u, pos1 = p.nib >> 2;
      double s0 = (double)p.p0, s1 = (double)p.p1;
      if (l1) {
        // L1-preserving scale: ||w||_1 over all four elements of the group, ||S_soft(w)||_1 over the recorded two
        num += (double)u2f((lo << 16) & 0x7FFFFFFFu) + (double)u2f(lo & 0x7FFF0000u) + (double)u2f((hi << 16) & 0x7FFFFFFFu) +
               (double)u2f(hi & 0x7FFF0000u);
        den += fabs(s0) + fabs(s1);
      } else {
        double a0 = (double)u2f(pick16_as_f32bits(lo, hi, pos0)), a1 = (double)u2f(pick16_as_f32bits(lo, hi, pos1));
        num += a0 * s0 + a1 * s1;
        den += s0 * s0 + s1 * s1;
      }
    }
  }
  __shared__ double sn[256], sd[256];
  sn[threadIdx.x] = num;
  sd[threadIdx.x] = den;
  __syncthreads();
  for (int off = 128; off > 0; off >>= 1) {
    if (threadIdx.x < off) {
      sn[threadIdx.x] += sn[threadIdx.x + off];
      sd[threadIdx.x] += sd[threadIdx.x + off];
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    partial[2 * blockIdx.x] = sn[0];
    partial[2 * blockIdx.x + 1] = sd[0];
  }
}

__global__ void __launch_bounds__(256) k_beta_final(const double* __restrict__ partial, int nblocks, float* beta_out) {
  __shared__ double sn[256], sd[256];
  double num = 0.0, den = 0.0;
  for (int i = threadIdx.x; i < nblocks; i += 256) {
    num += partial[2 * i];
    den += partial[2 * i + 1];
  }
  sn[threadIdx.x] = num;
  sd[threadIdx.x] = den;
  __syncthreads();
  for (int off = 128; off > 0; off >>= 1) {
    if (threadIdx.x < off) {
      sn[threadIdx.x] += sn[threadIdx.x + off];
      sd[threadIdx.x] += sd[threadIdx.x + off];
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) *beta_out = (sd[0] > 0.0) ? (float)(sn[0] / sd[0]) : __builtin_nanf("");
}

static int beta_blocks(int64_t n_chunks) {
  int64_t b = (n_chunks + 255) / 256;
  if (b > kBetaBlocks) b = kBetaBlocks;
  if (b < 1) b = 1;
  return (int)b;
}

size_t beta_workspace_bytes(int64_t O, int64_t I) { return (size_t)beta_blocks(O * (I / 8)) * 2 * sizeof(double); }

hipError_t launch_compute_beta(const void* W, int64_t O, int64_t I, int64_t ldw, int l1, float gamma, float* beta_out, void* ws,
                               hipStream_t s) {
  int64_t cpr = I / 8, n = O * cpr;
  int nb = beta_blocks(n);
  hipLaunchKernelGGL(k_beta_partial, dim3(nb), dim3(256), 0, s, (const uint4*)W, n, (int32_t)(cpr ? cpr : 1), ldw / 8, (double*)ws, l1, gamma);
  hipLaunchKernelGGL(k_beta_final, dim3(1), dim3(256), 0, s, (const double*)ws, nb, beta_out);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Flip count (Sec. 3.3): positions whose recorded / not-recorded state differs between two
// metadata arrays.  A nibble pos0 | pos1 << 2 expands to the 4-bit mask (1 << pos0) | (1 << pos1).
__device__ __forceinline__ uint32_t nibble_masks(uint32_t w) {
  uint32_t out = 0;
#pragma unroll
  for (int n = 0; n < 8; n++) {
    uint32_t nib = (w >> (4 * n)) & 0xFu;
    uint32_t m = (1u << (nib & 3u)) | (1u << (nib >> 2));
    out |= m << (4 * n);
  }
  return out;
}

__global__ void __launch_bounds__(256)
k_flip_count(const uint8_t* __restrict__ a, const uint8_t* __restrict__ b, int64_t nbytes, unsigned long long* out) {
  unsigned long long cnt = 0;
  int64_t nwords = nbytes / 4;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < nwords; i += (int64_t)gridDim.x * 256) {
    uint32_t wa = ((const uint32_t*)a)[i], wb = ((const uint32_t*)b)[i];
    cnt += __popc(nibble_masks(wa) ^ nibble_masks(wb));
  }
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    for (int64_t i = nwords * 4; i < nbytes; i++) cnt += __popc(nibble_masks(a[i]) ^ nibble_masks(b[i]));
  }
  __shared__ unsigned long long sc[256];
  sc[threadIdx.x] = cnt;
  __syncthreads();
  for (int off = 128; off > 0; off >>= 1) {
    if (threadIdx.x < off) sc[threadIdx.x] += sc[threadIdx.x + off];
    __syncthreads();
  }
  if (threadIdx.x == 0 && sc[0]) atomicAdd(out, sc[0]);
}

hipError_t launch_flip_count(const void* a, const void* b, int64_t nbytes, unsigned long long* out, hipStream_t s) {
  hipLaunchKernelGGL(k_fill_u64, dim3(1), dim3(1), 0, s, out, 0ull);
  if (nbytes > 0) {
    int64_t blocks = (nbytes / 4 + 255) / 256;
    if (blocks > 2048) blocks = 2048;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(k_flip_count, dim3((unsigned)blocks), dim3(256), 0, s, (const uint8_t*)a, (const uint8_t*)b, nbytes, out);
  }
  return hipGetLastError();
}

}  // namespace sste
