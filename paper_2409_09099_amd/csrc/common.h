// Shared host/device helpers for the S-STE sparse linear-layer kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/sste.h"

namespace sste {

// ---- host: status + thread-local message -----------------------------------------------------
int fail(int status, const char* fmt, ...);   // records the message, returns `status`
void clear_error();

// ---- host: size arithmetic that cannot overflow ------------------------------------------------------
// a * b >= limit for non-negative 64-bit a, b (limit > 0), without forming a product that may overflow
inline bool product_reaches(int64_t a, int64_t b, int64_t limit) {
  if (a <= 0 || b <= 0) return false;
  return a >= (limit + b - 1) / b;
}

// ---- optional per-kernel timing (sste_timing_begin / sste_timing_end) ---------------------------
// While timing is on, each launch of a hot-path kernel is bracketed by its own pair of HIP events on
// the launch stream, so the time reported is that kernel's alone.
struct TimingSlot { hipEvent_t start, stop; };
TimingSlot* timing_slot(int kind);   // nullptr when timing is off or the event pool is used up

#define SSTE_LAUNCH(kind, kernel, grid, block, stream, ...)                                           \
  do {                                                                                                \
    ::sste::TimingSlot* ts_ = ::sste::timing_slot(kind);                                              \
    if (ts_) hipExtLaunchKernelGGL(kernel, grid, block, 0, stream, ts_->start, ts_->stop, 0, __VA_ARGS__); \
    else hipLaunchKernelGGL(kernel, grid, block, 0, stream, __VA_ARGS__);                             \
  } while (0)

// ---- vector types for MFMA operands -----------------------------------------------------------
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(__bf16)))) __bf16 bf16x16;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(2 * sizeof(int)))) int i32x2;
typedef __attribute__((__vector_size__(4 * sizeof(int)))) int i32x4;
typedef __attribute__((__vector_size__(8 * sizeof(int)))) int i32x8;

// ---- device bit helpers -------------------------------------------------------------------------
__device__ __forceinline__ float u2f(uint32_t u) { return __uint_as_float(u); }
__device__ __forceinline__ uint32_t f2u(float f) { return __float_as_uint(f); }

// float32 -> bf16 pattern, round to nearest even (v_cvt_pk_bf16_f32 on gfx950)
__device__ __forceinline__ uint32_t bf16_rne(float f) {
  __bf16 b = (__bf16)f;
  uint16_t u;
  __builtin_memcpy(&u, &b, 2);
  return u;
}
// two floats -> packed bf16 pair (lo in bits 0..15)
__device__ __forceinline__ uint32_t bf16_rne_pack(float lo, float hi) {
  typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
  bf16x2 v;
  v[0] = (__bf16)lo;
  v[1] = (__bf16)hi;
  uint32_t u;
  __builtin_memcpy(&u, &v, 4);
  return u;
}

// 16-bit element `idx` (0..3) of the little-endian 64-bit pair {hi:lo}, moved to the top half of
// a dword with zeros below: the float32 value of that bf16 element.
__device__ __forceinline__ uint32_t pick16_as_f32bits(uint32_t lo, uint32_t hi, uint32_t idx) {
  // v_perm_b32: selector bytes 0..3 address `lo`, 4..7 address `hi`, 0x0c yields 0x00.
  // selector = 0x01000c0c + idx * 0x02020000.  Written as two shift-or/add instructions: the compiler
  // turns any C spelling of it back into a 32-bit multiply, which runs at quarter rate.
  uint32_t t, sel;
  asm("v_lshl_or_b32 %0, %1, 8, %1" : "=v"(t) : "v"(idx));
  asm("v_lshl_add_u32 %0, %1, 17, %2" : "=v"(sel) : "v"(t), "s"(0x01000c0cu));
  return __builtin_amdgcn_perm(hi, lo, sel);
}

// OCP e4m3 conversions (hardware: v_cvt_f32_fp8 / v_cvt_pk_fp8_f32, OCP flavour on gfx950)
__device__ __forceinline__ float e4m3_to_f32(uint32_t packed, int byte) {
  switch (byte) {
    case 0: return __builtin_amdgcn_cvt_f32_fp8(packed, 0);
    case 1: return __builtin_amdgcn_cvt_f32_fp8(packed, 1);
    case 2: return __builtin_amdgcn_cvt_f32_fp8(packed, 2);
    default: return __builtin_amdgcn_cvt_f32_fp8(packed, 3);
  }
}
// two floats (already clamped to +-448) -> two e4m3 codes in the low 16 bits
__device__ __forceinline__ uint32_t e4m3_rne_pack(float lo, float hi) {
  return (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(lo, hi, 0, false) & 0xFFFFu;
}
__device__ __forceinline__ float clamp448(float x) { return __builtin_amdgcn_fmed3f(x, -448.0f, 448.0f); }

// ---- activation between the two FFN linears -----------------------------------------------------------
// GELU in its tanh form, 0.5 x (1 + tanh(u)), u = sqrt(2/pi) (x + 0.044715 x^3) -- the form of the GPT-2 models
// whose layer shapes the workloads use (the paper does not name the activation).  Evaluated as x * s with
// s = 0.5 (1 + tanh(u)) = 1 / (1 + exp(-2u)) on the hardware exp2 / reciprocal: float32, about 1e-6 absolute.
// The ends behave: exp2 -> inf gives s = 0, exp2 -> 0 gives s = 1.
__device__ __forceinline__ float gelu_sigmoid(float x, float x2) {
  const float p = __builtin_fmaf(x2, 0.044715f, 1.0f);                    // 1 + 0.044715 x^2
  const float e = __builtin_amdgcn_exp2f((x * p) * -2.3022081981f);       // exp(-2u): -2 sqrt(2/pi) log2(e) = -2.3022082
  return __builtin_amdgcn_rcpf(1.0f + e);
}
__device__ __forceinline__ float gelu_tanh(float x) { return x * gelu_sigmoid(x, x * x); }
// d/dx: s + x s (1 - s) * 2 du/dx, du/dx = sqrt(2/pi) (1 + 3 * 0.044715 x^2)
__device__ __forceinline__ float gelu_tanh_grad(float x) {
  const float x2 = x * x;
  const float s = gelu_sigmoid(x, x2);
  const float q = __builtin_fmaf(x2, 0.2140644488f, 1.5957691216f);       // 2 sqrt(2/pi) (1 + 0.134145 x^2)
  return __builtin_fmaf(x * q, s - s * s, s);
}
__device__ __forceinline__ float bf16lo_f32(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16hi_f32(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// ---- buffer-descriptor loads ---------------------------------------------------------------------
// A raw buffer descriptor over [base, base + bytes): loads whose offset falls outside return zeros,
// which replaces per-lane bounds branches at tile edges.  Offsets are 32-bit.
typedef __amdgpu_buffer_rsrc_t BufferRsrc;
__device__ __forceinline__ BufferRsrc make_rsrc(const void* base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ uint4 buffer_load_b128(BufferRsrc r, uint32_t voffset, uint32_t soffset) {
  i32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)voffset, (int)soffset, 0);
  return make_uint4((uint32_t)v[0], (uint32_t)v[1], (uint32_t)v[2], (uint32_t)v[3]);
}
__device__ __forceinline__ uint2 buffer_load_b64(BufferRsrc r, uint32_t voffset, uint32_t soffset) {
  i32x2 v = __builtin_amdgcn_raw_buffer_load_b64(r, (int)voffset, (int)soffset, 0);
  return make_uint2((uint32_t)v[0], (uint32_t)v[1]);
}

// ---- direct-to-LDS loads and hand-tracked completion ------------------------------------------------
typedef __attribute__((address_space(3))) uint8_t lds_u8;

// s_waitcnt that constrains only the vector-memory counter (gfx9 encoding: vmcnt in bits 3:0 and
// 15:14; expcnt and lgkmcnt fields left at "no wait")
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  __builtin_amdgcn_s_waitcnt((N & 0xF) | 0x0F70 | ((N >> 4) << 14));
}

// 64 lanes x 16 B (or 4 B) from a buffer descriptor straight into LDS at lds_addr + lane * 16 (4).
// The statements overwrite M0 and say so in their clobber list, so the compiler never keeps a value
// of its own in M0 across them (it warns that M0 is a reserved register; that is the point).
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void dma_b128(i32x4 rsrc, uint32_t lds_addr, uint32_t voffset, uint32_t soffset) {
  asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
               :
               : "s"(lds_addr), "v"(voffset), "s"(rsrc), "s"(soffset)
               : "memory", "m0");
}
__device__ __forceinline__ void dma_b32(i32x4 rsrc, uint32_t lds_addr, uint32_t voffset, uint32_t soffset) {
  asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dword %1, %2, %3 offen lds"
               :
               : "s"(lds_addr), "v"(voffset), "s"(rsrc), "s"(soffset)
               : "memory", "m0");
}
#pragma clang diagnostic pop
// XOR key of the LDS tiles that are read with the transposing loads (ds_read_b64_tr_b16 / _b8): the X tile of
// the weight-gradient GEMM and the expanded S(W) tile of the input-gradient GEMM.  A tile row (one index of the
// contraction) is 512 B (bf16) or 256 B (8-bit), so every row starts at bank 0, and the 32-byte (16-byte) unit
// u of row r is stored at position u ^ x_swizzle(r).  One transposing read gathers, per 16 lanes, 4 (8)
// consecutive rows with the four lane quarters 8 (16) rows apart; the units of one such read must fall on
// different banks, and so must the 16 consecutive rows that 16 lanes of the input-gradient kernel write at
// once.  bf16: bits (r0, r1, r3) pick the 32-byte bank group, r2 the half of the row.  8-bit: bits
// (r0, r1, r2, r3 ^ r4).  (With r % 16 as the key the lane quarters of a read collided pairwise: bank
// conflicts were 25...45 % of these kernels' LDS cycles.)
template <bool FP8>
__device__ __forceinline__ int x_swizzle(int r) {
  return FP8 ? ((r & 7) | ((((r >> 3) ^ (r >> 4)) & 1) << 3))
             : ((r & 3) | (((r >> 3) & 1) << 2) | (((r >> 2) & 1) << 3));
}
__device__ __forceinline__ i32x4 rsrc_words(const void* base, uint32_t bytes) {
  uint64_t p = (uint64_t)base;
  i32x4 r;
  r[0] = __builtin_amdgcn_readfirstlane((int)(uint32_t)p);
  r[1] = __builtin_amdgcn_readfirstlane((int)((uint32_t)(p >> 32) & 0xFFFFu));
  r[2] = __builtin_amdgcn_readfirstlane((int)bytes);
  r[3] = 0x00020000;
  return r;
}

// The chip hands consecutive workgroup ids to its 8 XCDs in turn; this numbering gives each XCD a
// contiguous range of logical numbers instead, so that the workgroups sharing an L2 work on
// neighbouring tiles.
__device__ __forceinline__ int xcd_contiguous(int bid, int nblk) {
  constexpr int XCDS = 8;
  const int per_xcd = (nblk + XCDS - 1) / XCDS, rem = nblk % XCDS;
  const int xcd = bid % XCDS, slot = bid / XCDS;
  return (rem == 0 || xcd < rem) ? xcd * per_xcd + slot : rem * per_xcd + (xcd - rem) * (per_xcd - 1) + slot;
}
// MFMA group (0 .. groups-1) in which item idx of n evenly spread items is issued
constexpr int spread(int idx, int n, int groups) { return idx * groups / n; }

// Streaming (non-temporal) store for a final output that no kernel of the path reads again (Z): it
// leaves the L2 to the operands that are re-read, and no pile of dirty lines is left to flush when the
// kernel ends (measured on the 5120 x 1280 forward GEMM at 16384 tokens: 142 -> 113 us).  Intermediate
// results that the next kernel consumes (the packed estimator operand, the split partial sums) are
// stored normally: written with this hint they come back from HBM instead of the cache hierarchy and
// the consumer runs 15 % slower.
__device__ __forceinline__ void store_stream_b128(void* p, uint4 v) {
  i32x4 t;
  __builtin_memcpy(&t, &v, 16);
  __builtin_nontemporal_store(t, (i32x4*)p);
}
__device__ __forceinline__ void store_stream_b128(void* p, float4 v) {
  f32x4 t;
  __builtin_memcpy(&t, &v, 16);
  __builtin_nontemporal_store(t, (f32x4*)p);
}

// ---- host-side launch entry points implemented in the .hip files --------------------------------
// Key words of the draw, plus the global index of the tensor's first token group (the group id of
// token group k and channel o is (first_group + k) * O + o).
struct RngKey { uint32_t k0, k1; uint64_t first_group; };
RngKey derive_key(uint64_t seed, uint64_t offset);

hipError_t launch_project_pack(const void* W, int64_t O, int64_t I, int64_t ldw, float beta, float gamma, int val_dtype,
                               float val_scale, void* vals, void* meta, float* amax_out, hipStream_t s);
hipError_t launch_sgd_project_pack(void* W, bool w_f32, int64_t O, int64_t I, int64_t ldw, const float* G, int64_t ldg,
                                   float alpha, float beta, int val_dtype, float val_scale, void* vals, void* meta,
                                   hipStream_t s);
hipError_t launch_sgd_project_pack_batch(const void* table, int n_items, int64_t total_blocks, bool w_f32, int val_dtype,
                                         float alpha, hipStream_t s);
hipError_t launch_project_pack_batch(const void* table, int n_items, int64_t total_blocks, int val_dtype, hipStream_t s);
bool linear_dgrad_supported(int64_t T, int64_t O, int64_t lddy, int64_t I, int dtype);
hipError_t launch_linear_dgrad(const void* dY, int64_t T, int64_t O, int64_t lddy, int dtype, float scale, const void* vals,
                               const void* meta, int64_t I, void* dX, int64_t lddx, const void* H, int64_t ldh, hipStream_t s);
hipError_t launch_compute_beta(const void* W, int64_t O, int64_t I, int64_t ldw, int l1, float gamma, float* beta_out, void* ws,
                               hipStream_t s);
size_t beta_workspace_bytes(int64_t O, int64_t I);
hipError_t launch_cast_fp8(const void* X, int64_t R, int64_t C, int64_t ldx, int out_dtype, float scale, void* Q,
                           int64_t ldq, float* amax_out, hipStream_t s);
hipError_t launch_flip_count(const void* a, const void* b, int64_t nbytes, unsigned long long* out, hipStream_t s);
hipError_t launch_mvue_materialize(const void* dY, int64_t T, int64_t O, int64_t lddy, int dtype, RngKey key,
                                   void* vals, void* meta, hipStream_t s);
hipError_t launch_linear_fwd(const void* X, int64_t T, int64_t I, int64_t ldx, int dtype, float scale,
                             const void* vals, const void* meta, int64_t O, void* Z, int64_t ldz, int z_dtype,
                             float amax_scale, float* amax_out, hipStream_t s);
hipError_t launch_linear_fwd_act(const void* X, int64_t T, int64_t I, int64_t ldx, int dtype, float scale,
                                 const void* vals, const void* meta, int64_t O, void* H, int64_t ldh, void* A, int64_t lda,
                                 int a_dtype, float a_inv_scale, float* amax_out, hipStream_t s);
bool linear_fwd_supported(int64_t T, int64_t I, int64_t ldx, int64_t O, int dtype);
size_t wgrad_workspace_bytes(int64_t T, int64_t O, int64_t I, int dtype);
bool linear_wgrad_supported(int64_t T, int64_t O, int64_t I, int64_t ldx, int dtype);
bool wgrad_plan_override(int mi, int ni, int splits);
void* noalloc_scratch(hipError_t* err);   // this GPU's copy of the library's static scratch array
hipError_t launch_linear_wgrad(const void* dY, int64_t T, int64_t O, int64_t lddy, int dtype, const void* X,
                               int64_t I, int64_t ldx, float scale, RngKey key, float* dW, int64_t lddw,
                               int accumulate, void* ws, hipStream_t s);

}  // namespace sste
