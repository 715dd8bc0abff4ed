// Per-tensor rescaling and cast of bf16 activations / gradients to the 8-bit operand formats (paper
// Sec. 5.2: operands are rescaled per tensor before they are cast to FP8; e4m3 for the forward
// operands, e5m2 for the output gradient).  One streaming pass: 2 B read and 1 B written per element,
// plus the tensor's largest magnitude, from which the caller derives the scale of the next iteration.
#include "common.h"

namespace sste {

__global__ void k_fill_u32_cast(uint32_t* p, uint32_t v) { *p = v; }

// A lane converts 8 consecutive elements (16 bytes in, 8 bytes out) of kCastUnroll chunks per round, a
// workgroup 256 x kCastUnroll consecutive chunks.  q = x / scale is a true float32 division; clamp to
// the largest finite value; round to nearest even.
// Largest magnitude: atomics on one address serialise in L2 (about 12 ns each; one per workgroup would be
// 25 us for the 2048 workgroups of a large launch, as long as the streaming itself).  One workgroup in
// kEarlyPublishStride therefore publishes its maximum after its FIRST round -- few atomics, which run under
// the streaming of the remaining rounds and leave a value close to the tensor's maximum -- and every
// workgroup publishes at its end only if it can still raise the value it reads, which is then rare
// (a workgroup beats the maximum of a sample s times as large as its own share with probability 1/(s+1)).
constexpr int kCastUnroll = 4;
constexpr int kEarlyPublishStride = 16;

__device__ __forceinline__ void publish_max(uint32_t m, uint32_t* __restrict__ amax_bits, uint32_t* wave_max) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) m = max(m, (uint32_t)__shfl_xor((int)m, off, 64));
  __syncthreads();                                   // wave_max may still be read from the previous call
  if ((threadIdx.x & 63) == 0) wave_max[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
    m = max(max(wave_max[0], wave_max[1]), max(wave_max[2], wave_max[3]));
    if (m > __hip_atomic_load(amax_bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(amax_bits, m);
  }
}

// The quotient x / scale of the bit-spec is the IEEE float32 division.  For a bf16 numerator (at most eight
// significant bits) the sequence  q0 = x * r,  e = fma(-q0, scale, x),  q = fma(e, r, q0)  with r = RN(1 / scale)
// gives the same float32 for every one of the 128 x 2^23 pairs of significands (checked by enumeration on the
// GPU), in four instructions instead of the ten of the division expansion.  It needs the residual e to be
// exact, i.e. no underflow on the way: the host takes this form only for 2^-40 <= scale <= 2^40, where every
// quotient of magnitude 2^-20 ... 2^30 has a normal residual; smaller quotients round to zero in both 8-bit
// formats whatever their last bits, larger ones saturate (q0 is clamped to +-2^30 first so that an infinite
// product cannot turn into NaN), and the sign of x is put back at the end (a zero quotient loses it).
__device__ __forceinline__ float quotient_bf16_numerator(float x, float scale, float r) {
  const float q0 = __builtin_amdgcn_fmed3f(x * r, -0x1p30f, 0x1p30f);
  const float e = __builtin_fmaf(-q0, scale, x);
  const float q = __builtin_fmaf(e, r, q0);
  return u2f((f2u(q) & 0x7FFFFFFFu) | (f2u(x) & 0x80000000u));
}

// ROWS = false: X and Q are contiguous (leading dimension == row length), addressed as one long row; the
// 64-bit division per chunk of the strided case costs as much as the conversions themselves.
// FAST: the quotient by the sequence above (recip = RN(1 / scale) from the host).
template <bool BF8, bool STORE, bool ROWS, bool FAST>
__global__ void __launch_bounds__(256)
k_cast_fp8(const uint8_t* __restrict__ X, int64_t R, int64_t chunks_per_row, int64_t ldx_bytes, float scale, float recip,
           uint8_t* __restrict__ Q, int64_t ldq, uint32_t* __restrict__ amax_bits) {
  __shared__ uint32_t wave_max[4];
  const int64_t n = R * chunks_per_row;
  const int64_t stride = (int64_t)gridDim.x * 256 * kCastUnroll;
  float amaxf = 0.0f;                 // inputs are finite by contract
  bool first = true;
  for (int64_t base = (int64_t)blockIdx.x * 256 * kCastUnroll; base < n; base += stride) {
    i32x4 t[kCastUnroll];
    int64_t row[kCastUnroll], col[kCastUnroll];
#pragma unroll
    for (int u = 0; u < kCastUnroll; u++) {
      const int64_t c = base + u * 256 + threadIdx.x;
      row[u] = ROWS ? c / chunks_per_row : 0;
      col[u] = c - row[u] * chunks_per_row;
      t[u] = (i32x4){0, 0, 0, 0};
      if (c < n) t[u] = __builtin_nontemporal_load((const i32x4*)(X + row[u] * ldx_bytes + col[u] * 16));   // read once
    }
#pragma unroll
    for (int u = 0; u < kCastUnroll; u++) {
      uint32_t w[4] = {(uint32_t)t[u][0], (uint32_t)t[u][1], (uint32_t)t[u][2], (uint32_t)t[u][3]};
      uint32_t out[2] = {0, 0};
#pragma unroll
      for (int e = 0; e < 4; e++) {
        const uint32_t lo = w[e] << 16, hi = w[e] & 0xFFFF0000u;         // two bf16 as float32 bits
        amaxf = __builtin_fmaxf(amaxf, __builtin_fmaxf(__builtin_fabsf(u2f(lo)), __builtin_fabsf(u2f(hi))));   // one three-operand maximum
        if (STORE) {
          const float a = FAST ? quotient_bf16_numerator(u2f(lo), scale, recip) : u2f(lo) / scale;
          const float b = FAST ? quotient_bf16_numerator(u2f(hi), scale, recip) : u2f(hi) / scale;
          uint32_t pair;
          if (BF8)
            pair = (uint32_t)__builtin_amdgcn_cvt_pk_bf8_f32(__builtin_amdgcn_fmed3f(a, -57344.0f, 57344.0f),
                                                             __builtin_amdgcn_fmed3f(b, -57344.0f, 57344.0f), 0, false) & 0xFFFFu;
          else
            pair = e4m3_rne_pack(clamp448(a), clamp448(b));
          out[e >> 1] |= pair << (16 * (e & 1));
        }
      }
      if (STORE && base + u * 256 + threadIdx.x < n) *(uint2*)(Q + row[u] * ldq + col[u] * 8) = make_uint2(out[0], out[1]);
    }
    if (amax_bits && first && blockIdx.x % kEarlyPublishStride == 0 && base + stride < n)
      publish_max(f2u(amaxf), amax_bits, wave_max);                                        // uniform per workgroup
    first = false;
  }
  if (amax_bits) publish_max(f2u(amaxf), amax_bits, wave_max);
}

hipError_t launch_cast_fp8(const void* X, int64_t R, int64_t C, int64_t ldx, int out_dtype, float scale, void* Q,
                           int64_t ldq, float* amax_out, hipStream_t s) {
  if (amax_out) hipLaunchKernelGGL(k_fill_u32_cast, dim3(1), dim3(1), 0, s, (uint32_t*)amax_out, 0u);
  const int64_t chunks = C / 8, n = R * chunks;
  if (n == 0) return hipGetLastError();
  int64_t blocks = (n + 256 * kCastUnroll - 1) / (256 * kCastUnroll);
  if (blocks > 256 * 8) blocks = 256 * 8;                 // 8 workgroups (32 waves) per CU, grid-stride beyond
  dim3 grid((unsigned)blocks), block(256);
  const uint8_t* x = (const uint8_t*)X;
  uint32_t* ab = (uint32_t*)amax_out;
  const bool rows = !(ldx == C && (!Q || ldq == C));
  const bool fast = Q && scale >= 0x1p-40f && scale <= 0x1p40f;
  const float recip = 1.0f / scale;                       // IEEE division on the host: the correctly rounded reciprocal
#define CAST_LAUNCH(B8, ST, RW, FA)                                                                                    \
  SSTE_LAUNCH(SSTE_K_CAST, (k_cast_fp8<B8, ST, RW, FA>), grid, block, s, x, R, chunks, ldx * 2, scale, recip, (uint8_t*)Q, ldq, ab)
#define CAST_CASE(B8, ST)                                                                                              \
  do {                                                                                                                 \
    if (rows && fast) CAST_LAUNCH(B8, ST, true, ST);                                                                   \
    else if (rows) CAST_LAUNCH(B8, ST, true, false);                                                                   \
    else if (fast) CAST_LAUNCH(B8, ST, false, ST);                                                                     \
    else CAST_LAUNCH(B8, ST, false, false);                                                                            \
  } while (0)
  if (!Q) CAST_CASE(false, false);
  else if (out_dtype == SSTE_F8E5M2) CAST_CASE(true, true);
  else CAST_CASE(false, true);
#undef CAST_CASE
#undef CAST_LAUNCH
  return hipGetLastError();
}

}  // namespace sste
