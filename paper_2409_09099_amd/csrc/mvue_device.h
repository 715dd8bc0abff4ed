// Device code of the 2:4 minimum-variance unbiased estimator (paper Sec. 5.1) and its counter-based
// random draw.  The rule is stated in full in include/sste.h (sste_mvue_materialize).  Every float
// operation below is a single IEEE float32 operation in the order written; the translation unit is
// compiled with -ffp-contract=off so that tau1 = tau0 + h is not fused with tau0 = u * h.
#pragma once
#include "common.h"

namespace sste {

// 32-bit draw for a group id: three-round multiply-xorshift hash keyed by (k0, k1).  hi_term is the
// high word of the group id times 0x9E3779B9, which callers that walk consecutive ids hoist out of
// their loops.
__device__ __forceinline__ uint32_t draw_u32_pre(uint32_t k0, uint32_t k1, uint32_t gid_lo, uint32_t hi_term) {
  uint32_t x = gid_lo ^ k0;
  x += hi_term;
  x ^= x >> 17;
  x *= 0xED5AD4BBu;
  x += k1;
  x ^= x >> 11;
  x *= 0xAC4C1B51u;
  x ^= x >> 15;
  x *= 0x31848BABu;
  x ^= x >> 14;
  return x;
}
__device__ __forceinline__ uint32_t draw_u32(uint32_t k0, uint32_t k1, uint32_t gid_lo, uint32_t gid_hi) {
  return draw_u32_pre(k0, k1, gid_lo, gid_hi * 0x9E3779B9u);
}

struct Sel {
  float h;        // common magnitude of recorded elements that are not kept as they are
  uint32_t pos0;  // recorded positions, pos0 < pos1
  uint32_t pos1;
};

// Steps 1-4 of the rule on the four magnitudes m0..m3 (all >= 0, finite) and the 32-bit draw x.
// Non-negative floats order like their bit patterns, so minima, maxima and comparisons are taken on
// the bits as unsigned integers (same results, and no NaN canonicalisation instructions); sums and
// products are float32 operations.
__device__ __forceinline__ Sel mvue_select(float m0f, float m1f, float m2f, float m3f, uint32_t x) {
  uint32_t m0 = f2u(m0f), m1 = f2u(m1f), m2 = f2u(m2f), m3 = f2u(m3f);
  uint32_t a = max(m0, m1), b = min(m0, m1);
  uint32_t cc = max(m2, m3), d = min(m2, m3);
  uint32_t mx = max(a, cc), mid = min(a, cc);
  float Lo = (u2f(b) + u2f(d)) + u2f(mid);
  uint32_t clampv = (f2u(Lo) == 0u) ? mx : f2u(Lo);      // Lo is a sum of non-negative terms: +0 or positive
  float l0 = u2f(min(m0, clampv)), l1 = u2f(min(m1, clampv)), l2 = u2f(min(m2, clampv)), l3 = u2f(min(m3, clampv));
  float P0 = l0;
  float P1 = P0 + l1;
  float P2 = P1 + l2;
  float L = P2 + l3;
  float h = 0.5f * L;
  float u = (float)(x >> 8) * 0x1p-24f;     // exact: 24-bit integer times a power of two
  float tau0 = u * h;
  float tau1 = tau0 + h;
  uint32_t p0 = f2u(P0), p1 = f2u(P1), p2 = f2u(P2), t0 = f2u(tau0), t1 = f2u(tau1);
  // pos0 = min(#{k : P_k <= tau0}, 2): the prefix sums never decrease, so P2 <= tau0 implies the other
  // two and the count capped at 2 is the count over P0 and P1 alone.  pos1 = min(3, max(i1, pos0 + 1))
  // with i1 <= 3 and pos0 <= 2: the outer min never acts.
  Sel s;
  s.h = h;
  s.pos0 = (uint32_t)(p0 <= t0) + (uint32_t)(p1 <= t0);
  uint32_t i1 = (uint32_t)(p0 <= t1) + (uint32_t)(p1 <= t1) + (uint32_t)(p2 <= t1);
  s.pos1 = max(i1, s.pos0 + 1u);
  return s;
}

// bf16 group {hi:lo} = (g0 | g1 << 16, g2 | g3 << 16).  Returns the two recorded bf16 values packed
// (pos0's value in the low half) and writes the metadata nibble pos0 | pos1 << 2.
__device__ __forceinline__ uint32_t mvue_group_bf16(uint32_t lo, uint32_t hi, uint32_t x, uint32_t& nib) {
  float m0 = u2f((lo << 16) & 0x7FFFFFFFu), m1 = u2f(lo & 0x7FFF0000u);
  float m2 = u2f((hi << 16) & 0x7FFFFFFFu), m3 = u2f(hi & 0x7FFF0000u);
  Sel s = mvue_select(m0, m1, m2, m3, x);
  // Both recorded elements at once, as a pair of 16-bit patterns (pos0's in the low half): one byte
  // permute of {hi:lo} with selector bytes (2 pos0, 2 pos0 + 1, 2 pos1, 2 pos1 + 1).
  typedef __attribute__((__vector_size__(2 * sizeof(uint16_t)))) uint16_t u16x2;
  const uint32_t pp = s.pos0 | (s.pos1 << 16);
  const uint32_t sel = ((pp << 1) | (pp << 9)) + 0x01000100u;
  const uint32_t g = __builtin_amdgcn_perm(hi, lo, sel);
  // An element keeps its own pattern when m_p > h or m_p == 0.  On the 15-bit magnitude fields (the low
  // 16 bits of a bf16's float32 pattern are zero): field > bits(h) >> 16, or field == 0; both at once as
  // (field - 1) mod 2^16 >= bits(h) >> 16, evaluated for the pair with packed 16-bit arithmetic:
  // the saturating difference hh - (field - 1) is zero exactly for the elements that keep their pattern.
  const uint32_t hh = f2u(s.h) >> 16;
  u16x2 field, one = {1, 1}, hh2 = {(uint16_t)hh, (uint16_t)hh};
  const uint32_t gm = g & 0x7FFF7FFFu;
  __builtin_memcpy(&field, &gm, 4);
  u16x2 d = __builtin_elementwise_sub_sat(hh2, (u16x2)(field - one));
  u16x2 common_mask = (u16x2){0, 0} - __builtin_elementwise_min(d, one);        // 0xFFFF where sign | RNE(h) is stored
  uint32_t cm;
  __builtin_memcpy(&cm, &common_mask, 4);
  const uint32_t hq = bf16_rne(s.h);
  const uint32_t common = (g & 0x80008000u) | (hq | (hq << 16));
  nib = s.pos0 | (s.pos1 << 2);
  return (common & cm) | (g & ~cm);
}

// 8-bit group (e4m3, or e5m2 when BF8): the four codes of one group in one dword (g0 in byte 0).
// Returns the two recorded codes of theta / 2 in the low 16 bits (pos0's in byte 0).
template <bool BF8>
__device__ __forceinline__ float cvt8(uint32_t w) {
  return BF8 ? __builtin_amdgcn_cvt_f32_bf8((int)w, 0) : __builtin_amdgcn_cvt_f32_fp8((int)w, 0);
}
template <bool BF8>
__device__ __forceinline__ uint32_t mvue_group_f8(uint32_t g, uint32_t x, uint32_t& nib) {
  uint32_t ga = g & 0x7F7F7F7Fu;
  float m0, m1, m2, m3;
  if (BF8) {
    m0 = __builtin_amdgcn_cvt_f32_bf8(ga, 0), m1 = __builtin_amdgcn_cvt_f32_bf8(ga, 1);
    m2 = __builtin_amdgcn_cvt_f32_bf8(ga, 2), m3 = __builtin_amdgcn_cvt_f32_bf8(ga, 3);
  } else {
    m0 = __builtin_amdgcn_cvt_f32_fp8(ga, 0), m1 = __builtin_amdgcn_cvt_f32_fp8(ga, 1);
    m2 = __builtin_amdgcn_cvt_f32_fp8(ga, 2), m3 = __builtin_amdgcn_cvt_f32_fp8(ga, 3);
  }
  Sel s = mvue_select(m0, m1, m2, m3, x);
  // the two recorded codes side by side in bytes 0 and 1 (one byte permute; selector bytes 0x0c give zero)
  const uint32_t rec = __builtin_amdgcn_perm(g, g, s.pos0 | (s.pos1 << 8) | 0x0c0c0000u);
  const uint32_t reca = rec & 0x7F7Fu;
  float mp0, mp1;
  if (BF8) mp0 = __builtin_amdgcn_cvt_f32_bf8((int)reca, 0), mp1 = __builtin_amdgcn_cvt_f32_bf8((int)reca, 1);
  else mp0 = __builtin_amdgcn_cvt_f32_fp8((int)reca, 0), mp1 = __builtin_amdgcn_cvt_f32_fp8((int)reca, 1);
  // stored magnitudes: 0.5 * m_p where g_p is kept as it is, else 0.5 * h; all within the format's range
  bool own0 = (f2u(mp0) - 1u) >= f2u(s.h);
  bool own1 = (f2u(mp1) - 1u) >= f2u(s.h);
  float v0 = 0.5f * (own0 ? mp0 : s.h);
  float v1 = 0.5f * (own1 ? mp1 : s.h);
  uint32_t q = BF8 ? ((uint32_t)__builtin_amdgcn_cvt_pk_bf8_f32(v0, v1, 0, false) & 0xFFFFu) : e4m3_rne_pack(v0, v1);
  nib = s.pos0 | (s.pos1 << 2);
  return q | (rec & 0x8080u);
}
__device__ __forceinline__ uint32_t mvue_group_e4m3(uint32_t g, uint32_t x, uint32_t& nib) {
  return mvue_group_f8<false>(g, x, nib);
}

}  // namespace sste
