/*
 * Plain C versions of the oracle's three heaviest bit-spec routines, for the parity tests that run at
 * the full workload sizes (hundreds of millions of elements, where the numpy forms take minutes).
 *
 * TEST INFRASTRUCTURE, NOT PRODUCT CODE: nothing under the HIP library includes, links or calls this
 * file, and this file includes nothing of it.  Each routine is a scalar loop written from the same
 * specification text as its numpy counterpart (oracle/formats.py, oracle/mvue.py, oracle/rng.py,
 * oracle/projection.py) and is checked against that counterpart, element for element, by
 * tests/test_oracle_native.py; the numpy forms stay the reference and carry the pins to the paper.
 *
 *   orc_cast_fp8      Sec. 5.2: per-tensor rescale + cast of a bf16 tensor to e4m3 / e5m2
 *   orc_mvue_pack     Sec. 5.1: the 2:4 minimum-variance unbiased estimator on groups of four tokens,
 *                     with the counter-based draw, written as a row-major packed operand
 *   orc_decode_packed packed (values, 2-bit positions) -> dense-with-zeros float64 matrix
 *
 * Built with gcc -O2 -ffp-contract=off -fopenmp: every float operation below is one IEEE float32 (or
 * float64, where written) operation in the order written.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

enum { ORC_BF16 = 0, ORC_E4M3 = 1, ORC_E5M2 = 3 };

/* ---- storage formats ------------------------------------------------------------------------- */

static float bf16_to_f32(uint16_t b) {
  uint32_t u = (uint32_t)b << 16;
  float f;
  memcpy(&f, &u, 4);
  return f;
}

/* round to nearest, ties to even, on the upper 16 bits of the float32 pattern (no NaN handling) */
static uint16_t f32_to_bf16_rne(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  uint32_t lsb = (u >> 16) & 1u;
  return (uint16_t)((u + 0x7FFFu + lsb) >> 16);
}

/* e4m3fn: 1 sign, 4 exponent (bias 7), 3 mantissa bits; exponent 0 subnormal; no infinity */
static float e4m3_to_f32(uint8_t c) {
  int s = c >> 7, e = (c >> 3) & 15, m = c & 7;
  double mag = e == 0 ? m * ldexp(1.0, -9) : (1.0 + m / 8.0) * ldexp(1.0, e - 7);
  if (e == 15 && m == 7) mag = NAN;
  return (float)(s ? -mag : mag);
}

/* e5m2: 1 sign, 5 exponent (bias 15), 2 mantissa bits; exponent 0 subnormal; exponent 31 inf / NaN */
static float e5m2_to_f32(uint8_t c) {
  int s = c >> 7, e = (c >> 2) & 31, m = c & 3;
  double mag = e == 0 ? m * ldexp(1.0, -16) : (1.0 + m / 4.0) * ldexp(1.0, e - 15);
  if (e == 31) mag = m == 0 ? INFINITY : NAN;
  return (float)(s ? -mag : mag);
}

/* clamp to the largest finite magnitude, round to nearest even on the format's grid, keep subnormals
   and the sign of zero.  mbits = mantissa bits, emin = exponent of the smallest normal binade,
   emax = exponent of the largest binade, bias as in the format. */
static uint8_t f32_to_f8_rne_sat(float x, int mbits, int emin, int emax, int bias, double fmax) {
  int neg = signbit(x) ? 1 : 0;
  double a = fabs((double)x);
  if (a > fmax) a = fmax;
  int ex = 0;
  int e = emin;
  if (a > 0) {
    (void)frexp(a, &ex);            /* a = mant * 2^ex, mant in [0.5, 1) */
    e = ex - 1;
  }
  if (e < emin) e = emin;
  if (e > emax) e = emax;
  double step = ldexp(1.0, e - mbits);           /* spacing of the grid in that binade */
  double q = nearbyint(a / step);                /* ties to even (default rounding mode) */
  int one = 1 << mbits;                          /* q of the binade's first value */
  if (q >= 2 * one) {                            /* carried into the next binade */
    e += 1;
    q = one;
  }
  int qi = (int)q;
  int code = qi < one ? qi : (((e + bias) << mbits) | (qi - one));
  return (uint8_t)(code | (neg << 7));
}
static uint8_t f32_to_e4m3(float x) { return f32_to_f8_rne_sat(x, 3, -6, 8, 7, 448.0); }
static uint8_t f32_to_e5m2(float x) { return f32_to_f8_rne_sat(x, 2, -14, 15, 15, 57344.0); }

/* ---- Sec. 5.2: per-tensor rescale + cast ------------------------------------------------------- */

/* q = x / scale as ONE float32 division, clamped, rounded.  Returns max |x| through amax_out. */
void orc_cast_fp8(const uint16_t* x_bits, int64_t n, float scale, int fmt, uint8_t* codes, float* amax_out) {
  float amax = 0.0f;
#pragma omp parallel for reduction(max : amax) schedule(static)
  for (int64_t i = 0; i < n; i++) {
    float x = bf16_to_f32(x_bits[i]);
    volatile float q = x / scale;
    codes[i] = fmt == ORC_E4M3 ? f32_to_e4m3(q) : f32_to_e5m2(q);
    float ax = fabsf(x);
    if (ax > amax) amax = ax;
  }
  *amax_out = amax;
}

/* ---- counter-based draw ------------------------------------------------------------------------- */

static uint64_t mix64(uint64_t z) {
  z ^= z >> 30;
  z *= 0xBF58476D1CE4E5B9ull;
  z ^= z >> 27;
  z *= 0x94D049BB133111EBull;
  z ^= z >> 31;
  return z;
}

static uint32_t draw_u32(uint32_t k0, uint32_t k1, uint64_t gid) {
  uint32_t x = (uint32_t)(gid & 0xFFFFFFFFull) ^ k0;
  x += (uint32_t)(gid >> 32) * 0x9E3779B9u;
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

/* ---- Sec. 5.1: the estimator on one group ------------------------------------------------------- */

/* magnitudes m[4] (float32, >= 0) and the uniform u -> recorded positions and the common magnitude h */
static void mvue_select(const float m[4], float u, int* pos0, int* pos1, float* h_out) {
  float a = fmaxf(m[0], m[1]), b = fminf(m[0], m[1]);
  float cc = fmaxf(m[2], m[3]), d = fminf(m[2], m[3]);
  float mx = fmaxf(a, cc), mid = fminf(a, cc);
  volatile float bd = b + d;
  volatile float Lo = bd + mid;                  /* the three non-maximal magnitudes */
  float clamp = Lo == 0.0f ? mx : Lo;
  float l[4];
  for (int i = 0; i < 4; i++) l[i] = fminf(m[i], clamp);
  volatile float P0 = l[0];
  volatile float P1 = P0 + l[1];
  volatile float P2 = P1 + l[2];
  volatile float L = P2 + l[3];
  volatile float h = 0.5f * L;
  volatile float tau0 = u * h;
  volatile float tau1 = tau0 + h;
  int i0 = (P0 <= tau0) + (P1 <= tau0) + (P2 <= tau0);
  int i1 = (P0 <= tau1) + (P1 <= tau1) + (P2 <= tau1);
  int p0 = i0 < 2 ? i0 : 2;
  int p1 = i1 > p0 + 1 ? i1 : p0 + 1;
  if (p1 > 3) p1 = 3;
  *pos0 = p0;
  *pos1 = p1;
  *h_out = h;
}

/*
 * dy: (T, O) stored patterns, row-major with leading dimension O (uint16 for bf16, uint8 for the 8-bit
 * formats).  Group (k, o) = tokens 4k..4k+3 of channel o, group id (first_group + k) * O + o.
 * vals: (O, T/2) recorded values in ascending position order; meta: (O, T/8), the nibble
 * pos0 | pos1 << 2 of group k in byte k / 2, even k in the low nibble.  8-bit formats store theta / 2.
 */
void orc_mvue_pack(const void* dy, int64_t T, int64_t O, int fmt, uint64_t seed, uint64_t offset, uint64_t first_group,
                   void* vals, uint8_t* meta) {
  uint64_t key = mix64(seed ^ mix64(offset + 0x9E3779B97F4A7C15ull));
  uint32_t k0 = (uint32_t)key, k1 = (uint32_t)(key >> 32);
  int64_t G = T / 4;
  memset(meta, 0, (size_t)(O * (T / 8)));
#pragma omp parallel for schedule(static)
  for (int64_t o = 0; o < O; o++) {
    for (int64_t k = 0; k < G; k++) {
      uint64_t gid = (first_group + (uint64_t)k) * (uint64_t)O + (uint64_t)o;
      uint32_t x = draw_u32(k0, k1, gid);
      float u = (float)(x >> 8) * 0x1p-24f;
      float m[4], h;
      int p[2];
      if (fmt == ORC_BF16) {
        const uint16_t* g = (const uint16_t*)dy;
        uint16_t c[4];
        for (int i = 0; i < 4; i++) {
          c[i] = g[(4 * k + i) * O + o];
          m[i] = fabsf(bf16_to_f32(c[i]));
        }
        mvue_select(m, u, &p[0], &p[1], &h);
        uint16_t hq = f32_to_bf16_rne(h);
        uint16_t* out = (uint16_t*)vals + o * (T / 2) + 2 * k;
        for (int j = 0; j < 2; j++) {
          uint16_t code = c[p[j]];
          float mi = m[p[j]];
          out[j] = (mi > h || mi == 0.0f) ? code : (uint16_t)((code & 0x8000u) | hq);
        }
      } else {
        const uint8_t* g = (const uint8_t*)dy;
        uint8_t c[4];
        for (int i = 0; i < 4; i++) {
          c[i] = g[(4 * k + i) * O + o];
          m[i] = fabsf(fmt == ORC_E4M3 ? e4m3_to_f32(c[i]) : e5m2_to_f32(c[i]));
        }
        mvue_select(m, u, &p[0], &p[1], &h);
        volatile float half_h = 0.5f * h;
        uint8_t hq = fmt == ORC_E4M3 ? f32_to_e4m3(half_h) : f32_to_e5m2(half_h);
        uint8_t* out = (uint8_t*)vals + o * (T / 2) + 2 * k;
        for (int j = 0; j < 2; j++) {
          uint8_t code = c[p[j]];
          float mi = m[p[j]];
          volatile float half_m = 0.5f * mi;
          uint8_t own = (uint8_t)((code & 0x80u) | (fmt == ORC_E4M3 ? f32_to_e4m3(half_m) : f32_to_e5m2(half_m)));
          out[j] = (mi > h || mi == 0.0f) ? own : (uint8_t)((code & 0x80u) | hq);
        }
      }
      uint8_t nib = (uint8_t)(p[0] | (p[1] << 2));
      meta[o * (T / 8) + k / 2] |= (uint8_t)(nib << (4 * (k & 1)));
    }
  }
}

/* ---- packed -> dense ------------------------------------------------------------------------------ */

/* vals (R, K/2), meta (R, K/8) row-major -> dense (R, K) float64 holding the exact stored values; when
   the two positions of a group coincide the second value wins. */
void orc_decode_packed(const void* vals, const uint8_t* meta, int64_t R, int64_t K, int fmt, double* dense) {
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < R; r++) {
    for (int64_t g = 0; g < K / 4; g++) {
      uint8_t nib = (meta[r * (K / 8) + g / 2] >> (4 * (g & 1))) & 0xF;
      int p0 = nib & 3, p1 = (nib >> 2) & 3;
      double v[2];
      for (int j = 0; j < 2; j++) {
        if (fmt == ORC_BF16) v[j] = bf16_to_f32(((const uint16_t*)vals)[r * (K / 2) + 2 * g + j]);
        else {
          uint8_t c = ((const uint8_t*)vals)[r * (K / 2) + 2 * g + j];
          v[j] = fmt == ORC_E4M3 ? e4m3_to_f32(c) : e5m2_to_f32(c);
        }
      }
      double* d = dense + r * K + 4 * g;
      d[0] = d[1] = d[2] = d[3] = 0.0;
      d[p0] = v[0];
      d[p1] = v[1];
    }
  }
}
