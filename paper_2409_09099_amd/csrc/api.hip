// C ABI of the library: argument validation on the host, then kernel launches on the caller's
// stream.  Nothing here allocates, frees or synchronises.
#include "common.h"

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <vector>

namespace sste {

static thread_local char g_err[512] = "";

int fail(int status, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
  return status;
}
void clear_error() { g_err[0] = 0; }

// ---- per-kernel timing --------------------------------------------------------------------------
static std::mutex g_timing_mu;
static bool g_timing_on = false;
static std::vector<TimingSlot> g_slots;
static std::vector<int> g_slot_kind;
static size_t g_slots_used = 0;

TimingSlot* timing_slot(int kind) {
  if (!g_timing_on) return nullptr;
  std::lock_guard<std::mutex> lk(g_timing_mu);
  if (!g_timing_on || g_slots_used >= g_slots.size()) return nullptr;
  g_slot_kind[g_slots_used] = kind;
  return &g_slots[g_slots_used++];
}

static uint64_t mix64(uint64_t z) {
  z ^= z >> 30;
  z *= 0xBF58476D1CE4E5B9ull;
  z ^= z >> 27;
  z *= 0x94D049BB133111EBull;
  z ^= z >> 31;
  return z;
}

RngKey derive_key(uint64_t seed, uint64_t offset) {
  uint64_t k = mix64(seed ^ mix64(offset + 0x9E3779B97F4A7C15ull));
  RngKey r;
  r.k0 = (uint32_t)k;
  r.k1 = (uint32_t)(k >> 32);
  r.first_group = 0;
  return r;
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
static bool good_scale(float v) { return std::isfinite(v) && v > 0.0f; }
static bool good_dtype(int d) { return d == SSTE_BF16 || d == SSTE_F8E4M3; }
// the backward calls also take e5m2 output gradients (against e4m3 activations / weights)
static bool good_grad_dtype(int d) { return good_dtype(d) || d == SSTE_F8E5M2; }
static bool is_8bit(int d) { return d == SSTE_F8E4M3 || d == SSTE_F8E5M2; }
static int elems_per_16B(int d) { return is_8bit(d) ? 16 : 8; }

static int hip_status(hipError_t e, const char* what) {
  if (e == hipSuccess) return SSTE_OK;
  return fail(SSTE_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

}  // namespace sste

using namespace sste;

extern "C" {

int sste_version(void) { return 100; }

int sste_timing_begin(int max_launches) {
  clear_error();
  if (max_launches <= 0 || max_launches > (1 << 20)) return fail(SSTE_ERR_VALUE, "timing_begin: max_launches out of range");
  std::lock_guard<std::mutex> lk(g_timing_mu);
  if (g_timing_on) return fail(SSTE_ERR_VALUE, "timing_begin: timing is already on");
  g_slots.resize((size_t)max_launches);
  g_slot_kind.assign((size_t)max_launches, -1);
  for (size_t i = 0; i < g_slots.size(); i++) {
    hipError_t e = hipEventCreate(&g_slots[i].start);
    if (e == hipSuccess) e = hipEventCreate(&g_slots[i].stop);
    if (e != hipSuccess) {
      g_slots.resize(0);
      return fail(SSTE_ERR_HIP, "timing_begin: hipEventCreate: %s", hipGetErrorString(e));
    }
  }
  g_slots_used = 0;
  g_timing_on = true;
  return SSTE_OK;
}

int sste_timing_end(double* total_ms, int* launches) {
  clear_error();
  std::lock_guard<std::mutex> lk(g_timing_mu);
  if (!g_timing_on) return fail(SSTE_ERR_VALUE, "timing_end: timing is not on");
  g_timing_on = false;
  for (int k = 0; k < SSTE_K_COUNT; k++) {
    if (total_ms) total_ms[k] = 0.0;
    if (launches) launches[k] = 0;
  }
  int status = SSTE_OK;
  for (size_t i = 0; i < g_slots_used; i++) {
    float ms = 0.0f;
    hipError_t e = hipEventSynchronize(g_slots[i].stop);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, g_slots[i].start, g_slots[i].stop);
    if (e != hipSuccess) { status = fail(SSTE_ERR_HIP, "timing_end: %s", hipGetErrorString(e)); break; }
    int k = g_slot_kind[i];
    if (k >= 0 && k < SSTE_K_COUNT) {
      if (total_ms) total_ms[k] += (double)ms;
      if (launches) launches[k] += 1;
    }
  }
  for (size_t i = 0; i < g_slots.size(); i++) {
    (void)hipEventDestroy(g_slots[i].start);
    (void)hipEventDestroy(g_slots[i].stop);
  }
  g_slots.resize(0);
  g_slot_kind.resize(0);
  g_slots_used = 0;
  return status;
}

const char* sste_last_error(void) { return g_err; }

// Per-item argument checks shared by the single-tensor and the batch entry points.
static int check_pack_args(const char* who, const void* W, int64_t O, int64_t I, int64_t ldw, float beta, int val_dtype,
                           float val_scale, const void* vals, const void* meta, int ldw_multiple = 8) {
  if (O < 0 || I < 0) return fail(SSTE_ERR_SHAPE, "%s: negative size O=%lld I=%lld", who, (long long)O, (long long)I);
  if (I % 8 != 0) return fail(SSTE_ERR_SHAPE, "%s: I=%lld is not a multiple of 8 (whole groups of 4, two per metadata byte)", who, (long long)I);
  if (!good_dtype(val_dtype)) return fail(SSTE_ERR_DTYPE, "%s: unknown val_dtype %d", who, val_dtype);
  if (!good_scale(beta)) return fail(SSTE_ERR_VALUE, "%s: beta must be finite and > 0", who);
  if (!good_scale(val_scale)) return fail(SSTE_ERR_VALUE, "%s: val_scale must be finite and > 0", who);
  if (val_dtype == SSTE_BF16 && val_scale != 1.0f) return fail(SSTE_ERR_VALUE, "%s: val_scale must be 1 for bf16 values", who);
  if (I % (val_dtype == SSTE_F8E4M3 ? 128 : 64) != 0)
    return fail(SSTE_ERR_UNSUPPORTED, "%s: I=%lld must be a multiple of %d for this value type", who, (long long)I, val_dtype == SSTE_F8E4M3 ? 128 : 64);
  if (ldw < I) return fail(SSTE_ERR_SHAPE, "%s: ldw=%lld < I=%lld", who, (long long)ldw, (long long)I);
  if (product_reaches(O, ldw, 1ll << 40)) return fail(SSTE_ERR_UNSUPPORTED, "%s: more than 2^40 weights", who);
  if (ldw % ldw_multiple != 0) return fail(SSTE_ERR_ALIGN, "%s: ldw=%lld is not a multiple of %d", who, (long long)ldw, ldw_multiple);
  bool empty = (O == 0 || I == 0);
  if (!empty && (!W || !vals || !meta)) return fail(SSTE_ERR_NULL, "%s: NULL W, vals or meta", who);
  if (!aligned16(W) || !aligned16(vals)) return fail(SSTE_ERR_ALIGN, "%s: W and vals must be 16-byte aligned", who);
  return SSTE_OK;
}

// device-side table item of sste_project_pack_batch; must match PackTableItem in prune_pack.hip
struct PackTableItemHost {
  const void* W;
  void* vals;
  void* meta;
  int64_t O;
  int64_t ldw_bytes;
  int64_t first_block;
  int32_t steps;
  float beta;
  float val_scale;
  int32_t pad;
};
static_assert(sizeof(PackTableItemHost) == SSTE_PACK_TABLE_ITEM_BYTES, "table item size is part of the C ABI");

int sste_project_pack(const void* W, int64_t O, int64_t I, int64_t ldw, float beta, int val_dtype, float val_scale,
                      void* vals, void* meta, float* amax_out, void* hip_stream) {
  return sste_project_pack_gamma(W, O, I, ldw, beta, 0.0f, val_dtype, val_scale, vals, meta, amax_out, hip_stream);
}

int sste_project_pack_gamma(const void* W, int64_t O, int64_t I, int64_t ldw, float beta, float gamma, int val_dtype,
                            float val_scale, void* vals, void* meta, float* amax_out, void* hip_stream) {
  clear_error();
  int st = check_pack_args("project_pack", W, O, I, ldw, beta, val_dtype, val_scale, vals, meta);
  if (st != SSTE_OK) return st;
  if (!(gamma >= 0.0f && gamma <= 1.0f)) return fail(SSTE_ERR_VALUE, "project_pack: gamma must lie in [0, 1]");
  if (amax_out && (reinterpret_cast<uintptr_t>(amax_out) & 3u)) return fail(SSTE_ERR_ALIGN, "project_pack: amax_out must be 4-byte aligned");
  return hip_status(launch_project_pack(W, O, I, ldw, beta, gamma, val_dtype, val_scale, vals, meta, amax_out, (hipStream_t)hip_stream),
                    "project_pack launch");
}

static int check_update_args(const char* who, const void* W, int w_dtype, int64_t O, int64_t I, int64_t ldw, const float* G,
                             int64_t ldg, float beta, int val_dtype, float val_scale, const void* vals, const void* meta) {
  if (w_dtype != SSTE_BF16 && w_dtype != SSTE_F32) return fail(SSTE_ERR_DTYPE, "%s: w_dtype %d is neither bf16 nor float32", who, w_dtype);
  int st = check_pack_args(who, W, O, I, ldw, beta, val_dtype, val_scale, vals, meta, w_dtype == SSTE_F32 ? 4 : 8);
  if (st != SSTE_OK) return st;
  if (ldg < I) return fail(SSTE_ERR_SHAPE, "%s: ldg=%lld < I=%lld", who, (long long)ldg, (long long)I);
  if (ldg % 4 != 0) return fail(SSTE_ERR_ALIGN, "%s: ldg=%lld is not a multiple of 4", who, (long long)ldg);
  if (O > 0 && I > 0 && !G) return fail(SSTE_ERR_NULL, "%s: NULL G", who);
  if (!aligned16(G)) return fail(SSTE_ERR_ALIGN, "%s: G must be 16-byte aligned", who);
  return SSTE_OK;
}

int sste_sgd_project_pack(void* W, int w_dtype, int64_t O, int64_t I, int64_t ldw, const float* G, int64_t ldg, float alpha,
                          float beta, int val_dtype, float val_scale, void* vals, void* meta, void* hip_stream) {
  clear_error();
  int st = check_update_args("sgd_project_pack", W, w_dtype, O, I, ldw, G, ldg, beta, val_dtype, val_scale, vals, meta);
  if (st != SSTE_OK) return st;
  if (!std::isfinite(alpha)) return fail(SSTE_ERR_VALUE, "sgd_project_pack: alpha must be finite");
  return hip_status(launch_sgd_project_pack(W, w_dtype == SSTE_F32, O, I, ldw, G, ldg, alpha, beta, val_dtype, val_scale, vals, meta,
                                            (hipStream_t)hip_stream),
                    "sgd_project_pack launch");
}

// device-side table item of sste_sgd_project_pack_batch; must match UpdateTableItem in prune_pack.hip
struct UpdateTableItemHost {
  void* W;
  const float* G;
  void* vals;
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
static_assert(sizeof(UpdateTableItemHost) == SSTE_UPDATE_TABLE_ITEM_BYTES, "table item size is part of the C ABI");

int sste_sgd_project_pack_batch_prepare(const sste_update_item* items, int n_items, int w_dtype, int val_dtype, void* table_host,
                                        int64_t* total_blocks_out) {
  clear_error();
  if (n_items < 0) return fail(SSTE_ERR_SHAPE, "sgd_project_pack_batch_prepare: n_items=%d", n_items);
  if (!total_blocks_out || (n_items > 0 && (!items || !table_host)))
    return fail(SSTE_ERR_NULL, "sgd_project_pack_batch_prepare: NULL items, table_host or total_blocks_out");
  if (w_dtype != SSTE_BF16 && w_dtype != SSTE_F32) return fail(SSTE_ERR_DTYPE, "sgd_project_pack_batch_prepare: w_dtype %d is neither bf16 nor float32", w_dtype);
  if (!good_dtype(val_dtype)) return fail(SSTE_ERR_DTYPE, "sgd_project_pack_batch_prepare: unknown val_dtype %d", val_dtype);
  UpdateTableItemHost* out = (UpdateTableItemHost*)table_host;
  int64_t blocks = 0;
  for (int i = 0; i < n_items; i++) {
    const sste_update_item& it = items[i];
    char who[64];
    snprintf(who, sizeof who, "sgd_project_pack_batch_prepare item %d", i);
    int st = check_update_args(who, it.W, w_dtype, it.O, it.I, it.ldw, it.G, it.ldg, it.beta, val_dtype, it.val_scale, it.vals, it.meta);
    if (st != SSTE_OK) return st;
    int64_t steps = it.I / (val_dtype == SSTE_F8E4M3 ? 128 : 64);
    if (steps > 0x7FFFFFFFll) return fail(SSTE_ERR_UNSUPPORTED, "%s: I too large", who);
    UpdateTableItemHost t{};
    t.W = it.W;
    t.G = it.G;
    t.vals = it.vals;
    t.meta = it.meta;
    t.O = it.O;
    t.ldw_bytes = it.ldw * (w_dtype == SSTE_F32 ? 4 : 2);
    t.ldg = it.ldg;
    t.first_block = blocks;
    t.steps = (int32_t)(steps > 0 ? steps : 1);       // an empty item owns no block; the divisor only has to be non-zero
    t.beta = it.beta;
    t.val_scale = it.val_scale;
    out[i] = t;
    blocks += ((it.O + 15) / 16) * steps;
  }
  *total_blocks_out = blocks;
  return SSTE_OK;
}

int sste_sgd_project_pack_batch(const void* table_device, int n_items, int64_t total_blocks, int w_dtype, int val_dtype, float alpha,
                                void* hip_stream) {
  clear_error();
  if (n_items < 0 || total_blocks < 0) return fail(SSTE_ERR_SHAPE, "sgd_project_pack_batch: negative count");
  if (w_dtype != SSTE_BF16 && w_dtype != SSTE_F32) return fail(SSTE_ERR_DTYPE, "sgd_project_pack_batch: w_dtype %d is neither bf16 nor float32", w_dtype);
  if (!good_dtype(val_dtype)) return fail(SSTE_ERR_DTYPE, "sgd_project_pack_batch: unknown val_dtype %d", val_dtype);
  if (!std::isfinite(alpha)) return fail(SSTE_ERR_VALUE, "sgd_project_pack_batch: alpha must be finite");
  if (n_items > 0 && !table_device) return fail(SSTE_ERR_NULL, "sgd_project_pack_batch: NULL table");
  if (!aligned16(table_device)) return fail(SSTE_ERR_ALIGN, "sgd_project_pack_batch: the table must be 16-byte aligned");
  if ((total_blocks + 3) / 4 > 0x7FFFFFFFll) return fail(SSTE_ERR_UNSUPPORTED, "sgd_project_pack_batch: too many blocks for one grid");
  return hip_status(launch_sgd_project_pack_batch(table_device, n_items, total_blocks, w_dtype == SSTE_F32, val_dtype, alpha,
                                                  (hipStream_t)hip_stream),
                    "sgd_project_pack_batch launch");
}

int sste_project_pack_batch_prepare(const sste_pack_item* items, int n_items, int val_dtype, void* table_host,
                                    int64_t* total_blocks_out) {
  clear_error();
  if (n_items < 0) return fail(SSTE_ERR_SHAPE, "project_pack_batch_prepare: n_items=%d", n_items);
  if (!total_blocks_out || (n_items > 0 && (!items || !table_host)))
    return fail(SSTE_ERR_NULL, "project_pack_batch_prepare: NULL items, table_host or total_blocks_out");
  if (!good_dtype(val_dtype)) return fail(SSTE_ERR_DTYPE, "project_pack_batch_prepare: unknown val_dtype %d", val_dtype);
  PackTableItemHost* out = (PackTableItemHost*)table_host;
  int64_t blocks = 0;
  for (int i = 0; i < n_items; i++) {
    const sste_pack_item& it = items[i];
    char who[64];
    snprintf(who, sizeof who, "project_pack_batch_prepare item %d", i);
    int st = check_pack_args(who, it.W, it.O, it.I, it.ldw, it.beta, val_dtype, it.val_scale, it.vals, it.meta);
    if (st != SSTE_OK) return st;
    int64_t steps = it.I / (val_dtype == SSTE_F8E4M3 ? 128 : 64);
    if (steps > 0x7FFFFFFFll) return fail(SSTE_ERR_UNSUPPORTED, "%s: I too large", who);
    PackTableItemHost t{};
    t.W = it.W;
    t.vals = it.vals;
    t.meta = it.meta;
    t.O = it.O;
    t.ldw_bytes = it.ldw * 2;
    t.first_block = blocks;
    t.steps = (int32_t)(steps > 0 ? steps : 1);       // an empty item owns no block; the divisor only has to be non-zero
    t.beta = it.beta;
    t.val_scale = it.val_scale;
    out[i] = t;
    blocks += ((it.O + 15) / 16) * steps;
  }
  *total_blocks_out = blocks;
  return SSTE_OK;
}

int sste_project_pack_batch(const void* table_device, int n_items, int64_t total_blocks, int val_dtype, void* hip_stream) {
  clear_error();
  if (n_items < 0 || total_blocks < 0) return fail(SSTE_ERR_SHAPE, "project_pack_batch: negative count");
  if (!good_dtype(val_dtype)) return fail(SSTE_ERR_DTYPE, "project_pack_batch: unknown val_dtype %d", val_dtype);
  if (n_items > 0 && !table_device) return fail(SSTE_ERR_NULL, "project_pack_batch: NULL table");
  if (!aligned16(table_device)) return fail(SSTE_ERR_ALIGN, "project_pack_batch: the table must be 16-byte aligned");
  if ((total_blocks + 3) / 4 > 0x7FFFFFFFll) return fail(SSTE_ERR_UNSUPPORTED, "project_pack_batch: too many blocks for one grid");
  return hip_status(launch_project_pack_batch(table_device, n_items, total_blocks, val_dtype, (hipStream_t)hip_stream),
                    "project_pack_batch launch");
}

int sste_linear_fwd(const void* X, int64_t T, int64_t I, int64_t ldx, int dtype, float x_scale, const void* vals,
                    const void* meta, int64_t O, float w_scale, void* Z, int64_t ldz, void* hip_stream) {
  return sste_linear_fwd_ex(X, T, I, ldx, dtype, x_scale, vals, meta, O, w_scale, Z, ldz, SSTE_BF16, 1.0f, nullptr, hip_stream);
}

int sste_linear_fwd_ex(const void* X, int64_t T, int64_t I, int64_t ldx, int dtype, float x_scale, const void* vals,
                       const void* meta, int64_t O, float w_scale, void* Z, int64_t ldz, int z_dtype, float z_scale,
                       float* amax_out, void* hip_stream) {
  clear_error();
  if (T < 0 || I < 0 || O < 0) return fail(SSTE_ERR_SHAPE, "linear_fwd: negative size");
  if (!good_dtype(dtype)) return fail(SSTE_ERR_DTYPE, "linear_fwd: unknown dtype %d", dtype);
  if (!good_dtype(z_dtype)) return fail(SSTE_ERR_DTYPE, "linear_fwd: z_dtype %d is neither bf16 nor e4m3", z_dtype);
  if (I % 8 != 0) return fail(SSTE_ERR_SHAPE, "linear_fwd: I=%lld is not a multiple of 8", (long long)I);
  if (!good_scale(x_scale) || !good_scale(w_scale) || !good_scale(z_scale)) return fail(SSTE_ERR_VALUE, "linear_fwd: scales must be finite and > 0");
  const bool z8 = z_dtype == SSTE_F8E4M3;
  if (!z8 && z_scale != 1.0f) return fail(SSTE_ERR_VALUE, "linear_fwd: z_scale must be 1 for a bf16 output");
  if (z8 && !amax_out) return fail(SSTE_ERR_NULL, "linear_fwd: an e4m3 output needs amax_out (the next scale is derived from it)");
  if (reinterpret_cast<uintptr_t>(amax_out) & 3u) return fail(SSTE_ERR_ALIGN, "linear_fwd: amax_out must be 4-byte aligned");
  int kmult = dtype == SSTE_F8E4M3 ? 128 : 64;
  if (I % kmult != 0) return fail(SSTE_ERR_UNSUPPORTED, "linear_fwd: I=%lld must be a multiple of %d for this element type", (long long)I, kmult);
  const int zmult = z8 ? 16 : 8;
  if (O % zmult != 0) return fail(SSTE_ERR_UNSUPPORTED, "linear_fwd: O=%lld must be a multiple of %d", (long long)O, zmult);
  if (ldx < I || ldz < O) return fail(SSTE_ERR_SHAPE, "linear_fwd: leading dimension smaller than the row length");
  if (ldx % elems_per_16B(dtype) != 0 || ldz % zmult != 0) return fail(SSTE_ERR_ALIGN, "linear_fwd: ldx / ldz break the 16-byte row rule");
  bool empty = (T == 0 || O == 0);
  if (!empty && (!Z || (I > 0 && (!X || !vals || !meta)))) return fail(SSTE_ERR_NULL, "linear_fwd: NULL X, vals, meta or Z");
  if (!aligned16(X) || !aligned16(vals) || !aligned16(meta) || !aligned16(Z))
    return fail(SSTE_ERR_ALIGN, "linear_fwd: X, vals, meta and Z must be 16-byte aligned");
  if (!linear_fwd_supported(T, I, ldx, O, dtype)) return fail(SSTE_ERR_UNSUPPORTED, "linear_fwd: a tile of this problem does not fit 32-bit offsets");
  const float real_scale = x_scale * w_scale;                 // accumulator -> the tensor's real units
  const float store_scale = z8 ? real_scale / z_scale : real_scale;
  return hip_status(launch_linear_fwd(X, T, I, ldx, dtype, store_scale, vals, meta, O, Z, ldz, z_dtype, real_scale, amax_out,
                                      (hipStream_t)hip_stream),
                    "linear_fwd launch");
}

int sste_linear_fwd_act(const void* X, int64_t T, int64_t I, int64_t ldx, int dtype, float x_scale, const void* vals,
                        const void* meta, int64_t O, float w_scale, int act, void* H, int64_t ldh, void* A, int64_t lda,
                        int a_dtype, float a_scale, float* amax_out, void* hip_stream) {
  clear_error();
  if (T < 0 || I < 0 || O < 0) return fail(SSTE_ERR_SHAPE, "linear_fwd_act: negative size");
  if (!good_dtype(dtype)) return fail(SSTE_ERR_DTYPE, "linear_fwd_act: unknown dtype %d", dtype);
  if (!good_dtype(a_dtype)) return fail(SSTE_ERR_DTYPE, "linear_fwd_act: a_dtype %d is neither bf16 nor e4m3", a_dtype);
  if (act != SSTE_ACT_GELU_TANH) return fail(SSTE_ERR_VALUE, "linear_fwd_act: unknown activation %d", act);
  if (I % 8 != 0) return fail(SSTE_ERR_SHAPE, "linear_fwd_act: I=%lld is not a multiple of 8", (long long)I);
  if (!good_scale(x_scale) || !good_scale(w_scale) || !good_scale(a_scale)) return fail(SSTE_ERR_VALUE, "linear_fwd_act: scales must be finite and > 0");
  const bool a8 = a_dtype == SSTE_F8E4M3;
  if (!a8 && a_scale != 1.0f) return fail(SSTE_ERR_VALUE, "linear_fwd_act: a_scale must be 1 for a bf16 output");
  if (a8 && !amax_out) return fail(SSTE_ERR_NULL, "linear_fwd_act: an e4m3 output needs amax_out (the next scale is derived from it)");
  if (!a8 && amax_out) return fail(SSTE_ERR_VALUE, "linear_fwd_act: amax_out goes with an e4m3 output only");
  if (reinterpret_cast<uintptr_t>(amax_out) & 3u) return fail(SSTE_ERR_ALIGN, "linear_fwd_act: amax_out must be 4-byte aligned");
  int kmult = dtype == SSTE_F8E4M3 ? 128 : 64;
  if (I % kmult != 0) return fail(SSTE_ERR_UNSUPPORTED, "linear_fwd_act: I=%lld must be a multiple of %d for this element type", (long long)I, kmult);
  if (O % 8 != 0) return fail(SSTE_ERR_UNSUPPORTED, "linear_fwd_act: O=%lld must be a multiple of 8", (long long)O);
  if (ldx < I || lda < O || (H && ldh < O)) return fail(SSTE_ERR_SHAPE, "linear_fwd_act: leading dimension smaller than the row length");
  if (ldx % elems_per_16B(dtype) != 0 || lda % 8 != 0 || (H && ldh % 8 != 0)) return fail(SSTE_ERR_ALIGN, "linear_fwd_act: leading dimensions break the row rule");
  bool empty = (T == 0 || O == 0);
  if (!empty && (!A || (I > 0 && (!X || !vals || !meta)))) return fail(SSTE_ERR_NULL, "linear_fwd_act: NULL X, vals, meta or A");
  if (!aligned16(X) || !aligned16(vals) || !aligned16(meta) || !aligned16(H) || (reinterpret_cast<uintptr_t>(A) & (a8 ? 7u : 15u)))
    return fail(SSTE_ERR_ALIGN, "linear_fwd_act: X, vals, meta, H must be 16-byte aligned, A 16-byte (bf16) / 8-byte (e4m3)");
  if (!linear_fwd_supported(T, I, ldx, O, dtype)) return fail(SSTE_ERR_UNSUPPORTED, "linear_fwd_act: a tile of this problem does not fit 32-bit offsets");
  const float inv = 1.0f / a_scale;
  return hip_status(launch_linear_fwd_act(X, T, I, ldx, dtype, x_scale * w_scale, vals, meta, O, H, ldh, A, lda, a_dtype, inv, amax_out,
                                          (hipStream_t)hip_stream),
                    "linear_fwd_act launch");
}

// ---- delayed scaling (host only) ----------------------------------------------------------------------
void sste_amax_history_init(sste_amax_history* h, int length) {
  if (!h) return;
  if (length < 1) length = 1;
  if (length > SSTE_AMAX_HISTORY_MAX) length = SSTE_AMAX_HISTORY_MAX;
  for (int i = 0; i < SSTE_AMAX_HISTORY_MAX; i++) h->window[i] = 0.0f;
  h->length = length;
  h->next = 0;
}

float sste_amax_history_push(sste_amax_history* h, float amax, float format_max) {
  if (!h || h->length < 1 || h->length > SSTE_AMAX_HISTORY_MAX || !(format_max > 0.0f)) return 1.0f;
  if (std::isfinite(amax) && amax >= 0.0f) {                   // anything else leaves the window as it is
    h->window[h->next] = amax;
    h->next = (h->next + 1) % h->length;
  }
  float m = 0.0f;
  for (int i = 0; i < h->length; i++) m = h->window[i] > m ? h->window[i] : m;
  return m > 0.0f ? m / format_max : 1.0f;
}

static int wgrad_shape_check(int64_t T, int64_t O, int64_t I, int dtype, const char* who) {
  if (T < 0 || O < 0 || I < 0) return fail(SSTE_ERR_SHAPE, "%s: negative size", who);
  if (!good_grad_dtype(dtype)) return fail(SSTE_ERR_DTYPE, "%s: unknown dtype %d", who, dtype);
  if (T % 4 != 0) return fail(SSTE_ERR_SHAPE, "%s: T=%lld is not a multiple of 4 (groups of four tokens)", who, (long long)T);
  int kmult = is_8bit(dtype) ? 128 : 64, nmult = elems_per_16B(dtype);
  if (T % kmult != 0) return fail(SSTE_ERR_UNSUPPORTED, "%s: T=%lld must be a multiple of %d for this element type", who, (long long)T, kmult);
  if (O % nmult != 0 || I % nmult != 0) return fail(SSTE_ERR_UNSUPPORTED, "%s: O and I must be multiples of %d", who, nmult);
  return SSTE_OK;
}

int sste_wgrad_plan_override(int mi, int ni, int splits) {
  clear_error();
  if (!wgrad_plan_override(mi, ni, splits))
    return fail(SSTE_ERR_VALUE, "wgrad_plan_override: tile (%d, %d) is none of (8,4), (6,3), (8,3), (0,0), or splits=%d is outside 0..32", mi, ni, splits);
  return SSTE_OK;
}

size_t sste_wgrad_workspace_bytes(int64_t T, int64_t O, int64_t I, int dtype) {
  if (wgrad_shape_check(T, O, I, dtype, "wgrad_workspace_bytes") != SSTE_OK) return 0;
  return wgrad_workspace_bytes(T, O, I, dtype);
}

int sste_linear_dgrad(const void* dY, int64_t T, int64_t O, int64_t lddy, int dtype, float dy_scale, const void* vals,
                      const void* meta, int64_t I, float w_scale, void* dX, int64_t lddx, void* hip_stream) {
  return sste_linear_dgrad_act(dY, T, O, lddy, dtype, dy_scale, vals, meta, I, w_scale, SSTE_ACT_NONE, nullptr, 0, dX, lddx, hip_stream);
}

int sste_linear_dgrad_act(const void* dY, int64_t T, int64_t O, int64_t lddy, int dtype, float dy_scale, const void* vals,
                          const void* meta, int64_t I, float w_scale, int act, const void* H, int64_t ldh, void* dX,
                          int64_t lddx, void* hip_stream) {
  clear_error();
  if (act != SSTE_ACT_NONE && act != SSTE_ACT_GELU_TANH) return fail(SSTE_ERR_VALUE, "linear_dgrad: unknown activation %d", act);
  if (act == SSTE_ACT_NONE) {
    H = nullptr;
    ldh = 0;
  } else {
    if (T > 0 && I > 0 && !H) return fail(SSTE_ERR_NULL, "linear_dgrad: the activation's backward needs the stored pre-activation H");
    if (ldh < I) return fail(SSTE_ERR_SHAPE, "linear_dgrad: ldh < I");
    if (ldh % 8 != 0 || !aligned16(H)) return fail(SSTE_ERR_ALIGN, "linear_dgrad: H must be 16-byte aligned with ldh a multiple of 8");
  }
  if (T < 0 || I < 0 || O < 0) return fail(SSTE_ERR_SHAPE, "linear_dgrad: negative size");
  if (!good_grad_dtype(dtype)) return fail(SSTE_ERR_DTYPE, "linear_dgrad: unknown dtype %d", dtype);
  if (I % 8 != 0) return fail(SSTE_ERR_SHAPE, "linear_dgrad: I=%lld is not a multiple of 8", (long long)I);
  if (!good_scale(dy_scale) || !good_scale(w_scale)) return fail(SSTE_ERR_VALUE, "linear_dgrad: scales must be finite and > 0");
  const int ks = is_8bit(dtype) ? 128 : 64, e16 = elems_per_16B(dtype);
  if (I % ks != 0) return fail(SSTE_ERR_UNSUPPORTED, "linear_dgrad: I=%lld must be a multiple of %d", (long long)I, ks);
  if (O % e16 != 0) return fail(SSTE_ERR_UNSUPPORTED, "linear_dgrad: O=%lld must be a multiple of %d", (long long)O, e16);
  if (lddy < O || lddx < I) return fail(SSTE_ERR_SHAPE, "linear_dgrad: leading dimension smaller than the row length");
  if (lddy % e16 != 0 || lddx % 8 != 0) return fail(SSTE_ERR_ALIGN, "linear_dgrad: lddy / lddx break the 16-byte row rule");
  bool empty_out = (T == 0 || I == 0);
  if (!empty_out && !dX) return fail(SSTE_ERR_NULL, "linear_dgrad: NULL dX");
  if (!empty_out && O > 0 && (!dY || !vals || !meta)) return fail(SSTE_ERR_NULL, "linear_dgrad: NULL dY, vals or meta");
  if (!aligned16(dY) || !aligned16(vals) || !aligned16(dX)) return fail(SSTE_ERR_ALIGN, "linear_dgrad: dY, vals and dX must be 16-byte aligned");
  if (!linear_dgrad_supported(T, O, lddy, I, dtype)) return fail(SSTE_ERR_UNSUPPORTED, "linear_dgrad: problem too large for 32-bit tile offsets");
  return hip_status(launch_linear_dgrad(dY, T, O, lddy, dtype, dy_scale * w_scale, vals, meta, I, dX, lddx, H, ldh, (hipStream_t)hip_stream),
                    "linear_dgrad launch");
}

// Argument checks shared by sste_linear_wgrad and its variant that brings its own scratch.
static int check_wgrad_args(const char* who, const void* dY, int64_t T, int64_t O, int64_t lddy, int dtype, float dy_scale,
                            const void* X, int64_t I, int64_t ldx, float x_scale, const float* dW, int64_t lddw, int accumulate) {
  int st = wgrad_shape_check(T, O, I, dtype, who);
  if (st != SSTE_OK) return st;
  if (!good_scale(dy_scale) || !good_scale(x_scale)) return fail(SSTE_ERR_VALUE, "%s: scales must be finite and > 0", who);
  if (accumulate != 0 && accumulate != 1) return fail(SSTE_ERR_VALUE, "%s: accumulate must be 0 or 1", who);
  if (lddy < O || ldx < I || lddw < I) return fail(SSTE_ERR_SHAPE, "%s: leading dimension smaller than the row length", who);
  int e16 = elems_per_16B(dtype);
  if (lddy % e16 != 0 || ldx % e16 != 0 || lddw % 4 != 0) return fail(SSTE_ERR_ALIGN, "%s: leading dimensions break the 16-byte row rule", who);
  bool empty = (O == 0 || I == 0);
  if (!empty && (!dW || (T > 0 && (!dY || !X)))) return fail(SSTE_ERR_NULL, "%s: NULL dY, X or dW", who);
  if (!aligned16(dY) || !aligned16(X) || !aligned16(dW)) return fail(SSTE_ERR_ALIGN, "%s: dY, X and dW must be 16-byte aligned", who);
  if (!linear_wgrad_supported(T, O, I, ldx, dtype)) return fail(SSTE_ERR_UNSUPPORTED, "%s: this problem does not fit 32-bit tile offsets", who);
  return SSTE_OK;
}

int sste_linear_wgrad_noalloc(const void* dY, int64_t T, int64_t O, int64_t lddy, int dtype, float dy_scale, const void* X,
                              int64_t I, int64_t ldx, float x_scale, uint64_t seed, uint64_t offset, float* dW, int64_t lddw,
                              int accumulate, void* hip_stream) {
  clear_error();
  int st = check_wgrad_args("linear_wgrad_noalloc", dY, T, O, lddy, dtype, dy_scale, X, I, ldx, x_scale, dW, lddw, accumulate);
  if (st != SSTE_OK) return st;
  size_t need = sste_wgrad_workspace_bytes(T, O, I, dtype);
  if (need > (size_t)SSTE_NOALLOC_SCRATCH_BYTES)
    return fail(SSTE_ERR_WORKSPACE, "linear_wgrad_noalloc: this problem needs %zu bytes of scratch, the built-in scratch holds %zu; use sste_linear_wgrad with a workspace",
                need, (size_t)SSTE_NOALLOC_SCRATCH_BYTES);
  void* ws = nullptr;
  if (need > 0) {
    hipError_t e = hipSuccess;
    ws = noalloc_scratch(&e);
    if (!ws) return hip_status(e == hipSuccess ? hipErrorUnknown : e, "linear_wgrad_noalloc: address of the built-in scratch");
  }
  float scale = dy_scale * x_scale;
  if (is_8bit(dtype)) scale *= 2.0f;            // the sparsified 8-bit operand is stored halved
  return hip_status(launch_linear_wgrad(dY, T, O, lddy, dtype, X, I, ldx, scale, derive_key(seed, offset), dW, lddw, accumulate, ws,
                                        (hipStream_t)hip_stream),
                    "linear_wgrad_noalloc launch");
}

// first_token: global index of the tensor's first token row; whole groups, and (first_token / 4 + T / 4) * O < 2^64
static int check_first_token(const char* who, int64_t first_token, int64_t T, int64_t O) {
  if (first_token < 0 || first_token % 4 != 0) return fail(SSTE_ERR_SHAPE, "%s: first_token=%lld must be >= 0 and a multiple of 4", who, (long long)first_token);
  const unsigned __int128 last = ((unsigned __int128)(first_token / 4) + (unsigned __int128)(T / 4) + 1) * (unsigned __int128)(O > 0 ? O : 1);
  if (last >> 64) return fail(SSTE_ERR_UNSUPPORTED, "%s: group ids of this shard exceed 64 bits", who);
  return SSTE_OK;
}

int sste_linear_wgrad(const void* dY, int64_t T, int64_t O, int64_t lddy, int dtype, float dy_scale, const void* X,
                      int64_t I, int64_t ldx, float x_scale, uint64_t seed, uint64_t offset, float* dW, int64_t lddw,
                      int accumulate, void* workspace, size_t workspace_bytes, void* hip_stream) {
  return sste_linear_wgrad_at(dY, T, O, lddy, dtype, dy_scale, X, I, ldx, x_scale, seed, offset, 0, dW, lddw, accumulate, workspace,
                              workspace_bytes, hip_stream);
}

int sste_linear_wgrad_at(const void* dY, int64_t T, int64_t O, int64_t lddy, int dtype, float dy_scale, const void* X,
                         int64_t I, int64_t ldx, float x_scale, uint64_t seed, uint64_t offset, int64_t first_token,
                         float* dW, int64_t lddw, int accumulate, void* workspace, size_t workspace_bytes, void* hip_stream) {
  clear_error();
  int st = check_wgrad_args("linear_wgrad", dY, T, O, lddy, dtype, dy_scale, X, I, ldx, x_scale, dW, lddw, accumulate);
  if (st != SSTE_OK) return st;
  st = check_first_token("linear_wgrad", first_token, T, O);
  if (st != SSTE_OK) return st;
  size_t need = sste_wgrad_workspace_bytes(T, O, I, dtype);
  if (need > 0) {
    if (!workspace) return fail(SSTE_ERR_WORKSPACE, "linear_wgrad: workspace is NULL, %zu bytes needed", need);
    if (workspace_bytes < need) return fail(SSTE_ERR_WORKSPACE, "linear_wgrad: workspace has %zu bytes, %zu needed", workspace_bytes, need);
    if (!aligned16(workspace)) return fail(SSTE_ERR_ALIGN, "linear_wgrad: workspace must be 16-byte aligned");
  }
  float scale = dy_scale * x_scale;
  if (is_8bit(dtype)) scale *= 2.0f;            // the sparsified 8-bit operand is stored halved
  RngKey key = derive_key(seed, offset);
  key.first_group = (uint64_t)(first_token / 4);
  return hip_status(launch_linear_wgrad(dY, T, O, lddy, dtype, X, I, ldx, scale, key, dW, lddw, accumulate,
                                        workspace, (hipStream_t)hip_stream),
                    "linear_wgrad launch");
}

int sste_mvue_materialize(const void* dY, int64_t T, int64_t O, int64_t lddy, int dtype, uint64_t seed, uint64_t offset,
                          void* vals, void* meta, void* hip_stream) {
  return sste_mvue_materialize_at(dY, T, O, lddy, dtype, seed, offset, 0, vals, meta, hip_stream);
}

int sste_mvue_materialize_at(const void* dY, int64_t T, int64_t O, int64_t lddy, int dtype, uint64_t seed, uint64_t offset,
                             int64_t first_token, void* vals, void* meta, void* hip_stream) {
  clear_error();
  if (T < 0 || O < 0) return fail(SSTE_ERR_SHAPE, "mvue_materialize: negative size");
  if (!good_grad_dtype(dtype)) return fail(SSTE_ERR_DTYPE, "mvue_materialize: unknown dtype %d", dtype);
  if (T % 4 != 0) return fail(SSTE_ERR_SHAPE, "mvue_materialize: T=%lld is not a multiple of 4 (groups of four tokens)", (long long)T);
  if (T % (is_8bit(dtype) ? 128 : 64) != 0)
    return fail(SSTE_ERR_UNSUPPORTED, "mvue_materialize: T=%lld must be a multiple of %d for this element type", (long long)T, is_8bit(dtype) ? 128 : 64);
  if (lddy < O) return fail(SSTE_ERR_SHAPE, "mvue_materialize: lddy < O");
  // the kernel reads dY in 16-byte pieces of 8 (bf16) / 16 (8-bit) channels
  const int e16 = elems_per_16B(dtype);
  if (O % e16 != 0) return fail(SSTE_ERR_UNSUPPORTED, "mvue_materialize: O=%lld must be a multiple of %d", (long long)O, e16);
  if (lddy % e16 != 0) return fail(SSTE_ERR_ALIGN, "mvue_materialize: lddy=%lld is not a multiple of %d", (long long)lddy, e16);
  bool empty = (T == 0 || O == 0);
  if (!empty && (!dY || !vals || !meta)) return fail(SSTE_ERR_NULL, "mvue_materialize: NULL dY, vals or meta");
  if (!aligned16(dY) || !aligned16(vals) || (reinterpret_cast<uintptr_t>(meta) & 3u))
    return fail(SSTE_ERR_ALIGN, "mvue_materialize: dY and vals must be 16-byte aligned, meta 4-byte aligned");
  if (T / 8 > 65535) return fail(SSTE_ERR_UNSUPPORTED, "mvue_materialize: T=%lld exceeds 524280", (long long)T);
  int st = check_first_token("mvue_materialize", first_token, T, O);
  if (st != SSTE_OK) return st;
  RngKey key = derive_key(seed, offset);
  key.first_group = (uint64_t)(first_token / 4);
  return hip_status(launch_mvue_materialize(dY, T, O, lddy, dtype, key, vals, meta, (hipStream_t)hip_stream),
                    "mvue_materialize launch");
}

size_t sste_beta_workspace_bytes(int64_t O, int64_t I) {
  if (O < 0 || I < 0 || I % 8 != 0 || product_reaches(O, I, 1ll << 40)) return 0;
  return beta_workspace_bytes(O, I);
}

int sste_compute_beta(const void* W, int64_t O, int64_t I, int64_t ldw, float* beta_out, void* workspace,
                      size_t workspace_bytes, void* hip_stream) {
  return sste_compute_beta_ex(W, O, I, ldw, SSTE_BETA_MSE, 0.0f, beta_out, workspace, workspace_bytes, hip_stream);
}

int sste_compute_beta_ex(const void* W, int64_t O, int64_t I, int64_t ldw, int kind, float gamma, float* beta_out,
                         void* workspace, size_t workspace_bytes, void* hip_stream) {
  clear_error();
  if (kind != SSTE_BETA_MSE && kind != SSTE_BETA_L1) return fail(SSTE_ERR_VALUE, "compute_beta: unknown kind %d", kind);
  if (!(gamma >= 0.0f && gamma <= 1.0f)) return fail(SSTE_ERR_VALUE, "compute_beta: gamma must lie in [0, 1]");
  if (O < 0 || I < 0) return fail(SSTE_ERR_SHAPE, "compute_beta: negative size");
  if (I % 8 != 0) return fail(SSTE_ERR_SHAPE, "compute_beta: I=%lld is not a multiple of 8", (long long)I);
  if (ldw < I) return fail(SSTE_ERR_SHAPE, "compute_beta: ldw < I");
  if (ldw % 8 != 0) return fail(SSTE_ERR_ALIGN, "compute_beta: ldw is not a multiple of 8");
  if (!beta_out) return fail(SSTE_ERR_NULL, "compute_beta: beta_out is NULL");
  if (O > 0 && I > 0 && !W) return fail(SSTE_ERR_NULL, "compute_beta: W is NULL");
  if (product_reaches(O, ldw, 1ll << 40)) return fail(SSTE_ERR_UNSUPPORTED, "compute_beta: more than 2^40 weights");
  if (!aligned16(W)) return fail(SSTE_ERR_ALIGN, "compute_beta: W must be 16-byte aligned");
  size_t need = beta_workspace_bytes(O, I);
  if (!workspace || workspace_bytes < need) return fail(SSTE_ERR_WORKSPACE, "compute_beta: workspace needs %zu bytes", need);
  if (!aligned16(workspace)) return fail(SSTE_ERR_ALIGN, "compute_beta: workspace must be 16-byte aligned");
  return hip_status(launch_compute_beta(W, O, I, ldw, kind == SSTE_BETA_L1, gamma, beta_out, workspace, (hipStream_t)hip_stream),
                    "compute_beta launch");
}

int sste_cast_fp8(const void* X, int64_t R, int64_t C, int64_t ldx, int out_dtype, float scale, void* Q, int64_t ldq,
                  float* amax_out, void* hip_stream) {
  clear_error();
  if (R < 0 || C < 0) return fail(SSTE_ERR_SHAPE, "cast_fp8: negative size");
  if (C % 8 != 0) return fail(SSTE_ERR_SHAPE, "cast_fp8: C=%lld is not a multiple of 8", (long long)C);
  if (out_dtype != SSTE_F8E4M3 && out_dtype != SSTE_F8E5M2) return fail(SSTE_ERR_DTYPE, "cast_fp8: out_dtype %d is no 8-bit format", out_dtype);
  if (!good_scale(scale)) return fail(SSTE_ERR_VALUE, "cast_fp8: scale must be finite and > 0");
  if (ldx < C || (Q && ldq < C)) return fail(SSTE_ERR_SHAPE, "cast_fp8: leading dimension smaller than the row length");
  if (ldx % 8 != 0 || (Q && ldq % 8 != 0)) return fail(SSTE_ERR_ALIGN, "cast_fp8: ldx / ldq must be multiples of 8");
  if (!Q && !amax_out) return fail(SSTE_ERR_NULL, "cast_fp8: both Q and amax_out are NULL");
  if (R > 0 && C > 0 && !X) return fail(SSTE_ERR_NULL, "cast_fp8: NULL X");
  if (product_reaches(R, ldx, 1ll << 40) || product_reaches(R, Q ? ldq : 1, 1ll << 40)) return fail(SSTE_ERR_UNSUPPORTED, "cast_fp8: more than 2^40 elements");
  if (!aligned16(X) || (reinterpret_cast<uintptr_t>(Q) & 7u) || (reinterpret_cast<uintptr_t>(amax_out) & 3u))
    return fail(SSTE_ERR_ALIGN, "cast_fp8: X must be 16-byte, Q 8-byte, amax_out 4-byte aligned");
  return hip_status(launch_cast_fp8(X, R, C, ldx, out_dtype, scale, Q, ldq, amax_out, (hipStream_t)hip_stream), "cast_fp8 launch");
}

int sste_flip_count(const void* meta_a, const void* meta_b, int64_t O, int64_t I, unsigned long long* count_out, void* hip_stream) {
  clear_error();
  if (O < 0 || I < 0) return fail(SSTE_ERR_SHAPE, "flip_count: negative size");
  if (I % 8 != 0) return fail(SSTE_ERR_SHAPE, "flip_count: I=%lld is not a multiple of 8", (long long)I);
  if (!count_out) return fail(SSTE_ERR_NULL, "flip_count: count_out is NULL");
  if (product_reaches(O / 16 * 16 + 16, I, 1ll << 43)) return fail(SSTE_ERR_UNSUPPORTED, "flip_count: more than 2^40 bytes of metadata");
  int64_t nbytes = ((O + 15) / 16 * 16) * (I / 8);
  if (nbytes > 0 && (!meta_a || !meta_b)) return fail(SSTE_ERR_NULL, "flip_count: NULL metadata");
  if ((reinterpret_cast<uintptr_t>(meta_a) & 3u) || (reinterpret_cast<uintptr_t>(meta_b) & 3u) || (reinterpret_cast<uintptr_t>(count_out) & 7u))
    return fail(SSTE_ERR_ALIGN, "flip_count: metadata must be 4-byte and count_out 8-byte aligned");
  return hip_status(launch_flip_count(meta_a, meta_b, nbytes, count_out, (hipStream_t)hip_stream), "flip_count launch");
}

}  // extern "C"
