// Host-only driver for the argument-checking layer of the C ABI (csrc/api.hip), built with
// -fsanitize=address,undefined for the host pass and run on the CPU by tests/test_abi_sanitizers.py.
// Every call below must be refused before anything is launched, so the launch functions are stubs that
// abort if reached; what is exercised is the validation arithmetic (sizes near the 64-bit and 32-bit
// limits, misaligned and NULL pointers, table preparation writing into caller memory).
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../../include/sste.h"

static int failures = 0;
#define EXPECT(call, want)                                                                   \
  do {                                                                                       \
    int got_ = (call);                                                                       \
    if (got_ != (want)) {                                                                    \
      std::printf("line %d: status %d, expected %d (%s)\n", __LINE__, got_, (want), sste_last_error()); \
      failures++;                                                                            \
    }                                                                                        \
  } while (0)

int main() {
  void* fake = reinterpret_cast<void*>(0x1000);
  void* odd = reinterpret_cast<void*>(0x1004);
  const int64_t huge = INT64_MAX / 2;

  // project + pack
  EXPECT(sste_project_pack(fake, -1, 64, 64, 1.f, SSTE_BF16, 1.f, fake, fake, nullptr, nullptr), SSTE_ERR_SHAPE);
  EXPECT(sste_project_pack(fake, 4, 12, 12, 1.f, SSTE_BF16, 1.f, fake, fake, nullptr, nullptr), SSTE_ERR_SHAPE);
  EXPECT(sste_project_pack(odd, 4, 64, 64, 1.f, SSTE_BF16, 1.f, fake, fake, nullptr, nullptr), SSTE_ERR_ALIGN);
  EXPECT(sste_project_pack(nullptr, 4, 64, 64, 1.f, SSTE_BF16, 1.f, fake, fake, nullptr, nullptr), SSTE_ERR_NULL);
  EXPECT(sste_project_pack_gamma(fake, 4, 64, 64, 1.f, 2.f, SSTE_BF16, 1.f, fake, fake, nullptr, nullptr), SSTE_ERR_VALUE);
  EXPECT(sste_project_pack(fake, 4, 64, 64, 1.f, 99, 1.f, fake, fake, nullptr, nullptr), SSTE_ERR_DTYPE);

  // batch preparation: writes a table into caller memory; an offending item in the middle stops it
  {
    std::vector<sste_pack_item> items(3);
    for (auto& it : items) it = sste_pack_item{fake, fake, fake, 32, 128, 128, 1.5f, 1.f};
    std::vector<unsigned char> table(3 * SSTE_PACK_TABLE_ITEM_BYTES);
    int64_t blocks = -1;
    EXPECT(sste_project_pack_batch_prepare(items.data(), 3, SSTE_BF16, table.data(), &blocks), SSTE_OK);
    if (blocks != 3 * 2 * 2) { std::printf("blocks %lld\n", (long long)blocks); failures++; }
    items[1].I = 100;
    EXPECT(sste_project_pack_batch_prepare(items.data(), 3, SSTE_BF16, table.data(), &blocks), SSTE_ERR_SHAPE);
    EXPECT(sste_project_pack_batch_prepare(items.data(), -1, SSTE_BF16, table.data(), &blocks), SSTE_ERR_SHAPE);
    EXPECT(sste_project_pack_batch_prepare(nullptr, 0, SSTE_BF16, nullptr, &blocks), SSTE_OK);
    std::vector<sste_update_item> up(2);
    for (auto& it : up) it = sste_update_item{fake, reinterpret_cast<const float*>(fake), fake, fake, 16, 64, 64, 64, 1.5f, 1.f};
    std::vector<unsigned char> utable(2 * SSTE_UPDATE_TABLE_ITEM_BYTES);
    EXPECT(sste_sgd_project_pack_batch_prepare(up.data(), 2, SSTE_F32, SSTE_BF16, utable.data(), &blocks), SSTE_OK);
    up[1].ldg = 66;
    EXPECT(sste_sgd_project_pack_batch_prepare(up.data(), 2, SSTE_F32, SSTE_BF16, utable.data(), &blocks), SSTE_ERR_ALIGN);
  }

  // GEMMs: sizes at the edges of the offset arithmetic
  EXPECT(sste_linear_fwd(fake, huge, 64, 64, SSTE_BF16, 1.f, fake, fake, 8, 1.f, fake, 8, nullptr), SSTE_ERR_UNSUPPORTED);
  EXPECT(sste_linear_fwd(fake, 4, 64, huge - huge % 8, SSTE_BF16, 1.f, fake, fake, 8, 1.f, fake, 8, nullptr), SSTE_ERR_UNSUPPORTED);
  EXPECT(sste_linear_fwd_ex(fake, 4, 128, 128, SSTE_F8E4M3, 1.f, fake, fake, 16, 1.f, fake, 16, SSTE_F8E4M3, 1.f, nullptr, nullptr), SSTE_ERR_NULL);
  EXPECT(sste_linear_fwd_act(fake, 4, 64, 64, SSTE_BF16, 1.f, fake, fake, 8, 1.f, 5, fake, 8, fake, 8, SSTE_BF16, 1.f, nullptr, nullptr), SSTE_ERR_VALUE);
  EXPECT(sste_linear_dgrad(fake, 4, 16, 16, SSTE_BF16, 1.f, fake, fake, 96, 1.f, fake, 96, nullptr), SSTE_ERR_UNSUPPORTED);
  EXPECT(sste_linear_dgrad_act(fake, 4, 16, 16, SSTE_BF16, 1.f, fake, fake, 64, 1.f, SSTE_ACT_GELU_TANH, nullptr, 64, fake, 64, nullptr), SSTE_ERR_NULL);
  EXPECT(sste_linear_wgrad(fake, 100, 16, 16, SSTE_BF16, 1.f, fake, 16, 16, 1.f, 0, 0, reinterpret_cast<float*>(fake), 16, 0, nullptr, 0, nullptr), SSTE_ERR_UNSUPPORTED);
  EXPECT(sste_linear_wgrad(fake, 4096, 512, 512, SSTE_BF16, 1.f, fake, 512, 512, 1.f, 0, 0, reinterpret_cast<float*>(fake), 512, 0, nullptr, 0, nullptr), SSTE_ERR_WORKSPACE);
  EXPECT(sste_linear_wgrad(fake, 4096, 512, 512, SSTE_BF16, 1.f, fake, 512, 512, 1.f, 0, 0, reinterpret_cast<float*>(fake), 512, 0, fake, 16, nullptr), SSTE_ERR_WORKSPACE);
  EXPECT(sste_linear_wgrad_at(fake, 4096, 512, 512, SSTE_BF16, 1.f, fake, 512, 512, 1.f, 0, 0, 6, reinterpret_cast<float*>(fake), 512, 0, fake, size_t(1) << 40, nullptr), SSTE_ERR_SHAPE);
  EXPECT(sste_linear_wgrad_at(fake, 4096, 512, 512, SSTE_BF16, 1.f, fake, 512, 512, 1.f, 0, 0, INT64_MAX - 3, reinterpret_cast<float*>(fake), 512, 0, fake, size_t(1) << 40, nullptr), SSTE_ERR_UNSUPPORTED);
  EXPECT(sste_linear_wgrad_noalloc(fake, 16384, 5120, 5120, SSTE_BF16, 1.f, fake, 1280, 1280, 1.f, 0, 0, reinterpret_cast<float*>(fake), 1280, 0, nullptr), SSTE_ERR_WORKSPACE);
  if (sste_wgrad_workspace_bytes(16384, 5120, 1280, SSTE_BF16) == 0) { std::printf("workspace size 0\n"); failures++; }
  if (sste_wgrad_workspace_bytes(huge, huge, huge, SSTE_BF16) != 0 && sste_wgrad_workspace_bytes(100, 8, 8, SSTE_BF16) != 0) failures++;
  EXPECT(sste_wgrad_plan_override(5, 5, 0), SSTE_ERR_VALUE);
  EXPECT(sste_wgrad_plan_override(8, 3, 4), SSTE_OK);
  EXPECT(sste_wgrad_plan_override(0, 0, 0), SSTE_OK);
  EXPECT(sste_mvue_materialize(fake, 128, 333, 336, SSTE_BF16, 0, 0, fake, fake, nullptr), SSTE_ERR_UNSUPPORTED);
  EXPECT(sste_mvue_materialize_at(fake, 128, 8, 8, SSTE_BF16, 0, 0, -4, fake, fake, nullptr), SSTE_ERR_SHAPE);
  EXPECT(sste_cast_fp8(fake, 4, 60, 64, SSTE_F8E4M3, 1.f, fake, 64, nullptr, nullptr), SSTE_ERR_SHAPE);
  EXPECT(sste_compute_beta_ex(fake, 4, 64, 64, 7, 0.f, reinterpret_cast<float*>(fake), fake, 1 << 20, nullptr), SSTE_ERR_VALUE);
  EXPECT(sste_flip_count(fake, fake, 4, 60, nullptr, nullptr), SSTE_ERR_SHAPE);

  // absurd sizes must be refused by arithmetic that does not overflow
  EXPECT(sste_project_pack(fake, huge, 64, 64, 1.f, SSTE_BF16, 1.f, fake, fake, nullptr, nullptr), SSTE_ERR_UNSUPPORTED);
  EXPECT(sste_compute_beta(fake, huge, huge - huge % 8, huge - huge % 8, reinterpret_cast<float*>(fake), fake, 1 << 20, nullptr), SSTE_ERR_UNSUPPORTED);
  if (sste_beta_workspace_bytes(huge, huge - huge % 8) != 0) failures++;
  EXPECT(sste_flip_count(fake, fake, huge, huge - huge % 8, reinterpret_cast<unsigned long long*>(fake), nullptr), SSTE_ERR_UNSUPPORTED);
  EXPECT(sste_cast_fp8(fake, huge, 64, huge - huge % 8, SSTE_F8E4M3, 1.f, fake, huge - huge % 8, nullptr, nullptr), SSTE_ERR_UNSUPPORTED);

  // delayed-scaling helper: pure host code
  sste_amax_history h;
  sste_amax_history_init(&h, 1 << 20);
  for (int i = 0; i < 200; i++) (void)sste_amax_history_push(&h, float(i), 448.f);
  if (sste_amax_history_push(&h, 0.f, 448.f) != 199.f / 448.f) { std::printf("amax history\n"); failures++; }
  sste_amax_history_init(&h, -5);
  if (h.length != 1) failures++;

  std::printf(failures ? "FAILED: %d\n" : "abi driver ok%.0d\n", failures);
  return failures ? 1 : 0;
}
