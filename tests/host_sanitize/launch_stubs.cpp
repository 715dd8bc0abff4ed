// Stand-ins for the kernel launch functions of the library, for the host-only sanitizer build of the
// argument-checking layer: the driver only makes calls that must be refused before a launch, so reaching
// one of these is a failure.  Shape helpers return fixed answers.
#include <cstdio>
#include <cstdlib>

#include "../../paper_2409_09099_amd/csrc/common.h"

namespace sste {
[[noreturn]] static void reached(const char* what) {
  std::printf("launch function reached: %s\n", what);
  std::abort();
}
hipError_t launch_project_pack(const void*, int64_t, int64_t, int64_t, float, float, int, float, void*, void*, float*, hipStream_t) { reached("project_pack"); }
hipError_t launch_sgd_project_pack(void*, bool, int64_t, int64_t, int64_t, const float*, int64_t, float, float, int, float, void*, void*, hipStream_t) { reached("sgd_project_pack"); }
hipError_t launch_sgd_project_pack_batch(const void*, int, int64_t, bool, int, float, hipStream_t) { reached("sgd_project_pack_batch"); }
hipError_t launch_project_pack_batch(const void*, int, int64_t, int, hipStream_t) { reached("project_pack_batch"); }
bool linear_dgrad_supported(int64_t, int64_t, int64_t, int64_t, int) { return true; }
hipError_t launch_linear_dgrad(const void*, int64_t, int64_t, int64_t, int, float, const void*, const void*, int64_t, void*, int64_t, const void*, int64_t, hipStream_t) { reached("linear_dgrad"); }
hipError_t launch_compute_beta(const void*, int64_t, int64_t, int64_t, int, float, float*, void*, hipStream_t) { reached("compute_beta"); }
size_t beta_workspace_bytes(int64_t, int64_t) { return 16384; }
hipError_t launch_cast_fp8(const void*, int64_t, int64_t, int64_t, int, float, void*, int64_t, float*, hipStream_t) { reached("cast_fp8"); }
hipError_t launch_flip_count(const void*, const void*, int64_t, unsigned long long*, hipStream_t) { reached("flip_count"); }
hipError_t launch_mvue_materialize(const void*, int64_t, int64_t, int64_t, int, RngKey, void*, void*, hipStream_t) { reached("mvue_materialize"); }
hipError_t launch_linear_fwd(const void*, int64_t, int64_t, int64_t, int, float, const void*, const void*, int64_t, void*, int64_t, int, float, float*, hipStream_t) { reached("linear_fwd"); }
hipError_t launch_linear_fwd_act(const void*, int64_t, int64_t, int64_t, int, float, const void*, const void*, int64_t, void*, int64_t, void*, int64_t, int, float, float*, hipStream_t) { reached("linear_fwd_act"); }
bool linear_fwd_supported(int64_t T, int64_t I, int64_t ldx, int64_t O, int dtype) {
  int64_t eb = dtype == SSTE_F8E4M3 ? 1 : 2;
  if (product_reaches(ldx, 256 * eb, 1ll << 30) || product_reaches(I, 256 * eb, 1ll << 30)) return false;
  if (product_reaches(O / 256 + 1, T / 128 + 1, 0x80000000ll)) return false;
  return true;
}
size_t wgrad_workspace_bytes(int64_t T, int64_t O, int64_t I, int) { return (size_t)T * (size_t)O + (size_t)O * (size_t)I * 16; }   // unsigned: wraps, no overflow
bool linear_wgrad_supported(int64_t, int64_t, int64_t, int64_t, int) { return true; }
bool wgrad_plan_override(int mi, int ni, int splits) {
  return ((mi == 0 && ni == 0) || (mi == 8 && ni == 4) || (mi == 6 && ni == 3) || (mi == 8 && ni == 3)) && splits >= 0 && splits <= 32;
}
void* noalloc_scratch(hipError_t*) { reached("noalloc_scratch"); }
hipError_t launch_linear_wgrad(const void*, int64_t, int64_t, int64_t, int, const void*, int64_t, int64_t, float, RngKey, float*, int64_t, int, void*, hipStream_t) { reached("linear_wgrad"); }
}  // namespace sste
