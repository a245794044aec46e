// Host-only exerciser of the library's argument checking, built with AddressSanitizer and
// UndefinedBehaviorSanitizer on the host side (tests/test_host_sanitizers.py compiles and runs it).
// Every call below must be refused before any GPU call, so it runs on a machine without a GPU; the
// sanitizers turn any out-of-bounds access or undefined operation on the way into a failure.
#include <cstdio>
#include <cstdlib>
#include <cstring>

#include "fasth.h"

static int failures = 0;
#define EXPECT(call, want)                                                              \
  do {                                                                                  \
    const long long got_ = (long long)(call);                                           \
    if (got_ != (long long)(want)) {                                                    \
      std::printf("FAIL %s: got %lld, want %lld\n", #call, got_, (long long)(want));    \
      ++failures;                                                                       \
    }                                                                                   \
  } while (0)

int main() {
  float* p = reinterpret_cast<float*>(256);       // aligned, never dereferenced on the host
  float* odd = reinterpret_cast<float*>(260);     // not 16-byte aligned
  const size_t big = (size_t)1 << 40;
  fasth_shape ok = {64, 64, 32, 32, 0};
  fasth_shape bad_k = {64, 64, 32, 7, 0}, bad_m = {64, 64, 0, 32, 0}, bad_t = {64, 64, 32, 32, 2};
  fasth_shape too_big = {64, 256, 32, 256, 0}, many_blocks = {8, 1 << 20, 1, 1, 0};
  EXPECT(fasth_workspace_bytes(&ok) > 0, 1);
  EXPECT(fasth_workspace_bytes(&bad_k), 0);
  EXPECT(fasth_workspace_bytes(nullptr), 0);
  EXPECT(fasth_workspace_bytes(&many_blocks), 0);
  // shapes whose chains share a column between workgroups carry a hand-off area; the layout code is host code
  fasth_shape team2 = {1024, 1024, 32, 32, 0}, team8 = {4096, 128, 32, 128, 0}, split2 = {2048, 64, 100, 32, 0};
  EXPECT(fasth_workspace_bytes(&team2) > fasth_workspace_bytes(&ok), 1);
  EXPECT(fasth_workspace_bytes(&team8) > (size_t)32 * (256 + 8 * 2 * 8 * 64 * 8), 1);
  EXPECT(fasth_workspace_bytes(&split2) > 0, 1);
  EXPECT(fasth_set_wait_limit(0), FASTH_OK);
  EXPECT(fasth_set_wait_limit(-1), FASTH_OK);
  EXPECT(fasth_forward(&bad_k, p, p, p, p, big, nullptr), FASTH_EINVAL);
  EXPECT(fasth_forward(&bad_m, p, p, p, p, big, nullptr), FASTH_EINVAL);
  EXPECT(fasth_forward(&bad_t, p, p, p, p, big, nullptr), FASTH_EINVAL);
  EXPECT(fasth_forward(&too_big, p, p, p, p, big, nullptr), FASTH_EUNSUPPORTED);
  EXPECT(fasth_forward(&many_blocks, p, p, p, p, big, nullptr), FASTH_EUNSUPPORTED);
  EXPECT(fasth_forward(nullptr, p, p, p, p, big, nullptr), FASTH_EINVAL);
  EXPECT(fasth_forward(&ok, nullptr, p, p, p, big, nullptr), FASTH_EINVAL);
  EXPECT(fasth_forward(&ok, p, odd, p, p, big, nullptr), FASTH_EALIGN);
  EXPECT(fasth_forward(&ok, p, p, p, p, 128, nullptr), FASTH_EWORKSPACE);
  EXPECT(fasth_forward_static(&ok, nullptr, p, p, nullptr), FASTH_EINVAL);
  fasth_shape huge = {16384, 16384, 32, 128, 0};
  EXPECT(fasth_forward_static(&huge, p, p, p, nullptr), FASTH_EUNSUPPORTED);
  EXPECT(fasth_prepare(&ok, p, p, 16, nullptr), FASTH_EWORKSPACE);
  EXPECT(fasth_apply(&ok, p, p, odd, p, big, 0, nullptr), FASTH_EALIGN);
  EXPECT(fasth_backward(&ok, p, p, nullptr, p, p, big, nullptr), FASTH_EINVAL);
  EXPECT(fasth_backward(&ok, p, p, p, p, p, 16, nullptr), FASTH_EWORKSPACE);
  int best = 0;
  EXPECT(fasth_tune_block_size(&ok, nullptr, 0, 0, p, p, p, p, p, p, p, big, &best, nullptr, nullptr), FASTH_EINVAL);
  EXPECT(fasth_sequential_workspace_bytes(&ok), (size_t)32 * 64 * 64 * 4);
  EXPECT(fasth_sequential_forward(&ok, p, nullptr, p, nullptr), FASTH_EINVAL);
  EXPECT(fasth_sequential_backward(&ok, p, p, p, p, p, p, 16, nullptr), FASTH_EWORKSPACE);
  fasth_svd_shape s_bad = {64, 64, 32, 5}, s_ok = {64, 64, 32, 32};
  EXPECT(svd_layer_workspace_bytes(&s_bad), 0);
  EXPECT(svd_layer_workspace_bytes(&s_ok) > 2 * fasth_workspace_bytes(&ok), 1);
  EXPECT(svd_layer_apply(&s_bad, p, p, p, p, p, p, big, nullptr), FASTH_EINVAL);
  EXPECT(svd_layer_apply(&s_ok, p, p, p, p, p, p, 16, nullptr), FASTH_EWORKSPACE);
  EXPECT(svd_layer_inverse_apply(&s_ok, p, odd, p, p, p, p, big, nullptr), FASTH_EALIGN);
  EXPECT(svd_layer_apply_backward(&s_ok, p, p, p, p, p, p, p, nullptr, p, big, nullptr), FASTH_EINVAL);
  EXPECT(svd_layer_inverse_apply_backward(&s_ok, p, p, p, p, p, p, p, p, p, 16, nullptr), FASTH_EWORKSPACE);
  EXPECT(svd_sym_apply(&s_ok, 7, p, p, p, p, p, big, nullptr), FASTH_EINVAL);
  EXPECT(svd_sym_apply_backward(&s_ok, FASTH_DIAG_EXP, p, p, p, p, p, p, p, 16, nullptr), FASTH_EWORKSPACE);
  fasth_rect_shape r_ok = {96, 64, 96, 64, 8, 32}, r_bad = {96, 64, 96, 60, 8, 32};
  EXPECT(svd_rect_workspace_bytes(&r_bad), 0);
  EXPECT(svd_rect_workspace_bytes(&r_ok) > 0, 1);
  EXPECT(svd_rect_apply(&r_bad, p, p, p, p, p, p, big, nullptr), FASTH_EINVAL);
  EXPECT(svd_rect_apply(&r_ok, p, p, p, odd, p, p, big, nullptr), FASTH_EALIGN);
  EXPECT(svd_rect_apply_backward(&r_ok, p, p, p, p, p, p, p, p, p, 16, nullptr), FASTH_EWORKSPACE);
  EXPECT(svd_layer_log_abs_det(0, p, p, nullptr, nullptr), FASTH_EINVAL);
  float peaks[3];
  EXPECT(fasth_measure_peaks(nullptr, big, 1, peaks, peaks + 1, peaks + 2, nullptr), FASTH_EINVAL);
  EXPECT(fasth_measure_peaks(p, 1024, 1, peaks, peaks + 1, peaks + 2, nullptr), FASTH_EWORKSPACE);
  for (int code = -8; code <= 0; ++code) EXPECT(std::strlen(fasth_strerror(code)) > 0, 1);
  for (int id = -1; id <= FASTH_KERNEL_COUNT; ++id) {
    EXPECT(fasth_kernel_name(id) != nullptr, 1);
    EXPECT(fasth_profile_variant(id) != nullptr, 1);
  }
  float ms[FASTH_KERNEL_COUNT];
  int launches[FASTH_KERNEL_COUNT];
  EXPECT(fasth_profile_collect(nullptr, launches), FASTH_EINVAL);
  EXPECT(fasth_profile_collect(ms, launches), FASTH_OK);
  std::printf(failures ? "abi_host_check: %d failures\n" : "abi_host_check: ok\n", failures);
  return failures ? 1 : 0;
}
