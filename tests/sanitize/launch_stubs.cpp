// Stand-ins for the kernel launchers, so that the host side of the C ABI (argument
// validation, workspace planning, index description checks in csrc/api.hip) links into a
// CPU-only program that runs under the address and undefined-behaviour sanitizers.  Every
// stub reports a launch that the test does not expect to reach.
#include <cstdio>
#include <cstdlib>

#include "ivfpq_internal.h"

namespace ivfpq {
static int reached(const char *what) {
  std::fprintf(stderr, "launch stub reached: %s\n", what);
  return IVFPQ_ERR_HIP;
}
int launch_coarse(const ivfpq_index *, const float *, int64_t, int32_t, int32_t *, float *, float *, int64_t,
                  int32_t, int32_t *, hipStream_t) { return reached("coarse"); }
int launch_build_lut(const ivfpq_index *, const float *, int64_t, int32_t, const int32_t *, const RadiiSq &,
                     float *, uint64_t *, int32_t, const float *, hipStream_t) { return reached("build_lut"); }
int launch_scan(const ivfpq_index *, const float *, int64_t, int32_t, const int32_t *, int32_t, const RadiiSq &,
                int32_t, uint32_t *, int64_t *, int64_t *, float *, const int64_t *, float *, int64_t *,
                int32_t *, int32_t, const float *, float *, hipStream_t, const ScanView *) { return reached("scan"); }
int launch_query_radii(const ivfpq_index *, const ivfpq_radius_model *, const float *, int64_t, const int32_t *,
                       int32_t, float, float *, hipStream_t) { return reached("query_radii"); }
int launch_relayout(const ivfpq_index *, const uint8_t *, hipStream_t) { return reached("relayout"); }
int launch_list_boxes(const ivfpq_index *, const uint8_t *, hipStream_t) { return reached("list_boxes"); }
int launch_codebook_grid(const ivfpq_index *, hipStream_t) { return reached("codebook_grid"); }
int launch_iota(int64_t *, int64_t, hipStream_t) { return reached("iota"); }
int launch_fill_i32(int32_t *, int64_t, int32_t, hipStream_t) { return reached("fill_i32"); }
int coarse_fallbacks(int, unsigned int *out) { *out = 0; return IVFPQ_OK; }
bool list_major_supported(const ivfpq_index *, int32_t, int32_t) { return false; }
LmWorkspace plan_list_major(const ivfpq_index *, int64_t, int32_t) { return LmWorkspace(); }
int launch_scan_list_major(const ivfpq_index *, const float *, int64_t, int32_t, const int32_t *, int32_t,
                           const RadiiSq &, int32_t, const float *, float *, int64_t *, float *, const LmWorkspace &,
                           char *, hipStream_t) { return reached("scan_list_major"); }
void set_lm_first(int) {}
void set_lm_cap(int) {}
void set_scan_ablate(int) {}
void set_scan_variant(int) {}
void set_bound_grid(int) {}
void set_scan_waves(int) {}
}  // namespace ivfpq
