// Query-specific thresholds (paper Sec. 4.1 "Determining Proper Threshold"; the
// threshold step of Algorithm 2): density-map look-up at the projection of the
// query's residual w.r.t. its nearest list, polynomial, user scale.  One thread per
// (query, subspace); the maps (M * grid^2 floats, 2.6 MB for 64 subspaces of 100 x
// 100) stay in L2.  The work is a few loads per output: bound by launch latency for
// any realistic batch.

#include "ivfpq_internal.h"

namespace ivfpq {

namespace {

// floor((x - lo) * cells_per_unit) clamped to [0, G-1]; NaN -> 0
__device__ inline int grid_index(float x, float lo, float cpu, int G) {
  const float t = (x - lo) * cpu;
  int i = 0;
  if (t >= 1.0f) i = t >= (float)G ? G - 1 : (int)t;
  return i;
}

__global__ __launch_bounds__(256) void query_radii_kernel(
    const float *__restrict__ queries, const int32_t *__restrict__ probe_ids,
    const float *__restrict__ centroids, const float *__restrict__ lo, const float *__restrict__ cpu,
    const float *__restrict__ map, const float *__restrict__ coef, const float *__restrict__ fallback,
    int64_t total, int M, int D, int nlist, int nprobe, int G, int degree, float scale,
    float *__restrict__ out) {
  const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= total) return;
  const int64_t q = t / M;
  const int m = (int)(t - q * M);
  const int32_t c = probe_ids[q * nprobe];
  float r = fallback[m];
  if ((uint32_t)c < (uint32_t)nlist) {
    const float2 qv = make_float2(queries[q * D + 2 * m], queries[q * D + 2 * m + 1]);  // caller's pointer: no alignment assumed
    const float2 cv = *reinterpret_cast<const float2 *>(centroids + (int64_t)c * D + 2 * m);
    const float2 l = reinterpret_cast<const float2 *>(lo)[m];
    const float2 u = reinterpret_cast<const float2 *>(cpu)[m];
    const int i0 = grid_index(qv.x - cv.x, l.x, u.x, G);
    const int i1 = grid_index(qv.y - cv.y, l.y, u.y, G);
    const float f = map[((int64_t)m * G + i0) * G + i1];
    const float *cf = coef + (int64_t)m * (degree + 1);
    float p = cf[degree];
    for (int d = degree - 1; d >= 0; --d) p = fmaf(p, f, cf[d]);
    if (p > 0.0f && p < __builtin_inff()) r = p;
  }
  out[t] = r * scale;
}

}  // namespace

int launch_query_radii(const ivfpq_index *ix, const ivfpq_radius_model *md, const float *d_queries,
                       int64_t Q, const int32_t *d_probe_ids, int32_t nprobe, float scale,
                       float *d_radii, hipStream_t s) {
  const int64_t total = Q * md->M;
  const int64_t blocks = (total + 255) / 256;
  if (blocks > 0x7fffffff) {
    set_error("query_radii: Q * M = %lld is too large for one launch", (long long)total);
    return IVFPQ_ERR_UNSUPPORTED;
  }
  hipLaunchKernelGGL(query_radii_kernel, dim3((unsigned)blocks), dim3(256), 0, s, d_queries, d_probe_ids,
                     ix->d_centroids, md->d_lo, md->d_cpu, md->d_map, md->d_coef, md->d_fallback, total,
                     md->M, ix->D, ix->nlist, nprobe, md->grid, md->degree, scale, d_radii);
  IVFPQ_HIP_TRY(hipGetLastError());
  return IVFPQ_OK;
}

}  // namespace ivfpq
