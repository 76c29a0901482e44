// CPU oracle for the search path of sparsity-aware IVF-PQ (JUNO, arxiv 2312.01712).
//
// TEST INFRASTRUCTURE ONLY.  This file defines what the GPU library must
// compute; it is slow, single-threaded and written to be checked against the
// paper by eye.  It shares no code, header, table or helper with the HIP path,
// and only the tests, the smoke check and the benchmark's cpu_baseline leg may
// call it.
//
// Notation: the paper's Table 1 writes M for the subspace *dimension* and D/M
// for the number of subspaces.  Here M is the NUMBER of subspaces, dsub = D/M
// their dimension, E = 256 entries per subspace, nlist = the paper's C and
// nprobe = the paper's nprobs.
//
// All arithmetic that decides a result is IEEE fp32 in a fixed order (compile
// with -ffp-contract=off; fused multiply-adds are written explicitly as fmaf).
//
// Readings taken where the paper is silent or garbled (each is repeated at the
// function it concerns):
//   R1  entries outside the radius contribute the clamp r_m^2 (the paper only
//       says non-selected points get "a large constant", Sec. 5.3);
//   R3  the table holds SQUARED distances (metric definition in Sec. 2.1 and
//       the L2^2 identity of Sec. 4.2), not their roots as Algorithm 2 prints;
//   R4  an entry is kept when d2 <= r_m^2 (tangent rays hit);
//   R5  the radius test is made on the RESIDUAL projection (entries are trained
//       on residuals, Sec. 2.1 / Algorithm 1);
//   R6  one (query, probed list, subspace) ray writes one table row only;
//   R7  radii are per subspace and shared by all queries of a call;
//   R11 top-k order is (distance, id) lexicographic;
//   R14 hit-count scoring (Sec. 5.4) is expressed as a penalty that is summed like a
//       distance, so that smaller is better in every mode: a missed subspace costs 1
//       (hit count = M - sum); with the half-radius inner sphere of the reward /
//       penalty model, inside the inner sphere costs 0 (+1 in the paper), inside the
//       outer sphere only costs 1 (0), outside both costs 2 (-1), i.e. score = M - sum.
//       Rankings are those of the paper's scores; ties go to the smaller id;
//   R15 a per-query radius (Sec. 4.1 "Determining Proper Threshold": query-specific
//       thresholds times a user scale) is an input array radii[Q][M]; how it is
//       derived from densities is outside the search path;
//   R16 inner-product metric (Sec. 4.2 "Inner Product Similarity Support").  The
//       paper enlarges the sphere of entry e to R'^2 = R^2 + |e|^2 and shoots the ray
//       from the projection of the QUERY (its x_q, y_q are constant per query, so not
//       a residual).  The ray hits iff |q_m - e|^2 <= r_m^2 + |e|^2, which is the same
//       as IP(e, q_m) >= (|q_m|^2 - r_m^2) / 2 =: thr_m, the form used here (no
//       subtraction of nearly equal squares).  A kept entry stores -IP (smaller is
//       better in every mode), a missed one the bound -thr_m it cannot beat, which is
//       what the clamp r_m^2 is under L2 (R1).  The table depends on the query only;
//       a point of list c scores -IP(q, centroid_c) plus the sum of its table values,
//       i.e. minus the inner product of q with the point's reconstruction, and lists
//       are filtered by the same -IP(q, centroid).  For the hit-count modes the inner
//       sphere is the same construction with r_m / 2;
//   R17 dynamic threshold (Sec. 4.1 "Determining Proper Threshold"; the threshold step of
//       Algorithm 2).  Offline the paper cuts every (two-dimensional) subspace into a
//       G x G grid, G = 100, a cell's density being the number of search point
//       projections in it divided by its area, and fits a polynomial from that density
//       to the threshold a projection needs; online the density at the query's
//       projection is looked up, the polynomial evaluated and the result multiplied by
//       the user's scale.  The listing evaluates this inside the loop over the selected
//       lists, before the centroid is subtracted, and keeps overwriting (x, y); read
//       here as: ONE threshold per (query, subspace), looked up at the projection of
//       the residual w.r.t. the query's NEAREST list (entries and search point
//       projections live in residual space, R5), which fills radii[Q][M] of R15.  The
//       map stores the polynomial's input (the density, or whatever fixed transform of
//       it the fit used); a value that is not positive and finite is replaced by a
//       per-subspace fallback radius before scaling;
//
// Metric: 0 = squared L2, 1 = inner product (R16).
// Scoring modes: 0 = distances (the paper's JUNO-H), 1 = hit count (JUNO-L),
// 2 = reward/penalty hit count (JUNO-M).  radii_stride = 0 means one radii[M] for all
// queries, radii_stride = M means radii[Q][M].
//
// Pins (tests/test_oracle_pins.py): brute-force exact kNN on identity-codebook
// indexes, reconstruction identity of the unthresholded ADC sum, truncated-sum
// closed form and monotonicity of the thresholded one, the paper's ray/sphere
// formulation of the keep rule (t_hit <= t_max) with its printed 0.6/0.8/0.64
// example, argmin / full-permutation cases of the coarse stage, and
// sort-based selection for top-k; for the inner-product metric the enlarged-sphere
// form of the keep rule, the identity IP = (|e|^2 + |q|^2 - L2^2) / 2 against the L2
// table, reconstruction of -IP by the unthresholded sum, and brute-force maximum
// inner product search on identity-codebook indexes; for the dynamic threshold a
// hand-computed grid example, counting by cell inequalities, and the constant /
// identity polynomial cases.  No function here is "parity unpinned".

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <utility>
#include <vector>

namespace {

constexpr int E = 256;

struct Cand {
  float d;
  int64_t id;
};

inline bool cand_less(const Cand& a, const Cand& b) {
  return a.d < b.d || (a.d == b.d && a.id < b.id);
}

// Filtering stage (paper Sec. 2.1 "Online Search" step A; Sec. 5.3): squared L2
// distance from the query to every IVF centroid, then the nprobe closest.
// Distance: t = q_i - c_i, acc = fmaf(t, t, acc), i ascending, acc0 = 0.
// Order of the result: (distance, list id) ascending.
//
// Inner-product metric (R16): the score of a list is minus the inner product of the
// query with its centroid, acc = fmaf(q_i, c_i, acc), i ascending, acc0 = 0; "minus"
// is written 0 - acc here and in the table, so that no score is a negative zero (which
// would compare equal to +0 but differ in bits).
inline float list_score(const float* q, const float* cen, int D, int metric) {
  float acc = 0.0f;
  for (int i = 0; i < D; ++i) {
    if (metric == 0) {
      float t = q[i] - cen[i];
      acc = std::fmaf(t, t, acc);
    } else {
      acc = std::fmaf(q[i], cen[i], acc);
    }
  }
  return metric == 0 ? acc : 0.0f - acc;
}

void coarse_one(const float* q, int D, const float* centroids, int nlist, int nprobe, int metric,
                int32_t* out_ids, float* out_dist) {
  std::vector<std::pair<float, int32_t>> d(nlist);
  for (int c = 0; c < nlist; ++c) d[c] = {list_score(q, centroids + (size_t)c * D, D, metric), c};
  std::sort(d.begin(), d.end());
  for (int p = 0; p < nprobe; ++p) {
    out_ids[p] = d[p].second;
    if (out_dist) out_dist[p] = d[p].first;
  }
}

// Selective L2-LUT construction (paper Sec. 4.1; Algorithm 2) for one
// (query, probed list): for every subspace m and entry e,
//   res_j = q[m*dsub+j] - centroid[m*dsub+j]        (step B: residual)
//   t_j   = res_j - codebook[m][e][j]
//   d2    = t_0*t_0, then d2 = fmaf(t_j, t_j, d2) for j = 1..dsub-1   (step C)
//   keep  = d2 <= r_m^2   (entry inside the sphere of radius r_m around the
//                          residual projection; R4, R5)
//   lut[m][e] = keep ? d2 : r_m^2                                    (R1, R3)
// mask (optional) gets bit e of word [m][e/64] set when the entry is kept.
//
// Hit-count scoring (paper Sec. 5.4, R14): mode 1 stores 0 for a kept entry and 1
// otherwise; mode 2 stores 0 inside the inner sphere of radius r_m / 2
// (d2 <= r_m^2 / 4), 1 inside the outer sphere only, 2 outside both.
void lut_one(const float* q, const float* cen, int D, int M, const float* codebooks,
             const float* radii, int mode, float* lut, uint64_t* mask) {
  const int dsub = D / M;
  for (int m = 0; m < M; ++m) {
    const float r2 = radii[m] * radii[m];
    if (mask) for (int w = 0; w < 4; ++w) mask[m * 4 + w] = 0;
    for (int e = 0; e < E; ++e) {
      const float* cb = codebooks + ((size_t)m * E + e) * dsub;
      float d2 = 0.0f;
      for (int j = 0; j < dsub; ++j) {
        float res = q[m * dsub + j] - cen[m * dsub + j];
        float t = res - cb[j];
        d2 = (j == 0) ? t * t : std::fmaf(t, t, d2);
      }
      const bool keep = d2 <= r2;
      if (mode == 0) lut[m * E + e] = keep ? d2 : r2;
      else if (mode == 1) lut[m * E + e] = keep ? 0.0f : 1.0f;
      else lut[m * E + e] = d2 <= 0.25f * r2 ? 0.0f : (keep ? 1.0f : 2.0f);
      if (mask && keep) mask[m * 4 + (e >> 6)] |= (uint64_t)1 << (e & 63);
    }
  }
}

// The same table under the inner-product metric (paper Sec. 4.2, R16), for one query
// (it does not depend on the list): for every subspace m and entry e, with q_m the
// query's projection,
//   qq   = q_m0*q_m0, then qq = fmaf(q_mj, q_mj, qq)
//   thr  = 0.5 * (qq - r_m^2)
//   ip   = q_m0*e_0, then ip = fmaf(q_mj, e_j, ip)
//   keep = ip >= thr          (the ray from q_m hits the sphere of radius sqrt(r_m^2 + |e|^2))
//   lut[m][e] = keep ? 0 - ip : 0 - thr
// Hit-count modes: mode 1 stores 0 / 1 for kept / missed; mode 2 uses the inner
// threshold thr_in = 0.5 * (qq - r_m^2 / 4): 0 if ip >= thr_in, else 1 if kept, else 2.
void lut_one_ip(const float* q, int D, int M, const float* codebooks, const float* radii, int mode,
                float* lut, uint64_t* mask) {
  const int dsub = D / M;
  for (int m = 0; m < M; ++m) {
    const float* qm = q + m * dsub;
    const float r2 = radii[m] * radii[m];
    float qq = 0.0f;
    for (int j = 0; j < dsub; ++j) qq = (j == 0) ? qm[j] * qm[j] : std::fmaf(qm[j], qm[j], qq);
    const float thr = 0.5f * (qq - r2);
    const float thr_in = 0.5f * (qq - 0.25f * r2);
    if (mask) for (int w = 0; w < 4; ++w) mask[m * 4 + w] = 0;
    for (int e = 0; e < E; ++e) {
      const float* cb = codebooks + ((size_t)m * E + e) * dsub;
      float ip = 0.0f;
      for (int j = 0; j < dsub; ++j) ip = (j == 0) ? qm[j] * cb[j] : std::fmaf(qm[j], cb[j], ip);
      const bool keep = ip >= thr;
      if (mode == 0) lut[m * E + e] = keep ? 0.0f - ip : 0.0f - thr;
      else if (mode == 1) lut[m * E + e] = keep ? 0.0f : 1.0f;
      else lut[m * E + e] = ip >= thr_in ? 0.0f : (keep ? 1.0f : 2.0f);
      if (mask && keep) mask[m * 4 + (e >> 6)] |= (uint64_t)1 << (e & 63);
    }
  }
}

// Table of (query, list) under either metric.
void lut_any(const float* q, const float* cen, int D, int M, const float* codebooks,
             const float* radii, int mode, int metric, float* lut, uint64_t* mask) {
  if (metric == 0) lut_one(q, cen, D, M, codebooks, radii, mode, lut, mask);
  else lut_one_ip(q, D, M, codebooks, radii, mode, lut, mask);
}

// Distance calculation (paper Sec. 2.1 step D; Sec. 5.3): the distance of an
// encoded point is the sum over subspaces of the table value of its code,
// fp32, m ascending, starting from `start`: 0 under L2 and for the hit counts; under
// the inner-product metric with mode 0 the list's score -IP(q, centroid) (R16).
inline float adc_one(const float* lut, const uint8_t* code, int M, float start) {
  float dist = start;
  for (int m = 0; m < M; ++m) dist += lut[m * E + code[m]];
  return dist;
}

inline float adc_start(const float* q, const float* cen, int D, int mode, int metric) {
  return (metric == 1 && mode == 0) ? list_score(q, cen, D, 1) : 0.0f;
}

// Top-k (paper Sec. 2.1, last paragraph of "Online Search"): the k smallest by
// (distance, id), ascending; missing results are (id -1, distance +inf).
void topk_select(std::vector<Cand>& cand, int k, int64_t* out_ids, float* out_dist) {
  const size_t kk = std::min((size_t)k, cand.size());
  std::partial_sort(cand.begin(), cand.begin() + kk, cand.end(), cand_less);
  for (int i = 0; i < k; ++i) {
    if ((size_t)i < kk) {
      out_ids[i] = cand[i].id;
      out_dist[i] = cand[i].d;
    } else {
      out_ids[i] = -1;
      out_dist[i] = std::numeric_limits<float>::infinity();
    }
  }
}

}  // namespace

extern "C" {

// Batched filtering stage.  out_ids [Q][nprobe], out_dist [Q][nprobe] (may be null).
int oracle_coarse(int64_t Q, int32_t D, int32_t nlist, const float* queries,
                  const float* centroids, int32_t nprobe, int32_t metric, int32_t* out_ids,
                  float* out_dist) {
  if (nprobe > nlist || nprobe < 1 || metric < 0 || metric > 1) return -1;
  for (int64_t q = 0; q < Q; ++q)
    coarse_one(queries + q * D, D, centroids, nlist, nprobe, metric, out_ids + q * nprobe,
               out_dist ? out_dist + q * nprobe : nullptr);
  return 0;
}

// Batched thresholded look-up tables.  out_lut [Q][nprobe][M][256] fp32,
// out_mask [Q][nprobe][M][4] uint64 (may be null).
int oracle_build_lut(int64_t Q, int32_t D, int32_t M, const float* queries, const float* centroids,
                     const float* codebooks, const int32_t* probe_ids, int32_t nprobe,
                     const float* radii, int32_t radii_stride, int32_t mode, int32_t metric,
                     float* out_lut, uint64_t* out_mask) {
  if (D % M || mode < 0 || mode > 2 || metric < 0 || metric > 1 ||
      (radii_stride != 0 && radii_stride != M))
    return -1;
  for (int64_t q = 0; q < Q; ++q)
    for (int p = 0; p < nprobe; ++p) {
      const size_t row = (size_t)q * nprobe + p;
      lut_any(queries + q * D, centroids + (size_t)probe_ids[row] * D, D, M, codebooks,
              radii + q * radii_stride, mode, metric, out_lut + row * M * E,
              out_mask ? out_mask + row * M * 4 : nullptr);
    }
  return 0;
}

// Distances of every candidate of every query, in probe order then list order.
// cand_offsets [Q+1] is filled with the prefix sum of the probed list sizes;
// out_dist / out_ids must hold cand_offsets[Q] entries (call once with both
// null to size them).
int oracle_scan_all(int64_t Q, int32_t D, int32_t M, const float* queries, const float* centroids,
                    const float* codebooks, const int64_t* list_offsets, const uint8_t* codes,
                    const int64_t* ids, const int32_t* probe_ids, int32_t nprobe,
                    const float* radii, int32_t radii_stride, int32_t mode, int32_t metric,
                    int64_t* cand_offsets, float* out_dist, int64_t* out_ids) {
  if (D % M || mode < 0 || mode > 2 || metric < 0 || metric > 1 ||
      (radii_stride != 0 && radii_stride != M))
    return -1;
  std::vector<float> lut((size_t)M * E);
  int64_t pos = 0;
  for (int64_t q = 0; q < Q; ++q) {
    cand_offsets[q] = pos;
    for (int p = 0; p < nprobe; ++p) {
      const int32_t c = probe_ids[q * nprobe + p];
      const int64_t b = list_offsets[c], e = list_offsets[c + 1];
      if (out_dist) {
        lut_any(queries + q * D, centroids + (size_t)c * D, D, M, codebooks,
                radii + q * radii_stride, mode, metric, lut.data(), nullptr);
        const float start = adc_start(queries + q * D, centroids + (size_t)c * D, D, mode, metric);
        for (int64_t i = b; i < e; ++i) {
          out_dist[pos + (i - b)] = adc_one(lut.data(), codes + i * M, M, start);
          out_ids[pos + (i - b)] = ids ? ids[i] : i;
        }
      }
      pos += e - b;
    }
  }
  cand_offsets[Q] = pos;
  return 0;
}

// Top-k of one candidate array.
int oracle_topk(int64_t n, const float* dist, const int64_t* ids, int32_t k, int64_t* out_ids,
                float* out_dist) {
  std::vector<Cand> cand((size_t)n);
  for (int64_t i = 0; i < n; ++i) cand[i] = {dist[i], ids[i]};
  topk_select(cand, k, out_ids, out_dist);
  return 0;
}

// The whole search path for queries [q_begin, q_end): filtering, thresholded
// table per probed list, distance calculation over that list, top-k over all
// candidates of the query.  out_ids / out_dist are [Q][k] and only rows in the
// range are written, so disjoint ranges may be run from different threads.
int oracle_search(int64_t q_begin, int64_t q_end, int32_t D, int32_t nlist, int32_t M,
                  const float* queries, const float* centroids, const float* codebooks,
                  const int64_t* list_offsets, const uint8_t* codes, const int64_t* ids,
                  int32_t nprobe, int32_t k, const float* radii, int32_t radii_stride, int32_t mode,
                  int32_t metric, int64_t* out_ids, float* out_dist) {
  if (D % M || nprobe > nlist || nprobe < 1 || k < 1 || mode < 0 || mode > 2 || metric < 0 ||
      metric > 1 || (radii_stride != 0 && radii_stride != M))
    return -1;
  std::vector<float> lut((size_t)M * E);
  std::vector<int32_t> probes(nprobe);
  std::vector<Cand> cand;
  for (int64_t q = q_begin; q < q_end; ++q) {
    const float* qv = queries + q * D;
    coarse_one(qv, D, centroids, nlist, nprobe, metric, probes.data(), nullptr);
    cand.clear();
    for (int p = 0; p < nprobe; ++p) {
      const int32_t c = probes[p];
      lut_any(qv, centroids + (size_t)c * D, D, M, codebooks, radii + q * radii_stride, mode,
              metric, lut.data(), nullptr);
      const float start = adc_start(qv, centroids + (size_t)c * D, D, mode, metric);
      for (int64_t i = list_offsets[c]; i < list_offsets[c + 1]; ++i)
        cand.push_back({adc_one(lut.data(), codes + i * M, M, start), ids ? ids[i] : i});
    }
    topk_select(cand, k, out_ids + q * k, out_dist + q * k);
  }
  return 0;
}

// Exact k nearest neighbours by the metric definition L2(q,x) = sum (x_i-q_i)^2
// (paper Sec. 2.1), or k largest inner products sum x_i q_i (reported negated, so
// that smaller is better), accumulated in double, order (value, id).  Brute force.
int oracle_exact_knn(int64_t N, int32_t D, const float* base, int64_t Q, const float* queries,
                     int32_t k, int32_t metric, int64_t* out_ids, double* out_dist) {
  std::vector<std::pair<double, int64_t>> d((size_t)N);
  for (int64_t q = 0; q < Q; ++q) {
    for (int64_t i = 0; i < N; ++i) {
      double acc = 0.0;
      for (int j = 0; j < D; ++j) {
        if (metric == 0) {
          double t = (double)base[i * D + j] - (double)queries[q * D + j];
          acc += t * t;
        } else {
          acc -= (double)base[i * D + j] * (double)queries[q * D + j];
        }
      }
      d[i] = {acc, i};
    }
    const size_t kk = std::min((size_t)k, (size_t)N);
    std::partial_sort(d.begin(), d.begin() + kk, d.end());
    for (int i = 0; i < k; ++i) {
      out_ids[q * k + i] = (size_t)i < kk ? d[i].second : -1;
      out_dist[q * k + i] = (size_t)i < kk ? d[i].first : std::numeric_limits<double>::infinity();
    }
  }
  return 0;
}

// Grid cell of a coordinate (R17): t = (x - lo) * cells_per_unit in fp32, cell =
// floor(t) clamped to [0, G-1] (projections outside the map use the border cell).
static inline int grid_cell(float x, float lo, float cells_per_unit, int G) {
  const float t = (x - lo) * cells_per_unit;
  if (!(t >= 1.0f)) return 0;
  if (t >= (float)G) return G - 1;
  return (int)t;
}

// Density map (paper Sec. 4.1): for every subspace a G x G grid; density of a cell =
// (number of projections that fall into it) / (area of the cell).  proj is
// [n][M][2], lo and cells_per_unit are [M][2] (cell width along axis j is
// 1 / cells_per_unit[m][j]); out is [M][G][G] with cell (i0, i1) at i0 * G + i1.
int oracle_density_map(int64_t n, int32_t M, const float* proj, const float* lo,
                       const float* cells_per_unit, int32_t G, double* out) {
  if (n < 0 || M < 1 || G < 1) return 1;
  for (int64_t i = 0; i < (int64_t)M * G * G; ++i) out[i] = 0.0;
  for (int64_t p = 0; p < n; ++p)
    for (int m = 0; m < M; ++m) {
      const int i0 = grid_cell(proj[(p * M + m) * 2 + 0], lo[m * 2 + 0], cells_per_unit[m * 2 + 0], G);
      const int i1 = grid_cell(proj[(p * M + m) * 2 + 1], lo[m * 2 + 1], cells_per_unit[m * 2 + 1], G);
      out[((int64_t)m * G + i0) * G + i1] += 1.0;
    }
  for (int m = 0; m < M; ++m) {
    const double area = 1.0 / ((double)cells_per_unit[m * 2 + 0] * (double)cells_per_unit[m * 2 + 1]);
    for (int c = 0; c < G * G; ++c) out[(int64_t)m * G * G + c] /= area;
  }
  return 0;
}

// Query-specific thresholds (paper Sec. 4.1; Algorithm 2 threshold step; R17).
// For query q and subspace m (dsub = 2), with c = nearest[q]:
//   (x, y) = q[2m .. 2m+1] - centroid_c[2m .. 2m+1]
//   f      = map[m][cell(x)][cell(y)]
//   p      = coef[m][degree]; p = fmaf(p, f, coef[m][d]) for d = degree-1 .. 0
//   thres  = (0 < p < inf ? p : fallback[m]) * scale
int oracle_query_radii(int64_t Q, int32_t D, int32_t M, const float* queries, const float* centroids,
                       int32_t nlist, const int32_t* nearest, int32_t G, const float* lo,
                       const float* cells_per_unit, const float* map, int32_t degree,
                       const float* coef, const float* fallback, float scale, float* out) {
  if (Q < 0 || M < 1 || D != 2 * M || G < 1 || degree < 0) return 1;
  for (int64_t q = 0; q < Q; ++q) {
    const int32_t c = nearest[q];
    if (c < 0 || c >= nlist) return 1;
    for (int m = 0; m < M; ++m) {
      const float x = queries[q * D + 2 * m] - centroids[(int64_t)c * D + 2 * m];
      const float y = queries[q * D + 2 * m + 1] - centroids[(int64_t)c * D + 2 * m + 1];
      const int i0 = grid_cell(x, lo[m * 2 + 0], cells_per_unit[m * 2 + 0], G);
      const int i1 = grid_cell(y, lo[m * 2 + 1], cells_per_unit[m * 2 + 1], G);
      const float f = map[((int64_t)m * G + i0) * G + i1];
      float p = coef[m * (degree + 1) + degree];
      for (int d = degree - 1; d >= 0; --d) p = std::fmaf(p, f, coef[m * (degree + 1) + d]);
      const bool usable = p > 0.0f && p < std::numeric_limits<float>::infinity();
      out[q * M + m] = (usable ? p : fallback[m]) * scale;
    }
  }
  return 0;
}

}  // extern "C"
