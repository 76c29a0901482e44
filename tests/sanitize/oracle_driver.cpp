// Sanitizer leg for the CPU oracle: compiled together with oracle/ivfpq_oracle.cpp under
// -fsanitize=address,undefined and run on small seeded indexes that include the edge cases
// (empty lists, a single list, k above the number of candidates, every list probed, per-query
// radii, infinite and zero radii, all scoring modes, both metrics).  Any out-of-bounds access,
// overflow or misaligned access aborts the program; beyond that it checks that the fused search
// equals the composition of the stages.  Exit status 0 means clean.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <limits>
#include <vector>

extern "C" {
int oracle_coarse(int64_t Q, int32_t D, int32_t nlist, const float* queries, const float* centroids,
                  int32_t nprobe, int32_t metric, int32_t* out_ids, float* out_dist);
int oracle_build_lut(int64_t Q, int32_t D, int32_t M, const float* queries, const float* centroids,
                     const float* codebooks, const int32_t* probe_ids, int32_t nprobe, const float* radii,
                     int32_t radii_stride, int32_t mode, int32_t metric, float* out_lut, uint64_t* out_mask);
int oracle_scan_all(int64_t Q, int32_t D, int32_t M, const float* queries, const float* centroids,
                    const float* codebooks, const int64_t* list_offsets, const uint8_t* codes,
                    const int64_t* ids, const int32_t* probe_ids, int32_t nprobe, const float* radii,
                    int32_t radii_stride, int32_t mode, int32_t metric, int64_t* cand_offsets,
                    float* out_dist, int64_t* out_ids);
int oracle_topk(int64_t n, const float* dist, const int64_t* ids, int32_t k, int64_t* out_ids, float* out_dist);
int oracle_search(int64_t q_begin, int64_t q_end, int32_t D, int32_t nlist, int32_t M, const float* queries,
                  const float* centroids, const float* codebooks, const int64_t* list_offsets,
                  const uint8_t* codes, const int64_t* ids, int32_t nprobe, int32_t k, const float* radii,
                  int32_t radii_stride, int32_t mode, int32_t metric, int64_t* out_ids, float* out_dist);
int oracle_exact_knn(int64_t N, int32_t D, const float* base, int64_t Q, const float* queries, int32_t k,
                     int32_t metric, int64_t* out_ids, double* out_dist);
int oracle_density_map(int64_t n, int32_t M, const float* proj, const float* lo, const float* cells_per_unit,
                       int32_t G, double* out);
int oracle_query_radii(int64_t Q, int32_t D, int32_t M, const float* queries, const float* centroids,
                       int32_t nlist, const int32_t* nearest, int32_t G, const float* lo,
                       const float* cells_per_unit, const float* map, int32_t degree, const float* coef,
                       const float* fallback, float scale, float* out);
}

static uint64_t g_state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd() {
  g_state = g_state * 6364136223846793005ull + 1442695040888963407ull;
  return (uint32_t)(g_state >> 33);
}
static float unit() { return (float)(rnd() & 0xFFFFFF) / 16777216.0f; }

#define REQUIRE(c)                                                            \
  do {                                                                        \
    if (!(c)) {                                                               \
      std::fprintf(stderr, "oracle_driver: %s failed at line %d\n", #c, __LINE__); \
      std::exit(2);                                                           \
    }                                                                         \
  } while (0)

static void one_case(int N, int D, int M, int nlist, int Q, int nprobe, int k, int mode, int metric,
                     int radii_kind /*0 finite shared, 1 per query, 2 +inf, 3 zero*/, bool with_ids) {
  const int dsub = D / M;
  std::vector<float> cent((size_t)nlist * D), cb((size_t)M * 256 * dsub), q((size_t)Q * D);
  for (auto& v : cent) v = unit() * 2 - 1;
  for (auto& v : cb) v = (unit() * 2 - 1) * 0.5f;
  for (auto& v : q) v = unit() * 2 - 1;
  // list sizes: some empty, one long
  std::vector<int64_t> offs(nlist + 1, 0);
  std::vector<int> label(N);
  for (int i = 0; i < N; ++i) label[i] = (rnd() % 3 == 0) ? 0 : (int)(rnd() % nlist);
  if (nlist > 2) for (int i = 0; i < N; ++i) if (label[i] == 1) label[i] = 2;  // list 1 stays empty
  for (int i = 0; i < N; ++i) offs[label[i] + 1]++;
  for (int c = 0; c < nlist; ++c) offs[c + 1] += offs[c];
  std::vector<uint8_t> codes((size_t)N * M);
  for (auto& v : codes) v = (uint8_t)rnd();
  std::vector<int64_t> ids(N);
  for (int i = 0; i < N; ++i) ids[i] = 1000 + 7 * (int64_t)i;
  const int stride = radii_kind == 1 ? M : 0;
  std::vector<float> radii(radii_kind == 1 ? (size_t)Q * M : (size_t)M);
  for (auto& v : radii)
    v = radii_kind == 2 ? std::numeric_limits<float>::infinity() : (radii_kind == 3 ? 0.0f : 0.2f + unit());

  std::vector<int32_t> pid((size_t)Q * nprobe);
  std::vector<float> pd((size_t)Q * nprobe);
  REQUIRE(oracle_coarse(Q, D, nlist, q.data(), cent.data(), nprobe, metric, pid.data(), pd.data()) == 0);
  std::vector<float> lut((size_t)Q * nprobe * M * 256);
  std::vector<uint64_t> mask((size_t)Q * nprobe * M * 4);
  REQUIRE(oracle_build_lut(Q, D, M, q.data(), cent.data(), cb.data(), pid.data(), nprobe, radii.data(), stride,
                           mode, metric, lut.data(), mask.data()) == 0);
  std::vector<int64_t> co(Q + 1);
  const int64_t* idp = with_ids ? ids.data() : nullptr;
  REQUIRE(oracle_scan_all(Q, D, M, q.data(), cent.data(), cb.data(), offs.data(), codes.data(), idp, pid.data(),
                          nprobe, radii.data(), stride, mode, metric, co.data(), nullptr, nullptr) == 0);
  std::vector<float> cd((size_t)co[Q] + 1);
  std::vector<int64_t> ci((size_t)co[Q] + 1);
  REQUIRE(oracle_scan_all(Q, D, M, q.data(), cent.data(), cb.data(), offs.data(), codes.data(), idp, pid.data(),
                          nprobe, radii.data(), stride, mode, metric, co.data(), cd.data(), ci.data()) == 0);
  std::vector<int64_t> oi((size_t)Q * k), ti(k);
  std::vector<float> od((size_t)Q * k), td(k);
  REQUIRE(oracle_search(0, Q, D, nlist, M, q.data(), cent.data(), cb.data(), offs.data(), codes.data(), idp,
                        nprobe, k, radii.data(), stride, mode, metric, oi.data(), od.data()) == 0);
  for (int qi = 0; qi < Q; ++qi) {  // fused == stages composed
    REQUIRE(oracle_topk(co[qi + 1] - co[qi], cd.data() + co[qi], ci.data() + co[qi], k, ti.data(), td.data()) == 0);
    for (int j = 0; j < k; ++j) {
      REQUIRE(ti[j] == oi[(size_t)qi * k + j]);
      REQUIRE(td[j] == od[(size_t)qi * k + j] || (std::isinf(td[j]) && std::isinf(od[(size_t)qi * k + j])));
    }
  }
}

int main() {
  int cases = 0;
  for (int metric = 0; metric < 2; ++metric)
    for (int mode = 0; mode < 3; ++mode)
      for (int rk = 0; rk < 4; ++rk) {
        one_case(300, 12, 6, 5, 7, 3, 10, mode, metric, rk, true);
        one_case(40, 8, 8, 4, 3, 4, 64, mode, metric, rk, false);   // every list probed, k > candidates
        one_case(0, 6, 3, 2, 2, 1, 5, mode, metric, rk, true);      // an index without points
        one_case(65, 15, 5, 1, 4, 1, 3, mode, metric, rk, false);   // a single list, dsub = 3
        cases += 4;
      }
  // exact search, density map and per-query radii
  {
    const int N = 50, D = 6, Q = 4, k = 60;
    std::vector<float> base((size_t)N * D), q((size_t)Q * D);
    for (auto& v : base) v = unit();
    for (auto& v : q) v = unit();
    std::vector<int64_t> oi((size_t)Q * k);
    std::vector<double> od((size_t)Q * k);
    for (int metric = 0; metric < 2; ++metric)
      REQUIRE(oracle_exact_knn(N, D, base.data(), Q, q.data(), k, metric, oi.data(), od.data()) == 0);
    const int M = 3, G = 5, n = 200, degree = 2, nlist = 3;
    std::vector<float> proj((size_t)n * M * 2), lo(M * 2, -0.25f), cpu(M * 2, 4.0f);
    for (auto& v : proj) v = unit() * 3 - 1;  // a good share falls outside the map
    std::vector<double> dm((size_t)M * G * G);
    REQUIRE(oracle_density_map(n, M, proj.data(), lo.data(), cpu.data(), G, dm.data()) == 0);
    std::vector<float> fmap(dm.begin(), dm.end()), coef((size_t)M * (degree + 1), 0.01f), fb(M, 0.5f), cent((size_t)nlist * D, 0.1f);
    std::vector<int32_t> near(Q, 2);
    std::vector<float> out((size_t)Q * M);
    q[0] = std::numeric_limits<float>::quiet_NaN();  // NaN projection goes to cell 0
    REQUIRE(oracle_query_radii(Q, D, M, q.data(), cent.data(), nlist, near.data(), G, lo.data(), cpu.data(),
                               fmap.data(), degree, coef.data(), fb.data(), 0.75f, out.data()) == 0);
    near[1] = 3;  // outside the index: refused, nothing read
    REQUIRE(oracle_query_radii(Q, D, M, q.data(), cent.data(), nlist, near.data(), G, lo.data(), cpu.data(),
                               fmap.data(), degree, coef.data(), fb.data(), 0.75f, out.data()) != 0);
    cases += 4;
  }
  std::printf("oracle_driver: %d cases clean\n", cases);
  return 0;
}
