// Sanitizer leg for the host side of the C ABI: csrc/api.hip (host pass only) linked with
// launch stubs, run under -fsanitize=address,undefined without a GPU.  It walks the
// rejection paths of every entry point (null pointers, sizes outside the limits, bad radii,
// bad list offsets, workspace missing / misaligned / too small), checks that accepted calls
// reach the launchers, and sweeps the workspace planner for overlap and alignment.
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <limits>
#include <vector>

#include "ivfpq_internal.h"

#define REQUIRE(c)                                                                          \
  do {                                                                                      \
    if (!(c)) {                                                                             \
      std::fprintf(stderr, "api_driver: %s failed at line %d (last error: %s)\n", #c, __LINE__, \
                   ivfpq_last_error());                                                     \
      std::exit(2);                                                                         \
    }                                                                                       \
  } while (0)

static ivfpq_index fake_index(int64_t N, int D, int nlist, int M) {
  ivfpq_index ix;
  std::memset(&ix, 0, sizeof ix);
  ix.N = N; ix.D = D; ix.nlist = nlist; ix.M = M; ix.dsub = D / M; ix.Mp = (M + 3) & ~3;
  ix.metric = IVFPQ_METRIC_L2;
  ix.device = 0;
  return ix;
}

static void sweep_workspace() {
  const int nlists[] = {1, 7, 64, 1000, 1024, 16384, 100000};
  const int64_t Qs[] = {0, 1, 2, 63, 128, 2047, 2048, 10000, 300000};
  const int nprobes[] = {1, 8, 64, 1024};
  int n = 0;
  for (int nlist : nlists)
    for (int64_t Q : Qs)
      for (int nprobe : nprobes) {
        if (nprobe > nlist) continue;
        ivfpq_index ix = fake_index(1000, 128, nlist, 64);
        const ivfpq::Workspace w = ivfpq::plan_workspace(&ix, Q, nprobe, 100);
        REQUIRE(w.q_chunk >= 1 && w.nsplit >= 1 && w.nsplit <= nprobe && w.nlist_pad >= nlist);
        // scratch of the filtering stage: rows of the product, or keys + reference-order rows (many lists)
        const int nkeys = ivfpq::coarse_fused_keys(nlist, nprobe, 128);
        REQUIRE((nkeys > 0) == (nlist >= 16384 && nprobe <= 64));   // of the shapes swept here
        const size_t scratch = ivfpq::coarse_scratch_floats(w.nlist_pad, nkeys, w.q_chunk) * 4;
        REQUIRE(scratch <= ((size_t)1 << 30) + (size_t)(128 + ivfpq::FB_SLOTS) * w.nlist_pad * 4 + 1024);
        REQUIRE(nkeys == 0 || Q < 2000 || scratch < (size_t)Q * w.nlist_pad * 4 / 4);   // no full rows any more
        // regions in order, 256-byte aligned, inside the total
        const size_t ends[] = {w.coarse_dist + scratch,
                               w.probe_ids + (size_t)Q * nprobe * 4, w.probe_dist + (size_t)Q * nprobe * 4};
        REQUIRE(w.coarse_dist % 256 == 0 && w.probe_ids % 256 == 0 && w.probe_dist % 256 == 0 && w.coarse_flags % 256 == 0);
        REQUIRE(ends[0] <= w.probe_ids && ends[1] <= w.probe_dist && ends[2] <= w.coarse_flags);
        REQUIRE(w.coarse_flags + (size_t)Q * 4 <= w.total);
        if (w.nsplit > 1) {
          REQUIRE(w.part_d % 256 == 0 && w.part_id % 256 == 0 && w.coarse_flags + (size_t)Q * 4 <= w.part_d);
          REQUIRE(w.part_d + (size_t)Q * w.nsplit * 128 * 4 <= w.part_id);
          REQUIRE(w.part_id + (size_t)Q * w.nsplit * 128 * 8 <= w.total);
        }
        const size_t pub = ivfpq_search_workspace_bytes(&ix, Q, nprobe, 100);
        REQUIRE(pub >= w.total && pub >= 256);
        // k above 128: the slots of the one-pass selection lie behind the usual workspace
        REQUIRE(Q > 0 || ivfpq::plan_wide(&ix, Q, 1000, 0).total == 0);
        for (int k : {129, 1000, 1024}) {
          if (Q == 0) break;
          const ivfpq::WideWorkspace ww = ivfpq::plan_wide(&ix, Q, k, 0);
          REQUIRE(ww.total > 0 && ww.cap == 8192 && ww.q_chunk >= 1 && ww.q_chunk <= Q);
          REQUIRE(ww.q_chunk == Q || (size_t)ww.q_chunk * ww.cap * 12 <= ((size_t)1 << 30));
          REQUIRE(ww.d % 256 == 0 && ww.id % 256 == 0 && ww.n % 256 == 0 && ww.bound % 256 == 0 && ww.qmap % 256 == 0);
          REQUIRE(ww.d + (size_t)ww.q_chunk * ww.cap * 4 <= ww.id && ww.id + (size_t)ww.q_chunk * ww.cap * 8 <= ww.n);
          REQUIRE(ww.n + (size_t)ww.q_chunk * 4 <= ww.bound && ww.bound + (size_t)ww.q_chunk * 4 <= ww.qmap);
          REQUIRE(ww.qmap + (size_t)ww.q_chunk * 4 <= ww.total);
          const size_t pubk = ivfpq_search_workspace_bytes(&ix, Q, nprobe, k);
          REQUIRE(pubk >= ((ivfpq::plan_workspace(&ix, Q, nprobe, k).total + 255) & ~(size_t)255) + ww.total);
        }
        REQUIRE(ivfpq::plan_wide(&ix, Q, 128, 0).total == 0 && ivfpq::plan_wide(&ix, Q, 1000, 1).total == 0);
        ++n;
      }
  std::printf("api_driver: workspace planner clean on %d shapes\n", n);
}

static void index_descriptions() {
  const int nlist = 4, D = 8, M = 4;
  const int64_t N = 10;
  std::vector<float> cent((size_t)nlist * D, 0.0f), cb((size_t)M * 256 * (D / M), 0.0f);
  std::vector<uint8_t> codes((size_t)N * M, 0);
  int64_t offs[5] = {0, 3, 3, 7, 10};
  ivfpq_index_desc d;
  std::memset(&d, 0, sizeof d);
  d.N = N; d.D = D; d.nlist = nlist; d.M = M; d.ksub = 256;
  d.centroids = cent.data(); d.codebooks = cb.data(); d.list_offsets = offs; d.codes = codes.data();
  ivfpq_index *out = reinterpret_cast<ivfpq_index *>(0x1);
  auto expect = [&](ivfpq_index_desc v, int status) {
    out = reinterpret_cast<ivfpq_index *>(0x1);
    const int rc = ivfpq_index_create(&v, &out);
    REQUIRE(rc == status);
    REQUIRE(out == nullptr);
    REQUIRE(std::strlen(ivfpq_last_error()) > 0);
  };
  REQUIRE(ivfpq_index_create(nullptr, &out) == IVFPQ_ERR_INVALID_ARGUMENT);
  REQUIRE(ivfpq_index_create(&d, nullptr) == IVFPQ_ERR_INVALID_ARGUMENT);
  { auto v = d; v.ksub = 16; expect(v, IVFPQ_ERR_UNSUPPORTED); }
  { auto v = d; v.D = 9; expect(v, IVFPQ_ERR_INVALID_ARGUMENT); }
  { auto v = d; v.M = 0; expect(v, IVFPQ_ERR_INVALID_ARGUMENT); }
  { auto v = d; v.M = 256; v.D = 256; expect(v, IVFPQ_ERR_UNSUPPORTED); }
  { auto v = d; v.nlist = 0; expect(v, IVFPQ_ERR_INVALID_ARGUMENT); }
  { auto v = d; v.N = -1; expect(v, IVFPQ_ERR_INVALID_ARGUMENT); }
  { auto v = d; v.N = (int64_t)1 << 33; expect(v, IVFPQ_ERR_UNSUPPORTED); }
  { auto v = d; v.metric = 2; expect(v, IVFPQ_ERR_INVALID_ARGUMENT); }
  { auto v = d; v.centroids = nullptr; expect(v, IVFPQ_ERR_INVALID_ARGUMENT); }
  { auto v = d; v.codes = nullptr; expect(v, IVFPQ_ERR_INVALID_ARGUMENT); }
  { int64_t bad[5] = {0, 3, 2, 7, 10}; auto v = d; v.list_offsets = bad; expect(v, IVFPQ_ERR_INVALID_ARGUMENT); }
  { int64_t bad[5] = {1, 3, 3, 7, 10}; auto v = d; v.list_offsets = bad; expect(v, IVFPQ_ERR_INVALID_ARGUMENT); }
  { int64_t bad[5] = {0, 3, 3, 7, 9}; auto v = d; v.list_offsets = bad; expect(v, IVFPQ_ERR_INVALID_ARGUMENT); }
  // a list longer than 2^31 points (offsets only: nothing behind them is read before the refusal)
  { int64_t bad[5] = {0, 0, 0, 0, (int64_t)3 << 30}; auto v = d; v.N = (int64_t)3 << 30; v.list_offsets = bad;
    expect(v, IVFPQ_ERR_UNSUPPORTED); }
  std::printf("api_driver: index descriptions clean\n");
}

static void search_arguments() {
  ivfpq_index ix = fake_index(1000, 16, 8, 4);
  alignas(256) static unsigned char ws_mem[1 << 16];
  alignas(16) float q[4 * 16] = {0};
  float radii[4] = {1.0f, 2.0f, std::numeric_limits<float>::infinity(), 0.0f};
  int64_t ids[4 * 5];
  float dist[4 * 5];
  int32_t pid[4 * 2] = {0};
  const size_t need = ivfpq_search_workspace_bytes(&ix, 4, 2, 5);
  REQUIRE(need > 0 && need <= sizeof ws_mem);
  auto search = [&](const ivfpq_index *i, const float *qq, int64_t Q, int nprobe, int k, const float *r,
                    void *ws, size_t wsb) {
    return ivfpq_search(i, qq, Q, nprobe, k, r, ids, dist, ws, wsb, nullptr);
  };
  REQUIRE(search(nullptr, q, 4, 2, 5, radii, ws_mem, need) == IVFPQ_ERR_INVALID_ARGUMENT);
  REQUIRE(search(&ix, nullptr, 4, 2, 5, radii, ws_mem, need) == IVFPQ_ERR_INVALID_ARGUMENT);
  REQUIRE(search(&ix, q + 1, 4, 2, 5, radii, ws_mem, need) == IVFPQ_ERR_INVALID_ARGUMENT);   // misaligned queries
  REQUIRE(search(&ix, q, -1, 2, 5, radii, ws_mem, need) == IVFPQ_ERR_INVALID_ARGUMENT);
  REQUIRE(search(&ix, q, 4, 0, 5, radii, ws_mem, need) == IVFPQ_ERR_INVALID_ARGUMENT);
  REQUIRE(search(&ix, q, 4, 9, 5, radii, ws_mem, need) == IVFPQ_ERR_INVALID_ARGUMENT);
  REQUIRE(search(&ix, q, 4, 2, 0, radii, ws_mem, need) == IVFPQ_ERR_INVALID_ARGUMENT);
  REQUIRE(search(&ix, q, 4, 2, IVFPQ_MAX_K + 1, radii, ws_mem, need) == IVFPQ_ERR_UNSUPPORTED);
  REQUIRE(search(&ix, q, 4, 2, 5, nullptr, ws_mem, need) == IVFPQ_ERR_INVALID_ARGUMENT);
  { float bad[4] = {1.0f, -1.0f, 1.0f, 1.0f}; REQUIRE(search(&ix, q, 4, 2, 5, bad, ws_mem, need) == IVFPQ_ERR_INVALID_ARGUMENT); }
  { float bad[4] = {1.0f, 1.0f, std::nanf(""), 1.0f}; REQUIRE(search(&ix, q, 4, 2, 5, bad, ws_mem, need) == IVFPQ_ERR_INVALID_ARGUMENT); }
  REQUIRE(search(&ix, q, 4, 2, 5, radii, nullptr, need) == IVFPQ_ERR_WORKSPACE);
  REQUIRE(search(&ix, q, 4, 2, 5, radii, ws_mem + 64, need) == IVFPQ_ERR_WORKSPACE);
  REQUIRE(search(&ix, q, 4, 2, 5, radii, ws_mem, need - 1) == IVFPQ_ERR_WORKSPACE);
  REQUIRE(search(&ix, q, 0, 2, 5, radii, ws_mem, need) == IVFPQ_OK);  // an empty batch is a no-op
  // accepted: the call gets as far as the first launcher (a stub here)
  REQUIRE(search(&ix, q, 4, 2, 5, radii, ws_mem, need) == IVFPQ_ERR_HIP);
  { ivfpq_index big = fake_index(1000, 16, 4096, 4);
    REQUIRE(ivfpq_coarse(&big, q, 4, IVFPQ_MAX_NPROBE + 1, pid, nullptr, ws_mem, sizeof ws_mem, nullptr) == IVFPQ_ERR_UNSUPPORTED); }
  REQUIRE(ivfpq_coarse(&ix, q, 4, 2, nullptr, nullptr, ws_mem, need, nullptr) == IVFPQ_ERR_INVALID_ARGUMENT);
  REQUIRE(ivfpq_scan_topk(&ix, q, 4, 2, nullptr, 5, radii, ids, dist, ws_mem, need, nullptr) == IVFPQ_ERR_INVALID_ARGUMENT);
  REQUIRE(ivfpq_scan_topk(&ix, q, 4, 2, pid, 5, radii, ids, nullptr, ws_mem, need, nullptr) == IVFPQ_ERR_INVALID_ARGUMENT);
  REQUIRE(ivfpq_build_lut(&ix, q, 4, 2, pid, radii, nullptr, nullptr, nullptr) == IVFPQ_ERR_INVALID_ARGUMENT);
  { ivfpq_scoring sc = {7, nullptr, 0};
    REQUIRE(ivfpq_search_ex(&ix, q, 4, 2, 5, radii, &sc, ids, dist, ws_mem, need, nullptr) == IVFPQ_ERR_INVALID_ARGUMENT); }
  { ivfpq_scoring sc = {0, nullptr, 5};
    REQUIRE(ivfpq_search_ex(&ix, q, 4, 2, 5, radii, &sc, ids, dist, ws_mem, need, nullptr) == IVFPQ_ERR_INVALID_ARGUMENT); }
  REQUIRE(ivfpq_set_option("lm_first", 0) == IVFPQ_ERR_INVALID_ARGUMENT);
  REQUIRE(ivfpq_set_option("lm_cap", 8) == IVFPQ_ERR_INVALID_ARGUMENT);
  REQUIRE(ivfpq_set_option("lm_first", 1) == IVFPQ_OK && ivfpq_set_option("lm_cap", 4096) == IVFPQ_OK &&
          ivfpq_set_option("lm_cap", 0) == IVFPQ_OK);
  REQUIRE(ivfpq_set_option("wide_cap", 512) == IVFPQ_ERR_INVALID_ARGUMENT && ivfpq_set_option("wide_cap", 1 << 17) == IVFPQ_ERR_INVALID_ARGUMENT);
  REQUIRE(ivfpq_set_option("wide_cap", 0) == IVFPQ_OK && ivfpq_search_workspace_bytes(&ix, 4, 2, 1000) == ivfpq_search_workspace_bytes(&ix, 4, 2, 100));
  REQUIRE(ivfpq_set_option("wide_cap", 8192) == IVFPQ_OK && ivfpq_search_workspace_bytes(&ix, 4, 2, 1000) > ivfpq_search_workspace_bytes(&ix, 4, 2, 100));
  REQUIRE(ivfpq_scan_all(&ix, q, 4, 2, pid, radii, nullptr, nullptr, nullptr, nullptr, nullptr) == IVFPQ_ERR_INVALID_ARGUMENT);
  REQUIRE(ivfpq_set_option("scan_ablate", 1) == IVFPQ_ERR_INVALID_ARGUMENT);   // result-changing bits are gone
  REQUIRE(ivfpq_set_option("scan_ablate", 8 | 16 | 32 | 64 | 128) == IVFPQ_OK && ivfpq_set_option("scan_ablate", 256) == IVFPQ_ERR_INVALID_ARGUMENT);
  REQUIRE(ivfpq_set_option("bound_grid", 3) == IVFPQ_ERR_INVALID_ARGUMENT && ivfpq_set_option("bound_grid", 1) == IVFPQ_OK && ivfpq_set_option("bound_grid", 0) == IVFPQ_OK);
  REQUIRE(ivfpq_set_option("scan_ablate", 0) == IVFPQ_OK);
  REQUIRE(ivfpq_set_option("scan_loads", 4) == IVFPQ_ERR_INVALID_ARGUMENT);
  REQUIRE(ivfpq_set_option("scan_waves", 5) == IVFPQ_ERR_INVALID_ARGUMENT);
  REQUIRE(ivfpq_set_option(nullptr, 0) == IVFPQ_ERR_INVALID_ARGUMENT);
  // the entry point without a workspace: same argument checks, sizes beyond its built-in scratch refused
  REQUIRE(ivfpq_search_noalloc(nullptr, q, 4, 2, 5, radii, ids, dist, nullptr) == IVFPQ_ERR_INVALID_ARGUMENT);
  REQUIRE(ivfpq_search_noalloc(&ix, q, 4, 2, 0, radii, ids, dist, nullptr) == IVFPQ_ERR_INVALID_ARGUMENT);
  REQUIRE(ivfpq_search_noalloc(&ix, q, 4, 2, 5, nullptr, ids, dist, nullptr) == IVFPQ_ERR_INVALID_ARGUMENT);
  REQUIRE(ivfpq_search_noalloc(&ix, q, 4, 2, 5, radii, nullptr, dist, nullptr) == IVFPQ_ERR_INVALID_ARGUMENT);
  REQUIRE(ivfpq_search_noalloc(&ix, q, 0, 2, 5, radii, ids, dist, nullptr) == IVFPQ_OK);
  { ivfpq_index wide = fake_index(1000, 16, 100000, 4);   // 128 rows of 100 032 floats do not fit 32 MiB
    REQUIRE(ivfpq_search_noalloc(&wide, q, 4, 2, 5, radii, ids, dist, nullptr) == IVFPQ_OK ||
            std::strlen(ivfpq_last_error()) > 0);
    REQUIRE(ivfpq_search_noalloc(&wide, q, 200, 2, 5, radii, ids, dist, nullptr) == IVFPQ_ERR_WORKSPACE);
    REQUIRE(ivfpq_search_noalloc(&ix, q, 5000000, 8, 5, radii, ids, dist, nullptr) == IVFPQ_ERR_WORKSPACE); }
  // budgeted plans: whatever fits stays inside the budget, chunks are whole multiples of 128 or the batch
  { const int nlists[] = {8, 1024, 16384, 60000, 100000};
    const int64_t Qs[] = {1, 100, 127, 128, 3000, 10000, 200000};
    for (int nl : nlists)
      for (int64_t Q : Qs) {
        ivfpq_index b = fake_index(1000, 16, nl, 4);
        const int np = nl < 64 ? nl : 64;
        const ivfpq::Workspace w = ivfpq::plan_workspace(&b, Q, np, 100, IVFPQ_NOALLOC_SCRATCH_BYTES);
        if (w.total == SIZE_MAX) continue;
        REQUIRE(w.total <= IVFPQ_NOALLOC_SCRATCH_BYTES);
        REQUIRE(w.q_chunk >= 1 && (w.q_chunk == Q || w.q_chunk % 128 == 0) && w.q_chunk <= Q);
        REQUIRE(w.coarse_dist + ivfpq::coarse_scratch_floats(w.nlist_pad, ivfpq::coarse_fused_keys(nl, np, 16), w.q_chunk) * 4 <= w.probe_ids);
      } }
  ivfpq_index_info info;
  REQUIRE(ivfpq_index_get_info(&ix, &info) == IVFPQ_OK && info.D == 16 && info.dsub == 4);
  // radius model descriptions
  { ivfpq_index ix2 = fake_index(1000, 8, 8, 4);
    const int M = 4, G = 3;
    std::vector<float> lo(2 * M, 0.0f), cpu(2 * M, 1.0f), map((size_t)M * G * G, 0.0f), coef(M * 2, 0.0f), fb(M, 1.0f);
    ivfpq_radius_model_desc md = {M, G, 1, lo.data(), cpu.data(), map.data(), coef.data(), fb.data()};
    ivfpq_radius_model *out = nullptr;
    { auto v = md; v.M = 5; REQUIRE(ivfpq_radius_model_create(&ix2, &v, &out) == IVFPQ_ERR_INVALID_ARGUMENT); }
    { auto v = md; v.grid = 0; REQUIRE(ivfpq_radius_model_create(&ix2, &v, &out) == IVFPQ_ERR_INVALID_ARGUMENT); }
    { auto v = md; v.degree = 9; REQUIRE(ivfpq_radius_model_create(&ix2, &v, &out) == IVFPQ_ERR_INVALID_ARGUMENT); }
    { auto v = md; v.map = nullptr; REQUIRE(ivfpq_radius_model_create(&ix2, &v, &out) == IVFPQ_ERR_INVALID_ARGUMENT); }
    { cpu[3] = 0.0f; REQUIRE(ivfpq_radius_model_create(&ix2, &md, &out) == IVFPQ_ERR_INVALID_ARGUMENT); cpu[3] = 1.0f; }
    { fb[1] = -1.0f; REQUIRE(ivfpq_radius_model_create(&ix2, &md, &out) == IVFPQ_ERR_INVALID_ARGUMENT); fb[1] = 1.0f; }
    REQUIRE(ivfpq_radius_model_create(&ix, &md, &out) == IVFPQ_ERR_UNSUPPORTED);   // dsub = 4
    REQUIRE(out == nullptr);
  }
  std::printf("api_driver: search-side argument checks clean\n");
}

int main() {
  sweep_workspace();
  index_descriptions();
  search_arguments();
  std::printf("api_driver: clean\n");
  return 0;
}
