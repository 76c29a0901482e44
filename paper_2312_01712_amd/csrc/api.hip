// C ABI of the library: argument validation, index construction, workspace
// planning and the entry points declared in include/ivfpq.h.  No kernel lives
// here; every step of the search path runs in coarse.hip / scan.hip.

#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <atomic>
#include <new>
#include <vector>

#include "ivfpq_internal.h"

namespace ivfpq {

static thread_local char g_err[512] = "";

void set_error(const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
}

int hip_fail(hipError_t e, const char *what) {
  set_error("HIP error %d (%s) in %s", (int)e, hipGetErrorString(e), what);
  return IVFPQ_ERR_HIP;
}

static size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

// budget == 0: the proposal matrix of the filtering stage takes up to 1 GiB (queries are
// processed in chunks of q_chunk).  budget > 0: everything must fit in `budget` bytes; the
// chunk shrinks (in steps of 128 queries) to make it fit, and total = SIZE_MAX says that not
// even the smallest chunk does.
Workspace plan_workspace(const ivfpq_index *ix, int64_t Q, int32_t nprobe, int32_t k, size_t budget) {
  (void)k;
  Workspace w;
  memset(&w, 0, sizeof w);
  w.nlist_pad = (ix->nlist + 63) & ~63;
  // enough workgroups to fill 256 CUs a few times over when the batch is small
  int64_t ns = Q > 0 ? (2048 + Q - 1) / Q : 1;
  if (ns > nprobe) ns = nprobe;
  if (ns > 64) ns = 64;
  if (ns < 1) ns = 1;
  w.nsplit = (int32_t)ns;
  size_t fixed = 2 * align256((size_t)Q * nprobe * 4) + align256((size_t)Q * 4);
  if (w.nsplit > 1) fixed += align256((size_t)Q * w.nsplit * 128 * 4) + align256((size_t)Q * w.nsplit * 128 * 8);
  // scratch of the filtering stage per query: a row of the product, or (many lists) the keys
  // the product keeps plus a sixteenth of a row for the queries that need every distance
  const int32_t nkeys = coarse_fused_keys(ix->nlist, nprobe, ix->D);
  const size_t row_bytes = nkeys > 0 ? (size_t)nkeys * 4 + (size_t)w.nlist_pad / 4 + 1 : (size_t)w.nlist_pad * 4;
  int64_t qc = ((int64_t)1 << 30) / (int64_t)row_bytes;
  qc &= ~(int64_t)127;
  if (qc < 128) qc = 128;
  if (budget > 0) {
    const size_t spare = 256 + (nkeys > 0 ? (size_t)(FB_SLOTS + 1) * w.nlist_pad * 4 + 1024 : 0);   // fixed part and rounding of the scratch size
    const int64_t fit = fixed + spare <= budget ? (int64_t)((budget - fixed - spare) / row_bytes) : 0;
    if (fit < qc) qc = fit >= Q ? fit : (fit & ~(int64_t)127);
    if (qc < 1 || (qc < 128 && qc < Q)) {
      w.total = SIZE_MAX;
      return w;
    }
  }
  if (qc > Q) qc = Q;
  w.q_chunk = qc < 1 ? 1 : qc;
  size_t off = 0;
  w.coarse_dist = off; off += align256(coarse_scratch_floats(w.nlist_pad, nkeys, w.q_chunk) * 4);
  w.probe_ids = off;   off += align256((size_t)Q * nprobe * 4);
  w.probe_dist = off;  off += align256((size_t)Q * nprobe * 4);
  w.coarse_flags = off; off += align256((size_t)Q * 4);
  if (w.nsplit > 1) {
    w.part_d = off;    off += align256((size_t)Q * w.nsplit * 128 * 4);
    w.part_id = off;   off += align256((size_t)Q * w.nsplit * 128 * 8);
  }
  w.total = off;
  return w;
}

static std::atomic<int> g_wide_cap{8192};  // slots per query of the wide selection

void set_wide_cap(int v) { g_wide_cap.store(v, std::memory_order_relaxed); }

WideWorkspace plan_wide(const ivfpq_index *ix, int64_t Q, int32_t k, int32_t mode) {
  WideWorkspace w = {};
  if (ix->metric != IVFPQ_METRIC_L2 || mode != 0 || k <= 128 || k > 8 * 128 || Q < 1) return w;
  w.cap = g_wide_cap.load(std::memory_order_relaxed);
  if (w.cap == 0) return w;  // switched off: pass by pass
  // the slot arrays take at most 1 GiB: larger batches go through them in chunks
  int64_t qc = ((int64_t)1 << 30) / ((int64_t)w.cap * 12);
  if (qc < 1024) qc = 1024;
  w.q_chunk = qc < Q ? qc : Q;
  auto a256 = [](size_t v) { return (v + 255) & ~(size_t)255; };
  size_t off = 0;
  w.d = off;     off += a256((size_t)w.q_chunk * w.cap * 4);
  w.id = off;    off += a256((size_t)w.q_chunk * w.cap * 8);
  w.n = off;     off += a256((size_t)w.q_chunk * 4);
  w.bound = off; off += a256((size_t)w.q_chunk * 4);
  w.qmap = off;  off += a256((size_t)w.q_chunk * 4);
  w.total = off;
  return w;
}

static int check_common(const ivfpq_index *ix, const void *q, int64_t Q, int32_t nprobe, const char *fn) {
  if (!ix) { set_error("%s: index is NULL", fn); return IVFPQ_ERR_INVALID_ARGUMENT; }
  if (Q < 0) { set_error("%s: Q = %lld is negative", fn, (long long)Q); return IVFPQ_ERR_INVALID_ARGUMENT; }
  if (Q > 0 && !q) { set_error("%s: queries pointer is NULL", fn); return IVFPQ_ERR_INVALID_ARGUMENT; }
  if ((uintptr_t)q % 16) { set_error("%s: queries pointer must be 16-byte aligned", fn); return IVFPQ_ERR_INVALID_ARGUMENT; }
  if (Q > 0) {  // the index lives on one device; the kernels would fault on another one's pointers
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) (void)hipGetLastError();
    else if (dev != ix->device) {
      set_error("%s: the index was created on device %d, the current device is %d", fn, ix->device, dev);
      return IVFPQ_ERR_INVALID_ARGUMENT;
    }
  }
  if (nprobe < 1 || nprobe > ix->nlist) {
    set_error("%s: nprobe = %d outside [1, nlist = %d]", fn, nprobe, ix->nlist);
    return IVFPQ_ERR_INVALID_ARGUMENT;
  }
  if (nprobe > IVFPQ_MAX_NPROBE) {
    set_error("%s: nprobe = %d above the limit %d", fn, nprobe, IVFPQ_MAX_NPROBE);
    return IVFPQ_ERR_UNSUPPORTED;
  }
  return IVFPQ_OK;
}

static int check_k(int32_t k, const char *fn) {
  if (k < 1) { set_error("%s: k = %d must be positive", fn, k); return IVFPQ_ERR_INVALID_ARGUMENT; }
  if (k > IVFPQ_MAX_K) { set_error("%s: k = %d above the limit %d", fn, k, IVFPQ_MAX_K); return IVFPQ_ERR_UNSUPPORTED; }
  return IVFPQ_OK;
}

static int make_radii(const ivfpq_index *ix, const float *radii, RadiiSq *out, const char *fn) {
  if (!radii) { set_error("%s: radii pointer is NULL", fn); return IVFPQ_ERR_INVALID_ARGUMENT; }
  memset(out, 0, sizeof *out);
  for (int m = 0; m < ix->M; ++m) {
    const float r = radii[m];
    if (!(r >= 0.0f)) {  // catches NaN and negatives
      set_error("%s: radii[%d] = %g must be >= 0 (or +inf)", fn, m, (double)r);
      return IVFPQ_ERR_INVALID_ARGUMENT;
    }
    out->v[m] = r * r;  // fp32 product; +inf stays +inf
  }
  return IVFPQ_OK;
}

static int check_workspace(const Workspace &w, const void *ws, size_t bytes, const char *fn) {
  if (w.total == 0) return IVFPQ_OK;
  if (!ws) { set_error("%s: workspace pointer is NULL (%zu bytes needed)", fn, w.total); return IVFPQ_ERR_WORKSPACE; }
  if ((uintptr_t)ws % 256) { set_error("%s: workspace must be 256-byte aligned", fn); return IVFPQ_ERR_WORKSPACE; }
  if (bytes < w.total) { set_error("%s: workspace has %zu bytes, %zu needed", fn, bytes, w.total); return IVFPQ_ERR_WORKSPACE; }
  return IVFPQ_OK;
}

// Which way stages 2-4 run.  A request for the list-major scan is honoured where that scan is
// built (L2, k <= 128, the specialised shapes), anything else runs query-major.  Left to the
// library (AUTO), the list-major scan serves batches with enough (query, list) pairs to group,
// over indexes whose lists are short: there the per-query fixed costs of the query-major
// kernel dominate, while long lists (the 100M-point configuration) gain more from its
// per-block pruning.  Measured: faster on every 1M-point workload and on the 10M-point one,
// four times slower on the 100M-point one.
static bool use_list_major(const ivfpq_index *ix, int64_t Q, int32_t nprobe, int32_t k, int32_t mode,
                           int32_t requested) {
  if (requested == IVFPQ_SCAN_QUERY_MAJOR || !list_major_supported(ix, nprobe, k)) return false;
  if (requested == IVFPQ_SCAN_LIST_MAJOR) return true;
  (void)mode;
  return Q * (int64_t)nprobe >= 16384 && ix->N <= (int64_t)4096 * ix->nlist;
}

}  // namespace ivfpq

using namespace ivfpq;

extern "C" {

const char *ivfpq_last_error(void) { return g_err; }

int ivfpq_set_option(const char *name, int value) {
  if (name && !strcmp(name, "scan_waves")) {
    if (value != 0 && value != 4 && value != 8 && value != 16) {
      set_error("set_option: scan_waves must be 0, 4, 8 or 16");
      return IVFPQ_ERR_INVALID_ARGUMENT;
    }
    set_scan_waves(value);
    return IVFPQ_OK;
  }
  if (name && !strcmp(name, "scan_ablate")) {
    if (value & ~(8 | 16 | 32 | 64 | 128)) {
      set_error("set_option: scan_ablate accepts the bits 8, 16, 32, 64 and 128 only");
      return IVFPQ_ERR_INVALID_ARGUMENT;
    }
    set_scan_ablate(value);
    return IVFPQ_OK;
  }
  if (name && !strcmp(name, "scan_loads")) {
    if (value < 0 || value > 3) { set_error("set_option: scan_loads must be 0, 1, 2 or 3"); return IVFPQ_ERR_INVALID_ARGUMENT; }
    set_scan_variant(value);
    return IVFPQ_OK;
  }
  if (name && !strcmp(name, "lm_first")) {
    if (value < 1 || value > 64) { set_error("set_option: lm_first must be in [1, 64]"); return IVFPQ_ERR_INVALID_ARGUMENT; }
    set_lm_first(value);
    return IVFPQ_OK;
  }
  if (name && !strcmp(name, "lm_cap")) {
    if (value != 0 && (value < 64 || value > 65536)) { set_error("set_option: lm_cap must be 0 or in [64, 65536]"); return IVFPQ_ERR_INVALID_ARGUMENT; }
    set_lm_cap(value);
    return IVFPQ_OK;
  }
  if (name && !strcmp(name, "bound_grid")) {
    if (value < 0 || value > 2) { set_error("set_option: bound_grid must be 0, 1 or 2"); return IVFPQ_ERR_INVALID_ARGUMENT; }
    set_bound_grid(value);
    return IVFPQ_OK;
  }
  if (name && !strcmp(name, "wide_cap")) {
    if (value != 0 && (value < 1024 || value > 65536)) { set_error("set_option: wide_cap must be 0 or in [1024, 65536]"); return IVFPQ_ERR_INVALID_ARGUMENT; }
    set_wide_cap(value);
    return IVFPQ_OK;
  }
  set_error("set_option: unknown option");
  return IVFPQ_ERR_INVALID_ARGUMENT;
}

int64_t ivfpq_coarse_fallbacks(int reset) {
  unsigned int n = 0;
  const int rc = coarse_fallbacks(reset, &n);
  return rc == IVFPQ_OK ? (int64_t)n : (int64_t)rc;
}

void ivfpq_index_destroy(ivfpq_index *ix) {
  if (!ix) return;
  (void)hipFree(ix->d_centroids);
  (void)hipFree(ix->d_cnorm);
  (void)hipFree(ix->d_box);
  (void)hipFree(ix->d_grid);
  (void)hipFree(ix->d_grid_par);
  (void)hipFree(ix->d_codebooks);
  (void)hipFree(ix->d_list_offsets);
  (void)hipFree(ix->d_list_blocks);
  (void)hipFree(ix->d_codes);
  (void)hipFree(ix->d_ids);
  delete ix;
}

int ivfpq_index_create(const ivfpq_index_desc *d, ivfpq_index **out) {
  const char *fn = "index_create";
  if (!d || !out) { set_error("%s: NULL argument", fn); return IVFPQ_ERR_INVALID_ARGUMENT; }
  *out = nullptr;
  if (d->ksub != IVFPQ_KSUB) { set_error("%s: ksub = %d, only 256 is supported", fn, d->ksub); return IVFPQ_ERR_UNSUPPORTED; }
  if (d->N < 0 || d->D < 1 || d->nlist < 1 || d->M < 1) {
    set_error("%s: N, D, nlist, M must be positive (N may be 0)", fn);
    return IVFPQ_ERR_INVALID_ARGUMENT;
  }
  if (d->D % d->M) { set_error("%s: D = %d is not a multiple of M = %d", fn, d->D, d->M); return IVFPQ_ERR_INVALID_ARGUMENT; }
  if (d->metric != IVFPQ_METRIC_L2 && d->metric != IVFPQ_METRIC_IP) {
    set_error("%s: metric = %d unknown", fn, d->metric);
    return IVFPQ_ERR_INVALID_ARGUMENT;
  }
  if (d->M > IVFPQ_MAX_M) { set_error("%s: M = %d above the limit %d", fn, d->M, IVFPQ_MAX_M); return IVFPQ_ERR_UNSUPPORTED; }
  if (d->N >= ((int64_t)1 << 32)) { set_error("%s: N = %lld must be below 2^32", fn, (long long)d->N); return IVFPQ_ERR_UNSUPPORTED; }
  if (!d->centroids || !d->codebooks || !d->list_offsets || (d->N > 0 && !d->codes)) {
    set_error("%s: NULL array in the description", fn);
    return IVFPQ_ERR_INVALID_ARGUMENT;
  }
  // list offsets: host copy (works for host and device sources once a device exists;
  // a plain host pointer is read directly so that bad input is caught without a GPU)
  std::vector<int64_t> offs((size_t)d->nlist + 1);
  hipPointerAttribute_t attr;
  bool on_device = false;
  if (hipPointerGetAttributes(&attr, d->list_offsets) == hipSuccess)
    on_device = attr.type == hipMemoryTypeDevice;
  else
    (void)hipGetLastError();
  if (on_device) {
    IVFPQ_HIP_TRY(hipMemcpy(offs.data(), d->list_offsets, offs.size() * 8, hipMemcpyDeviceToHost));
  } else {
    memcpy(offs.data(), d->list_offsets, offs.size() * 8);
  }
  if (offs[0] != 0 || offs[d->nlist] != d->N) {
    set_error("%s: list_offsets must start at 0 and end at N", fn);
    return IVFPQ_ERR_INVALID_ARGUMENT;
  }
  std::vector<int64_t> blocks((size_t)d->nlist + 1);
  blocks[0] = 0;
  int64_t max_len = 0;
  for (int c = 0; c < d->nlist; ++c) {
    const int64_t len = offs[c + 1] - offs[c];
    if (len < 0) { set_error("%s: list_offsets decrease at list %d", fn, c); return IVFPQ_ERR_INVALID_ARGUMENT; }
    if (len > 0x7FFFFFC0ll) { set_error("%s: list %d longer than 2^31 points", fn, c); return IVFPQ_ERR_UNSUPPORTED; }
    if (len > max_len) max_len = len;
    blocks[c + 1] = blocks[c] + (len + 63) / 64;
  }

  ivfpq_index *ix = new (std::nothrow) ivfpq_index;
  if (!ix) { set_error("%s: out of host memory", fn); return IVFPQ_ERR_NO_MEMORY; }
  memset(ix, 0, sizeof *ix);
  ix->N = d->N; ix->D = d->D; ix->nlist = d->nlist; ix->M = d->M; ix->dsub = d->D / d->M;
  ix->metric = d->metric;
  ix->Mp = (d->M + 3) & ~3;
  ix->total_blocks = blocks[d->nlist];
  ix->code_bytes = ix->total_blocks * ivfpq_block_bytes(ix->Mp);
  ix->max_list_len = max_len;

  int rc = IVFPQ_OK;
  uint8_t *d_rows = nullptr;
  bool rows_owned = false;
  std::vector<float> cent_h, cnorm;
#define TRY_OR_FAIL(expr)                                   \
  do {                                                      \
    hipError_t _e = (expr);                                 \
    if (_e != hipSuccess) {                                 \
      rc = _e == hipErrorOutOfMemory ? IVFPQ_ERR_NO_MEMORY : IVFPQ_ERR_HIP; \
      set_error("%s: HIP error %d (%s) in %s", fn, (int)_e, hipGetErrorString(_e), #expr); \
      goto fail;                                            \
    }                                                       \
  } while (0)
  TRY_OR_FAIL(hipGetDevice(&ix->device));
  {
    const size_t cb = (size_t)d->nlist * d->D * 4, kb = (size_t)d->M * 256 * ix->dsub * 4;
    TRY_OR_FAIL(hipMalloc(&ix->d_centroids, cb));
    TRY_OR_FAIL(hipMalloc(&ix->d_cnorm, (size_t)d->nlist * 4));
    TRY_OR_FAIL(hipMalloc(&ix->d_codebooks, kb));
    TRY_OR_FAIL(hipMalloc(&ix->d_list_offsets, offs.size() * 8));
    TRY_OR_FAIL(hipMalloc(&ix->d_list_blocks, blocks.size() * 8));
    // padding behind the last list: for an empty list the scan reads (and ignores) one
    // 1 KiB chunk at the list's base
    TRY_OR_FAIL(hipMalloc(&ix->d_codes, (size_t)ix->code_bytes + 4096));
    TRY_OR_FAIL(hipMemset(ix->d_codes + ix->code_bytes, 0, 4096));
    TRY_OR_FAIL(hipMalloc(&ix->d_ids, d->N > 0 ? (size_t)d->N * 8 : 256));
    TRY_OR_FAIL(hipMemcpy(ix->d_centroids, d->centroids, cb, hipMemcpyDefault));
    TRY_OR_FAIL(hipMemcpy(ix->d_codebooks, d->codebooks, kb, hipMemcpyDefault));
    TRY_OR_FAIL(hipMemcpy(ix->d_list_offsets, offs.data(), offs.size() * 8, hipMemcpyHostToDevice));
    TRY_OR_FAIL(hipMemcpy(ix->d_list_blocks, blocks.data(), blocks.size() * 8, hipMemcpyHostToDevice));
    // squared centroid norms: only rank proposals in the filtering stage
    cent_h.resize((size_t)d->nlist * d->D);
    TRY_OR_FAIL(hipMemcpy(cent_h.data(), ix->d_centroids, cb, hipMemcpyDeviceToHost));
    cnorm.resize(d->nlist);
    float mx = 0.0f;
    for (int c = 0; c < d->nlist; ++c) {
      double s = 0.0;
      for (int i = 0; i < d->D; ++i) s += (double)cent_h[(size_t)c * d->D + i] * cent_h[(size_t)c * d->D + i];
      cnorm[c] = (float)s;
      if (cnorm[c] > mx) mx = cnorm[c];
    }
    ix->max_cnorm = mx;
    TRY_OR_FAIL(hipMemcpy(ix->d_cnorm, cnorm.data(), (size_t)d->nlist * 4, hipMemcpyHostToDevice));
    // per list and subspace, the bounding box of the entries the list's points use (filled
    // below from the codes; an empty list keeps the all-zero box)
    TRY_OR_FAIL(hipMalloc(&ix->d_box, (size_t)d->nlist * d->D * 2 * 4));
    TRY_OR_FAIL(hipMemset(ix->d_box, 0, (size_t)d->nlist * d->D * 2 * 4));
    // two-dimensional subspaces, L2: a grid per subspace with, for every cell, a lower bound on
    // the squared distance from any point of the cell to the nearest entry (the second
    // ingredient of the list-level bound, see probe_bound_kernel)
    if (ix->dsub == 2 && d->metric == IVFPQ_METRIC_L2) {
      TRY_OR_FAIL(hipMalloc(&ix->d_grid, (size_t)d->M * GRID_G * GRID_G * 4));
      TRY_OR_FAIL(hipMalloc(&ix->d_grid_par, (size_t)d->M * 8 * 4));
      rc = launch_codebook_grid(ix, nullptr);
      if (rc != IVFPQ_OK) goto fail;
      TRY_OR_FAIL(hipDeviceSynchronize());
    }
    if (d->N > 0) {
      bool codes_dev = false;
      if (hipPointerGetAttributes(&attr, d->codes) == hipSuccess) codes_dev = attr.type == hipMemoryTypeDevice;
      else (void)hipGetLastError();
      if (codes_dev) {
        d_rows = const_cast<uint8_t *>(d->codes);
      } else {
        TRY_OR_FAIL(hipMalloc(&d_rows, (size_t)d->N * d->M));
        rows_owned = true;
        TRY_OR_FAIL(hipMemcpy(d_rows, d->codes, (size_t)d->N * d->M, hipMemcpyHostToDevice));
      }
      rc = launch_relayout(ix, d_rows, nullptr);
      if (rc != IVFPQ_OK) goto fail;
      rc = launch_list_boxes(ix, d_rows, nullptr);
      if (rc != IVFPQ_OK) goto fail;
      if (d->ids) TRY_OR_FAIL(hipMemcpy(ix->d_ids, d->ids, (size_t)d->N * 8, hipMemcpyDefault));
      else {
        rc = launch_iota(ix->d_ids, d->N, nullptr);
        if (rc != IVFPQ_OK) goto fail;
      }
      TRY_OR_FAIL(hipDeviceSynchronize());
    }
  }
  if (rows_owned) (void)hipFree(d_rows);
  *out = ix;
  return IVFPQ_OK;
fail:
  if (rows_owned) (void)hipFree(d_rows);
  ivfpq_index_destroy(ix);
  return rc;
#undef TRY_OR_FAIL
}

int ivfpq_index_get_info(const ivfpq_index *ix, ivfpq_index_info *info) {
  if (!ix || !info) { set_error("index_get_info: NULL argument"); return IVFPQ_ERR_INVALID_ARGUMENT; }
  info->N = ix->N; info->D = ix->D; info->nlist = ix->nlist; info->M = ix->M; info->dsub = ix->dsub;
  info->code_bytes = ix->code_bytes; info->max_list_len = ix->max_list_len;
  info->metric = ix->metric;
  return IVFPQ_OK;
}

void ivfpq_radius_model_destroy(ivfpq_radius_model *md) {
  if (!md) return;
  (void)hipFree(md->d_block);
  delete md;
}

int ivfpq_radius_model_create(const ivfpq_index *ix, const ivfpq_radius_model_desc *d,
                              ivfpq_radius_model **out) {
  const char *fn = "radius_model_create";
  if (!ix || !d || !out) { set_error("%s: NULL argument", fn); return IVFPQ_ERR_INVALID_ARGUMENT; }
  *out = nullptr;
  if (!d->lo || !d->cells_per_unit || !d->map || !d->coef || !d->fallback) {
    set_error("%s: NULL array in the description", fn);
    return IVFPQ_ERR_INVALID_ARGUMENT;
  }
  if (d->M != ix->M) {
    set_error("%s: M = %d differs from the index's %d", fn, d->M, ix->M);
    return IVFPQ_ERR_INVALID_ARGUMENT;
  }
  if (ix->dsub != 2) {
    set_error("%s: the density map is two-dimensional; the index has dsub = %d", fn, ix->dsub);
    return IVFPQ_ERR_UNSUPPORTED;
  }
  if (d->grid < 1 || d->grid > 1024 || d->degree < 0 || d->degree > 8) {
    set_error("%s: grid = %d outside [1, 1024] or degree = %d outside [0, 8]", fn, d->grid, d->degree);
    return IVFPQ_ERR_INVALID_ARGUMENT;
  }
  const int M = d->M, G = d->grid, nc = d->degree + 1;
  for (int i = 0; i < 2 * M; ++i) {
    if (!isfinite(d->lo[i]) || !isfinite(d->cells_per_unit[i]) || !(d->cells_per_unit[i] > 0.0f)) {
      set_error("%s: lo / cells_per_unit of subspace %d not finite or not positive", fn, i / 2);
      return IVFPQ_ERR_INVALID_ARGUMENT;
    }
  }
  for (int m = 0; m < M; ++m) {
    if (!isfinite(d->fallback[m]) || d->fallback[m] < 0.0f) {
      set_error("%s: fallback[%d] must be finite and >= 0", fn, m);
      return IVFPQ_ERR_INVALID_ARGUMENT;
    }
  }
  ivfpq_radius_model *md = new (std::nothrow) ivfpq_radius_model;
  if (!md) { set_error("%s: out of host memory", fn); return IVFPQ_ERR_NO_MEMORY; }
  memset(md, 0, sizeof *md);
  md->M = M; md->grid = G; md->degree = d->degree;
  // lo | cells_per_unit | coef | fallback | map; every part starts on a multiple of 8 bytes
  const size_t n_lo = 2 * (size_t)M, n_coef = ((size_t)M * nc + 1) & ~(size_t)1, n_fb = ((size_t)M + 1) & ~(size_t)1;
  const size_t n_map = (size_t)M * G * G;
  std::vector<float> host(2 * n_lo + n_coef + n_fb + n_map, 0.0f);
  memcpy(host.data(), d->lo, n_lo * 4);
  memcpy(host.data() + n_lo, d->cells_per_unit, n_lo * 4);
  memcpy(host.data() + 2 * n_lo, d->coef, (size_t)M * nc * 4);
  memcpy(host.data() + 2 * n_lo + n_coef, d->fallback, (size_t)M * 4);
  memcpy(host.data() + 2 * n_lo + n_coef + n_fb, d->map, n_map * 4);
  hipError_t e = hipGetDevice(&md->device);
  if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&md->d_block), host.size() * 4);
  if (e == hipSuccess) e = hipMemcpy(md->d_block, host.data(), host.size() * 4, hipMemcpyHostToDevice);
  if (e != hipSuccess) {
    ivfpq_radius_model_destroy(md);
    if (e == hipErrorOutOfMemory) { set_error("%s: out of device memory", fn); return IVFPQ_ERR_NO_MEMORY; }
    return hip_fail(e, fn);
  }
  md->d_lo = md->d_block;
  md->d_cpu = md->d_lo + n_lo;
  md->d_coef = md->d_cpu + n_lo;
  md->d_fallback = md->d_coef + n_coef;
  md->d_map = md->d_fallback + n_fb;
  *out = md;
  return IVFPQ_OK;
}

int ivfpq_query_radii(const ivfpq_index *ix, const ivfpq_radius_model *md, const float *d_queries,
                      int64_t Q, const int32_t *d_probe_ids, int32_t nprobe, float scale,
                      float *d_radii, void *stream) {
  const char *fn = "query_radii";
  int rc = check_common(ix, d_queries, Q, nprobe, fn);
  if (rc) return rc;
  if (!md) { set_error("%s: model is NULL", fn); return IVFPQ_ERR_INVALID_ARGUMENT; }
  if (md->M != ix->M || ix->dsub != 2) {
    set_error("%s: the model was made for another index shape", fn);
    return IVFPQ_ERR_INVALID_ARGUMENT;
  }
  if (!isfinite(scale) || scale < 0.0f) {
    set_error("%s: scale must be finite and >= 0", fn);
    return IVFPQ_ERR_INVALID_ARGUMENT;
  }
  if (Q == 0) return IVFPQ_OK;
  if (!d_probe_ids || !d_radii) { set_error("%s: NULL pointer", fn); return IVFPQ_ERR_INVALID_ARGUMENT; }
  return launch_query_radii(ix, md, d_queries, Q, d_probe_ids, nprobe, scale, d_radii,
                            static_cast<hipStream_t>(stream));
}

size_t ivfpq_search_workspace_bytes(const ivfpq_index *ix, int64_t Q, int32_t nprobe, int32_t k) {
  return ivfpq_search_workspace_bytes_ex(ix, Q, nprobe, k, nullptr);
}

size_t ivfpq_search_workspace_bytes_ex(const ivfpq_index *ix, int64_t Q, int32_t nprobe, int32_t k,
                                       const ivfpq_scoring *sc) {
  if (!ix || Q < 0 || nprobe < 1 || nprobe > ix->nlist || k < 1) return 0;
  const Workspace w = plan_workspace(ix, Q, nprobe, k);
  size_t n = w.total;
  if (use_list_major(ix, Q, nprobe, k, sc ? sc->mode : IVFPQ_SCORE_DISTANCE, sc ? sc->strategy : IVFPQ_SCAN_AUTO))
    n = align256(w.total) + plan_list_major(ix, Q, nprobe).total;
  else if (const size_t wide = plan_wide(ix, Q, k, sc ? sc->mode : IVFPQ_SCORE_DISTANCE).total)
    n = align256(w.total) + wide;
  return n < 256 ? 256 : n;
}

int ivfpq_resolve_strategy(const ivfpq_index *ix, int64_t Q, int32_t nprobe, int32_t k, const ivfpq_scoring *sc) {
  if (!ix || Q < 0 || nprobe < 1 || nprobe > ix->nlist || k < 1) {
    set_error("resolve_strategy: invalid argument");
    return IVFPQ_ERR_INVALID_ARGUMENT;
  }
  if (sc && (sc->strategy < IVFPQ_SCAN_AUTO || sc->strategy > IVFPQ_SCAN_LIST_MAJOR)) {
    set_error("resolve_strategy: scan strategy %d unknown", sc->strategy);
    return IVFPQ_ERR_INVALID_ARGUMENT;
  }
  return use_list_major(ix, Q, nprobe, k, sc ? sc->mode : IVFPQ_SCORE_DISTANCE, sc ? sc->strategy : IVFPQ_SCAN_AUTO)
             ? IVFPQ_SCAN_LIST_MAJOR : IVFPQ_SCAN_QUERY_MAJOR;
}

int ivfpq_coarse(const ivfpq_index *ix, const float *d_queries, int64_t Q, int32_t nprobe,
                 int32_t *d_probe_ids, float *d_probe_dist, void *ws, size_t ws_bytes, void *stream) {
  const char *fn = "coarse";
  int rc = check_common(ix, d_queries, Q, nprobe, fn);
  if (rc) return rc;
  if (Q == 0) return IVFPQ_OK;
  if (!d_probe_ids) { set_error("%s: output pointer is NULL", fn); return IVFPQ_ERR_INVALID_ARGUMENT; }
  const Workspace w = plan_workspace(ix, Q, nprobe, 1);
  if ((rc = check_workspace(w, ws, ws_bytes, fn))) return rc;
  char *base = static_cast<char *>(ws);
  return launch_coarse(ix, d_queries, Q, nprobe, d_probe_ids, d_probe_dist,
                       reinterpret_cast<float *>(base + w.coarse_dist), w.q_chunk, w.nlist_pad,
                       reinterpret_cast<int32_t *>(base + w.coarse_flags), static_cast<hipStream_t>(stream));
}

// scoring defaults (distances, shared radii) when the caller passes none
static int unpack_scoring(const ivfpq_index *ix, const ivfpq_scoring *sc, const float *radii, RadiiSq *r2,
                          int32_t *mode, const float **d_query_radii, const char *fn,
                          int32_t *strategy = nullptr) {
  *mode = IVFPQ_SCORE_DISTANCE;
  *d_query_radii = nullptr;
  if (strategy) *strategy = IVFPQ_SCAN_AUTO;
  if (sc) {
    if (sc->mode < IVFPQ_SCORE_DISTANCE || sc->mode > IVFPQ_SCORE_HIT_REWARD) {
      set_error("%s: scoring mode %d unknown", fn, sc->mode);
      return IVFPQ_ERR_INVALID_ARGUMENT;
    }
    if (sc->strategy < IVFPQ_SCAN_AUTO || sc->strategy > IVFPQ_SCAN_LIST_MAJOR) {
      set_error("%s: scan strategy %d unknown", fn, sc->strategy);
      return IVFPQ_ERR_INVALID_ARGUMENT;
    }
    *mode = sc->mode;
    *d_query_radii = sc->d_query_radii;
    if (strategy) *strategy = sc->strategy;
  }
  if (*d_query_radii) {  // per-query radii replace the shared ones
    memset(r2, 0, sizeof *r2);
    return IVFPQ_OK;
  }
  return make_radii(ix, radii, r2, fn);
}

// Stages 2-4 query-major.  For k above 128 the slots of the wide selection lie behind the usual
// workspace; a workspace without room for them still serves the call, pass by pass.
static int scan_query_major(const ivfpq_index *ix, const float *d_queries, int64_t Q, int32_t nprobe,
                            const int32_t *d_probe_ids, int32_t k, const RadiiSq &r2, int32_t mode, const float *qr,
                            int64_t *d_out_ids, float *d_out_dist, const Workspace &w, char *base, size_t ws_bytes,
                            hipStream_t s) {
  const WideWorkspace ww = plan_wide(ix, Q, k, mode);
  ScanView view = {0, nullptr, false, nullptr, nullptr};
  if (ww.total > 0 && ws_bytes >= align256(w.total) + ww.total) {
    view.wide = &ww;
    view.wide_base = base + align256(w.total);
  }
  return launch_scan(ix, d_queries, Q, nprobe, d_probe_ids, k, r2, w.nsplit,
                     reinterpret_cast<uint32_t *>(base + w.part_d), reinterpret_cast<int64_t *>(base + w.part_id),
                     d_out_ids, d_out_dist, nullptr, nullptr, nullptr, nullptr, mode, qr,
                     reinterpret_cast<float *>(base + w.probe_dist), s, &view);
}

// Stages 2-4 list-major: the usual workspace, then the list-major part behind it.
static int scan_list_major(const ivfpq_index *ix, const float *d_queries, int64_t Q, int32_t nprobe,
                           const int32_t *d_probe_ids, int32_t k, const RadiiSq &r2, int32_t mode, const float *qr,
                           int64_t *d_out_ids, float *d_out_dist, const Workspace &w, void *ws, size_t ws_bytes,
                           hipStream_t s, const char *fn) {
  const LmWorkspace lw = plan_list_major(ix, Q, nprobe);
  Workspace both = w;
  both.total = align256(w.total) + lw.total;
  if (int rc = check_workspace(both, ws, ws_bytes, fn)) return rc;
  char *base = static_cast<char *>(ws);
  return launch_scan_list_major(ix, d_queries, Q, nprobe, d_probe_ids, k, r2, mode, qr,
                                reinterpret_cast<float *>(base + w.probe_dist), d_out_ids, d_out_dist, lw,
                                base + align256(w.total), s);
}

int ivfpq_build_lut_ex(const ivfpq_index *ix, const float *d_queries, int64_t Q, int32_t nprobe,
                       const int32_t *d_probe_ids, const float *radii, const ivfpq_scoring *scoring,
                       float *d_lut, uint64_t *d_mask, void *stream) {
  const char *fn = "build_lut";
  int rc = check_common(ix, d_queries, Q, nprobe, fn);
  if (rc) return rc;
  RadiiSq r2;
  int32_t mode;
  const float *qr;
  if ((rc = unpack_scoring(ix, scoring, radii, &r2, &mode, &qr, fn))) return rc;
  if (Q == 0) return IVFPQ_OK;
  if (!d_probe_ids || !d_lut) { set_error("%s: NULL pointer", fn); return IVFPQ_ERR_INVALID_ARGUMENT; }
  return launch_build_lut(ix, d_queries, Q, nprobe, d_probe_ids, r2, d_lut, d_mask, mode, qr,
                          static_cast<hipStream_t>(stream));
}

int ivfpq_build_lut(const ivfpq_index *ix, const float *d_queries, int64_t Q, int32_t nprobe,
                    const int32_t *d_probe_ids, const float *radii, float *d_lut, uint64_t *d_mask,
                    void *stream) {
  return ivfpq_build_lut_ex(ix, d_queries, Q, nprobe, d_probe_ids, radii, nullptr, d_lut, d_mask, stream);
}

int ivfpq_scan_topk_ex(const ivfpq_index *ix, const float *d_queries, int64_t Q, int32_t nprobe,
                       const int32_t *d_probe_ids, int32_t k, const float *radii,
                       const ivfpq_scoring *scoring, int64_t *d_out_ids, float *d_out_dist, void *ws,
                       size_t ws_bytes, void *stream) {
  const char *fn = "scan_topk";
  int rc = check_common(ix, d_queries, Q, nprobe, fn);
  if (rc) return rc;
  if ((rc = check_k(k, fn))) return rc;
  RadiiSq r2;
  int32_t mode, strategy;
  const float *qr;
  if ((rc = unpack_scoring(ix, scoring, radii, &r2, &mode, &qr, fn, &strategy))) return rc;
  if (Q == 0) return IVFPQ_OK;
  if (!d_probe_ids || !d_out_ids || !d_out_dist) { set_error("%s: NULL pointer", fn); return IVFPQ_ERR_INVALID_ARGUMENT; }
  const Workspace w = plan_workspace(ix, Q, nprobe, k);
  char *base = static_cast<char *>(ws);
  if (use_list_major(ix, Q, nprobe, k, mode, strategy))
    return scan_list_major(ix, d_queries, Q, nprobe, d_probe_ids, k, r2, mode, qr, d_out_ids, d_out_dist, w, ws,
                           ws_bytes, static_cast<hipStream_t>(stream), fn);
  if ((rc = check_workspace(w, ws, ws_bytes, fn))) return rc;
  return scan_query_major(ix, d_queries, Q, nprobe, d_probe_ids, k, r2, mode, qr, d_out_ids, d_out_dist, w, base,
                          ws_bytes, static_cast<hipStream_t>(stream));
}

int ivfpq_scan_topk(const ivfpq_index *ix, const float *d_queries, int64_t Q, int32_t nprobe,
                    const int32_t *d_probe_ids, int32_t k, const float *radii, int64_t *d_out_ids,
                    float *d_out_dist, void *ws, size_t ws_bytes, void *stream) {
  return ivfpq_scan_topk_ex(ix, d_queries, Q, nprobe, d_probe_ids, k, radii, nullptr, d_out_ids, d_out_dist,
                            ws, ws_bytes, stream);
}

// ---- the search that allocates nothing and takes no workspace -----------------------------
// Its workspace is this array: one copy per GPU, held from the moment the library is loaded
// on that GPU until the process ends.  The name is a host-side stand-in, not a device
// address: host code only ever uses the pointer that hipGetSymbolAddress returns for the
// current device (scratch_address), and the kernels receive that pointer as an argument,
// exactly as they receive a caller's workspace.
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[IVFPQ_NOALLOC_SCRATCH_BYTES];

static constexpr int MAX_DEVICES = 64;
static std::atomic<void *> g_scratch_ptr[MAX_DEVICES];

// Device address of `scratch` on the current device, looked up once per device.
static int scratch_address(void **out, const char *fn) {
  int dev = -1;
  IVFPQ_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= MAX_DEVICES) {
    set_error("%s: device ordinal %d outside [0, %d)", fn, dev, MAX_DEVICES);
    return IVFPQ_ERR_UNSUPPORTED;
  }
  void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    IVFPQ_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p || (uintptr_t)p % 256) {
      set_error("%s: the static scratch array has no usable device address", fn);
      return IVFPQ_ERR_HIP;
    }
    g_scratch_ptr[dev].store(p, std::memory_order_release);  // two threads racing here store the same address
  }
  *out = p;
  return IVFPQ_OK;
}

// Stages 1-4 with the workspace `base` carved as `w` says.
static int search_in_workspace(const ivfpq_index *ix, const float *d_queries, int64_t Q, int32_t nprobe,
                               int32_t k, const RadiiSq &r2, int32_t mode, const float *qr, int64_t *d_out_ids,
                               float *d_out_dist, const Workspace &w, char *base, size_t ws_bytes, hipStream_t s) {
  int32_t *probe_ids = reinterpret_cast<int32_t *>(base + w.probe_ids);
  int rc = launch_coarse(ix, d_queries, Q, nprobe, probe_ids, nullptr,
                         reinterpret_cast<float *>(base + w.coarse_dist), w.q_chunk, w.nlist_pad,
                         reinterpret_cast<int32_t *>(base + w.coarse_flags), s);
  if (rc) return rc;
  return scan_query_major(ix, d_queries, Q, nprobe, probe_ids, k, r2, mode, qr, d_out_ids, d_out_dist, w, base,
                          ws_bytes, s);
}

int ivfpq_search_noalloc(const ivfpq_index *ix, const float *d_queries, int64_t Q, int32_t nprobe, int32_t k,
                         const float *radii, int64_t *d_out_ids, float *d_out_dist, void *stream) {
  const char *fn = "search_noalloc";
  int rc = check_common(ix, d_queries, Q, nprobe, fn);
  if (rc) return rc;
  if ((rc = check_k(k, fn))) return rc;
  RadiiSq r2;
  if ((rc = make_radii(ix, radii, &r2, fn))) return rc;
  if (Q == 0) return IVFPQ_OK;
  if (!d_out_ids || !d_out_dist) { set_error("%s: NULL pointer", fn); return IVFPQ_ERR_INVALID_ARGUMENT; }
  const Workspace w = plan_workspace(ix, Q, nprobe, k, IVFPQ_NOALLOC_SCRATCH_BYTES);
  if (w.total == SIZE_MAX || w.total > IVFPQ_NOALLOC_SCRATCH_BYTES) {
    set_error("%s: Q = %lld, nprobe = %d with nlist = %d need more than the %u bytes of built-in scratch; "
              "use ivfpq_search with a workspace, or smaller batches", fn, (long long)Q, nprobe, ix->nlist,
              (unsigned)IVFPQ_NOALLOC_SCRATCH_BYTES);
    return IVFPQ_ERR_WORKSPACE;
  }
  void *base = nullptr;
  if ((rc = scratch_address(&base, fn))) return rc;
  // Nothing in the workspace has to start at zero: every region is written in full (for the
  // rows and probes of this call) before it is read, so the previous call's contents do not matter.
  return search_in_workspace(ix, d_queries, Q, nprobe, k, r2, IVFPQ_SCORE_DISTANCE, nullptr, d_out_ids,
                             d_out_dist, w, static_cast<char *>(base), IVFPQ_NOALLOC_SCRATCH_BYTES,
                             static_cast<hipStream_t>(stream));
}

int ivfpq_search_ex(const ivfpq_index *ix, const float *d_queries, int64_t Q, int32_t nprobe, int32_t k,
                    const float *radii, const ivfpq_scoring *scoring, int64_t *d_out_ids,
                    float *d_out_dist, void *ws, size_t ws_bytes, void *stream) {
  const char *fn = "search";
  int rc = check_common(ix, d_queries, Q, nprobe, fn);
  if (rc) return rc;
  if ((rc = check_k(k, fn))) return rc;
  RadiiSq r2;
  int32_t mode, strategy;
  const float *qr;
  if ((rc = unpack_scoring(ix, scoring, radii, &r2, &mode, &qr, fn, &strategy))) return rc;
  if (Q == 0) return IVFPQ_OK;
  if (!d_out_ids || !d_out_dist) { set_error("%s: NULL pointer", fn); return IVFPQ_ERR_INVALID_ARGUMENT; }
  const Workspace w = plan_workspace(ix, Q, nprobe, k);
  if (use_list_major(ix, Q, nprobe, k, mode, strategy)) {
    Workspace both = w;
    both.total = align256(w.total) + plan_list_major(ix, Q, nprobe).total;
    if ((rc = check_workspace(both, ws, ws_bytes, fn))) return rc;   // before anything is enqueued
    char *base = static_cast<char *>(ws);
    int32_t *probe_ids = reinterpret_cast<int32_t *>(base + w.probe_ids);
    rc = launch_coarse(ix, d_queries, Q, nprobe, probe_ids, nullptr, reinterpret_cast<float *>(base + w.coarse_dist),
                       w.q_chunk, w.nlist_pad, reinterpret_cast<int32_t *>(base + w.coarse_flags),
                       static_cast<hipStream_t>(stream));
    if (rc) return rc;
    return scan_list_major(ix, d_queries, Q, nprobe, probe_ids, k, r2, mode, qr, d_out_ids, d_out_dist, w, ws,
                           ws_bytes, static_cast<hipStream_t>(stream), fn);
  }
  if ((rc = check_workspace(w, ws, ws_bytes, fn))) return rc;
  return search_in_workspace(ix, d_queries, Q, nprobe, k, r2, mode, qr, d_out_ids, d_out_dist, w,
                             static_cast<char *>(ws), ws_bytes, static_cast<hipStream_t>(stream));
}

int ivfpq_search(const ivfpq_index *ix, const float *d_queries, int64_t Q, int32_t nprobe, int32_t k,
                 const float *radii, int64_t *d_out_ids, float *d_out_dist, void *ws, size_t ws_bytes,
                 void *stream) {
  return ivfpq_search_ex(ix, d_queries, Q, nprobe, k, radii, nullptr, d_out_ids, d_out_dist, ws, ws_bytes,
                         stream);
}

int ivfpq_scan_all_ex(const ivfpq_index *ix, const float *d_queries, int64_t Q, int32_t nprobe,
                      const int32_t *d_probe_ids, const float *radii, const ivfpq_scoring *scoring,
                      const int64_t *d_cand_offsets, float *d_all_dist, int64_t *d_all_ids,
                      int32_t *d_errors, void *stream) {
  const char *fn = "scan_all";
  int rc = check_common(ix, d_queries, Q, nprobe, fn);
  if (rc) return rc;
  RadiiSq r2;
  int32_t mode;
  const float *qr;
  if ((rc = unpack_scoring(ix, scoring, radii, &r2, &mode, &qr, fn))) return rc;
  if (!d_errors) { set_error("%s: NULL pointer", fn); return IVFPQ_ERR_INVALID_ARGUMENT; }
  if (Q > 0 && (!d_probe_ids || !d_cand_offsets || !d_all_dist || !d_all_ids)) {
    set_error("%s: NULL pointer", fn);
    return IVFPQ_ERR_INVALID_ARGUMENT;
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  rc = launch_fill_i32(d_errors, 1, 0, s);
  if (rc || Q == 0) return rc;
  // the dump variant of the scan kernel keeps no top-k, so k and the result pointers are unused
  return launch_scan(ix, d_queries, Q, nprobe, d_probe_ids, 0, r2, 1, nullptr, nullptr, nullptr, nullptr,
                     d_cand_offsets, d_all_dist, d_all_ids, d_errors, mode, qr, nullptr, s);
}

int ivfpq_scan_all(const ivfpq_index *ix, const float *d_queries, int64_t Q, int32_t nprobe,
                   const int32_t *d_probe_ids, const float *radii, const int64_t *d_cand_offsets,
                   float *d_all_dist, int64_t *d_all_ids, int32_t *d_errors, void *stream) {
  return ivfpq_scan_all_ex(ix, d_queries, Q, nprobe, d_probe_ids, radii, nullptr, d_cand_offsets, d_all_dist,
                           d_all_ids, d_errors, stream);
}

}  // extern "C"
