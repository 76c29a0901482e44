// Internal declarations shared by the translation units of the HIP library.
// Not part of the public interface (see include/ivfpq.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ivfpq.h"

// Device-side image of an index.
struct ivfpq_index {
  int64_t N;
  int32_t D, nlist, M, dsub;
  int32_t metric;           // IVFPQ_METRIC_L2 or IVFPQ_METRIC_IP
  int32_t Mp;               // code bytes per point in the device layout, M rounded up to 4
  int device;
  float *d_centroids;       // [nlist][D]
  float *d_cnorm;           // [nlist] squared norms (only used to propose probe lists)
  float *d_box;             // [nlist][M][2][dsub] per list and subspace: bounding box (low corner, high corner) of the entries its points use
  float *d_grid;            // dsub == 2, L2 metric: [M][GRID_G * GRID_G] lower bound on the squared distance from any point of a grid cell to the subspace's nearest entry; else NULL
  float *d_grid_par;        // [M][8]: low corner (x, y), high corner (x, y), cells per unit (x, y), 0, 0
  float *d_codebooks;       // [M][256][dsub]
  int64_t *d_list_offsets;  // [nlist+1] in points
  int64_t *d_list_blocks;   // [nlist+1] in 64-point blocks of the interleaved layout
  uint8_t *d_codes;         // interleaved blocks, see layout note below
  int64_t *d_ids;           // [N]
  int64_t code_bytes;
  int64_t total_blocks;
  int64_t max_list_len;
  float max_cnorm;
};

// Device-side image of a threshold model (ivfpq_radius_model_desc); one allocation.
struct ivfpq_radius_model {
  int32_t M, grid, degree;
  int device;
  float *d_block;     // the allocation: lo | cells_per_unit | coef | fallback | map
  float *d_lo;        // [M][2]
  float *d_cpu;       // [M][2]
  float *d_coef;      // [M][degree+1]
  float *d_fallback;  // [M]
  float *d_map;       // [M][grid][grid]
};

// Device layout of the codes.  Every inverted list is padded to a multiple of 64
// points (nb blocks) and occupies nb*64*Mp bytes, stored chunk-major: a point's Mp
// code bytes are cut into Mp/16 chunks of 16 bytes followed by (Mp%16)/4 chunks of
// 4 bytes; chunk j of the whole list comes first for j = 0, then j = 1, ...:
// [chunk][block][lane][16 B], then [chunk][block][lane][4 B].  A wavefront that
// assigns lane l to point l of a block reads 1 KiB (or 256 B) contiguous per load
// instruction, consecutive blocks of one chunk are contiguous, and the later
// chunks of blocks that are abandoned early are never touched.  Padding bytes and
// padding points are 0; 4 KiB of zero padding follow the last list.
__host__ __device__ inline int64_t ivfpq_block_bytes(int Mp) { return (int64_t)64 * Mp; }

// r_m^2 for every subspace, passed to kernels by value (kernel-argument
// segment), so that a search needs no device copy of the radii.
struct RadiiSq {
  float v[IVFPQ_MAX_M];
};

namespace ivfpq {

void set_error(const char *fmt, ...);
int hip_fail(hipError_t e, const char *what);

#define IVFPQ_HIP_TRY(expr)                              \
  do {                                                   \
    hipError_t _e = (expr);                              \
    if (_e != hipSuccess) return ivfpq::hip_fail(_e, #expr); \
  } while (0)

// ---- filtering stage with many lists ---------------------------------------------------------
// There the matrix product does not write its rows: per query and group of 64 lists it keeps
// the COARSE_FT smallest values as keys (coarse_gemm_top_kernel).  Keys per query, or 0 where
// rows are written (few lists: a group would hold several of a query's nearest lists, and the
// bound on what it left out would reject the proposal).
constexpr int COARSE_FT = 6;
inline int32_t coarse_fused_keys(int32_t nlist, int32_t nprobe, int32_t D) {
  int slack = nprobe / 4;
  if (slack < 16) slack = 16;
  const int64_t kprop = (int64_t)nprobe + slack;
  const int64_t groups = 2 * (((int64_t)nlist + 127) / 128);
  const int64_t keys = groups * COARSE_FT;
  if (kprop > 128 || keys > 16384 || groups < 3 * kprop || D > 2048) return 0;
  return (int32_t)keys;
}
// Floats of scratch the filtering stage takes for a chunk of qc queries: rows of the product,
// or keys, then reference-order rows for the queries that need every distance (one per 16
// queries and FB_SLOTS more), then the list of the first FB_SLOTS such queries.
constexpr int FB_SLOTS = 64;
inline size_t coarse_scratch_floats(int32_t nlist_pad, int32_t nkeys, int64_t qc) {
  if (nkeys <= 0) return (size_t)qc * nlist_pad;
  return (((size_t)qc * nkeys + 63) & ~(size_t)63) + (size_t)((qc + 15) / 16 + FB_SLOTS) * nlist_pad + FB_SLOTS + 64;
}

// ---- workspace carving (all offsets 256-byte aligned) -----------------------
struct Workspace {
  size_t coarse_dist;   // scratch of the filtering stage for one query chunk (coarse_scratch_floats)
  size_t probe_ids;     // [Q][nprobe] int32
  size_t probe_dist;    // [Q][nprobe] fp32: list-level lower bounds for the scan
  size_t coarse_flags;  // [Q] int32: queries the one-wavefront selection of the filtering stage leaves to the workgroup one
  size_t part_d;        // [Q][nsplit][128] uint32 (only when nsplit > 1)
  size_t part_id;       // [Q][nsplit][128] int64
  size_t total;
  int64_t q_chunk;      // queries per coarse chunk
  int32_t nlist_pad;    // row stride of coarse_dist
  int32_t nsplit;       // probe groups per query in the scan
};
Workspace plan_workspace(const ivfpq_index *ix, int64_t Q, int32_t nprobe, int32_t k, size_t budget = 0);

// ---- launchers (enqueue only) -------------------------------------------------
int launch_coarse(const ivfpq_index *ix, const float *d_queries, int64_t Q, int32_t nprobe,
                  int32_t *d_probe_ids, float *d_probe_dist, float *d_scratch, int64_t q_chunk,
                  int32_t nlist_pad, int32_t *d_flags, hipStream_t s);
int launch_build_lut(const ivfpq_index *ix, const float *d_queries, int64_t Q, int32_t nprobe,
                     const int32_t *d_probe_ids, const RadiiSq &r2, float *d_lut, uint64_t *d_mask,
                     int32_t mode, const float *d_query_radii, hipStream_t s);
// Workspace of the wide selection (more than 128 neighbours per query in one pass of the
// query-major scan): offsets into its part of the workspace, 256-byte aligned.
struct WideWorkspace {
  size_t d, id;      // [q_chunk][cap] distance keys / rows within the bound
  size_t n, bound;   // [q_chunk] slots in use (-1: overflow) / final bound
  size_t qmap;       // [q_chunk] int32: 0 for the queries left to the pass-by-pass path, else -1
  size_t total;      // 0: the wide selection does not apply
  int64_t q_chunk;   // queries that share the slot arrays at a time
  int32_t cap;       // slots per query
};
// total == 0 unless the wide selection serves this call (L2 distances, 128 < k <= 1024).
WideWorkspace plan_wide(const ivfpq_index *ix, int64_t Q, int32_t k, int32_t mode);
void set_wide_cap(int v);  // slots per query of the wide selection (1024 .. 65536)

// Which part of the probe table a scan launch covers, and for which queries (NULL: all of it).
struct ScanView {
  int32_t probe_stride;  // row stride of d_probe_ids / d_probe_lb when only the first nprobe of a longer row are scanned (0: nprobe)
  const int32_t *qmap;   // device [Q] or NULL: queries with a negative entry are left out
  bool bounds_ready;     // d_probe_lb already holds the list-level bounds of every row
  const WideWorkspace *wide;  // NULL: k above 128 is produced pass by pass
  char *wide_base;            // device base of the wide selection's part of the workspace
};
int launch_scan(const ivfpq_index *ix, const float *d_queries, int64_t Q, int32_t nprobe,
                const int32_t *d_probe_ids, int32_t k, const RadiiSq &r2, int32_t nsplit,
                uint32_t *d_part_d, int64_t *d_part_id, int64_t *d_out_ids, float *d_out_dist,
                const int64_t *d_cand_offsets, float *d_all_dist, int64_t *d_all_ids,
                int32_t *d_errors, int32_t mode, const float *d_query_radii, float *d_probe_lb,
                hipStream_t s, const ScanView *view = nullptr);
int launch_probe_bounds(const ivfpq_index *ix, const float *d_queries, int64_t Q, int32_t nprobe,
                        const int32_t *d_probe_ids, const RadiiSq &r2, int32_t mode, const float *d_query_radii,
                        float *d_probe_lb, hipStream_t s, int32_t *d_zero = nullptr, int64_t zero_n = 0);
// ---- list-major batched scan (scan_lm.hip) --------------------------------------------------
struct LmWorkspace {      // offsets into the list-major part of the workspace, 256-byte aligned
  size_t cnt, base;       // [nlist], [nlist+1] int32
  size_t pairs;           // [pairs_cap] (query, list) int32 pairs bucketed by list
  size_t rank;            // [pairs_cap] int32: a pair's position among the pairs of its list
  size_t gcnt, qmap;      // [Q] uint32 / int32
  size_t qmap_head;       // [Q] int32
  size_t cand;            // [Q][cap] (distance bits, row) candidates of the list-major scan
  size_t total;
  int64_t pairs_cap;
  int32_t first;          // probed lists per query that are scanned query-major first
  int32_t cap;            // candidate slots per query
};
bool list_major_supported(const ivfpq_index *ix, int32_t nprobe, int32_t k);
LmWorkspace plan_list_major(const ivfpq_index *ix, int64_t Q, int32_t nprobe);
int launch_scan_list_major(const ivfpq_index *ix, const float *d_queries, int64_t Q, int32_t nprobe,
                           const int32_t *d_probe_ids, int32_t k, const RadiiSq &r2, int32_t mode,
                           const float *d_query_radii, float *d_probe_lb, int64_t *d_out_ids, float *d_out_dist,
                           const LmWorkspace &w, char *lm_base, hipStream_t s);
void set_lm_first(int v);  // lists per query scanned query-major before the list-major scan (1 .. 64)
void set_lm_cap(int v);    // candidate slots per query of the list-major scan (64 .. 65536; 0: by the number of probes)
int get_scan_ablate();

int launch_query_radii(const ivfpq_index *ix, const ivfpq_radius_model *md, const float *d_queries,
                       int64_t Q, const int32_t *d_probe_ids, int32_t nprobe, float scale,
                       float *d_radii, hipStream_t s);
int launch_relayout(const ivfpq_index *ix, const uint8_t *d_rows, hipStream_t s);
int launch_list_boxes(const ivfpq_index *ix, const uint8_t *d_rows, hipStream_t s);
constexpr int GRID_G = 64;   // cells per side of the per-subspace grid of nearest-entry bounds
int launch_codebook_grid(const ivfpq_index *ix, hipStream_t s);
int launch_iota(int64_t *d, int64_t n, hipStream_t s);
int coarse_fallbacks(int reset, unsigned int *out);
int launch_fill_i32(int32_t *d, int64_t n, int32_t v, hipStream_t s);
void set_scan_ablate(int bits);   // pruning switches 8 | 32 | 64 (results unchanged)
void set_scan_variant(int v);     // code loads: 0 adaptive, 1 whole blocks, 2 first half + rest on demand
void set_scan_waves(int nw);  // wavefronts per scan workgroup: 0 (auto), 4, 8 or 16
void set_bound_grid(int v);   // nearest-entry grid in the list-level bound: 0 (long lists only), 1 always, 2 never

}  // namespace ivfpq
