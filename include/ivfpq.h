/*
 * ivfpq.h -- C ABI of the MI355X (gfx950) search path of sparsity-aware IVF-PQ
 * (JUNO, arxiv 2312.01712).
 *
 * Notation.  The paper's Table 1 writes M for the subspace DIMENSION and D/M
 * for the number of subspaces.  This interface writes M for the NUMBER of
 * subspaces and dsub = D / M for their dimension; ksub (the paper's E) is fixed
 * at 256 so that a code is one byte; nlist is the paper's C, nprobe its nprobs.
 *
 * One query batch runs four stages (paper Sec. 2.1 "Online Search", Sec. 4.1,
 * Sec. 5.3):
 *   1. filtering: squared L2 distance from each query to the nlist IVF
 *      centroids, the nprobe nearest lists are probed;
 *   2. selective L2-LUT construction: for every probed list and subspace, a
 *      codebook entry is kept only if it lies within the subspace's radius of
 *      the query residual's projection; a kept entry stores its squared
 *      distance, any other entry stores the clamp r_m^2;
 *   3. distance calculation: the distance of an encoded point is the sum over
 *      subspaces of the table value of its code;
 *   4. top-k over all points of the probed lists, by (distance, id).
 *
 * Conventions for every call
 *   - "host" pointers are ordinary process memory, "device" pointers are HIP
 *     device memory on the current device, which must be the device the index
 *     was created on.  Nothing passed in is retained except by
 *     ivfpq_index_create, which copies what it needs.
 *   - d_queries must be 16-byte aligned (rows are read with vector loads); other
 *     device arrays need the natural alignment of their element type.
 *   - Search-side calls allocate nothing and never synchronise: they enqueue
 *     kernels on `hip_stream` (a hipStream_t, NULL = the default stream) and
 *     return.  Results are valid once the stream has reached that point.
 *   - Return value: IVFPQ_OK or a negative ivfpq_status.  On an argument error
 *     nothing is enqueued and no output is written.  ivfpq_last_error() gives a
 *     text for the last failure on the calling thread.
 *   - Limits: ksub == 256; D % M == 0; M <= 128; 1 <= k <= 1024;
 *     1 <= nprobe <= min(nlist, 1024); N < 2^32; radii finite >= 0 or +inf.
 *   - k > 128 (the paper's second quality metric retrieves 1000 neighbours,
 *     Sec. 6.1) is served 128 results at a time: ceil(k / 128) passes over the
 *     probed lists, each keeping the keys after the last (distance, id) of the
 *     pass before.  For that the ids of the index must be distinct and >= 0.
 *   - NaN in queries or in the index gives unspecified (but in-bounds) results.
 */
#ifndef IVFPQ_H
#define IVFPQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  IVFPQ_OK = 0,
  IVFPQ_ERR_INVALID_ARGUMENT = -1, /* null pointer, size out of range, bad offsets, bad radius */
  IVFPQ_ERR_UNSUPPORTED = -2,      /* a shape outside the stated limits                          */
  IVFPQ_ERR_WORKSPACE = -3,        /* workspace missing, misaligned or too small                 */
  IVFPQ_ERR_HIP = -4,              /* a HIP runtime call failed (text in ivfpq_last_error)       */
  IVFPQ_ERR_NO_MEMORY = -5         /* host or device allocation failed in index_create           */
} ivfpq_status;

#define IVFPQ_KSUB 256
#define IVFPQ_MAX_M 128
#define IVFPQ_MAX_K 1024
#define IVFPQ_MAX_NPROBE 1024

typedef struct ivfpq_index ivfpq_index; /* opaque; owns its device copies */

/* Similarity an index is searched by.
 *   IVFPQ_METRIC_L2  squared L2 distance (paper Sec. 2.1), everything above.
 *   IVFPQ_METRIC_IP  maximum inner product (paper Sec. 4.2, "Inner Product Similarity
 *     Support").  All results are NEGATED inner products, so that smaller is better and
 *     the (value, id) order of every output stays as for L2:
 *       lists      are ranked by -IP(q, centroid), acc = fmaf(q_i, c_i, acc), i ascending;
 *       the table  is one per QUERY (the paper's ray starts at the query's projection q_m,
 *                  not at a residual); entry e of subspace m is kept iff the ray hits its
 *                  enlarged sphere, |q_m - e|^2 <= r_m^2 + |e|^2, evaluated in the equivalent
 *                  form IP(e, q_m) >= thr_m = (|q_m|^2 - r_m^2) / 2; a kept entry stores
 *                  0 - IP(e, q_m), a missed one the bound 0 - thr_m that it cannot beat;
 *       a point    of list c scores -IP(q, centroid_c) plus the sum of its table values
 *                  (fp32, subspaces ascending), i.e. minus the inner product of the query
 *                  with the point's reconstruction when nothing is missed.
 *     With the hit-count scorings the table holds the same penalties as under L2 (inner
 *     sphere: the same construction with r_m / 2) and the list term is left out.
 *     ivfpq_build_lut returns the per-query table once per probe, [Q][nprobe][M][256]. */
typedef enum { IVFPQ_METRIC_L2 = 0, IVFPQ_METRIC_IP = 1 } ivfpq_metric;

/* A trained index as the offline phase leaves it (paper Sec. 2.1, Algorithm 1:
 * IVF centroids and labels, residual codebooks, encoded points).  All pointers
 * are caller-owned and read-only; they may be host or device pointers. */
typedef struct {
  int64_t N;                   /* number of encoded points                                  */
  int32_t D;                   /* vector dimension                                          */
  int32_t nlist;               /* number of inverted lists                                  */
  int32_t M;                   /* number of subspaces, D % M == 0                           */
  int32_t ksub;                /* entries per subspace, must be 256                         */
  const float *centroids;      /* [nlist][D] row-major                                      */
  const float *codebooks;      /* [M][256][dsub], trained on residuals                      */
  const int64_t *list_offsets; /* [nlist+1], non-decreasing, [0] = 0, [nlist] = N           */
  const uint8_t *codes;        /* [N][M]; rows list_offsets[c] .. list_offsets[c+1] are list c */
  const int64_t *ids;          /* [N] result ids in the same row order; NULL = row number   */
  int32_t metric;              /* an ivfpq_metric                                           */
} ivfpq_index_desc;

/* Copies the index to the current device, re-laid out for the scan (codes in
 * blocks of 64 points, interleaved so that one wavefront load is contiguous).
 * Synchronous; allocates device memory that *out owns until destroy. */
int ivfpq_index_create(const ivfpq_index_desc *desc, ivfpq_index **out);
void ivfpq_index_destroy(ivfpq_index *index);

/* Bytes of device workspace the search-side calls need for a batch of Q
 * queries (0 on invalid arguments), with the scan strategy left to the library.
 * The workspace must be 256-byte aligned.  For 128 < k <= 1024 with L2 distances
 * the figure includes the per-query slots ("wide_cap" below, 12 bytes each, for
 * at most 1 GiB at a time) that let one pass over the lists produce all k
 * neighbours; a workspace sized for k = 128 is accepted too, and the call then
 * takes ceil(k / 128) passes.  Results are the same either way. */
size_t ivfpq_search_workspace_bytes(const ivfpq_index *index, int64_t Q, int32_t nprobe, int32_t k);

/* The whole search path (stages 1-4) for a batch.
 *   d_queries   device [Q][D] fp32 row-major
 *   radii       host   [M] fp32, per-subspace radius r_m shared by the batch
 *               (paper Sec. 4.1: user-set threshold); +inf keeps every entry
 *   d_out_ids   device [Q][k] int64, ascending by (distance, id); -1 when the
 *               probed lists hold fewer than k points
 *   d_out_dist  device [Q][k] fp32, +inf where the id is -1
 *   d_workspace device, at least ivfpq_search_workspace_bytes(...) bytes
 * Q == 0 is a no-op. */
int ivfpq_search(const ivfpq_index *index, const float *d_queries, int64_t Q, int32_t nprobe,
                 int32_t k, const float *radii, int64_t *d_out_ids, float *d_out_dist,
                 void *d_workspace, size_t workspace_bytes, void *hip_stream);

/* The whole search path for callers that cannot allocate and have no workspace to pass:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same stages, same results and same argument conventions as ivfpq_search (distance
 * scoring, shared radii), with the workspace in a static device array inside the library:
 * IVFPQ_NOALLOC_SCRATCH_BYTES per GPU, held from library load to process end.  The call
 * allocates nothing (no hipMalloc / hipFree, no allocating library routine), takes no
 * workspace and never synchronises.
 *   Limit: the batch's workspace must fit the array.  The filtering stage works through the
 *   batch in chunks of at least 128 queries x nlist floats, so roughly
 *   8 Q nprobe + 128 * 4 nlist bytes (+ 3 KiB per query when Q < 2048) must stay under the
 *   array's size: e.g. Q = 10 000 with nprobe = 64 and nlist = 16 384, or nlist up to about
 *   60 000 for small batches.  Beyond it the call returns IVFPQ_ERR_WORKSPACE with a text that
 *   says so, and writes nothing.
 *   Every call on a GPU uses that GPU's one array: calls that overlap in time on the same
 *   GPU (two streams, two host threads) race on it and give wrong results; serialise them
 *   or use ivfpq_search with separate workspaces.  Nothing in the array has to be cleared
 *   between calls (every region is written before it is read). */
#define IVFPQ_NOALLOC_SCRATCH_BYTES (32u << 20)
int ivfpq_search_noalloc(const ivfpq_index *index, const float *d_queries, int64_t Q, int32_t nprobe,
                         int32_t k, const float *radii, int64_t *d_out_ids, float *d_out_dist,
                         void *hip_stream);

/* Stage 1 alone (paper Sec. 2.1 step A; Sec. 5.3 on computing it as a matrix
 * product): d_probe_ids device [Q][nprobe] int32 ordered by (distance, list
 * id); d_probe_dist device [Q][nprobe] fp32 or NULL.  Distances are
 * sum_i fmaf(t_i, t_i, .) with t_i = q_i - c_i, i ascending. */
int ivfpq_coarse(const ivfpq_index *index, const float *d_queries, int64_t Q, int32_t nprobe,
                 int32_t *d_probe_ids, float *d_probe_dist, void *d_workspace,
                 size_t workspace_bytes, void *hip_stream);

/* Stage 2 alone (paper Sec. 4.1; Algorithm 2), materialised for inspection:
 * d_lut device [Q][nprobe][M][256] fp32; d_mask device [Q][nprobe][M][4]
 * uint64 (bit e%64 of word e/64 set when entry e is kept) or NULL. */
int ivfpq_build_lut(const ivfpq_index *index, const float *d_queries, int64_t Q, int32_t nprobe,
                    const int32_t *d_probe_ids, const float *radii, float *d_lut,
                    uint64_t *d_mask, void *hip_stream);

/* Stages 2-4 for given probe lists (device [Q][nprobe] int32, every id in
 * [0, nlist)).  Same outputs as ivfpq_search. */
int ivfpq_scan_topk(const ivfpq_index *index, const float *d_queries, int64_t Q, int32_t nprobe,
                    const int32_t *d_probe_ids, int32_t k, const float *radii, int64_t *d_out_ids,
                    float *d_out_dist, void *d_workspace, size_t workspace_bytes,
                    void *hip_stream);

/* Stages 2-3 with every candidate's distance written out (paper Sec. 5.3: the
 * list of search points and distances handed to top-k).  d_cand_offsets device
 * [Q+1] int64: query q's candidates occupy [off[q], off[q+1]) in probe order
 * then list order, so off[q+1]-off[q] must equal the summed sizes of its probed
 * lists (checked on the device: a mismatching query is skipped and counted in
 * *d_errors, device int32, which the call first sets to 0).  Meant for small
 * inputs. */
int ivfpq_scan_all(const ivfpq_index *index, const float *d_queries, int64_t Q, int32_t nprobe,
                   const int32_t *d_probe_ids, const float *radii, const int64_t *d_cand_offsets,
                   float *d_all_dist, int64_t *d_all_ids, int32_t *d_errors, void *hip_stream);

/* ---- scoring variants --------------------------------------------------------
 * The calls above rank by distances with one radius per subspace for the whole
 * batch (the paper's JUNO-H).  The *_ex calls take an ivfpq_scoring that selects
 *   - per-query radii (paper Sec. 4.1 "Determining Proper Threshold": a threshold
 *     specific to the query, times a user scale): d_query_radii, device [Q][M] fp32,
 *     each >= 0 or +inf (not validated: a NaN radius keeps no entry and yields NaN
 *     sums); when it is non-NULL the host `radii` argument is ignored and may be NULL;
 *   - hit-count scoring (paper Sec. 5.4), expressed as a penalty that is summed and
 *     ranked exactly like a distance, smaller is better:
 *       IVFPQ_SCORE_HIT_COUNT   an entry inside the radius stores 0, any other 1,
 *                               so the result is M - (number of subspaces hit)
 *                               (the paper's JUNO-L);
 *       IVFPQ_SCORE_HIT_REWARD  with the inner sphere of half the radius: 0 inside it
 *                               (the paper's +1), 1 inside the outer sphere only (0),
 *                               2 outside both (-1), so the result is M - score
 *                               (the paper's JUNO-M).
 *     The returned "distances" are these sums (small integers held in fp32); ties are
 *     frequent and go to the smaller id.  Keep masks are those of the outer radius.
 * scoring == NULL means distances and shared radii, i.e. the plain call. */
typedef enum {
  IVFPQ_SCORE_DISTANCE = 0,
  IVFPQ_SCORE_HIT_COUNT = 1,
  IVFPQ_SCORE_HIT_REWARD = 2
} ivfpq_score_mode;

/* How stages 2-4 walk the (query, probed list) pairs.  Results do not depend on it.
 *   IVFPQ_SCAN_QUERY_MAJOR  one workgroup per query scans the query's lists nearest first and
 *     prunes against its running k-th distance (per list, per block of 64 points, per partial
 *     sum).  Best on long lists.
 *   IVFPQ_SCAN_LIST_MAJOR   the CDNA4 counterpart of the paper's entry -> points map
 *     (Sec. 5.2, Algorithm 1; Sec. 5.3): the queries that selected a list are served together,
 *     two per pass over the list's codes, with their tables interleaved so that one look-up
 *     serves both.  The nearest list of every query is ranked first (its k-th distance is the
 *     bound that filters the query's other lists).  Best where the per-query fixed costs or
 *     the look-up rate dominate: short lists, data without cluster structure.
 *     Needs the L2 metric, k <= 128 and an (M, dsub) of (48, 2), (64, 2) or (16, 4); any other
 *     call is served query-major.  Takes a larger workspace.
 *   IVFPQ_SCAN_AUTO         the library chooses: list-major where it is available, when the
 *     batch has at least 16 384 (query, list) pairs and the index's mean list length is at
 *     most 4096; query-major otherwise.
 * ivfpq_search_workspace_bytes sizes the workspace for AUTO with distance scoring;
 * ivfpq_search_workspace_bytes_ex for the scoring actually passed. */
typedef enum { IVFPQ_SCAN_AUTO = 0, IVFPQ_SCAN_QUERY_MAJOR = 1, IVFPQ_SCAN_LIST_MAJOR = 2 } ivfpq_scan_strategy;

typedef struct {
  int32_t mode;               /* an ivfpq_score_mode                              */
  const float *d_query_radii; /* device [Q][M], or NULL for the shared host radii */
  int32_t strategy;           /* an ivfpq_scan_strategy                            */
} ivfpq_scoring;

/* Workspace bytes for the *_ex calls with this scoring (the strategy decides). */
size_t ivfpq_search_workspace_bytes_ex(const ivfpq_index *index, int64_t Q, int32_t nprobe, int32_t k,
                                       const ivfpq_scoring *scoring);

/* The strategy such a call will run with: IVFPQ_SCAN_QUERY_MAJOR or IVFPQ_SCAN_LIST_MAJOR
 * (scoring NULL: AUTO, distance scoring); a negative ivfpq_status on invalid arguments. */
int ivfpq_resolve_strategy(const ivfpq_index *index, int64_t Q, int32_t nprobe, int32_t k,
                           const ivfpq_scoring *scoring);

int ivfpq_search_ex(const ivfpq_index *index, const float *d_queries, int64_t Q, int32_t nprobe,
                    int32_t k, const float *radii, const ivfpq_scoring *scoring, int64_t *d_out_ids,
                    float *d_out_dist, void *d_workspace, size_t workspace_bytes, void *hip_stream);
int ivfpq_build_lut_ex(const ivfpq_index *index, const float *d_queries, int64_t Q, int32_t nprobe,
                       const int32_t *d_probe_ids, const float *radii, const ivfpq_scoring *scoring,
                       float *d_lut, uint64_t *d_mask, void *hip_stream);
int ivfpq_scan_topk_ex(const ivfpq_index *index, const float *d_queries, int64_t Q, int32_t nprobe,
                       const int32_t *d_probe_ids, int32_t k, const float *radii,
                       const ivfpq_scoring *scoring, int64_t *d_out_ids, float *d_out_dist,
                       void *d_workspace, size_t workspace_bytes, void *hip_stream);
int ivfpq_scan_all_ex(const ivfpq_index *index, const float *d_queries, int64_t Q, int32_t nprobe,
                      const int32_t *d_probe_ids, const float *radii, const ivfpq_scoring *scoring,
                      const int64_t *d_cand_offsets, float *d_all_dist, int64_t *d_all_ids,
                      int32_t *d_errors, void *hip_stream);

/* ---- dynamic thresholds ------------------------------------------------------
 * Paper Sec. 4.1 "Determining Proper Threshold" and the threshold step of
 * Algorithm 2: offline, every two-dimensional subspace is cut into a grid x grid
 * map (the paper uses 100 x 100) that records the density of search point
 * projections per cell, and a polynomial is fitted from that density to the
 * threshold a projection needs; online, the value at the query's projection is
 * looked up, the polynomial evaluated and the result multiplied by the user's
 * scale.  Here: one threshold per (query, subspace), looked up at the projection
 * of the residual of the query w.r.t. its NEAREST list (the space the entries and
 * the encoded points live in); the result is the d_query_radii array of
 * ivfpq_scoring.  The map and the polynomial are inputs (the offline fit is not
 * part of the search path). */
typedef struct {
  int32_t M;                   /* number of subspaces; must equal the index's, with dsub == 2   */
  int32_t grid;                /* cells per axis, 1 .. 1024                                      */
  int32_t degree;              /* degree of the polynomial, 0 .. 8                               */
  const float *lo;             /* host [M][2]  low corner of the map                             */
  const float *cells_per_unit; /* host [M][2]  1 / cell width along each axis, finite and > 0    */
  const float *map;            /* host [M][grid][grid]  the polynomial's input per cell (the
                                  density or a fixed transform of it); cell (i0, i1), i0 from the
                                  subspace's first coordinate, at i0 * grid + i1                 */
  const float *coef;           /* host [M][degree + 1]  lowest power first                       */
  const float *fallback;       /* host [M]  radius used where the polynomial gives no positive
                                  finite value                                                   */
} ivfpq_radius_model_desc;

typedef struct ivfpq_radius_model ivfpq_radius_model; /* opaque; owns its device copy */

/* Copies the model to the current device.  Synchronous; allocates. */
int ivfpq_radius_model_create(const ivfpq_index *index, const ivfpq_radius_model_desc *desc,
                              ivfpq_radius_model **out);
void ivfpq_radius_model_destroy(ivfpq_radius_model *model);

/* d_radii[q][m] for a batch, all in fp32, with c = d_probe_ids[q * nprobe] (the first
 * entry of a row of ivfpq_coarse's output: the nearest list):
 *   x_j  = q[2m + j] - centroid_c[2m + j],                       j = 0, 1
 *   i_j  = floor((x_j - lo[m][j]) * cells_per_unit[m][j]) clamped to [0, grid - 1]
 *          (NaN goes to cell 0)
 *   f    = map[m][i_0][i_1]
 *   p    = coef[m][degree];  p = fmaf(p, f, coef[m][d]) for d = degree - 1 .. 0
 *   d_radii[q][m] = (0 < p < inf ? p : fallback[m]) * scale
 * d_queries device [Q][D]; d_probe_ids device [Q][nprobe] int32 with ids in [0, nlist)
 * (a row whose first id is outside gets the fallback); d_radii device [Q][M] fp32.
 * scale must be finite and >= 0.  Enqueues one kernel; allocates nothing. */
int ivfpq_query_radii(const ivfpq_index *index, const ivfpq_radius_model *model,
                      const float *d_queries, int64_t Q, const int32_t *d_probe_ids, int32_t nprobe,
                      float scale, float *d_radii, void *hip_stream);

/* Shape of an index and of its device layout. */
typedef struct {
  int64_t N;
  int32_t D, nlist, M, dsub;
  int64_t code_bytes;   /* bytes of the interleaved code array on the device   */
  int64_t max_list_len; /* longest inverted list                                */
  int32_t metric;       /* the ivfpq_metric it was created with                 */
} ivfpq_index_info;
int ivfpq_index_get_info(const ivfpq_index *index, ivfpq_index_info *info);

/* Diagnostic: number of queries, on the current device since the last reset, whose
 * probe lists were not accepted from the matrix-product proposal and were instead
 * computed from reference-order distances to every centroid (the result is the
 * same either way; the count says how often the slower path ran).  Synchronises
 * the device.  Negative: an ivfpq_status. */
int64_t ivfpq_coarse_fallbacks(int reset);

/* Tuning switches, process-wide.  None of them changes a result; each takes effect for the
 * calls that start after it returns and may be set from any thread.  Unknown names and values
 * outside the stated sets give IVFPQ_ERR_INVALID_ARGUMENT.
 *   "scan_waves"   wavefronts per workgroup of the fused scan kernel: 0 (default: chosen from
 *                  the shape), 4, 8 or 16.
 *   "scan_loads"   how the scan kernel fetches code blocks: 0 (default) the first chunk (16
 *                  subspaces) of a block ahead and the rest only when the block needs it, whole
 *                  blocks once pruning has been switched off for a query; 1 always whole blocks;
 *                  2 / 3 always the first half / the first chunk ahead.
 *   "lm_first"     list-major scan: probed lists per query that are ranked first (1 .. 64,
 *                  default 1); their k-th distance is the bound that filters the other lists.
 *                  1: the nearest list is ranked list-major as well (queries that share it
 *                  share its pass); more: those lists are scanned query-major.
 *   "lm_cap"       list-major scan: candidate slots per query (64 .. 65536; default 0: 256 per
 *                  probed list, at least 4096 and at most 16384; 8 bytes of workspace per
 *                  slot); a query that overflows them is redone query-major.  Set both
 *                  before sizing the workspace.
 *   "wide_cap"     128 < k <= 1024: slots per query for the keys within the running bound on the
 *                  k-th distance (1024 .. 65536, default 8192).  Between lists the bound, which
 *                  only tightens, clears the slots it has overtaken; a query that still runs
 *                  out of slots is redone pass by pass.  0: no slots, every query pass by
 *                  pass (128 neighbours per pass).  Set before sizing the workspace.
 *   "scan_ablate"  bit mask that switches exact pruning off, to measure what it saves: 8 the
 *                  early exit of the distance sums, 16 all of the per-block pruning from the
 *                  first list on (no row minima, no checks: what the kernel otherwise switches
 *                  to by itself for queries whose blocks rarely end early), 32 that switch,
 *                  64 the list-level bound that skips a list before its table is built.
 *                  8 | 16 | 64 with "scan_loads" 1 is the plain scan: every code byte of every
 *                  probed list is read and looked up.  128: the hit-count scorings use the
 *                  float table of the distance scoring instead of their byte table.
 *   "bound_grid"   the list-level bound (two-dimensional subspaces, L2) can add, to the per-list
 *                  boxes, a per-subspace grid of distances to the nearest codebook entry: 0
 *                  (default) on indexes with more than 4096 points per list, where a list that
 *                  slips through the bound costs most; 1 always; 2 never. */
int ivfpq_set_option(const char *name, int value);

/* Text for the most recent failure on this thread ("" if none). */
const char *ivfpq_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* IVFPQ_H */
