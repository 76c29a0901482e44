// List-major batched scan: the queries that probe the same inverted list are served
// together, two at a time, from ONE pass over the list's codes.
//
// Paper Sec. 5.2 / Algorithm 1 builds an inverted entry -> points map per list so that the
// distance calculation (Sec. 5.3) touches a list's points once per hit entry.  On CDNA4 the
// dense code stream is the better carrier, and what the map buys -- work shared inside a list
// -- is had by turning the loop nest around: the outer loop runs over lists, the queries that
// selected a list (Sec. 2.1 step A) are grouped, and the group shares the list's code stream
// and ONE table look-up per (point, subspace): the tables of the two queries of a group are
// interleaved entry by entry, so a single 8-byte LDS read returns both queries' values for a
// point's code.  The LDS gather rate, which bounds the query-major scan on data where
// nothing can be pruned, is per lane-address and not per byte, so two queries cost what one
// did.  Sums keep the subspace order of the plain loop: results are bit for bit those of the
// query-major scan.
//
// A query's lists are now scanned by different workgroups at different times, so the running
// k-th distance is not at hand.  Instead:
//   A  the query-major kernel scans the first few probed lists of every query (the nearest
//      ones) and leaves each query's top-k of those; tau_q = its k-th distance bounds the
//      final k-th distance from above;
//   B  (query, list) pairs of the remaining probes whose list-level lower bound exceeds tau_q
//      are dropped; the others are bucketed by list (count, offsets, fill);
//   C  the list-major scan appends every point with distance <= tau_q to the query's
//      candidate buffer (a few hundred per query: anything above tau_q cannot be in the
//      result);
//   D  one wavefront per query merges its buffer into the top-k of phase A by (distance, id).
// A query whose buffer overflows is redone by the query-major kernel, so the result is
// always that of the plain loop.

#include "scan_device.h"

namespace {

constexpr int LM_G = 2;        // queries per group (interleaved tables, 8-byte look-ups)
constexpr int LM_NW = 8;       // wavefronts per workgroup: one workgroup per CU (the table fills most of its LDS), 2 per SIMD, 256 registers each
constexpr int LM_QUEUE = 64;   // accepted candidates a wavefront holds per query before it appends them
constexpr int LM_SEL_WORDS = 16;     // head pass: small LDS block of selection state
constexpr int LM_BINS = 1024;        // head pass: bins of the selection histogram
constexpr int LM_COLLECT = 128;      // head pass: candidates a query may collect (the sorted list of a wavefront)

typedef float floatx2 __attribute__((ext_vector_type(2)));

struct LmArgs {
  const float *queries;         // [Q][D]
  const int32_t *probe_ids;     // [Q][nprobe]
  const float *probe_lb;        // [Q][nprobe] list-level lower bounds, or NULL
  const float *centroids;       // [nlist][D]
  const float *codebooks;       // [M][256][dsub]
  const int64_t *list_offsets;  // [nlist+1]
  const int64_t *list_blocks;   // [nlist+1]
  const uint8_t *codes;         // interleaved blocks
  const int64_t *ids;           // [N]
  int64_t *out_ids;             // [Q][k]: phase A's top-k on entry to the merge, the result after it
  float *out_dist;              // [Q][k]
  int32_t *cnt;                 // [nlist] pairs per list
  int32_t *rank;                // [max(Q, Q*(nprobe-first))] position of a pair among its list's pairs, -1: no pair
  int32_t *base;                // [nlist+1] first pair slot of a list (ranges padded to LM_G); [nlist] = slots in use
  int2 *pairs;                  // [Q*(nprobe-first) + nlist] (query, list); query -1 pads a list's range
  uint32_t *gcnt;               // [Q] candidates appended (may run past cap: the query then counts as overflowed)
  uint2 *cand;                  // [Q][cap] (distance bits, row in the index)
  int32_t *qmap;                // [Q] out: q for a query to be redone query-major, -1 otherwise
  int32_t *qmap_head;           // [Q] head pass: q for a query whose nearest list is left to the query-major kernel, else -1
  int32_t head_max;             // head pass: longest list (points) whose distances fit the workgroup's LDS
  const float *query_radii;     // [Q][M] or NULL
  int64_t Q;
  int32_t D, M, dsub, Mp, nlist, nprobe, first, k, cap, mode;
  int32_t head_done;            // the head pass has run: queries it left out (qmap_head) have no first-list result yet
};

// One thread per (query, probe >= first).  fill == 0: count the surviving pairs of every list
// (and clear the query's candidate count); the value the count returns is the pair's position
// among its list's pairs and is kept (rank, -1 for a pair that takes no part), so that
// fill == 1 only has to write the pair to that position of the list's slot range: no second
// evaluation of the predicate and no second atomic operation on the per-list words.
// head == 1 (the head pass): one thread per query, the pair is (query, its nearest list); a
// query whose nearest list is missing, empty or too long for the head pass is handed to the
// query-major kernel through qmap_head instead.
__global__ __launch_bounds__(256) void lm_pairs_kernel(LmArgs a, int fill, int head) {
  const int np2 = head ? 1 : a.nprobe - a.first;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= a.Q * np2) return;
  const int64_t q = idx / np2;
  const int p = head ? 0 : a.first + (int)(idx % np2);
  const int32_t c = a.probe_ids[q * a.nprobe + p];
  if (fill) {
    const int32_t r = a.rank[idx];
    if (r >= 0) a.pairs[a.base[c] + r] = make_int2((int)q, c);
    return;
  }
  if (!head && p == a.first) a.gcnt[q] = 0u;
  bool take = true;
  // a query the head pass left out has no bound yet: it takes no part here and is redone
  // query-major over all of its lists (lm_merge_kernel puts it on that list)
  if (!head && a.head_done && a.qmap_head[q] >= 0) take = false;
  const bool exists = (uint32_t)c < (uint32_t)a.nlist;
  const int64_t len = exists ? a.list_offsets[c + 1] - a.list_offsets[c] : 0;
  if (head) {
    const bool ok = len > 0 && len <= a.head_max;
    a.qmap_head[q] = ok ? -1 : (int32_t)q;
    take = ok;
  }
  if (len <= 0) take = false;
  if (take && !head && a.probe_lb) {
    // no point of the list can reach the k-th distance that phase A already guarantees
    const float tau = a.out_dist[q * a.k + a.k - 1];
    if (a.probe_lb[q * a.nprobe + p] > tau) take = false;
  }
  a.rank[idx] = take ? atomicAdd(&a.cnt[c], 1) : -1;
}

// Slot ranges of the lists: base[c] = sum over c' < c of cnt[c'] rounded up to LM_G.  The
// padding slot of an odd range is marked (query -1), the counts are cleared.
// One workgroup.
__global__ __launch_bounds__(1024) void lm_offsets_kernel(LmArgs a) {
  __shared__ int part[1024];
  const int tid = threadIdx.x;
  const int chunk = (a.nlist + 1023) / 1024;
  const int lo = tid * chunk < a.nlist ? tid * chunk : a.nlist;
  const int hi = lo + chunk < a.nlist ? lo + chunk : a.nlist;
  int sum = 0;
  for (int c = lo; c < hi; ++c) sum += (a.cnt[c] + LM_G - 1) / LM_G * LM_G;
  part[tid] = sum;
  __syncthreads();
  for (int off = 1; off < 1024; off <<= 1) {
    const int v = tid >= off ? part[tid - off] : 0;
    __syncthreads();
    part[tid] += v;
    __syncthreads();
  }
  int run = part[tid] - sum;
  for (int c = lo; c < hi; ++c) {
    const int n = a.cnt[c], padded = (n + LM_G - 1) / LM_G * LM_G;
    a.base[c] = run;
    for (int j = n; j < padded; ++j) a.pairs[run + j] = make_int2(-1, c);
    run += padded;
    a.cnt[c] = 0;   // left clear for the next pass over this workspace
  }
  if (tid == 1023) a.base[a.nlist] = part[1023];
}

// 8-byte look-up of a point's code in an interleaved table row (2 KiB per row): the byte
// select of the sub-dword addressing form extracts the code and scales it by 8.
__device__ __forceinline__ uint32_t code_offset8(uint32_t w, int j) {
  uint32_t a;
  const uint32_t three = 3u;
  switch (j) {
    case 0: asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_0" : "=v"(a) : "s"(three), "v"(w)); break;
    case 1: asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_1" : "=v"(a) : "s"(three), "v"(w)); break;
    case 2: asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_2" : "=v"(a) : "s"(three), "v"(w)); break;
    default: asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_3" : "=v"(a) : "s"(three), "v"(w)); break;
  }
  return a;
}

// d0 += table value of query 0, d1 += that of query 1, for subspaces [h, h1) in subspace order;
// the look-ups of a group are issued together and added afterwards (see lookup_group).
template <int MT>
__device__ __forceinline__ void lookup_group2(const CodeRegs<((MT + 3) / 4 * 4) / 4> &r, int h, int h1, float &d0,
                                              float &d1) {
  floatx2 t[LOOKUP_GROUP];
#pragma unroll
  for (int j = 0; j < LOOKUP_GROUP; ++j) {
    const int m = h + j;
    if (m < h1) {
      // the table starts at LDS address 0 (no static LDS: checked when the kernel is prepared)
      const uint32_t off = code_offset8(r.w[m >> 2], m & 3);
      t[j] = *(const LDS floatx2 *)(uintptr_t)(uint32_t)(m * 2048 + off);
    }
  }
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int j = 0; j < LOOKUP_GROUP; ++j)
    if (h + j < h1) {
      d0 += t[j][0];
      d1 += t[j][1];
    }
  __builtin_amdgcn_sched_barrier(0);
}

// Append a wavefront's queued candidates of one query to the query's buffer: `slot` is where
// the buffer's counter stood when the wavefront reserved its n entries.
__device__ __forceinline__ void lm_store(const LmArgs &a, int64_t q, uint32_t slot, LDS uint32_t *qd,
                                         LDS uint32_t *qrow, int n, int lane) {
  // past the capacity nothing is stored; the counter has grown all the same, which marks the
  // query as overflowed
  if (slot + (uint32_t)n <= (uint32_t)a.cap && lane < n)
    a.cand[q * a.cap + slot + lane] = make_uint2(qd[lane], qrow[lane]);
}

__device__ __forceinline__ void lm_flush(const LmArgs &a, int64_t q, LDS uint32_t *qd, LDS uint32_t *qrow, int n,
                                         int lane) {
  uint32_t slot = 0;
  if (lane == 0) slot = atomicAdd(&a.gcnt[q], (uint32_t)n);
  slot = (uint32_t)__builtin_amdgcn_readfirstlane((int)slot);
  lm_store(a, q, slot, qd, qrow, n, lane);
}

// Offer a block's distances for one query: every valid point with distance <= tau is queued.
__device__ __forceinline__ void lm_offer(const LmArgs &a, int64_t q, float dist, bool valid, uint32_t tau,
                                         uint32_t row, LDS uint32_t *qd, LDS uint32_t *qrow, int &qcount, int lane) {
  const uint32_t bits = __float_as_uint(dist);
  const bool pass = valid && bits <= tau;
  const unsigned long long bal = __ballot(pass);
  if (bal == 0) return;
  const int n = __popcll(bal);
  if (qcount + n > LM_QUEUE) {
    lm_flush(a, q, qd, qrow, qcount, lane);
    qcount = 0;
  }
  if (pass) {
    const int slot = qcount + __popcll(bal & ((1ull << lane) - 1ull));
    qd[slot] = bits;
    qrow[slot] = row;
  }
  qcount += n;
}

// ---- head pass: exact top-k of ONE list per query, without a bound to filter by ----------
// The nearest list of a query has to be ranked in full.  Its distances (bit patterns of
// non-negative floats, which order like the values) are kept in LDS; a histogram of 1024 bins
// of equal width finds the bin of the k-th smallest, everything up to that bin is collected (k keys plus the few that share the last bin) and one wavefront per query
// sorts the collected keys by (distance, id).  More than LM_COLLECT collected keys (masses of
// equal distances) hand the query to the query-major kernel.

// bin b of a histogram lives at word (b % 16) * 64 + b / 16, so that lane l, which owns the 16
// consecutive bins 16 l .. 16 l + 15, reads them without bank conflicts
__device__ __forceinline__ uint32_t lds_add(LDS uint32_t *p) {   // LDS atomic increment, returns the old value
  return __hip_atomic_fetch_add(p, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}
constexpr int LM_BPL = LM_BINS / 64;   // bins per lane
__device__ __forceinline__ int lm_hidx(uint32_t bin) { return (int)(((bin % LM_BPL) << 6) | (bin / LM_BPL)); }

// One wavefront: the bin that holds the need-th smallest key (need >= 1, at most the number
// of keys counted) and the number of keys in the bins below it.
__device__ inline void lm_find_bin(const LDS uint32_t *hist, uint32_t need, int lane, uint32_t &bin, uint32_t &below) {
  uint32_t sum = 0;
  for (int j = 0; j < LM_BPL; ++j) sum += hist[j * 64 + lane];
  uint32_t incl = sum;
  for (int off = 1; off < 64; off <<= 1) {
    const uint32_t v = (uint32_t)__shfl_up((int)incl, off);
    if (lane >= off) incl += v;
  }
  const uint32_t excl = incl - sum;
  const bool mine = excl < need && need <= incl;   // exactly one lane
  uint32_t b = 0, bl = 0, run = excl;
  if (mine) {
    for (int j = 0; j < LM_BPL; ++j) {
      const uint32_t c = hist[j * 64 + lane];
      if (run < need && need <= run + c) {
        b = (uint32_t)LM_BPL * lane + j;
        bl = run;
      }
      run += c;
    }
  }
  const unsigned long long bal = __ballot(mine);
  const int src = bal ? __ffsll((long long)bal) - 1 : 0;
  bin = (uint32_t)__shfl((int)b, src);
  below = (uint32_t)__shfl((int)bl, src);
}

// One task: a list and the (up to) LM_G queries of a group that probe it.
struct LmTask {
  int32_t c;
  int64_t q0, q1;      // q1 == q0 when the group is half empty (has1 false): its copy is dropped
  bool has1;
  int64_t row0;
  int32_t len, nb;
  const uint8_t *base;
  float tauv;          // main pass: lane 0 holds tau of q0, the other lanes tau of q1 (a vector load, like the metadata)
};

// Persistent workgroups, one per CU.  Tasks are sorted by list; in every round the grid takes
// the next gridDim.x tasks, and within a round the workgroups of one XCD (workgroup b runs on
// XCD b % 8) take a run of consecutive tasks, so that the tasks which stream the same list's
// codes share an L2.  Everything a task needs from global memory -- its pair entries, the
// list's metadata, the two query rows, the centroid, the first code block -- is requested
// while the task before it is still being scanned, so that a workgroup (the only one on its
// CU: the interleaved table fills most of the LDS) does not sit idle through a chain of
// dependent loads at every task boundary.
// HEAD: the head pass -- a task's list is the nearest list of its queries; no bound exists yet,
// every distance is kept (in LDS) and the exact top-k of the list is selected per query and
// written to the query's output row, where the main pass and the merge find it.
template <int MT, int DSUB, bool HEAD>
__global__ __launch_bounds__(LM_NW * 64) __attribute__((amdgpu_waves_per_eu(LM_NW / 4))) void lm_scan_kernel(LmArgs a, RadiiSq r2) {
  constexpr int NW = LM_NW;
  constexpr int MPT = (MT + 3) / 4 * 4;
  constexpr int ITER = (MT + NW - 1) / NW;
  constexpr int NCH = MPT / 16 + (MPT % 16) / 4;
  extern __shared__ __align__(16) unsigned char smem[];
  LDS unsigned char *smem3 = (LDS unsigned char *)smem;
  const int D = a.D;   // LM_G * D <= NT and LM_G * MT <= NT: one element per thread (checked by the launcher)
  const int dpad = (D + 3) & ~3;
  // LDS carve: interleaved table [MT][256][2] | residuals [2][dpad] | r_m^2 [2][MAX_M] | queues
  LDS float *lut = (LDS float *)smem3;
  LDS float *sres = (LDS float *)(smem3 + MT * 2048);
  LDS float *sr2 = sres + LM_G * dpad;
  LDS uint32_t *queue = (LDS uint32_t *)(sr2 + LM_G * IVFPQ_MAX_M);  // main pass: [NW][G][2][LM_QUEUE]
  // head pass: selection state, the histograms, then the distances [2][head_max]; the
  // collected keys use the table's LDS once the list has been scanned
  LDS uint32_t *ssel = queue;                      // [LM_SEL_WORDS]
  LDS uint32_t *hist = queue + LM_SEL_WORDS;       // [2][LM_BINS]
  LDS uint32_t *sdist = hist + LM_G * LM_BINS;     // [2][head_max]
  LDS uint32_t *coll_d = (LDS uint32_t *)smem3;    // [2][LM_COLLECT] collected keys: distance bits ...
  LDS uint32_t *coll_pos = coll_d + LM_G * LM_COLLECT;    // ... their positions in the list ...
  LDS uint32_t *coll_rank = coll_pos + LM_G * LM_COLLECT;  // ... and in sorted order

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  LDS uint32_t *qd0 = queue + (wave * LM_G + 0) * 2 * LM_QUEUE, *qrow0 = qd0 + LM_QUEUE;
  LDS uint32_t *qd1 = queue + (wave * LM_G + 1) * 2 * LM_QUEUE, *qrow1 = qd1 + LM_QUEUE;

  // this wavefront's codebook rows (rows wave, wave + NW, ...) stay in registers for the whole
  // kernel; the head pass at 64 subspaces has registers for three of its eight rows and fetches
  // the others (from the L2) when a task's table is built (four and five resident rows spill 2
  // and 6 registers; the batch takes the same time with 3 and 4)
  constexpr int RES = (HEAD && ITER > 6) ? 3 : ITER;
  float4 cbr[RES][DSUB];
  auto load_row = [&](int it, float4 (&row)[DSUB]) __attribute__((always_inline)) {
    const int m = wave + it * NW;
    const int mc = m < MT ? m : MT - 1;
    const uint8_t *cb = uniform_ptr(reinterpret_cast<const uint8_t *>(a.codebooks + (int64_t)mc * 256 * DSUB));
#pragma unroll
    for (int x = 0; x < DSUB; ++x)
      row[x] = *reinterpret_cast<const float4 *>(cb + (uint32_t)(lane * 16 * DSUB + 16 * x));
  };
#pragma unroll
  for (int it = 0; it < RES; ++it) load_row(it, cbr[it]);

  const int ntasks = a.base[a.nlist] / LM_G;
  const int nwg = gridDim.x, b = blockIdx.x;
  const int in_round = (nwg & 7) == 0 ? (b & 7) * (nwg >> 3) + (b >> 3) : b;

  // what this thread contributes to a task's residuals and radii: element tid of [2][D] / [2][MT]
  const int rg = tid >= D ? 1 : 0, rd = tid - rg * D;
  const bool r_on = tid < LM_G * D;
  const int mg = tid >= MT ? 1 : 0, mm = tid - mg * MT;
  const bool m_on = tid < LM_G * MT;

  // A task's pair entries and its list's metadata are requested with VECTOR loads (a lane each:
  // even lanes the first pair entry, odd lanes the second; lanes 0 and 1 the list's row range,
  // the others its first block), although every lane of the wavefront wants the same values:
  // scalar loads share their counter with the LDS, so a scalar load in flight makes the next
  // LDS read of the scan wait for it, whereas vector loads complete in order behind the code
  // stream and cost nothing when they are consumed a scan later.
  auto fetch_pairs = [&](int t) __attribute__((always_inline)) { return a.pairs[(int64_t)t * LM_G + (lane & 1)]; };
  auto fetch_meta = [&](const int2 &pv) __attribute__((always_inline)) {
    const int c = __builtin_amdgcn_readlane(pv.y, 0);
    const int64_t *src = lane < 2 ? a.list_offsets + c + lane : a.list_blocks + c;
    return *src;
  };
  auto lane64 = [&](int64_t v, int l) __attribute__((always_inline)) {
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, l);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)((uint64_t)v >> 32), l);
    return (int64_t)(((uint64_t)hi << 32) | lo);
  };
  // everything else a task needs, requested together: bounds, this thread's residual and radius
  // element, the wavefront's first code block
  auto fetch_task = [&](const int2 &pv, int64_t mv, LmTask &tk, float &qv, float &cv, float &rv,
                        CodeRegs<MPT / 4> &first) __attribute__((always_inline)) {
    tk.c = __builtin_amdgcn_readlane(pv.y, 0);
    tk.q0 = __builtin_amdgcn_readlane(pv.x, 0);
    tk.has1 = __builtin_amdgcn_readlane(pv.x, 1) >= 0;
    tk.q1 = tk.has1 ? __builtin_amdgcn_readlane(pv.x, 1) : tk.q0;
    tk.row0 = lane64(mv, 0);
    tk.len = (int)(lane64(mv, 1) - tk.row0);
    tk.nb = (tk.len + 63) >> 6;
    tk.base = a.codes + lane64(mv, 2) * ivfpq_block_bytes(MPT);
    tk.tauv = 0.0f;
    if constexpr (!HEAD) tk.tauv = a.out_dist[(lane == 0 ? tk.q0 : tk.q1) * a.k + a.k - 1];
    qv = cv = 0.0f;
    if (r_on) {
      qv = a.queries[(rg ? tk.q1 : tk.q0) * D + rd];
      cv = a.centroids[(int64_t)tk.c * D + rd];
    }
    rv = 0.0f;
    if (m_on) {
      rv = r2.v[mm];
      if (a.query_radii) {
        const float r = a.query_radii[(mg ? tk.q1 : tk.q0) * MT + mm];
        rv = r * r;
      }
    }
    const int b0 = wave < tk.nb ? wave : tk.nb - 1;   // nb >= 1: only non-empty lists have tasks
    load_chunks<MPT, 0, NCH>(tk.base, tk.nb, b0, lane, first);
  };

  LmTask tk;
  float qv, cv, rv;
  CodeRegs<MPT / 4> nxt;
  int t = in_round;
  if (t >= ntasks) return;
  int2 npv = make_int2(0, 0);   // pair entries of the next task
  {
    const int2 pv = fetch_pairs(t);
    if (t + nwg < ntasks) npv = fetch_pairs(t + nwg);
    fetch_task(pv, fetch_meta(pv), tk, qv, cv, rv, nxt);
  }
  // main pass: the candidates of the task before, queued in LDS, and where they go
  uint32_t pend_slot = 0;
  int64_t pend_q0 = 0, pend_q1 = 0;
  int pend_c0 = 0, pend_c1 = 0;
  auto drain_pending = [&]() __attribute__((always_inline)) {
    const uint32_t s0 = (uint32_t)__builtin_amdgcn_readlane((int)pend_slot, 0);
    const uint32_t s1 = (uint32_t)__builtin_amdgcn_readlane((int)pend_slot, 1);
    if (pend_c0 > 0) lm_store(a, pend_q0, s0, qd0, qrow0, pend_c0, lane);
    if (pend_c1 > 0) lm_store(a, pend_q1, s1, qd1, qrow1, pend_c1, lane);
    pend_c0 = pend_c1 = 0;
  };
  for (;;) {
    if (r_on) sres[rg * dpad + rd] = qv - cv;
    if (m_on) sr2[mg * IVFPQ_MAX_M + mm] = rv;
    if (HEAD && tid < LM_SEL_WORDS)   // [0..1] keys collected, [2..3] bin of the k-th key, [4..5] smallest key, [6..7] largest key
      ssel[tid] = (tid == 4 || tid == 5) ? 0xFFFFFFFFu : 0u;
    if constexpr (HEAD)
      for (int i = tid; i < LM_G * LM_BINS; i += NW * 64) hist[i] = 0u;
    __syncthreads();
    // ---- the two tables, interleaved: row m holds (query 0, query 1) of entry 0, of entry 1, ... ----
    auto build_rows = [&](auto mode_tag) __attribute__((always_inline)) {
      constexpr int MODE = decltype(mode_tag)::value;
      float4 cbs[ITER > RES ? ITER - RES : 1][DSUB];   // streamed rows, requested together
#pragma unroll
      for (int it = RES; it < ITER; ++it) load_row(it, cbs[it - RES]);
#pragma unroll
      for (int it = 0; it < ITER; ++it) {
        const int m = wave + it * NW;
        if (m < MT) {
          const float4 *row = it < RES ? cbr[it < RES ? it : 0] : cbs[it >= RES ? it - RES : 0];
          float res0[DSUB], res1[DSUB];
#pragma unroll
          for (int j = 0; j < DSUB; ++j) {
            res0[j] = sres[m * DSUB + j];
            res1[j] = sres[dpad + m * DSUB + j];
          }
          const float4 v0 = lut_entry4<DSUB, MODE>(res0, row, sr2[m]);
          const float4 v1 = lut_entry4<DSUB, MODE>(res1, row, sr2[IVFPQ_MAX_M + m]);
          LDS floatx4 *dst = (LDS floatx4 *)(lut + m * 512 + 8 * lane);
          dst[0] = floatx4{v0.x, v1.x, v0.y, v1.y};
          dst[1] = floatx4{v0.z, v1.z, v0.w, v1.w};
        }
      }
    };
    if (a.mode == 0) build_rows(std::integral_constant<int, 0>{});
    else if (a.mode == 1) build_rows(std::integral_constant<int, 1>{});
    else build_rows(std::integral_constant<int, 2>{});
    // on their way while this task is scanned: the next task's list metadata, the pair
    // entries of the task after it
    const int tn = t + nwg;
    const bool more = tn < ntasks;
    int64_t nmv = 0;
    int2 nnv = make_int2(0, 0);
    if (more) nmv = fetch_meta(npv);
    if (tn + nwg < ntasks) nnv = fetch_pairs(tn + nwg);
    if constexpr (!HEAD) drain_pending();   // the queues are free again before this task fills them
    __syncthreads();
    // ---- one pass over the list's codes serves both queries ----
    int qc0 = 0, qc1 = 0;
    uint32_t mn0 = 0xFFFFFFFFu, mn1 = 0xFFFFFFFFu, mx0 = 0u, mx1 = 0u;   // head pass: key range of this wavefront's points
    // Head pass: the histogram's window.  No table entry exceeds its row's r_m^2, so a distance
    // lies in [0, sum of the r_m^2]: with finite radii the window is known before the scan and
    // every distance is counted as it is produced.  Otherwise (infinite radii) the window is
    // the range the distances turn out to span, and they are counted in a pass of their own.
    // Bins have equal width in value; bin_of is monotone in the distance, which is all the
    // selection needs.
    float wlo[2] = {0.0f, 0.0f}, wscale[2] = {0.0f, 0.0f};
    bool window_known = false;
    if constexpr (HEAD) {
      float s0 = lane < MT ? sr2[lane] : 0.0f, s1 = lane < MT ? sr2[IVFPQ_MAX_M + lane] : 0.0f;
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) {
        s0 += __shfl_xor(s0, off);
        s1 += __shfl_xor(s1, off);
      }
      window_known = s0 > 0.0f && s0 < __builtin_inff() && s1 > 0.0f && s1 < __builtin_inff();   // same in every wavefront
      wscale[0] = (float)LM_BINS / s0;
      wscale[1] = (float)LM_BINS / s1;
    }
    auto bin_of = [&](int g, uint32_t key) __attribute__((always_inline)) {
      const float x = (__uint_as_float(key) - wlo[g]) * wscale[g];
      return x >= (float)(LM_BINS - 1) ? (uint32_t)(LM_BINS - 1) : (x > 0.0f ? (uint32_t)x : 0u);
    };
    // tau_q as the bit pattern of a non-negative float (orders like the value; +inf when the
    // first lists held fewer than k points)
    const uint32_t tau0 = (uint32_t)__builtin_amdgcn_readlane((int)__float_as_uint(tk.tauv), 0);
    const uint32_t tau1 = (uint32_t)__builtin_amdgcn_readlane((int)__float_as_uint(tk.tauv), 1);
    const int last = tk.nb - 1;
    for (int blk = wave; blk < tk.nb; blk += NW) {
      CodeRegs<MPT / 4> cur = nxt;
      const int bn = blk + NW < last ? blk + NW : last;
      load_chunks<MPT, 0, NCH>(tk.base, tk.nb, bn, lane, nxt);   // past the end: re-reads the last block, in bounds
      float d0 = 0.0f, d1 = 0.0f;
#pragma unroll
      for (int h = 0; h < MT; h += LOOKUP_GROUP) lookup_group2<MT>(cur, h, cmin(h + LOOKUP_GROUP, MT), d0, d1);
      const int i = blk * 64 + lane;
      const bool valid = i < tk.len;
      const uint32_t row = (uint32_t)(tk.row0 + i);
      if constexpr (HEAD) {
        if (valid) {
          const uint32_t k0 = __float_as_uint(d0), k1 = __float_as_uint(d1);
          sdist[i] = k0;
          sdist[a.head_max + i] = k1;
          if (window_known) {
            lds_add(&hist[lm_hidx(bin_of(0, k0))]);
            lds_add(&hist[LM_BINS + lm_hidx(bin_of(1, k1))]);
          } else {
            mn0 = k0 < mn0 ? k0 : mn0;
            mx0 = k0 > mx0 ? k0 : mx0;
            mn1 = k1 < mn1 ? k1 : mn1;
            mx1 = k1 > mx1 ? k1 : mx1;
          }
        }
      } else {
        lm_offer(a, tk.q0, d0, valid, tau0, row, qd0, qrow0, qc0, lane);
        if (tk.has1) lm_offer(a, tk.q1, d1, valid, tau1, row, qd1, qrow1, qc1, lane);
      }
    }
    // the rest of the next task's inputs is requested before this task's candidates are
    // appended: both wait on the memory system at the same time
    const LmTask done = tk;
    if (more) {
      fetch_task(npv, nmv, tk, qv, cv, rv, nxt);
      npv = nnv;
    }
    if constexpr (HEAD) {
      const int L = done.len, k = a.k;
      const int ng = done.has1 ? 2 : 1;
      // window not known: smallest and largest key of each query's list (this wavefront's share first)
      if (!window_known)
        for (int g = 0; g < ng; ++g) {
          uint32_t lo = g ? mn1 : mn0, hi = g ? mx1 : mx0;
#pragma unroll
          for (int off = 32; off > 0; off >>= 1) {
            const uint32_t ol = (uint32_t)__shfl_xor((int)lo, off), oh = (uint32_t)__shfl_xor((int)hi, off);
            lo = ol < lo ? ol : lo;
            hi = oh > hi ? oh : hi;
          }
          if (lane == 0) {
            __hip_atomic_fetch_min(&ssel[4 + g], lo, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            __hip_atomic_fetch_max(&ssel[6 + g], hi, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
          }
        }
      __syncthreads();   // the list is scanned: every distance is in LDS and the table's LDS is free
      uint32_t top[2] = {LM_BINS, LM_BINS};   // collect keys whose bin is <= top (everything when the list is short)
      if (tid < LM_G * LM_COLLECT) {           // empty slots: the sentinel, and rank 0
        coll_d[tid] = SENT_D;
        coll_rank[tid] = 0u;
      }
      if (L <= LM_COLLECT) __syncthreads();    // (else the barriers of the histogram come before the slots are filled)
      if (L > LM_COLLECT) {                    // uniform; then k <= LM_COLLECT < L: the k-th smallest exists
        if (!window_known) {
          for (int g = 0; g < 2; ++g) {
            wlo[g] = __uint_as_float(ssel[4 + g]);
            wscale[g] = (float)LM_BINS / (__uint_as_float(ssel[6 + g]) - wlo[g]);   // one value only: every key in bin 0
          }
          for (int i = tid; i < L; i += NW * 64)
            for (int g = 0; g < ng; ++g) lds_add(&hist[g * LM_BINS + lm_hidx(bin_of(g, sdist[g * a.head_max + i]))]);
          __syncthreads();
        }
        if (wave < ng) {                       // wavefront g ranks query g's histogram
          uint32_t bin, below;
          lm_find_bin(hist + wave * LM_BINS, (uint32_t)k, lane, bin, below);
          if (lane == 0) ssel[2 + wave] = bin;
        }
        __syncthreads();
        top[0] = ssel[2];
        top[1] = ssel[3];
      }
      // collect (distance, position in the list) of the keys up to that bin; a wavefront reserves
      // the slots of its keys with one atomic operation
      for (int i0 = wave * 64; i0 < L; i0 += NW * 64) {
        const int i = i0 + lane;
        for (int g = 0; g < ng; ++g) {
          const uint32_t key = i < L ? sdist[g * a.head_max + i] : 0u;
          const bool take = i < L && bin_of(g, key) <= top[g];
          const unsigned long long bal = __ballot(take);
          if (bal == 0ull) continue;
          uint32_t first = 0;
          if (lane == 0) first = __hip_atomic_fetch_add(&ssel[g], (uint32_t)__popcll(bal), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
          first = (uint32_t)__builtin_amdgcn_readfirstlane((int)first);
          const uint32_t slot = first + (uint32_t)__popcll(bal & ((1ull << lane) - 1ull));
          if (take && slot < (uint32_t)LM_COLLECT) {
            coll_d[g * LM_COLLECT + slot] = key;
            coll_pos[g * LM_COLLECT + slot] = (uint32_t)i;
          }
        }
      }
      __syncthreads();
      // Rank sort, all wavefronts: thread (query g, key i, half h) counts the keys of half h of
      // query g's collected keys that precede key i in (distance, id) order; the two halves add
      // up to the key's position in the sorted order.  Unused slots hold the sentinel, which
      // precedes nothing, so the count runs over a fixed 64 slots, four per LDS read.  The id of
      // a key is requested before the count and only needed after it; where distances tie (rare)
      // the ids of the tying keys are fetched on the spot.
      {
        typedef uint32_t uintx4 __attribute__((ext_vector_type(4)));
        const int g = tid >> 8, i = tid & (LM_COLLECT - 1), h = (tid >> 7) & 1;
        const uint32_t n = ssel[g];
        const bool live = g < ng && n <= (uint32_t)LM_COLLECT && (uint32_t)i < n;
        const uint32_t md = live ? coll_d[g * LM_COLLECT + i] : SENT_D;
        const uint32_t mpos = live ? coll_pos[g * LM_COLLECT + i] : 0u;
        int64_t mid = SENT_ID;
        if (live) mid = a.ids[done.row0 + mpos];
        uint32_t before = 0, ties = 0;
        const LDS uintx4 *half = (const LDS uintx4 *)(coll_d + g * LM_COLLECT + h * (LM_COLLECT / 2));
#pragma unroll
        for (int j = 0; j < LM_COLLECT / 8; ++j) {
          const uintx4 od = half[j];
#pragma unroll
          for (int x = 0; x < 4; ++x) {
            before += od[x] < md ? 1u : 0u;
            ties += od[x] == md ? 1u : 0u;
          }
        }
        if (live) {
          if (ties > ((i >> 6) == h ? 1u : 0u)) {
            const int j0 = h * (LM_COLLECT / 2);
            for (int j = j0; j < j0 + LM_COLLECT / 2 && j < (int)n; ++j)
              if (coll_d[g * LM_COLLECT + j] == md && a.ids[done.row0 + coll_pos[g * LM_COLLECT + j]] < mid) ++before;
          }
          if (before) __hip_atomic_fetch_add(&coll_rank[g * LM_COLLECT + i], before, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
        __syncthreads();
        const int64_t q = g ? done.q1 : done.q0;
        if (g < ng && h == 0) {
          if (n > (uint32_t)LM_COLLECT) {
            if (i == 0) a.qmap_head[q] = (int32_t)q;   // too many equal distances: left to the query-major kernel
          } else if ((uint32_t)i < n) {
            const uint32_t r = coll_rank[g * LM_COLLECT + i];
            if (r < (uint32_t)k) {
              a.out_ids[q * k + r] = mid;
              a.out_dist[q * k + r] = __uint_as_float(md);
            }
          } else if (i < k) {                           // fewer than k points in the list
            a.out_ids[q * k + i] = -1;
            a.out_dist[q * k + i] = __builtin_inff();
          }
        }
      }
    } else {
      // One atomic instruction reserves the space of both queues: lane g for query g.  Its
      // result is not waited for here: the queued candidates are written to the reserved slots
      // after the next task's table is built (drain_pending), so the round trip of the atomic
      // is hidden behind that work.
      pend_slot = 0;
      const int n_mine = lane == 0 ? qc0 : (lane == 1 ? qc1 : 0);
      if (n_mine > 0) pend_slot = atomicAdd(&a.gcnt[lane == 0 ? done.q0 : done.q1], (uint32_t)n_mine);
      pend_q0 = done.q0;
      pend_q1 = done.q1;
      pend_c0 = qc0;
      pend_c1 = qc1;
    }
    if (!more) {
      if constexpr (!HEAD) drain_pending();
      break;
    }
    t = tn;
    __syncthreads();  // every wavefront is done with the table and the residuals before the next task rewrites them
  }
}

// One wavefront per query: the candidates of the list-major scan are merged into the top-k of
// the first lists by (distance, id).  Queries whose buffer overflowed are handed to the
// query-major kernel through qmap.
__global__ __launch_bounds__(256) void lm_merge_kernel(LmArgs a) {
  const int lane = threadIdx.x & 63;
  const int64_t q = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (q >= a.Q) return;
  const uint32_t n = a.gcnt[q];
  const bool overflow = n > (uint32_t)a.cap || (a.head_done && a.qmap_head[q] >= 0);
  if (lane == 0) a.qmap[q] = overflow ? (int32_t)q : -1;
  if (overflow || n == 0) return;   // redone elsewhere / phase A's result stands
  const int k = a.k;
  Key L0, L1;
  {
    const int64_t o = q * k;
    const bool in0 = lane < k, in1 = 64 + lane < k;
    const int64_t id0 = in0 ? a.out_ids[o + lane] : -1, id1 = in1 ? a.out_ids[o + 64 + lane] : -1;
    L0.d = id0 >= 0 ? __float_as_uint(a.out_dist[o + lane]) : SENT_D;
    L0.id = id0 >= 0 ? id0 : SENT_ID;
    L1.d = id1 >= 0 ? __float_as_uint(a.out_dist[o + 64 + lane]) : SENT_D;
    L1.id = id1 >= 0 ? id1 : SENT_ID;
  }
  Key tau;
  {
    const Key t0 = bcast_key(L0, (k - 1) & 63), t1 = bcast_key(L1, (k - 1) & 63);
    tau = (k - 1) < 64 ? t0 : t1;
  }
  for (uint32_t off = 0; off < n; off += 64) {
    Key c;
    c.d = SENT_D;
    c.id = SENT_ID;
    if (off + lane < n) {
      const uint2 e = a.cand[q * a.cap + off + lane];
      c.d = e.x;
      if (e.x <= tau.d) c.id = a.ids[e.y];   // a larger distance fails the test below whatever its id: no id fetched
    }
    const bool pass = kless(c, tau);
    if (__ballot(pass) == 0) continue;
    if (!pass) {
      c.d = SENT_D;
      c.id = SENT_ID;
    }
    wave_sort_desc<true>(c, lane);
    wave_merge<true>(L0, L1, c, lane);
    const Key t0 = bcast_key(L0, (k - 1) & 63), t1 = bcast_key(L1, (k - 1) & 63);
    tau = (k - 1) < 64 ? t0 : t1;
  }
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const Key e = h ? L1 : L0;
    const int i = h * 64 + lane;
    if (i < k) {
      const bool real = e.d != SENT_D;
      a.out_ids[q * k + i] = real ? e.id : -1;
      a.out_dist[q * k + i] = real ? __uint_as_float(e.d) : __builtin_inff();
    }
  }
}

std::atomic<int> g_lm_first{1};     // lists per query that are ranked first (their k-th distance filters the rest)
std::atomic<int> g_lm_cap{0};       // candidate slots per query; 0: by the number of probes (lm_auto_cap)

size_t lm_fixed_lds(int M, int D) {   // table, residuals, radii
  const int dpad = (D + 3) & ~3;
  return (size_t)M * 2048 + (size_t)LM_G * dpad * 4 + (size_t)LM_G * IVFPQ_MAX_M * 4;
}
size_t lm_scan_lds(int M, int D) { return lm_fixed_lds(M, D) + (size_t)LM_NW * LM_G * 2 * LM_QUEUE * 4; }
// head pass: the distances of the list's points for both queries live in LDS next to the table
int lm_head_max(int M, int D) {
  const int64_t spare = (int64_t)LDS_PER_CU - (int64_t)lm_fixed_lds(M, D) - LM_SEL_WORDS * 4 - LM_G * LM_BINS * 4;
  int64_t n = spare / (LM_G * 4);
  n &= ~(int64_t)63;
  return (int)(n > 8192 ? 8192 : (n < 0 ? 0 : n));
}
size_t lm_head_lds(int M, int D) { return lm_fixed_lds(M, D) + (size_t)LM_G * lm_head_max(M, D) * 4 + LM_SEL_WORDS * 4 + LM_G * LM_BINS * 4; }

template <int MT, int DSUB, bool HEAD>
int launch_lm_scan_t(const LmArgs &a, const RadiiSq &r2, int grid, hipStream_t s) {
  auto kern = lm_scan_kernel<MT, DSUB, HEAD>;
  static std::atomic<uint64_t> prepared;
  if (int rc = prepare_kernel(kern, prepared)) return rc;
  const size_t lds = HEAD ? lm_head_lds(MT, a.D) : lm_scan_lds(MT, a.D);
  hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(LM_NW * 64), lds, s, a, r2);
  return IVFPQ_OK;
}

template <bool HEAD>
int launch_lm_scan(const ivfpq_index *ix, const LmArgs &a, const RadiiSq &r2, int grid, hipStream_t s) {
  if (ix->M == 48) return launch_lm_scan_t<48, 2, HEAD>(a, r2, grid, s);
  if (ix->M == 64) return launch_lm_scan_t<64, 2, HEAD>(a, r2, grid, s);
  return launch_lm_scan_t<16, 4, HEAD>(a, r2, grid, s);
}

}  // namespace

namespace ivfpq {

void set_lm_first(int v) { g_lm_first.store(v, std::memory_order_relaxed); }
void set_lm_cap(int v) { g_lm_cap.store(v, std::memory_order_relaxed); }

bool list_major_supported(const ivfpq_index *ix, int32_t nprobe, int32_t k) {
  if (ix->metric != IVFPQ_METRIC_L2 || k > KP) return false;
  const bool shape = (ix->M == 48 && ix->dsub == 2) || (ix->M == 64 && ix->dsub == 2) || (ix->M == 16 && ix->dsub == 4);
  if (!shape || lm_scan_lds(ix->M, ix->D) > (size_t)LDS_PER_CU || LM_G * ix->D > LM_NW * 64 || LM_G * ix->M > LM_NW * 64) return false;
  return nprobe > g_lm_first.load(std::memory_order_relaxed);
}

static size_t lm_align(size_t v) { return (v + 255) & ~(size_t)255; }

LmWorkspace plan_list_major(const ivfpq_index *ix, int64_t Q, int32_t nprobe) {
  LmWorkspace w;
  w.first = g_lm_first.load(std::memory_order_relaxed);
  // Candidates that pass the first lists' bound grow with the number of lists probed; a query
  // that runs out of slots costs a query-major pass over all of its lists.  Measured on the
  // 1M x 96 configuration (64 probes): 4096 slots 11.39 ms per batch, 8192 10.88, 16384 10.71.
  w.cap = g_lm_cap.load(std::memory_order_relaxed);
  if (w.cap == 0) w.cap = nprobe >= 64 ? 16384 : (nprobe * 256 > 4096 ? nprobe * 256 : 4096);
  w.pairs_cap = Q * (nprobe - w.first > 1 ? nprobe - w.first : 1) + ix->nlist;   // also holds the head pass's Q pairs
  size_t off = 0;
  w.cnt = off;   off += lm_align((size_t)ix->nlist * 4);
  w.base = off;  off += lm_align(((size_t)ix->nlist + 1) * 4);
  w.pairs = off; off += lm_align((size_t)w.pairs_cap * 8);
  w.rank = off;  off += lm_align((size_t)w.pairs_cap * 4);
  w.gcnt = off;  off += lm_align((size_t)Q * 4);
  w.qmap = off;  off += lm_align((size_t)Q * 4);
  w.qmap_head = off; off += lm_align((size_t)Q * 4);
  w.cand = off;  off += lm_align((size_t)Q * w.cap * 8);
  w.total = off;
  return w;
}

int launch_scan_list_major(const ivfpq_index *ix, const float *d_queries, int64_t Q, int32_t nprobe,
                           const int32_t *d_probe_ids, int32_t k, const RadiiSq &r2, int32_t mode,
                           const float *d_query_radii, float *d_probe_lb, int64_t *d_out_ids, float *d_out_dist,
                           const LmWorkspace &w, char *lm_base, hipStream_t s) {
  if (Q * (int64_t)nprobe > 0x7FFFFFFFll || w.pairs_cap > 0x7FFFFFFFll) {
    set_error("scan (list-major): %lld (query, probe) pairs exceed 2^31", (long long)(Q * (int64_t)nprobe));
    return IVFPQ_ERR_UNSUPPORTED;
  }

  LmArgs a;
  a.queries = d_queries;
  a.probe_ids = d_probe_ids;
  a.probe_lb = (get_scan_ablate() & 64) ? nullptr : d_probe_lb;
  a.centroids = ix->d_centroids;
  a.codebooks = ix->d_codebooks;
  a.list_offsets = ix->d_list_offsets;
  a.list_blocks = ix->d_list_blocks;
  a.codes = ix->d_codes;
  a.ids = ix->d_ids;
  a.out_ids = d_out_ids;
  a.out_dist = d_out_dist;
  a.cnt = reinterpret_cast<int32_t *>(lm_base + w.cnt);
  a.rank = reinterpret_cast<int32_t *>(lm_base + w.rank);
  a.base = reinterpret_cast<int32_t *>(lm_base + w.base);
  a.pairs = reinterpret_cast<int2 *>(lm_base + w.pairs);
  a.gcnt = reinterpret_cast<uint32_t *>(lm_base + w.gcnt);
  a.cand = reinterpret_cast<uint2 *>(lm_base + w.cand);
  a.qmap = reinterpret_cast<int32_t *>(lm_base + w.qmap);
  a.qmap_head = reinterpret_cast<int32_t *>(lm_base + w.qmap_head);
  a.head_max = lm_head_max(ix->M, ix->D);
  a.query_radii = d_query_radii;
  a.Q = Q;
  a.D = ix->D; a.M = ix->M; a.dsub = ix->dsub; a.Mp = ix->Mp; a.nlist = ix->nlist;
  a.nprobe = nprobe; a.first = w.first; a.k = k; a.cap = w.cap; a.mode = mode;
  a.head_done = 0;

  // list-level lower bounds of every (query, probe); the same launch clears the per-list counts
  // (lm_offsets_kernel leaves them clear for the pass after it)
  int rc = launch_probe_bounds(ix, d_queries, Q, nprobe, d_probe_ids, r2, mode, d_query_radii, d_probe_lb, s, a.cnt,
                               ix->nlist);
  if (rc) return rc;

  int dev = 0, cus = 0;
  IVFPQ_HIP_TRY(hipGetDevice(&dev));
  IVFPQ_HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
  if (cus < 1) cus = 1;

  // ---- the first lists of every query: they give the bound tau_q that filters the rest ----
  // One list per query under distance scoring: the head pass ranks it list-major (queries that
  // share a nearest list share its table pass); what the head pass leaves out (qmap_head) skips
  // the list-major scan and is redone query-major at the end.  Otherwise (several first lists, or the hit-count scorings,
  // whose masses of equal scores the head pass's selection is not made for): query-major.
  const bool head_pass = w.first == 1 && mode == IVFPQ_SCORE_DISTANCE && a.head_max >= 64;
  if (head_pass) {
    const unsigned qgrid = (unsigned)((Q + 255) / 256);
    hipLaunchKernelGGL(lm_pairs_kernel, dim3(qgrid), dim3(256), 0, s, a, 0, 1);
    hipLaunchKernelGGL(lm_offsets_kernel, dim3(1), dim3(1024), 0, s, a);
    hipLaunchKernelGGL(lm_pairs_kernel, dim3(qgrid), dim3(256), 0, s, a, 1, 1);
    rc = launch_lm_scan<true>(ix, a, r2, cus, s);
    if (rc) return rc;
  }
  a.head_done = head_pass ? 1 : 0;
  if (!head_pass) {
    ScanView head = {nprobe, nullptr, true};
    rc = launch_scan(ix, d_queries, Q, w.first, d_probe_ids, k, r2, 1, nullptr, nullptr, d_out_ids, d_out_dist,
                     nullptr, nullptr, nullptr, nullptr, mode, d_query_radii, d_probe_lb, s, &head);
    if (rc) return rc;
  }

  // ---- the other lists, list-major: pairs bucketed by list, scan, merge ----
  const int64_t npairs = Q * (nprobe - w.first);
  const unsigned pair_grid = (unsigned)((npairs + 255) / 256);
  hipLaunchKernelGGL(lm_pairs_kernel, dim3(pair_grid), dim3(256), 0, s, a, 0, 0);
  hipLaunchKernelGGL(lm_offsets_kernel, dim3(1), dim3(1024), 0, s, a);
  hipLaunchKernelGGL(lm_pairs_kernel, dim3(pair_grid), dim3(256), 0, s, a, 1, 0);
  rc = launch_lm_scan<false>(ix, a, r2, cus, s);
  if (rc) return rc;
  hipLaunchKernelGGL(lm_merge_kernel, dim3((unsigned)((Q + 3) / 4)), dim3(256), 0, s, a);
  IVFPQ_HIP_TRY(hipGetLastError());
  // queries whose candidate buffer overflowed: the query-major kernel over all of their probes
  ScanView redo = {0, a.qmap, true};
  return launch_scan(ix, d_queries, Q, nprobe, d_probe_ids, k, r2, 1, nullptr, nullptr, d_out_ids, d_out_dist,
                     nullptr, nullptr, nullptr, nullptr, mode, d_query_radii, d_probe_lb, s, &redo);
}

}  // namespace ivfpq
