// Selective L2-LUT construction, distance calculation and top-k, fused
// (paper Sec. 4.1 and Algorithm 2 for the table; Sec. 2.1 step D and Sec. 5.3
// for the accumulation; Sec. 2.1 for the final selection).
//
// One workgroup serves one (query, probe group).  For each probed list it
//   1. builds the thresholded table for (query, list) in LDS: entry e of
//      subspace m stores d2 = ||res_m - codebook[m][e]||^2 if d2 <= r_m^2 and
//      the clamp r_m^2 otherwise (res = query - list centroid);
//   2. streams the list's codes from HBM, one point per lane, 16 bytes per load,
//      and sums the table values of the point's codes in subspace order (fp32,
//      the same order as a plain loop, so sums are reproducible bit for bit).
//      A block of 64 points is dropped as soon as partial sum + (sum of the row
//      minima of the remaining subspaces) exceeds the current k-th distance for
//      all of its points, and code bytes that were not needed are never requested:
//      exact, i.e. the result is that of the plain loop;
//   3. keeps, per wavefront, the 128 best (distance, id) pairs seen so far as a
//      sorted list spread over the lanes' registers; candidates that beat the
//      current k-th best are queued in LDS and folded in 64 at a time with a
//      bitonic merge.
// At the end the wavefronts' lists are merged and the first k written out.
//
// The paper builds the table on RT cores (a ray per (query, list, subspace)
// against one sphere per entry) and accumulates on tensor cores.  CDNA4 has
// neither RT cores nor a reason to turn a byte-indexed gather into a matrix
// product: the radius test is a compare on the vector ALU and the accumulation
// is bound by HBM and LDS gather rates.

#include "scan_device.h"

namespace {

using ivfpq::GRID_G;

// BYTE: the hit-count scorings with a byte table (one byte per entry, 256 bytes per row,
// integer sums) instead of the float table; the sums are the same small integers either way.
template <int MT, int DSUB, int NW, bool DUMP, bool BYTE = false>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(scan_wpe(BYTE ? (MT + 3) / 4 : MT, NW)))) void scan_kernel(ScanArgs a, RadiiSq r2) {
  constexpr int NT = NW * 64;
  using Acc = std::conditional_t<BYTE, uint32_t, float>;
  constexpr int MPT = (MT + 3) / 4 * 4;
  extern __shared__ __align__(16) unsigned char smem[];
  const int M = MT > 0 ? MT : a.M;
  const int Mp = MT > 0 ? MPT : a.Mp;
  const int D = a.D;
  const int dsub = DSUB > 0 ? DSUB : a.dsub;
  // LDS carve: table | merge staging (aliases the table) | query | queues | tau
  const int lut_bytes = M * (BYTE ? 256 : 1024);
  const int stage_bytes = NW * KP * 12;
  const int region0 = lut_bytes > stage_bytes ? lut_bytes : stage_bytes;
  LDS unsigned char *smem3 = (LDS unsigned char *)smem;
  LDS float *lut = (LDS float *)smem3;
  LDS float *sq = (LDS float *)(smem3 + region0);
  const int sq_bytes = 2 * ((D * 4 + 15) & ~15);  // the query, then the residual of the current list
  LDS float *sres = sq + (sq_bytes >> 3);
  LDS int64_t *queue_id = (LDS int64_t *)(smem3 + region0 + sq_bytes);
  LDS uint32_t *queue_d = (LDS uint32_t *)(smem3 + region0 + sq_bytes + NW * 64 * 8);
  LDS uint32_t *tau_words = (LDS uint32_t *)(smem3 + region0 + sq_bytes + NW * 64 * 12);
  // per-probe list metadata of up to META probes, staged once per chunk of probes so
  // that a probe does not start with a chain of dependent scalar loads
  constexpr int META = 64;
  const int tau_bytes = (4 * (2 * NW + 4) + 15) & ~15;  // bound | ranks [NW] | wide: slots taken, overflow | wide: counts [NW]
  LDS int64_t *meta_row0 = (LDS int64_t *)(smem3 + region0 + sq_bytes + NW * 64 * 12 + tau_bytes);
  LDS int64_t *meta_blk = meta_row0 + META;
  LDS int32_t *meta_len = (LDS int32_t *)(meta_blk + META);
  LDS int32_t *meta_c = meta_len + META;
  LDS float *meta_lb = (LDS float *)(meta_c + META);
  LDS float *sr2 = meta_lb + META;  // [M] r_m^2 of this query
  LDS uint32_t *srmin = (LDS uint32_t *)(sr2 + IVFPQ_MAX_M);  // [M][4] partial minima (bit patterns) of each row of the current table

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform, kept in a scalar register
  LDS float *ssuf = (LDS float *)(srmin + 4 * IVFPQ_MAX_M) + wave * SUF_SLOTS;  // this wavefront's suffix sums of srmin, per 8 subspaces
  LDS uint32_t *stat = (LDS uint32_t *)((LDS float *)(srmin + 4 * IVFPQ_MAX_M) + NW * SUF_SLOTS);  // blocks scanned / scanned to the end
  const int64_t q = blockIdx.x / a.nsplit;
  const int split = blockIdx.x % a.nsplit;
  const int p_begin = (int)((int64_t)a.nprobe * split / a.nsplit);
  const int p_end = (int)((int64_t)a.nprobe * (split + 1) / a.nsplit);
  const int32_t *probes = a.probe_ids + q * a.probe_stride;
  // with a query map only the queries it names are served (uniform over the workgroup)
  if (a.qmap && a.qmap[q] < 0) return;

  int64_t dump_pos = 0;
  if (DUMP) {
    int64_t total = 0;
    for (int p = 0; p < a.nprobe; ++p) {
      const int32_t c = probes[p];
      if ((uint32_t)c < (uint32_t)a.nlist) total += a.list_offsets[c + 1] - a.list_offsets[c];
    }
    if (total != a.cand_offsets[q + 1] - a.cand_offsets[q]) {
      if (tid == 0) atomicAdd(a.errors, 1);
      return;
    }
    dump_pos = a.cand_offsets[q];
  }

  for (int i = tid; i < D; i += NT) sq[i] = a.queries[q * D + i];
  for (int m = tid; m < M; m += NT) {
    float v = r2.v[m];
    if (a.query_radii) {
      const float r = a.query_radii[q * M + m];
      v = r * r;
    }
    sr2[m] = v;
    srmin[4 * m] = srmin[4 * m + 1] = srmin[4 * m + 2] = srmin[4 * m + 3] = 0u;
  }
  const int mode = a.mode;
  if (tid <= NW) tau_words[tid] = SENT_D;
  if (tid < 2) stat[tid] = 0u;
  const bool wide = !DUMP && a.wide_cap > 0;
  if (tid < 2) tau_words[NW + 1 + tid] = 0u;
  SharedTau sh;
  sh.bound = tau_words;
  sh.rank = tau_words + 1;
  sh.nw = NW;
  sh.wave = wave;
  // wide selection: the bound is on the k_out-th distance, from ceil(k_out / NW) keys per wavefront
  sh.jrank = ((wide ? a.k_out : a.k) + NW - 1) / NW;
  sh.wide = wide ? tau_words + NW + 1 : nullptr;
  sh.wide_d = wide ? a.wide_d + q * a.wide_cap : nullptr;
  sh.wide_id = wide ? a.wide_id + q * a.wide_cap : nullptr;
  sh.wide_cap = a.wide_cap;

  WaveTop st;
  init_wave_top<false, DUMP>(st, a, q);
  LDS uint32_t *qd = queue_d + wave * 64;
  LDS int64_t *qid = queue_id + wave * 64;

  // Codebook rows of this wavefront (rows wave, wave + NW, ...): the first RES of them
  // stay in registers for the whole kernel -- the codebook is the same for every list
  // and re-reading all of it per list costs a quarter of the kernel on short lists --
  // the remaining STR are streamed per list.  RES is what fits beside the scan's
  // registers at 4 wavefronts per SIMD.
  constexpr bool VEC = MT > 0 && (DSUB == 2 || DSUB == 4);
  constexpr int ITER = VEC ? (MT + NW - 1) / NW : 1;
  constexpr int DS4 = VEC ? DSUB : 1;
  constexpr int WPE = scan_wpe(BYTE ? (MT + 3) / 4 : MT, NW);
  // (a dsub = 4 row takes 16 registers and its table arithmetic more temporaries: with resident
  // rows the kernel spilled up to 198 registers, so those rows are all streamed)
  constexpr int RES_REGS = DS4 == 4 ? 0 : res_regs(WPE), RES_MAX_TOTAL = res_max_total(WPE);
  constexpr int RES_BUDGET = RES_REGS < RES_MAX_TOTAL - 2 * (MPT / 4) ? RES_REGS : RES_MAX_TOTAL - 2 * (MPT / 4);
  constexpr int RES_CAP = (RES_BUDGET > 0 ? RES_BUDGET : 0) / (4 * DS4);
  constexpr int RES = !VEC ? 0 : (ITER < RES_CAP ? ITER : RES_CAP);
  constexpr int STR = VEC ? ITER - RES : 0;
  float4 cbr[RES > 0 ? RES : 1][DS4];
  if constexpr (VEC) {
#pragma unroll
    for (int it = 0; it < RES; ++it) {
      const int m = wave + it * NW;
      const int mc = m < MT ? m : MT - 1;
      const uint8_t *cb = uniform_ptr(reinterpret_cast<const uint8_t *>(a.codebooks + (int64_t)mc * 256 * DSUB));
#pragma unroll
      for (int x = 0; x < DSUB; ++x)
        cbr[it][x] = *reinterpret_cast<const float4 *>(cb + (uint32_t)(lane * 16 * DSUB + 16 * x));
    }
  }
  // Code chunks per point (16-byte chunks, then 4-byte chunks) and how many of them
  // the "first half" loading mode fetches ahead; that mode exists when it splits the
  // chunks in two non-empty parts.
  constexpr int NCH = MPT / 16 + (MPT % 16) / 4;
  constexpr int HCH = (MPT / 16 + 1) / 2;
  constexpr int MH = 16 * HCH;  // subspaces covered by the first HCH chunks
  constexpr bool HALF_OK = MT > 0 && HCH >= 1 && HCH < NCH && MH < MT;
  constexpr bool QUARTER_OK = HALF_OK && HCH >= 2;  // the first chunk alone (16 subspaces) is a proper part
  // How much of a block is fetched ahead: 0 all chunks, 1 the first half, 2 the first chunk;
  // the rest is fetched when a block turns out to need it.  While pruning, most blocks end
  // within their first chunk.
  int depth = 0, depth_later = 0;
  if (HALF_OK && !DUMP && a.load_mode != 1) depth_later = (QUARTER_OK && a.load_mode != 2) ? 2 : 1;
  // the first list of a query is scanned without any bound, so every block of it is needed
  // whole: it is fetched whole (in the default mode), the lists after it by parts
  if (a.load_mode != 0) depth = depth_later;
  auto load_ahead = [&](const uint8_t *lb, int nblk, int blk, CodeRegs<MPT / 4> &r) __attribute__((always_inline)) {
    if constexpr (MT > 0) {
      load_chunks<MPT, 0, HALF_OK ? 1 : NCH>(lb, nblk, blk, lane, r);
      if constexpr (HALF_OK) {
        if (depth < 2) load_chunks<MPT, 1, HCH>(lb, nblk, blk, lane, r);
        if (depth < 1) load_chunks<MPT, HCH, NCH>(lb, nblk, blk, lane, r);
      }
    }
  };
  bool sres_ready = false;
  // Pruning (row minima, checks of the partial sums, partial loads) pays only where blocks
  // do end early.  The workgroup counts, over the first PROBE_LISTS lists of its query, how
  // many blocks were scanned and how many of them to the end; if nearly all were, the rest
  // of the lists are scanned plainly.  Results do not depend on it.
  constexpr int PROBE_LISTS = 4;
  bool prune = VEC && !DUMP && !(a.ablate & 16);
  uint32_t tot_blocks = 0, tot_full = 0;
  bool pushed = false, decided = (a.ablate & 16) != 0;
  auto push_counts = [&](int last_list) __attribute__((always_inline)) {
    if (VEC && !DUMP && !pushed && last_list - p_begin >= PROBE_LISTS - 1) {
      pushed = true;
      if (lane == 0) {
        __hip_atomic_fetch_add(stat, tot_blocks, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        __hip_atomic_fetch_add(stat + 1, tot_full, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      }
    }
  };
  for (int p = p_begin; p < p_end; ++p) {
    const int pm = (p - p_begin) & (META - 1);
    if (pm == 0) {
      // every wavefront has passed the second barrier of the previous probe, so nobody
      // still reads the old entries
      if (tid < META && p + tid < p_end) {
        const int32_t cc = probes[p + tid];
        const bool ok = (uint32_t)cc < (uint32_t)a.nlist;
        const int64_t r0 = ok ? a.list_offsets[cc] : 0;
        meta_c[tid] = ok ? cc : 0;  // a probe id outside [0, nlist) becomes an empty list
        meta_row0[tid] = r0;
        meta_len[tid] = ok ? (int)(a.list_offsets[cc + 1] - r0) : 0;
        meta_blk[tid] = ok ? a.list_blocks[cc] : 0;
        meta_lb[tid] = (ok && a.probe_lb) ? a.probe_lb[q * a.probe_stride + p + tid] : 0.0f;
      }
      __syncthreads();
    }
    const int32_t c = __builtin_amdgcn_readfirstlane(meta_c[pm]);
    const int64_t row0 = meta_row0[pm];
    const int len = __builtin_amdgcn_readfirstlane(meta_len[pm]);
    const int nb = (len + 63) >> 6;
    const uint8_t *base = a.codes + meta_blk[pm] * ivfpq_block_bytes(Mp);
    const float *cen = a.centroids + (int64_t)c * D;
    // Loads that do not depend on LDS go out before the barrier, so that their
    // latency overlaps the tail of the previous list: the streamed part of this
    // wavefront's codebook rows and the first code block of the new list.
    float4 cbs[STR > 0 ? STR : 1][DS4];
    CodeRegs<MPT / 4> nxt;
    // The residual q - centroid of a list is formed once, in LDS.  For the list after
    // this one the centroid is requested now and the residual written after this
    // list's table is finished, so the next table does not wait for it.
    const bool next_known = VEC && D <= NT && pm + 1 < META && p + 1 < p_end;
    float cen_next = 0.0f;
    if constexpr (VEC) {
      if (!sres_ready)
        for (int i = tid; i < D; i += NT) sres[i] = sq[i] - cen[i];
      if (next_known && tid < D)
        cen_next = *reinterpret_cast<const float *>(
            uniform_ptr(reinterpret_cast<const uint8_t *>(
                a.centroids + (int64_t)__builtin_amdgcn_readfirstlane(meta_c[pm + 1]) * D)) +
            (uint32_t)(tid * 4));
#pragma unroll
      for (int it = 0; it < STR; ++it) {
        const int m = wave + (RES + it) * NW;
        const int mc = m < MT ? m : MT - 1;
        const uint8_t *cb = uniform_ptr(reinterpret_cast<const uint8_t *>(a.codebooks + (int64_t)mc * 256 * DSUB));
#pragma unroll
        for (int x = 0; x < DSUB; ++x)
          cbs[it][x] = *reinterpret_cast<const float4 *>(cb + (uint32_t)(lane * 16 * DSUB + 16 * x));
      }
    }
    if constexpr (MT > 0) {
      // an empty list still has readable padding behind its base
      // (with 128 registers only the first chunk goes out here, whatever the depth: the
      // registers of the other chunks stay free while the table is built)
      const int b0 = wave < nb ? wave : (nb > 0 ? nb - 1 : 0);
      if constexpr (WPE == 2) load_ahead(base, nb, b0, nxt);
      else load_chunks<MPT, 0, HALF_OK ? 1 : NCH>(base, nb, b0, lane, nxt);
    }
    __syncthreads();  // previous list fully scanned (and sq written) before the table changes
    if (!DUMP && wide && sh.wide[0] > (uint32_t)(a.wide_cap >> 2) && sh.wide[1] == 0u)
      wide_compact<NW>(sh, tau_words + NW + 3, tid, lane, wave);
    if (VEC && !DUMP && !decided && p - p_begin >= PROBE_LISTS) {  // every wavefront has pushed its counts
      decided = true;
      if (!(a.ablate & 32)) {
        const uint32_t nblk = stat[0], nfull = stat[1];
        prune = 8 * (uint64_t)nfull < 7 * (uint64_t)nblk;
      }
    }
    // List-level bound (probe_bound_kernel): if not even the lower bound on any point of
    // this list is within the workgroup's bound on the k-th distance, neither table nor scan
    // is needed.  Between the two barriers nobody scans, so every wavefront reads the same
    // shared bound and the decision is uniform over the workgroup.
    bool skip_list = false;
    if (VEC && !DUMP) {
      const uint32_t bnd = *(volatile LDS uint32_t *)sh.bound;
      skip_list = bnd != SENT_D && meta_lb[pm] > __uint_as_float(bnd);
    }
    if (skip_list) {
      // Ruled out.  The bound cannot change while nobody scans, so the following probes of
      // this metadata chunk are checked right here and the workgroup goes on with the first
      // one that is not ruled out: a run of skipped lists costs one barrier.
      const float bound_f = __uint_as_float(*(volatile LDS uint32_t *)sh.bound);
      int pn = p;
      do {
        const int pmn = (pn - p_begin) & (META - 1);
        const int nbn = (meta_len[pmn] + 63) >> 6;
        if (wave < nbn) tot_blocks += (nbn - 1 - wave) / NW + 1;  // all pruned: counts for the switch
        ++pn;
      } while (pn < p_end && ((pn - p_begin) & (META - 1)) != 0 && meta_lb[(pn - p_begin) & (META - 1)] > bound_f);
      push_counts(pn - 1);
      __syncthreads();  // nobody still reads the metadata when the next chunk is staged
      sres_ready = false;
      p = pn - 1;
      continue;
    }
    // ---- selective table for (query, list c) ----
    if constexpr (VEC) {
      // one subspace per wavefront and pass, four consecutive entries per lane; the
      // scoring mode is resolved once per list, outside the unrolled passes
      auto build_rows = [&](auto mode_tag) __attribute__((always_inline)) {
        constexpr int MODE = decltype(mode_tag)::value;
        constexpr int NBATCH = (ITER + 7) / 8;
        uint32_t lo[NBATCH][8];  // this lane's minimum over its entries of each row (for the early exit)
#pragma unroll
        for (int it = 0; it < NBATCH * 8; ++it) lo[it >> 3][it & 7] = 0xFFFFFFFFu;
        // With 256 registers (WPE == 2) the passes form straight-line code (the validity of
        // a row is known at compile time for every pass but the last) and the compiler
        // overlaps their LDS reads.  With 128 registers that form spills, so each row stays
        // a block of its own.
        constexpr bool STRAIGHT = WPE == 2;
#pragma unroll
        for (int it = 0; it < ITER; ++it) {
          const int m = wave + it * NW;
          if ((STRAIGHT && (it + 1) * NW <= MT) || m < MT) {
            float res[DS4];
#pragma unroll
            for (int j = 0; j < DS4; ++j) res[j] = sres[m * DSUB + j];
            const float4 v = lut_entry4<DSUB, MODE>(res, it < RES ? cbr[it < RES ? it : 0] : cbs[it >= RES ? it - RES : 0], sr2[m]);
            if constexpr (BYTE)   // penalties 0, 1, 2: four entries in one dword
              *((LDS uint32_t *)lut + m * 64 + lane) = (uint32_t)v.x | ((uint32_t)v.y << 8) | ((uint32_t)v.z << 16) | ((uint32_t)v.w << 24);
            else
              *(LDS floatx4 *)(lut + m * 256 + 4 * lane) = floatx4{v.x, v.y, v.z, v.w};
            if (!DUMP)
              lo[it >> 3][it & 7] = umin32(umin32(__float_as_uint(v.x), __float_as_uint(v.y)),
                                           umin32(__float_as_uint(v.z), __float_as_uint(v.w)));
          }
        }
        if (!DUMP && prune) {
          // one partial minimum per row and 16 lanes goes to LDS; the reader takes the
          // smallest of the four
#pragma unroll
          for (int bt = 0; bt < NBATCH; ++bt) {
            const uint32_t d = rows8_min16(lo[bt], lane);
            const int it = bt * 8 + (lane & 7);
            const int m = wave + it * NW;
            if ((lane & 15) < 8 && it < ITER && m < MT) srmin[4 * m + (lane >> 4)] = d;
          }
        }
      };
      if (mode == 0) build_rows(std::integral_constant<int, 0>{});
      else if (mode == 1) build_rows(std::integral_constant<int, 1>{});
      else build_rows(std::integral_constant<int, 2>{});
    } else {
      const int e = tid & 255;
      for (int m = tid >> 8; m < M; m += NT >> 8) {
        const int mu = __builtin_amdgcn_readfirstlane(m);
        bool keep;
        lut[mu * 256 + e] = lut_entry<DSUB>(sq + mu * dsub, cen + mu * dsub,
                                            a.codebooks + ((int64_t)mu * 256 + e) * dsub, dsub,
                                            sr2[mu], mode, keep);
      }
    }
    __syncthreads();
    if constexpr (VEC) {
      if (next_known && tid < D) sres[tid] = sq[tid] - cen_next;  // this list's table is complete
      sres_ready = next_known;
    }
    // ---- distance calculation over list c ----
    if (MT > 0) {
      // Two register sets: `nxt` receives the loads of the next block while `cur` is
      // looked up.  Loads are issued for every iteration (past the end they re-read the
      // list's last block, which is in bounds), so the block in flight never has to
      // complete before the current one can be used.
      // Suffix sums of the row minima at the check points (every 8 subspaces), per wavefront:
      // lane l holds rows l and 64 + l, groups of 8 lanes are summed in place, then the
      // groups are accumulated from the last one down.
      float suf0 = 0.0f;
      if (VEC && !DUMP && prune) {
        constexpr int NG = (MT + 7) / 8;
        typedef uint32_t uintx4 __attribute__((ext_vector_type(4)));
        auto row_min = [&](int m) {
          const uintx4 p = *(const LDS uintx4 *)(srmin + 4 * m);
          return __uint_as_float(umin32(umin32(p[0], p[1]), umin32(p[2], p[3])));
        };
        float v0 = lane < MT ? row_min(lane) : 0.0f;
        float v1 = (MT > 64 && lane + 64 < MT) ? row_min((MT > 64 ? 64 : 0) + lane) : 0.0f;
        v0 = group8_sum(v0);
        v1 = group8_sum(v1);
        float acc = 0.0f;
#pragma unroll
        for (int j = NG - 1; j >= 0; --j) {
          const int gl = __builtin_amdgcn_readlane((int)__float_as_uint(j < 8 ? v0 : v1), (j & 7) * 8);
          acc += __uint_as_float((uint32_t)gl);
          if (lane == 0) ssuf[j] = acc;
        }
        if (lane == 0) ssuf[NG] = 0.0f;
        suf0 = acc;
      }
      if (wave < nb) {
        const int last = nb - 1;
        int blocks = 0, full = 0;
        if constexpr (HALF_OK && WPE != 2) {  // the rest of what is fetched ahead of the first block
          if (depth < 2) load_chunks<MPT, 1, HCH>(base, nb, wave, lane, nxt);
          if (depth < 1) load_chunks<MPT, HCH, NCH>(base, nb, wave, lane, nxt);
        }
        for (int b = wave; b < nb; b += NW) {
          CodeRegs<MPT / 4> cur = nxt;
          const int bn = b + NW < last ? b + NW : last;
          load_ahead(base, nb, bn, nxt);
          const int i = b * 64 + lane;
          const bool valid = i < len;
          if (DUMP) {
            const float dist = BYTE ? adc_sum_bytes<MT>(lut, cur) : adc_sum<MT>(lut, cur);
            if (valid) {
              a.all_dist[dump_pos + i] = dist;
              a.all_ids[dump_pos + i] = a.ids[row0 + i];
            }
          } else {
            const uint32_t shared = *(volatile LDS uint32_t *)sh.bound;
            const uint32_t pref = (a.ablate & 8) ? SENT_D : ((wide || shared < st.tau.d) ? shared : st.tau.d);
            // bound on the k-th smallest distance, enlarged as adc_part_exit needs it
            const float tauf = pref == SENT_D ? __builtin_inff() : __uint_as_float(pref) * 1.0001220703125f;
            Acc dist = 0;
            ++blocks;
            // no point of this list can reach the bound any more (it only tightens): the
            // wavefront is done with the list, and requests no further blocks of it
            if (prune && !(suf0 <= tauf)) {
              blocks += (nb - 1 - b) / NW;
              break;
            }
            // The block in up to three parts (first chunk, rest of the first half, second
            // half); most blocks end in an early part, and a part that was not fetched ahead
            // is fetched when a block turns out to need it.
            if constexpr (QUARTER_OK) {
              if (!adc_part_exit<MT, 0, 16>(lut, cur, ssuf, tauf, prune, valid, dist)) continue;
              if (depth == 2) load_chunks<MPT, 1, HCH>(base, nb, b, lane, cur);
              if (!adc_part_exit<MT, 16, MH>(lut, cur, ssuf, tauf, prune, valid, dist)) continue;
            } else if constexpr (HALF_OK) {
              if (!adc_part_exit<MT, 0, MH>(lut, cur, ssuf, tauf, prune, valid, dist)) continue;
            }
            if (HALF_OK && depth >= 1) load_chunks<MPT, HCH, NCH>(base, nb, b, lane, cur);
            if (!adc_part_exit<MT, HALF_OK ? MH : 0, MT>(lut, cur, ssuf, tauf, prune, valid, dist)) continue;
            ++full;
            wave_offer(st, acc_value(dist), valid, row0 + i, a.ids, qd, qid, lane, a.k, sh);
          }
        }
        tot_blocks += blocks;
        tot_full += full;
      }
      // without pruning every block is needed whole; the list during which pruning was
      // switched off still had its blocks fetched by halves
      depth = (!prune && a.load_mode < 2) ? 0 : depth_later;
      push_counts(p);
    } else {
      for (int b = wave; b < nb; b += NW) {
        const float dist = adc_sum_rt(lut, base, nb, b, lane, M, Mp);
        const int i = b * 64 + lane;
        const bool valid = i < len;
        if (DUMP && valid) {
          a.all_dist[dump_pos + i] = dist;
          a.all_ids[dump_pos + i] = a.ids[row0 + i];
        }
        if (!DUMP) wave_offer(st, dist, valid, row0 + i, a.ids, qd, qid, lane, a.k, sh);
      }
    }
    if (DUMP) dump_pos += len;
  }
  if (DUMP) return;

  if (wide) finish_wide(st, qd, qid, lane, tid, sh, a, q);
  else finish_topk<NW>(st, qd, qid, lane, wave, sh, smem3, a, q, split);
}


// ---------------------------------------------------------------------------
// Inner-product metric (paper Sec. 4.2 "Inner Product Similarity Support").
//
// The paper enlarges the sphere of entry e to radius^2 = r_m^2 + |e|^2 and starts the
// ray at the projection q_m of the QUERY; it hits iff |q_m - e|^2 <= r_m^2 + |e|^2, i.e.
// iff IP(e, q_m) >= thr_m = (|q_m|^2 - r_m^2) / 2, which is the form evaluated here.
// A kept entry stores 0 - IP, a missed one the bound 0 - thr_m.  The table depends on
// the query only, so a workgroup builds it once and then streams the probed lists with
// no barrier between them; a point of list c scores (0 - IP(q, centroid_c)) plus the
// sum of its table values, subspaces ascending.  Scores have either sign: keys go
// through the order-preserving map of dist_key, and the early exit of the sums works
// from a lower bound on what the remaining subspaces can still add (adc_ip_exit).

template <int MODE>
__device__ inline float table_value_ip(float ip, float thr, float thr_in) {
  if (MODE == 0) return ip >= thr ? 0.0f - ip : 0.0f - thr;
  if (MODE == 1) return ip >= thr ? 0.0f : 1.0f;
  return ip >= thr_in ? 0.0f : (ip >= thr ? 1.0f : 2.0f);
}
__device__ inline float table_value_ip(float ip, float thr, float thr_in, int mode) {
  return mode == 0 ? table_value_ip<0>(ip, thr, thr_in)
                   : (mode == 1 ? table_value_ip<1>(ip, thr, thr_in) : table_value_ip<2>(ip, thr, thr_in));
}

// ip = q_0 e_0, then ip = fmaf(q_j, e_j, ip)
template <typename SP>
__device__ inline float entry_ip(SP qm, const float *__restrict__ cb, int dsub) {
  float ip = qm[0] * cb[0];
  for (int j = 1; j < dsub; ++j) ip = fmaf(qm[j], cb[j], ip);
  return ip;
}

// thr = (|q_m|^2 - r2) / 2 and the same with the half radius; |q_m|^2 as q_0 q_0, then fmaf
template <typename SP>
__device__ inline void ip_thresholds(SP qm, int dsub, float r2, float &thr, float &thr_in) {
  float qq = qm[0] * qm[0];
  for (int j = 1; j < dsub; ++j) qq = fmaf(qm[j], qm[j], qq);
  thr = 0.5f * (qq - r2);
  thr_in = 0.5f * (qq - 0.25f * r2);
}

// 0 - q.c with acc = fmaf(q_i, c_i, acc), i ascending (the list term of a score)
template <typename SP>
__device__ inline float neg_ip_chain(SP sq, const float *__restrict__ cen, int D) {
  float acc = 0.0f;
  int i = 0;
  if ((D & 3) == 0 && (reinterpret_cast<uintptr_t>(cen) & 15) == 0) {
    for (; i < D; i += 4) {
      const float4 c4 = *reinterpret_cast<const float4 *>(cen + i);
      acc = fmaf(sq[i], c4.x, acc);
      acc = fmaf(sq[i + 1], c4.y, acc);
      acc = fmaf(sq[i + 2], c4.z, acc);
      acc = fmaf(sq[i + 3], c4.w, acc);
    }
  }
  for (; i < D; ++i) acc = fmaf(sq[i], cen[i], acc);
  return 0.0f - acc;
}

// Sum with early exit for terms of either sign.  suf[j] is the fp32 sum of the row minima
// of subspaces >= 8 j, and slack >= (4 M + 8) 2^-24 (|start| + sum_m max_e |table[m][e]|).
// Every fp32 addition is monotone in both operands, so the final sum is at least what the
// chain gives when each remaining term is replaced by its row minimum; that in turn is at
// least partial + (exact sum of the minima) - M 2^-24 (|start| + sum of max |term|) by the
// usual bound on sequential summation.  suf, slack and the test expression are themselves
// rounded; all of these errors together stay below half of slack.  So if
// fl(partial + fl(suf - slack)) is above the bound on the k-th best score for every point of
// the block, no point of it can enter the result and the rest of the block is skipped.
// Points that survive get exactly the sum adc_sum computes.
template <int MT, int M0, int M1>
__device__ inline bool adc_ip_exit(const LDS float *lut, const CodeRegs<((MT + 3) / 4 * 4) / 4> &r,
                                   uint32_t pref, bool valid, const LDS float *suf, float slack, float &dist) {
#pragma unroll
  for (int g = M0; g < M1; g += 8) {
    // requested ahead of the look-ups, so that it has arrived when they have
    float rest = 0.0f;
    if (cmin(g + 8, M1) < MT) rest = suf[cmin(g + 8, M1) >> 3];
#pragma unroll
    for (int h = g; h < cmin(g + 8, M1); h += LOOKUP_GROUP)
      lookup_group<MT>(lut, r, h, cmin(h + LOOKUP_GROUP, cmin(g + 8, M1)), dist);
    if (cmin(g + 8, M1) < MT) {
      const float lb = dist + (rest - slack);
      if (__ballot(valid && dist_key<true>(lb) <= pref) == 0) return false;
    }
  }
  return true;
}

template <int MT, int NW, bool DUMP>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(4))) void scan_ip_kernel(ScanArgs a, RadiiSq r2) {
  constexpr int NT = NW * 64;
  constexpr int MPT = (MT + 3) / 4 * 4;
  constexpr int META = 64;
  extern __shared__ __align__(16) unsigned char smem[];
  const int M = MT > 0 ? MT : a.M;
  const int Mp = MT > 0 ? MPT : a.Mp;
  const int D = a.D, dsub = a.dsub;
  // LDS carve: table | merge staging (aliases the table) | query | queues | bounds | list metadata | thresholds
  const int lut_bytes = M * 1024;
  const int stage_bytes = NW * KP * 12;
  const int region0 = lut_bytes > stage_bytes ? lut_bytes : stage_bytes;
  LDS unsigned char *smem3 = (LDS unsigned char *)smem;
  LDS float *lut = (LDS float *)smem3;
  LDS float *sq = (LDS float *)(smem3 + region0);
  const int sq_bytes = (D * 4 + 15) & ~15;
  LDS int64_t *queue_id = (LDS int64_t *)(smem3 + region0 + sq_bytes);
  LDS uint32_t *queue_d = (LDS uint32_t *)(smem3 + region0 + sq_bytes + NW * 64 * 8);
  LDS uint32_t *tau_words = (LDS uint32_t *)(smem3 + region0 + sq_bytes + NW * 64 * 12);
  const int tau_bytes = (4 * (2 * NW + 4) + 15) & ~15;  // bound | ranks [NW] | wide: slots taken, overflow | wide: counts [NW]
  LDS int64_t *meta_row0 = (LDS int64_t *)(smem3 + region0 + sq_bytes + NW * 64 * 12 + tau_bytes);
  LDS int64_t *meta_blk = meta_row0 + META;
  LDS int32_t *meta_len = (LDS int32_t *)(meta_blk + META);
  LDS float *meta_start = (LDS float *)(meta_len + META);
  LDS float *meta_lb = meta_start + META;  // lower bound on the score of any point of the list
  LDS float *sthr = meta_lb + META;  // [M]
  LDS float *sthr_in = sthr + IVFPQ_MAX_M;
  LDS float *srmin = sthr_in + IVFPQ_MAX_M;    // [M] smallest value of each table row
  LDS float *srabs = srmin + IVFPQ_MAX_M;      // [M] largest magnitude of each table row
  LDS float *ssuf = srabs + IVFPQ_MAX_M;       // [M/8 + 2] suffix sums of srmin at the check points, then sum srabs

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int64_t q = blockIdx.x / a.nsplit;
  const int split = blockIdx.x % a.nsplit;
  const int p_begin = (int)((int64_t)a.nprobe * split / a.nsplit);
  const int p_end = (int)((int64_t)a.nprobe * (split + 1) / a.nsplit);
  const int32_t *probes = a.probe_ids + q * a.probe_stride;
  const int mode = a.mode;

  int64_t dump_pos = 0;
  if (DUMP) {
    int64_t total = 0;
    for (int p = 0; p < a.nprobe; ++p) {
      const int32_t c = probes[p];
      if ((uint32_t)c < (uint32_t)a.nlist) total += a.list_offsets[c + 1] - a.list_offsets[c];
    }
    if (total != a.cand_offsets[q + 1] - a.cand_offsets[q]) {
      if (tid == 0) atomicAdd(a.errors, 1);
      return;
    }
    dump_pos = a.cand_offsets[q];
  }

  for (int i = tid; i < D; i += NT) sq[i] = a.queries[q * D + i];
  if (tid <= NW) tau_words[tid] = SENT_D;
  __syncthreads();
  for (int m = tid; m < M; m += NT) {
    float v = r2.v[m];
    if (a.query_radii) {
      const float r = a.query_radii[q * M + m];
      v = r * r;
    }
    float thr, thr_in;
    ip_thresholds(sq + m * dsub, dsub, v, thr, thr_in);
    sthr[m] = thr;
    sthr_in[m] = thr_in;
  }
  SharedTau sh;
  sh.bound = tau_words;
  sh.rank = tau_words + 1;
  sh.nw = NW;
  sh.wave = wave;
  sh.jrank = (a.k + NW - 1) / NW;
  sh.wide = nullptr;  // the inner-product scan produces k above KP pass by pass
  sh.wide_d = nullptr;
  sh.wide_id = nullptr;
  sh.wide_cap = 0;
  WaveTop st;
  init_wave_top<true, DUMP>(st, a, q);
  LDS uint32_t *qd = queue_d + wave * 64;
  LDS int64_t *qid = queue_id + wave * 64;
  __syncthreads();
  // ---- the query's table, built once ----
  {
    const int e = tid & 255;
    for (int m = tid >> 8; m < M; m += NT >> 8) {
      const int mu = __builtin_amdgcn_readfirstlane(m);
      const float ip = entry_ip(sq + mu * dsub, a.codebooks + ((int64_t)mu * 256 + e) * dsub, dsub);
      lut[mu * 256 + e] = table_value_ip(ip, sthr[mu], sthr_in[mu], mode);
    }
  }
  // ---- row minima and magnitudes for the early exit (one row per wavefront and pass) ----
  if constexpr (MT > 0 && !DUMP) {
    __syncthreads();
    for (int m = wave; m < M; m += NW) {
      const floatx4 v = *(const LDS floatx4 *)(lut + m * 256 + 4 * lane);
      float lo = fminf(fminf(v[0], v[1]), fminf(v[2], v[3]));
      float hi = fmaxf(fmaxf(fabsf(v[0]), fabsf(v[1])), fmaxf(fabsf(v[2]), fabsf(v[3])));
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) {
        lo = fminf(lo, __shfl_xor(lo, off));
        hi = fmaxf(hi, __shfl_xor(hi, off));
      }
      if (lane == 0) {
        srmin[m] = lo;
        srabs[m] = hi;
      }
    }
    __syncthreads();
    if (tid == 0) {
      float acc = 0.0f, mag = 0.0f;
      for (int m = M - 1; m >= 0; --m) {
        acc += srmin[m];
        mag += srabs[m];
        if ((m & 7) == 0) ssuf[m >> 3] = acc;
      }
      ssuf[(M + 7) / 8] = mag;
    }
  }
  // ---- the probed lists, META at a time ----
  for (int p0 = p_begin; p0 < p_end; p0 += META) {
    __syncthreads();  // table written; nobody still reads the previous metadata
    if (tid < META && p0 + tid < p_end) {
      const int32_t cc = probes[p0 + tid];
      const bool ok = (uint32_t)cc < (uint32_t)a.nlist;
      const int64_t r0 = ok ? a.list_offsets[cc] : 0;
      meta_row0[tid] = r0;
      meta_len[tid] = ok ? (int)(a.list_offsets[cc + 1] - r0) : 0;  // outside [0, nlist): an empty list
      meta_blk[tid] = ok ? a.list_blocks[cc] : 0;
      meta_start[tid] = (ok && mode == 0) ? neg_ip_chain(sq, a.centroids + (int64_t)cc * D, D) : 0.0f;
    }
    __syncthreads();
    const int pn = p_end - p0 < META ? p_end - p0 : META;
    // List-level bound (distance scoring; a wavefront per list, a lane per subspace).  Every
    // point of the list uses, in subspace m, an entry inside the list's box, so its inner
    // product with q_m is at most u_m = sum_j max(q_j lo_j, q_j hi_j) and its table value
    // 0 - max(IP, thr_m) at least 0 - max(u_m, thr_m).  The margins cover the roundings of u_m
    // and of the table's inner product (dsub products each), of the sum below, and of the
    // scan's own sum (the slack of adc_ip_exit).
    if constexpr (MT > 0 && !DUMP) {
      const bool bound_on = mode == 0 && !(a.ablate & (64 | 8));
      for (int pm = wave; pm < pn; pm += NW) {
        const int32_t cc = probes[p0 + pm];
        float lbv = -__builtin_inff();
        if (bound_on && (uint32_t)cc < (uint32_t)a.nlist) {
          const float *bx = a.list_box + (int64_t)cc * D * 2;
          const float eps_m = (float)(2 * dsub + 4) * 5.9604645e-08f;
          float acc = 0.0f, amag = 0.0f;
          for (int m = lane; m < M; m += 64) {
            float u = 0.0f, mag = 0.0f;
            for (int j = 0; j < dsub; ++j) {
              const float qj = sq[m * dsub + j], lo = bx[m * 2 * dsub + j], hi = bx[m * 2 * dsub + dsub + j];
              u += fmaxf(qj * lo, qj * hi);
              mag += fabsf(qj) * fmaxf(fabsf(lo), fabsf(hi));
            }
            const float thr = sthr[m];
            const float t = fmaxf(u, thr) + eps_m * (mag + fabsf(thr));
            acc += t;
            amag += fabsf(t);
          }
#pragma unroll
          for (int off = 32; off > 0; off >>= 1) {
            acc += __shfl_xor(acc, off);
            amag += __shfl_xor(amag, off);
          }
          const float start_l = meta_start[pm];
          const float eps_s = 5.9604645e-08f * (fabsf(start_l) + amag + ssuf[(M + 7) / 8]);
          lbv = (start_l - acc) - (float)(5 * M + 80) * eps_s;
        }
        if (lane == 0) meta_lb[pm] = lbv;
      }
      __syncthreads();
    }
    for (int pm = 0; pm < pn; ++pm) {
      const int64_t row0 = meta_row0[pm];
      const int len = __builtin_amdgcn_readfirstlane(meta_len[pm]);
      const int nb = (len + 63) >> 6;
      const uint8_t *base = a.codes + meta_blk[pm] * ivfpq_block_bytes(Mp);
      const float start = meta_start[pm];
      if constexpr (MT > 0 && !DUMP) {  // ruled out by the list-level bound: nothing of the list is requested
        const uint32_t shared0 = *(volatile LDS uint32_t *)sh.bound;
        const uint32_t pref0 = shared0 < st.tau.d ? shared0 : st.tau.d;
        if (dist_key<true>(meta_lb[pm]) > pref0) continue;
      }
      if constexpr (MT > 0) {
        if (wave < nb) {
          const int last = nb - 1;
          const float slack = (float)(4 * MT + 8) * 5.9604645e-08f * (fabsf(start) + ssuf[(MT + 7) / 8]);
          // as in the L2 kernel: only the first chunk (16 subspaces) of a block is fetched
          // ahead, the rest of the first half and the second half when a block needs them
          constexpr int NCH = MPT / 16 + (MPT % 16) / 4;
          constexpr int HCH = (MPT / 16 + 1) / 2;
          constexpr int MH = 16 * HCH;
          constexpr bool PARTS = !DUMP && HCH >= 2 && HCH < NCH && MH < MT;
          const bool ahead1 = PARTS && a.load_mode != 1;  // wave-uniform
          auto load_ahead = [&](int blk, CodeRegs<MPT / 4> &r) __attribute__((always_inline)) {
            load_chunks<MPT, 0, PARTS ? 1 : NCH>(base, nb, blk, lane, r);
            if constexpr (PARTS)
              if (!ahead1) load_chunks<MPT, 1, NCH>(base, nb, blk, lane, r);
          };
          CodeRegs<MPT / 4> nxt;
          load_ahead(wave, nxt);
          for (int b = wave; b < nb; b += NW) {
            CodeRegs<MPT / 4> cur = nxt;
            const int bn = b + NW < last ? b + NW : last;
            load_ahead(bn, nxt);
            const int i = b * 64 + lane;
            const bool valid = i < len;
            if (DUMP) {
              const float dist = adc_sum<MT>(lut, cur, start);
              if (valid) {
                a.all_dist[dump_pos + i] = dist;
                a.all_ids[dump_pos + i] = a.ids[row0 + i];
              }
            } else {
              const uint32_t shared = *(volatile LDS uint32_t *)sh.bound;
              const uint32_t pref = (a.ablate & 8) ? SENT_D : (shared < st.tau.d ? shared : st.tau.d);
              // no point of this list can reach the bound any more (it only tightens): the
              // wavefront is done with the list and requests no further blocks of it
              if (dist_key<true>(start + (ssuf[0] - slack)) > pref) break;
              float dist = start;
              if constexpr (PARTS) {
                if (!adc_ip_exit<MT, 0, 16>(lut, cur, pref, valid, ssuf, slack, dist)) continue;
                if (ahead1) load_chunks<MPT, 1, HCH>(base, nb, b, lane, cur);
                if (!adc_ip_exit<MT, 16, MH>(lut, cur, pref, valid, ssuf, slack, dist)) continue;
                if (ahead1) load_chunks<MPT, HCH, NCH>(base, nb, b, lane, cur);
                if (!adc_ip_exit<MT, MH, MT>(lut, cur, pref, valid, ssuf, slack, dist)) continue;
              } else {
                if (!adc_ip_exit<MT, 0, MT>(lut, cur, pref, valid, ssuf, slack, dist)) continue;
              }
              wave_offer<true>(st, dist, valid, row0 + i, a.ids, qd, qid, lane, a.k, sh);
            }
          }
        }
      } else {
        for (int b = wave; b < nb; b += NW) {
          const float dist = adc_sum_rt(lut, base, nb, b, lane, M, Mp, start);
          const int i = b * 64 + lane;
          const bool valid = i < len;
          if (DUMP) {
            if (valid) {
              a.all_dist[dump_pos + i] = dist;
              a.all_ids[dump_pos + i] = a.ids[row0 + i];
            }
          } else {
            wave_offer<true>(st, dist, valid, row0 + i, a.ids, qd, qid, lane, a.k, sh);
          }
        }
      }
      if (DUMP) dump_pos += len;
    }
  }
  if (DUMP) return;
  finish_topk<NW, true>(st, qd, qid, lane, wave, sh, smem3, a, q, split);
}

// List-level lower bound for the L2 metric.  For every list and subspace the index holds
// the bounding box of the entries that the list's points use (list_box_kernel), so the
// squared distance from the residual projection to the entry of any point of the list is at
// least the squared distance to that box, and the point's table value is at least
// min(that, r_m^2).  out[q][p] is the sum over the subspaces, reduced by 2^-12 relative
// against the handful of roundings that separate this evaluation from the table's (the
// residual is the same fp32 value q - c the table uses).  For the hit-count scorings the bound
// of a subspace is the penalty that every such entry gets when the whole box lies outside the
// (inner) sphere, decided with the same margin.  One wavefront per BOUND_PAIRS (query, probe)
// pairs, lane = subspace.  zero[0 .. zero_n) is set to 0 by the same launch (the list-major
// scan's per-list counters).
constexpr int BOUND_PAIRS = 2;  // (query, probe) pairs per wavefront: their loads are issued together

__global__ __launch_bounds__(256) void probe_bound_kernel(const float *__restrict__ queries,
                                                          const int32_t *__restrict__ probe_ids,
                                                          const float *__restrict__ centroids,
                                                          const float *__restrict__ box,
                                                          const float *__restrict__ grid,
                                                          const float *__restrict__ grid_par, int D, int M, int dsub,
                                                          int nlist, int64_t total, int nprobe, RadiiSq r2,
                                                          const float *__restrict__ query_radii, int mode,
                                                          float *__restrict__ out, int32_t *__restrict__ zero,
                                                          int64_t zero_n) {
  const int lane = threadIdx.x & 63;
  // (on the side: clear the caller's counters, so that they need no launch of their own)
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < zero_n; i += (int64_t)gridDim.x * 256) zero[i] = 0;
  const int64_t qp0 = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * BOUND_PAIRS;
  if (qp0 >= total) return;
  int64_t qs[BOUND_PAIRS];
  int32_t cs[BOUND_PAIRS];
  bool ok[BOUND_PAIRS];
  float lb[BOUND_PAIRS];
#pragma unroll
  for (int i = 0; i < BOUND_PAIRS; ++i) {
    const int64_t qp = qp0 + i < total ? qp0 + i : total - 1;  // a clamped pair is computed and not stored
    qs[i] = qp / nprobe;
    cs[i] = probe_ids[qp];
    ok[i] = (uint32_t)cs[i] < (uint32_t)nlist;
    if (!ok[i]) cs[i] = 0;
    lb[i] = 0.0f;
  }
  for (int m = lane; m < M; m += 64) {
    float best[BOUND_PAIRS];
    if (dsub == 2) {  // a box is one 16-byte load: (low x, low y, high x, high y)
      float2 qv[BOUND_PAIRS], cv[BOUND_PAIRS];
      float4 v[BOUND_PAIRS];
#pragma unroll
      for (int i = 0; i < BOUND_PAIRS; ++i) {
        qv[i] = *reinterpret_cast<const float2 *>(queries + qs[i] * D + 2 * m);
        cv[i] = *reinterpret_cast<const float2 *>(centroids + (int64_t)cs[i] * D + 2 * m);
        v[i] = reinterpret_cast<const float4 *>(box + (int64_t)cs[i] * D * 2)[m];
      }
      float4 gp0 = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
      float2 gp1 = make_float2(0.0f, 0.0f);
      if (grid) {
        gp0 = reinterpret_cast<const float4 *>(grid_par)[2 * m];
        gp1 = reinterpret_cast<const float2 *>(grid_par)[4 * m + 2];
      }
#pragma unroll
      for (int i = 0; i < BOUND_PAIRS; ++i) {
        const float x0 = qv[i].x - cv[i].x, x1 = qv[i].y - cv[i].y;
        const float t0 = fmaxf(fmaxf(v[i].x - x0, x0 - v[i].z), 0.0f);
        const float t1 = fmaxf(fmaxf(v[i].y - x1, x1 - v[i].w), 0.0f);
        best[i] = fmaf(t1, t1, t0 * t0);
        if (grid) {
          // Second bound: every entry of the subspace (used by this list or not) lies in the
          // grid's rectangle.  Inside it, the cell of the residual projection holds a lower
          // bound on the squared distance to the nearest entry; outside, the projection p' onto
          // the rectangle satisfies |p - e|^2 >= |p - p'|^2 + |p' - e|^2 for every e in it.
          const float fx = fminf(fmaxf((x0 - gp0.x) * gp1.x, 0.0f), (float)(GRID_G - 1));
          const float fy = fminf(fmaxf((x1 - gp0.y) * gp1.y, 0.0f), (float)(GRID_G - 1));
          const float cell = grid[(int64_t)m * (GRID_G * GRID_G) + (int)fy * GRID_G + (int)fx];
          const float o0 = fmaxf(fmaxf(gp0.x - x0, x0 - gp0.z), 0.0f);
          const float o1 = fmaxf(fmaxf(gp0.y - x1, x1 - gp0.w), 0.0f);
          best[i] = fmaxf(best[i], cell + fmaf(o1, o1, o0 * o0));
        }
      }
    } else {
#pragma unroll
      for (int i = 0; i < BOUND_PAIRS; ++i) {
        const float *bx = box + (int64_t)cs[i] * D * 2 + (int64_t)m * 2 * dsub;  // this list's boxes: [M][2][dsub]
        float acc = 0.0f;
        for (int j = 0; j < dsub; ++j) {
          const int d = m * dsub + j;
          const float x = queries[qs[i] * D + d] - centroids[(int64_t)cs[i] * D + d];
          const float t = fmaxf(fmaxf(bx[j] - x, x - bx[dsub + j]), 0.0f);
          acc = fmaf(t, t, acc);
        }
        best[i] = acc;
      }
    }
#pragma unroll
    for (int i = 0; i < BOUND_PAIRS; ++i) {
      float rm2 = r2.v[m];
      if (query_radii) {
        const float r = query_radii[qs[i] * M + m];
        rm2 = r * r;
      }
      if (mode == 0) {
        lb[i] += fminf(best[i], rm2);
      } else {  // 1 per subspace whose box is outside the sphere; mode 2: 2, and 1 if only outside the inner sphere
        const float b = best[i] * 0.999755859375f;
        lb[i] += b > rm2 ? (mode == 1 ? 1.0f : 2.0f) : ((mode == 2 && b > 0.25f * rm2) ? 1.0f : 0.0f);
      }
    }
  }
#pragma unroll
  for (int i = 0; i < BOUND_PAIRS; ++i) {
    float v = lb[i];
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    if (lane == 0 && qp0 + i < total)
      out[qp0 + i] = !ok[i] ? 0.0f : (mode == 0 ? v * 0.999755859375f : v);  // the counts are exact
  }
}

// ---------------------------------------------------------------------------
// Wide selection, second step: the keys a query's workgroup kept (all within its final
// bound on the k-th distance, plus those the bound overtook after they were stored) are
// filtered by that bound, given their ids, sorted by (distance, id) in LDS and the first k
// written out.
// A query whose slots overflowed, or that has more than WIDE_SORT keys within the bound
// (long runs of equal distances), gets map[q] = 0 and is served pass by pass afterwards;
// every other query gets map[q] = -1.
constexpr int WIDE_SORT = 2048;

__global__ __launch_bounds__(256) void wide_select_kernel(const uint32_t *__restrict__ wd, const int64_t *__restrict__ wid,
                                                          const int32_t *__restrict__ wn,
                                                          const uint32_t *__restrict__ wbound,
                                                          const int64_t *__restrict__ ids, int cap, int k,
                                                          int64_t *__restrict__ out_ids, float *__restrict__ out_dist,
                                                          int32_t *__restrict__ map) {
  __shared__ uint32_t sd[WIDE_SORT];
  __shared__ int64_t sid[WIDE_SORT];
  __shared__ uint32_t cnt;
  const int tid = threadIdx.x;
  const int64_t q = blockIdx.x;
  const int n = wn[q];
  if (n < 0) {
    if (tid == 0) map[q] = 0;
    return;
  }
  const uint32_t bound = wbound[q];
  if (tid == 0) cnt = 0u;
  __syncthreads();
  const uint32_t *d = wd + q * cap;
  const int64_t *id = wid + q * cap;
  for (int i = tid; i < n; i += 256) {
    const uint32_t v = d[i];
    if (v <= bound) {
      const uint32_t slot = __hip_atomic_fetch_add(&cnt, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      if (slot < (uint32_t)WIDE_SORT) {
        sd[slot] = v;
        sid[slot] = ids[id[i]];  // the slots hold rows
      }
    }
  }
  __syncthreads();
  const int m = (int)cnt;
  if (m > WIDE_SORT) {
    if (tid == 0) map[q] = 0;
    return;
  }
  if (tid == 0) map[q] = -1;
  int P = 2;
  while (P < m) P <<= 1;
  for (int i = m + tid; i < P; i += 256) {
    sd[i] = SENT_D;
    sid[i] = SENT_ID;
  }
  __syncthreads();
  for (int k2 = 2; k2 <= P; k2 <<= 1) {
    for (int j = k2 >> 1; j > 0; j >>= 1) {
      for (int t = tid; t < (P >> 1); t += 256) {
        const int lo = ((t & ~(j - 1)) << 1) | (t & (j - 1)), hi = lo | j;
        const uint32_t a0 = sd[lo], a1 = sd[hi];
        const bool greater = a0 != a1 ? a0 > a1 : sid[lo] > sid[hi];
        const bool asc = (lo & k2) == 0;  // direction of this pair's run
        if (greater == asc) {
          const int64_t i0 = sid[lo], i1 = sid[hi];
          sd[lo] = a1;
          sd[hi] = a0;
          sid[lo] = i1;
          sid[hi] = i0;
        }
      }
      __syncthreads();
    }
  }
  for (int i = tid; i < k; i += 256) {
    const bool real = i < m;
    out_ids[q * k + i] = real ? sid[i] : -1;
    out_dist[q * k + i] = real ? key_dist<false>(sd[i]) : __builtin_inff();
  }
}


// Merge the probe groups' partial lists of a query (one wavefront per query).
__global__ __launch_bounds__(64) void merge_kernel(const uint32_t *__restrict__ part_d,
                                                   const int64_t *__restrict__ part_id, int nsplit,
                                                   int k, int k_out, int k_off, int sgn,
                                                   int64_t *__restrict__ out_ids,
                                                   float *__restrict__ out_dist) {
  const int lane = threadIdx.x;
  const int64_t q = blockIdx.x;
  const int64_t o = q * nsplit * KP;
  Key L0, L1;
  L0.d = part_d[o + lane];
  L0.id = part_id[o + lane];
  L1.d = part_d[o + 64 + lane];
  L1.id = part_id[o + 64 + lane];
  for (int s = 1; s < nsplit; ++s)
    for (int h = 0; h < 2; ++h) {
      Key qk;
      qk.d = part_d[o + s * KP + h * 64 + (63 - lane)];
      qk.id = part_id[o + s * KP + h * 64 + (63 - lane)];
      wave_merge<true>(L0, L1, qk, lane);
    }
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const Key e = h ? L1 : L0;
    const int i = h * 64 + lane;
    if (i < k) {
      const bool real = e.d != SENT_D;
      out_ids[q * k_out + k_off + i] = real ? e.id : -1;
      out_dist[q * k_out + k_off + i] = real ? (sgn ? key_dist<true>(e.d) : key_dist<false>(e.d)) : __builtin_inff();
    }
  }
}

// Stand-alone table construction (same entry routine as the fused kernel).
// One workgroup of 256 threads per (query, probe): thread e handles entry e.
template <int DSUB>
__global__ __launch_bounds__(256) void lut_kernel(const float *__restrict__ queries,
                                                  const int32_t *__restrict__ probe_ids,
                                                  const float *__restrict__ centroids,
                                                  const float *__restrict__ codebooks, int D, int M,
                                                  int dsub_rt, int nlist, int nprobe, RadiiSq r2,
                                                  const float *__restrict__ query_radii, int mode, int ip,
                                                  float *__restrict__ out_lut,
                                                  uint64_t *__restrict__ out_mask) {
  extern __shared__ float sqv[];
  const int dsub = DSUB > 0 ? DSUB : dsub_rt;
  const int e = threadIdx.x, lane = e & 63, wave = e >> 6;
  const int64_t qp = blockIdx.x;
  const int64_t q = qp / nprobe;
  const int32_t c = probe_ids[qp];
  if ((uint32_t)c >= (uint32_t)nlist) return;  // uniform
  for (int i = e; i < D; i += 256) sqv[i] = queries[q * D + i];
  __syncthreads();
  const float *cen = centroids + (int64_t)c * D;
  for (int m = 0; m < M; ++m) {
    bool keep;
    float rm2 = r2.v[m];
    if (query_radii) {
      const float r = query_radii[q * M + m];
      rm2 = r * r;
    }
    float v;
    if (ip) {  // inner-product metric: the table of the query (the list does not enter)
      float thr, thr_in;
      ip_thresholds(sqv + m * dsub, dsub, rm2, thr, thr_in);
      const float x = entry_ip(sqv + m * dsub, codebooks + ((int64_t)m * 256 + e) * dsub, dsub);
      keep = x >= thr;
      v = table_value_ip(x, thr, thr_in, mode);
    } else {
      v = lut_entry<DSUB>(sqv + m * dsub, cen + m * dsub, codebooks + ((int64_t)m * 256 + e) * dsub, dsub,
                          rm2, mode, keep);
    }
    out_lut[(qp * M + m) * 256 + e] = v;
    const unsigned long long bal = __ballot(keep);
    if (out_mask && lane == 0) out_mask[(qp * M + m) * 4 + wave] = bal;
  }
}

// Index build: for every list and subspace the bounding box of the entries that the list's
// points use, box[c][m] = (low corner [dsub], high corner [dsub]).  One workgroup per list,
// thread = (slice of the list's points, subspace); the slices are combined through LDS.
__global__ __launch_bounds__(256) void list_box_kernel(const uint8_t *__restrict__ rows,
                                                       const int64_t *__restrict__ list_offsets,
                                                       const float *__restrict__ codebooks, int M, int dsub,
                                                       float *__restrict__ box) {
  extern __shared__ float sred[];  // [slices][M][2 * dsub]
  const int c = blockIdx.x;
  const int64_t r0 = list_offsets[c], n = list_offsets[c + 1] - r0;
  if (n <= 0) return;  // keeps the zero box
  const int slices = 256 / M >= 4 ? 4 : (256 / M > 0 ? 256 / M : 1);
  const int sl = threadIdx.x / M, m = threadIdx.x % M;
  const int w = 2 * dsub;
  if (sl < slices) {
    float *mine = sred + ((size_t)sl * M + m) * w;
    for (int j = 0; j < dsub; ++j) {
      mine[j] = __builtin_inff();
      mine[dsub + j] = -__builtin_inff();
    }
    for (int64_t i = sl; i < n; i += slices) {
      const int code = rows[(r0 + i) * M + m];
      const float *e = codebooks + ((int64_t)m * 256 + code) * dsub;
      for (int j = 0; j < dsub; ++j) {
        mine[j] = fminf(mine[j], e[j]);
        mine[dsub + j] = fmaxf(mine[dsub + j], e[j]);
      }
    }
  }
  __syncthreads();
  if (sl == 0) {
    float *out = box + ((int64_t)c * M + m) * w;
    for (int j = 0; j < dsub; ++j) {
      float lo = __builtin_inff(), hi = -__builtin_inff();
      for (int s2 = 0; s2 < slices; ++s2) {
        if (s2 < n) {  // a slice beyond the list's length saw no point
          lo = fminf(lo, sred[((size_t)s2 * M + m) * w + j]);
          hi = fmaxf(hi, sred[((size_t)s2 * M + m) * w + dsub + j]);
        }
      }
      out[j] = lo;
      out[dsub + j] = hi;
    }
  }
}

// Index build: raw rows [N][M] -> 64-point blocks, chunk-major within each list
// (one wavefront per block).
__global__ __launch_bounds__(256) void relayout_kernel(const uint8_t *__restrict__ rows,
                                                       const int64_t *__restrict__ list_offsets,
                                                       const int64_t *__restrict__ list_blocks,
                                                       int nlist, int M, int Mp, int64_t total_blocks,
                                                       uint8_t *__restrict__ out) {
  const int lane = threadIdx.x & 63;
  const int64_t B = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (B >= total_blocks) return;
  int lo = 0, hi = nlist;  // largest c with list_blocks[c] <= B (skips empty lists)
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (list_blocks[mid] <= B) lo = mid; else hi = mid;
  }
  const int c = lo;
  const int64_t b = B - list_blocks[c];
  const int64_t nb = list_blocks[c + 1] - list_blocks[c];
  const int64_t i = b * 64 + lane;
  const bool valid = i < list_offsets[c + 1] - list_offsets[c];
  const uint8_t *src = rows + (list_offsets[c] + i) * M;
  uint8_t *list_base = out + list_blocks[c] * ivfpq_block_bytes(Mp);
  const int n16 = Mp >> 4;
  for (int d = 0; d < (Mp >> 2); ++d) {
    uint32_t w = 0;
    if (valid)
      for (int bb = 0; bb < 4; ++bb)
        if (4 * d + bb < M) w |= (uint32_t)src[4 * d + bb] << (8 * bb);
    uint8_t *p = d < 4 * n16 ? list_base + ((int64_t)(d >> 2) * nb + b) * 1024 + lane * 16 + (d & 3) * 4
                             : list_base + (int64_t)n16 * nb * 1024 + ((int64_t)(d - 4 * n16) * nb + b) * 256 + lane * 4;
    *reinterpret_cast<uint32_t *>(p) = w;
  }
}

// Index build, two-dimensional subspaces: one workgroup per subspace lays a GRID_G x GRID_G
// grid over the bounding rectangle of the subspace's 256 entries (one cell of margin all
// round) and stores, per cell, min over the entries of the squared distance from the entry to
// the cell -- the cell enlarged by 1/256 of its size on every side, so that a point whose cell
// index is off by a rounding is still covered.  par[m] = (low x, low y, high x, high y,
// cells per unit x, cells per unit y, 0, 0).
__global__ __launch_bounds__(256) void codebook_grid_kernel(const float *__restrict__ codebooks, float *__restrict__ grid,
                                                            float *__restrict__ par) {
  __shared__ float ex[256], ey[256];
  __shared__ float red[4][4];
  const int m = blockIdx.x, tid = threadIdx.x;
  const float x = codebooks[((int64_t)m * 256 + tid) * 2], y = codebooks[((int64_t)m * 256 + tid) * 2 + 1];
  ex[tid] = x;
  ey[tid] = y;
  float lox = x, hix = x, loy = y, hiy = y;
  for (int off = 32; off > 0; off >>= 1) {
    lox = fminf(lox, __shfl_xor(lox, off));
    hix = fmaxf(hix, __shfl_xor(hix, off));
    loy = fminf(loy, __shfl_xor(loy, off));
    hiy = fmaxf(hiy, __shfl_xor(hiy, off));
  }
  if ((tid & 63) == 0) {
    red[tid >> 6][0] = lox;
    red[tid >> 6][1] = hix;
    red[tid >> 6][2] = loy;
    red[tid >> 6][3] = hiy;
  }
  __syncthreads();
  lox = fminf(fminf(red[0][0], red[1][0]), fminf(red[2][0], red[3][0]));
  hix = fmaxf(fmaxf(red[0][1], red[1][1]), fmaxf(red[2][1], red[3][1]));
  loy = fminf(fminf(red[0][2], red[1][2]), fminf(red[2][2], red[3][2]));
  hiy = fmaxf(fmaxf(red[0][3], red[1][3]), fmaxf(red[2][3], red[3][3]));
  // a degenerate extent (all entries equal in a coordinate) gets an arbitrary positive one
  float wx = hix - lox, wy = hiy - loy;
  if (!(wx > 0.0f)) wx = 1.0f;
  if (!(wy > 0.0f)) wy = 1.0f;
  const float cx = wx / (float)(GRID_G - 2), cy = wy / (float)(GRID_G - 2);   // cell size: the entries span G - 2 cells
  const float gx0 = lox - cx, gy0 = loy - cy;
  const float gx1 = gx0 + cx * (float)GRID_G, gy1 = gy0 + cy * (float)GRID_G;
  if (tid == 0) {
    float *o = par + (int64_t)m * 8;
    o[0] = gx0;
    o[1] = gy0;
    o[2] = fmaxf(gx1, hix);   // the rectangle must hold every entry whatever the sums above round to
    o[3] = fmaxf(gy1, hiy);
    o[4] = 1.0f / cx;
    o[5] = 1.0f / cy;
    o[6] = o[7] = 0.0f;
  }
  for (int c = tid; c < GRID_G * GRID_G; c += 256) {
    const int ix = c % GRID_G, iy = c / GRID_G;
    const float eps = 1.0f / 256.0f;
    const float ax = gx0 + cx * ((float)ix - eps), bx = gx0 + cx * ((float)(ix + 1) + eps);
    const float ay = gy0 + cy * ((float)iy - eps), by = gy0 + cy * ((float)(iy + 1) + eps);
    float best = __builtin_inff();
    for (int e = 0; e < 256; ++e) {
      const float dx = fmaxf(fmaxf(ax - ex[e], ex[e] - bx), 0.0f), dy = fmaxf(fmaxf(ay - ey[e], ey[e] - by), 0.0f);
      best = fminf(best, fmaf(dy, dy, dx * dx));
    }
    grid[(int64_t)m * (GRID_G * GRID_G) + c] = best;
  }
}

__global__ void iota_kernel(int64_t *d, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) d[i] = i;
}

__global__ void fill_i32_kernel(int32_t *d, int64_t n, int32_t v) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) d[i] = v;
}

// Tuning switches (ivfpq_set_option).  None of them changes a result.  Atomics: a setter may run
// on one host thread while another enqueues a search; a launch reads each switch once.
std::atomic<int> g_scan_waves{0};    // 0 = choose from the shape
std::atomic<int> g_scan_ablate{0};   // pruning switches: 8 | 32 | 64
std::atomic<int> g_bound_grid{0};    // list-level bound: 0 = the nearest-entry grid on long lists only, 1 = always, 2 = never
std::atomic<int> g_scan_variant{0};  // code loads: 0 = default (first chunk ahead while pruning), 1 = always whole blocks, 2 = always the first half ahead, 3 = always the first chunk ahead

template <int MT, int DSUB, int NW, bool BYTE = false>
int launch_scan_t(const ScanArgs &a, const RadiiSq &r2, int64_t grid, bool dump, hipStream_t s) {
  const int lut_bytes = a.M * (BYTE ? 256 : 1024), stage = NW * KP * 12;
  const size_t lds = (size_t)(lut_bytes > stage ? lut_bytes : stage) + 2 * ((a.D * 4 + 15) & ~15) +
                     (size_t)NW * 64 * 12 + ((4 * (2 * NW + 4) + 15) & ~15) + 64 * 28 + 5 * IVFPQ_MAX_M * 4 +
                     (size_t)NW * SUF_SLOTS * 4 + 16;
  if (lds > (size_t)LDS_PER_CU) {
    ivfpq::set_error("scan: %zu bytes of LDS needed, 163840 available", lds);
    return IVFPQ_ERR_UNSUPPORTED;
  }
  auto kern = dump ? scan_kernel<MT, DSUB, NW, true, BYTE> : scan_kernel<MT, DSUB, NW, false, BYTE>;
  static std::atomic<uint64_t> prepared[2];
  if (int rc = prepare_kernel(kern, prepared[dump ? 1 : 0])) return rc;
  hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(NW * 64), lds, s, a, r2);
  return IVFPQ_OK;
}

template <int MT, int DSUB>
int launch_scan_nw(const ScanArgs &a, const RadiiSq &r2, int64_t grid, bool dump, hipStream_t s) {
  int nw = g_scan_waves.load(std::memory_order_relaxed);
  // One workgroup per CU once the table passes 72 KiB: the specialised kernels then run 8
  // wavefronts with twice the registers, the run-time-M kernel (few registers) runs 16.
  // Tables of at most 32 KiB leave room for four workgroups per CU: 4 wavefronts each, so that
  // a workgroup's serial phases (table, barriers, final merge) overlap with three others'.
  // hit-count scorings on a specialised shape: the byte table (8 wavefronts, whatever M)
  if (MT > 0 && a.mode != 0 && !(a.ablate & 128) && (nw == 0 || nw == 8)) return launch_scan_t<MT, DSUB, 8, true>(a, r2, grid, dump, s);
  if (nw == 0) nw = (MT == 0 && a.M > 72) ? 16 : (a.M <= 32 ? 4 : 8);
  if (a.wide_cap > 0 && nw * KP < a.k_out) nw = 8;  // the bound takes ceil(k_out / nw) <= KP keys of every wavefront
  if (nw >= 16) return launch_scan_t<MT, DSUB, 16>(a, r2, grid, dump, s);
  if (nw >= 8) return launch_scan_t<MT, DSUB, 8>(a, r2, grid, dump, s);
  return launch_scan_t<MT, DSUB, 4>(a, r2, grid, dump, s);
}

size_t scan_ip_lds(const ScanArgs &a, int nw) {
  const int lut_bytes = a.M * 1024, stage = nw * KP * 12;
  return (size_t)(lut_bytes > stage ? lut_bytes : stage) + ((a.D * 4 + 15) & ~15) + (size_t)nw * 64 * 12 +
         ((4 * (nw + 1) + 15) & ~15) + 64 * 28 + 4 * IVFPQ_MAX_M * 4 + (IVFPQ_MAX_M / 8 + 2) * 4;
}

template <int MT, int NW>
int launch_scan_ip_t(const ScanArgs &a, const RadiiSq &r2, int64_t grid, bool dump, hipStream_t s) {
  const size_t lds = scan_ip_lds(a, NW);
  if (lds > (size_t)LDS_PER_CU) {
    ivfpq::set_error("scan: %zu bytes of LDS needed, 163840 available", lds);
    return IVFPQ_ERR_UNSUPPORTED;
  }
  auto kern = dump ? scan_ip_kernel<MT, NW, true> : scan_ip_kernel<MT, NW, false>;
  static std::atomic<uint64_t> prepared[2];
  if (int rc = prepare_kernel(kern, prepared[dump ? 1 : 0])) return rc;
  hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(NW * 64), lds, s, a, r2);
  return IVFPQ_OK;
}

// Inner-product metric: 8 wavefronts while two workgroups fit a CU, else 16.
template <int MT>
int launch_scan_ip(const ScanArgs &a, const RadiiSq &r2, int64_t grid, bool dump, hipStream_t s) {
  if (2 * scan_ip_lds(a, 8) <= (size_t)LDS_PER_CU) return launch_scan_ip_t<MT, 8>(a, r2, grid, dump, s);
  return launch_scan_ip_t<MT, 16>(a, r2, grid, dump, s);
}

}  // namespace

namespace ivfpq {

void set_scan_waves(int nw) { g_scan_waves.store(nw, std::memory_order_relaxed); }
void set_bound_grid(int v) { g_bound_grid.store(v, std::memory_order_relaxed); }
void set_scan_ablate(int bits) { g_scan_ablate.store(bits, std::memory_order_relaxed); }
void set_scan_variant(int v) { g_scan_variant.store(v, std::memory_order_relaxed); }
int get_scan_ablate() { return g_scan_ablate.load(std::memory_order_relaxed); }

int launch_scan(const ivfpq_index *ix, const float *d_queries, int64_t Q, int32_t nprobe,
                const int32_t *d_probe_ids, int32_t k, const RadiiSq &r2, int32_t nsplit,
                uint32_t *d_part_d, int64_t *d_part_id, int64_t *d_out_ids, float *d_out_dist,
                const int64_t *d_cand_offsets, float *d_all_dist, int64_t *d_all_ids,
                int32_t *d_errors, int32_t mode, const float *d_query_radii, float *d_probe_lb,
                hipStream_t s, const ScanView *view) {
  ScanArgs a;
  a.queries = d_queries;
  a.probe_ids = d_probe_ids;
  a.centroids = ix->d_centroids;
  a.codebooks = ix->d_codebooks;
  a.probe_lb = nullptr;
  a.qmap = view ? view->qmap : nullptr;
  a.probe_stride = (view && view->probe_stride > 0) ? view->probe_stride : nprobe;
  a.list_box = ix->d_box;
  a.list_offsets = ix->d_list_offsets;
  a.list_blocks = ix->d_list_blocks;
  a.codes = ix->d_codes;
  a.ids = ix->d_ids;
  a.out_ids = d_out_ids;
  a.out_dist = d_out_dist;
  a.part_d = d_part_d;
  a.part_id = d_part_id;
  a.cand_offsets = d_cand_offsets;
  a.all_dist = d_all_dist;
  a.all_ids = d_all_ids;
  a.errors = d_errors;
  a.D = ix->D;
  a.M = ix->M;
  a.dsub = ix->dsub;
  a.Mp = ix->Mp;
  a.nlist = ix->nlist;
  a.nprobe = nprobe;
  a.nsplit = nsplit;
  a.ablate = g_scan_ablate.load(std::memory_order_relaxed);
  a.mode = mode;
  a.query_radii = d_query_radii;
  a.load_mode = g_scan_variant.load(std::memory_order_relaxed);
  a.wide_d = nullptr;
  a.wide_id = nullptr;
  a.wide_n = nullptr;
  a.wide_bound = nullptr;
  a.wide_cap = 0;
  const bool dump = d_all_dist != nullptr;
  const int64_t grid = Q * nsplit;
  if (grid > 0x7FFFFFFFll) {
    set_error("scan: %lld workgroups exceed the grid limit", (long long)grid);
    return IVFPQ_ERR_UNSUPPORTED;
  }
  const int M = ix->M, ds = ix->dsub;
  const bool ip = ix->metric == IVFPQ_METRIC_IP;
  if (d_probe_lb && !dump && !ip && !(a.ablate & 64)) {
    if (!(view && view->bounds_ready))
      if (int rc = launch_probe_bounds(ix, d_queries, Q, nprobe, d_probe_ids, r2, mode, d_query_radii, d_probe_lb, s))
        return rc;
    a.probe_lb = d_probe_lb;
  }
  auto dispatch = [&](const ScanArgs &x, int64_t g) -> int {
    if (ip) {
      if (M == 64) return launch_scan_ip<64>(x, r2, g, dump, s);
      if (M == 48) return launch_scan_ip<48>(x, r2, g, dump, s);
      if (M == 100) return launch_scan_ip<100>(x, r2, g, dump, s);
      if (M == 16) return launch_scan_ip<16>(x, r2, g, dump, s);
      return launch_scan_ip<0>(x, r2, g, dump, s);
    }
    if (M == 64 && ds == 2) return launch_scan_nw<64, 2>(x, r2, g, dump, s);
    if (M == 48 && ds == 2) return launch_scan_nw<48, 2>(x, r2, g, dump, s);
    if (M == 100 && ds == 2) return launch_scan_nw<100, 2>(x, r2, g, dump, s);
    if (M == 16 && ds == 4) return launch_scan_nw<16, 4>(x, r2, g, dump, s);
    return launch_scan_nw<0, 0>(x, r2, g, dump, s);
  };
  a.k_out = k;
  // k above KP in one pass (wide selection): chunks of queries share the slot arrays; each
  // chunk is scanned once with every key within the bound kept, sorted by wide_select_kernel,
  // and the queries that kernel could not finish go through the passes below.
  const WideWorkspace *ww = view ? view->wide : nullptr;
  if (ww && ww->total > 0 && k > KP && k <= 8 * KP && !dump && !ip && mode == 0 && !a.qmap) {
    char *wb = view->wide_base;
    for (int64_t q0 = 0; q0 < Q; q0 += ww->q_chunk) {
      const int64_t qc = Q - q0 < ww->q_chunk ? Q - q0 : ww->q_chunk;
      ScanArgs c = a;
      c.queries = d_queries + q0 * ix->D;
      c.probe_ids = d_probe_ids + q0 * a.probe_stride;
      if (a.probe_lb) c.probe_lb = a.probe_lb + q0 * a.probe_stride;
      if (d_query_radii) c.query_radii = d_query_radii + q0 * ix->M;
      c.out_ids = d_out_ids + q0 * k;
      c.out_dist = d_out_dist + q0 * k;
      c.nsplit = 1;
      c.k = KP;
      c.k_off = 0;
      c.wide_d = reinterpret_cast<uint32_t *>(wb + ww->d);
      c.wide_id = reinterpret_cast<int64_t *>(wb + ww->id);
      c.wide_n = reinterpret_cast<int32_t *>(wb + ww->n);
      c.wide_bound = reinterpret_cast<uint32_t *>(wb + ww->bound);
      c.wide_cap = ww->cap;
      int32_t *map = reinterpret_cast<int32_t *>(wb + ww->qmap);
      if (int rc = dispatch(c, qc)) return rc;
      hipLaunchKernelGGL(wide_select_kernel, dim3((unsigned)qc), dim3(256), 0, s, c.wide_d, c.wide_id, c.wide_n,
                         c.wide_bound, ix->d_ids, ww->cap, k, c.out_ids, c.out_dist, map);
      ScanView rest;
      rest.probe_stride = a.probe_stride;
      rest.qmap = map;
      rest.bounds_ready = true;
      rest.wide = nullptr;
      rest.wide_base = nullptr;
      if (int rc = launch_scan(ix, c.queries, qc, nprobe, c.probe_ids, k, r2, 1, nullptr, nullptr, c.out_ids, c.out_dist,
                               nullptr, nullptr, nullptr, nullptr, mode, c.query_radii,
                               a.probe_lb ? d_probe_lb + q0 * a.probe_stride : nullptr, s, &rest))
        return rc;
    }
    IVFPQ_HIP_TRY(hipGetLastError());
    return IVFPQ_OK;
  }
  // A wavefront's sorted list holds KP keys, so k > KP takes ceil(k / KP) passes over the
  // lists; pass j keeps the keys above the last key pass j - 1 wrote.
  for (int32_t off = 0; off == 0 || off < k; off += KP) {
    a.k_off = off;
    a.k = k - off < KP ? k - off : KP;
    if (int rc = dispatch(a, grid)) return rc;
    if (dump) break;
    if (nsplit > 1)
      hipLaunchKernelGGL(merge_kernel, dim3((unsigned)Q), dim3(64), 0, s, d_part_d, d_part_id, nsplit, a.k,
                         a.k_out, a.k_off, (int)ip, d_out_ids, d_out_dist);
  }
  IVFPQ_HIP_TRY(hipGetLastError());
  return IVFPQ_OK;
}

int launch_probe_bounds(const ivfpq_index *ix, const float *d_queries, int64_t Q, int32_t nprobe,
                        const int32_t *d_probe_ids, const RadiiSq &r2, int32_t mode, const float *d_query_radii,
                        float *d_probe_lb, hipStream_t s, int32_t *d_zero, int64_t zero_n) {
  const int64_t total = Q * nprobe;
  if (total == 0) return zero_n > 0 ? launch_fill_i32(d_zero, zero_n, 0, s) : IVFPQ_OK;
  // The grid of nearest-entry distances tightens the bound (on the 100M-point configuration it
  // rules out 59.4 instead of 55.9 of a query's 64 lists, and the tables built per query drop
  // from 8.1 to 4.6) at the price of a slower bound kernel (three more loads per pair and
  // subspace, one of them a gather): it pays where a list that slips through is expensive,
  // i.e. on long lists (measured: 4 % faster there, 7-14 % slower on the 1M-point ones).
  const int grid_mode = g_bound_grid.load(std::memory_order_relaxed);
  const bool use_grid = ix->d_grid && grid_mode != 2 && (grid_mode == 1 || ix->N > (int64_t)4096 * ix->nlist);
  const int64_t per_block = 4 * BOUND_PAIRS;
  if ((total + per_block - 1) / per_block > 0x7FFFFFFFll) {
    set_error("scan: %lld (query, probe) pairs exceed the grid limit of the bound kernel", (long long)total);
    return IVFPQ_ERR_UNSUPPORTED;
  }
  hipLaunchKernelGGL(probe_bound_kernel, dim3((unsigned)((total + per_block - 1) / per_block)), dim3(256), 0, s,
                     d_queries, d_probe_ids, ix->d_centroids, ix->d_box,
                     use_grid ? ix->d_grid : nullptr, ix->d_grid_par, ix->D, ix->M, ix->dsub, ix->nlist, total,
                     nprobe, r2, d_query_radii, mode, d_probe_lb, d_zero, d_zero ? zero_n : 0);
  IVFPQ_HIP_TRY(hipGetLastError());
  return IVFPQ_OK;
}

int launch_build_lut(const ivfpq_index *ix, const float *d_queries, int64_t Q, int32_t nprobe,
                     const int32_t *d_probe_ids, const RadiiSq &r2, float *d_lut, uint64_t *d_mask,
                     int32_t mode, const float *d_query_radii, hipStream_t s) {
  const int64_t grid = Q * nprobe;
  if (grid > 0x7FFFFFFFll) {
    set_error("build_lut: %lld workgroups exceed the grid limit", (long long)grid);
    return IVFPQ_ERR_UNSUPPORTED;
  }
  const size_t lds = (size_t)ix->D * sizeof(float);
#define LUT_LAUNCH(DS)                                                                           \
  hipLaunchKernelGGL(lut_kernel<DS>, dim3((unsigned)grid), dim3(256), lds, s, d_queries,         \
                     d_probe_ids, ix->d_centroids, ix->d_codebooks, ix->D, ix->M, ix->dsub,      \
                     ix->nlist, nprobe, r2, d_query_radii, mode, (int)(ix->metric == IVFPQ_METRIC_IP), d_lut, \
                     d_mask)
  if (ix->dsub == 2) LUT_LAUNCH(2);
  else if (ix->dsub == 4) LUT_LAUNCH(4);
  else LUT_LAUNCH(0);
#undef LUT_LAUNCH
  IVFPQ_HIP_TRY(hipGetLastError());
  return IVFPQ_OK;
}

int launch_relayout(const ivfpq_index *ix, const uint8_t *d_rows, hipStream_t s) {
  if (ix->total_blocks == 0) return IVFPQ_OK;
  const int64_t grid = (ix->total_blocks + 3) / 4;
  hipLaunchKernelGGL(relayout_kernel, dim3((unsigned)grid), dim3(256), 0, s, d_rows, ix->d_list_offsets,
                     ix->d_list_blocks, ix->nlist, ix->M, ix->Mp, ix->total_blocks, ix->d_codes);
  IVFPQ_HIP_TRY(hipGetLastError());
  return IVFPQ_OK;
}

int launch_codebook_grid(const ivfpq_index *ix, hipStream_t s) {
  hipLaunchKernelGGL(codebook_grid_kernel, dim3((unsigned)ix->M), dim3(256), 0, s, ix->d_codebooks, ix->d_grid,
                     ix->d_grid_par);
  IVFPQ_HIP_TRY(hipGetLastError());
  return IVFPQ_OK;
}

int launch_list_boxes(const ivfpq_index *ix, const uint8_t *d_rows, hipStream_t s) {
  if (ix->N == 0) return IVFPQ_OK;
  const int slices = 256 / ix->M >= 4 ? 4 : (256 / ix->M > 0 ? 256 / ix->M : 1);
  const size_t lds = (size_t)slices * ix->D * 2 * sizeof(float);
  hipLaunchKernelGGL(list_box_kernel, dim3((unsigned)ix->nlist), dim3(256), lds, s, d_rows, ix->d_list_offsets,
                     ix->d_codebooks, ix->M, ix->dsub, ix->d_box);
  IVFPQ_HIP_TRY(hipGetLastError());
  return IVFPQ_OK;
}

int launch_fill_i32(int32_t *d, int64_t n, int32_t v, hipStream_t s) {
  if (n == 0) return IVFPQ_OK;
  hipLaunchKernelGGL(fill_i32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, d, n, v);
  IVFPQ_HIP_TRY(hipGetLastError());
  return IVFPQ_OK;
}

int launch_iota(int64_t *d, int64_t n, hipStream_t s) {
  if (n == 0) return IVFPQ_OK;
  hipLaunchKernelGGL(iota_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, d, n);
  IVFPQ_HIP_TRY(hipGetLastError());
  return IVFPQ_OK;
}

}  // namespace ivfpq
