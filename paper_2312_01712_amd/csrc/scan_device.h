// Device-side building blocks shared by the scan kernels (query-major scan in scan.hip,
// list-major scan in scan_lm.hip): (distance, id) keys and the cross-lane sorting network,
// per-wavefront top-k lists, table entries (paper Sec. 4.1, Algorithm 2), the interleaved code
// layout's loads and the byte-select look-up (paper Sec. 2.1 step D, Sec. 5.3).
// Everything here is inline device code; each translation unit gets its own copy.
#pragma once

#include <limits.h>

#include <atomic>
#include <type_traits>

#include "ivfpq_internal.h"

namespace {

// Pointers into LDS carry their address space in the type, so that every access
// is a DS instruction and no generic-pointer dispatch is ever generated.
#define LDS __attribute__((address_space(3)))
typedef float floatx4 __attribute__((ext_vector_type(4)));

// Wavefronts per SIMD the scan kernel is compiled for: 4 (two 8-wave workgroups per CU, 128
// vector registers each).  Tables of more than 72 KiB allow one workgroup per CU anyway;
// with at most 8 wavefronts in it each SIMD holds 2 and a wavefront may use 256 registers,
// enough to keep every codebook row it needs resident.
constexpr int scan_wpe(int mt, int nw) { return mt > 72 && nw <= 8 ? 2 : 4; }
// Vector registers a wavefront may devote to resident codebook rows ...
constexpr int res_regs(int wpe) { return wpe == 2 ? 112 : 48; }
// ... as long as they and the two code register sets stay under this.
constexpr int res_max_total(int wpe) { return wpe == 2 ? 200 : 82; }
constexpr int KP = 128;                    // capacity of a wavefront's sorted list
constexpr int cmin(int a, int b) { return a < b ? a : b; }
constexpr int SUF_SLOTS = IVFPQ_MAX_M / 8 + 4;  // floats per wavefront for the suffix sums of the row minima
constexpr int LOOKUP_GROUP = 8;            // table look-ups a wavefront keeps in flight
constexpr uint32_t SENT_D = 0xFFFFFFFFu;   // sentinel key: larger than any distance
constexpr int64_t SENT_ID = LLONG_MAX;

struct Key {
  uint32_t d;  // distance as an unsigned integer that orders like the value (see dist_key)
  int64_t id;
};

// Distances are >= 0 under L2 and for the hit counts, so their bits already order like
// the values.  Scores under the inner-product metric have either sign (SGN): the usual
// order-preserving map is applied (flip all bits of a negative, set the top bit of a
// non-negative), and undone on output.
template <bool SGN>
__device__ inline uint32_t dist_key(float v) {
  const uint32_t u = __float_as_uint(v);
  if (!SGN) return u;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
template <bool SGN>
__device__ inline float key_dist(uint32_t k) {
  if (!SGN) return __uint_as_float(k);
  return __uint_as_float((k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k);
}

__device__ inline bool kless(const Key &a, const Key &b) {
  return a.d < b.d || (a.d == b.d && a.id < b.id);
}

// Cross-lane helpers on the data-parallel-primitive path (no LDS traffic).  XOR1 / XOR2 swap
// lanes within a quad, QUAD_MIRROR reverses a quad, HALF_MIRROR reverses each group of 8
// lanes, ROR4 / ROR8 rotate each row of 16 lanes by 4 / 8.
constexpr int DPP_XOR1 = 0xB1, DPP_XOR2 = 0x4E, DPP_QUAD_MIRROR = 0x1B, DPP_HALF_MIRROR = 0x141, DPP_ROR4 = 0x124,
              DPP_ROR8 = 0x128;
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, CTRL, 0xF, 0xF, false);
}
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
  return __uint_as_float(dpp_u32<CTRL>(__float_as_uint(v)));
}

// The value of lane ^ J.  With DPP, J = 1, 2, 8 are one register-to-register move (8: a
// rotation by half a row of 16), J = 4 is two (reverse the group of 8, then reverse the quad:
// 7 ^ 3 = 4) and only J = 16 and 32 go through the LDS crossbar; a 64-key bitonic sort has 18
// of its 21 stages at J <= 8.  Measured: 2-3 % faster in the L2 kernels (C2, C3), 10 % slower in
// the 16-wavefront inner-product kernel (C4: 11.3 -> 12.4 ms), which therefore keeps the
// crossbar shuffles (DPP = false).
template <int J, bool DPP>
__device__ __forceinline__ uint32_t xor_u32(uint32_t v) {
  if constexpr (DPP && J == 1) return dpp_u32<DPP_XOR1>(v);
  else if constexpr (DPP && J == 2) return dpp_u32<DPP_XOR2>(v);
  else if constexpr (DPP && J == 4) return dpp_u32<DPP_QUAD_MIRROR>(dpp_u32<DPP_HALF_MIRROR>(v));
  else if constexpr (DPP && J == 8) return dpp_u32<DPP_ROR8>(v);
  else return (uint32_t)__shfl_xor((int)v, J);
}

template <int J, bool DPP>
__device__ __forceinline__ Key xor_key(const Key &a) {
  Key o;
  o.d = xor_u32<J, DPP>(a.d);
  const uint32_t lo = xor_u32<J, DPP>((uint32_t)a.id);
  const uint32_t hi = xor_u32<J, DPP>((uint32_t)((uint64_t)a.id >> 32));
  o.id = (int64_t)(((uint64_t)hi << 32) | lo);
  return o;
}

// compare-exchange with lane ^ J; this lane keeps the smaller key iff keep_small
template <int J, bool DPP>
__device__ __forceinline__ void cx_lane(Key &a, bool keep_small) {
  const Key o = xor_key<J, DPP>(a);
  const bool take = keep_small ? kless(o, a) : kless(a, o);
  if (take) a = o;
}

// the stages J, J/2, ..., 1 of one bitonic level; desc: this lane's block sorts descending
template <int J, bool DPP>
__device__ __forceinline__ void cx_cascade(Key &a, int lane, bool desc) {
  const bool lower = (lane & J) == 0;
  cx_lane<J, DPP>(a, desc ? !lower : lower);
  if constexpr (J > 1) cx_cascade<J / 2, DPP>(a, lane, desc);
}

template <int K2, bool DPP>
__device__ __forceinline__ void sort_levels_desc(Key &a, int lane) {
  cx_cascade<K2 / 2, DPP>(a, lane, (lane & K2) == 0 || K2 == 64);
  if constexpr (K2 < 64) sort_levels_desc<K2 * 2, DPP>(a, lane);
}

// Sort 64 keys (one per lane) in DESCENDING lane order.
template <bool DPP>
__device__ inline void wave_sort_desc(Key &a, int lane) { sort_levels_desc<2, DPP>(a, lane); }

// L0/L1 hold a sorted list of 128 keys (element i lives in lane i%64, register
// i/64).  qd holds 64 keys sorted descending by lane.  Afterwards L0/L1 hold the
// 128 smallest of the 192, sorted ascending.
template <bool DPP>
__device__ inline void wave_merge(Key &L0, Key &L1, const Key &qd, int lane) {
  // element 64+l against the l-th largest queued key: the 128 survivors form a
  // bitonic sequence
  if (kless(qd, L1)) L1 = qd;
  if (kless(L1, L0)) {
    const Key t = L0;
    L0 = L1;
    L1 = t;
  }
  cx_cascade<32, DPP>(L0, lane, false);
  cx_cascade<32, DPP>(L1, lane, false);
}

__device__ inline Key bcast_key(const Key &a, int src) {
  Key o;
  o.d = (uint32_t)__shfl((int)a.d, src);
  const int lo = __shfl((int)(uint32_t)a.id, src);
  const int hi = __shfl((int)(uint32_t)((uint64_t)a.id >> 32), src);
  o.id = (int64_t)(((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo);
  return o;
}

__device__ __forceinline__ uint32_t umin32(uint32_t a, uint32_t b) { return a < b ? a : b; }

// Minima of eight table rows at once.  lo[j] is this lane's minimum over its entries of row
// j (bit patterns of non-negative floats, which order like the values).  Three exchange
// steps halve the number of rows a lane carries while doubling the lanes a value covers
// (lane bit 0, 1, 2 select which row is kept), two more combine the groups of a row of 16
// lanes.  Afterwards lane l with (l & 15) < 8 holds the minimum of row (l & 7) over its 16
// lanes: 5 + 2 + 1 + 1 exchanges instead of 8 x 4.
__device__ __forceinline__ uint32_t rows8_min16(const uint32_t (&lo)[8], int lane) {
  const bool b0 = lane & 1, b1 = lane & 2, b2 = lane & 4;
  uint32_t a[4], c[2];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t keep = b0 ? lo[2 * i + 1] : lo[2 * i], send = b0 ? lo[2 * i] : lo[2 * i + 1];
    a[i] = umin32(keep, dpp_u32<DPP_XOR1>(send));        // row 2 i + b0 over a lane pair
  }
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const uint32_t keep = b1 ? a[2 * i + 1] : a[2 * i], send = b1 ? a[2 * i] : a[2 * i + 1];
    c[i] = umin32(keep, dpp_u32<DPP_XOR2>(send));        // row 4 i + 2 b1 + b0 over a quad
  }
  // a rotation by 4 within the 16 lanes pairs every lane with one whose bit 2 differs and
  // whose bits 0 and 1 agree; over the two lanes that end up with a row (l and l + 8) the
  // four quads of the 16 lanes are all covered
  const uint32_t keep = b2 ? c[1] : c[0], send = b2 ? c[0] : c[1];
  uint32_t d = umin32(keep, dpp_u32<DPP_ROR4>(send));    // row 4 b2 + 2 b1 + b0 over two quads
  d = umin32(d, dpp_u32<DPP_ROR8>(d));                   // ... over the 16 lanes
  return d;
}

// Sum over each group of 8 consecutive lanes, left in every lane of the group.
__device__ __forceinline__ float group8_sum(float v) {
  v += dpp_f32<DPP_XOR1>(v);
  v += dpp_f32<DPP_XOR2>(v);
  v += dpp_f32<DPP_HALF_MIRROR>(v);
  return v;
}

// What an entry at squared distance d2 stores (r2 = r_m^2).  Mode 0: the distance,
// clamped at r2 (written as a minimum: equal bit for bit to keep ? d2 : r2, and a NaN
// d2, whose pattern is above every number's, yields r2 in both forms).  Modes 1 and 2 are the hit-count scorings of paper
// Sec. 5.4, expressed as penalties so that smaller is better: mode 1 stores 0 for a hit
// and 1 for a miss (hit count = M - sum); mode 2 adds the inner sphere of radius
// r_m / 2: 0 inside it, 1 inside the outer sphere only, 2 outside both (score = M - sum).
template <int MODE>
__device__ inline float table_value(float d2, float r2) {
  if (MODE == 0) {  // min(d2, r2) on the bit patterns: both are >= +0, so bits order like values
    const uint32_t a = __float_as_uint(d2), b = __float_as_uint(r2);
    return __uint_as_float(a < b ? a : b);
  }
  if (MODE == 1) return d2 <= r2 ? 0.0f : 1.0f;
  return d2 <= 0.25f * r2 ? 0.0f : (d2 <= r2 ? 1.0f : 2.0f);
}
__device__ inline float table_value(float d2, float r2, int mode) {
  return mode == 0 ? table_value<0>(d2, r2) : (mode == 1 ? table_value<1>(d2, r2) : table_value<2>(d2, r2));
}

// One table entry (paper Sec. 4.1; Algorithm 2): squared distance between the
// residual projection and a codebook entry, thresholded at r2.
template <int DSUB, typename SP>
__device__ inline float lut_entry(SP sq, const float *__restrict__ cen,
                                  const float *__restrict__ cb, int dsub_rt, float r2, int mode, bool &keep) {
  const int dsub = DSUB > 0 ? DSUB : dsub_rt;
  float d2 = 0.0f;
  if (DSUB == 2) {
    const float2 e = *reinterpret_cast<const float2 *>(cb);
    const float t0 = (sq[0] - cen[0]) - e.x;
    const float t1 = (sq[1] - cen[1]) - e.y;
    d2 = fmaf(t1, t1, t0 * t0);
  } else if (DSUB == 4) {
    const float4 e = *reinterpret_cast<const float4 *>(cb);
    const float t0 = (sq[0] - cen[0]) - e.x;
    const float t1 = (sq[1] - cen[1]) - e.y;
    const float t2 = (sq[2] - cen[2]) - e.z;
    const float t3 = (sq[3] - cen[3]) - e.w;
    d2 = fmaf(t3, t3, fmaf(t2, t2, fmaf(t1, t1, t0 * t0)));
  } else {
    for (int j = 0; j < dsub; ++j) {
      const float t = (sq[j] - cen[j]) - cb[j];
      d2 = j == 0 ? t * t : fmaf(t, t, d2);
    }
  }
  keep = d2 <= r2;
  return table_value(d2, r2, mode);
}

// Four consecutive entries of one subspace (same arithmetic per entry as above);
// ev holds their 4 * DSUB coordinates as loaded from the codebook.
template <int DSUB, int MODE>
__device__ inline float4 lut_entry4(const float (&res)[DSUB > 0 ? DSUB : 1], const float4 *ev, float r2) {
  constexpr int DS = DSUB > 0 ? DSUB : 1;  // res: residual projection q_m - centroid_m, computed once per list
  float e[4 * DS];
#pragma unroll
  for (int x = 0; x < DSUB; ++x) {
    e[4 * x + 0] = ev[x].x; e[4 * x + 1] = ev[x].y; e[4 * x + 2] = ev[x].z; e[4 * x + 3] = ev[x].w;
  }
  float d2[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float t0 = res[0] - e[i * DSUB];
    float acc = t0 * t0;
#pragma unroll
    for (int j = 1; j < DSUB; ++j) {
      const float t = res[j] - e[i * DSUB + j];
      acc = fmaf(t, t, acc);
    }
    d2[i] = table_value<MODE>(acc, r2);
  }
  return make_float4(d2[0], d2[1], d2[2], d2[3]);
}

struct ScanArgs {
  const float *queries;         // [Q][D]
  const int32_t *probe_ids;     // [Q][probe_stride]; the first nprobe of a row are scanned
  const float *centroids;       // [nlist][D]
  const float *codebooks;       // [M][256][dsub]
  const float *probe_lb;        // [Q][probe_stride] lower bound on the distance of any point of the probed list, or NULL
  const int32_t *qmap;          // [Q] or NULL: a query with a negative entry is left out (its workgroups exit at once)
  const float *list_box;        // [nlist][M][2][dsub] per list and subspace the bounding box of the entries in use
  const int64_t *list_offsets;  // [nlist+1]
  const int64_t *list_blocks;   // [nlist+1]
  const uint8_t *codes;         // interleaved blocks
  const int64_t *ids;           // [N]
  int64_t *out_ids;             // [Q][k]
  float *out_dist;              // [Q][k]
  uint32_t *part_d;             // [Q][nsplit][KP] (nsplit > 1)
  int64_t *part_id;
  const int64_t *cand_offsets;  // [Q+1] (DUMP)
  float *all_dist;              // (DUMP)
  int64_t *all_ids;             // (DUMP)
  int32_t *errors;              // (DUMP)
  int32_t D, M, dsub, Mp, nlist, nprobe, probe_stride, k, nsplit;
  int32_t k_out, k_off;  // rows of the outputs hold k_out keys; this launch fills [k_off, k_off + k)
  const float *query_radii;     // [Q][M] per-query radii, or NULL: the shared r_m^2 of the call
  int32_t mode;       // scoring: 0 distances, 1 hit count, 2 reward/penalty hit count
  int32_t load_mode;  // 0 default policy, 1 whole blocks, 2 always the first half of the chunks ahead, 3 always the first chunk
  int32_t ablate;  // pruning switches (results do not depend on them): 8 disables the early exit of the
                   // distance sums, 16 scans plainly from the first list on (no row minima, no checks),
                   // 32 disables the switch to plain scanning, 64 the list-level bound, 128 the byte
                   // table of the hit-count scorings
  // Wide selection (k_out above KP in one pass, wide_cap > 0): every candidate within the
  // workgroup's bound on the k_out-th distance goes to the query's slots; wide_select_kernel
  // sorts them afterwards.  The wavefronts' own lists (KP keys each) only feed the bound.
  uint32_t *wide_d;      // [Q][wide_cap] distance keys
  int64_t *wide_id;      // [Q][wide_cap] rows (positions in the index, not ids)
  int32_t *wide_n;       // [Q] slots in use, or -1: they did not suffice
  uint32_t *wide_bound;  // [Q] the bound at the end of the scan
  int32_t wide_cap;
};

// Codes of one point (the lane's) in registers.
template <int NDW>
struct CodeRegs {
  uint32_t w[NDW > 0 ? NDW : 1];
};

// A pointer that is the same in every lane, moved to scalar registers so that loads
// through it use the scalar-base + 32-bit lane-offset addressing form.
__device__ inline const uint8_t *uniform_ptr(const uint8_t *p) {
  const uint64_t v = reinterpret_cast<uint64_t>(p);
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return reinterpret_cast<const uint8_t *>(((uint64_t)hi << 32) | lo);
}

// Chunks [J0, J1) of block b of a list with nb blocks (J counts the 16-byte chunks
// first, then the 4-byte chunks).  Within a list the layout is chunk-major: chunk j of
// all blocks is contiguous, so a wavefront that stops needing the later chunks of its
// blocks leaves whole streams of the list unread.
template <int MP, int J0, int J1>
__device__ inline void load_chunks(const uint8_t *__restrict__ list_base, int nb, int b, int lane,
                                   CodeRegs<MP / 4> &r) {
  constexpr int N16 = MP / 16;
#pragma unroll
  for (int j = J0; j < J1; ++j) {
    if (j < N16) {
      const uint8_t *sp = uniform_ptr(list_base + ((int64_t)j * nb + b) * 1024);
      const uint4 v = *reinterpret_cast<const uint4 *>(sp + (uint32_t)(lane * 16));
      r.w[4 * j + 0] = v.x;
      r.w[4 * j + 1] = v.y;
      r.w[4 * j + 2] = v.z;
      r.w[4 * j + 3] = v.w;
    } else {
      const int t = j - N16;
      const uint8_t *sp = uniform_ptr(list_base + (int64_t)N16 * nb * 1024 + ((int64_t)t * nb + b) * 256);
      r.w[4 * N16 + t] = *reinterpret_cast<const uint32_t *>(sp + (uint32_t)(lane * 4));
    }
  }
}

template <int MP>
__device__ inline void load_codes(const uint8_t *__restrict__ list_base, int nb, int b, int lane,
                                  CodeRegs<MP / 4> &r) {
  load_chunks<MP, 0, MP / 16 + (MP % 16) / 4>(list_base, nb, b, lane, r);
}

// Byte offset of a point's code in a 1 KiB table row: 4 * byte j of w.  The byte select of
// the sub-dword addressing form does the extraction and the shift in one instruction
// (the compiler emits a bit-field extract plus a shift-add for the plain expression, which
// makes the vector ALU the limit of the look-up loop).
__device__ __forceinline__ uint32_t code_offset(uint32_t w, int j) {
  uint32_t a;
  const uint32_t two = 2u;
  switch (j) {
    case 0: asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_0" : "=v"(a) : "s"(two), "v"(w)); break;
    case 1: asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_1" : "=v"(a) : "s"(two), "v"(w)); break;
    case 2: asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_2" : "=v"(a) : "s"(two), "v"(w)); break;
    default: asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_3" : "=v"(a) : "s"(two), "v"(w)); break;
  }
  return a;
}

// dist += table value of the point's code, for subspaces [h, h1), in subspace order.  The
// look-ups are issued together and only then added: the sums form a dependent chain, and
// without the fences the scheduler pairs every read with its add, so that a wavefront has
// one LDS read in flight at a time.
template <int MT>
__device__ __forceinline__ void lookup_group(const LDS float *lut, const CodeRegs<((MT + 3) / 4 * 4) / 4> &r,
                                             int h, int h1, float &dist) {
  float t[LOOKUP_GROUP];
#pragma unroll
  for (int j = 0; j < LOOKUP_GROUP; ++j) {
    const int m = h + j;
    if (m < h1) {
      // The table starts at LDS address 0 (the kernels declare no static LDS; the launcher
      // checks it), so the row offset fits the instruction's immediate and the look-up
      // needs no address arithmetic beyond code_offset.
      const uint32_t off = code_offset(r.w[m >> 2], m & 3);
      t[j] = *(const LDS float *)(uintptr_t)(uint32_t)(m * 1024 + off);
    }
  }
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int j = 0; j < LOOKUP_GROUP; ++j)
    if (h + j < h1) dist += t[j];
  __builtin_amdgcn_sched_barrier(0);
}

// The same for a BYTE table (hit-count scorings, paper Sec. 5.4: an entry stores its penalty
// 0, 1 or 2 in one byte; a row is 256 bytes, one dword per LDS bank, so a wavefront's look-ups
// of a row never conflict): acc += penalty of the point's code, as an integer.
template <int MT>
__device__ __forceinline__ void lookup_group(const LDS float *, const CodeRegs<((MT + 3) / 4 * 4) / 4> &r,
                                             int h, int h1, uint32_t &acc) {
  uint32_t t[LOOKUP_GROUP];
#pragma unroll
  for (int j = 0; j < LOOKUP_GROUP; ++j) {
    const int m = h + j;
    if (m < h1) {
      const uint32_t code = (r.w[m >> 2] >> (8 * (m & 3))) & 0xFFu;
      t[j] = *(const LDS unsigned char *)(uintptr_t)(uint32_t)(m * 256 + code);   // the table starts at LDS address 0
    }
  }
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int j = 0; j < LOOKUP_GROUP; ++j)
    if (h + j < h1) acc += t[j];
  __builtin_amdgcn_sched_barrier(0);
}

__device__ __forceinline__ float acc_value(float a) { return a; }
__device__ __forceinline__ float acc_value(uint32_t a) { return (float)a; }   // exact: sums of at most 2 M

template <int MT>
__device__ inline float adc_sum(const LDS float *lut, const CodeRegs<((MT + 3) / 4 * 4) / 4> &r,
                                float start = 0.0f) {
  float dist = start;
#pragma unroll
  for (int h = 0; h < MT; h += LOOKUP_GROUP) lookup_group<MT>(lut, r, h, cmin(h + LOOKUP_GROUP, MT), dist);
  return dist;
}
template <int MT>
__device__ inline float adc_sum_bytes(const LDS float *lut, const CodeRegs<((MT + 3) / 4 * 4) / 4> &r) {
  uint32_t acc = 0;
#pragma unroll
  for (int h = 0; h < MT; h += LOOKUP_GROUP) lookup_group<MT>(lut, r, h, cmin(h + LOOKUP_GROUP, MT), acc);
  return (float)acc;
}

// Same sum, over subspaces [M0, M1), with early exit.  Table values are >= 0 and fp32
// addition is monotone in both operands, so the final sum is at least what the chain gives
// when every remaining term is replaced by the minimum of its table row; for non-negative
// terms that is at least (partial + exact sum of those minima) (1 - M 2^-24).  suf[j] is an
// fp32 sum (in some order) of the row minima of subspaces >= 8 j, itself within M 2^-24 of
// the exact one, and tauf is the bound on the k-th smallest distance enlarged by 2^-13,
// which covers these errors and the rounding of the test itself many times over (M <= 128).
// Every 8 subspaces the wavefront checks whether any of its points can still reach the
// bound; if none can, the rest of the block is skipped and false returned.  Points that
// survive get exactly the sum adc_sum computes.  With `checks` off it is the plain sum.
// (ACC: float for a table of distances, uint32_t for a byte table of penalties.)
template <int MT, int M0, int M1, typename ACC>
__device__ inline bool adc_part_exit(const LDS float *lut, const CodeRegs<((MT + 3) / 4 * 4) / 4> &r,
                                     const LDS float *suf, float tauf, bool checks, bool valid, ACC &dist) {
#pragma unroll
  for (int g = M0; g < M1; g += 8) {
    // requested ahead of the look-ups, so that it has arrived when they have
    float rest = 0.0f;
    if (checks && cmin(g + 8, M1) < MT) rest = suf[cmin(g + 8, M1) >> 3];
#pragma unroll
    for (int h = g; h < cmin(g + 8, M1); h += LOOKUP_GROUP)
      lookup_group<MT>(lut, r, h, cmin(h + LOOKUP_GROUP, cmin(g + 8, M1)), dist);
    if (checks && cmin(g + 8, M1) < MT) {  // `checks` is uniform: off, a check costs a scalar branch
      if (__ballot(valid && acc_value(dist) + rest <= tauf) == 0) return false;
    }
  }
  return true;
}

// runtime-M variant: dwords are fetched as they are needed
__device__ inline float adc_sum_rt(const LDS float *lut, const uint8_t *__restrict__ list_base, int nb, int b,
                                   int lane, int M, int Mp, float start = 0.0f) {
  const int n16 = Mp >> 4;
  float dist = start;
  for (int d = 0; d < (Mp >> 2); ++d) {
    const uint8_t *p = d < 4 * n16
                           ? list_base + ((int64_t)(d >> 2) * nb + b) * 1024 + lane * 16 + (d & 3) * 4
                           : list_base + (int64_t)n16 * nb * 1024 + ((int64_t)(d - 4 * n16) * nb + b) * 256 + lane * 4;
    const uint32_t w = *reinterpret_cast<const uint32_t *>(p);
    for (int bb = 0; bb < 4; ++bb) {
      const int m = 4 * d + bb;
      if (m < M) dist += lut[m * 256 + ((w >> (8 * bb)) & 0xFFu)];
    }
  }
  return dist;
}

// Per-wavefront top-k state.
struct WaveTop {
  Key L0, L1;       // sorted list, 2 keys per lane
  Key tau;          // k-th best so far (sentinel while fewer than k are known)
  Key floor;        // only keys above this one are wanted (the last key of the previous pass)
  int qcount;       // keys waiting in the LDS queue
};

// Bounds shared by the wavefronts of a workgroup (LDS): word 0 is an upper bound
// on the k-th smallest distance over everything the workgroup has seen; words
// 1..NW hold each wavefront's ceil(k/NW)-th smallest distance.
struct SharedTau {
  LDS uint32_t *bound;
  LDS uint32_t *rank;  // [NW]
  int nw, wave, jrank;
  // wide selection: [0] slots taken so far, [1] set when they ran out; NULL otherwise
  LDS uint32_t *wide;
  uint32_t *wide_d;    // this query's slots
  int64_t *wide_id;
  int wide_cap;
};

// Fold the queued keys into the sorted list and refresh the bounds.  Two rules
// tighten the shared bound, both by atomic min so that a stale value can only
// be looser, never wrong:
//   (i)  a wavefront that knows k keys publishes its k-th smallest distance;
//   (ii) the wavefronts see disjoint points, so if each of the NW wavefronts
//        knows j = ceil(k/NW) keys no larger than x_w, at least k keys are no
//        larger than max_w x_w.
template <bool DPP>
__device__ __forceinline__ void wave_flush(WaveTop &st, LDS uint32_t *qd, LDS int64_t *qid, int lane, int k,
                                  const SharedTau &sh) {
  Key q;
  q.d = lane < st.qcount ? qd[lane] : SENT_D;
  q.id = lane < st.qcount ? qid[lane] : SENT_ID;
  wave_sort_desc<DPP>(q, lane);
  wave_merge<DPP>(st.L0, st.L1, q, lane);
  st.qcount = 0;
  const Key t0 = bcast_key(st.L0, (k - 1) & 63), t1 = bcast_key(st.L1, (k - 1) & 63);
  st.tau = (k - 1) < 64 ? t0 : t1;
  const int jr = sh.jrank - 1;
  const uint32_t j0 = (uint32_t)__shfl((int)st.L0.d, jr & 63), j1 = (uint32_t)__shfl((int)st.L1.d, jr & 63);
  volatile LDS uint32_t *rank = sh.rank;
  if (lane == 0) {
    // (rule (i) needs a list that can hold k keys: not so in the wide selection)
    if (!sh.wide && st.tau.d != SENT_D) __hip_atomic_fetch_min(sh.bound, st.tau.d, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    rank[sh.wave] = jr < 64 ? j0 : j1;
  }
  uint32_t mx = lane < sh.nw ? rank[lane] : 0u;
#pragma unroll
  for (int off = 8; off > 0; off >>= 1) {
    const uint32_t o = (uint32_t)__shfl_xor((int)mx, off);
    mx = o > mx ? o : mx;
  }
  if (lane == 0 && mx != SENT_D) __hip_atomic_fetch_min(sh.bound, mx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

// Offer this block's distances to the wavefront's top-k.
template <bool SGN = false>
__device__ __forceinline__ void wave_offer(WaveTop &st, float dist, bool valid, int64_t row,
                                  const int64_t *__restrict__ ids, LDS uint32_t *qd, LDS int64_t *qid,
                                  int lane, int k, const SharedTau &sh) {
  const uint32_t bits = dist_key<SGN>(dist);
  const uint32_t shared = *(volatile LDS uint32_t *)sh.bound;
  const uint32_t pref = (sh.wide || shared < st.tau.d) ? shared : st.tau.d;
  bool pass = valid && bits <= pref;
  if (__ballot(pass) == 0) return;
  Key c;
  c.d = bits;
  // (wide selection: the wavefront's list only feeds the bound, which is a distance, so the
  // row number breaks ties as well as the id would, and no id is fetched during the scan)
  c.id = sh.wide ? row : (pass ? ids[row] : SENT_ID);
  if (sh.wide) {
    // every key within the bound is kept: one slot range per wavefront and block
    const unsigned long long wb = __ballot(pass);
    const uint32_t wn = (uint32_t)__popcll(wb);
    uint32_t pos = 0;
    if (lane == 0) pos = __hip_atomic_fetch_add(sh.wide, wn, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    pos = (uint32_t)__builtin_amdgcn_readfirstlane((int)pos);
    if (pos + wn <= (uint32_t)sh.wide_cap) {
      if (pass) {
        const uint32_t slot = pos + (uint32_t)__popcll(wb & ((1ull << lane) - 1ull));
        sh.wide_d[slot] = c.d;
        sh.wide_id[slot] = c.id;
      }
    } else if (lane == 0) {
      sh.wide[1] = 1u;
    }
  }
  pass = pass && kless(c, st.tau) && kless(st.floor, c);
  unsigned long long bal = __ballot(pass);
  int n = __popcll(bal);
  if (n == 0) return;
  if (st.qcount + n > 64) {
    wave_flush<!SGN>(st, qd, qid, lane, k, sh);
    pass = pass && kless(c, st.tau);
    bal = __ballot(pass);
    n = __popcll(bal);
    if (n == 0) return;
  }
  if (pass) {
    const int slot = st.qcount + __popcll(bal & ((1ull << lane) - 1ull));
    qd[slot] = c.d;
    qid[slot] = c.id;
  }
  st.qcount += n;
}

// Empty top-k state.  More than KP keys per query are produced KP at a time: a later pass
// keeps only the keys above the last one of the pass before it (which that pass has
// already written to the output row).
template <bool SGN, bool DUMP>
__device__ inline void init_wave_top(WaveTop &st, const ScanArgs &a, int64_t q) {
  st.L0.d = st.L1.d = SENT_D;
  st.L0.id = st.L1.id = SENT_ID;
  st.tau.d = SENT_D;
  st.tau.id = SENT_ID;
  st.qcount = 0;
  st.floor.d = 0u;
  st.floor.id = INT64_MIN;
  if (!DUMP && a.k_off > 0) {
    const int64_t o = q * a.k_out + a.k_off - 1;
    const int64_t fid = a.out_ids[o];
    const uint32_t fd = fid == -1 ? SENT_D : dist_key<SGN>(a.out_dist[o]);  // -1: nothing is left
    st.floor.d = __builtin_amdgcn_readfirstlane(fd);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)(uint64_t)fid);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)((uint64_t)fid >> 32));
    st.floor.id = (int64_t)(((uint64_t)hi << 32) | lo);
  }
}

// End of a workgroup's work: fold the queues, merge the wavefronts' sorted lists
// through LDS (the table region is free by then) and write the first k keys, or
// the whole list when the probes of the query were split over several workgroups.
template <int NW, bool SGN = false>
__device__ __forceinline__ void finish_topk(WaveTop &st, LDS uint32_t *qd, LDS int64_t *qid, int lane,
                                            int wave, const SharedTau &sh, LDS unsigned char *smem3,
                                            const ScanArgs &a, int64_t q, int split) {
  if (st.qcount > 0) wave_flush<!SGN>(st, qd, qid, lane, a.k, sh);
  __syncthreads();  // tables no longer needed: their LDS becomes the staging area
  LDS uint32_t *stage_d = (LDS uint32_t *)smem3;
  LDS int64_t *stage_id = (LDS int64_t *)(smem3 + NW * KP * 4);
  auto put = [&]() __attribute__((always_inline)) {
    stage_d[wave * KP + lane] = st.L0.d;
    stage_d[wave * KP + 64 + lane] = st.L1.d;
    stage_id[wave * KP + lane] = st.L0.id;
    stage_id[wave * KP + 64 + lane] = st.L1.id;
  };
  if (wave > 0) put();
  __syncthreads();
  // pairwise rounds: wavefront w takes the list of w + stride, for stride = 1, 2, 4, ...
  for (int stride = 1; stride < NW; stride <<= 1) {
    if ((wave & (2 * stride - 1)) == 0 && wave + stride < NW) {
      const int w = wave + stride;
      for (int h = 0; h < 2; ++h) {
        Key qk;  // the half is sorted ascending: read it reversed to get descending
        qk.d = stage_d[w * KP + h * 64 + (63 - lane)];
        qk.id = stage_id[w * KP + h * 64 + (63 - lane)];
        wave_merge<!SGN>(st.L0, st.L1, qk, lane);
      }
      if (wave > 0 && 2 * stride < NW) put();  // read by another wavefront in a later round
    }
    if (2 * stride < NW) __syncthreads();
  }
  if (wave == 0) {
    if (a.nsplit > 1) {
      const int64_t o = (q * a.nsplit + split) * KP;
      a.part_d[o + lane] = st.L0.d;
      a.part_d[o + 64 + lane] = st.L1.d;
      a.part_id[o + lane] = st.L0.id;
      a.part_id[o + 64 + lane] = st.L1.id;
    } else {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const Key e = h ? st.L1 : st.L0;  // by value: a reference would pin the state in scratch
        const int i = h * 64 + lane;
        if (i < a.k) {
          const bool real = e.d != SENT_D;
          const int64_t o = q * a.k_out + a.k_off + i;
          a.out_ids[o] = real ? e.id : -1;
          a.out_dist[o] = real ? key_dist<SGN>(e.d) : __builtin_inff();
        }
      }
    }
  }
}

// Wide selection, between two lists (nobody scans): drop the slots whose key the bound has
// since ruled out.  Chunks of NT slots are read, counted and written back in order; a key
// never moves to a higher slot, so the chunk being written never reaches the one read next.
// `wcnt` holds NW words.  Ends with a barrier.
template <int NW>
__device__ inline void wide_compact(const SharedTau &sh, LDS uint32_t *wcnt, int tid, int lane, int wave) {
  constexpr int NT = NW * 64;
  const uint32_t taken = sh.wide[0];
  const uint32_t n = taken < (uint32_t)sh.wide_cap ? taken : (uint32_t)sh.wide_cap;
  const uint32_t bound = *(volatile LDS uint32_t *)sh.bound;
  uint32_t out = 0;
  for (uint32_t base = 0; base < n; base += NT) {
    const uint32_t i = base + tid;
    uint32_t d = SENT_D;
    int64_t id = SENT_ID;
    if (i < n) {
      d = sh.wide_d[i];
      id = sh.wide_id[i];
    }
    const bool keep = i < n && d <= bound;
    const unsigned long long bal = __ballot(keep);
    if (lane == 0) wcnt[wave] = (uint32_t)__popcll(bal);
    __syncthreads();  // the counts are there, and every read of this chunk has completed
    uint32_t before = 0, total = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const uint32_t c = wcnt[w];
      total += c;
      if (w < wave) before += c;
    }
    if (keep) {
      const uint32_t pos = out + before + (uint32_t)__popcll(bal & ((1ull << lane) - 1ull));
      sh.wide_d[pos] = d;
      sh.wide_id[pos] = id;
    }
    out += total;
    __syncthreads();  // counts free for the next chunk
  }
  if (tid == 0) sh.wide[0] = out;
  __syncthreads();
}

// End of a workgroup's work in the wide selection: the final bound and the slot count go to
// global memory for wide_select_kernel; a query whose slots ran out is marked -1 and served
// by the pass-by-pass path afterwards.
__device__ inline void finish_wide(WaveTop &st, LDS uint32_t *qd, LDS int64_t *qid, int lane, int tid,
                                   const SharedTau &sh, const ScanArgs &a, int64_t q) {
  if (st.qcount > 0) wave_flush<true>(st, qd, qid, lane, a.k, sh);
  __syncthreads();
  if (tid == 0) {
    const uint32_t taken = sh.wide[0];
    const bool over = sh.wide[1] != 0u || taken > (uint32_t)sh.wide_cap;
    a.wide_n[q] = over ? -1 : (int32_t)taken;
    a.wide_bound[q] = *(volatile LDS uint32_t *)sh.bound;
  }
}

constexpr int LDS_PER_CU = 160 * 1024;

// Once per kernel and device: the look-up code addresses the table at LDS address 0, which
// holds as long as the kernel has no static LDS in front of its dynamic allocation (checked
// here), and the kernel is allowed the whole LDS of a CU as dynamic allocation.  `done` has
// one bit per device; two host threads that race through here do the same idempotent calls.
template <typename K>
int prepare_kernel(K kern, std::atomic<uint64_t> &done) {
  int dev = 0;
  IVFPQ_HIP_TRY(hipGetDevice(&dev));
  const uint64_t bit = 1ull << (dev & 63);
  if (done.load(std::memory_order_acquire) & bit) return IVFPQ_OK;
  hipFuncAttributes attr;
  IVFPQ_HIP_TRY(hipFuncGetAttributes(&attr, reinterpret_cast<const void *>(kern)));
  if (attr.sharedSizeBytes != 0) {
    ivfpq::set_error("scan: kernel has %zu bytes of static LDS, 0 expected", (size_t)attr.sharedSizeBytes);
    return IVFPQ_ERR_UNSUPPORTED;
  }
  IVFPQ_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, LDS_PER_CU));
  done.fetch_or(bit, std::memory_order_release);
  return IVFPQ_OK;
}

}  // namespace
