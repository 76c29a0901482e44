// Filtering stage (paper Sec. 2.1 "Online Search" step A; Sec. 5.3, last
// paragraph): squared L2 distance from each query to every IVF centroid, the
// nprobe nearest lists are probed.
//
// The paper computes ||x||^2 - 2 x q^T + ||q||^2 with one matrix product on
// tensor cores.  Here the product runs on the MFMA units (fp32 inputs, fp32
// accumulate).  Its rounding differs from the reference order of operations
// (t = q_i - c_i; acc = fmaf(t, t, acc), i ascending), so the product only
// PROPOSES nprobe + slack lists per query; their distances are then recomputed
// in the reference order and the final (distance, list id) selection is made
// on those.  A proposal is accepted only if the slack window is provably wide
// enough under a rounding-error bound; otherwise that query falls back to
// reference-order distances for all lists.  The result is therefore identical
// to a plain scan in the reference order, whatever the matrix unit rounds.
//
// Under the inner-product metric (paper Sec. 4.2, last sentence) lists are ranked
// by 0 - IP(q, centroid), reference order acc = fmaf(q_i, c_i, acc); the same
// scheme applies with the product itself as the proposal.

#include "ivfpq_internal.h"

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
using ivfpq::COARSE_FT;

constexpr int BM = 128;  // queries per tile
constexpr int BN = 128;  // lists per tile
constexpr int BK = 16;   // depth per LDS stage
constexpr int LDT = BM + 4;

// Four consecutive elements k .. k + 3 of row `row` of a [nrows][D] matrix, in two steps so that
// a slice's loads are all in flight while the previous slice is multiplied: load4_issue reads
// from an address clamped into the matrix (no branch; a conditional load made the compiler wait
// inside each condition), load4_mask, called when the values are needed, zeroes what stands for
// a row or an element that does not exist.  VEC: D is a multiple of 4 and the matrix 16-byte
// aligned, one 16-byte load.
template <bool VEC>
__device__ __forceinline__ void load4_issue(const float *__restrict__ base, int row, int nrows, int k, int D,
                                            float out[4]) {
  const float *p = base + (int64_t)(row < nrows ? row : 0) * D;
  if (VEC) {
    const float4 v = *reinterpret_cast<const float4 *>(p + (k < D ? k : 0));
    out[0] = v.x;
    out[1] = v.y;
    out[2] = v.z;
    out[3] = v.w;
  } else {
#pragma unroll
    for (int x = 0; x < 4; ++x) out[x] = p[k + x < D ? k + x : 0];
  }
}
template <bool VEC>
__device__ __forceinline__ void load4_mask(int row, int nrows, int k, int D, float v[4]) {
#pragma unroll
  for (int x = 0; x < 4; ++x)
    if (!(row < nrows && k + (VEC ? 0 : x) < D)) v[x] = 0.0f;
}

// out[q][c] = ||c||^2 - 2 q.c  (the ||q||^2 term is constant per query and does
// not change the ranking); -q.c under the inner-product metric.  One workgroup of 4 wavefronts computes a 128 x 128
// tile; each wavefront owns a 64 x 64 quadrant as 2 x 2 MFMA 32x32x2 blocks.
template <bool VEC>
__global__ __launch_bounds__(256) void coarse_gemm_kernel(const float *__restrict__ Qm,
                                                          const float *__restrict__ Cm,
                                                          const float *__restrict__ cnorm,
                                                          float *__restrict__ out, int Qn, int nlist,
                                                          int D, int ldo, int ip) {
  __shared__ float sA[BK][LDT];
  __shared__ float sB[BK][LDT];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int q0 = blockIdx.y * BM, c0 = blockIdx.x * BN;
  floatx16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

  for (int k0 = 0; k0 < D; k0 += BK) {
#pragma unroll
    for (int r = 0; r < 2; ++r) {
      const int f = tid + 256 * r;
      const int row = f >> 2, kq = (f & 3) * 4;
      float va[4], vb[4];
      load4_issue<VEC>(Qm, q0 + row, Qn, k0 + kq, D, va);
      load4_issue<VEC>(Cm, c0 + row, nlist, k0 + kq, D, vb);
      load4_mask<VEC>(q0 + row, Qn, k0 + kq, D, va);
      load4_mask<VEC>(c0 + row, nlist, k0 + kq, D, vb);
#pragma unroll
      for (int x = 0; x < 4; ++x) {
        sA[kq + x][row] = va[x];
        sB[kq + x][row] = vb[x];
      }
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < BK; kk += 2) {
      const int kr = kk + (lane >> 5), l31 = lane & 31;
      const float a0 = sA[kr][wm * 64 + l31], a1 = sA[kr][wm * 64 + 32 + l31];
      const float b0 = sB[kr][wn * 64 + l31], b1 = sB[kr][wn * 64 + 32 + l31];
      acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);
      acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);
      acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);
      acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);
    }
    __syncthreads();
  }
  // accumulator layout of the 32x32 block: column = lane % 32,
  // row = 8 * (v / 4) + 4 * (lane / 32) + v % 4
#pragma unroll
  for (int bi = 0; bi < 2; ++bi)
#pragma unroll
    for (int bj = 0; bj < 2; ++bj) {
      const int c = c0 + wn * 64 + bj * 32 + (lane & 31);
      const float cn = c < nlist ? cnorm[c] : 0.0f;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int q = q0 + wm * 64 + bi * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        if (q < Qn && c < nlist) out[(int64_t)q * ldo + c] = ip ? -acc[bi][bj][v] : cn - 2.0f * acc[bi][bj][v];
      }
    }
}

// ---------------------------------------------------------------------------
// Many lists (coarse_fused_keys() > 0): the product's rows are never written.  The tile is
// computed with the lists along the accumulator rows, so that a lane holds, for ONE query
// (column lane % 32), 64 of the tile's 128 lists (rows 8 (v / 4) + 4 (lane / 32) + v % 4 of each
// of the four 32 x 32 blocks); it keeps the COARSE_FT smallest of them as sorted integer keys
// -- the proposal value mapped to an int32 that orders like the float, its low 6 bits replaced
// by the position (block, v) of the list -- and writes those.  What a lane leaves out is no
// smaller than its last key: the selection kernel works on the keys and uses that bound for
// the lists it never sees.  K slices are double-buffered in LDS, the next slice's global
// loads in flight while the current one is multiplied.

constexpr int32_t KEY_PAD = 0x7F000000;   // key of a list that does not exist: above every real key
constexpr float PAD_VALUE = 1.7e38f;      // its proposal value

__device__ __forceinline__ int32_t prop_key(float v) {   // monotone float -> int32, its own inverse
  const int32_t b = (int32_t)__float_as_uint(v);
  return b ^ ((b >> 31) & 0x7FFFFFFF);
}
__device__ __forceinline__ float prop_value(int32_t k) {
  return __uint_as_float((uint32_t)(k ^ ((k >> 31) & 0x7FFFFFFF)));
}
__device__ __forceinline__ int32_t med3i(int32_t a, int32_t b, int32_t c) {
  const int32_t lo = a < b ? a : b, hi = a < b ? b : a;
  const int32_t m = hi < c ? hi : c;
  return lo > m ? lo : m;
}

template <bool VEC>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4))) void coarse_gemm_top_kernel(
    const float *__restrict__ Qm, const float *__restrict__ Cm, const float *__restrict__ cnorm,
    int32_t *__restrict__ keys, int Qn, int nlist, int D, int ldk, int ip, int32_t *__restrict__ fb_count) {
  // Tiles stay [row][k] in LDS, as they come from memory (one 16-byte store per 16-byte load),
  // rows LDK floats apart: 16-byte aligned, and eight lanes reading 16 bytes of eight consecutive
  // rows touch 32 different banks.  The MFMA step (2 along k) lets each half of the wavefront
  // bring its own k: half h takes k = 8 h .. 8 h + 7 of the slice, two 16-byte reads per row.
  // (The order of the sum over k differs from a plain loop's; the product only proposes.)
  constexpr int LDK = BK + 4;
  __shared__ __align__(16) float sA[2][BN][LDK];  // [stage][list of the tile][k]
  __shared__ __align__(16) float sB[2][BM][LDK];  // [stage][query of the tile][k]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l31 = lane & 31, half = lane >> 5;
  const int c0 = blockIdx.x * BN, q0 = blockIdx.y * BM;
  floatx16 acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[i][v] = 0.0f;
  if (blockIdx.x == 0 && blockIdx.y == 0 && tid == 0) *fb_count = 0;  // flagged queries of this chunk: none yet
  float va[2][4], vb[2][4];
  auto fetch = [&](int k0) __attribute__((always_inline)) {
#pragma unroll
    for (int r = 0; r < 2; ++r) {
      const int f = tid + 256 * r;
      const int row = f >> 2, kq = (f & 3) * 4;
      load4_issue<VEC>(Cm, c0 + row, nlist, k0 + kq, D, va[r]);
      load4_issue<VEC>(Qm, q0 + row, Qn, k0 + kq, D, vb[r]);
    }
  };
  auto stash = [&](int st, int k0) __attribute__((always_inline)) {
#pragma unroll
    for (int r = 0; r < 2; ++r) {
      const int f = tid + 256 * r;
      const int row = f >> 2, kq = (f & 3) * 4;
      load4_mask<VEC>(c0 + row, nlist, k0 + kq, D, va[r]);
      load4_mask<VEC>(q0 + row, Qn, k0 + kq, D, vb[r]);
      *reinterpret_cast<float4 *>(&sA[st][row][kq]) = make_float4(va[r][0], va[r][1], va[r][2], va[r][3]);
      *reinterpret_cast<float4 *>(&sB[st][row][kq]) = make_float4(vb[r][0], vb[r][1], vb[r][2], vb[r][3]);
    }
  };
  fetch(0);
  stash(0, 0);
  __syncthreads();
  int st = 0;
  for (int k0 = 0; k0 < D; k0 += BK) {
    const bool more = k0 + BK < D;
    if (more) fetch(k0 + BK);
    const int kh = 8 * half;
    const float4 b0 = *reinterpret_cast<const float4 *>(&sB[st][wave * 32 + l31][kh]);
    const float4 b1 = *reinterpret_cast<const float4 *>(&sB[st][wave * 32 + l31][kh + 4]);
    // two accumulators at a time, alternating, so that a product never waits for the one before it
#pragma unroll
    for (int i = 0; i < 4; i += 2) {
      const float4 a0 = *reinterpret_cast<const float4 *>(&sA[st][i * 32 + l31][kh]);
      const float4 a1 = *reinterpret_cast<const float4 *>(&sA[st][i * 32 + l31][kh + 4]);
      const float4 c0v = *reinterpret_cast<const float4 *>(&sA[st][i * 32 + 32 + l31][kh]);
      const float4 c1v = *reinterpret_cast<const float4 *>(&sA[st][i * 32 + 32 + l31][kh + 4]);
      acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0.x, b0.x, acc[i], 0, 0, 0);
      acc[i + 1] = __builtin_amdgcn_mfma_f32_32x32x2f32(c0v.x, b0.x, acc[i + 1], 0, 0, 0);
      acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0.y, b0.y, acc[i], 0, 0, 0);
      acc[i + 1] = __builtin_amdgcn_mfma_f32_32x32x2f32(c0v.y, b0.y, acc[i + 1], 0, 0, 0);
      acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0.z, b0.z, acc[i], 0, 0, 0);
      acc[i + 1] = __builtin_amdgcn_mfma_f32_32x32x2f32(c0v.z, b0.z, acc[i + 1], 0, 0, 0);
      acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0.w, b0.w, acc[i], 0, 0, 0);
      acc[i + 1] = __builtin_amdgcn_mfma_f32_32x32x2f32(c0v.w, b0.w, acc[i + 1], 0, 0, 0);
      acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1.x, b1.x, acc[i], 0, 0, 0);
      acc[i + 1] = __builtin_amdgcn_mfma_f32_32x32x2f32(c1v.x, b1.x, acc[i + 1], 0, 0, 0);
      acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1.y, b1.y, acc[i], 0, 0, 0);
      acc[i + 1] = __builtin_amdgcn_mfma_f32_32x32x2f32(c1v.y, b1.y, acc[i + 1], 0, 0, 0);
      acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1.z, b1.z, acc[i], 0, 0, 0);
      acc[i + 1] = __builtin_amdgcn_mfma_f32_32x32x2f32(c1v.z, b1.z, acc[i + 1], 0, 0, 0);
      acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1.w, b1.w, acc[i], 0, 0, 0);
      acc[i + 1] = __builtin_amdgcn_mfma_f32_32x32x2f32(c1v.w, b1.w, acc[i + 1], 0, 0, 0);
    }
    if (more) stash(st ^ 1, k0 + BK);
    __syncthreads();  // the other stage is complete, and nobody still reads this one
    st ^= 1;
  }
  // the tiles are done with: their LDS now holds the lists' squared norms
  float *scn = &sA[0][0][0];
  if (tid < BN) {
    const int c = c0 + tid;
    scn[tid] = c < nlist ? (ip ? 0.0f : cnorm[c]) : PAD_VALUE;
  }
  __syncthreads();
  int32_t t[COARSE_FT];
#pragma unroll
  for (int x = 0; x < COARSE_FT; ++x) t[x] = KEY_PAD;
  const float coef = ip ? -1.0f : -2.0f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int r = i * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
      const float val = scn[r] + coef * acc[i][v];
      const int32_t key = (prop_key(val) & ~63) | (i * 16 + v);
#pragma unroll
      for (int x = COARSE_FT - 1; x > 0; --x) t[x] = med3i(t[x - 1], t[x], key);
      t[0] = t[0] < key ? t[0] : key;
    }
  const int q = q0 + wave * 32 + l31;
  if (q < Qn) {
    int32_t *o = keys + (int64_t)q * ldk + (int64_t)(blockIdx.x * 2 + half) * COARSE_FT;
#pragma unroll
    for (int x = 0; x < COARSE_FT; x += 2) *reinterpret_cast<int2 *>(o + x) = make_int2(t[x], t[x + 1]);
  }
}

// list of the key at position p of a query's key row
__device__ __forceinline__ int fused_list(int p, int32_t key) {
  const int g = p / COARSE_FT, pos = key & 63;
  return (g >> 1) * BN + (pos >> 4) * 32 + 8 * ((pos & 15) >> 2) + 4 * (g & 1) + (pos & 3);
}

// ---------------------------------------------------------------------------

constexpr int SEL_THREADS = 256;
constexpr int MAX_PROPOSE = 2048;
using ivfpq::FB_SLOTS;   // flagged queries per chunk whose reference-order rows are filled by many workgroups
constexpr int FB_SLICES = 64;

__device__ inline uint32_t orderable(float f) {
  const uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ inline float unorderable(uint32_t k) {
  return __uint_as_float((k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k);
}

// Reference-order distance (see header).  The chain over D is sequential by definition; what
// can overlap is the fetch of the centroid row: eight 16-byte loads are issued before the
// chain consumes them (one load per step left the chain waiting a memory round trip per 4
// dimensions).  Same operations in the same order either way.
constexpr int ROW_BATCH = 8;

__device__ inline float exact_dist(const float *sq, const float *__restrict__ cen, int D) {
  float acc = 0.0f;
  int i = 0;
  if ((D & 3) == 0 && (reinterpret_cast<uintptr_t>(cen) & 15) == 0) {
    for (; i + 4 * ROW_BATCH <= D; i += 4 * ROW_BATCH) {
      float4 c[ROW_BATCH];
#pragma unroll
      for (int b = 0; b < ROW_BATCH; ++b) c[b] = *reinterpret_cast<const float4 *>(cen + i + 4 * b);
#pragma unroll
      for (int b = 0; b < ROW_BATCH; ++b) {
        float t = sq[i + 4 * b] - c[b].x;
        acc = fmaf(t, t, acc);
        t = sq[i + 4 * b + 1] - c[b].y;
        acc = fmaf(t, t, acc);
        t = sq[i + 4 * b + 2] - c[b].z;
        acc = fmaf(t, t, acc);
        t = sq[i + 4 * b + 3] - c[b].w;
        acc = fmaf(t, t, acc);
      }
    }
    for (; i < D; i += 4) {
      const float4 c4 = *reinterpret_cast<const float4 *>(cen + i);
      float t = sq[i] - c4.x;
      acc = fmaf(t, t, acc);
      t = sq[i + 1] - c4.y;
      acc = fmaf(t, t, acc);
      t = sq[i + 2] - c4.z;
      acc = fmaf(t, t, acc);
      t = sq[i + 3] - c4.w;
      acc = fmaf(t, t, acc);
    }
  }
  for (; i < D; ++i) {
    const float t = sq[i] - cen[i];
    acc = fmaf(t, t, acc);
  }
  return acc;
}

// Reference-order list score under the inner-product metric: 0 - q.c
__device__ inline float exact_neg_ip(const float *sq, const float *__restrict__ cen, int D) {
  float acc = 0.0f;
  int i = 0;
  if ((D & 3) == 0 && (reinterpret_cast<uintptr_t>(cen) & 15) == 0) {
    for (; i + 4 * ROW_BATCH <= D; i += 4 * ROW_BATCH) {
      float4 c[ROW_BATCH];
#pragma unroll
      for (int b = 0; b < ROW_BATCH; ++b) c[b] = *reinterpret_cast<const float4 *>(cen + i + 4 * b);
#pragma unroll
      for (int b = 0; b < ROW_BATCH; ++b) {
        acc = fmaf(sq[i + 4 * b], c[b].x, acc);
        acc = fmaf(sq[i + 4 * b + 1], c[b].y, acc);
        acc = fmaf(sq[i + 4 * b + 2], c[b].z, acc);
        acc = fmaf(sq[i + 4 * b + 3], c[b].w, acc);
      }
    }
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

__device__ inline float exact_score(const float *sq, const float *__restrict__ cen, int D, int ip) {
  return ip ? exact_neg_ip(sq, cen, D) : exact_dist(sq, cen, D);
}

// Reference-order distances from the queries in the flagged-query list `fb` (count, then
// queries) to every list: workgroup (x, y) fills slice x of row y.  A single workgroup takes
// 0.3 ms for 16384 lists, and the rest of the batch would wait for it.
__global__ __launch_bounds__(256) void coarse_exact_rows_kernel(const float *__restrict__ Qm,
                                                                const float *__restrict__ cent,
                                                                const int32_t *__restrict__ fb,
                                                                float *__restrict__ rows, int nlist, int D, int ldo,
                                                                int ip) {
  extern __shared__ float sqx[];  // [D]
  const int nflag = fb[0] < FB_SLOTS ? fb[0] : FB_SLOTS;
  if ((int)blockIdx.y >= nflag) return;
  const int64_t q = fb[1 + blockIdx.y];
  for (int i = threadIdx.x; i < D; i += 256) sqx[i] = Qm[q * D + i];
  __syncthreads();
  float *row = rows + (int64_t)blockIdx.y * ldo;
  for (int c = blockIdx.x * 256 + threadIdx.x; c < nlist; c += gridDim.x * 256)
    row[c] = exact_score(sqx, cent + (int64_t)c * D, D, ip);
}

// inclusive prefix sum over the 256 threads of the workgroup (tmp: 2 x 256)
__device__ inline uint32_t scan256(uint32_t v, uint32_t *tmp, int tid) {
  int cur = 0;
  tmp[tid] = v;
  __syncthreads();
  for (int off = 1; off < SEL_THREADS; off <<= 1) {
    uint32_t x = tmp[cur * SEL_THREADS + tid];
    if (tid >= off) x += tmp[cur * SEL_THREADS + tid - off];
    cur ^= 1;
    tmp[cur * SEL_THREADS + tid] = x;
    __syncthreads();
  }
  const uint32_t r = tmp[cur * SEL_THREADS + tid];
  __syncthreads();
  return r;
}

// queries that needed the exact fallback since the counter was last reset (diagnostic)
__device__ unsigned int g_coarse_fallbacks = 0;

constexpr int NBINS = 2048;                       // histogram bins per refinement level
constexpr int BINS_PER_THREAD = NBINS / SEL_THREADS;

__device__ inline unsigned long long row_key(const float *row, int c) {
  return ((unsigned long long)orderable(row[c]) << 32) | (uint32_t)c;
}

// One workgroup per query.  Keys are (proposal value, list id) packed in 64 bits, so
// they are distinct.  A histogram over equal-width key intervals finds a cut that
// holds at least kprop and at most MAX_PROPOSE keys below it (refining the interval
// of the kprop-th key when a level is too coarse; at width 1 a bin holds one key, so
// the loop ends).  The selected lists get their distances in the reference order,
// are sorted by (distance, list id), and the first nprobe are emitted.
// With `flags` (device [qn]) a workgroup serves the queries of its group of `group` consecutive
// queries whose flag is set, one after the other, and nothing else: the second line behind
// coarse_select_wave_kernel, launched with few workgroups because it usually finds no work.
__global__ __launch_bounds__(SEL_THREADS) __attribute__((amdgpu_waves_per_eu(4))) void coarse_select_kernel(
    float *__restrict__ rows, const float *__restrict__ Qm, const float *__restrict__ cent, int nlist,
    int D, int ldo, int nprobe, int kprop, float err_scale, float max_cnorm, int ip,
    int32_t *__restrict__ out_ids, float *__restrict__ out_dist, const int32_t *__restrict__ flags, int qn,
    int group, int mode, int flag_min, const int32_t *__restrict__ fb) {
  extern __shared__ float sq[];  // [D]
  __shared__ uint32_t hist[NBINS];
  __shared__ uint32_t tmp[2 * SEL_THREADS];
  __shared__ unsigned long long keys[MAX_PROPOSE];
  __shared__ unsigned long long red_lo[SEL_THREADS / 64], red_hi[SEL_THREADS / 64];
  __shared__ uint32_t sel[3];
  __shared__ uint32_t sel_cut[2];
  __shared__ uint32_t count;
  __shared__ float red[SEL_THREADS / 64];

  const int tid = threadIdx.x;
  for (int gq = 0; gq < group; ++gq) {
  // mode 0: `rows` holds the product's rows, one per query.  The other modes serve queries for
  // which there are no such rows, from reference-order distances to every list.  Mode 1: the
  // flagged queries of the group with a flag above flag_min, one scratch row per workgroup,
  // filled here.  Mode 2: the query in slot blockIdx.x of the flagged-query list `fb` (count,
  // then queries), its row already filled by coarse_exact_rows_kernel.
  int64_t q;
  float *row;
  if (mode == 2) {
    const int nflag = fb[0] < FB_SLOTS ? fb[0] : FB_SLOTS;
    if (gq > 0 || (int)blockIdx.x >= nflag) break;
    q = fb[1 + blockIdx.x];
    row = rows + (int64_t)blockIdx.x * ldo;
  } else {
    q = (int64_t)blockIdx.x * group + gq;
    if (q >= qn) break;
    if (flags && flags[q] <= flag_min) continue;   // uniform over the workgroup
    row = rows + (mode == 1 ? (int64_t)blockIdx.x : q) * ldo;
  }
  __syncthreads();                         // the shared arrays are free of the query before
  const float *qv = Qm + q * D;

  float part = 0.0f;
  for (int i = tid; i < D; i += SEL_THREADS) {
    const float x = qv[i];
    sq[i] = x;
    part += x * x;
  }
  for (int off = 32; off > 0; off >>= 1) part += __shfl_xor(part, off);
  if ((tid & 63) == 0) red[tid >> 6] = part;
  __syncthreads();
  const float qq = red[0] + red[1] + red[2] + red[3];

  for (int attempt = mode ? 1 : 0; attempt < 2; ++attempt) {
    if (attempt == 1) {
      // fallback: reference-order distances for every list
      if (tid == 0) atomicAdd(&g_coarse_fallbacks, 1u);
      if (mode != 2)
        for (int c = tid; c < nlist; c += SEL_THREADS) row[c] = exact_score(sq, cent + (int64_t)c * D, D, ip);
      __syncthreads();
    }
    int nsel = 0;
    unsigned long long cut = 0ull;  // exclusive upper bound of the selected keys
    for (bool allow_fast = true;; allow_fast = false) {
    // ---- smallest and largest key of the row ----
    unsigned long long kmin = ~0ull, kmax = 0ull;
    for (int c = tid; c < nlist; c += SEL_THREADS) {
      const unsigned long long k = row_key(row, c);
      kmin = k < kmin ? k : kmin;
      kmax = k > kmax ? k : kmax;
    }
    // Shortcut for kprop <= 256 and long rows, or rows of 1024 lists and more when D is large
    // (its fixed cost, ranking 256 minima, is more than a histogram over a short row unless the
    // histogram's coarser cut buys many long reference-order distances: measured, 1024 lists,
    // D = 200: 0.39 -> 0.22 ms per 10 000 queries; D = 128: 0.12 -> 0.15).  The threads' own minima are distinct keys of the
    // row, so the kprop-th smallest of them is an upper bound on the kprop-th smallest key
    // of the row.  Everything up to that bound is selected (typically 1.2-1.5 kprop keys)
    // and the histogram is not needed; it remains the way out if too many keys tie under
    // the bound.
    const bool fast = allow_fast && kprop <= SEL_THREADS && (nlist >= 16 * SEL_THREADS || (nlist >= 4 * SEL_THREADS && D > 160));
    unsigned long long fast_cut = 0ull;
    if (fast) {
      keys[tid] = kmin;  // this thread's minimum (every thread has elements)
      __syncthreads();
      uint32_t rank = 0;
#pragma unroll 4
      for (int j = 0; j < SEL_THREADS; ++j) rank += keys[j] < kmin ? 1u : 0u;
      if (rank == (uint32_t)kprop - 1u) {
        sel_cut[0] = (uint32_t)(kmin + 1ull);
        sel_cut[1] = (uint32_t)((kmin + 1ull) >> 32);
      }
      __syncthreads();
      fast_cut = ((unsigned long long)sel_cut[1] << 32) | sel_cut[0];
    }
    for (int off = 32; off > 0; off >>= 1) {
      const unsigned long long a = __shfl_xor(kmin, off), b = __shfl_xor(kmax, off);
      kmin = a < kmin ? a : kmin;
      kmax = b > kmax ? b : kmax;
    }
    if ((tid & 63) == 0) {
      red_lo[tid >> 6] = kmin;
      red_hi[tid >> 6] = kmax;
    }
    __syncthreads();
    for (int w = 0; w < SEL_THREADS / 64; ++w) {
      kmin = red_lo[w] < kmin ? red_lo[w] : kmin;
      kmax = red_hi[w] > kmax ? red_hi[w] : kmax;
    }
    // ---- histogram levels: window [lo, lo + (NBINS << shift)) ----
    unsigned long long lo = kmin;
    int shift = 64 - __clzll((kmax - kmin) | 1ull) - 11;  // (kmax - lo) >> shift < NBINS
    if (shift < 0) shift = 0;
    uint32_t need = kprop;   // keys still wanted from the window
    uint32_t below = 0;      // keys under the window (all selected)
    for (;;) {
      if (fast) {
        cut = fast_cut;
        break;
      }
      for (int i = tid; i < NBINS; i += SEL_THREADS) hist[i] = 0;
      __syncthreads();
      for (int c = tid; c < nlist; c += SEL_THREADS) {
        const unsigned long long k = row_key(row, c);
        if (k >= lo) {
          const unsigned long long bin = (k - lo) >> shift;
          if (bin < NBINS) atomicAdd(&hist[(uint32_t)bin], 1u);
        }
      }
      __syncthreads();
      uint32_t local[BINS_PER_THREAD], sum = 0;
#pragma unroll
      for (int i = 0; i < BINS_PER_THREAD; ++i) {
        local[i] = hist[tid * BINS_PER_THREAD + i];
        sum += local[i];
      }
      const uint32_t incl = scan256(sum, tmp, tid);
      uint32_t run = incl - sum;
      if (run < need && incl >= need) {  // the bin of the need-th key is one of this thread's
#pragma unroll
        for (int i = 0; i < BINS_PER_THREAD; ++i) {
          if (run < need && run + local[i] >= need) {
            sel[0] = tid * BINS_PER_THREAD + i;  // bin
            sel[1] = run;                        // keys of the window under that bin
            sel[2] = local[i];                   // keys in that bin
          }
          run += local[i];
        }
      }
      __syncthreads();
      const uint32_t bin = sel[0], under = sel[1], inbin = sel[2];
      __syncthreads();
      if (below + under + inbin <= (uint32_t)MAX_PROPOSE || shift == 0) {
        cut = lo + (((unsigned long long)bin + 1) << shift);
        if (cut < lo) cut = ~0ull;  // wrapped: the window reaches the top of the key range
        break;
      }
      below += under;
      need -= under;
      lo += (unsigned long long)bin << shift;
      shift = shift > 11 ? shift - 11 : 0;
    }
    // ---- collect the selected lists ----
    if (tid == 0) count = 0;
    __syncthreads();
    for (int c = tid; c < nlist; c += SEL_THREADS) {
      const unsigned long long k = row_key(row, c);
      if (k < cut || cut == ~0ull) {
        const uint32_t slot = atomicAdd(&count, 1u);
        if (slot < (uint32_t)MAX_PROPOSE) keys[slot] = (uint32_t)c;
      }
    }
    __syncthreads();
    nsel = count < (uint32_t)MAX_PROPOSE ? (int)count : MAX_PROPOSE;
    const bool overflow = fast && count > (uint32_t)MAX_PROPOSE;
    __syncthreads();
    if (!overflow) break;  // else masses of ties under the bound: once more, with the histogram
    }
    int psort = 2;
    while (psort < nsel) psort <<= 1;
    // reference-order distances, one selected list per thread (dense: the sequential
    // chain over D runs once per wavefront, not once per selected list)
    for (int i = tid; i < psort; i += SEL_THREADS) {
      unsigned long long key = ~0ull;
      if (i < nsel) {
        const int c = (int)(uint32_t)keys[i];
        const float d = attempt == 1 ? row[c] : exact_score(sq, cent + (int64_t)c * D, D, ip);
        key = ((unsigned long long)orderable(d) << 32) | (uint32_t)c;
      }
      keys[i] = key;
    }
    __syncthreads();
    // ---- sort the proposals by (reference distance, list id) ----
    for (int k2 = 2; k2 <= psort; k2 <<= 1)
      for (int j = k2 >> 1; j > 0; j >>= 1) {
        for (int t = tid; t < (psort >> 1); t += SEL_THREADS) {
          const int i = ((t & ~(j - 1)) << 1) | (t & (j - 1));
          const int p = i + j;
          const unsigned long long a = keys[i], b = keys[p];
          const bool up = (i & k2) == 0;
          if (up ? (b < a) : (a < b)) {
            keys[i] = b;
            keys[p] = a;
          }
        }
        __syncthreads();
      }
    if (attempt == 1 || nsel >= nlist) break;
    // every list that was not selected has a proposal value >= the cut's; accept if
    // that lower bound clears the nprobe-th reference distance by more than the
    // rounding-error bound of the matrix product
    // (|q.c| <= (|q|^2 + |c|^2) / 2, so the same bound covers the product alone)
    const float t_prop = unorderable((uint32_t)(cut >> 32)) + (ip ? 0.0f : qq);
    const float tau = unorderable((uint32_t)(keys[nprobe - 1] >> 32));
    const float bound = err_scale * (qq + max_cnorm);
    const bool ok = (t_prop - tau) > bound;  // false for NaN
    __syncthreads();
    if (ok) break;
  }
  for (int p = tid; p < nprobe; p += SEL_THREADS) {
    const unsigned long long key = keys[p];
    out_ids[q * nprobe + p] = (int32_t)(uint32_t)key;
    if (out_dist) out_dist[q * nprobe + p] = unorderable((uint32_t)(key >> 32));
  }
  }
}

// ---------------------------------------------------------------------------
// The same selection with one WAVEFRONT per query and no workgroup barrier, for rows of up
// to 4096 lists: a histogram of 1024 bins over the range of the row's proposal values finds
// the bin of the kprop-th smallest, the lists up to that bin (and far enough past the
// nprobe-th for the acceptance test) are collected, get their reference-order distances (one
// list per lane) and are put in (distance, list) order by a rank sort.  The proposal is
// accepted under the same rounding bound as above.  Whatever does not fit -- more than CS_CAND lists up to the bin (masses of equal
// proposal values), a proposal that the bound does not accept -- is flagged and left to
// coarse_select_kernel, so the result is that of the reference order in every case.

#define LDS __attribute__((address_space(3)))
constexpr int CS_BINS = 1024;   // histogram bins; bin b lives at word (b % 16) * 64 + b / 16 (lane l owns bins 16 l .. 16 l + 15)
constexpr int CS_CAND = 256;    // lists a query may collect
constexpr int CS_WAVES = 4;     // queries per workgroup

__device__ __forceinline__ int cs_hidx(uint32_t bin) { return (int)(((bin & 15u) << 6) | (bin >> 4)); }

// FUSED: `rows` holds the key rows of coarse_gemm_top_kernel (nrow keys per query) instead of
// the product's rows (nrow = nlist values); a key gives its list and, to 64 units in the last
// place, the proposal value, and the last key of every group of COARSE_FT bounds the lists of
// that group that were not written.
template <bool FUSED>
__global__ __launch_bounds__(CS_WAVES * 64) void coarse_select_wave_kernel(
    const float *__restrict__ rows, const float *__restrict__ Qm, const float *__restrict__ cent, int qn, int nlist,
    int nrow, int D, int ldo, int nprobe, int kprop, float err_scale, float max_cnorm, int ip,
    int32_t *__restrict__ out_ids, float *__restrict__ out_dist, int32_t *__restrict__ flags,
    int32_t *__restrict__ fb) {
  extern __shared__ __align__(16) unsigned char cs_smem[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t q = (int64_t)blockIdx.x * CS_WAVES + wave;
  if (q >= qn) return;   // no workgroup barrier anywhere in this kernel
  const int dpad = (D + 3) & ~3;
  const size_t per_wave = (size_t)CS_BINS * 4 + (size_t)CS_CAND * 8 + (size_t)dpad * 4;
  LDS unsigned char *mine = (LDS unsigned char *)cs_smem + wave * per_wave;
  LDS uint32_t *hist = (LDS uint32_t *)mine;
  LDS unsigned long long *cand = (LDS unsigned long long *)(mine + CS_BINS * 4);
  LDS float *sq = (LDS float *)(mine + CS_BINS * 4 + CS_CAND * 8);
  const float *row = rows + q * ldo;
  const float *qv = Qm + q * D;
  // The row's entries, raw: rows of up to 64 * ROW_REGS entries are read once, with all loads
  // in flight together, and stay in registers for the three passes below; longer rows are read
  // by each pass.  `each(fn)` calls fn(position, raw entry) for
  // the whole row, every lane in every call (positions past the end included).
  constexpr int ROW_REGS = 24;
  const uint32_t *raw_row = reinterpret_cast<const uint32_t *>(row);
  const bool in_regs = nrow <= 64 * ROW_REGS;
  uint32_t kreg[ROW_REGS];
  if (in_regs) {
#pragma unroll
    for (int j = 0; j < ROW_REGS; ++j) kreg[j] = j * 64 + lane < nrow ? raw_row[j * 64 + lane] : 0u;
  }
  auto each = [&](auto fn) __attribute__((always_inline)) {
    if (in_regs) {
#pragma unroll
      for (int j = 0; j < ROW_REGS; ++j)
        if (j * 64 < nrow) fn(j * 64 + lane, kreg[j]);
    } else {
      for (int c0 = 0; c0 < nrow; c0 += 64) fn(c0 + lane, c0 + lane < nrow ? raw_row[c0 + lane] : 0u);
    }
  };
  // what an entry stands for: its list (nlist: none), its proposal value
  auto list_of = [&](int p, uint32_t raw) __attribute__((always_inline)) {
    if (p >= nrow) return nlist;
    const int list = FUSED ? fused_list(p, (int32_t)raw) : p;
    return list < nlist ? list : nlist;
  };
  auto value_of = [&](uint32_t raw) __attribute__((always_inline)) {
    return FUSED ? prop_value((int32_t)raw) : __uint_as_float(raw);
  };

  float part = 0.0f;
  for (int i = lane; i < D; i += 64) {
    const float x = qv[i];
    sq[i] = x;
    part += x * x;
  }
  for (int off = 32; off > 0; off >>= 1) part += __shfl_xor(part, off);
  const float qq = part;

  // range of the row's proposal values
  float vmin = __builtin_inff(), vmax = -__builtin_inff();
  each([&](int p, uint32_t raw) __attribute__((always_inline)) {
    if (list_of(p, raw) < nlist) {
      const float v = value_of(raw);
      vmin = fminf(vmin, v);
      vmax = fmaxf(vmax, v);
    }
  });
  for (int off = 32; off > 0; off >>= 1) {
    vmin = fminf(vmin, __shfl_xor(vmin, off));
    vmax = fmaxf(vmax, __shfl_xor(vmax, off));
  }
  // bins of equal width in value: bin(v) is monotone in v whatever the roundings, which is all
  // the selection needs (NaN and a degenerate range go to bin 0 / the last bin)
  const float scale = (float)CS_BINS / (vmax - vmin);
  auto bin_of = [&](float v) __attribute__((always_inline)) {
    const float x = (v - vmin) * scale;
    return x >= (float)(CS_BINS - 1) ? (uint32_t)(CS_BINS - 1) : (x > 0.0f ? (uint32_t)x : 0u);
  };
  for (int i = lane; i < CS_BINS; i += 64) hist[i] = 0u;
  each([&](int p, uint32_t raw) __attribute__((always_inline)) {
    if (list_of(p, raw) < nlist)
      __hip_atomic_fetch_add(&hist[cs_hidx(bin_of(value_of(raw)))], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
  });
  __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
  // bin of the need-th smallest value: lane l owns bins 16 l .. 16 l + 15
  uint32_t own[16], sum = 0;
  for (int j = 0; j < 16; ++j) {
    own[j] = hist[j * 64 + lane];
    sum += own[j];
  }
  uint32_t incl = sum;
  for (int off = 1; off < 64; off <<= 1) {
    const uint32_t v = (uint32_t)__shfl_up((int)incl, off);
    if (lane >= off) incl += v;
  }
  const uint32_t excl = incl - sum;
  auto bin_of_rank = [&](uint32_t need) __attribute__((always_inline)) {   // 1 <= need <= nlist
    const bool hit = excl < need && need <= incl;   // exactly one lane
    uint32_t b = 0, run = excl;
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      if (hit && run < need && need <= run + own[j]) b = 16u * lane + j;
      run += own[j];
    }
    const unsigned long long bal = __ballot(hit);
    return (uint32_t)__shfl((int)b, bal ? __ffsll((long long)bal) - 1 : 0);
  };
  // The cut: the bin of the kprop-th smallest proposal, and far enough beyond the bin of the
  // nprobe-th for the acceptance test below to hold (twice the rounding bound past that bin's
  // upper edge), whichever is later.
  // (a key is within 64 units in the last place of its proposal value, which is at most
  // 2 (|q|^2 + max |c|^2) in magnitude: 2^-15 of that sum covers it)
  const float bound = (err_scale + (FUSED ? 3.0517578125e-05f : 0.0f)) * (qq + max_cnorm);
  uint32_t top = bin_of_rank((uint32_t)kprop);
  {
    const float reach = (float)(bin_of_rank((uint32_t)nprobe) + 2u) + 2.0f * bound * scale;
    const uint32_t top2 = reach >= (float)(CS_BINS - 1) ? (uint32_t)(CS_BINS - 1) : (reach > 0.0f ? (uint32_t)reach : 0u);
    top = top2 > top ? top2 : top;
  }
  // collect the lists up to that bin; the smallest proposal among the others bounds them all
  uint32_t count = 0;
  float rest_min = __builtin_inff();
  each([&](int p, uint32_t raw) __attribute__((always_inline)) {
    const int list = list_of(p, raw);
    const bool real = list < nlist;
    const float v = real ? value_of(raw) : __builtin_inff();
    const bool take = real && bin_of(v) <= top;
    // (the last key of a group bounds the lists its lane left out, taken or not)
    if (!take || (FUSED && p % COARSE_FT == COARSE_FT - 1)) rest_min = fminf(rest_min, v);
    const unsigned long long bal = __ballot(take);
    if (take) {
      const uint32_t slot = count + (uint32_t)__popcll(bal & ((1ull << lane) - 1ull));
      if (slot < (uint32_t)CS_CAND) cand[slot] = (uint32_t)list;
    }
    count += (uint32_t)__popcll(bal);
  });
  for (int off = 32; off > 0; off >>= 1) rest_min = fminf(rest_min, __shfl_xor(rest_min, off));
  bool ok = count <= (uint32_t)CS_CAND;
  const int n = ok ? (int)count : 0;
  __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
  // reference-order distances, one list per lane and round; keys (distance, list) back to LDS
  constexpr int ROUNDS = CS_CAND / 64;
  unsigned long long key[ROUNDS];
#pragma unroll
  for (int r = 0; r < ROUNDS; ++r) {
    key[r] = ~0ull;
    const int i = r * 64 + lane;
    if (r * 64 < n) {   // uniform
      if (i < n) {
        const int c = (int)(uint32_t)cand[i];
        const float d = exact_score((const float *)sq, cent + (int64_t)c * D, D, ip);
        key[r] = ((unsigned long long)orderable(d) << 32) | (uint32_t)c;
      }
    }
  }
  __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
#pragma unroll
  for (int r = 0; r < ROUNDS; ++r)
    if (r * 64 + lane < n) cand[r * 64 + lane] = key[r];
  __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
  // rank sort: position of a key = number of keys below it (keys are distinct)
  uint32_t rank[ROUNDS];
#pragma unroll
  for (int r = 0; r < ROUNDS; ++r) rank[r] = 0;
  for (int j = 0; j < n; ++j) {
    const unsigned long long o = cand[j];
#pragma unroll
    for (int r = 0; r < ROUNDS; ++r) rank[r] += o < key[r] ? 1u : 0u;
  }
  // the nprobe-th reference distance, for the acceptance test
  float tau = 0.0f;
#pragma unroll
  for (int r = 0; r < ROUNDS; ++r) {
    const bool has = r * 64 + lane < n && rank[r] == (uint32_t)nprobe - 1u;
    const unsigned long long bal = __ballot(has);
    if (bal) tau = unorderable((uint32_t)(__shfl((unsigned long long)key[r], __ffsll((long long)bal) - 1) >> 32));
  }
  if (ok && (FUSED || n < nlist)) {
    // every list that was not collected has a proposal value of at least rest_min; accept if
    // that clears the nprobe-th reference distance by more than the rounding bound of the
    // matrix product
    const float t_prop = rest_min + (ip ? 0.0f : qq);
    ok = (t_prop - tau) > bound;   // false for NaN
  }
  ok = ok && n >= nprobe;
  if (lane == 0) {
    int32_t f = ok ? 0 : 1;
    if (FUSED && !ok) {   // a flagged query takes a number; the first FB_SLOTS also a slot of the list
      const int32_t slot = (int32_t)atomicAdd(reinterpret_cast<unsigned int *>(fb), 1u);
      if (slot < FB_SLOTS) fb[1 + slot] = (int32_t)q;
      f = slot + 1;
    }
    flags[q] = f;
  }
  if (!ok) return;
#pragma unroll
  for (int r = 0; r < ROUNDS; ++r)
    if (r * 64 + lane < n && rank[r] < (uint32_t)nprobe) {
      out_ids[q * nprobe + rank[r]] = (int32_t)(uint32_t)key[r];
      if (out_dist) out_dist[q * nprobe + rank[r]] = unorderable((uint32_t)(key[r] >> 32));
    }
}

}  // namespace

namespace ivfpq {

int coarse_fallbacks(int reset, unsigned int *out) {
  IVFPQ_HIP_TRY(hipMemcpyFromSymbol(out, HIP_SYMBOL(g_coarse_fallbacks), sizeof(unsigned int)));
  if (reset) {
    const unsigned int zero = 0;
    IVFPQ_HIP_TRY(hipMemcpyToSymbol(HIP_SYMBOL(g_coarse_fallbacks), &zero, sizeof zero));
  }
  return IVFPQ_OK;
}

int launch_coarse(const ivfpq_index *ix, const float *d_queries, int64_t Q, int32_t nprobe,
                  int32_t *d_probe_ids, float *d_probe_dist, float *d_scratch, int64_t q_chunk,
                  int32_t nlist_pad, int32_t *d_flags, hipStream_t s) {
  const int D = ix->D, nlist = ix->nlist;
  int slack = nprobe / 4;
  if (slack < 16) slack = 16;
  int kprop = nprobe + slack;
  if (kprop > nlist) kprop = nlist;
  if (kprop > MAX_PROPOSE) {
    set_error("coarse: nprobe %d too large", nprobe);
    return IVFPQ_ERR_UNSUPPORTED;
  }
  const float err_scale = 4.0f * (float)D * 1.1920929e-07f;
  const int vec = (D % 4 == 0) && (((uintptr_t)d_queries | (uintptr_t)ix->d_centroids) % 16 == 0);
  const int nkeys = coarse_fused_keys(nlist, nprobe, D);   // the workspace was sized by the same rule
  if (nkeys > 0 && !d_flags) {
    set_error("coarse: no flag array");
    return IVFPQ_ERR_INVALID_ARGUMENT;
  }
  for (int64_t q0 = 0; q0 < Q; q0 += q_chunk) {
    const int qn = (int)((Q - q0) < q_chunk ? (Q - q0) : q_chunk);
    const float *qm = d_queries + q0 * D;
    dim3 grid((nlist + BN - 1) / BN, (qn + BM - 1) / BM);
    const int ip = ix->metric == IVFPQ_METRIC_IP;
    int32_t *ids = d_probe_ids + q0 * nprobe;
    float *dist = d_probe_dist ? d_probe_dist + q0 * nprobe : nullptr;
    const size_t wave_lds = CS_WAVES * ((size_t)CS_BINS * 4 + (size_t)CS_CAND * 8 + (size_t)((D + 3) & ~3) * 4);
    if (nkeys > 0) {
      // many lists: keys instead of rows, then the one-wavefront selection on the keys; the
      // queries it flags get reference-order distances to every list, one scratch row per
      // workgroup of the second-line kernel (behind the keys, see coarse_scratch_bytes)
      // The first FB_SLOTS flagged queries have their rows filled by FB_SLICES workgroups each
      // and are then selected one workgroup per query; any beyond that (centroids whose order
      // follows their geometry flag every query) are served sixteen queries per workgroup.
      const int group = 16;
      int32_t *keys = reinterpret_cast<int32_t *>(d_scratch);
      float *group_rows = d_scratch + (((size_t)q_chunk * nkeys + 63) & ~(size_t)63);
      float *slot_rows = group_rows + (size_t)((q_chunk + group - 1) / group) * nlist_pad;
      int32_t *fb = reinterpret_cast<int32_t *>(slot_rows + (size_t)FB_SLOTS * nlist_pad);
      hipLaunchKernelGGL(vec ? coarse_gemm_top_kernel<true> : coarse_gemm_top_kernel<false>, grid, dim3(256), 0, s, qm,
                         ix->d_centroids, ix->d_cnorm, keys, qn, nlist, D, nkeys, ip, fb);
      hipLaunchKernelGGL(coarse_select_wave_kernel<true>, dim3((qn + CS_WAVES - 1) / CS_WAVES), dim3(CS_WAVES * 64),
                         wave_lds, s, d_scratch, qm, ix->d_centroids, qn, nlist, nkeys, D, nkeys, nprobe, kprop,
                         err_scale, ix->max_cnorm, ip, ids, dist, d_flags + q0, fb);
      hipLaunchKernelGGL(coarse_exact_rows_kernel, dim3(FB_SLICES, FB_SLOTS), dim3(256), (size_t)D * sizeof(float), s, qm,
                         ix->d_centroids, fb, slot_rows, nlist, D, nlist_pad, ip);
      hipLaunchKernelGGL(coarse_select_kernel, dim3(FB_SLOTS), dim3(SEL_THREADS), (size_t)D * sizeof(float), s,
                         slot_rows, qm, ix->d_centroids, nlist, D, nlist_pad, nprobe, kprop, err_scale, ix->max_cnorm,
                         ip, ids, dist, nullptr, qn, 1, 2, 0, fb);
      hipLaunchKernelGGL(coarse_select_kernel, dim3((qn + group - 1) / group), dim3(SEL_THREADS),
                         (size_t)D * sizeof(float), s, group_rows, qm, ix->d_centroids, nlist, D, nlist_pad, nprobe,
                         kprop, err_scale, ix->max_cnorm, ip, ids, dist, d_flags + q0, qn, group, 1, FB_SLOTS, fb);
      continue;
    }
    hipLaunchKernelGGL(vec ? coarse_gemm_kernel<true> : coarse_gemm_kernel<false>, grid, dim3(256), 0, s, qm,
                       ix->d_centroids, ix->d_cnorm, d_scratch, qn, nlist, D, nlist_pad, ip);
    // One wavefront per query where the proposal is small enough for it; the workgroup-per-query
    // kernel then only serves the queries the wavefront kernel flags (16 queries per workgroup,
    // so that the usual case of no flag costs a few hundred idle workgroups).
    const bool by_wave = d_flags && kprop <= CS_CAND / 2 && nlist <= 4096 && wave_lds <= 64 * 1024;
    if (by_wave) {
      hipLaunchKernelGGL(coarse_select_wave_kernel<false>, dim3((qn + CS_WAVES - 1) / CS_WAVES), dim3(CS_WAVES * 64),
                         wave_lds, s, d_scratch, qm, ix->d_centroids, qn, nlist, nlist, D, nlist_pad, nprobe, kprop,
                         err_scale, ix->max_cnorm, ip, ids, dist, d_flags + q0, nullptr);
      const int group = 16;
      hipLaunchKernelGGL(coarse_select_kernel, dim3((qn + group - 1) / group), dim3(SEL_THREADS),
                         (size_t)D * sizeof(float), s, d_scratch, qm, ix->d_centroids, nlist, D, nlist_pad, nprobe,
                         kprop, err_scale, ix->max_cnorm, ip, ids, dist, d_flags + q0, qn, group, 0, 0, nullptr);
    } else {
      hipLaunchKernelGGL(coarse_select_kernel, dim3(qn), dim3(SEL_THREADS), (size_t)D * sizeof(float), s,
                         d_scratch, qm, ix->d_centroids, nlist, D, nlist_pad, nprobe, kprop, err_scale,
                         ix->max_cnorm, ip, ids, dist, nullptr, qn, 1, 0, 0, nullptr);
    }
  }
  IVFPQ_HIP_TRY(hipGetLastError());
  return IVFPQ_OK;
}

}  // namespace ivfpq
