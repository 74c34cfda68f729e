// Aggregation kernels for the selection aggregators (max / min) with per-dimension argument
// tracking: full re-aggregation ("recompute", Sec. 2.5.2) and the event-driven incremental
// update with reset detection (Sec. 2.5.1).  One wave64 owns one target row; a lane holds four
// consecutive dimensions, so a row of d floats occupies LPR = 16/32/64 lanes and a wave works on
// 64 / LPR neighbour rows at a time.  Rows are read as coalesced 16-byte lane loads.
//
// Next to the selected value and its holder the cache keeps, per dimension, a bound on the best
// value among the OTHER neighbours (exact after a recompute, afterwards only ever loosened).  A
// holder that got worse but still strictly beats that bound stays the holder, and a candidate that
// strictly beats it covers a reset even if it is worse than the old value: both save the
// recompute that the value-only rule of Sec. 2.5.1 would need.
#include <algorithm>

#include "bigrows.h"

#ifndef INK_EV_INLINE_WIDE
#define INK_EV_INLINE_WIDE 1       // inline recompute of exposed rows: 0 never, 1 rows of 64 lanes and short launches, 2 also 32 lanes, 3 always
#endif
#ifndef INK_EVENT_GRID
#define INK_EVENT_GRID 8192        // workgroups of the event kernel (measured: 4096-8192 best, fewer leave a tail)
#endif

namespace ink {



struct F4 { float v[4]; };
struct I4 { int v[4]; };

template <bool IS_MIN> __device__ __forceinline__ bool better(float x, float y) {
  return IS_MIN ? (x < y) : (x > y);
}
template <bool IS_MIN> __device__ __forceinline__ float worst() {
  return IS_MIN ? __builtin_huge_valf() : -__builtin_huge_valf();
}
// lexicographic: better value first, lower id on equal value
template <bool IS_MIN> __device__ __forceinline__ void take(float x, int id, float &bv, int &bi) {
  if (better<IS_MIN>(x, bv) || (x == bv && id < bi)) { bv = x; bi = id; }
}

template <bool IS_MIN> __device__ __forceinline__ float best_of(float x, float y) { return better<IS_MIN>(x, y) ? x : y; }
// the same with the runner-up value sv (best value among the entries that are not the holder)
template <bool IS_MIN> __device__ __forceinline__ void take2(float x, int id, float &bv, int &bi, float &sv) {
  if (better<IS_MIN>(x, bv) || (x == bv && id < bi)) { sv = bv; bv = x; bi = id; }
  else if (better<IS_MIN>(x, sv)) sv = x;
}
// merge of the triples of two disjoint sets
template <bool IS_MIN> __device__ __forceinline__ void merge2(float ov, int oi, float os, float &bv, int &bi, float &sv) {
  float loser;
  if (better<IS_MIN>(ov, bv) || (ov == bv && oi < bi)) { loser = bv; bv = ov; bi = oi; }
  else loser = ov;
  sv = best_of<IS_MIN>(loser, best_of<IS_MIN>(sv, os));
}
// ... and with the runner-up's id si (lowest id among the non-holders that have the value sv)
// ASC: the caller feeds ids in ascending order, so on equal values the entry seen first keeps its
// place and the id comparisons drop out (8 instead of 12 vector instructions per value; the
// re-gather is bound by them, not by memory, on wide rows)
template <bool IS_MIN, bool ASC>
__device__ __forceinline__ void take2i(float x, int id, float &bv, int &bi, float &sv, int &si) {
  const bool first = better<IS_MIN>(x, bv) || (!ASC && x == bv && id < bi);
  const bool second = better<IS_MIN>(x, sv) || (!ASC && x == sv && id < si);
  const float nsv = first ? bv : (second ? x : sv);
  const int nsi = first ? bi : (second ? id : si);
  bv = first ? x : bv;
  bi = first ? id : bi;
  sv = nsv;
  si = nsi;
}
// merge of the (best, runner-up) pairs of two disjoint sets
template <bool IS_MIN>
__device__ __forceinline__ void merge2i(float ov, int oi, float os, int osi, float &bv, int &bi, float &sv, int &si) {
  float lv; int li;
  if (better<IS_MIN>(ov, bv) || (ov == bv && oi < bi)) { lv = bv; li = bi; bv = ov; bi = oi; }
  else { lv = ov; li = oi; }
  if (better<IS_MIN>(lv, sv) || (lv == sv && li < si)) { sv = lv; si = li; }
  if (better<IS_MIN>(os, sv) || (os == sv && osi < si)) { sv = os; si = osi; }
}

__device__ __forceinline__ float4 ld4(const float *p) { return *reinterpret_cast<const float4 *>(p); }


// Reduce (bv, bi) over the lane groups of a wave (groups are LPR lanes wide); every lane ends
// with the result for its 4 dimensions.
template <bool IS_MIN, int LPR> __device__ __forceinline__ void reduce_groups(F4 &bv, I4 &bi, F4 &sv) {
#pragma unroll
  for (int off = LPR; off < kWave; off <<= 1) {
#pragma unroll
    for (int c = 0; c < 4; c++) {
      float ov = __shfl_xor(bv.v[c], off, kWave);
      int oi = __shfl_xor(bi.v[c], off, kWave);
      float os = __shfl_xor(sv.v[c], off, kWave);
      merge2<IS_MIN>(ov, oi, os, bv.v[c], bi.v[c], sv.v[c]);
    }
  }
}
template <bool IS_MIN, int LPR> __device__ __forceinline__ void reduce_groups_i(F4 &bv, I4 &bi, F4 &sv, I4 &si) {
#pragma unroll
  for (int off = LPR; off < kWave; off <<= 1) {
#pragma unroll
    for (int c = 0; c < 4; c++) {
      float ov = __shfl_xor(bv.v[c], off, kWave);
      int oi = __shfl_xor(bi.v[c], off, kWave);
      float os = __shfl_xor(sv.v[c], off, kWave);
      int oj = __shfl_xor(si.v[c], off, kWave);
      merge2i<IS_MIN>(ov, oi, os, oj, bv.v[c], bi.v[c], sv.v[c], si.v[c]);
    }
  }
}

// Selection over neighbours ids[j0 .. j1) of one row, by the whole wave.  On return every lane
// holds the best (value, id) and the runner-up value of its 4 dimensions over the range;
// (worst, INT_MAX, worst) if empty.
template <bool IS_MIN, int LPR, bool ASC>
__device__ __forceinline__ void gather_range_t(const int32_t *ids, int64_t j0, int64_t j1, const float *M,
                                               int ldm, bool lane_on, int q, F4 &bv, I4 &bi, F4 &sv, I4 &si) {
  constexpr int G = kWave / LPR;
  const int l = lane_id();
  const int g = l / LPR;
#pragma unroll
  for (int c = 0; c < 4; c++) { bv.v[c] = worst<IS_MIN>(); bi.v[c] = 0x7fffffff; sv.v[c] = worst<IS_MIN>(); si.v[c] = 0x7fffffff; }
  for (int64_t jb = j0; jb < j1; jb += kWave) {
    int64_t jj = jb + l;
    int myid = jj < j1 ? ids[jj] : -1;
    int cnt = (int)((j1 - jb) < kWave ? (j1 - jb) : kWave);
    constexpr int U = LPR == 16 ? INK_U_SEL16 : (LPR == 32 ? INK_U_SEL32 : INK_U_SEL64);
    for (int it = 0; it < cnt; it += G * U) {
      int id[U];
      float4 row[U];
#pragma unroll
      for (int u = 0; u < U; u++) {
        int k = it + u * G + g;
        id[u] = __shfl(myid, k < kWave ? k : 0, kWave);
        if (k >= cnt) id[u] = -1;
        if (id[u] >= 0 && lane_on) row[u] = ld4(M + (int64_t)id[u] * ldm + 4 * q);
      }
#pragma unroll
      for (int u = 0; u < U; u++) {
        if (id[u] >= 0 && lane_on) {
          take2i<IS_MIN, ASC>(row[u].x, id[u], bv.v[0], bi.v[0], sv.v[0], si.v[0]);
          take2i<IS_MIN, ASC>(row[u].y, id[u], bv.v[1], bi.v[1], sv.v[1], si.v[1]);
          take2i<IS_MIN, ASC>(row[u].z, id[u], bv.v[2], bi.v[2], sv.v[2], si.v[2]);
          take2i<IS_MIN, ASC>(row[u].w, id[u], bv.v[3], bi.v[3], sv.v[3], si.v[3]);
        }
      }
    }
  }
  reduce_groups_i<IS_MIN, LPR>(bv, bi, sv, si);
}
// asc (wave-uniform): ids[j0 .. j1) are ascending, as they are for every node no op has touched yet
template <bool IS_MIN, int LPR>
__device__ __forceinline__ void gather_range(const int32_t *ids, int64_t j0, int64_t j1, const float *M, int ldm,
                                             bool lane_on, int q, bool asc, F4 &bv, I4 &bi, F4 &sv, I4 &si) {
  if (asc) gather_range_t<IS_MIN, LPR, true>(ids, j0, j1, M, ldm, lane_on, q, bv, bi, sv, si);
  else gather_range_t<IS_MIN, LPR, false>(ids, j0, j1, M, ldm, lane_on, q, bv, bi, sv, si);
}

struct RowOut {
  float *A; int32_t *ARG; float *UB; int32_t *ARG2; int ld; int d;
};

// Writes (bv, bi) as the new aggregated row of v if it differs from what is stored; returns
// (wave-uniform) whether any VALUE of the first d dimensions changed bitwise.
template <int LPR>
__device__ __forceinline__ bool store_row(const RowOut &o, int v, bool lane_on, int q, const F4 &bv,
                                          const I4 &bi, const F4 &sv, const I4 &si, bool have_old, const F4 &ov,
                                          const I4 &oi) {
  const int l = lane_id();
  bool writer = lane_on && l < LPR;
  bool vchg = false, ichg = false;
  if (writer) {    // bound and runner-up are rewritten unconditionally (they never decide whether a row "changed")
    *reinterpret_cast<float4 *>(o.UB + (int64_t)v * o.ld + 4 * q) = make_float4(sv.v[0], sv.v[1], sv.v[2], sv.v[3]);
    *reinterpret_cast<int4 *>(o.ARG2 + (int64_t)v * o.ld + 4 * q) = make_int4(si.v[0], si.v[1], si.v[2], si.v[3]);
  }
  if (writer) {
    F4 cv = ov; I4 ci = oi;
    if (!have_old) {
      float4 a = ld4(o.A + (int64_t)v * o.ld + 4 * q);
      int4 b = *reinterpret_cast<const int4 *>(o.ARG + (int64_t)v * o.ld + 4 * q);
      cv.v[0] = a.x; cv.v[1] = a.y; cv.v[2] = a.z; cv.v[3] = a.w;
      ci.v[0] = b.x; ci.v[1] = b.y; ci.v[2] = b.z; ci.v[3] = b.w;
    }
#pragma unroll
    for (int c = 0; c < 4; c++) {
      if (4 * q + c < o.d) vchg |= __float_as_uint(cv.v[c]) != __float_as_uint(bv.v[c]);
      ichg |= ci.v[c] != bi.v[c];
    }
    if (vchg || ichg) {
      *reinterpret_cast<float4 *>(o.A + (int64_t)v * o.ld + 4 * q) = make_float4(bv.v[0], bv.v[1], bv.v[2], bv.v[3]);
      *reinterpret_cast<int4 *>(o.ARG + (int64_t)v * o.ld + 4 * q) = make_int4(bi.v[0], bi.v[1], bi.v[2], bi.v[3]);
    }
  }
  return __ballot(vchg) != 0ull;
}

// no in-neighbours: alpha = 0, arg = -1; fewer than two: no runner-up
template <bool IS_MIN>
__device__ __forceinline__ void finish_empty(F4 &bv, I4 &bi, F4 &sv, I4 &si) {
#pragma unroll
  for (int c = 0; c < 4; c++) {
    if (bi.v[c] == 0x7fffffff) { bv.v[c] = 0.f; bi.v[c] = -1; sv.v[c] = worst<IS_MIN>(); }
    if (si.v[c] == 0x7fffffff) si.v[c] = -1;
  }
}

__device__ __forceinline__ void mark_bit(uint64_t *bm, int v) {
  atomicOr((unsigned long long *)&bm[v >> 6], 1ull << (v & 63));
}

// ------------------------------------------------------------------ full re-aggregation
// what a recompute launch does besides storing the rows
enum { FULL_COMPARE = 1,        // compare with the cached row: store and mark only what changed
       FULL_COUNT_GATHER = 2,   // tally the neighbour rows fetched
       FULL_COUNT_CHANGED = 4,  // tally the rows whose value changed
       FULL_COUNT_LONG = 8 };   // tally the neighbour rows that go to the long-row path

// One wave per row, the grid strides over the rows; n_targets_dev (optional) is the device-side
// row count, n_targets then only bounds it.
template <bool IS_MIN, int LPR>
__global__ __launch_bounds__(256) void k_agg_full(AggArgs a, const int32_t *targets, int64_t n_targets,
                                                  const int32_t *n_targets_dev, uint64_t *chg, int32_t *big_list,
                                                  int32_t *n_big, int flags, Counters *cnt) {
  const int l = lane_id();
  const int q = l % LPR;
  const bool lane_on = 4 * q < a.wd;
  if (n_targets_dev) { int64_t nd = *n_targets_dev; n_targets = nd < n_targets ? nd : n_targets; }
  const int64_t stride = (int64_t)gridDim.x * (blockDim.x / kWave);
  for (int64_t wid = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / kWave; wid < n_targets; wid += stride) {
    int v = targets ? targets[wid] : (int)wid;
    int deg = a.in_deg[v];
    if ((flags & FULL_COUNT_GATHER) && l == 0)
      atomicAdd(&cnt->stripe[blockIdx.x % kStripes][ST_REGATHER], (unsigned long long)deg);
    if ((flags & FULL_COUNT_LONG) && deg > a.big_deg && l == 0)     // few rows: also tallied when every row is recomputed
      atomicAdd(&cnt->stripe[blockIdx.x % kStripes][ST_REGATHER_LONG], (unsigned long long)deg);
    if (deg > a.big_deg) {
      if (l == 0) big_list[atomicAdd(n_big, 1)] = v;
      continue;
    }
    int64_t off = a.in_off[v];
    F4 bv; I4 bi; F4 sv; I4 si;
    gather_range<IS_MIN, LPR>(a.in_ids + off, 0, deg, a.M, a.ldm, lane_on, q, a.in_asc[v] != 0, bv, bi, sv, si);
    finish_empty<IS_MIN>(bv, bi, sv, si);
    RowOut o{a.A, a.ARG, a.UB, a.ARG2, a.ld, a.d};
    F4 dum; I4 dumi;
    bool ch;
    if (flags & FULL_COMPARE) ch = store_row<LPR>(o, v, lane_on, q, bv, bi, sv, si, false, dum, dumi);
    else {
      if (lane_on && l < LPR) {
        *reinterpret_cast<float4 *>(a.A + (int64_t)v * a.ld + 4 * q) = make_float4(bv.v[0], bv.v[1], bv.v[2], bv.v[3]);
        *reinterpret_cast<int4 *>(a.ARG + (int64_t)v * a.ld + 4 * q) = make_int4(bi.v[0], bi.v[1], bi.v[2], bi.v[3]);
        *reinterpret_cast<float4 *>(a.UB + (int64_t)v * a.ld + 4 * q) = make_float4(sv.v[0], sv.v[1], sv.v[2], sv.v[3]);
        *reinterpret_cast<int4 *>(a.ARG2 + (int64_t)v * a.ld + 4 * q) = make_int4(si.v[0], si.v[1], si.v[2], si.v[3]);
      }
      ch = false;
    }
    if (ch && chg && l == 0) {
      mark_bit(chg, v);
      if ((flags & FULL_COUNT_CHANGED) && a.count_cond) atomicAdd(&cnt->stripe[blockIdx.x % kStripes][ST_ACHG], 1ull);
    }
  }
}

// cooperative path for rows with more than kBigDeg in-neighbours: a workgroup per chunk of
// kBigChunk neighbours (its 4 waves take a quarter each), partial rows to scratch
template <bool IS_MIN, int LPR, int NW>
__global__ __launch_bounds__(NW * kWave) void k_big_partial(AggArgs a, const int32_t *big_list, const int32_t *n_big_p,
                                                      const int32_t *pref, const int32_t *total_p, float *part_v,
                                                      int32_t *part_i, float *part_s, int32_t *part_j) {
  __shared__ float sv[NW][kWave * 4];    // sized per variant: the 4-wave form must not pay the LDS of the 16-wave one
  __shared__ int si[NW][kWave * 4];
  __shared__ float ss[NW][kWave * 4];
  __shared__ int sj[NW][kWave * 4];
  const int l = lane_id(), w = threadIdx.x / kWave;
  constexpr int nw = NW;
  const int q = l % LPR;
  const bool lane_on = 4 * q < a.wd;
  const int total = *total_p, n_big = *n_big_p;
  for (int cg = blockIdx.x; cg < total; cg += gridDim.x) {
    int i, v;
    int64_t j0, j1;
    big_chunk(pref, n_big, cg, big_list, a.in_deg, i, v, j0, j1);
    int64_t off = a.in_off[v];
    int64_t len = j1 - j0;
    int64_t w0 = j0 + len * w / nw, w1 = j0 + len * (w + 1) / nw;
    F4 bv; I4 bi; F4 s2; I4 j2;
    gather_range<IS_MIN, LPR>(a.in_ids + off, w0, w1, a.M, a.ldm, lane_on, q, a.in_asc[v] != 0, bv, bi, s2, j2);
#pragma unroll
    for (int c = 0; c < 4; c++) {
      sv[w][l * 4 + c] = bv.v[c]; si[w][l * 4 + c] = bi.v[c]; ss[w][l * 4 + c] = s2.v[c]; sj[w][l * 4 + c] = j2.v[c];
    }
    __syncthreads();
    if (w == 0) {
      for (int ww = 1; ww < nw; ww++)
#pragma unroll
        for (int c = 0; c < 4; c++)
          merge2i<IS_MIN>(sv[ww][l * 4 + c], si[ww][l * 4 + c], ss[ww][l * 4 + c], sj[ww][l * 4 + c], bv.v[c], bi.v[c],
                          s2.v[c], j2.v[c]);
      if (lane_on && l < LPR) {
        int64_t o = (int64_t)cg * a.wd + 4 * q;
#pragma unroll
        for (int c = 0; c < 4; c++) {
          part_v[o + c] = bv.v[c]; part_i[o + c] = bi.v[c]; part_s[o + c] = s2.v[c]; part_j[o + c] = j2.v[c];
        }
      }
    }
    __syncthreads();
  }
}

// one wave per big row: reduce its partial rows and store
template <bool IS_MIN, int LPR>
__global__ __launch_bounds__(64) void k_big_final(AggArgs a, const int32_t *big_list, const int32_t *n_big_p,
                                                  const int32_t *pref, const float *part_v, const int32_t *part_i,
                                                  const float *part_s, const int32_t *part_j, uint64_t *chg,
                                                  int compare, Counters *cnt) {
  const int l = lane_id();
  const int q = l % LPR;
  const bool lane_on = 4 * q < a.wd;
  const int n_big = *n_big_p;
  for (int i = blockIdx.x; i < n_big; i += gridDim.x) {
    int v = big_list[i];
    F4 bv; I4 bi; F4 s2; I4 j2;
#pragma unroll
    for (int c = 0; c < 4; c++) {
      bv.v[c] = worst<IS_MIN>(); bi.v[c] = 0x7fffffff; s2.v[c] = worst<IS_MIN>(); j2.v[c] = 0x7fffffff;
    }
    if (lane_on && l < LPR) {
      for (int p = pref[i]; p < pref[i + 1]; p++) {
        int64_t o = (int64_t)p * a.wd + 4 * q;
#pragma unroll
        for (int c = 0; c < 4; c++)
          merge2i<IS_MIN>(part_v[o + c], part_i[o + c], part_s[o + c], part_j[o + c], bv.v[c], bi.v[c], s2.v[c], j2.v[c]);
      }
    }
    finish_empty<IS_MIN>(bv, bi, s2, j2);
    RowOut o{a.A, a.ARG, a.UB, a.ARG2, a.ld, a.d};
    F4 dum; I4 dumi;
    bool ch = store_row<LPR>(o, v, lane_on, q, bv, bi, s2, j2, false, dum, dumi);
    if (compare && ch && chg && l == 0) {
      mark_bit(chg, v);
      if (a.count_cond) atomicAdd(&cnt->stripe[blockIdx.x % kStripes][ST_ACHG], 1ull);
    }
  }
}

// ------------------------------------------------------------------ event-driven incremental update
// Events of a target arrive as one contiguous segment of ev_val (kind << 30 | source id).
//   DEL  (edge u -> v removed):    dimension i needs a reset iff arg[v][i] == u
//   ADD  (edge s -> v inserted):   (m_s[i], s) is a candidate
//   CHG  (message of u changed, edge kept): (m_u[i], u) is a candidate; if u held dimension i and
//        its value got worse the dimension needs a reset, if equal nothing happened there
// A reset dimension is covered when the best candidate strictly beats the old value, otherwise
// the row is exposed and recomputed from its whole current neighbourhood.
//
// A target has a handful of events, and what bounds the kernel is the traffic of its random row
// accesses (one source row per event, four cached rows per target, up to four written back), not
// the latency of one target's chain: keeping the next targets' rows in flight across targets
// (register double-buffering, event words staged in LDS) was measured and bought nothing, so the
// loop is the plain one.

#ifndef INK_EV_U
#define INK_EV_U 2                 // source rows in flight per lane group and batch
#endif
#ifndef INK_EV_BLOCK
#define INK_EV_BLOCK 8             // consecutive targets per wave visit (at most 62)
#endif
constexpr int kEvBlock = INK_EV_BLOCK;
constexpr uint32_t kEvNone = 0xFFFFFFFFu;     // no event: its kind bits name no kind

template <bool IS_MIN> struct Cached {        // this lane's four dimensions of a target's cached row
  F4 ov; I4 oi; F4 ou; I4 o2;                 // value, holder, bound on the other neighbours, runner-up id or -1
};
template <bool IS_MIN>
__device__ __forceinline__ void load_cached(const AggArgs &a, int v, bool lane_on, int q, Cached<IS_MIN> &k) {
#pragma unroll
  for (int c = 0; c < 4; c++) { k.ov.v[c] = 0.f; k.oi.v[c] = -1; k.ou.v[c] = worst<IS_MIN>(); k.o2.v[c] = -1; }
  if (lane_on) {
    const int64_t o = (int64_t)v * a.ld + 4 * q;
    const float4 x = ld4(a.A + o);
    const int4 y = *reinterpret_cast<const int4 *>(a.ARG + o);
    const float4 z = ld4(a.UB + o);
    const int4 y2 = *reinterpret_cast<const int4 *>(a.ARG2 + o);
    k.ov.v[0] = x.x; k.ov.v[1] = x.y; k.ov.v[2] = x.z; k.ov.v[3] = x.w;
    k.oi.v[0] = y.x; k.oi.v[1] = y.y; k.oi.v[2] = y.z; k.oi.v[3] = y.w;
    k.ou.v[0] = z.x; k.ou.v[1] = z.y; k.ou.v[2] = z.z; k.ou.v[3] = z.w;
    k.o2.v[0] = y2.x; k.o2.v[1] = y2.y; k.o2.v[2] = y2.z; k.o2.v[3] = y2.w;
  }
}

// U events per lane group: their words and, unless they are deletions, their sources' message rows
template <int U> struct EvBatch { uint32_t code[U]; float4 row[U]; };

// events it + u G + g (u < U) of the window `mine` (lane j holds event j, cntw of them are real)
template <bool IS_MIN, int LPR, int U>
__device__ __forceinline__ void issue_batch(const AggArgs &a, uint32_t mine, int it, int cntw, bool lane_on, int q,
                                            EvBatch<U> &b) {
  constexpr int G = kWave / LPR;
  const float W = worst<IS_MIN>();
  const int g = lane_id() / LPR;
#pragma unroll
  for (int u = 0; u < U; u++) {
    const int k = it + u * G + g;
    const uint32_t x = __shfl(mine, k < kWave ? k : 0, kWave);
    const bool valid = k < cntw && lane_on;
    b.code[u] = valid ? x : kEvNone;
    b.row[u] = make_float4(W, W, W, W);        // an event without a row offers the worst value: it never wins
    if (valid && (x >> kEvKindShift) != EV_DEL) b.row[u] = ld4(a.M + (int64_t)(x & kEvIdMask) * a.ldm + 4 * q);
  }
}

template <bool IS_MIN> struct EvAcc {
  F4 cv; I4 ci; F4 cs;       // best candidate, its source, runner-up candidate value
  bool reset[4];             // per dimension: the holder left or got worse
  bool inv2[4];              // per dimension: the recorded runner-up left or changed its message
  bool any_del;              // wave-uniform: the segment cancels something (a removed edge or a changed source)
  __device__ __forceinline__ void init() {
    any_del = false;
#pragma unroll
    for (int c = 0; c < 4; c++) {
      cv.v[c] = worst<IS_MIN>(); ci.v[c] = 0x7fffffff; cs.v[c] = worst<IS_MIN>();
      reset[c] = false; inv2[c] = false;
    }
  }
};

// Written without branches: the per-lane conditions become wave masks in scalar registers and the
// updates selects and min / max (this loop runs once per event and lane group and is half of the
// kernel's vector instructions, and the kernel's time follows their number).  What keeps it short:
//  * an event without a row (a removed edge, an empty slot) carries the worst value, so it needs no
//    mask of its own: it never becomes a candidate, and as "new value of the holder" it is a reset;
//  * an inserted edge cannot name the old holder or runner-up (it was no neighbour), so the id
//    tests need no kind;
//  * the runner-up among the candidates is max(cs, min(r, cv)) (mirrored for min) whichever of the
//    two wins;
//  * TIES false (wave-uniform): the candidates so far are changed sources in ascending id order (the order the
//    events are created in), so on equal values the earlier one keeps the dimension and the id
//    comparison is skipped.  The caller sets TIES from a target's first inserted edge on.
// v_max_f32 / v_min_f32 as they are: the library forms first canonicalise both operands (two more
// instructions each), which matters in a loop whose time follows its instruction count.  No NaN
// reaches them (inputs are finite, the sentinels are infinities).
__device__ __forceinline__ float vmax(float a, float b) { float d; asm("v_max_f32 %0, %1, %2" : "=v"(d) : "v"(a), "v"(b)); return d; }
__device__ __forceinline__ float vmin(float a, float b) { float d; asm("v_min_f32 %0, %1, %2" : "=v"(d) : "v"(a), "v"(b)); return d; }

template <bool IS_MIN, int U>
__device__ __forceinline__ void consume_batch(const EvBatch<U> &b, const Cached<IS_MIN> &k, EvAcc<IS_MIN> &s, bool TIES) {
#pragma unroll
  for (int u = 0; u < U; u++) {
    const uint32_t x = b.code[u];
    const int id = (int)(x & kEvIdMask);               // "no event": an id no node has
    const float r[4] = {b.row[u].x, b.row[u].y, b.row[u].z, b.row[u].w};
    bool first[4];
#pragma unroll
    for (int c = 0; c < 4; c++) {      // & and | on purpose: no short-circuit, no branch
      s.inv2[c] |= k.o2.v[c] == id;
      s.reset[c] |= (k.oi.v[c] == id) & better<IS_MIN>(k.ov.v[c], r[c]);
      first[c] = better<IS_MIN>(r[c], s.cv.v[c]);
    }
    if (TIES) {
      asm volatile("");                // keeps this a (wave-uniform) branch: only targets with an inserted edge pay for it
      const uint32_t kind = x >> kEvKindShift;
      const bool has_row = (kind == EV_ADD) | (kind == EV_CHG);
#pragma unroll
      for (int c = 0; c < 4; c++) first[c] |= has_row & (r[c] == s.cv.v[c]) & (id < s.ci.v[c]);
    }
#pragma unroll
    for (int c = 0; c < 4; c++) {
      s.cs.v[c] = IS_MIN ? vmin(s.cs.v[c], vmax(r[c], s.cv.v[c])) : vmax(s.cs.v[c], vmin(r[c], s.cv.v[c]));
      s.cv.v[c] = first[c] ? r[c] : s.cv.v[c];
      s.ci.v[c] = first[c] ? id : s.ci.v[c];
    }
  }
}

// The decision for target v once its events are reduced (the lane groups still hold partial
// results), the recompute of an exposed row of moderate length, and the store.
template <bool IS_MIN, int LPR, bool INLINE>
__device__ __forceinline__ void finish_target(const AggArgs &a, int v, const Cached<IS_MIN> &k, EvAcc<IS_MIN> &s,
                                              bool lane_on, int q, uint64_t *chg, int32_t *big_list, int32_t *exp_list,
                                              Counters *cnt) {
  const int l = lane_id();
  const F4 &ov = k.ov; const I4 &oi = k.oi; const F4 &ou = k.ou; const I4 &o2 = k.o2;
  F4 &cv = s.cv; I4 &ci = s.ci; F4 &cs = s.cs;
  // combine the lane groups: the flags travel packed in one register
  unsigned fl = 0u;
#pragma unroll
  for (int c = 0; c < 4; c++) fl |= ((unsigned)s.reset[c] << c) | ((unsigned)s.inv2[c] << (4 + c));
#pragma unroll
  for (int off = LPR; off < kWave; off <<= 1) fl |= (unsigned)__shfl_xor((int)fl, off, kWave);
  bool reset[4], inv2[4];
#pragma unroll
  for (int c = 0; c < 4; c++) { reset[c] = (fl >> c) & 1u; inv2[c] = (fl >> (4 + c)) & 1u; }
  reduce_groups<IS_MIN, LPR>(cv, ci, cs);
  // Per dimension: (nv, ni) new value and holder, nu new bound on the others, n2 the other neighbour
  // that has exactly the value nu (lowest such id) where that is certain, else -1.  A recorded
  // runner-up is trusted only while it neither left nor changed; it lets a reset that no candidate
  // covers be settled by promotion instead of a recompute, once per dimension between recomputes.
  F4 nv = ov; I4 ni = oi; F4 nu = ou; I4 n2;
  bool exposed = false;
  bool vchg = false, ichg = false, uchg = false;      // what of the cached row changes (short live ranges: per dimension)
#pragma unroll
  for (int c = 0; c < 4; c++) {
    const bool has_cand = ci.v[c] != 0x7fffffff;
    const int r2 = inv2[c] ? -1 : o2.v[c];               // runner-up still known to hold ou
    const bool ou_beats_cs = better<IS_MIN>(ou.v[c], cs.v[c]);
    n2.v[c] = r2;
    if (oi.v[c] < 0) {                       // no neighbours before this batch
      n2.v[c] = -1;
      if (has_cand) { nv.v[c] = cv.v[c]; ni.v[c] = ci.v[c]; nu.v[c] = cs.v[c]; }
    } else if (reset[c]) {
      // the holder left or got worse (then its new value is one of the candidates); every other
      // old neighbour is bounded by ou, and those that reach ou have ids above r2
      if (has_cand && better<IS_MIN>(cv.v[c], ou.v[c])) {
        nv.v[c] = cv.v[c]; ni.v[c] = ci.v[c]; nu.v[c] = best_of<IS_MIN>(ou.v[c], cs.v[c]);
        n2.v[c] = ou_beats_cs ? r2 : -1;
      } else if (r2 >= 0 && has_cand && cv.v[c] == ou.v[c] && ci.v[c] < r2) {
        nv.v[c] = cv.v[c]; ni.v[c] = ci.v[c];            // candidate and runner-up tie: the lower id holds
        n2.v[c] = ou_beats_cs ? r2 : -1;                 // nu stays ou, held by r2
      } else if (r2 >= 0) {
        nv.v[c] = ou.v[c]; ni.v[c] = r2;                 // the runner-up takes over; who follows is not known
        n2.v[c] = -1;                                    // nu stays ou: it bounds the old others and every candidate
      } else exposed = true;
    } else if (has_cand) {
      if (ci.v[c] == oi.v[c]) {              // the holder itself, unchanged or better at this dimension
        nv.v[c] = cv.v[c]; nu.v[c] = best_of<IS_MIN>(ou.v[c], cs.v[c]);
        n2.v[c] = ou_beats_cs ? r2 : -1;
      } else if (better<IS_MIN>(cv.v[c], ov.v[c]) || (cv.v[c] == ov.v[c] && ci.v[c] < oi.v[c])) {
        nv.v[c] = cv.v[c]; ni.v[c] = ci.v[c];          // the old holder joins the others
        nu.v[c] = best_of<IS_MIN>(best_of<IS_MIN>(ou.v[c], ov.v[c]), cs.v[c]);
        n2.v[c] = -1;
        if (better<IS_MIN>(ov.v[c], cs.v[c])) {        // it is their best unless the old runner-up ties with it
          if (better<IS_MIN>(ov.v[c], ou.v[c])) n2.v[c] = oi.v[c];
          else if (r2 >= 0) n2.v[c] = oi.v[c] < r2 ? oi.v[c] : r2;
        }
      } else {
        nu.v[c] = best_of<IS_MIN>(ou.v[c], cv.v[c]);
        n2.v[c] = better<IS_MIN>(ou.v[c], cv.v[c]) ? r2 : -1;
      }
    }
    vchg |= (4 * q + c < a.d) & (__float_as_uint(ov.v[c]) != __float_as_uint(nv.v[c]));
    ichg |= oi.v[c] != ni.v[c];
    uchg |= (__float_as_uint(ou.v[c]) != __float_as_uint(nu.v[c])) | (o2.v[c] != n2.v[c]);
  }
  exposed = __ballot(exposed && lane_on) != 0ull;
  if (a.count_cond) {   // condition of this target (Sec. 2.5.1; the distribution shown in Sec. 5.2)
    bool rs = (reset[0] || reset[1] || reset[2] || reset[3]) && lane_on;
    bool any_reset = __ballot(rs) != 0ull;
    bool dl = s.any_del;
    if (l == 0 && !exposed) {
      int which = !dl ? ST_NODEL : (!any_reset ? ST_NOEFFECT : ST_COVERED);
      atomicAdd(&cnt->stripe[blockIdx.x % kStripes][which], 1ull);
    }
  }
  if (exposed) {
    int deg = a.in_deg[v];
    if (l == 0) {
      if (a.count_cond) atomicAdd(&cnt->stripe[blockIdx.x % kStripes][ST_EXPOSED], 1ull);
      atomicAdd(&cnt->stripe[blockIdx.x % kStripes][ST_REGATHER], (unsigned long long)deg);
    }
    if constexpr (INLINE) {      // rows of moderate length are recomputed on the spot
      if (deg <= a.big_deg) {
        F4 bv; I4 bi; F4 sv; I4 si;
        gather_range<IS_MIN, LPR>(a.in_ids + a.in_off[v], 0, deg, a.M, a.ldm, lane_on, q, a.in_asc[v] != 0, bv, bi, sv, si);
        finish_empty<IS_MIN>(bv, bi, sv, si);
        RowOut o{a.A, a.ARG, a.UB, a.ARG2, a.ld, a.d};
        const bool ch = store_row<LPR>(o, v, lane_on, q, bv, bi, sv, si, true, ov, oi);
        if (ch && l == 0) { mark_bit(chg, v); if (a.count_cond) atomicAdd(&cnt->stripe[blockIdx.x % kStripes][ST_ACHG], 1ull); }
        return;
      }
    }
    // recomputed by the kernels that follow: long rows chunk by chunk, the others one wave per row
    if (l == 0) {
      if (deg > a.big_deg) {
        big_list[atomicAdd(&cnt->v[C_NBIG], 1)] = v;
        atomicAdd(&cnt->stripe[blockIdx.x % kStripes][ST_REGATHER_LONG], (unsigned long long)deg);
      } else {
        exp_list[atomicAdd(&cnt->v[C_NEXP], 1)] = v;
      }
    }
    return;
  }
  // each half of the cached row is rewritten only if it changed: most targets keep their bound and
  // runner-up, many keep value and holder
  const bool writer = lane_on && l < LPR;
  vchg &= writer;
  if (writer) {
    if (vchg || ichg) {
      *reinterpret_cast<float4 *>(a.A + (int64_t)v * a.ld + 4 * q) = make_float4(nv.v[0], nv.v[1], nv.v[2], nv.v[3]);
      *reinterpret_cast<int4 *>(a.ARG + (int64_t)v * a.ld + 4 * q) = make_int4(ni.v[0], ni.v[1], ni.v[2], ni.v[3]);
    }
    if (uchg) {
      *reinterpret_cast<float4 *>(a.UB + (int64_t)v * a.ld + 4 * q) = make_float4(nu.v[0], nu.v[1], nu.v[2], nu.v[3]);
      *reinterpret_cast<int4 *>(a.ARG2 + (int64_t)v * a.ld + 4 * q) = make_int4(n2.v[0], n2.v[1], n2.v[2], n2.v[3]);
    }
  }
  const bool ch = __ballot(vchg) != 0ull;
  if (ch && l == 0) { mark_bit(chg, v); if (a.count_cond) atomicAdd(&cnt->stripe[blockIdx.x % kStripes][ST_ACHG], 1ull); }
}

// The grid is sized to what the chip holds at once; every wave walks blocks of kEvBlock consecutive
// targets with the grid's wave count as stride.  One load per block brings the targets' ids and
// segment bounds (lane j holds those of target j), so a target's own chain is: cached row and event
// words (issued together), then the source rows.
// INLINE: exposed rows of moderate length are recomputed by the wave that finds them instead of
// being listed for a follow-up launch.  Measured: on large launches over 128-float rows the listing
// form is 3 % faster (waves that recompute leave their neighbours in the block waiting), on rows of
// 256 floats the inline form saves 0.1 of 0.9 ms of aggregation, and on short launches it saves a
// launch.  The launcher picks per call.
template <bool IS_MIN, int LPR, bool INLINE>
__global__ __launch_bounds__(256) void k_agg_events(AggArgs a, const int32_t *targets, const int32_t *seg,
                                                    const int32_t *n_targets_p, const uint32_t *ev, uint64_t *chg,
                                                    int32_t *big_list, int32_t *exp_list, Counters *cnt, int ev_block) {
  constexpr int G = kWave / LPR;
  constexpr int U = INK_EV_U;
  static_assert(kEvBlock + 2 <= kWave, "a lane per target and bound of the block");
  const int l = lane_id();
  const int q = l % LPR;
  const bool lane_on = 4 * q < a.wd;
  const int n = *n_targets_p;
  const int n_blk = (n + ev_block - 1) / ev_block;      // ev_block <= kEvBlock: 1 for short launches, whose targets should not queue behind each other in one wave
  const int n_waves = (int)gridDim.x * (int)(blockDim.x / kWave);
  const int wave0 = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave));
  for (int blk = wave0; blk < n_blk; blk += n_waves) {
    const int w0 = blk * ev_block;
    const int kt = n - w0 < ev_block ? n - w0 : ev_block;
    const int my_t = targets[w0 + (l < kt ? l : kt - 1)];
    const int my_s = seg[w0 + (l <= kt ? l : kt)];
    for (int t = 0; t < kt; t++) {
      const int v = __builtin_amdgcn_readlane(my_t, t);
      const int e0 = __builtin_amdgcn_readlane(my_s, t), e1 = __builtin_amdgcn_readlane(my_s, t + 1);
      Cached<IS_MIN> c;
      load_cached<IS_MIN>(a, v, lane_on, q, c);
      EvAcc<IS_MIN> s;
      s.init();
      bool ties = false;
      for (int eb = e0; eb < e1; eb += kWave) {
        const int ee = eb + l;
        const uint32_t mine = ee < e1 ? ev[ee] : kEvNone;
        const int cntw = e1 - eb < kWave ? e1 - eb : kWave;
        // wave-uniform: from the first inserted edge of the window on, equal values are settled by id
        const uint64_t adds = __ballot(ee < e1 && (mine >> kEvKindShift) == EV_ADD);
        s.any_del |= __ballot(ee < e1 && (mine >> kEvKindShift) != EV_ADD) != 0ull;
        const int first_add = adds ? __builtin_ctzll(adds) : kWave;
        for (int it = 0; it < cntw; it += G * U) {
          EvBatch<U> bx;
          issue_batch<IS_MIN, LPR, U>(a, mine, it, cntw, lane_on, q, bx);
          ties |= it + G * U > first_add;
          consume_batch<IS_MIN, U>(bx, c, s, ties);
        }
      }
      finish_target<IS_MIN, LPR, INLINE>(a, v, c, s, lane_on, q, chg, big_list, exp_list, cnt);
    }
  }
}

// ------------------------------------------------------------------ host side
static int lanes_per_row(int ld) { return ld <= 64 ? 16 : (ld <= 128 ? 32 : 64); }

template <bool IS_MIN, int LPR>
static hipError_t run_big(ink_ctx *c, const AggArgs &a, uint64_t *chg, int compare, int block_threads,
                          int64_t n_rows_max) {
  const int32_t *list = c->big_list.as<int32_t>();
  int32_t *pref = c->big_pref.as<int32_t>();
  int32_t *n_big = &c->d_cnt->v[C_NBIG], *total = &c->d_cnt->v[C_NCHUNK];
  INK_TRY(plan_big_rows(c, n_rows_max, a.in_deg));
  const dim3 grid(big_partial_grid(c, a.big_grid, block_threads));
  if (block_threads == 1024)
    hipLaunchKernelGGL((k_big_partial<IS_MIN, LPR, 16>), grid, dim3(1024), 0, c->stream, a, list, (const int32_t *)n_big,
                       (const int32_t *)pref, (const int32_t *)total, c->big_part_v.as<float>(),
                       c->big_part_i.as<int32_t>(), c->big_part_s.as<float>(), c->big_part_j.as<int32_t>());
  else
    hipLaunchKernelGGL((k_big_partial<IS_MIN, LPR, 4>), grid, dim3(256), 0, c->stream, a, list, (const int32_t *)n_big,
                       (const int32_t *)pref, (const int32_t *)total, c->big_part_v.as<float>(),
                       c->big_part_i.as<int32_t>(), c->big_part_s.as<float>(), c->big_part_j.as<int32_t>());
  hipLaunchKernelGGL((k_big_final<IS_MIN, LPR>), dim3(kBigGrid), dim3(64), 0, c->stream, a, list,
                     (const int32_t *)n_big, (const int32_t *)pref, (const float *)c->big_part_v.as<float>(),
                     (const int32_t *)c->big_part_i.as<int32_t>(), (const float *)c->big_part_s.as<float>(),
                     (const int32_t *)c->big_part_j.as<int32_t>(), chg, compare, c->d_cnt);
  return hipGetLastError();
}

constexpr int64_t kFullGrid = 1 << 20;     // workgroups of a recompute launch (4 rows each per stride)

template <bool IS_MIN, int LPR>
static hipError_t full_t(ink_ctx *c, const AggArgs &a_in, const int32_t *targets, int64_t n_targets, uint64_t *chg) {
  if (n_targets <= 0) return hipSuccess;
  AggArgs a = a_in;
  a.big_deg = big_threshold(n_targets, LPR, kBigDeg);
  int compare = chg != nullptr;
  INK_TRY(ensure_big_buffers(c, a.wd, true));
  INK_TRY(hipMemsetAsync(&c->d_cnt->v[C_NBIG], 0, sizeof(int32_t), c->stream));
  int64_t blocks = std::min<int64_t>((n_targets + 3) / 4, kFullGrid);
  {
    KernelTimer kt(c, a.layer, INK_K_AGG_FULL);
    hipLaunchKernelGGL((k_agg_full<IS_MIN, LPR>), dim3((unsigned)blocks), dim3(256), 0, c->stream, a, targets, n_targets,
                       (const int32_t *)nullptr, chg, c->big_list.as<int32_t>(), &c->d_cnt->v[C_NBIG],
                       (compare ? FULL_COMPARE : 0) | (targets ? FULL_COUNT_GATHER : 0) | FULL_COUNT_LONG, c->d_cnt);
    INK_TRY(hipGetLastError());
  }
  KernelTimer kt(c, a.layer, INK_K_AGG_LONG);
  return run_big<IS_MIN, LPR>(c, a, chg, compare, big_block_threads(n_targets), n_targets);
}

// n_targets may be an upper bound: the kernel stops at the device-side count n_targets_dev.
// Exposed rows are listed by the event kernel and recomputed by the two launches after it.
template <bool IS_MIN, int LPR>
static hipError_t events_t(ink_ctx *c, const AggArgs &a_in, const int32_t *targets, const int32_t *seg,
                           int64_t n_targets, const int32_t *n_targets_dev, const uint32_t *ev, uint64_t *chg) {
  if (n_targets <= 0) return hipSuccess;
  AggArgs a = a_in;
  a.big_deg = big_threshold(n_targets, LPR, kBigDeg);
  INK_TRY(ensure_big_buffers(c, a.wd, true));
  INK_TRY(c->exp_list.reserve((size_t)n_targets * 4));
  const int ev_block = latency_mode(n_targets) ? 1 : kEvBlock;
  int64_t blocks = std::min<int64_t>(((n_targets + ev_block - 1) / ev_block + 3) / 4, INK_EVENT_GRID);
  const bool inline_exposed = INK_EV_INLINE_WIDE == 0 ? false : (LPR >= (INK_EV_INLINE_WIDE == 1 ? 64 : (INK_EV_INLINE_WIDE == 2 ? 32 : 16)) || latency_mode(n_targets));
  {
    KernelTimer kt(c, a.layer, INK_K_AGG_EVENTS);
    if (inline_exposed)
      hipLaunchKernelGGL((k_agg_events<IS_MIN, LPR, true>), dim3((unsigned)blocks), dim3(256), 0, c->stream, a, targets, seg,
                         n_targets_dev, ev, chg, c->big_list.as<int32_t>(), c->exp_list.as<int32_t>(), c->d_cnt, ev_block);
    else
      hipLaunchKernelGGL((k_agg_events<IS_MIN, LPR, false>), dim3((unsigned)blocks), dim3(256), 0, c->stream, a, targets, seg,
                         n_targets_dev, ev, chg, c->big_list.as<int32_t>(), c->exp_list.as<int32_t>(), c->d_cnt, ev_block);
    INK_TRY(hipGetLastError());
  }
  if (!inline_exposed) {
    KernelTimer kt(c, a.layer, INK_K_AGG_EXPOSED);
    int64_t rb = std::min<int64_t>((n_targets + 3) / 4, latency_mode(n_targets) ? 2048 : 16384);
    hipLaunchKernelGGL((k_agg_full<IS_MIN, LPR>), dim3((unsigned)rb), dim3(256), 0, c->stream, a,
                       (const int32_t *)c->exp_list.as<int32_t>(), n_targets, (const int32_t *)&c->d_cnt->v[C_NEXP], chg,
                       c->big_list.as<int32_t>(), &c->d_cnt->v[C_NBIG], FULL_COMPARE | FULL_COUNT_CHANGED, c->d_cnt);
    INK_TRY(hipGetLastError());
  }
  KernelTimer kt(c, a.layer, INK_K_AGG_LONG);
  return run_big<IS_MIN, LPR>(c, a, chg, 1, big_block_threads(n_targets), n_targets);
}

#define DISPATCH(fn, ...)                                                         \
  do {                                                                            \
    int lpr_ = lanes_per_row(a.wd);                                               \
    if (a.is_min) {                                                               \
      if (lpr_ == 16) return fn<true, 16>(__VA_ARGS__);                           \
      if (lpr_ == 32) return fn<true, 32>(__VA_ARGS__);                           \
      return fn<true, 64>(__VA_ARGS__);                                           \
    } else {                                                                      \
      if (lpr_ == 16) return fn<false, 16>(__VA_ARGS__);                          \
      if (lpr_ == 32) return fn<false, 32>(__VA_ARGS__);                          \
      return fn<false, 64>(__VA_ARGS__);                                          \
    }                                                                             \
  } while (0)

hipError_t agg_select_full(ink_ctx *c, const AggArgs &a, const int32_t *targets, int64_t n_targets, uint64_t *chg) {
  DISPATCH(full_t, c, a, targets, n_targets, chg);
}

hipError_t agg_select_events(ink_ctx *c, const AggArgs &a, const int32_t *targets, const int32_t *seg,
                             int64_t n_targets, const int32_t *n_targets_dev, const uint32_t *ev_val, uint64_t *chg) {
  DISPATCH(events_t, c, a, targets, seg, n_targets, n_targets_dev, ev_val, chg);
}

}  // namespace ink
