// Aggregation kernels for the accumulative aggregators (sum, mean, degree-normalised sum):
// the cached state is the plain sum S_v of the (possibly pre-scaled) message rows of the
// in-neighbours, updated by adding deltas (the extension sketched in Sec. 7): for a removed edge
// the old message is subtracted, for an inserted edge the new one is added, and for a kept edge
// whose source changed the difference new - old is added.  The three edge sets are disjoint, so
// no message is counted twice.  Events of a target are consumed in their stored order and lane
// groups are combined in a fixed pattern: results are reproducible run to run.
#include <algorithm>

#include "bigrows.h"

namespace ink {

struct S4 { float v[4]; };

__device__ __forceinline__ float4 ldf4(const float *p) { return *reinterpret_cast<const float4 *>(p); }

// Lanes per row: 16 / 32 / 64 (64 / LPR groups fill the wave) or 12 (five groups, lanes 60-63 idle:
// rows of at most 48 floats, five of them per load instead of four).
template <int LPR> __device__ __forceinline__ void sum_groups(S4 &a) {
  if constexpr ((LPR & (LPR - 1)) == 0) {
#pragma unroll
    for (int off = LPR; off < kWave; off <<= 1)
#pragma unroll
      for (int c = 0; c < 4; c++) a.v[c] = __fadd_rn(a.v[c], __shfl_xor(a.v[c], off, kWave));
  } else {       // group 0 + group 1 + ... in that order; valid in the lanes of group 0
    constexpr int G = kWave / LPR;
    const int q = lane_id() % LPR;
    S4 r = a;
#pragma unroll
    for (int g = 1; g < G; g++)
#pragma unroll
      for (int c = 0; c < 4; c++) r.v[c] = __fadd_rn(r.v[c], __shfl(a.v[c], q + g * LPR, kWave));
    a = r;
  }
}
template <int LPR> __device__ __forceinline__ bool lane_in_groups() { return lane_id() < (kWave / LPR) * LPR; }

// sum of rows M[ids[j]] for j in [j0, j1): group g takes j0 + g, j0 + g + G, ... in order
template <int LPR>
__device__ __forceinline__ void sum_range(const int32_t *ids, int64_t j0, int64_t j1, const float *M, int ldm,
                                          bool lane_on, int q, S4 &acc) {
  constexpr int G = kWave / LPR;
  const int l = lane_id();
  const int g = l / LPR;
#pragma unroll
  for (int c = 0; c < 4; c++) acc.v[c] = 0.f;
  for (int64_t jb = j0; jb < j1; jb += kWave) {
    int64_t jj = jb + l;
    int myid = jj < j1 ? ids[jj] : -1;
    int cnt = (int)((j1 - jb) < kWave ? (j1 - jb) : kWave);
    constexpr int U = LPR <= 16 ? INK_U_SUM16 : (LPR == 32 ? INK_U_SUM32 : INK_U_SUM64);
    for (int it = 0; it < cnt; it += G * U) {
      int id[U];
      float4 row[U];
#pragma unroll
      for (int u = 0; u < U; u++) {
        int k = it + u * G + g;
        id[u] = __shfl(myid, k < kWave ? k : 0, kWave);
        if (k >= cnt) id[u] = -1;
        if (id[u] >= 0 && lane_on) row[u] = ldf4(M + (int64_t)id[u] * ldm + 4 * q);
      }
#pragma unroll
      for (int u = 0; u < U; u++) {
        if (id[u] >= 0 && lane_on) {
          acc.v[0] = __fadd_rn(acc.v[0], row[u].x); acc.v[1] = __fadd_rn(acc.v[1], row[u].y);
          acc.v[2] = __fadd_rn(acc.v[2], row[u].z); acc.v[3] = __fadd_rn(acc.v[3], row[u].w);
        }
      }
    }
  }
  sum_groups<LPR>(acc);
}

__device__ __forceinline__ void mark_bit_s(uint64_t *bm, int v) {
  atomicOr((unsigned long long *)&bm[v >> 6], 1ull << (v & 63));
}

// stores the row; returns wave-uniform "some value of the first d dimensions changed"
template <int LPR>
__device__ __forceinline__ bool store_sum(float *A, int ld, int d, int v, bool lane_on, int q, const S4 &nv,
                                          bool compare) {
  const int l = lane_id();
  bool writer = lane_on && l < LPR;
  bool chg = false;
  if (writer) {
    float *p = A + (int64_t)v * ld + 4 * q;
    if (compare) {
      float4 o = ldf4(p);
      float ov[4] = {o.x, o.y, o.z, o.w};
#pragma unroll
      for (int c = 0; c < 4; c++)
        if (4 * q + c < d) chg |= __float_as_uint(ov[c]) != __float_as_uint(nv.v[c]);
    }
    if (!compare || chg) *reinterpret_cast<float4 *>(p) = make_float4(nv.v[0], nv.v[1], nv.v[2], nv.v[3]);
  }
  return __ballot(chg) != 0ull;
}

template <int LPR>
__global__ __launch_bounds__(256) void k_sum_full(AggArgs a, const int32_t *targets, int64_t n_targets, uint64_t *chg,
                                                  int32_t *big_list, int32_t *n_big, int compare, Counters *cnt) {
  const int l = lane_id();
  const int q = l % LPR;
  const bool lane_on = 4 * q < a.wd && lane_in_groups<LPR>();
  int64_t wid = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / kWave;
  if (wid >= n_targets) return;
  int v = targets ? targets[wid] : (int)wid;
  int deg = a.in_deg[v];
  if (targets && l == 0) atomicAdd(&cnt->stripe[blockIdx.x % kStripes][ST_REGATHER], (unsigned long long)deg);
  if (deg > a.big_deg && l == 0)      // few rows: also tallied when every row is recomputed
    atomicAdd(&cnt->stripe[blockIdx.x % kStripes][ST_REGATHER_LONG], (unsigned long long)deg);
  if (deg > a.big_deg) {
    if (l == 0) big_list[atomicAdd(n_big, 1)] = v;
    return;
  }
  S4 acc;
  sum_range<LPR>(a.in_ids + a.in_off[v], 0, deg, a.M, a.ldm, lane_on, q, acc);
  bool ch = store_sum<LPR>(a.A, a.ld, a.d, v, lane_on, q, acc, compare != 0);
  if (ch && chg && l == 0) mark_bit_s(chg, v);
}

template <int LPR>
__global__ __launch_bounds__(INK_BIG_LB) void k_sum_big_partial(AggArgs a, const int32_t *big_list, const int32_t *n_big_p,
                                                          const int32_t *pref, const int32_t *total_p, float *part) {
  __shared__ float sv[kBigMaxWaves][kWave * 4];
  const int l = lane_id(), w = threadIdx.x / kWave, nw = blockDim.x / kWave;
  const int q = l % LPR;
  const bool lane_on = 4 * q < a.wd && lane_in_groups<LPR>();
  const int total = *total_p, n_big = *n_big_p;
  for (int cg = blockIdx.x; cg < total; cg += gridDim.x) {
    int i, v;
    int64_t j0, j1;
    big_chunk(pref, n_big, cg, big_list, a.in_deg, i, v, j0, j1);
    int64_t off = a.in_off[v];
    int64_t len = j1 - j0;
    int64_t w0 = j0 + len * w / nw, w1 = j0 + len * (w + 1) / nw;
    S4 acc;
    sum_range<LPR>(a.in_ids + off, w0, w1, a.M, a.ldm, lane_on, q, acc);
#pragma unroll
    for (int c = 0; c < 4; c++) sv[w][l * 4 + c] = acc.v[c];
    __syncthreads();
    if (w == 0) {
      for (int ww = 1; ww < nw; ww++)
#pragma unroll
        for (int c = 0; c < 4; c++) acc.v[c] = __fadd_rn(acc.v[c], sv[ww][l * 4 + c]);
      if (lane_on && l < LPR) {
        int64_t o = (int64_t)cg * a.wd + 4 * q;
#pragma unroll
        for (int c = 0; c < 4; c++) part[o + c] = acc.v[c];
      }
    }
    __syncthreads();
  }
}

template <int LPR>
__global__ __launch_bounds__(64) void k_sum_big_final(AggArgs a, const int32_t *big_list, const int32_t *n_big_p,
                                                      const int32_t *pref, const float *part, uint64_t *chg,
                                                      int compare) {
  const int l = lane_id();
  const int q = l % LPR;
  const bool lane_on = 4 * q < a.wd;
  const int n_big = *n_big_p;
  for (int i = blockIdx.x; i < n_big; i += gridDim.x) {
    int v = big_list[i];
    S4 acc;
#pragma unroll
    for (int c = 0; c < 4; c++) acc.v[c] = 0.f;
    if (lane_on && l < LPR) {
      for (int p = pref[i]; p < pref[i + 1]; p++) {
        int64_t o = (int64_t)p * a.wd + 4 * q;
#pragma unroll
        for (int c = 0; c < 4; c++) acc.v[c] = __fadd_rn(acc.v[c], part[o + c]);
      }
    }
    bool ch = store_sum<LPR>(a.A, a.ld, a.d, v, lane_on, q, acc, compare != 0);
    if (ch && chg && l == 0) mark_bit_s(chg, v);
  }
}

__device__ __forceinline__ int find_in(const int32_t *F, int nF, int u) {   // position of u in ascending F, or -1
  int lo = 0, hi = nF - 1;
  while (lo <= hi) {
    int m = (lo + hi) >> 1;
    int x = F[m];
    if (x == u) return m;
    if (x < u) lo = m + 1; else hi = m - 1;
  }
  return -1;
}

__global__ void k_delta_rows(const float *M, int ldm, const int32_t *F, int nF, const float *f_old, float *f_delta,
                             int ld_old) {
  int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  int64_t i = t / ld_old;
  int k = (int)(t % ld_old);
  if (i < nF) f_delta[i * ld_old + k] = __fsub_rn(M[(int64_t)F[i] * ldm + k], f_old[i * ld_old + k]);
}

template <int LPR>
__global__ __launch_bounds__(256) void k_sum_events(AggArgs a, const int32_t *targets, const int32_t *seg,
                                                    const int32_t *n_targets_p, const uint32_t *ev, const int32_t *F,
                                                    int nF, const float *f_old, const float *f_delta, int ld_old,
                                                    uint64_t *chg, Counters *cnt) {
  constexpr int G = kWave / LPR;
  const int l = lane_id();
  const int q = l % LPR, g = l / LPR;
  const bool lane_on = 4 * q < a.wd;
  int64_t wid = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / kWave;
  if (wid >= *n_targets_p) return;
  int v = targets[wid];
  int e0 = seg[wid], e1 = seg[wid + 1];
  S4 acc;
#pragma unroll
  for (int c = 0; c < 4; c++) acc.v[c] = 0.f;
  for (int eb = e0; eb < e1; eb += kWave) {
    int ee = eb + l;
    uint32_t mine = ee < e1 ? ev[ee] : 0xFFFFFFFFu;
    int cntw = (e1 - eb) < kWave ? (e1 - eb) : kWave;
    constexpr int U = 4;       // events in flight per lane group
    for (int it = 0; it < cntw; it += G * U) {
      const float *p[U];
      bool neg[U];
      float4 r[U];
#pragma unroll
      for (int u = 0; u < U; u++) {
        int k = it + u * G + g;
        uint32_t x = __shfl(mine, k < kWave ? k : 0, kWave);
        p[u] = nullptr;
        neg[u] = false;
        if (k < cntw && lane_on) {
          uint32_t kind = x >> kEvKindShift;
          int id = (int)(x & kEvIdMask);
          if (kind == EV_CHG) {          // id = position of the source in F: add (new - old)
            p[u] = f_delta + (int64_t)id * ld_old + 4 * q;
          } else if (kind == EV_ADD) {
            p[u] = a.M + (int64_t)id * a.ldm + 4 * q;
          } else {                        // removed edge: subtract what the source contributed before
            int pos = nF > 0 ? find_in(F, nF, id) : -1;
            p[u] = pos >= 0 ? f_old + (int64_t)pos * ld_old + 4 * q : a.M + (int64_t)id * a.ldm + 4 * q;
            neg[u] = true;
          }
          r[u] = ldf4(p[u]);
        }
      }
#pragma unroll
      for (int u = 0; u < U; u++) {
        if (!p[u]) continue;
        if (neg[u]) {
          acc.v[0] = __fsub_rn(acc.v[0], r[u].x); acc.v[1] = __fsub_rn(acc.v[1], r[u].y);
          acc.v[2] = __fsub_rn(acc.v[2], r[u].z); acc.v[3] = __fsub_rn(acc.v[3], r[u].w);
        } else {
          acc.v[0] = __fadd_rn(acc.v[0], r[u].x); acc.v[1] = __fadd_rn(acc.v[1], r[u].y);
          acc.v[2] = __fadd_rn(acc.v[2], r[u].z); acc.v[3] = __fadd_rn(acc.v[3], r[u].w);
        }
      }
    }
  }
  sum_groups<LPR>(acc);
  S4 nv;
#pragma unroll
  for (int c = 0; c < 4; c++) nv.v[c] = 0.f;
  if (lane_on) {
    float4 o = ldf4(a.A + (int64_t)v * a.ld + 4 * q);
    nv.v[0] = __fadd_rn(o.x, acc.v[0]); nv.v[1] = __fadd_rn(o.y, acc.v[1]);
    nv.v[2] = __fadd_rn(o.z, acc.v[2]); nv.v[3] = __fadd_rn(o.w, acc.v[3]);
  }
  bool ch = store_sum<LPR>(a.A, a.ld, a.d, v, lane_on, q, nv, true);
  if (ch && l == 0) { mark_bit_s(chg, v); if (a.count_cond) atomicAdd(&cnt->stripe[blockIdx.x % kStripes][ST_ACHG], 1ull); }
}

static int lanes_per_row(int ld) { return ld <= 64 ? 16 : (ld <= 128 ? 32 : 64); }
// full re-aggregation only: narrow rows take 12 lanes (config 2, layer 2: 4.5 % less aggregation time)
static int lanes_per_row_full(int ld) { return ld <= 48 ? 12 : lanes_per_row(ld); }

template <int LPR>
static hipError_t sum_full_t(ink_ctx *c, const AggArgs &a_in, const int32_t *targets, int64_t n_targets,
                             uint64_t *chg) {
  if (n_targets <= 0) return hipSuccess;
  AggArgs a = a_in;
  a.big_deg = big_threshold(n_targets, LPR, kBigDegSum);
  int compare = chg != nullptr;
  INK_TRY(ensure_big_buffers(c, a.wd, false));
  INK_TRY(hipMemsetAsync(&c->d_cnt->v[C_NBIG], 0, sizeof(int32_t), c->stream));
  {
    KernelTimer kt(c, a.layer, INK_K_AGG_FULL);
    hipLaunchKernelGGL((k_sum_full<LPR>), dim3((unsigned)((n_targets + 3) / 4)), dim3(256), 0, c->stream, a, targets,
                       n_targets, chg, c->big_list.as<int32_t>(), &c->d_cnt->v[C_NBIG], compare, c->d_cnt);
    INK_TRY(hipGetLastError());
  }
  KernelTimer kt(c, a.layer, INK_K_AGG_LONG);
  const int32_t *list = c->big_list.as<int32_t>();
  int32_t *pref = c->big_pref.as<int32_t>();
  int32_t *n_big = &c->d_cnt->v[C_NBIG], *total = &c->d_cnt->v[C_NCHUNK];
  INK_TRY(plan_big_rows(c, n_targets, a.in_deg));
  hipLaunchKernelGGL((k_sum_big_partial<LPR>), dim3(big_partial_grid(c, a.big_grid, big_block_threads(n_targets))),
                     dim3(big_block_threads(n_targets)), 0, c->stream, a, list, (const int32_t *)n_big,
                     (const int32_t *)pref, (const int32_t *)total, c->big_part_v.as<float>());
  hipLaunchKernelGGL((k_sum_big_final<LPR>), dim3(kBigGrid), dim3(64), 0, c->stream, a, list, (const int32_t *)n_big,
                     (const int32_t *)pref, (const float *)c->big_part_v.as<float>(), chg, compare);
  return hipGetLastError();
}

template <int LPR>
static hipError_t sum_events_t(ink_ctx *c, const AggArgs &a, const int32_t *targets, const int32_t *seg,
                               int64_t n_targets, const int32_t *n_targets_dev, const uint32_t *ev, const int32_t *F,
                               int nF, const float *f_old, const float *f_delta, int ld_old, uint64_t *chg) {
  if (n_targets <= 0) return hipSuccess;
  KernelTimer kt(c, a.layer, INK_K_AGG_EVENTS);
  hipLaunchKernelGGL((k_sum_events<LPR>), dim3((unsigned)((n_targets + 3) / 4)), dim3(256), 0, c->stream, a, targets,
                     seg, n_targets_dev, ev, F, nF, f_old, f_delta, ld_old, chg, c->d_cnt);
  return hipGetLastError();
}

hipError_t agg_sum_full(ink_ctx *c, const AggArgs &a, const int32_t *targets, int64_t n_targets, uint64_t *chg) {
  switch (lanes_per_row_full(a.wd)) {
    case 12: return sum_full_t<12>(c, a, targets, n_targets, chg);
    case 16: return sum_full_t<16>(c, a, targets, n_targets, chg);
    case 32: return sum_full_t<32>(c, a, targets, n_targets, chg);
    default: return sum_full_t<64>(c, a, targets, n_targets, chg);
  }
}

hipError_t agg_sum_events(ink_ctx *c, const AggArgs &a, const int32_t *targets, const int32_t *seg,
                          int64_t n_targets, const int32_t *n_targets_dev, const uint32_t *ev_val, const int32_t *F,
                          int nF, const float *f_old, const float *f_delta, int ld_old, uint64_t *chg) {
  switch (lanes_per_row(a.wd)) {
    case 16: return sum_events_t<16>(c, a, targets, seg, n_targets, n_targets_dev, ev_val, F, nF, f_old, f_delta, ld_old, chg);
    case 32: return sum_events_t<32>(c, a, targets, seg, n_targets, n_targets_dev, ev_val, F, nF, f_old, f_delta, ld_old, chg);
    default: return sum_events_t<64>(c, a, targets, seg, n_targets, n_targets_dev, ev_val, F, nF, f_old, f_delta, ld_old, chg);
  }
}

hipError_t agg_sum_delta_rows(ink_ctx *c, const AggArgs &a, const int32_t *F, int nF, const float *f_old,
                              float *f_delta, int ld_old) {
  if (nF <= 0) return hipSuccess;
  int64_t n = (int64_t)nF * ld_old;
  hipLaunchKernelGGL(k_delta_rows, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, c->stream, a.M, a.ldm, F, nF, f_old,
                     f_delta, ld_old);
  return hipGetLastError();
}

}  // namespace ink
