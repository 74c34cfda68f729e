// C ABI entry points and the per-layer driver of the incremental update (Sec. 2.3 workflow):
// for every aggregation layer  seed events from the changed edges -> expand events from the
// changed sources -> group by target -> incremental aggregation / recompute -> dense combination
// on the changed rows -> compare-and-emit the next layer's sources.
#include <algorithm>
#include <chrono>
#include <cstring>
#include <cstdio>
#include <mutex>
#include <new>
#include <vector>

#include "bigrows.h"

using namespace ink;

#define API_TRY(x)                                                                         \
  do {                                                                                     \
    hipError_t e_ = (x);                                                                   \
    if (e_ != hipSuccess) {                                                                \
      c->err = std::string("HIP error: ") + hipGetErrorString(e_) + " at " #x;             \
      return e_ == hipErrorOutOfMemory ? INK_E_OOM : INK_E_DEVICE;                         \
    }                                                                                      \
  } while (0)

static thread_local std::string g_create_err;

static inline int round_up(int x, int m) { return (x + m - 1) / m * m; }
static inline dim3 grid1(int64_t n, int per = 256) { return dim3((unsigned)std::max<int64_t>(1, (n + per - 1) / per)); }

// ------------------------------------------------------------------------------------ kernels
// The events of a layer are created in this order: removed edges, changed sources (by ascending
// source, each over its kept out-edges), inserted edges.  The grouping is stable, so every target
// sees its events in that order: among the events that carry a row, the changed sources come first
// and in ascending id order, which is what lets the max / min kernel drop the id comparison of ties
// until the first inserted edge shows up (consume_batch in agg.hip).
// seed i of the applied edge changes: deletions first, then insertions; key = target
__device__ __forceinline__ void seed_event(int i, const int32_t *del_s, const int32_t *del_d, const int32_t *ins_s,
                                           const int32_t *ins_d, int n_del, uint32_t *key, uint32_t *val) {
  if (i < n_del) { *key = (uint32_t)del_d[i]; *val = (EV_DEL << kEvKindShift) | (uint32_t)del_s[i]; }
  else {
    int j = i - n_del;
    *key = (uint32_t)ins_d[j]; *val = (EV_ADD << kEvKindShift) | (uint32_t)ins_s[j];
  }
}

// deletions go to [0, n_del), insertions behind the n_chg events of the changed sources
__global__ void k_seed_events(const int32_t *del_s, const int32_t *del_d, const int32_t *ins_s, const int32_t *ins_d,
                              int n_del, int n_ins, int64_t n_chg, uint32_t *key, uint32_t *val) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_del + n_ins) return;
  const int64_t p = i < n_del ? i : i + n_chg;
  seed_event((int)i, del_s, del_d, ins_s, ins_d, n_del, &key[p], &val[p]);
}

// out-edges of a changed source that exist in both snapshots: the block minus the ids appended
// by this batch
struct KeptOutDeg {
  const int32_t *F; const int32_t *deg; const int32_t *new_out;
  const int32_t *n_dev;      // optional device-side length of F (the launch may cover more)
  __device__ int operator()(int64_t i) const {
    if (n_dev && i >= *n_dev) return 0;
    int u = F[i];
    return deg[u] - new_out[u];
  }
};
struct StorePref { int32_t *p; __device__ void operator()(int64_t i, int, int ex) const { p[i] = ex; } };

// propagated event e: source = the changed node owning it, target = its e-th kept out-neighbour.
// payload_index: store the position in F instead of the node id.
__device__ __forceinline__ void expand_event(int e, const int32_t *F, int nF, const int32_t *pref, const int64_t *off,
                                             const int32_t *ids, int payload_index, uint32_t *key, uint32_t *val) {
  int lo = 0, hi = nF - 1;
  while (lo < hi) {
    int mid = (lo + hi + 1) >> 1;
    if (pref[mid] <= e) lo = mid; else hi = mid - 1;
  }
  int u = F[lo];
  int p = e - pref[lo];
  *key = (uint32_t)ids[off[u] + p];
  *val = (EV_CHG << kEvKindShift) | (uint32_t)(payload_index ? lo : u);
}

// A wave creates kExpandPerWave consecutive events.  It finds the sources of its first and last
// event with two wave-wide searches (64 probes per round); a lane then looks for the source of each
// of its events only between those two, usually one or two candidates, instead of searching the
// whole prefix array once per event.
constexpr int kExpandPerWave = 4 * kWave;
__global__ __launch_bounds__(256) void k_expand_events(const int32_t *F, int nF, const int32_t *pref, int n_ev,
                                                       const int64_t *off, const int32_t *ids, uint32_t *key,
                                                       uint32_t *val, int payload_index) {
  const int l = lane_id();
  const int64_t wv = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / kWave;
  const int64_t e_base = wv * kExpandPerWave;
  if (e_base >= n_ev) return;
  const int e_end = (int)(e_base + kExpandPerWave < n_ev ? e_base + kExpandPerWave : n_ev);
  const int lo = wave_last_le(pref, nF, (int)e_base);                      // pref[0] = 0 <= every event
  const int hi = lo + wave_last_le(pref + lo, nF - lo, e_end - 1);         // pref[lo] <= e_base <= e_end - 1
  for (int e = (int)e_base + l; e < e_end; e += kWave) {
    int a = lo, b = hi;
    while (a < b) {
      int mid = (a + b + 1) >> 1;
      if (pref[mid] <= e) a = mid; else b = mid - 1;
    }
    const int u = F[a];
    key[e] = (uint32_t)ids[off[u] + (e - pref[a])];
    val[e] = (EV_CHG << kEvKindShift) | (uint32_t)(payload_index ? a : u);
  }
}

// The counters reach the host through pinned host memory: one wave writes the slots and the
// stripe totals, then a sequence number that the host polls.  A blocking stream synchronisation
// costs an interrupt round trip per read-back, and a short batch has four of them.  The loads
// bypass the L1 so that a workgroup may publish what its own threads stored before a barrier.
__device__ __forceinline__ void publish_wave(const Counters *d, HostCounters *h, uint32_t *h_seq, uint32_t seq) {
  const int l = lane_id();
  if (l < 32) h->v[l] = __hip_atomic_load(&d->v[l], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
  for (int w = 0; w < ST_N; w++) {
    unsigned long long t = __hip_atomic_load(&d->stripe[l][w], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    for (int o = 32; o > 0; o >>= 1) t += __shfl_xor(t, o, kWave);
    if (l == 0) h->total[w] = t;
  }
  __threadfence_system();
  if (l == 0) __hip_atomic_store(h_seq, seq, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
}
static_assert(kStripes == kWave, "one stripe per lane");

__global__ __launch_bounds__(64) void k_publish(const Counters *d, HostCounters *h, uint32_t *h_seq, uint32_t seq) {
  publish_wave(d, h, h_seq, seq);
}

// A layer with few events (at most THREADS * ITEMS): clearing the counters, creating the events,
// grouping them by target (stable, so deletions stay ahead of changes ahead of insertions) and
// the segment heads in one workgroup.  Output as from the separate kernels: val in grouped
// order, the distinct targets, the start of each target's events plus the closing offset, and
// the target count in the counter block.
template <int THREADS, int ITEMS>
__global__ __launch_bounds__(THREADS) void k_small_group(const int32_t *del_s, const int32_t *del_d, const int32_t *ins_s,
                                                         const int32_t *ins_d, int n_del, int n_ins, const int32_t *F,
                                                         int nF, const int32_t *pref, int n_chg, const int64_t *off,
                                                         const int32_t *ids, int payload_index, int passes,
                                                         uint32_t *key_out, uint32_t *val_out, int32_t *t_list,
                                                         int32_t *t_seg, Counters *cnt) {
  __shared__ SmallSortLds<THREADS, ITEMS> S;
  __shared__ int sm[THREADS / kWave + 1];
  {
    int32_t *z = (int32_t *)cnt;
    for (int i = threadIdx.x; i < (int)(sizeof(Counters) / sizeof(int32_t)); i += THREADS)
      if (i != C_NT) z[i] = 0;
  }
  const int n_seed = n_del + n_ins, nE = n_seed + n_chg;
  for (int e = threadIdx.x; e < nE; e += THREADS) {
    uint32_t k, v;
    if (e < n_del) seed_event(e, del_s, del_d, ins_s, ins_d, n_del, &k, &v);
    else if (e < n_del + n_chg) expand_event(e - n_del, F, nF, pref, off, ids, payload_index, &k, &v);
    else seed_event(e - n_chg, del_s, del_d, ins_s, ins_d, n_del, &k, &v);
    S.sk[e] = k; S.sv[e] = v;
  }
  small_sort_lds<THREADS, ITEMS>(S, nE, passes);
  const int t0 = threadIdx.x * ITEMS;
  int h[ITEMS], c = 0;
#pragma unroll
  for (int k = 0; k < ITEMS; k++) {
    int i = t0 + k;
    h[k] = i < nE && (i == 0 || S.sk[i] != S.sk[i - 1]);
    c += h[k];
    if (i < nE) { key_out[i] = S.sk[i]; val_out[i] = S.sv[i]; }
  }
  int nT;
  int ex = block_excl_scan<THREADS>(c, sm, &nT);
#pragma unroll
  for (int k = 0; k < ITEMS; k++)
    if (h[k]) { t_list[ex] = (int32_t)S.sk[t0 + k]; t_seg[ex] = t0 + k; ex++; }
  if (threadIdx.x == 0) { t_seg[nT] = nE; cnt->v[C_NT] = nT; }
}

// The rows a layer with few events has to transform, in one workgroup: the targets whose bit the
// aggregation set in the bitmap (the bits are cleared on the way), the sources F (self term) and
// the nodes D whose in-degree changed, sorted and made unique -> rows[], their number -> C_NC.
// Also clears the first n_flags bytes of flag (the transform sets the flags of changed rows).
// n_t_bound + nF + nD is at most THREADS * ITEMS.
template <int THREADS, int ITEMS>
__global__ __launch_bounds__(THREADS) void k_small_collect(const int32_t *t_list, const int32_t *n_t_dev, int n_t_bound,
                                                           unsigned long long *bm, const int32_t *F, int nF,
                                                           const int32_t *D, int nD, int passes, int32_t *rows,
                                                           uint8_t *flag, int n_flags, Counters *cnt) {
  __shared__ SmallSortLds<THREADS, ITEMS> S;
  __shared__ int sm[THREADS / kWave + 1];
  for (int i = threadIdx.x; i < n_flags; i += THREADS) flag[i] = 0;
  const int nT = n_t_bound > 0 ? min(*n_t_dev, n_t_bound) : 0;
  const int M = n_t_bound + nF + nD;
  const int t0 = threadIdx.x * ITEMS;
  int id[ITEMS], c = 0;
#pragma unroll
  for (int k = 0; k < ITEMS; k++) {
    int i = t0 + k;
    id[k] = -1;
    if (i < n_t_bound) {
      if (i < nT) {
        int v = t_list[i];
        unsigned long long bit = 1ull << (v & 63);
        if (atomicAnd(&bm[v >> 6], ~bit) & bit) id[k] = v;
      }
    } else if (i < n_t_bound + nF) id[k] = F[i - n_t_bound];
    else if (i < M) id[k] = D[i - n_t_bound - nF];
    c += id[k] >= 0;
  }
  int m;
  int ex = block_excl_scan<THREADS>(c, sm, &m);
#pragma unroll
  for (int k = 0; k < ITEMS; k++)
    if (id[k] >= 0) { S.sk[ex] = (uint32_t)id[k]; S.sv[ex] = 0; ex++; }
  small_sort_lds<THREADS, ITEMS>(S, m, passes);
  int h[ITEMS];
  c = 0;
#pragma unroll
  for (int k = 0; k < ITEMS; k++) {
    int i = t0 + k;
    h[k] = i < m && (i == 0 || S.sk[i] != S.sk[i - 1]);
    c += h[k];
  }
  int nC;
  ex = block_excl_scan<THREADS>(c, sm, &nC);
#pragma unroll
  for (int k = 0; k < ITEMS; k++)
    if (h[k]) rows[ex++] = (int32_t)S.sk[t0 + k];
  if (threadIdx.x == 0) cnt->v[C_NC] = nC;
}

// The emission of a layer with few transformed rows (at most THREADS * ITEMS) in one workgroup:
// rows whose flag is set -> their positions (idx) and ids (f_list), the count, and, with
// want_events, the exclusive prefix of their kept out-degrees and its total.
template <int THREADS, int ITEMS>
__global__ __launch_bounds__(THREADS) void k_small_emit(const uint8_t *flag, const int32_t *rows, int nC, int32_t *idx,
                                                        int32_t *f_list, int want_events, const int32_t *deg,
                                                        const int32_t *new_out, int32_t *f_pref, Counters *cnt,
                                                        HostCounters *h, uint32_t *h_seq, uint32_t seq) {
  __shared__ int s_f[THREADS * ITEMS];
  __shared__ int sm[THREADS / kWave + 1];
  const int t0 = threadIdx.x * ITEMS;
  int f[ITEMS], c = 0;
#pragma unroll
  for (int k = 0; k < ITEMS; k++) {
    int i = t0 + k;
    f[k] = i < nC && flag[i] != 0;
    c += f[k];
  }
  int nF;
  int ex = block_excl_scan<THREADS>(c, sm, &nF);
#pragma unroll
  for (int k = 0; k < ITEMS; k++)
    if (f[k]) { int u = rows[t0 + k]; idx[ex] = t0 + k; f_list[ex] = u; s_f[ex] = u; ex++; }
  if (threadIdx.x == 0) cnt->v[C_NEXT] = nF;
  if (!want_events) {
    __threadfence();
    __syncthreads();
    if (threadIdx.x < kWave) publish_wave(cnt, h, h_seq, seq);
    return;
  }
  __syncthreads();
  int kd[ITEMS];
  c = 0;
#pragma unroll
  for (int k = 0; k < ITEMS; k++) {
    int i = t0 + k;
    kd[k] = i < nF ? deg[s_f[i]] - new_out[s_f[i]] : 0;
    c += kd[k];
  }
  int n_ev;
  ex = block_excl_scan<THREADS>(c, sm, &n_ev);
#pragma unroll
  for (int k = 0; k < ITEMS; k++) {
    if (t0 + k < nC) f_pref[t0 + k] = ex;
    ex += kd[k];
  }
  if (threadIdx.x == 0) cnt->v[C_NEV] = n_ev;
  __threadfence();
  __syncthreads();
  if (threadIdx.x < kWave) publish_wave(cnt, h, h_seq, seq);
}

__global__ void k_mark_nodes(const int32_t *list, int n, uint64_t *bm) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) { int v = list[i]; atomicOr((unsigned long long *)&bm[v >> 6], 1ull << (v & 63)); }
}

__global__ void k_gather_i32(const int32_t *table, const int32_t *idx, int n, const int32_t *n_dev, int32_t *out) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (n_dev) n = *n_dev;
  if (i < n) out[i] = table[idx[i]];
}

__global__ void k_gather_rows(const float *table, int ld, int d, const int32_t *rows, int64_t n, const int32_t *n_dev,
                              float *out) {
  int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (n_dev) n = *n_dev;
  int64_t r = t / d;
  int k = (int)(t % d);
  if (r < n) out[r * d + k] = table[(int64_t)rows[r] * ld + k];
}

// the same, 16 bytes per thread, for d a multiple of 4
__global__ void k_gather_rows4(const float *table, int ld, int d4, const int32_t *rows, int64_t n, const int32_t *n_dev,
                               float *out) {
  int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (n_dev) n = *n_dev;
  int64_t r = t / d4;
  int k = (int)(t - r * d4);
  if (r < n)
    reinterpret_cast<float4 *>(out)[r * d4 + k] = *reinterpret_cast<const float4 *>(table + (int64_t)rows[r] * ld + 4 * k);
}

// n bounds the row count (and sizes the launch); with n_dev the exact count is read on the device
static void gather_rows(hipStream_t s, const float *table, int ld, int d, const int32_t *rows, int64_t n, float *out,
                        const int32_t *n_dev = nullptr) {
  if (n <= 0) return;
  if (d % 4 == 0)
    hipLaunchKernelGGL(k_gather_rows4, grid1(n * (d / 4)), dim3(256), 0, s, table, ld, d / 4, rows, n, n_dev, out);
  else hipLaunchKernelGGL(k_gather_rows, grid1(n * d), dim3(256), 0, s, table, ld, d, rows, n, n_dev, out);
}

__global__ void k_pack_rows(const void *table, int ld, int d, int64_t row0, int64_t nrows, void *out) {
  int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  int64_t r = t / d;
  int k = (int)(t % d);
  if (r < nrows) ((uint32_t *)out)[r * d + k] = ((const uint32_t *)table)[(row0 + r) * ld + k];
}

__global__ void k_unpack_rows(const float *in, int d, int ld, int64_t n, float *table) {
  int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  int64_t r = t / d;
  int k = (int)(t % d);
  if (r < n) table[r * ld + k] = in[r * d + k];
}

__global__ void k_iota_u32(uint32_t *out, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) out[i] = (uint32_t)i;
}

// adjacent equal keys in a sorted list -> *flag = 1
__global__ void k_any_adjacent_equal(const uint32_t *keys, int64_t n, int32_t *flag) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i + 1 < n && keys[i] == keys[i + 1]) *flag = 1;
}

// any id outside [0, n_nodes) (a negative id is a huge unsigned one) -> *flag = 1
__global__ void k_any_out_of_range(const uint32_t *ids, int64_t n, uint32_t n_nodes, int32_t *flag) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n && ids[i] >= n_nodes) *flag = 1;
}

// New input features for the nodes ids[i] (ascending); the caller's row of ids[i] is rows[perm[i]].
// Writes the feature table with compare-and-emit: flag[i] = 1 if the row changed bitwise,
// old_rows[i] = the previous row (optional), dense[i] = the new row padded to ld (optional).
__global__ void k_set_features(const uint32_t *ids, const uint32_t *perm, int64_t n, const float *rows, int d, float *X,
                               int ld, float *old_rows, float *dense, uint8_t *flag, int32_t *list) {
  int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  int64_t i = t / ld;
  int k = (int)(t % ld);
  if (i >= n) return;
  int64_t v = ids[i];
  if (k == 0) list[i] = (int32_t)v;
  float nv = k < d ? rows[(int64_t)perm[i] * d + k] : 0.f;
  float o = X[v * ld + k];
  if (old_rows) old_rows[i * ld + k] = o;
  if (dense) dense[i * ld + k] = nv;
  if (__float_as_uint(o) != __float_as_uint(nv)) {
    X[v * ld + k] = nv;
    flag[i] = 1;
  }
}

__global__ void k_gather_rows_ld(const float *in, int ld, const int32_t *idx, int64_t n, const int32_t *n_dev,
                                 float *out) {
  // out[i][:] = in[idx[i]][:], both with row stride ld (a multiple of 4): 16 bytes per thread
  const int ld4 = ld >> 2;
  int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  int64_t r = t / ld4;
  int k = (int)(t - r * ld4);
  if (n_dev) n = *n_dev;
  if (r < n)
    reinterpret_cast<float4 *>(out)[r * ld4 + k] = *reinterpret_cast<const float4 *>(in + (int64_t)idx[r] * ld + 4 * k);
}

__device__ __forceinline__ float gcn_coef(int indeg) {      // (indeg + 1)^(-1/2)
  return __fdiv_rn(1.0f, __fsqrt_rn((float)(indeg + 1)));
}

__global__ void k_gcn_coef_all(const int32_t *deg, int n, float *cnorm) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) cnorm[i] = gcn_coef(deg[i]);
}

// scaled = c_v * raw for the nodes in `nodes` (null: all); optionally keeps the old scaled rows
// and flags rows that changed bitwise (flag must be pre-zeroed)
__global__ void k_gcn_rescale(const int32_t *nodes, int64_t n, const int32_t *deg, float *cnorm, const float *raw,
                              float *scaled, int ld, int d, float *old_rows, uint8_t *flag) {
  int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  int64_t i = t / ld;
  int k = (int)(t % ld);
  if (i >= n) return;
  int v = nodes ? nodes[i] : (int)i;
  float cv = gcn_coef(deg[v]);
  if (k == 0) cnorm[v] = cv;
  float o = scaled[(int64_t)v * ld + k];
  float nv = k < d ? __fmul_rn(cv, raw[(int64_t)v * ld + k]) : 0.f;
  if (old_rows) old_rows[i * ld + k] = o;
  if (__float_as_uint(o) != __float_as_uint(nv)) {
    scaled[(int64_t)v * ld + k] = nv;
    if (flag) flag[i] = 1;
  }
}

// last GCN layer: h = act(c_v (S + own scaled message) + b) for the listed rows, compare-and-emit
__global__ void k_gcn_final(const int32_t *rows, int64_t n, const float *S, const float *Msc, const float *cnorm,
                            const float *bias, const float *user, int ld_user, int relu, float *H, int ld, int d,
                            uint8_t *flag) {
  int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  int64_t i = t / ld;
  int k = (int)(t % ld);
  if (i >= n || k >= d) return;
  int64_t v = rows ? rows[i] : i;
  float x = __fmul_rn(cnorm[v], __fadd_rn(S[v * ld + k], Msc[v * ld + k]));
  if (bias) x = __fadd_rn(x, bias[k]);
  if (user) x = __fadd_rn(x, user[v * ld_user + k]);
  if (relu) x = x > 0.f ? x : 0.f;
  float o = H[v * ld + k];
  if (__float_as_uint(o) != __float_as_uint(x)) {
    H[v * ld + k] = x;
    if (flag) flag[i] = 1;
  }
}

// ------------------------------------------------------------------------------------ helpers
static ink_status fail(ink_ctx *c, ink_status st, const std::string &msg) {
  if (c) c->err = msg; else g_create_err = msg;
  return st;
}

// An updating call that fails on the device side (allocation or HIP error) may have rewritten part of
// the graph store or of the cache: the context is then marked unusable and every later call but
// ink_last_error / ink_destroy returns INK_E_STATE.
static ink_status seal(ink_ctx *c, ink_status st) {
  if (st == INK_E_OOM || st == INK_E_DEVICE) c->broken = true;
  return st;
}
static const char *kBrokenMsg = "the context is unusable after a failed update (INK_E_OOM / INK_E_DEVICE): destroy it";

static hipError_t wait_published(ink_ctx *c, uint32_t seq);

static hipError_t alloc_table(Table &t, int64_t n, int d) {
  // rows start on 64-byte boundaries: a gathered row then touches the fewest cache lines (config 2,
  // 41-wide rows: 176 -> 192 bytes per row and 5 % less aggregation time; 128-byte alignment loses
  // that again to the larger table)
  t.d = d;
  t.ld = round_up(d, 16);
  size_t bytes = (size_t)n * t.ld * 4;
  hipError_t e = hipMalloc(&t.p, bytes);
  if (e != hipSuccess) return e;
  return hipMemset(t.p, 0, bytes);
}

// uploads rows [row_off, row_off + K) of a weight matrix W ([K][N], host or device) into the
// zero-initialised padded device matrix `dst` ([Kp][Np] elements) in the order the transform
// kernel stages it (xform_weight_index)
static hipError_t upload_padded(const float *src, int K, int N, int Kp, int Np, int row_off, float *dst, bool src_dev) {
  std::vector<float> h((size_t)K * N);
  hipError_t e = hipMemcpy(h.data(), src, h.size() * 4, src_dev ? hipMemcpyDeviceToHost : hipMemcpyHostToHost);
  if (e != hipSuccess) return e;
  std::vector<float> p((size_t)Kp * Np);
  e = hipMemcpy(p.data(), dst, p.size() * 4, hipMemcpyDeviceToHost);
  if (e != hipSuccess) return e;
  for (int k = 0; k < K; k++)
    for (int j = 0; j < N; j++) p[xform_weight_index(row_off + k, j, Np)] = h[(size_t)k * N + j];
  return hipMemcpy(dst, p.data(), p.size() * 4, hipMemcpyHostToDevice);
}

static hipError_t upload_vec(const float *src, int n, float **dst, bool src_dev) {
  if (!src) { *dst = nullptr; return hipSuccess; }
  hipError_t e = hipMalloc((void **)dst, (size_t)round_up(n, 32) * 4);
  if (e != hipSuccess) return e;
  e = hipMemset(*dst, 0, (size_t)round_up(n, 32) * 4);
  if (e != hipSuccess) return e;
  return hipMemcpy(*dst, src, (size_t)n * 4, src_dev ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice);
}

static void prof_collect(ink_ctx *c) {
  for (auto &p : c->ev_pending) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, p.a, p.b) == hipSuccess) {
      if (p.cls >= 0) c->stats.ms[p.cls] += ms;
      if (p.kern >= 0 && p.layer >= 1 && p.layer <= INK_MAX_LAYERS) c->stats.layer[p.layer - 1].ms_kernel[p.kern] += ms;
    }
    c->ev_free.push_back(p.a); c->ev_free.push_back(p.b);
  }
  c->ev_pending.clear();
}

hipError_t ink::read_counters(ink_ctx *c) {
  const uint32_t seq = ++c->pub_seq;
  hipLaunchKernelGGL(k_publish, dim3(1), dim3(64), 0, c->stream, (const Counters *)c->d_cnt, c->h_cnt, c->h_seq, seq);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return wait_published(c, seq);
}

// waits until the record with this sequence number has arrived: a short spin, then the blocking wait
static hipError_t wait_published(ink_ctx *c, uint32_t seq) {
  hipError_t e;
  const auto t0 = std::chrono::steady_clock::now();
  for (int spin = 0;; spin++) {
    if (__atomic_load_n(c->h_seq, __ATOMIC_ACQUIRE) == seq) return hipSuccess;
    if ((spin & 63) == 63 &&
        std::chrono::duration<double, std::micro>(std::chrono::steady_clock::now() - t0).count() > 150.0)
      break;
  }
  e = hipStreamSynchronize(c->stream);
  if (e != hipSuccess) return e;
  return __atomic_load_n(c->h_seq, __ATOMIC_ACQUIRE) == seq ? hipSuccess : hipErrorUnknown;
}

static const Table &msg_table(ink_ctx *c, int l) {   // m_l: h_{l-1} (aggregate first) or GCN's scaled h_{l-1} W_l
  return c->kind == INK_MODEL_GCN ? c->Msc[l] : c->H[l - 1];
}

static AggArgs agg_args(ink_ctx *c, int l) {       // layer l in 1..k
  AggArgs a;
  a.n = c->n;
  a.in_off = c->gin.off; a.in_deg = c->gin.deg; a.in_ids = c->gin.ids; a.in_asc = c->gin.asc;
  const Table &M = msg_table(c, l);
  a.M = M.f(); a.ldm = M.ld;
  a.A = c->A[l].f(); a.ARG = c->is_select ? c->ARG[l].i() : nullptr; a.ld = c->A[l].ld; a.d = c->A[l].d;
  a.UB = c->is_select ? c->UB[l].f() : nullptr;
  a.ARG2 = c->is_select ? c->ARG2[l].i() : nullptr;
  a.wd = round_up(a.d, 4);
  a.is_min = c->is_min;
  a.big_deg = kBigDeg;
  a.big_grid = 2 * c->big_hint[l] + 1024;
  a.count_cond = 1;
  a.layer = l;
  return a;
}

// dense combination of layer l for the rows in `rows` (null: all nodes).  With flags != null the
// layer's table is updated with compare-and-emit.
static hipError_t run_transform(ink_ctx *c, int l, const int32_t *rows, int64_t n_rows, uint8_t *flags,
                                float *old_rows = nullptr, const int32_t *n_rows_dev = nullptr) {
  const DevLayer &L = c->layers[l - 1];
  XformArgs x;
  memset(&x, 0, sizeof(x));
  x.rows = rows; x.n_rows = n_rows; x.n_rows_dev = n_rows_dev;
  x.old_rows = old_rows; x.ld_old = c->H[l].ld;
  if (c->agg == INK_AGG_MEAN) x.mean_deg = c->gin.deg;
  x.A = c->A[l].f(); x.lda = c->A[l].ld;
  x.Hp = c->H[l - 1].f(); x.ldh = c->H[l - 1].ld;
  x.d_in = L.in_dim; x.eps = c->eps;
  if (c->kind == INK_MODEL_SAGE) {
    x.mode = 0;
    x.W = L.W1; x.Kp = L.K1p; x.Np = L.N1p; x.bias = L.b1; x.n_out = L.out_dim; x.relu = L.act == INK_ACT_RELU;
    x.out = c->H[l].f(); x.ld_out = c->H[l].ld; x.to_table = 1; x.row_changed = flags;
    x.user = c->USER[l].f(); x.ld_user = c->USER[l].ld;
    return xform_run(c, x);
  }
  // GIN: two linear maps through a staging buffer
  hipError_t e = c->stage0.reserve((size_t)n_rows * L.N1p * 4);
  if (e != hipSuccess) return e;
  x.mode = 1;
  x.W = L.W1; x.Kp = L.K1p; x.Np = L.N1p; x.bias = L.b1; x.n_out = L.hidden; x.relu = 1;
  x.out = c->stage0.as<float>(); x.ld_out = L.N1p; x.to_table = 0; x.old_rows = nullptr;
  e = xform_run(c, x);
  if (e != hipSuccess) return e;
  XformArgs y;
  memset(&y, 0, sizeof(y));
  y.mode = 2; y.rows = rows; y.n_rows = n_rows; y.n_rows_dev = n_rows_dev;
  y.Hp = c->stage0.as<float>(); y.ldh = L.N1p; y.d_in = L.hidden;
  y.W = L.W2; y.Kp = L.K2p; y.Np = L.N2p; y.bias = L.b2; y.n_out = L.out_dim; y.relu = L.act == INK_ACT_RELU;
  y.out = c->H[l].f(); y.ld_out = c->H[l].ld; y.to_table = 1; y.row_changed = flags; y.out_rows = rows;
  y.old_rows = old_rows; y.ld_old = c->H[l].ld;
  y.user = c->USER[l].f(); y.ld_user = c->USER[l].ld;
  return xform_run(c, y);
}

// ------------------------------------------------------------------------------------ static work memory
// Work memory of ink_full_infer_noalloc: the list of long rows, its chunk prefix, the partial rows
// of the chunks, the block sums of the scan that plans them and GIN's staging rows.  One array per
// GPU for the life of the process, shared by every call on that GPU.  Nothing in it has to start
// from zero: every part is written by the launch that reads it afterwards.
static __device__ __align__(256) unsigned char scratch[INK_NOALLOC_SCRATCH_BYTES];

// device address of `scratch` per GPU, looked up once with that GPU current (ink_create does it);
// host code uses these pointers, never the array's name
constexpr int kMaxDevices = 64;
static void *g_scratch_ptr[kMaxDevices];
static std::mutex g_scratch_mu;

static hipError_t scratch_lookup(int *dev_out, void **ptr_out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    g_scratch_ptr[dev] = p;
  }
  if (dev_out) *dev_out = dev;
  if (ptr_out) *ptr_out = g_scratch_ptr[dev];
  return hipSuccess;
}

static inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// ------------------------------------------------------------------------------------ create
// Event records of a layer are addressed with 32-bit offsets: at most one per edge plus one per
// list entry of the batch (below 2^30), so the edge count is held below 2^31 - 2^30.
constexpr int64_t kMaxEdges = (1ll << 31) - (1ll << 30) - 1;

static ink_status validate_model(const ink_model *m, int feat_dim, std::string &why) {
  if (m->n_layers < 1 || m->n_layers > INK_MAX_LAYERS || !m->layers) { why = "n_layers out of range or layers NULL"; return INK_E_ARG; }
  if (m->kind != INK_MODEL_SAGE && m->kind != INK_MODEL_GIN && m->kind != INK_MODEL_GCN) { why = "unknown model kind"; return INK_E_ARG; }
  if (m->agg < INK_AGG_MAX || m->agg > INK_AGG_GCN_SYM) { why = "unknown aggregator"; return INK_E_ARG; }
  if ((m->kind == INK_MODEL_GCN) != (m->agg == INK_AGG_GCN_SYM)) { why = "GCN needs INK_AGG_GCN_SYM (and only GCN takes it)"; return INK_E_ARG; }
  int d = feat_dim;
  for (int l = 0; l < m->n_layers; l++) {
    const ink_layer &L = m->layers[l];
    if (L.in_dim != d) { why = "layer in_dim does not match the previous width"; return INK_E_ARG; }
    int agg_w = m->kind == INK_MODEL_GCN ? L.out_dim : L.in_dim;      // GCN aggregates after the linear map
    (void)agg_w;
    if (L.in_dim < 1 || L.out_dim < 1 || L.out_dim > INK_MAX_OUT_DIM || L.in_dim > INK_MAX_IN_DIM) { why = "layer width out of range"; return INK_E_ARG; }
    if (!L.W_neigh) { why = "W_neigh is NULL"; return INK_E_ARG; }
    if (m->kind == INK_MODEL_SAGE && !L.W_self) { why = "GraphSAGE needs W_self"; return INK_E_ARG; }
    if (m->kind == INK_MODEL_GIN && (!L.W_mlp2 || L.mlp_hidden < 1 || L.mlp_hidden > 256)) { why = "GIN needs W_mlp2 and 1 <= mlp_hidden <= 256"; return INK_E_ARG; }
    if (L.act != INK_ACT_NONE && L.act != INK_ACT_RELU) { why = "unknown activation"; return INK_E_ARG; }
    d = L.out_dim;
  }
  return INK_OK;
}

extern "C" ink_status ink_create(const ink_csr *g, const float *features, int32_t feat_dim, const ink_model *model,
                                 const ink_options *opts, ink_ctx **out) {
  if (out) *out = nullptr;
  if (!g || !features || !model || !out || !g->rowptr || (g->n_edges > 0 && !g->col))
    return fail(nullptr, INK_E_ARG, "ink_create: NULL argument");
  if (g->n_nodes < 1 || g->n_edges < 0 || feat_dim < 1 || g->n_nodes >= (1 << 30))
    return fail(nullptr, INK_E_ARG, "ink_create: bad n_nodes / n_edges / feat_dim");
  std::string why;
  ink_status st = validate_model(model, feat_dim, why);
  if (st != INK_OK) return fail(nullptr, st, "ink_create: " + why);
  const bool dev = opts && opts->mem == INK_MEM_DEVICE;
  const int n = g->n_nodes;
  const int64_t E = g->n_edges;
  if (E > kMaxEdges) return fail(nullptr, INK_E_ARG, "ink_create: more than 2^31 - 2^30 edges (event offsets are 32-bit)");
  // graph to the host (validation and block layout are host work)
  std::vector<int64_t> rowptr((size_t)n + 1);
  std::vector<int32_t> col((size_t)E);
  if (hipMemcpy(rowptr.data(), g->rowptr, rowptr.size() * 8, dev ? hipMemcpyDeviceToHost : hipMemcpyHostToHost) != hipSuccess ||
      (E && hipMemcpy(col.data(), g->col, col.size() * 4, dev ? hipMemcpyDeviceToHost : hipMemcpyHostToHost) != hipSuccess))
    return fail(nullptr, INK_E_DEVICE, "ink_create: cannot read the graph arrays");
  if (rowptr[0] != 0 || rowptr[n] != E) return fail(nullptr, INK_E_ARG, "ink_create: rowptr[0] != 0 or rowptr[n] != n_edges");
  for (int v = 0; v < n; v++) {
    if (rowptr[v + 1] < rowptr[v]) return fail(nullptr, INK_E_ARG, "ink_create: rowptr not monotone");
    for (int64_t e = rowptr[v]; e < rowptr[v + 1]; e++) {
      int32_t u = col[e];
      if (u < 0 || u >= n) return fail(nullptr, INK_E_RANGE, "ink_create: column id out of range");
      if (u == v) return fail(nullptr, INK_E_ARG, "ink_create: self loop in the graph");
      if (e > rowptr[v] && col[e - 1] >= u) return fail(nullptr, INK_E_ARG, "ink_create: row not strictly ascending");
    }
  }
  if (opts && opts->node_capacity >= (1 << 30)) return fail(nullptr, INK_E_ARG, "ink_create: node_capacity too large");
  ink_ctx *c = new (std::nothrow) ink_ctx();
  if (!c) return fail(nullptr, INK_E_OOM, "ink_create: host allocation failed");
  c->n = n; c->n_edges = E; c->n_edges_now = E;
  c->n_cap = (opts && opts->node_capacity > n) ? opts->node_capacity : n;
  c->id_bits = 1; while ((1ll << c->id_bits) < c->n_cap) c->id_bits++;
  c->kind = model->kind; c->agg = model->agg; c->n_layers = model->n_layers; c->eps = model->gin_eps;
  c->is_select = model->agg == INK_AGG_MAX || model->agg == INK_AGG_MIN; c->is_min = model->agg == INK_AGG_MIN;
  c->mem = dev ? INK_MEM_DEVICE : INK_MEM_HOST;
  c->slack = (opts && opts->slack_factor > 0.f) ? opts->slack_factor : 0.25f;
  c->profile = opts ? opts->profile : 0;
  c->pool_reserve = opts ? opts->pool_reserve : 0;
  if (opts && opts->small_batch_limit != 0)
    c->small_batch = opts->small_batch_limit < 0 ? 0 : std::min<int64_t>(opts->small_batch_limit, 4096);
  c->batch_dev = dev || (opts && opts->batch_mem == INK_MEM_DEVICE);
  if (opts && opts->dense_threshold != 0.f) c->dense_frac = opts->dense_threshold < 0.f ? 1e30 : opts->dense_threshold;
  memset(&c->stats, 0, sizeof(c->stats));
#define CREATE_TRY(x)                                                                              \
  do {                                                                                             \
    hipError_t e_ = (x);                                                                           \
    if (e_ != hipSuccess) {                                                                        \
      g_create_err = std::string("ink_create: HIP error: ") + hipGetErrorString(e_) + " at " #x;   \
      ink_destroy(c);                                                                              \
      return e_ == hipErrorOutOfMemory ? INK_E_OOM : INK_E_DEVICE;                                 \
    }                                                                                              \
  } while (0)
  if (opts && opts->hip_stream) c->stream = (hipStream_t)opts->hip_stream;
  else { CREATE_TRY(hipStreamCreate(&c->stream)); c->own_stream = true; }
  CREATE_TRY(scratch_lookup(&c->device, &c->scratch));
  CREATE_TRY(graph_build(c, rowptr.data(), col.data()));
  const int64_t nc = c->n_cap;     // every per-node array is allocated for the capacity
  CREATE_TRY(hipMalloc(&c->new_out, (size_t)nc * 4));
  CREATE_TRY(hipMemset(c->new_out, 0, (size_t)nc * 4));
  CREATE_TRY(hipMalloc(&c->d_cnt, sizeof(Counters)));
  CREATE_TRY(hipMemset(c->d_cnt, 0, sizeof(Counters)));
  CREATE_TRY(hipHostMalloc((void **)&c->h_cnt, sizeof(HostCounters) + 64, hipHostMallocCoherent));
  memset(c->h_cnt, 0, sizeof(HostCounters) + 64);
  c->h_seq = reinterpret_cast<uint32_t *>(reinterpret_cast<char *>(c->h_cnt) + sizeof(HostCounters));
  size_t bmw = ((size_t)nc + 63) / 64;
  CREATE_TRY(hipMalloc(&c->bm_a, bmw * 8));
  CREATE_TRY(hipMemset(c->bm_a, 0, bmw * 8));
  if (opts && opts->max_batch > 0) {       // size the batch staging up front
    CREATE_TRY(c->b_raw.reserve((size_t)opts->max_batch * sizeof(ink_edge_update)));
    const size_t per = (((size_t)opts->max_batch + 64) * 4 + 255) / 256 * 256;
    CREATE_TRY(c->b_misc.reserve(per * 28));
    for (DevBuf *b : {&c->b_del_s, &c->b_del_d, &c->b_ins_s, &c->b_ins_d, &c->b_touch_in, &c->b_uniq}) CREATE_TRY(b->reserve(per));
    CREATE_TRY(c->c_list.reserve((size_t)nc * 4));
  }
  CREATE_TRY(c->big_list.reserve((size_t)(c->gin.pool_cap / kBigDeg + 4096) * 4));
  // tables
  c->H.resize(c->n_layers + 1); c->A.resize(c->n_layers + 1); c->ARG.resize(c->n_layers + 1);
  c->UB.resize(c->n_layers + 1); c->ARG2.resize(c->n_layers + 1);
  c->XW.resize(c->n_layers + 1); c->Msc.resize(c->n_layers + 1); c->USER.resize(c->n_layers + 1);
  if (c->kind == INK_MODEL_GCN) CREATE_TRY(hipMalloc(&c->cnorm, (size_t)nc * 4));
  CREATE_TRY(alloc_table(c->H[0], nc, feat_dim));
  {
    DevBuf tmp;
    const float *src = features;
    if (!dev) {
      CREATE_TRY(tmp.reserve((size_t)n * feat_dim * 4));
      CREATE_TRY(hipMemcpy(tmp.p, features, (size_t)n * feat_dim * 4, hipMemcpyHostToDevice));
      src = tmp.as<float>();
    }
    hipLaunchKernelGGL(k_unpack_rows, grid1((int64_t)n * feat_dim), dim3(256), 0, c->stream, src, (int)feat_dim,
                       c->H[0].ld, (int64_t)n, c->H[0].f());
    CREATE_TRY(hipStreamSynchronize(c->stream));
    tmp.release();
  }
  c->layers.resize(c->n_layers);
  for (int l = 1; l <= c->n_layers; l++) {
    const ink_layer &S = model->layers[l - 1];
    DevLayer &L = c->layers[l - 1];
    L.in_dim = S.in_dim; L.out_dim = S.out_dim; L.hidden = S.mlp_hidden; L.act = S.act;
    CREATE_TRY(alloc_table(c->H[l], nc, S.out_dim));
    CREATE_TRY(alloc_table(c->A[l], nc, c->kind == INK_MODEL_GCN ? S.out_dim : S.in_dim));
    if (c->is_select) { CREATE_TRY(alloc_table(c->ARG[l], nc, S.in_dim)); CREATE_TRY(alloc_table(c->UB[l], nc, S.in_dim)); CREATE_TRY(alloc_table(c->ARG2[l], nc, S.in_dim)); }
    if (c->kind == INK_MODEL_GCN) {
      CREATE_TRY(alloc_table(c->Msc[l], nc, S.out_dim));
      if (l == 1) CREATE_TRY(alloc_table(c->XW[1], nc, S.out_dim));
      L.K1 = S.in_dim; L.K1p = round_up(L.K1, 32); L.N1 = S.out_dim; L.N1p = round_up(L.N1, 32);
      CREATE_TRY(hipMalloc(&L.W1, (size_t)L.K1p * L.N1p * 4));
      CREATE_TRY(hipMemset(L.W1, 0, (size_t)L.K1p * L.N1p * 4));
      CREATE_TRY(upload_padded(S.W_neigh, S.in_dim, S.out_dim, L.K1p, L.N1p, 0, L.W1, dev));
      CREATE_TRY(upload_vec(S.bias, S.out_dim, &L.b1, dev));
    } else if (c->kind == INK_MODEL_SAGE) {
      L.K1 = 2 * S.in_dim; L.K1p = round_up(L.K1, 32); L.N1 = S.out_dim; L.N1p = round_up(L.N1, 32);
      CREATE_TRY(hipMalloc(&L.W1, (size_t)L.K1p * L.N1p * 4));
      CREATE_TRY(hipMemset(L.W1, 0, (size_t)L.K1p * L.N1p * 4));
      CREATE_TRY(upload_padded(S.W_neigh, S.in_dim, S.out_dim, L.K1p, L.N1p, 0, L.W1, dev));
      CREATE_TRY(upload_padded(S.W_self, S.in_dim, S.out_dim, L.K1p, L.N1p, S.in_dim, L.W1, dev));
      CREATE_TRY(upload_vec(S.bias, S.out_dim, &L.b1, dev));
    } else {   // GIN
      L.K1 = S.in_dim; L.K1p = round_up(L.K1, 32); L.N1 = S.mlp_hidden; L.N1p = round_up(L.N1, 32);
      L.K2 = S.mlp_hidden; L.K2p = round_up(L.K2, 32); L.N2 = S.out_dim; L.N2p = round_up(L.N2, 32);
      CREATE_TRY(hipMalloc(&L.W1, (size_t)L.K1p * L.N1p * 4));
      CREATE_TRY(hipMemset(L.W1, 0, (size_t)L.K1p * L.N1p * 4));
      CREATE_TRY(upload_padded(S.W_neigh, S.in_dim, S.mlp_hidden, L.K1p, L.N1p, 0, L.W1, dev));
      CREATE_TRY(upload_vec(S.bias, S.mlp_hidden, &L.b1, dev));
      CREATE_TRY(hipMalloc(&L.W2, (size_t)L.K2p * L.N2p * 4));
      CREATE_TRY(hipMemset(L.W2, 0, (size_t)L.K2p * L.N2p * 4));
      CREATE_TRY(upload_padded(S.W_mlp2, S.mlp_hidden, S.out_dim, L.K2p, L.N2p, 0, L.W2, dev));
      CREATE_TRY(upload_vec(S.bias_mlp2, S.out_dim, &L.b2, dev));
    }
  }
  *out = c;
  return INK_OK;
}

extern "C" void ink_destroy(ink_ctx *c) {
  if (!c) return;
  if (c->stream) (void)hipStreamSynchronize(c->stream);
  for (GraphSide *g : {&c->gin, &c->gout}) {
    if (g->off) (void)hipFree(g->off);
    if (g->deg) (void)hipFree(g->deg);
    if (g->cap) (void)hipFree(g->cap);
    if (g->asc) (void)hipFree(g->asc);
    if (g->ids) (void)hipFree(g->ids);
  }
  if (c->new_out) (void)hipFree(c->new_out);
  for (auto &L : c->layers) for (float *p : {L.W1, L.b1, L.W2, L.b2}) if (p) (void)hipFree(p);
  for (auto *vec : {&c->H, &c->A, &c->ARG, &c->UB, &c->ARG2, &c->XW, &c->Msc, &c->USER}) for (auto &t : *vec) if (t.p) (void)hipFree(t.p);
  if (c->cnorm) (void)hipFree(c->cnorm);
  if (c->d_cnt) (void)hipFree(c->d_cnt);
  if (c->h_cnt) (void)hipHostFree(c->h_cnt);
  if (c->bm_a) (void)hipFree(c->bm_a);
  for (DevBuf *b : {&c->ws.blk, &c->ws.hist, &c->ws.tmpk, &c->ws.tmpv, &c->b_raw, &c->b_misc, &c->b_uniq, &c->b_del_s,
                    &c->b_del_d, &c->b_ins_s, &c->b_ins_d, &c->f_list[0], &c->f_list[1], &c->f_old[0], &c->f_old[1],
                    &c->f_pref, &c->ev_key, &c->ev_val, &c->t_list, &c->t_seg, &c->c_list, &c->c_flag, &c->c_idx, &c->c_old,
                    &c->b_touch_in,
                    &c->u_ev, &c->u_rows, &c->u_key, &c->u_val, &c->u_uniq, &c->u_seg, &c->u_flag, &c->u_idx, &c->u_list, &c->exp_list, &c->big_list, &c->big_part_v, &c->big_part_i, &c->big_part_s, &c->big_part_j, &c->big_pref, &c->f_delta, &c->stage0, &c->stage1, &c->res_ids, &c->res_emb})
    b->release();
  for (auto e : c->ev_free) (void)hipEventDestroy(e);
  for (auto &p : c->ev_pending) { (void)hipEventDestroy(p.a); (void)hipEventDestroy(p.b); }
  if (c->own_stream && c->stream) (void)hipStreamDestroy(c->stream);
  delete c;
}

extern "C" const char *ink_last_error(const ink_ctx *c) { return c ? c->err.c_str() : g_create_err.c_str(); }

// ------------------------------------------------------------------------------------ full inference
// Aggregated rows wider than one wave covers (256 floats) are handled one 256-column block at a
// time: the aggregators act per dimension, so the blocks are independent.
constexpr int kAggBlock = 256;
static int agg_blocks(const AggArgs &a) { return (a.d + kAggBlock - 1) / kAggBlock; }
static AggArgs agg_block(const AggArgs &a, int b) {
  AggArgs r = a;
  int c0 = b * kAggBlock;
  r.M += c0; r.A += c0;
  if (r.ARG) { r.ARG += c0; r.UB += c0; r.ARG2 += c0; }
  r.d = std::min(kAggBlock, a.d - c0);
  r.wd = round_up(r.d, 4);
  r.count_cond = b == 0;      // a target's condition is tallied once, for its first block
  return r;
}

// recompute of every node (targets == null) or of the listed ones
static hipError_t agg_full_any(ink_ctx *c, const AggArgs &a_in, uint64_t *chg, const int32_t *targets = nullptr,
                               int64_t n_targets = -1) {
  AggArgs a = a_in;
  if (!targets) {        // every node: the chunk count is bounded by the edge count
    n_targets = c->n;
    a.big_grid = c->n_edges_now / kBigChunk + std::min<int64_t>(c->n, c->n_edges_now / kBigDeg) + 1;
  }
  for (int b = 0; b < agg_blocks(a); b++) {
    AggArgs ab = agg_block(a, b);
    hipError_t e = c->is_select ? agg_select_full(c, ab, targets, n_targets, chg)
                                : agg_sum_full(c, ab, targets, n_targets, chg);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

// GCN: message table of layer l + 1 from the finished layer l (rows == null: every node):
// h_l = act(c (S_l + m_l) + b_l) is stored, then m_{l+1} = c * (h_l W_{l+1}) with compare-and-emit
static hipError_t gcn_next_messages(ink_ctx *c, int l, const int32_t *rows, int64_t n_rows, uint8_t *flags,
                                    float *old_rows) {
  const DevLayer &L = c->layers[l - 1], &Ln = c->layers[l];
  XformArgs x;
  memset(&x, 0, sizeof(x));
  x.mode = 3; x.rows = rows; x.n_rows = n_rows;
  x.A = c->A[l].f(); x.lda = c->A[l].ld; x.Hp = c->Msc[l].f(); x.ldh = c->Msc[l].ld; x.d_in = L.out_dim;
  x.cnorm = c->cnorm; x.in_bias = L.b1; x.in_relu = L.act == INK_ACT_RELU;
  x.in_user = c->USER[l].f(); x.ld_in_user = c->USER[l].ld;
  x.h_store = c->H[l].f(); x.ld_hs = c->H[l].ld;
  x.W = Ln.W1; x.Kp = Ln.K1p; x.Np = Ln.N1p; x.bias = nullptr; x.n_out = Ln.out_dim; x.relu = 0;
  x.out_scale = c->cnorm;
  x.out = c->Msc[l + 1].f(); x.ld_out = c->Msc[l + 1].ld; x.to_table = 1; x.row_changed = flags;
  x.old_rows = old_rows; x.ld_old = c->Msc[l + 1].ld;
  return xform_run(c, x);
}

static hipError_t gcn_final(ink_ctx *c, const int32_t *rows, int64_t n_rows, uint8_t *flags) {
  int k = c->n_layers;
  const DevLayer &L = c->layers[k - 1];
  if (n_rows <= 0) return hipSuccess;
  hipLaunchKernelGGL(k_gcn_final, grid1(n_rows * c->H[k].ld), dim3(256), 0, c->stream, rows, n_rows,
                     (const float *)c->A[k].f(), (const float *)c->Msc[k].f(), (const float *)c->cnorm,
                     (const float *)L.b1, (const float *)c->USER[k].f(), c->USER[k].ld, (int)(L.act == INK_ACT_RELU),
                     c->H[k].f(), c->H[k].ld, c->H[k].d, flags);
  return hipGetLastError();
}

static ink_status full_infer_impl(ink_ctx *c) {
  auto t0 = std::chrono::steady_clock::now();
  memset(&c->stats, 0, sizeof(c->stats));
  c->stats.n_layers = c->n_layers;
  hipStream_t s = c->stream;
  if (c->kind == INK_MODEL_GCN) {
    Prof p(c, INK_T_TRANSFORM);
    const DevLayer &L = c->layers[0];
    XformArgs x;
    memset(&x, 0, sizeof(x));
    x.mode = 2; x.n_rows = c->n; x.Hp = c->H[0].f(); x.ldh = c->H[0].ld; x.d_in = L.in_dim;
    x.W = L.W1; x.Kp = L.K1p; x.Np = L.N1p; x.n_out = L.out_dim;
    x.out = c->XW[1].f(); x.ld_out = c->XW[1].ld; x.to_table = 0;
    API_TRY(xform_run(c, x));
    hipLaunchKernelGGL(k_gcn_rescale, grid1((int64_t)c->n * c->Msc[1].ld), dim3(256), 0, s, (const int32_t *)nullptr,
                       (int64_t)c->n, (const int32_t *)c->gin.deg, c->cnorm, (const float *)c->XW[1].f(),
                       c->Msc[1].f(), c->Msc[1].ld, c->Msc[1].d, (float *)nullptr, (uint8_t *)nullptr);
    API_TRY(hipGetLastError());
  }
  for (int l = 1; l <= c->n_layers; l++) {
    AggArgs a = agg_args(c, l);
    { Prof p(c, INK_T_AGG); API_TRY(agg_full_any(c, a, nullptr)); }
    {
      Prof p(c, INK_T_TRANSFORM, l, INK_K_XFORM);
      if (c->kind != INK_MODEL_GCN) API_TRY(run_transform(c, l, nullptr, c->n, nullptr));
      else if (l < c->n_layers) API_TRY(gcn_next_messages(c, l, nullptr, c->n, nullptr, nullptr));
      else API_TRY(gcn_final(c, nullptr, c->n, nullptr));
    }
    ink_layer_stats &S = c->stats.layer[l - 1];
    S.dense = 1; S.n_targets = c->n; S.n_exposed = c->n; S.n_regather_nb = c->n_edges_now; S.n_transformed = c->n;
  }
  API_TRY(hipStreamSynchronize(s));
  prof_collect(c);
  c->inferred = true;
  c->stats.ms_total = std::chrono::duration<float, std::milli>(std::chrono::steady_clock::now() - t0).count();
  return INK_OK;
}

extern "C" ink_status ink_full_infer(ink_ctx *c) {
  if (!c) return INK_E_ARG;
  if (c->broken) return fail(c, INK_E_STATE, kBrokenMsg);
  return seal(c, full_infer_impl(c));
}

// ------------------------------------------------------------------------------------ full inference without allocation
extern "C" ink_status ink_full_infer_noalloc(ink_ctx *c) {
  if (!c) return INK_E_ARG;
  if (c->broken) return fail(c, INK_E_STATE, kBrokenMsg);
  void *base = c->scratch;
  if (!base) return fail(c, INK_E_DEVICE, "ink_full_infer_noalloc: the scratch array's address was not found at ink_create");
  // what the full inference reserves, from the same bounds its kernels' launchers use
  int wd_max = 0, n1p_max = 0;
  for (int l = 1; l <= c->n_layers; l++) {
    wd_max = std::max(wd_max, std::min(round_up(c->A[l].d, 4), kAggBlock));
    if (c->kind == INK_MODEL_GIN) n1p_max = std::max(n1p_max, c->layers[l - 1].N1p);
  }
  const size_t list_b = align256((size_t)big_rows_capacity(c) * 4);
  const size_t pref_b = align256((list_b / 4 + 1) * 4);
  const size_t part_b = align256((size_t)big_chunk_capacity(c) * wd_max * 4);
  const int n_part = c->is_select ? 4 : 1;
  const size_t blk_b = align256((size_t)nblocks((int64_t)(list_b / 4), kScanTile) * 4);
  const size_t stage_b = align256((size_t)c->n * n1p_max * 4);
  const size_t need = list_b + pref_b + (size_t)n_part * part_b + blk_b + stage_b;
  if (need > (size_t)INK_NOALLOC_SCRATCH_BYTES) {
    char msg[256];
    snprintf(msg, sizeof(msg), "ink_full_infer_noalloc: this graph and model need %zu bytes of work memory, the static "
             "scratch holds %zu: use ink_full_infer", need, (size_t)INK_NOALLOC_SCRATCH_BYTES);
    return fail(c, INK_E_RANGE, msg);
  }
  // lend the carve-outs to the buffers the kernels' launchers use, run, and put the owners back
  DevBuf *bufs[] = {&c->big_list, &c->big_pref, &c->big_part_v, &c->big_part_i, &c->big_part_s, &c->big_part_j,
                    &c->ws.blk, &c->stage0};
  const size_t sizes[] = {list_b, pref_b, part_b, c->is_select ? part_b : 0, c->is_select ? part_b : 0,
                          c->is_select ? part_b : 0, blk_b, stage_b};
  constexpr int NB = sizeof(bufs) / sizeof(bufs[0]);
  DevBuf saved[NB];
  size_t used = 0;
  for (int i = 0; i < NB; i++) {
    saved[i] = *bufs[i];
    bufs[i]->p = sizes[i] ? (char *)base + used : nullptr;
    bufs[i]->cap = sizes[i];
    bufs[i]->fixed = true;
    used += sizes[i];
  }
  const int profile = c->profile;
  c->profile = 0;                    // HIP events are created on demand: not in this call
  ink_status st = full_infer_impl(c);
  c->profile = profile;
  for (int i = 0; i < NB; i++) *bufs[i] = saved[i];
  return seal(c, st);
}

// ------------------------------------------------------------------------------------ updates
// Events + grouping + aggregation of layer l.  F (nF ids, ascending) are the sources whose message
// changed and n_chg the events they propagate (their kept out-edges, prefix already in f_pref);
// f_old holds their previous message rows (sum-type only).  Marks targets whose aggregate changed
// in c->bm_a.  Counters are read back by the caller's next synchronisation.
constexpr int64_t kSmallLayer = 4096;           // events / rows up to which a layer's bookkeeping runs in one workgroup
constexpr int64_t kBitmapOneLaunch = 16384;     // nodes up to which the bitmap scan is a single launch
constexpr int64_t kNoSyncEvents = 1 << 18;     // below this the target count stays on the device

static ink_status layer_aggregate(ink_ctx *c, int l, const int32_t *F, int64_t nF, int64_t n_chg, const float *f_old,
                                  int ld_old, int64_t n_ins, int64_t n_del) {
  hipStream_t s = c->stream;
  ink_layer_stats &S = c->stats.layer[l - 1];
  Counters *dc = c->d_cnt;
  AggArgs a = agg_args(c, l);
  const int64_t n_seed = n_ins + n_del;
  S.n_sources = nF;
  int64_t nE = n_seed + n_chg;
  S.n_events = nE;
  uint64_t *bm = c->bm_a;
  bool dense = nE > 0 && (double)nE > c->dense_frac * (double)std::max<int64_t>(c->n_edges_now, 1);
  S.dense = dense;
  const bool small = !dense && nE > 0 && nE <= kSmallLayer;
  if (!small) API_TRY(hipMemsetAsync(dc, 0, sizeof(Counters), s));
  if (dense) {
    // so many events that re-aggregating every node costs less than grouping them (Sec. 5.1)
    Prof p(c, INK_T_AGG);
    API_TRY(agg_full_any(c, a, bm));
    return INK_OK;
  }
  if (nE == 0) return INK_OK;
  API_TRY(c->ev_key.reserve((size_t)nE * 4));
  API_TRY(c->ev_val.reserve((size_t)nE * 4));
  API_TRY(c->t_list.reserve((size_t)(nE + 1) * 4));
  API_TRY(c->t_seg.reserve((size_t)(nE + 2) * 4));
  uint32_t *key = c->ev_key.as<uint32_t>(), *val = c->ev_val.as<uint32_t>();
  int64_t nT = std::min<int64_t>(nE, c->n);       // upper bound unless read back below
  if (small) {
    // few events: counters, events, grouping and segment heads in one launch
    Prof p(c, INK_T_GROUP);
    const int passes = (c->id_bits + kRadixBits - 1) / kRadixBits;
#define INK_SMALL_GROUP(T, I)                                                                                      \
  hipLaunchKernelGGL((k_small_group<T, I>), dim3(1), dim3(T), 0, s, (const int32_t *)c->del_src,                    \
                     (const int32_t *)c->del_dst, (const int32_t *)c->ins_src, (const int32_t *)c->ins_dst,        \
                     (int)n_del, (int)n_ins, F, (int)nF, (const int32_t *)c->f_pref.as<int32_t>(), (int)n_chg,     \
                     (const int64_t *)c->gout.off, (const int32_t *)c->gout.ids, c->is_select ? 0 : 1, passes, key, \
                     val, c->t_list.as<int32_t>(), c->t_seg.as<int32_t>(), dc)
    if (nE <= 256) INK_SMALL_GROUP(256, 1);
    else if (nE <= 1024) INK_SMALL_GROUP(256, 4);
    else INK_SMALL_GROUP(1024, 4);
#undef INK_SMALL_GROUP
    API_TRY(hipGetLastError());
  } else {
    {
      Prof p(c, INK_T_EVENTS);
      if (n_seed > 0)
        hipLaunchKernelGGL(k_seed_events, grid1(n_seed), dim3(256), 0, s, (const int32_t *)c->del_src,
                           (const int32_t *)c->del_dst, (const int32_t *)c->ins_src, (const int32_t *)c->ins_dst,
                           (int)n_del, (int)n_ins, (int64_t)n_chg, key, val);
      if (n_chg > 0)
        hipLaunchKernelGGL(k_expand_events, grid1(n_chg, 256 / kWave * kExpandPerWave), dim3(256), 0, s, F, (int)nF,
                           (const int32_t *)c->f_pref.as<int32_t>(), (int)n_chg, (const int64_t *)c->gout.off,
                           (const int32_t *)c->gout.ids, key + n_del, val + n_del, c->is_select ? 0 : 1);
      API_TRY(hipGetLastError());
    }
    Prof p(c, INK_T_GROUP);
    { KernelTimer kt(c, l, INK_K_SORT); API_TRY(radix_sort_pairs(c->ws, key, val, nE, c->id_bits, s)); }
    API_TRY(segment_heads(c->ws, key, nE, c->t_list.as<int32_t>(), c->t_seg.as<int32_t>(), &dc->v[C_NT], s));
    if (nE > kNoSyncEvents) {
      API_TRY(read_counters(c));
      nT = c->h_cnt->v[C_NT];
    }
  }
  if (c->affected_mode) {
    // baseline "Affected" (Sec. 4.1): every node an event reaches is recomputed from its whole
    // neighbourhood, without looking at the events' content, and counts as affected
    Prof p(c, INK_T_AGG);
    if (nE <= kNoSyncEvents) {
      API_TRY(read_counters(c));
      nT = c->h_cnt->v[C_NT];
    }
    API_TRY(agg_full_any(c, a, bm, c->t_list.as<int32_t>(), nT));
    if (nT > 0) hipLaunchKernelGGL(k_mark_nodes, grid1(nT), dim3(256), 0, s, (const int32_t *)c->t_list.as<int32_t>(), (int)nT, bm);
    API_TRY(hipGetLastError());
    return INK_OK;
  }
  {
    Prof p(c, INK_T_AGG);
    if (!c->is_select && nF > 0) {
      API_TRY(c->f_delta.reserve((size_t)nF * ld_old * 4));
      API_TRY(agg_sum_delta_rows(c, a, F, (int)nF, f_old, c->f_delta.as<float>(), ld_old));
    }
    for (int b = 0; b < agg_blocks(a); b++) {
      AggArgs ab = agg_block(a, b);
      int c0 = b * kAggBlock;
      if (b > 0) API_TRY(hipMemsetAsync(&dc->v[C_NBIG], 0, 2 * sizeof(int32_t), s));   // long and exposed row lists
      if (c->is_select)
        API_TRY(agg_select_events(c, ab, c->t_list.as<int32_t>(), c->t_seg.as<int32_t>(), nT, &dc->v[C_NT],
                                  c->ev_val.as<uint32_t>(), bm));
      else
        API_TRY(agg_sum_events(c, ab, c->t_list.as<int32_t>(), c->t_seg.as<int32_t>(), nT, &dc->v[C_NT],
                               c->ev_val.as<uint32_t>(), F, (int)nF, f_old ? f_old + c0 : nullptr,
                               c->f_delta.as<float>() ? c->f_delta.as<float>() + c0 : nullptr, ld_old, bm));
    }
  }
  return INK_OK;
}

// fills the layer's statistics from the counters of the last read-back
static void layer_stats_from_counters(ink_ctx *c, int l) {
  ink_layer_stats &S = c->stats.layer[l - 1];
  if (S.dense) {
    S.n_targets = c->n; S.n_exposed = c->n; S.n_regather_nb = c->n_edges_now;
    S.n_regather_nb_long = (int64_t)c->h_cnt->sum(ST_REGATHER_LONG);
    return;
  }
  c->big_hint[l] = c->h_cnt->v[C_NCHUNK];
  S.n_targets = c->h_cnt->v[C_NT];
  if (c->affected_mode) {
    S.n_exposed = S.n_targets; S.n_regather_nb = (int64_t)c->h_cnt->sum(ST_REGATHER);
    return;
  }
  S.n_exposed = (int64_t)c->h_cnt->sum(ST_EXPOSED);
  S.n_regather_nb = (int64_t)c->h_cnt->sum(ST_REGATHER);
  S.n_regather_nb_long = (int64_t)c->h_cnt->sum(ST_REGATHER_LONG);
  S.n_alpha_changed = (int64_t)c->h_cnt->sum(ST_ACHG);
  S.n_no_deletion = (int64_t)c->h_cnt->sum(ST_NODEL);
  S.n_deletion_no_effect = (int64_t)c->h_cnt->sum(ST_NOEFFECT);
  S.n_covered = (int64_t)c->h_cnt->sum(ST_COVERED);
}

// bitmap (plus extra id lists) -> ascending row list in c->c_list; returns the count, or, with
// bound >= 0, that upper bound without waiting for the device (the count stays in C_NC).
// n_t_bound >= 0 says that only the first *C_NT (at most n_t_bound) entries of c->t_list can have
// their bit set; a short candidate list is then collected in one workgroup, which also clears
// the row flags (*flags_cleared), unless the graph is so small that scanning the whole bitmap is
// one launch as well (then sorting the candidates costs more than the scan).
static ink_status collect_rows(ink_ctx *c, const int32_t *extra0, int64_t n0, const int32_t *extra1, int64_t n1,
                               int64_t *nC, int64_t bound = -1, int64_t n_t_bound = -1, bool *flags_cleared = nullptr) {
  hipStream_t s = c->stream;
  Prof p(c, INK_T_COMPACT);
  API_TRY(c->c_list.reserve((size_t)c->n * 4));
  const int64_t M = n_t_bound + n0 + n1;
  if (n_t_bound >= 0 && M <= kSmallLayer && c->n > kBitmapOneLaunch) {
    const int64_t n_flags = std::min<int64_t>(M, c->n);
    API_TRY(c->c_flag.reserve((size_t)n_flags + 64));
    const int passes = (c->id_bits + kRadixBits - 1) / kRadixBits;
#define INK_SMALL_COLLECT(T, I)                                                                                    \
  hipLaunchKernelGGL((k_small_collect<T, I>), dim3(1), dim3(T), 0, s, (const int32_t *)c->t_list.as<int32_t>(),     \
                     (const int32_t *)&c->d_cnt->v[C_NT], (int)n_t_bound, (unsigned long long *)c->bm_a, extra0,   \
                     (int)n0, extra1, (int)n1, passes, c->c_list.as<int32_t>(), c->c_flag.as<uint8_t>(),           \
                     (int)n_flags, c->d_cnt)
    if (M <= 256) INK_SMALL_COLLECT(256, 1);
    else if (M <= 1024) INK_SMALL_COLLECT(256, 4);
    else INK_SMALL_COLLECT(1024, 4);
#undef INK_SMALL_COLLECT
    API_TRY(hipGetLastError());
    if (flags_cleared) *flags_cleared = true;
  } else {
    if (n0 > 0) hipLaunchKernelGGL(k_mark_nodes, grid1(n0), dim3(256), 0, s, extra0, (int)n0, c->bm_a);
    if (n1 > 0) hipLaunchKernelGGL(k_mark_nodes, grid1(n1), dim3(256), 0, s, extra1, (int)n1, c->bm_a);
    API_TRY(bitmap_to_list(c->ws, c->bm_a, c->n, c->c_list.as<int32_t>(), &c->d_cnt->v[C_NC], 1, s));
  }
  if (bound >= 0) { *nC = bound; return INK_OK; }
  API_TRY(read_counters(c));
  *nC = c->h_cnt->v[C_NC];
  return INK_OK;
}

// rows of c_list whose flag is set -> f_list[nxt] (ids) and, for sum-type, f_old[nxt] (old rows
// taken from c_old with row stride ld).  With want_events the events those rows will propagate in
// the next layer are counted in the same round trip (prefix of kept out-degrees in f_pref).
// With `result` (the last layer's output table) and a modest nC, the new rows of the changed nodes
// are gathered into res_emb and the batch's marks are cleared before that round trip, so nothing
// is left to launch after it; *result_done says whether that happened.
constexpr size_t kEagerResultBytes = (size_t)64 << 20;
static ink_status emit_changed(ink_ctx *c, int64_t nC, int nxt, bool keep_old, int ld, bool want_events,
                               int64_t *nF2, int64_t *n_chg, const Table *result = nullptr,
                               bool *result_done = nullptr) {
  hipStream_t s = c->stream;
  Prof p(c, INK_T_COMPACT);
  Counters *dc = c->d_cnt;
  *nF2 = 0; *n_chg = 0;
  API_TRY(c->f_list[nxt].reserve((size_t)nC * 4));
  const bool small = nC <= kSmallLayer;
  uint32_t published = 0;
  if (small) {
    if (want_events) API_TRY(c->f_pref.reserve((size_t)(nC + 1) * 4));
#define INK_SMALL_EMIT(T, I)                                                                                       \
  hipLaunchKernelGGL((k_small_emit<T, I>), dim3(1), dim3(T), 0, s, (const uint8_t *)c->c_flag.as<uint8_t>(),        \
                     (const int32_t *)c->c_list.as<int32_t>(), (int)nC, c->c_idx.as<int32_t>(),                    \
                     c->f_list[nxt].as<int32_t>(), want_events ? 1 : 0, (const int32_t *)c->gout.deg,              \
                     (const int32_t *)c->new_out, c->f_pref.as<int32_t>(), dc, c->h_cnt, c->h_seq, seq)
    const uint32_t seq = ++c->pub_seq;       // the kernel publishes the counters itself
    published = seq;
    if (nC <= 256) INK_SMALL_EMIT(256, 1);
    else if (nC <= 1024) INK_SMALL_EMIT(256, 4);
    else INK_SMALL_EMIT(1024, 4);
#undef INK_SMALL_EMIT
  } else {
    API_TRY(compact_flags_u8(c->ws, c->c_flag.as<uint8_t>(), nC, c->c_idx.as<int32_t>(), &dc->v[C_NEXT], s));
    hipLaunchKernelGGL(k_gather_i32, grid1(nC), dim3(256), 0, s, (const int32_t *)c->c_list.as<int32_t>(),
                       (const int32_t *)c->c_idx.as<int32_t>(), 0, (const int32_t *)&dc->v[C_NEXT],
                       c->f_list[nxt].as<int32_t>());
  }
  if (keep_old) {
    API_TRY(c->f_old[nxt].reserve((size_t)nC * ld * 4));
    hipLaunchKernelGGL(k_gather_rows_ld, grid1(nC * (ld / 4)), dim3(256), 0, s, (const float *)c->c_old.as<float>(), ld,
                       (const int32_t *)c->c_idx.as<int32_t>(), (int64_t)0, (const int32_t *)&dc->v[C_NEXT],
                       c->f_old[nxt].as<float>());
  }
  if (want_events && !small) {
    API_TRY(c->f_pref.reserve((size_t)(nC + 1) * 4));
    API_TRY(tile_scan(c->ws, KeptOutDeg{c->f_list[nxt].as<int32_t>(), c->gout.deg, c->new_out, &dc->v[C_NEXT]},
                      StorePref{c->f_pref.as<int32_t>()}, nC, &dc->v[C_NEV], s));
  }
  if (result && (size_t)nC * result->d * 4 <= kEagerResultBytes) {
    API_TRY(c->res_emb.reserve((size_t)nC * result->d * 4));
    gather_rows(s, (const float *)result->f(), result->ld, result->d, (const int32_t *)c->f_list[nxt].as<int32_t>(), nC,
                c->res_emb.as<float>(), &dc->v[C_NEXT]);
    API_TRY(graph_end_batch(c));
    *result_done = true;
  }
  API_TRY(hipGetLastError());
  if (small) API_TRY(wait_published(c, published));
  else API_TRY(read_counters(c));
  *nF2 = c->h_cnt->v[C_NEXT];
  if (want_events) *n_chg = (uint32_t)c->h_cnt->v[C_NEV];
  return INK_OK;
}

// Layers 1..k for the sources F_1 = f_list[cur] (nF ids whose layer-1 message changed, n_chg events
// along their kept out-edges) and the applied edge changes; D (nD ids) are nodes whose in-degree
// changed (normalised aggregators).  Fills the result for layer k.
// Rows that have to be re-transformed at a layer for a reason of their own (their user term changed):
// asked for at the start of every layer up to `last_layer`.
struct LayerRows {
  int last_layer;
  ink_status (*rows_of)(ink_ctx *c, int l, void *state, const int32_t **rows, int64_t *n);
  void *state;
};

static ink_status propagate_layers(ink_ctx *c, int64_t nF, int64_t n_chg, int cur, int64_t n_ins, int64_t n_del,
                                   const int32_t *D_all, int64_t nD_all, ink_update_result *out,
                                   const LayerRows *own = nullptr) {
  hipStream_t s = c->stream;
  const int64_t n_seed = n_ins + n_del;
  const bool gcn = c->kind == INK_MODEL_GCN;
  const bool keep_old = !c->is_select && !c->affected_mode;   // delta updates subtract the old message rows
  for (int l = 1; l <= c->n_layers && (n_seed > 0 || nF > 0 || (own && l <= own->last_layer)); l++) {
    ink_layer_stats &S = c->stats.layer[l - 1];
    const int32_t *D = D_all;
    int64_t nD = nD_all;
    if (own) {
      ink_status st_own = own->rows_of(c, l, own->state, &D, &nD);
      if (st_own != INK_OK) return st_own;
    }
    const int32_t *F = c->f_list[cur].as<int32_t>();
    int ld_msg = msg_table(c, l).ld;
    ink_status st = layer_aggregate(c, l, F, nF, n_chg, keep_old ? c->f_old[cur].as<float>() : nullptr, ld_msg,
                                    n_ins, n_del);
    if (st != INK_OK) return st;
    // rows to transform: aggregate changed; own message changed (self term); degree changed.
    // A layer with few events keeps the row count on the device: the transform and the emission
    // are launched for an upper bound and stop at the count, which saves one host round trip.
    int64_t nC = 0;
    const bool lazy = !gcn && !S.dense && !c->affected_mode && S.n_events <= kNoSyncEvents;
    const int64_t bound = lazy ? std::min<int64_t>(std::min<int64_t>(S.n_events, c->n) + nF + nD, c->n) : -1;
    // without the dense fallback and the baseline only grouped targets can have changed aggregates
    const int64_t n_t_bound = (S.dense || c->affected_mode) ? -1 : (S.n_events > 0 ? std::min<int64_t>(S.n_events, c->n) : 0);
    bool flags_cleared = false;
    st = collect_rows(c, F, nF, D, nD, &nC, bound, n_t_bound, &flags_cleared);
    if (st != INK_OK) return st;
    const int32_t *nC_dev = lazy ? &c->d_cnt->v[C_NC] : nullptr;
    if (!lazy) { S.n_transformed = nC; layer_stats_from_counters(c, l); }
    int nxt = cur ^ 1;
    int64_t nF2 = 0, n_chg2 = 0;
    bool result_done = false;
    if (nC > 0) {
      const bool last = l == c->n_layers;
      int ld_next = gcn ? (last ? c->H[l].ld : c->Msc[l + 1].ld) : c->H[l].ld;
      API_TRY(c->c_flag.reserve((size_t)nC + 64));
      API_TRY(c->c_idx.reserve((size_t)nC * 4));
      bool want_old = keep_old && !last;
      if (want_old) API_TRY(c->c_old.reserve((size_t)nC * ld_next * 4));
      {
        Prof p(c, INK_T_TRANSFORM, l, INK_K_XFORM);
        const int32_t *rows = c->c_list.as<int32_t>();
        float *old_rows = want_old ? c->c_old.as<float>() : nullptr;
        if (!gcn) {
          if (lazy && !flags_cleared) API_TRY(hipMemsetAsync(c->c_flag.p, 0, (size_t)nC, s));   // flags past the count stay 0
          API_TRY(run_transform(c, l, rows, nC, c->c_flag.as<uint8_t>(), old_rows, nC_dev));
        } else {
          if (!flags_cleared) API_TRY(hipMemsetAsync(c->c_flag.p, 0, (size_t)nC, s));
          if (!last) API_TRY(gcn_next_messages(c, l, rows, nC, c->c_flag.as<uint8_t>(), old_rows));
          else API_TRY(gcn_final(c, rows, nC, c->c_flag.as<uint8_t>()));
        }
        // the baseline propagates from every node of the affected area, changed or not
        if (c->affected_mode && !last) API_TRY(hipMemsetAsync(c->c_flag.p, 1, (size_t)nC, s));
      }
      st = emit_changed(c, nC, nxt, want_old, ld_next, !last, &nF2, &n_chg2, last ? &c->H[l] : nullptr, &result_done);
      if (st != INK_OK) return st;
    } else if (lazy) {
      API_TRY(read_counters(c));
    }
    if (lazy) { S.n_transformed = c->h_cnt->v[C_NC]; layer_stats_from_counters(c, l); }
    S.n_changed = nF2;
    nF = nF2;
    n_chg = n_chg2;
    cur = nxt;
    if (l == c->n_layers) {
      out->n_changed = nF;
      if (nF > 0) {
        int d = c->H[l].d;
        out->changed_ids = c->f_list[cur].as<int32_t>();    // stays untouched until the next call
        if (!result_done) {
          API_TRY(c->res_emb.reserve((size_t)nF * d * 4));
          gather_rows(s, (const float *)c->H[l].f(), c->H[l].ld, d, out->changed_ids, nF, c->res_emb.as<float>());
        }
        out->embeddings = c->res_emb.as<float>();
      }
    }
  }
  return INK_OK;
}

static ink_status apply_updates_impl(ink_ctx *c, const ink_edge_update *upd, int64_t n, ink_update_result *out);

extern "C" ink_status ink_apply_updates(ink_ctx *c, const ink_edge_update *upd, int64_t n, ink_update_result *out) {
  if (!c) return INK_E_ARG;
  if (c->broken) return fail(c, INK_E_STATE, kBrokenMsg);
  c->affected_mode = false;
  return seal(c, apply_updates_impl(c, upd, n, out));
}

extern "C" ink_status ink_apply_updates_affected(ink_ctx *c, const ink_edge_update *upd, int64_t n,
                                                 ink_update_result *out) {
  if (!c) return INK_E_ARG;
  if (c->broken) return fail(c, INK_E_STATE, kBrokenMsg);
  c->affected_mode = true;
  ink_status st = apply_updates_impl(c, upd, n, out);
  c->affected_mode = false;
  return seal(c, st);
}

static ink_status apply_updates_impl(ink_ctx *c, const ink_edge_update *upd, int64_t n, ink_update_result *out) {
  if (!out || n < 0 || (n > 0 && !upd)) return fail(c, INK_E_ARG, "ink_apply_updates: NULL argument or negative n");
  if (!c->inferred) return fail(c, INK_E_STATE, "ink_apply_updates: call ink_full_infer first");
  if (n >= (1ll << 30)) return fail(c, INK_E_ARG, "ink_apply_updates: batch too large");
  if (c->n_edges_now + n > kMaxEdges) return fail(c, INK_E_ARG, "ink_apply_updates: the graph would exceed the edge limit");
  auto t0 = std::chrono::steady_clock::now();
  memset(out, 0, sizeof(*out));
  hipStream_t s = c->stream;
  // Validation before anything is touched: a host-resident batch is checked here; a device-resident
  // one by the first kernel of the graph stage, which drops the whole batch on a bad entry (the
  // graph stage reports it after its first read-back, before any block is modified).
  if (!c->batch_dev) {
    for (int64_t i = 0; i < n; i++) {
      if (upd[i].op > 1) return fail(c, INK_E_ARG, "ink_apply_updates: op must be 0 (insert) or 1 (delete)");
      if (upd[i].src < 0 || upd[i].src >= c->n || upd[i].dst < 0 || upd[i].dst >= c->n)
        return fail(c, INK_E_RANGE, "ink_apply_updates: node id out of range");
    }
  }
  memset(&c->stats, 0, sizeof(c->stats));
  c->stats.n_layers = c->n_layers;
  int64_t n_ins = 0, n_del = 0;
  if (n > 0) {
    Prof p(c, INK_T_GRAPH);
    API_TRY(c->b_raw.reserve((size_t)n * sizeof(ink_edge_update)));
    API_TRY(hipMemcpyAsync(c->b_raw.p, upd, (size_t)n * sizeof(ink_edge_update),
                           c->batch_dev ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice, s));
    ink_status st = graph_apply_batch(c, n, &n_ins, &n_del);
    if (st != INK_OK) return st;
  }
  out->n_applied_ins = n_ins; out->n_applied_del = n_del; out->n_noop = n - n_ins - n_del;
  c->n_edges_now += n_ins - n_del;
  const int64_t n_seed = n_ins + n_del;
  const bool gcn = c->kind == INK_MODEL_GCN;
  // nodes whose in-degree may have changed: their normalisation (GCN, mean) changes row-locally
  const int32_t *D = (const int32_t *)c->b_touch_in.p;
  const int64_t nD = (n_seed > 0 && (gcn || c->agg == INK_AGG_MEAN)) ? c->n_touched_in : 0;

  int64_t nF = 0;            // |F_l|: sources whose message m_l changed
  int64_t n_chg = 0;         // events F_l propagates along its kept out-edges
  int cur = 0;               // f_list[cur] / f_old[cur] describe F_l
  if (gcn && nD > 0) {
    // layer-1 messages are c_u * (x_u W_1): a degree change rescales the row
    Prof p(c, INK_T_TRANSFORM);
    int ld = c->Msc[1].ld;
    API_TRY(c->c_flag.reserve((size_t)nD + 64));
    API_TRY(c->c_idx.reserve((size_t)nD * 4));
    API_TRY(c->c_old.reserve((size_t)nD * ld * 4));
    API_TRY(c->c_list.reserve((size_t)c->n * 4));
    API_TRY(hipMemsetAsync(c->c_flag.p, 0, (size_t)nD, s));
    API_TRY(hipMemcpyAsync(c->c_list.p, D, (size_t)nD * 4, hipMemcpyDeviceToDevice, s));
    hipLaunchKernelGGL(k_gcn_rescale, grid1(nD * ld), dim3(256), 0, s, D, nD, (const int32_t *)c->gin.deg, c->cnorm,
                       (const float *)c->XW[1].f(), c->Msc[1].f(), ld, c->Msc[1].d, c->c_old.as<float>(),
                       c->c_flag.as<uint8_t>());
    API_TRY(hipGetLastError());
    ink_status st = emit_changed(c, nD, cur, true, ld, true, &nF, &n_chg);
    if (st != INK_OK) return st;
  }
  {
    ink_status st = propagate_layers(c, nF, n_chg, cur, n_ins, n_del, D, nD, out);
    if (st != INK_OK) return st;
  }
  API_TRY(graph_end_batch(c));
  API_TRY(hipStreamSynchronize(s));
  prof_collect(c);
  c->stats.ms_total = std::chrono::duration<float, std::milli>(std::chrono::steady_clock::now() - t0).count();
  return INK_OK;
}

// ------------------------------------------------------------------------------------ feature updates
static ink_status update_features_impl(ink_ctx *c, const int32_t *node_ids, const float *rows, int64_t n,
                                       ink_update_result *out);
extern "C" ink_status ink_update_features(ink_ctx *c, const int32_t *node_ids, const float *rows, int64_t n,
                                          ink_update_result *out) {
  if (!c) return INK_E_ARG;
  if (c->broken) return fail(c, INK_E_STATE, kBrokenMsg);
  return seal(c, update_features_impl(c, node_ids, rows, n, out));
}

static ink_status update_features_impl(ink_ctx *c, const int32_t *node_ids, const float *rows, int64_t n,
                                       ink_update_result *out) {
  if (!out || n < 0 || (n > 0 && (!node_ids || !rows))) return fail(c, INK_E_ARG, "ink_update_features: NULL argument or negative n");
  if (!c->inferred) return fail(c, INK_E_STATE, "ink_update_features: call ink_full_infer first");
  if (n > c->n) return fail(c, INK_E_ARG, "ink_update_features: more rows than nodes (ids must be distinct)");
  auto t0 = std::chrono::steady_clock::now();
  memset(out, 0, sizeof(*out));
  hipStream_t s = c->stream;
  c->affected_mode = false;
  const int d0 = c->H[0].d, ld0 = c->H[0].ld;
  // validation before anything is touched: host-resident ids are range-checked here, device-resident
  // ones by a kernel; distinctness is checked on the sorted device copy (one read-back for both)
  if (!c->batch_dev)
    for (int64_t i = 0; i < n; i++)
      if (node_ids[i] < 0 || node_ids[i] >= c->n) return fail(c, INK_E_RANGE, "ink_update_features: node id out of range");
  memset(&c->stats, 0, sizeof(c->stats));
  c->stats.n_layers = c->n_layers;
  if (n == 0) return INK_OK;
  const bool gcn = c->kind == INK_MODEL_GCN;
  const bool keep_old = !c->is_select;
  Counters *dc = c->d_cnt;
  int64_t nF = 0, n_chg = 0;
  int cur = 0;
  {
    Prof p(c, INK_T_GRAPH);
    const hipMemcpyKind kind = c->batch_dev ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice;
    size_t per = ((size_t)n * 4 + 255) & ~(size_t)255;
    API_TRY(c->b_misc.reserve(per * 2));
    uint32_t *ids = c->b_misc.as<uint32_t>(), *perm = (uint32_t *)((char *)c->b_misc.p + per);
    API_TRY(hipMemcpyAsync(ids, node_ids, (size_t)n * 4, kind, s));
    const float *drows = rows;
    if (!c->batch_dev) {
      API_TRY(c->stage1.reserve((size_t)n * d0 * 4));
      API_TRY(hipMemcpyAsync(c->stage1.p, rows, (size_t)n * d0 * 4, hipMemcpyHostToDevice, s));
      drows = c->stage1.as<float>();
    }
    hipLaunchKernelGGL(k_iota_u32, grid1(n), dim3(256), 0, s, perm, n);
    API_TRY(radix_sort_pairs(c->ws, ids, perm, n, c->id_bits, s));
    API_TRY(hipMemsetAsync(dc, 0, sizeof(Counters), s));
    hipLaunchKernelGGL(k_any_adjacent_equal, grid1(n), dim3(256), 0, s, (const uint32_t *)ids, n, &dc->v[C_TMP0]);
    if (c->batch_dev)
      hipLaunchKernelGGL(k_any_out_of_range, grid1(n), dim3(256), 0, s, (const uint32_t *)ids, n, (uint32_t)c->n, &dc->v[C_TMP1]);
    API_TRY(hipGetLastError());
    API_TRY(read_counters(c));
    if (c->h_cnt->v[C_TMP1]) return fail(c, INK_E_RANGE, "ink_update_features: node id out of range");
    if (c->h_cnt->v[C_TMP0]) return fail(c, INK_E_ARG, "ink_update_features: a node id appears more than once");
    API_TRY(c->c_flag.reserve((size_t)n + 64));
    API_TRY(c->c_idx.reserve((size_t)n * 4));
    API_TRY(c->c_list.reserve((size_t)c->n * 4));
    API_TRY(hipMemsetAsync(c->c_flag.p, 0, (size_t)n, s));
    float *old0 = nullptr, *dense = nullptr;
    if (keep_old && !gcn) { API_TRY(c->c_old.reserve((size_t)n * ld0 * 4)); old0 = c->c_old.as<float>(); }
    if (gcn) { API_TRY(c->stage0.reserve((size_t)n * ld0 * 4)); dense = c->stage0.as<float>(); }
    hipLaunchKernelGGL(k_set_features, grid1(n * ld0), dim3(256), 0, s, (const uint32_t *)ids, (const uint32_t *)perm, n,
                       drows, d0, c->H[0].f(), ld0, old0, dense, c->c_flag.as<uint8_t>(), c->c_list.as<int32_t>());
    API_TRY(hipGetLastError());
  }
  int ld_msg = ld0;
  if (gcn) {
    // layer-1 messages are c_u (x_u W_1): redo the product for the listed rows, then rescale
    Prof p(c, INK_T_TRANSFORM);
    const DevLayer &L = c->layers[0];
    ld_msg = c->Msc[1].ld;
    XformArgs x;
    memset(&x, 0, sizeof(x));
    x.mode = 2; x.n_rows = n; x.Hp = c->stage0.as<float>(); x.ldh = ld0; x.d_in = L.in_dim;
    x.W = L.W1; x.Kp = L.K1p; x.Np = L.N1p; x.n_out = L.out_dim;
    x.out = c->XW[1].f(); x.ld_out = c->XW[1].ld; x.to_table = 1; x.out_rows = c->c_list.as<int32_t>();
    API_TRY(xform_run(c, x));
    API_TRY(c->c_old.reserve((size_t)n * ld_msg * 4));
    API_TRY(hipMemsetAsync(c->c_flag.p, 0, (size_t)n, s));
    hipLaunchKernelGGL(k_gcn_rescale, grid1(n * ld_msg), dim3(256), 0, s, (const int32_t *)c->c_list.as<int32_t>(), n,
                       (const int32_t *)c->gin.deg, c->cnorm, (const float *)c->XW[1].f(), c->Msc[1].f(), ld_msg,
                       c->Msc[1].d, c->c_old.as<float>(), c->c_flag.as<uint8_t>());
    API_TRY(hipGetLastError());
  }
  ink_status st = emit_changed(c, n, cur, keep_old, ld_msg, true, &nF, &n_chg);
  if (st != INK_OK) return st;
  st = propagate_layers(c, nF, n_chg, cur, 0, 0, nullptr, 0, out);
  if (st != INK_OK) return st;
  API_TRY(hipStreamSynchronize(s));
  prof_collect(c);
  c->stats.ms_total = std::chrono::duration<float, std::milli>(std::chrono::steady_clock::now() - t0).count();
  return INK_OK;
}

// ------------------------------------------------------------------------------------ user-defined events
// key of event i for the pass over layer l: its target, or n_nodes (sorts behind every node) if it
// belongs to another layer; value = its position in the list
__global__ void k_user_keys(const ink_user_event *ev, int64_t n, int layer, uint32_t n_nodes, uint32_t *key, uint32_t *val) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  key[i] = ev[i].layer == layer ? (uint32_t)ev[i].target : n_nodes;
  val[i] = (uint32_t)i;
}

// One wave per target: its events (positions pos[seg[j] .. seg[j + 1]) of the list, in list order)
// are applied to the node's term; flag[j] = 1 if the term changed bitwise.
__global__ __launch_bounds__(256) void k_user_apply(const int32_t *uniq, const int32_t *seg, const int32_t *n_uniq,
                                                    const uint32_t *pos, const ink_user_event *ev, const float *rows,
                                                    int stride, float *U, int ld, int d, uint8_t *flag) {
  const int l = lane_id();
  int64_t j = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / kWave;
  if (j >= *n_uniq) return;
  const int64_t v = uniq[j];
  const int e0 = seg[j], e1 = seg[j + 1];
  bool chg = false;
  for (int k = l; k < d; k += kWave) {
    const float old = U[v * ld + k];
    float u = old;
    for (int e = e0; e < e1; e++) {
      const uint32_t i = pos[e];
      const int op = ev[i].op;
      const float r = rows[(int64_t)i * stride + k];
      u = op == INK_USER_SET ? r : (op == INK_USER_ADD ? __fadd_rn(u, r) : 0.f);
    }
    if (__float_as_uint(u) != __float_as_uint(old)) { U[v * ld + k] = u; chg = true; }
  }
  const bool any = __ballot(chg) != 0ull;
  if (l == 0) flag[j] = any ? 1 : 0;
}

struct UserState {
  int64_t n;                       // events in the list
  int row_stride;                  // floats between the rows of two events
  int64_t per_layer[INK_MAX_LAYERS + 1];   // events that name each layer
};

// the nodes whose term of layer l changed -> ascending list (the rows this layer re-transforms for its own reasons)
static ink_status user_rows_of(ink_ctx *c, int l, void *state, const int32_t **rows, int64_t *n_rows) {
  const UserState *u = (const UserState *)state;
  *rows = nullptr; *n_rows = 0;
  const int64_t m = u->per_layer[l];
  if (m == 0) return INK_OK;
  hipStream_t s = c->stream;
  Prof p(c, INK_T_EVENTS);
  uint32_t *key = c->u_key.as<uint32_t>(), *val = c->u_val.as<uint32_t>();
  hipLaunchKernelGGL(k_user_keys, grid1(u->n), dim3(256), 0, s, (const ink_user_event *)c->u_ev.p, u->n, l, (uint32_t)c->n, key, val);
  API_TRY(hipGetLastError());
  // stable: the layer's events come first, grouped by target, each group in list order
  API_TRY(radix_sort_pairs(c->ws, key, val, u->n, c->id_bits + 1, s));
  int32_t *n_uniq = &c->d_cnt->v[C_TMP0], *n_chg = &c->d_cnt->v[C_TMP1];
  API_TRY(segment_heads(c->ws, key, m, c->u_uniq.as<int32_t>(), c->u_seg.as<int32_t>(), n_uniq, s));
  hipLaunchKernelGGL(k_user_apply, grid1(m * kWave), dim3(256), 0, s, (const int32_t *)c->u_uniq.as<int32_t>(),
                     (const int32_t *)c->u_seg.as<int32_t>(), (const int32_t *)n_uniq, (const uint32_t *)val,
                     (const ink_user_event *)c->u_ev.p, (const float *)c->u_rows.p, u->row_stride,
                     c->USER[l].f(), c->USER[l].ld, c->USER[l].d, c->u_flag.as<uint8_t>());
  API_TRY(hipGetLastError());
  API_TRY(read_counters(c));
  const int64_t nu = c->h_cnt->v[C_TMP0];
  API_TRY(compact_flags_u8(c->ws, c->u_flag.as<uint8_t>(), nu, c->u_idx.as<int32_t>(), n_chg, s));
  hipLaunchKernelGGL(k_gather_i32, grid1(nu), dim3(256), 0, s, (const int32_t *)c->u_uniq.as<int32_t>(),
                     (const int32_t *)c->u_idx.as<int32_t>(), 0, (const int32_t *)n_chg, c->u_list.as<int32_t>());
  API_TRY(hipGetLastError());
  API_TRY(read_counters(c));
  *rows = c->u_list.as<int32_t>();
  *n_rows = c->h_cnt->v[C_TMP1];
  return INK_OK;
}

static ink_status apply_user_events_impl(ink_ctx *c, const ink_user_event *events, const float *rows, int32_t row_stride,
                                         int64_t n, ink_update_result *out) {
  if (!out || n < 0 || (n > 0 && (!events || !rows))) return fail(c, INK_E_ARG, "ink_apply_user_events: NULL argument or negative n");
  if (!c->inferred) return fail(c, INK_E_STATE, "ink_apply_user_events: call ink_full_infer first");
  if (n >= (1ll << 30)) return fail(c, INK_E_ARG, "ink_apply_user_events: too many events");
  UserState u;
  memset(&u, 0, sizeof(u));
  u.n = n;
  u.row_stride = row_stride;
  int last = 0;
  for (int64_t i = 0; i < n; i++) {
    const ink_user_event &e = events[i];
    if (e.layer < 1 || e.layer > c->n_layers) return fail(c, INK_E_RANGE, "ink_apply_user_events: layer out of range");
    if (e.target < 0 || e.target >= c->n) return fail(c, INK_E_RANGE, "ink_apply_user_events: node id out of range");
    if (e.op < INK_USER_SET || e.op > INK_USER_CLEAR) return fail(c, INK_E_ARG, "ink_apply_user_events: unknown op");
    if (row_stride < c->H[e.layer].d) return fail(c, INK_E_ARG, "ink_apply_user_events: row_stride below the layer's width");
    u.per_layer[e.layer]++;
    last = std::max(last, (int)e.layer);
  }
  auto t0 = std::chrono::steady_clock::now();
  memset(out, 0, sizeof(*out));
  memset(&c->stats, 0, sizeof(c->stats));
  c->stats.n_layers = c->n_layers;
  if (n == 0) return INK_OK;
  c->affected_mode = false;
  hipStream_t s = c->stream;
  // everything that can fail for lack of memory comes before the first term is touched
  for (int l = 1; l <= last; l++)
    if (u.per_layer[l] > 0 && !c->USER[l].p) API_TRY(alloc_table(c->USER[l], c->n_cap, c->H[l].d));
  API_TRY(c->u_ev.reserve((size_t)n * sizeof(ink_user_event)));
  API_TRY(c->u_rows.reserve((size_t)n * row_stride * 4));
  for (DevBuf *b : {&c->u_key, &c->u_val, &c->u_uniq, &c->u_seg, &c->u_idx, &c->u_list}) API_TRY(b->reserve((size_t)(n + 2) * 4));
  API_TRY(c->u_flag.reserve((size_t)n + 64));
  API_TRY(c->c_list.reserve((size_t)c->n * 4));
  API_TRY(hipMemcpyAsync(c->u_ev.p, events, (size_t)n * sizeof(ink_user_event), hipMemcpyHostToDevice, s));
  API_TRY(hipMemcpyAsync(c->u_rows.p, rows, (size_t)n * row_stride * 4, hipMemcpyHostToDevice, s));
  LayerRows own{last, user_rows_of, &u};
  ink_status st = propagate_layers(c, 0, 0, 0, 0, 0, nullptr, 0, out, &own);
  if (st != INK_OK) return st;
  API_TRY(hipStreamSynchronize(s));
  prof_collect(c);
  c->stats.ms_total = std::chrono::duration<float, std::milli>(std::chrono::steady_clock::now() - t0).count();
  return INK_OK;
}

extern "C" ink_status ink_apply_user_events(ink_ctx *c, const ink_user_event *events, const float *rows,
                                            int32_t row_stride, int64_t n, ink_update_result *out) {
  if (!c) return INK_E_ARG;
  if (c->broken) return fail(c, INK_E_STATE, kBrokenMsg);
  return seal(c, apply_user_events_impl(c, events, rows, row_stride, n, out));
}

// ------------------------------------------------------------------------------------ node arrival
__global__ void k_iota_i32(int32_t *out, int64_t n, int32_t first) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) out[i] = first + (int32_t)i;
}

__global__ void k_unpack_rows_at(const float *in, int d, int ld, int64_t row0, int64_t n, float *table) {
  int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  int64_t i = t / ld;
  int k = (int)(t % ld);
  if (i >= n) return;
  table[(row0 + i) * ld + k] = k < d ? in[i * d + k] : 0.f;
}

static ink_status add_nodes_impl(ink_ctx *c, const float *features, int64_t n_new, ink_update_result *out);
extern "C" ink_status ink_add_nodes(ink_ctx *c, const float *features, int64_t n_new, ink_update_result *out) {
  if (!c) return INK_E_ARG;
  if (c->broken) return fail(c, INK_E_STATE, kBrokenMsg);
  return seal(c, add_nodes_impl(c, features, n_new, out));
}

static ink_status add_nodes_impl(ink_ctx *c, const float *features, int64_t n_new, ink_update_result *out) {
  if (!out || n_new < 0 || (n_new > 0 && !features)) return fail(c, INK_E_ARG, "ink_add_nodes: NULL argument or negative n_new");
  if (!c->inferred) return fail(c, INK_E_STATE, "ink_add_nodes: call ink_full_infer first");
  if ((int64_t)c->n + n_new > c->n_cap) return fail(c, INK_E_RANGE, "ink_add_nodes: beyond ink_options.node_capacity");
  auto t0 = std::chrono::steady_clock::now();
  memset(out, 0, sizeof(*out));
  memset(&c->stats, 0, sizeof(c->stats));
  c->stats.n_layers = c->n_layers;
  if (n_new == 0) return INK_OK;
  hipStream_t s = c->stream;
  c->affected_mode = false;
  const int n0 = c->n;
  const int d0 = c->H[0].d, ld0 = c->H[0].ld;
  const bool gcn = c->kind == INK_MODEL_GCN;
  {
    Prof p(c, INK_T_GRAPH);
    ink_status st = graph_add_nodes(c, n_new);
    if (st != INK_OK) return st;
    const float *drows = features;
    if (!c->batch_dev) {
      API_TRY(c->stage1.reserve((size_t)n_new * d0 * 4));
      API_TRY(hipMemcpyAsync(c->stage1.p, features, (size_t)n_new * d0 * 4, hipMemcpyHostToDevice, s));
      drows = c->stage1.as<float>();
    }
    hipLaunchKernelGGL(k_unpack_rows_at, grid1(n_new * ld0), dim3(256), 0, s, drows, d0, ld0, (int64_t)n0, n_new, c->H[0].f());
    API_TRY(c->res_ids.reserve((size_t)n_new * 4));
    hipLaunchKernelGGL(k_iota_i32, grid1(n_new), dim3(256), 0, s, c->res_ids.as<int32_t>(), n_new, (int32_t)n0);
    API_TRY(hipGetLastError());
  }
  c->n = n0 + (int)n_new;          // from here on the new ids are valid rows
  const int32_t *rows = c->res_ids.as<int32_t>();
  if (gcn) {
    // layer-1 message of a node without in-edges: d-hat = 1, so c_v = 1 and m_1 = x W_1
    Prof p(c, INK_T_TRANSFORM);
    const DevLayer &L = c->layers[0];
    XformArgs x;
    memset(&x, 0, sizeof(x));
    x.mode = 2; x.n_rows = n_new; x.Hp = c->H[0].f() + (int64_t)n0 * ld0; x.ldh = ld0; x.d_in = L.in_dim;
    x.W = L.W1; x.Kp = L.K1p; x.Np = L.N1p; x.n_out = L.out_dim;
    x.out = c->XW[1].f(); x.ld_out = c->XW[1].ld; x.to_table = 1; x.out_rows = rows;
    API_TRY(xform_run(c, x));
    hipLaunchKernelGGL(k_gcn_rescale, grid1(n_new * c->Msc[1].ld), dim3(256), 0, s, rows, n_new, (const int32_t *)c->gin.deg,
                       c->cnorm, (const float *)c->XW[1].f(), c->Msc[1].f(), c->Msc[1].ld, c->Msc[1].d, (float *)nullptr,
                       (uint8_t *)nullptr);
    API_TRY(hipGetLastError());
  }
  for (int l = 1; l <= c->n_layers; l++) {
    API_TRY(hipMemsetAsync(c->d_cnt, 0, sizeof(Counters), s));
    AggArgs a = agg_args(c, l);
    { Prof p(c, INK_T_AGG); API_TRY(agg_full_any(c, a, nullptr, rows, n_new)); }
    {
      Prof p(c, INK_T_TRANSFORM);
      if (!gcn) API_TRY(run_transform(c, l, rows, n_new, nullptr));
      else if (l < c->n_layers) API_TRY(gcn_next_messages(c, l, rows, n_new, nullptr, nullptr));
      else API_TRY(gcn_final(c, rows, n_new, nullptr));
    }
    ink_layer_stats &S = c->stats.layer[l - 1];
    S.n_targets = n_new; S.n_exposed = n_new; S.n_transformed = n_new; S.n_changed = n_new;
  }
  {
    int k = c->n_layers, d = c->H[k].d;
    API_TRY(c->res_emb.reserve((size_t)n_new * d * 4));
    gather_rows(s, (const float *)c->H[k].f(), c->H[k].ld, d, rows, n_new, c->res_emb.as<float>());
    API_TRY(hipGetLastError());
    out->n_changed = n_new;
    out->changed_ids = c->res_ids.as<int32_t>();
    out->embeddings = c->res_emb.as<float>();
  }
  API_TRY(hipStreamSynchronize(s));
  prof_collect(c);
  c->stats.ms_total = std::chrono::duration<float, std::milli>(std::chrono::steady_clock::now() - t0).count();
  return INK_OK;
}

// ------------------------------------------------------------------------------------ inspection
extern "C" ink_status ink_get_layer(ink_ctx *c, int32_t layer, int32_t which, int64_t row0, int64_t nrows, void *dst,
                                    int32_t dst_mem, int32_t *width_out) {
  if (!c) return INK_E_ARG;
  if (c->broken) return fail(c, INK_E_STATE, kBrokenMsg);
  if (!c->inferred) return fail(c, INK_E_STATE, "ink_get_layer: call ink_full_infer first");
  if (layer < 0 || layer > c->n_layers || which < 0 || which > 5 || (which > 0 && layer == 0))
    return fail(c, INK_E_RANGE, "ink_get_layer: layer / which out of range");
  if (row0 < 0 || nrows < 0 || row0 + nrows > c->n) return fail(c, INK_E_RANGE, "ink_get_layer: rows out of range");
  if (which >= 2 && which <= 4 && !c->is_select) return fail(c, INK_E_ARG, "ink_get_layer: no argument table for sum-type aggregators");
  const Table &t = which == 0 ? c->H[layer] : (which == 1 ? c->A[layer] : (which == 2 ? c->ARG[layer] : (which == 3 ? c->UB[layer] : (which == 4 ? c->ARG2[layer] : c->USER[layer]))));
  if (!t.p) return fail(c, INK_E_ARG, "ink_get_layer: table not kept for this model");
  if (width_out) *width_out = t.d;
  if (nrows == 0) return INK_OK;
  if (!dst) return fail(c, INK_E_ARG, "ink_get_layer: dst is NULL");
  size_t bytes = (size_t)nrows * t.d * 4;
  void *dev_dst = dst;
  if (dst_mem != INK_MEM_DEVICE) { API_TRY(c->stage1.reserve(bytes)); dev_dst = c->stage1.p; }
  hipLaunchKernelGGL(k_pack_rows, grid1(nrows * t.d), dim3(256), 0, c->stream, (const void *)t.p, t.ld, t.d, row0, nrows,
                     dev_dst);
  API_TRY(hipGetLastError());
  if (dst_mem != INK_MEM_DEVICE) API_TRY(hipMemcpyAsync(dst, dev_dst, bytes, hipMemcpyDeviceToHost, c->stream));
  API_TRY(hipStreamSynchronize(c->stream));
  return INK_OK;
}

extern "C" ink_status ink_get_graph(ink_ctx *c, int64_t *rowptr, int32_t *col) {
  if (!c || !rowptr) return INK_E_ARG;
  if (c->broken) return fail(c, INK_E_STATE, kBrokenMsg);
  API_TRY(hipStreamSynchronize(c->stream));
  API_TRY(graph_export(c, rowptr, col));
  return INK_OK;
}

extern "C" ink_status ink_set_profiling(ink_ctx *c, int32_t on) {
  if (!c) return INK_E_ARG;
  c->profile = on != 0;
  return INK_OK;
}

extern "C" ink_status ink_get_stats(ink_ctx *c, void *dst, size_t bytes) {
  if (!c || !dst) return INK_E_ARG;
  memcpy(dst, &c->stats, std::min(bytes, sizeof(ink_stats)));
  return INK_OK;
}
