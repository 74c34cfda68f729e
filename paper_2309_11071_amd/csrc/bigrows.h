// Work list for rows with more than kBigDeg in-neighbours: each such row is cut into chunks of
// kBigChunk neighbours, one workgroup per chunk, then one wave per row combines its chunks in
// order.  The plan (chunk prefix over the listed rows) is built on the device from the device-side
// row count, and the chunk / row kernels run a fixed grid that strides over it, so no host
// round trip is needed; with no long rows they return at once.
#pragma once
#include "ctx.h"

namespace ink {

#ifndef INK_BIG_LB
#define INK_BIG_LB 1024
#endif

constexpr int kBigGrid = 4096;             // workgroups of the per-row combine kernel

// Few targets (small batches): latency matters more than throughput, so rows are handed to the
// cooperative path much earlier and each chunk is shared by 16 waves instead of 4.
constexpr int kLatencyTargets = 8192;

// upper bound of the long rows one launch can list: with at most kLatencyTargets targets every
// target may be one, otherwise a long row has more than kBigDeg in-neighbours; never more than nodes
inline int64_t big_rows_capacity(const ink_ctx *c) {
  int64_t e = c->n_edges_now > c->n_edges ? c->n_edges_now : c->n_edges;
  int64_t r = e / kBigDeg > kLatencyTargets ? e / kBigDeg : kLatencyTargets;
  return (r < c->n_cap ? r : c->n_cap) + 1;
}
// ... and of their chunks: a row of deg neighbours has at most deg / chunk + 1
inline int64_t big_chunk_capacity(const ink_ctx *c) {
  int64_t e = c->n_edges_now > c->n_edges ? c->n_edges_now : c->n_edges;
  return e / kBigChunk + big_rows_capacity(c);
}

// one workgroup per expected chunk (the hardware balances them); never fewer than fill the chip
inline unsigned big_partial_grid(const ink_ctx *c, int64_t want, int block_threads) {
  int64_t lo = block_threads >= 1024 ? 512 : 2048, hi = big_chunk_capacity(c);
  if (want < lo) want = lo;
  if (want > hi) want = hi;
  return (unsigned)want;
}

// buffers of the long-row path; call before the kernel that fills the list (growing drops contents)
inline hipError_t ensure_big_buffers(ink_ctx *c, int ld, bool with_ids) {
  INK_TRY(c->big_list.reserve((size_t)big_rows_capacity(c) * 4));
  INK_TRY(c->big_pref.reserve((size_t)(c->big_list.cap / 4 + 1) * 4));
  int64_t cap = big_chunk_capacity(c);
  INK_TRY(c->big_part_v.reserve((size_t)cap * ld * sizeof(float)));
  if (with_ids) {
    INK_TRY(c->big_part_i.reserve((size_t)cap * ld * sizeof(int32_t)));
    INK_TRY(c->big_part_s.reserve((size_t)cap * ld * sizeof(float)));
    INK_TRY(c->big_part_j.reserve((size_t)cap * ld * sizeof(int32_t)));
  }
  return hipSuccess;
}

inline bool latency_mode(int64_t n_targets) { return n_targets <= kLatencyTargets; }
inline int big_threshold(int64_t n_targets, int lanes_per_row, int throughput_deg) {
  return latency_mode(n_targets) ? 32 * (kWave / lanes_per_row) : throughput_deg;
}
inline int big_block_threads(int64_t n_targets) { return latency_mode(n_targets) ? (INK_BIG_LB >= 1024 ? 1024 : 256) : 256; }
constexpr int kBigMaxWaves = INK_BIG_LB / 64;

// plan: pref[i] = chunks of the listed rows before i (i <= n_big), *total = all chunks
struct BigChunkCount {
  const int32_t *list; const int32_t *n_big; const int32_t *deg;
  __device__ int operator()(int64_t i) const { return i < *n_big ? (deg[list[i]] + kBigChunk - 1) / kBigChunk : 0; }
};
struct BigPrefStore {
  int32_t *pref; const int32_t *n_big;
  __device__ void operator()(int64_t i, int v, int ex) const {
    int n = *n_big;
    if (i < n) pref[i] = ex;
    if (i == n - 1) pref[n] = ex + v;
  }
};
// n_rows_max bounds the device-side row count
inline hipError_t plan_big_rows(ink_ctx *c, int64_t n_rows_max, const int32_t *in_deg) {
  int64_t cap = (int64_t)(c->big_list.cap / 4);
  if (n_rows_max > cap) n_rows_max = cap;
  const int32_t *n_big = &c->d_cnt->v[C_NBIG];
  return tile_scan<BigChunkCount, BigPrefStore, kScanItems, true>(
      c->ws, BigChunkCount{c->big_list.as<int32_t>(), n_big, in_deg}, BigPrefStore{c->big_pref.as<int32_t>(), n_big},
      n_rows_max, &c->d_cnt->v[C_NCHUNK], c->stream);
}

// row (index in the list), node id and neighbour range of global chunk cg
__device__ __forceinline__ void big_chunk(const int32_t *pref, int n_big, int cg, const int32_t *list,
                                          const int32_t *in_deg, int &i, int &v, int64_t &j0, int64_t &j1) {
  i = wave_last_le(pref, n_big, cg);      // called by whole waves with wave-uniform arguments
  v = list[i];
  int64_t deg = in_deg[v];
  j0 = (int64_t)(cg - pref[i]) * kBigChunk;
  j1 = j0 + kBigChunk < deg ? j0 + kBigChunk : deg;
}

}  // namespace ink
