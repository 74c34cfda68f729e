// Scan, compaction and radix sort kernels (gfx950, wave64).
#include "prim.h"

namespace ink {


// ---------------------------------------------------------------- scan of an int array
struct LoadI32 { const int32_t *p; __device__ int operator()(int64_t i) const { return p[i]; } };
struct StoreExcl { int32_t *p; __device__ void operator()(int64_t i, int, int ex) const { p[i] = ex; } };

hipError_t scan_excl_i32(PrimWorkspace &ws, const int32_t *in, int32_t *out, int64_t n,
                         int32_t *total, hipStream_t s) {
  return tile_scan<LoadI32, StoreExcl, kScanItems, true>(ws, LoadI32{in}, StoreExcl{out}, n, total, s);
}

// ---------------------------------------------------------------- flag compaction
struct LoadFlag { const uint8_t *p; __device__ int operator()(int64_t i) const { return p[i] != 0; } };
struct StoreIdx {
  int32_t *p;
  __device__ void operator()(int64_t i, int v, int ex) const { if (v) p[ex] = (int32_t)i; }
};

hipError_t compact_flags_u8(PrimWorkspace &ws, const uint8_t *flags, int64_t n, int32_t *out_idx,
                            int32_t *count, hipStream_t s) {
  return tile_scan<LoadFlag, StoreIdx, kScanItems, true>(ws, LoadFlag{flags}, StoreIdx{out_idx}, n, count, s);
}

// ---------------------------------------------------------------- bitmap -> ascending id list
struct LoadPop { const uint64_t *p; __device__ int operator()(int64_t i) const { return __popcll(p[i]); } };
struct StoreBits {
  uint64_t *words; int32_t *out; int clear;
  __device__ void operator()(int64_t i, int v, int ex) const {
    if (!v) return;
    uint64_t w = words[i];
    while (w) {
      int b = __ffsll((unsigned long long)w) - 1;
      out[ex++] = (int32_t)(i * 64 + b);
      w &= w - 1;
    }
    if (clear) words[i] = 0;
  }
};

hipError_t bitmap_to_list(PrimWorkspace &ws, uint64_t *words, int64_t n_bits, int32_t *out_idx,
                          int32_t *count, int clear, hipStream_t s) {
  int64_t nw = (n_bits + 63) / 64;
  return tile_scan<LoadPop, StoreBits, 1>(ws, LoadPop{words}, StoreBits{words, out_idx, clear}, nw, count, s);
}

// ---------------------------------------------------------------- segment heads of sorted keys
struct LoadHead {
  const uint32_t *k; const int32_t *n_dev;
  __device__ int operator()(int64_t i) const {
    if (n_dev && i >= *n_dev) return 0;
    return i == 0 || k[i] != k[i - 1];
  }
};
struct StoreHead {
  const uint32_t *k; int32_t *uniq; int32_t *seg; int64_t n; const int32_t *n_dev;
  __device__ void operator()(int64_t i, int v, int ex) const {
    if (v) { uniq[ex] = (int32_t)k[i]; seg[ex] = (int32_t)i; }
    int64_t nn = n_dev ? (int64_t)*n_dev : n;
    if (i == nn - 1) seg[ex + v] = (int32_t)nn;    // closing offset after the last run
  }
};

hipError_t segment_heads(PrimWorkspace &ws, const uint32_t *keys, int64_t n, int32_t *uniq,
                         int32_t *seg, int32_t *count, hipStream_t s, const int32_t *n_dev) {
  return tile_scan<LoadHead, StoreHead, kScanItems, true>(ws, LoadHead{keys, n_dev}, StoreHead{keys, uniq, seg, n, n_dev}, n, count,
                                                             s);
}

// ---------------------------------------------------------------- stable LSD radix sort
constexpr int kSortThreads = 256;
constexpr int kSortWaves = kSortThreads / kWave;
#ifndef INK_SORT_ITEMS
#define INK_SORT_ITEMS 12     // measured on 3.4 x 10^7 pairs: 8 -> 1.25 ms, 12 -> 1.18 ms, 16 -> 1.18 ms
#endif
constexpr int kSortItems = INK_SORT_ITEMS;                    // keys per thread
constexpr int kSortTile = kSortThreads * kSortItems;          // keys per workgroup

// hist[d * nb + b] = number of keys of tile b with digit d
__global__ __launch_bounds__(kSortThreads) void k_radix_hist(const uint32_t *keys, int64_t n, int shift,
                                                              int32_t *hist, int nb) {
  __shared__ int h[kRadix];
  h[threadIdx.x] = 0;
  __syncthreads();
  int64_t base = (int64_t)blockIdx.x * kSortTile;
#pragma unroll
  for (int k = 0; k < kSortItems; k++) {
    int64_t i = base + k * kSortThreads + threadIdx.x;
    if (i < n) atomicAdd(&h[(keys[i] >> shift) & (kRadix - 1)], 1);
  }
  __syncthreads();
  hist[(int64_t)threadIdx.x * nb + blockIdx.x] = h[threadIdx.x];
}

// Each wave owns a contiguous run of kSortItems * 64 keys of the tile and walks it in rounds of
// 64 consecutive keys, so ranks follow the input order (stability).  The pairs are first put in
// digit order inside LDS and written out from there, so that neighbouring lanes store to
// neighbouring addresses (runs of one digit) instead of 64 unrelated ones per instruction.
__global__ __launch_bounds__(kSortThreads) void k_radix_scatter(const uint32_t *keys, const uint32_t *vals,
                                                                 uint32_t *okeys, uint32_t *ovals, int64_t n,
                                                                 int shift, const int32_t *hist_scanned, int nb) {
  static_assert(kSortThreads == kRadix, "one thread per digit");
  __shared__ int cnt[kSortWaves][kRadix];      // per-wave digit counts, then the wave's first slot of the digit in the tile
  __shared__ int tile_first[kRadix];           // first slot of the digit in the tile
  __shared__ int64_t out_first[kRadix];        // first position of the tile's keys of the digit in the output
  __shared__ uint32_t skey[kSortTile], sval[kSortTile];
  __shared__ int sm[kSortWaves + 1];
  int w = threadIdx.x / kWave, l = lane_id();
  for (int i = threadIdx.x; i < kSortWaves * kRadix; i += kSortThreads) (&cnt[0][0])[i] = 0;
  __syncthreads();
  const int64_t tbase = (int64_t)blockIdx.x * kSortTile;
  int64_t wbase = tbase + (int64_t)w * (kSortItems * kWave);
  uint32_t key[kSortItems], val[kSortItems];
  int rank[kSortItems];
#pragma unroll
  for (int k = 0; k < kSortItems; k++) {
    int64_t i = wbase + k * kWave + l;
    bool ok = i < n;
    key[k] = ok ? keys[i] : 0xFFFFFFFFu;
    val[k] = ok ? vals[i] : 0;
    int dg = ok ? (int)((key[k] >> shift) & (kRadix - 1)) : kRadix;   // kRadix = "no key"
    // lanes holding the same digit
    uint64_t same = __ballot(ok);
#pragma unroll
    for (int b = 0; b < kRadixBits; b++) {
      uint64_t m = __ballot((dg >> b) & 1);
      same &= ((dg >> b) & 1) ? m : ~m;
    }
    uint64_t lt = (l == 0) ? 0ull : (~0ull >> (kWave - l));
    int before = __popcll(same & lt);
    int prev = 0;
    if (ok) prev = cnt[w][dg];                 // all lanes of a digit group read the same value
    rank[k] = prev + before;
    // the last lane of each group publishes the new count (after every lane has read)
    bool leader = ok && ((same >> l) >> 1) == 0;
    if (leader) cnt[w][dg] = prev + before + 1;
  }
  __syncthreads();
  // thread t handles digit t: its total in the tile, the exclusive prefix over digits, the waves' slots
  {
    const int d = threadIdx.x;
    int tot = 0;
#pragma unroll
    for (int i = 0; i < kSortWaves; i++) tot += cnt[i][d];
    int all;
    int first = block_excl_scan<kSortThreads>(tot, sm, &all);
    tile_first[d] = first;
    out_first[d] = (int64_t)hist_scanned[(int64_t)d * nb + blockIdx.x];
    int run = first;
#pragma unroll
    for (int i = 0; i < kSortWaves; i++) {
      int c = cnt[i][d];
      cnt[i][d] = run;
      run += c;
    }
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < kSortItems; k++) {
    int64_t i = wbase + k * kWave + l;
    if (i < n) {
      int dg = (key[k] >> shift) & (kRadix - 1);
      int slot = cnt[w][dg] + rank[k];
      skey[slot] = key[k];
      sval[slot] = val[k];
    }
  }
  __syncthreads();
  const int in_tile = (int)(n - tbase < kSortTile ? n - tbase : kSortTile);
  for (int s = threadIdx.x; s < in_tile; s += kSortThreads) {
    uint32_t kk = skey[s];
    int dg = (kk >> shift) & (kRadix - 1);
    int64_t pos = out_first[dg] + (s - tile_first[dg]);
    okeys[pos] = kk;
    ovals[pos] = sval[s];
  }
}

// Whole sort in one workgroup: the same stable digit ranking, all passes in LDS, one launch.
// Keys live in registers between the ranking and the scatter of a pass, so one LDS copy of the
// pairs is enough.  THREADS x ITEMS pairs at most: 256 x {1,4,16} for short lists, 1024 x 16
// (128 KB of pairs) up to kSmallSort.
constexpr int kWideThreads = 1024;
constexpr int kSmallItems = 16;
constexpr int kSmallSort = kWideThreads * kSmallItems;     // 16384 pairs

template <int THREADS, int ITEMS>
__global__ __launch_bounds__(THREADS) void k_small_sort(uint32_t *keys, uint32_t *vals, int n, int passes) {
  __shared__ SmallSortLds<THREADS, ITEMS> S;
  for (int i = threadIdx.x; i < n; i += THREADS) { S.sk[i] = keys[i]; S.sv[i] = vals[i]; }
  small_sort_lds<THREADS, ITEMS>(S, n, passes);
  for (int i = threadIdx.x; i < n; i += THREADS) { keys[i] = S.sk[i]; vals[i] = S.sv[i]; }
}

hipError_t radix_sort_pairs(PrimWorkspace &ws, uint32_t *keys, uint32_t *vals, int64_t n, int bits,
                            hipStream_t s) {
  if (n <= 1 || bits <= 0) return hipSuccess;
  int passes = (bits + kRadixBits - 1) / kRadixBits;
  if (n <= kSmallSort) {
    if (n <= 256)
      hipLaunchKernelGGL((k_small_sort<256, 1>), dim3(1), dim3(256), 0, s, keys, vals, (int)n, passes);
    else if (n <= 1024)
      hipLaunchKernelGGL((k_small_sort<256, 4>), dim3(1), dim3(256), 0, s, keys, vals, (int)n, passes);
    else if (n <= 4096)
      hipLaunchKernelGGL((k_small_sort<kWideThreads, 4>), dim3(1), dim3(kWideThreads), 0, s, keys, vals, (int)n, passes);
    else
      hipLaunchKernelGGL((k_small_sort<kWideThreads, kSmallItems>), dim3(1), dim3(kWideThreads), 0, s, keys, vals, (int)n, passes);
    return hipGetLastError();
  }
  int nb = nblocks(n, kSortTile);
  INK_TRY(ws.hist.reserve((size_t)kRadix * nb * sizeof(int32_t)));
  INK_TRY(ws.tmpk.reserve((size_t)n * sizeof(uint32_t)));
  INK_TRY(ws.tmpv.reserve((size_t)n * sizeof(uint32_t)));
  int32_t *hist = ws.hist.as<int32_t>();
  uint32_t *ka = keys, *va = vals, *kb = ws.tmpk.as<uint32_t>(), *vb = ws.tmpv.as<uint32_t>();
  for (int p = 0; p < passes; p++) {
    int shift = p * kRadixBits;
    hipLaunchKernelGGL(k_radix_hist, dim3(nb), dim3(kSortThreads), 0, s, (const uint32_t *)ka, n, shift, hist, nb);
    INK_TRY(scan_excl_i32(ws, hist, hist, (int64_t)kRadix * nb, nullptr, s));
    hipLaunchKernelGGL(k_radix_scatter, dim3(nb), dim3(kSortThreads), 0, s, (const uint32_t *)ka,
                       (const uint32_t *)va, kb, vb, n, shift, (const int32_t *)hist, nb);
    uint32_t *t = ka; ka = kb; kb = t;
    t = va; va = vb; vb = t;
  }
  if (ka != keys) {
    INK_TRY(hipMemcpyAsync(keys, ka, (size_t)n * sizeof(uint32_t), hipMemcpyDeviceToDevice, s));
    INK_TRY(hipMemcpyAsync(vals, va, (size_t)n * sizeof(uint32_t), hipMemcpyDeviceToDevice, s));
  }
  return hipGetLastError();
}

}  // namespace ink
