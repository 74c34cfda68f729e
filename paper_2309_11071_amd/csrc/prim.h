// Device-wide primitives on one HIP stream: exclusive scan, stream compaction and a stable
// LSD radix sort of (u32 key, u32 value) pairs.  All are multi-kernel (reduce / scan the
// block sums / apply), never spin on other workgroups, and are deterministic.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ink {

constexpr int kWave = 64;
constexpr int kScanThreads = 256;
constexpr int kScanItems = 8;
constexpr int kScanTile = kScanThreads * kScanItems;   // items per workgroup

struct DevBuf {            // grow-only device buffer (contents are NOT kept across growth)
  void *p = nullptr;
  size_t cap = 0;
  bool fixed = false;      // p is borrowed memory of exactly cap bytes: never freed, never grown
  hipError_t reserve(size_t bytes) {
    if (bytes <= cap) return hipSuccess;
    if (fixed) return hipErrorOutOfMemory;
    if (p) { hipError_t e = hipFree(p); p = nullptr; cap = 0; if (e != hipSuccess) return e; }
    size_t want = 2 * bytes + 256;       // generous: a buffer that grows again stalls the stream (free + allocate)
    hipError_t e = hipMalloc(&p, want);
    if (e != hipSuccess) { p = nullptr; return e; }
    cap = want;
    return hipSuccess;
  }
  void release() { if (p && !fixed) (void)hipFree(p); p = nullptr; cap = 0; fixed = false; }
  template <class T> T *as() const { return reinterpret_cast<T *>(p); }
};

struct PrimWorkspace {     // scratch shared by scan / compaction / sort calls on one stream
  DevBuf blk;              // block sums
  DevBuf hist;             // radix histograms
  DevBuf tmpk, tmpv;       // radix ping-pong
};

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }

// inclusive scan across the 64 lanes of a wave
__device__ __forceinline__ int wave_incl_scan(int x) {
  int l = lane_id();
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    int y = __shfl_up(x, o, kWave);
    if (l >= o) x += y;
  }
  return x;
}

// exclusive scan over a workgroup of THREADS threads; *total gets the block sum.
// smem must hold THREADS / kWave + 1 ints.  Contains __syncthreads.
template <int THREADS = kScanThreads>
__device__ __forceinline__ int block_excl_scan(int x, int *smem, int *total) {
  int incl = wave_incl_scan(x);
  int w = threadIdx.x / kWave, l = lane_id();
  constexpr int nw = THREADS / kWave;
  __syncthreads();
  if (l == kWave - 1) smem[w] = incl;
  __syncthreads();
  int base = 0, tot = 0;
#pragma unroll
  for (int i = 0; i < nw; i++) {
    int s = smem[i];
    if (i < w) base += s;
    tot += s;
  }
  *total = tot;
  return base + incl - x;
}

// Last index i in [0, n) with a[i] <= key, for ascending a with a[0] <= key.  The whole wave
// searches together, 64 probes per round, so a list of n entries costs ceil(log64 n) dependent
// loads instead of log2 n.  Every lane must call it with the same arguments; all lanes get the result.
__device__ __forceinline__ int wave_last_le(const int32_t *a, int n, int key) {
  const int l = lane_id();
  int lo = 0, len = n;
  while (len > 1) {
    int step = (len + kWave - 1) / kWave;
    int idx = lo + l * step;
    bool ok = idx < lo + len && a[idx] <= key;
    int hit = __popcll(__ballot(ok));          // probes are ascending, so the hits are lanes 0 .. hit-1
    int j = hit > 0 ? hit - 1 : 0;
    int end = lo + len;
    lo += j * step;
    len = end - lo < step ? end - lo : step;
  }
  return lo;
}

// ---------------------------------------------------------------- stable LSD radix sort, 8 bits a pass
constexpr int kRadixBits = 8;
constexpr int kRadix = 1 << kRadixBits;

// One workgroup sorts up to THREADS * ITEMS (key, value) pairs that sit in LDS: per pass every
// wave ranks its own slice digit by digit with ballots, the digit totals are scanned, and the
// pairs are scattered in place (a thread holds its pairs in registers across the barrier).
template <int THREADS, int ITEMS>
struct SmallSortLds {
  uint32_t sk[THREADS * ITEMS];
  uint32_t sv[THREADS * ITEMS];
  int cnt[THREADS / kWave][kRadix];
  int wsum[kRadix / kWave];
};

// On entry sk / sv [0, n) are written (no barrier needed after the writes); on return they hold
// the pairs in ascending key order, equal keys in their input order, and a barrier has passed.
// `passes` 8-bit digits of the key are sorted, lowest first.
template <int THREADS, int ITEMS>
__device__ __forceinline__ void small_sort_lds(SmallSortLds<THREADS, ITEMS> &S, int n, int passes) {
  constexpr int kWaves = THREADS / kWave;
  constexpr int kDigitWaves = kRadix / kWave;    // the waves whose threads own one digit each
  static_assert(THREADS >= kRadix, "one thread per digit");
  const int w = threadIdx.x / kWave, l = lane_id();
  const int per_wave = ITEMS * kWave;
  for (int p = 0; p < passes; p++) {
    int shift = p * kRadixBits;
    for (int i = threadIdx.x; i < kWaves * kRadix; i += THREADS) (&S.cnt[0][0])[i] = 0;
    __syncthreads();
    uint32_t key[ITEMS], val[ITEMS];
    int rank[ITEMS];
#pragma unroll
    for (int k = 0; k < ITEMS; k++) {
      int i = w * per_wave + k * kWave + l;
      bool ok = i < n;
      key[k] = ok ? S.sk[i] : 0xFFFFFFFFu;
      val[k] = ok ? S.sv[i] : 0;
      int dg = ok ? (int)((key[k] >> shift) & (kRadix - 1)) : kRadix;
      uint64_t same = __ballot(ok);
#pragma unroll
      for (int b = 0; b < kRadixBits; b++) {
        uint64_t m = __ballot((dg >> b) & 1);
        same &= ((dg >> b) & 1) ? m : ~m;
      }
      uint64_t lt = (l == 0) ? 0ull : (~0ull >> (kWave - l));
      int before = __popcll(same & lt);
      int prev = 0;
      if (ok) prev = S.cnt[w][dg];
      rank[k] = prev + before;
      bool leader = ok && ((same >> l) >> 1) == 0;
      if (leader) S.cnt[w][dg] = prev + before + 1;
    }
    __syncthreads();
    // digit totals -> exclusive prefix over digits (thread t < kRadix = digit t), then per-wave bases
    const bool digit_thread = threadIdx.x < kRadix;
    int tot = 0, incl = 0;
    if (digit_thread) {
#pragma unroll
      for (int i = 0; i < kWaves; i++) tot += S.cnt[i][threadIdx.x];
      incl = wave_incl_scan(tot);
      if (l == kWave - 1) S.wsum[w] = incl;
    }
    __syncthreads();
    if (digit_thread) {
      int base = 0;
#pragma unroll
      for (int i = 0; i < kDigitWaves; i++) if (i < w) base += S.wsum[i];
      int run = base + incl - tot;
#pragma unroll
      for (int i = 0; i < kWaves; i++) { int c = S.cnt[i][threadIdx.x]; S.cnt[i][threadIdx.x] = run; run += c; }
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < ITEMS; k++) {
      int i = w * per_wave + k * kWave + l;
      if (i < n) {
        int dg = (key[k] >> shift) & (kRadix - 1);
        int pos = S.cnt[w][dg] + rank[k];
        S.sk[pos] = key[k];
        S.sv[pos] = val[k];
      }
    }
    __syncthreads();
  }
}

#define INK_TRY(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) return e_; } while (0)

inline int nblocks(int64_t n, int per) { return (int)((n + per - 1) / per); }

// ---------------------------------------------------------------- generic tile scan machinery
// Functor F: __device__ int operator()(int64_t i) const  -> value of item i
// Functor W: __device__ void operator()(int64_t i, int v, int excl) const -> consume exclusive prefix

template <class F, int ITEMS>
__global__ __launch_bounds__(kScanThreads) void k_tile_reduce(F f, int64_t n, int32_t *blk) {
  __shared__ int sm[kScanThreads / kWave + 1];
  int64_t base = (int64_t)blockIdx.x * (kScanThreads * ITEMS) + (int64_t)threadIdx.x * ITEMS;
  int s = 0;
#pragma unroll
  for (int k = 0; k < ITEMS; k++) {
    int64_t i = base + k;
    if (i < n) s += f(i);
  }
  int tot;
  block_excl_scan(s, sm, &tot);
  if (threadIdx.x == 0) blk[blockIdx.x] = tot;
}

// single workgroup: exclusive scan of blk[0..nb) in place, total to *total
template <int DUMMY>
__global__ __launch_bounds__(kScanThreads) void k_scan_blk(int32_t *blk, int nb, int32_t *total) {
  __shared__ int sm[kScanThreads / kWave + 1];
  int carry = 0;
  for (int b0 = 0; b0 < nb; b0 += kScanThreads) {
    int i = b0 + threadIdx.x;
    int x = i < nb ? blk[i] : 0;
    int tot;
    int ex = block_excl_scan(x, sm, &tot);
    if (i < nb) blk[i] = carry + ex;
    carry += tot;
    __syncthreads();
  }
  if (threadIdx.x == 0 && total) *total = carry;
}

template <class F, class W, int ITEMS>
__global__ __launch_bounds__(kScanThreads) void k_tile_apply(F f, W w, int64_t n, const int32_t *blk,
                                                              int32_t *total_single) {
  __shared__ int sm[kScanThreads / kWave + 1];
  int64_t base = (int64_t)blockIdx.x * (kScanThreads * ITEMS) + (int64_t)threadIdx.x * ITEMS;
  int v[ITEMS];
  int s = 0;
#pragma unroll
  for (int k = 0; k < ITEMS; k++) {
    int64_t i = base + k;
    v[k] = i < n ? f(i) : 0;
    s += v[k];
  }
  int tot;
  int ex = block_excl_scan(s, sm, &tot);
  ex += blk ? blk[blockIdx.x] : 0;
#pragma unroll
  for (int k = 0; k < ITEMS; k++) {
    int64_t i = base + k;
    if (i < n) w(i, v[k], ex);
    ex += v[k];
  }
  if (total_single && threadIdx.x == 0) *total_single = tot;   // only used when gridDim.x == 1
}

// short inputs: the whole scan in one workgroup and one launch, tile after tile with a carry
constexpr int kOneWgThreads = 1024;
constexpr int kOneWgItems = 4;
constexpr int64_t kOneWgLimit = 16384;
template <class F, class W>
__global__ __launch_bounds__(kOneWgThreads) void k_tile_scan_one(F f, W w, int64_t n, int32_t *total) {
  __shared__ int sm[kOneWgThreads / kWave + 1];
  int carry = 0;
  for (int64_t t0 = 0; t0 < n; t0 += kOneWgThreads * kOneWgItems) {
    int64_t base = t0 + (int64_t)threadIdx.x * kOneWgItems;
    int v[kOneWgItems];
    int s = 0;
#pragma unroll
    for (int k = 0; k < kOneWgItems; k++) {
      int64_t i = base + k;
      v[k] = i < n ? f(i) : 0;
      s += v[k];
    }
    int tot;
    int ex = carry + block_excl_scan<kOneWgThreads>(s, sm, &tot);
#pragma unroll
    for (int k = 0; k < kOneWgItems; k++) {
      int64_t i = base + k;
      if (i < n) w(i, v[k], ex);
      ex += v[k];
    }
    carry += tot;
    __syncthreads();
  }
  if (total && threadIdx.x == 0) *total = carry;
}

// ONE_WG: only for functors that do O(1) work per item
template <class F, class W, int ITEMS = kScanItems, bool ONE_WG = false>
inline hipError_t tile_scan(PrimWorkspace &ws, F f, W w, int64_t n, int32_t *total, hipStream_t s) {
  if (n <= 0) {
    if (total) INK_TRY(hipMemsetAsync(total, 0, sizeof(int32_t), s));
    return hipSuccess;
  }
  int nb = nblocks(n, kScanThreads * ITEMS);
  if (nb == 1) {
    hipLaunchKernelGGL((k_tile_apply<F, W, ITEMS>), dim3(1), dim3(kScanThreads), 0, s, f, w, n,
                       (const int32_t *)nullptr, total);
    return hipGetLastError();
  }
  if (ONE_WG && n <= kOneWgLimit) {
    hipLaunchKernelGGL((k_tile_scan_one<F, W>), dim3(1), dim3(kOneWgThreads), 0, s, f, w, n, total);
    return hipGetLastError();
  }
  INK_TRY(ws.blk.reserve((size_t)nb * sizeof(int32_t)));
  int32_t *blk = ws.blk.as<int32_t>();
  hipLaunchKernelGGL((k_tile_reduce<F, ITEMS>), dim3(nb), dim3(kScanThreads), 0, s, f, n, blk);
  hipLaunchKernelGGL((k_scan_blk<0>), dim3(1), dim3(kScanThreads), 0, s, blk, nb, total);
  hipLaunchKernelGGL((k_tile_apply<F, W, ITEMS>), dim3(nb), dim3(kScanThreads), 0, s, f, w, n,
                     (const int32_t *)blk, (int32_t *)nullptr);
  return hipGetLastError();
}

// out[i] = sum_{j<i} in[j] for i < n, *total = sum of all (device pointers; total may alias nothing)
hipError_t scan_excl_i32(PrimWorkspace &ws, const int32_t *in, int32_t *out, int64_t n,
                         int32_t *total, hipStream_t s);

// indices i < n with flags[i] != 0, ascending, to out_idx; *count = how many
hipError_t compact_flags_u8(PrimWorkspace &ws, const uint8_t *flags, int64_t n, int32_t *out_idx,
                            int32_t *count, hipStream_t s);

// set bits of a bitmap of n_bits bits (uint64 words, bit b of word w = item 64 w + b) as an
// ascending list; words are cleared to zero afterwards if clear != 0
hipError_t bitmap_to_list(PrimWorkspace &ws, uint64_t *words, int64_t n_bits, int32_t *out_idx,
                          int32_t *count, int clear, hipStream_t s);

// segment heads of a sorted key array: uniq[j] = j-th distinct key, seg[j] = first index of its
// run, seg[*count] = n
// n_dev (optional): device-side number of valid keys, n is then an upper bound
hipError_t segment_heads(PrimWorkspace &ws, const uint32_t *keys, int64_t n, int32_t *uniq,
                         int32_t *seg, int32_t *count, hipStream_t s, const int32_t *n_dev = nullptr);

// stable sort of (key, val) pairs by the low `bits` bits of key, in place (uses ws.tmpk / tmpv)
hipError_t radix_sort_pairs(PrimWorkspace &ws, uint32_t *keys, uint32_t *vals, int64_t n, int bits,
                            hipStream_t s);

}  // namespace ink
