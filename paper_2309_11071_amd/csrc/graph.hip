// Device graph store: for each direction (in-neighbours for aggregation / recompute, Sec. 2.5.2;
// out-neighbours for event propagation, Sec. 2.4.2) every node owns a block of ids with slack
// inside one pool.  A batch is normalised to its net effect on the edge set, then applied per
// touched node: deleted slots are refilled from the block's tail, inserted ids are appended, a
// full block moves to a larger one at the pool's end.  Every step is a deterministic function of
// the batch and the current store.
#include <algorithm>
#include <vector>

#include "ctx.h"

namespace ink {


#define INK_TRYS(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { c->err = std::string("HIP error: ") + hipGetErrorString(e_); return INK_E_DEVICE; } } while (0)

static inline int64_t align4(int64_t x) { return (x + 3) & ~(int64_t)3; }

static int32_t block_cap(int64_t deg, float slack) {
  int64_t extra = (int64_t)(deg * (double)slack + 0.999);
  if (extra < 4) extra = 4;
  return (int32_t)align4(deg + extra);
}

static hipError_t side_alloc(GraphSide &g, int n, const std::vector<int64_t> &off, const std::vector<int32_t> &deg,
                             const std::vector<int32_t> &cap, const std::vector<int32_t> &ids, int64_t top,
                             int64_t reserve_opt) {
  int64_t reserve = reserve_opt > 0 ? reserve_opt : std::max<int64_t>(top / 4, 1 << 20);
  g.pool_cap = top + reserve;
  g.pool_top = top;
  INK_TRY(hipMalloc(&g.off, sizeof(int64_t) * (size_t)n));
  INK_TRY(hipMalloc(&g.deg, sizeof(int32_t) * (size_t)n));
  INK_TRY(hipMalloc(&g.cap, sizeof(int32_t) * (size_t)n));
  INK_TRY(hipMalloc(&g.asc, (size_t)n));
  INK_TRY(hipMemset(g.asc, 1, (size_t)n));       // built from ascending CSR rows; empty blocks are ascending too
  INK_TRY(hipMalloc(&g.ids, sizeof(int32_t) * (size_t)g.pool_cap));
  INK_TRY(hipMemcpy(g.off, off.data(), sizeof(int64_t) * (size_t)n, hipMemcpyHostToDevice));
  INK_TRY(hipMemcpy(g.deg, deg.data(), sizeof(int32_t) * (size_t)n, hipMemcpyHostToDevice));
  INK_TRY(hipMemcpy(g.cap, cap.data(), sizeof(int32_t) * (size_t)n, hipMemcpyHostToDevice));
  INK_TRY(hipMemcpy(g.ids, ids.data(), sizeof(int32_t) * (size_t)top, hipMemcpyHostToDevice));
  return hipSuccess;
}

hipError_t graph_build(ink_ctx *c, const int64_t *rowptr, const int32_t *col) {
  const int n = c->n;
  const int nc = (int)c->n_cap;        // per-node arrays cover the capacity; nodes >= n own no block yet
  const int64_t E = rowptr[n];
  std::vector<int64_t> off(nc, 0);
  std::vector<int32_t> deg(nc, 0), cap(nc, 0);
  // in side straight from the CSR
  int64_t top = 0;
  for (int v = 0; v < n; v++) {
    int64_t d = rowptr[v + 1] - rowptr[v];
    off[v] = top; deg[v] = (int32_t)d; cap[v] = block_cap(d, c->slack);
    top += cap[v];
  }
  {
    std::vector<int32_t> ids((size_t)top, -1);
    for (int v = 0; v < n; v++) std::copy(col + rowptr[v], col + rowptr[v + 1], ids.begin() + off[v]);
    INK_TRY(side_alloc(c->gin, nc, off, deg, cap, ids, top, c->pool_reserve));
  }
  // out side: transpose
  std::vector<int32_t> odeg(n, 0);
  for (int64_t e = 0; e < E; e++) odeg[col[e]]++;
  top = 0;
  for (int v = 0; v < n; v++) {
    off[v] = top; deg[v] = odeg[v]; cap[v] = block_cap(odeg[v], c->slack);
    top += cap[v];
  }
  {
    std::vector<int32_t> ids((size_t)top, -1);
    std::vector<int64_t> cur(off);
    for (int v = 0; v < n; v++)
      for (int64_t e = rowptr[v]; e < rowptr[v + 1]; e++) ids[cur[col[e]]++] = v;
    INK_TRY(side_alloc(c->gout, nc, off, deg, cap, ids, top, c->pool_reserve));
  }
  return hipSuccess;
}

hipError_t graph_export(ink_ctx *c, int64_t *rowptr, int32_t *col) {
  const int n = c->n;
  std::vector<int64_t> off(n);
  std::vector<int32_t> deg(n);
  INK_TRY(hipMemcpy(off.data(), c->gin.off, sizeof(int64_t) * (size_t)n, hipMemcpyDeviceToHost));
  INK_TRY(hipMemcpy(deg.data(), c->gin.deg, sizeof(int32_t) * (size_t)n, hipMemcpyDeviceToHost));
  rowptr[0] = 0;
  for (int v = 0; v < n; v++) rowptr[v + 1] = rowptr[v] + deg[v];
  if (!col) return hipSuccess;
  std::vector<int32_t> pool((size_t)c->gin.pool_top);
  INK_TRY(hipMemcpy(pool.data(), c->gin.ids, sizeof(int32_t) * pool.size(), hipMemcpyDeviceToHost));
  for (int v = 0; v < n; v++) {
    std::copy(pool.begin() + off[v], pool.begin() + off[v] + deg[v], col + rowptr[v]);
    std::sort(col + rowptr[v], col + rowptr[v + 1]);
  }
  return hipSuccess;
}

// ------------------------------------------------------------------------------- batch kernels
struct RawUpdate { uint8_t op; uint8_t pad[3]; int32_t src, dst; };

// what is wrong with a list entry: bit 0 = op is neither insert nor delete, bit 1 = id out of range
__device__ __forceinline__ int entry_error(const RawUpdate &a, int n_nodes) {
  int e = a.op > 1 ? 1 : 0;
  if (a.src < 0 || a.src >= n_nodes || a.dst < 0 || a.dst >= n_nodes) e |= 2;
  return e;
}

// Also validates the batch: a bad entry sets *err, and no kernel uses an id as an index before
// k_mark_last has seen *err and dropped every entry.
__global__ void k_unpack(const RawUpdate *raw, int64_t n, int n_nodes, uint32_t *src, uint32_t *dst, uint32_t *pos,
                         int32_t *err) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  RawUpdate a = raw[i];
  int e = entry_error(a, n_nodes);
  if (e) atomicOr(err, e);
  src[i] = (uint32_t)a.src;
  dst[i] = (uint32_t)a.dst;
  pos[i] = (uint32_t)i;
}

__global__ void k_gather_u32(const uint32_t *table, const uint32_t *idx, int64_t n, uint32_t *out) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) out[i] = table[idx[i]];
}

// entry j (in (dst, src, position) order) is the final word on its edge if the next entry names
// another edge; self loops never count
__global__ void k_mark_last(const RawUpdate *raw, const uint32_t *perm, int64_t n, uint8_t *flag, const int32_t *err) {
  int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= n) return;
  if (*err) { flag[j] = 0; return; }
  RawUpdate a = raw[perm[j]];
  bool last = true;
  if (j + 1 < n) {
    RawUpdate b = raw[perm[j + 1]];
    last = (a.src != b.src) || (a.dst != b.dst);
  }
  flag[j] = last && a.src != a.dst;
}

// unique ops in (dst, src) order: node = dst, other = src, op = final op
__global__ void k_take_ops(const RawUpdate *raw, const uint32_t *perm, const int32_t *idx, const int32_t *count,
                           uint32_t *node, int32_t *other, uint8_t *op, int32_t *pos) {
  int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (k >= *count) return;
  RawUpdate a = raw[perm[idx[k]]];
  node[k] = (uint32_t)a.dst;
  other[k] = a.src;
  op[k] = a.op;
  pos[k] = -1;
}

// chunks of 2048 block slots per touched node
constexpr int kChunk = 2048;
__global__ void k_chunk_counts(const int32_t *nodes, const int32_t *n_nodes, int64_t n_max, const int32_t *deg,
                               int32_t *chunks) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_max) return;
  chunks[i] = i < *n_nodes ? (deg[nodes[i]] + kChunk - 1) / kChunk : 0;
}

// Walk the blocks of the touched nodes; an id found in the node's op list records its slot and,
// if the op is a delete, becomes a tombstone (-1).
__global__ __launch_bounds__(256) void k_classify(const int32_t *nodes, const int32_t *n_nodes, const int32_t *seg,
                                                  const int32_t *chunk_pref, const int32_t *n_chunks,
                                                  const int64_t *off, const int32_t *deg, int32_t *ids,
                                                  const int32_t *other, const uint8_t *op, int32_t *pos) {
  int total = *n_chunks, nn = *n_nodes;
  for (int ch = blockIdx.x; ch < total; ch += gridDim.x) {
    // node owning this chunk: last i with chunk_pref[i] <= ch
    int i = wave_last_le(chunk_pref, nn, ch);
    int v = nodes[i];
    int s0 = seg[i], s1 = seg[i + 1];
    int d = deg[v];
    int64_t base = off[v];
    int p0 = (ch - chunk_pref[i]) * kChunk;
    int p1 = p0 + kChunk < d ? p0 + kChunk : d;
    for (int p = p0 + threadIdx.x; p < p1; p += blockDim.x) {
      int e = ids[base + p];
      int a = s0, b = s1 - 1;
      while (a <= b) {
        int m = (a + b) >> 1;
        int x = other[m];
        if (x == e) {
          pos[m] = p;
          if (op[m] == 1) ids[base + p] = -1;
          break;
        }
        if (x < e) a = m + 1; else b = m - 1;
      }
    }
  }
}

// per touched node: effective op flags, counts and the pool space a relocation would need.
// eff: 0 no-op, 1 insert, 2 delete.  One wave per node.
__global__ __launch_bounds__(256) void k_effect(const int32_t *nodes, const int32_t *n_nodes, const int32_t *seg,
                                                const uint8_t *op, const int32_t *pos, uint8_t *eff,
                                                const int32_t *deg, const int32_t *cap, int32_t *nd_ins,
                                                int32_t *nd_del, float slack, Counters *cnt, int st_need,
                                                int st_ins, int st_del) {
  int64_t w = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / kWave;
  int l = threadIdx.x & (kWave - 1);
  if (w >= *n_nodes) return;
  int s0 = seg[w], s1 = seg[w + 1];
  int ni = 0, nd = 0;
  for (int k = s0 + l; k < s1; k += kWave) {
    int e = 0;
    if (op[k] == 0) e = pos[k] < 0 ? 1 : 0;
    else e = pos[k] >= 0 ? 2 : 0;
    eff[k] = (uint8_t)e;
    ni += e == 1;
    nd += e == 2;
  }
  for (int o = 32; o > 0; o >>= 1) { ni += __shfl_xor(ni, o, kWave); nd += __shfl_xor(nd, o, kWave); }
  if (l == 0) {
    int v = nodes[w];
    nd_ins[w] = ni; nd_del[w] = nd;
    int nd2 = deg[v] - nd + ni;
    if (nd2 > cap[v]) {
      long long want = 2ll * cap[v];
      long long extra = (long long)(nd2 * (double)slack + 0.999);
      if (extra < 4) extra = 4;
      if (want < nd2 + extra) want = nd2 + extra;
      want = (want + 3) & ~3ll;
      atomicAdd(&cnt->stripe[blockIdx.x % kStripes][st_need], (unsigned long long)want);   // pool space needed
    }
    if (ni) atomicAdd(&cnt->stripe[blockIdx.x % kStripes][st_ins], (unsigned long long)ni);  // effective inserts
    if (nd) atomicAdd(&cnt->stripe[blockIdx.x % kStripes][st_del], (unsigned long long)nd);  // effective deletes
  }
}

// One workgroup per touched node: refill deleted slots from the tail, relocate if the block is
// too small, append inserted ids.  `fill` is scratch with one slot per op of the batch.
__global__ __launch_bounds__(256) void k_apply(const int32_t *nodes, const int32_t *seg, const int32_t *other,
                                               const uint8_t *eff, const int32_t *pos, const int32_t *nd_ins,
                                               const int32_t *nd_del, int64_t *off, int32_t *deg, int32_t *cap,
                                               int32_t *ids, unsigned long long *pool_used,
                                               unsigned long long pool_base, float slack, int32_t *fill,
                                               int32_t *new_cnt, uint8_t *asc) {
  __shared__ int sm[kScanThreads / kWave + 1];
  __shared__ long long s_off, s_newoff;
  __shared__ int s_deg, s_cap;
  const int i = blockIdx.x;
  const int v = nodes[i];
  const int s0 = seg[i], s1 = seg[i + 1];
  const int ni = nd_ins[i], nd = nd_del[i];
  if (ni == 0 && nd == 0) return;
  // The block's descriptor is read once, by one thread, and handed to the others through LDS;
  // it is written back only after the last barrier.  (Every wave reading off / cap from global
  // memory raced with the relocation below, which rewrites both.)
  if (threadIdx.x == 0) { s_off = off[v]; s_deg = deg[v]; s_cap = cap[v]; }
  __syncthreads();
  const int d0 = s_deg;
  const int cap0 = s_cap;
  const int d1 = d0 - nd;             // survivors of the old block
  int64_t base = s_off;
  if (nd > 0) {
    // survivors in the tail [d1, d0), in slot order -> fill[s0 ...]
    int carry = 0;
    for (int p0 = d1; p0 < d0; p0 += kScanThreads) {
      int p = p0 + threadIdx.x;
      int e = p < d0 ? ids[base + p] : -1;
      int tot;
      int ex = block_excl_scan(e >= 0 ? 1 : 0, sm, &tot);
      if (e >= 0) fill[s0 + carry + ex] = e;
      carry += tot;
      __syncthreads();
    }
    __threadfence_block();
    __syncthreads();
    // holes in the head [0, d1), in op order, take them in turn
    carry = 0;
    for (int k0 = s0; k0 < s1; k0 += kScanThreads) {
      int k = k0 + threadIdx.x;
      bool hole = k < s1 && eff[k] == 2 && pos[k] < d1;
      int tot;
      int ex = block_excl_scan(hole ? 1 : 0, sm, &tot);
      if (hole) ids[base + pos[k]] = fill[s0 + carry + ex];
      carry += tot;
      __syncthreads();
    }
  }
  const int d2 = d1 + ni;
  const bool move = d2 > cap0;        // workgroup-uniform: taken from the LDS copy
  long long want = cap0;
  if (move) {
    want = 2ll * cap0;
    long long extra = (long long)(d2 * (double)slack + 0.999);
    if (extra < 4) extra = 4;
    if (want < d2 + extra) want = d2 + extra;
    want = (want + 3) & ~3ll;
    if (threadIdx.x == 0) s_newoff = (long long)(pool_base + atomicAdd(pool_used, (unsigned long long)want));
    __syncthreads();
    int64_t nb = s_newoff;
    for (int p = threadIdx.x; p < d1; p += blockDim.x) ids[nb + p] = ids[base + p];
    base = nb;
    __syncthreads();
  }
  if (ni > 0) {
    int carry = 0;
    for (int k0 = s0; k0 < s1; k0 += kScanThreads) {
      int k = k0 + threadIdx.x;
      bool ins = k < s1 && eff[k] == 1;
      int tot;
      int ex = block_excl_scan(ins ? 1 : 0, sm, &tot);
      if (ins) ids[base + d1 + carry + ex] = other[k];
      carry += tot;
      __syncthreads();
    }
  }
  if (threadIdx.x == 0) {
    if (move) { cap[v] = (int32_t)want; off[v] = base; }
    deg[v] = d2;
    asc[v] = 0;              // holes were refilled from the tail / ids appended: order no longer known
    if (new_cnt) new_cnt[v] = ni;
  }
}

// effective ops -> Delta E lists in (node, other) order
__global__ void k_split_ops(const uint32_t *node, const int32_t *other, const uint8_t *eff, const int32_t *n_ops,
                            const int32_t *idx_ins, const int32_t *idx_del, int32_t *ins_s, int32_t *ins_d,
                            int32_t *del_s, int32_t *del_d, const int32_t *n_ins, const int32_t *n_del) {
  int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (k < *n_ins) { int j = idx_ins[k]; ins_s[k] = other[j]; ins_d[k] = (int32_t)node[j]; }
  if (k < *n_del) { int j = idx_del[k]; del_s[k] = other[j]; del_d[k] = (int32_t)node[j]; }
}
__global__ void k_flag_eq(const uint8_t *eff, const int32_t *n_ops, int64_t n_max, uint8_t want, uint8_t *flag) {
  int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (k < n_max) flag[k] = k < *n_ops && eff[k] == want;
}

// out side: ops = [deletes | inserts] keyed by source
__global__ void k_out_ops(const int32_t *del_s, const int32_t *del_d, const int32_t *ins_s, const int32_t *ins_d,
                          int n_del, int n_ins, uint32_t *key, uint32_t *val) {
  int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (k < n_del) { key[k] = (uint32_t)del_s[k]; val[k] = (uint32_t)k; }
  else if (k < n_del + n_ins) { key[k] = (uint32_t)ins_s[k - n_del]; val[k] = (uint32_t)k; }
}
// after a stable sort by source of entries that were in (dst, src) order per kind, entries of one
// source are not yet ordered by destination across the two kinds; a second stable sort fixes the
// order: we sort by destination first, then by source (both stable)
__global__ void k_out_dst_key(const int32_t *del_d, const int32_t *ins_d, int n_del, int n_ins, uint32_t *key,
                              uint32_t *val) {
  int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (k < n_del) { key[k] = (uint32_t)del_d[k]; val[k] = (uint32_t)k; }
  else if (k < n_del + n_ins) { key[k] = (uint32_t)ins_d[k - n_del]; val[k] = (uint32_t)k; }
}
__global__ void k_out_take(const uint32_t *perm, const int32_t *del_s, const int32_t *del_d, const int32_t *ins_s,
                           const int32_t *ins_d, int n_del, int n_ins, uint32_t *node, int32_t *other, uint8_t *op,
                           int32_t *pos) {
  int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (k >= n_del + n_ins) return;
  int j = (int)perm[k];
  if (j < n_del) { node[k] = (uint32_t)del_s[j]; other[k] = del_d[j]; op[k] = 1; }
  else { node[k] = (uint32_t)ins_s[j - n_del]; other[k] = ins_d[j - n_del]; op[k] = 0; }
  pos[k] = -1;
}

__global__ void k_zero_at(const int32_t *nodes, int n, int32_t *arr) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) arr[nodes[i]] = 0;
}

__global__ void k_copy_blocks(int n, const int64_t *off, const int32_t *deg, const int32_t *src, int32_t *dst) {
  // one wave per node; offsets are unchanged (same layout in a larger pool)
  int64_t w = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / kWave;
  int l = threadIdx.x & (kWave - 1);
  if (w >= n) return;
  int64_t o = off[w];
  int d = deg[w];
  for (int p = l; p < d; p += kWave) dst[o + p] = src[o + p];
}

static inline dim3 grid1(int64_t n, int per = 256) { return dim3((unsigned)std::max<int64_t>(1, (n + per - 1) / per)); }

struct Arena {
  char *base; size_t used = 0, cap;
  Arena(DevBuf &b) : base((char *)b.p), cap(b.cap) {}
  template <class T> T *get(size_t n) {
    size_t bytes = (n * sizeof(T) + 255) & ~(size_t)255;
    T *p = (T *)(base + used);
    used += bytes;
    return p;
  }
};

static hipError_t grow_pool(ink_ctx *c, GraphSide &g, int64_t need_total) {
  int64_t new_cap = std::max<int64_t>(g.pool_cap * 2, g.pool_top + need_total + (1 << 20));
  int32_t *np = nullptr;
  INK_TRY(hipMalloc(&np, sizeof(int32_t) * (size_t)new_cap));
  hipLaunchKernelGGL(k_copy_blocks, grid1((int64_t)c->n * kWave), dim3(256), 0, c->stream, c->n,
                     (const int64_t *)g.off, (const int32_t *)g.deg, (const int32_t *)g.ids, np);
  INK_TRY(hipStreamSynchronize(c->stream));
  INK_TRY(hipFree(g.ids));
  g.ids = np;
  g.pool_cap = new_cap;
  return hipSuccess;
}

// empty blocks of kNewNodeCap slots for the nodes n0 .. n0 + n_new - 1 at the pool's top
constexpr int kNewNodeCap = 4;
__global__ void k_init_blocks(int64_t *off, int32_t *deg, int32_t *cap, int32_t *ids, int n0, int64_t n_new, int64_t top) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_new) return;
  int64_t o = top + i * kNewNodeCap;
  off[n0 + i] = o; deg[n0 + i] = 0; cap[n0 + i] = kNewNodeCap;
  for (int k = 0; k < kNewNodeCap; k++) ids[o + k] = -1;
}

ink_status graph_add_nodes(ink_ctx *c, int64_t n_new) {
  for (GraphSide *g : {&c->gin, &c->gout}) {
    int64_t need = n_new * kNewNodeCap;
    if (g->pool_top + need > g->pool_cap) {
      hipError_t e = grow_pool(c, *g, need);
      if (e == hipErrorOutOfMemory) { c->err = "out of device memory while growing the edge pool"; return INK_E_OOM; }
      INK_TRYS(e);
    }
    hipLaunchKernelGGL(k_init_blocks, grid1(n_new), dim3(256), 0, c->stream, g->off, g->deg, g->cap, g->ids, c->n, n_new,
                       g->pool_top);
    INK_TRYS(hipGetLastError());
    g->pool_top += need;
  }
  return INK_OK;
}

// A kernel found a malformed entry and dropped the whole batch before any block was touched:
// clear the flag and report.
static ink_status batch_error(ink_ctx *c) {
  int e = c->h_cnt->v[C_ERR];
  INK_TRYS(hipMemsetAsync(&c->d_cnt->v[C_ERR], 0, sizeof(int32_t), c->stream));
  INK_TRYS(hipStreamSynchronize(c->stream));
  if (e & 2) { c->err = "ink_apply_updates: node id out of range"; return INK_E_RANGE; }
  c->err = "ink_apply_updates: op must be 0 (insert) or 1 (delete)";
  return INK_E_ARG;
}

// One direction.  Ops (node, other, op, pos) are in (node, other) order on the device; n_ops is
// known on the host.  all_effective: presence was already established (out side).
struct SideBufs {
  uint32_t *node; int32_t *other; uint8_t *op; int32_t *pos; uint8_t *eff;
  int32_t *uniq, *seg, *chunks, *chunk_pref, *nd_ins, *nd_del, *fill;
};

// n_ops_max bounds the number of ops; the exact count sits on the device in *n_ops_dev.  One host
// round trip per direction: it returns the touched-node count, the totals and the pool space
// that relocations need.
static ink_status apply_side(ink_ctx *c, GraphSide &g, SideBufs &b, int64_t n_ops_max, const int32_t *n_ops_dev,
                             int32_t *new_cnt, int *n_touched_out, int64_t *tot_ins, int64_t *tot_del) {
  hipStream_t s = c->stream;
  Counters *dc = c->d_cnt;
  // scratch slots, the 64-bit slot and the stripes in one fill (the batch's op count sits before them)
  INK_TRYS(hipMemsetAsync(&dc->v[C_TMP0], 0, sizeof(Counters) - C_TMP0 * sizeof(int32_t), s));
  INK_TRYS(segment_heads(c->ws, b.node, n_ops_max, b.uniq, b.seg, &dc->v[C_TMP0], s, n_ops_dev));
  hipLaunchKernelGGL(k_chunk_counts, grid1(n_ops_max), dim3(256), 0, s, (const int32_t *)b.uniq,
                     (const int32_t *)&dc->v[C_TMP0], n_ops_max, (const int32_t *)g.deg, b.chunks);
  INK_TRYS(scan_excl_i32(c->ws, b.chunks, b.chunk_pref, n_ops_max, &dc->v[C_TMP1], s));
  hipLaunchKernelGGL(k_classify, dim3(2048), dim3(256), 0, s, (const int32_t *)b.uniq, (const int32_t *)&dc->v[C_TMP0],
                     (const int32_t *)b.seg, (const int32_t *)b.chunk_pref, (const int32_t *)&dc->v[C_TMP1],
                     (const int64_t *)g.off, (const int32_t *)g.deg, g.ids, (const int32_t *)b.other,
                     (const uint8_t *)b.op, b.pos);
  hipLaunchKernelGGL(k_effect, grid1(n_ops_max * kWave), dim3(256), 0, s, (const int32_t *)b.uniq,
                     (const int32_t *)&dc->v[C_TMP0], (const int32_t *)b.seg, (const uint8_t *)b.op,
                     (const int32_t *)b.pos, b.eff, (const int32_t *)g.deg, (const int32_t *)g.cap, b.nd_ins, b.nd_del,
                     c->slack, dc, (int)ST_REGATHER, (int)ST_EXPOSED, (int)ST_ACHG);
  INK_TRYS(read_counters(c));
  if (c->h_cnt->v[C_ERR]) return batch_error(c);
  int n_touched = c->h_cnt->v[C_TMP0];
  *n_touched_out = n_touched;
  int64_t need = (int64_t)c->h_cnt->sum(ST_REGATHER);
  *tot_ins = (int64_t)c->h_cnt->sum(ST_EXPOSED);
  *tot_del = (int64_t)c->h_cnt->sum(ST_ACHG);
  if (n_touched == 0) return INK_OK;
  if (g.pool_top + need > g.pool_cap) {
    hipError_t e = grow_pool(c, g, need);
    if (e == hipErrorOutOfMemory) { c->err = "out of device memory while growing the edge pool"; return INK_E_OOM; }
    INK_TRYS(e);
  }
  // blocks that move take their space at the pool's top: base by value, the amount handed out so
  // far in a 64-bit slot of the counter block (zero since the fill above)
  unsigned long long *d_used = (unsigned long long *)&dc->v[C_TOP64];
  hipLaunchKernelGGL(k_apply, dim3(n_touched), dim3(256), 0, s, (const int32_t *)b.uniq, (const int32_t *)b.seg,
                     (const int32_t *)b.other, (const uint8_t *)b.eff, (const int32_t *)b.pos,
                     (const int32_t *)b.nd_ins, (const int32_t *)b.nd_del, g.off, g.deg, g.cap, g.ids, d_used,
                     (unsigned long long)g.pool_top, c->slack, b.fill, new_cnt, g.asc);
  INK_TRYS(hipGetLastError());
  g.pool_top += need;      // exact: the apply kernel allocates precisely what k_effect summed
  return INK_OK;
}

// ------------------------------------------------------------ short batches: one workgroup
// A batch of at most kSmallBatch entries goes through the same steps in two single-workgroup
// kernels (one per direction) instead of some thirty launches: everything up to the per-node
// op lists, their segment heads and the chunk plan of the blocks to walk happens in LDS.  Both
// directions are classified before the host looks at the counters, so the batch costs one round
// trip instead of two.  The lists these kernels write are the ones the general path writes.
constexpr int kSmallBatch = 4096;      // largest batch of the single-workgroup form (1024 threads x 4)

struct SmallSide {           // what one direction's kernels hand on (device pointers)
  uint32_t *node; int32_t *other; uint8_t *op; int32_t *pos; uint8_t *eff;
  int32_t *uniq, *seg, *chunk_pref, *nd_ins, *nd_del, *fill;
};

// Ops [0, n_ops) are in (node, other) order with their node ids in S.sk.  Writes the distinct
// nodes, the start of each node's ops (plus the closing offset) and the exclusive prefix of the
// chunk counts of their blocks; *n_uniq_out / *n_chunks_out get the totals.  s_u is LDS scratch
// for THREADS * ITEMS ints, sm for the block scan.
template <int THREADS, int ITEMS>
__device__ __forceinline__ void small_heads_and_chunks(SmallSortLds<THREADS, ITEMS> &S, int *s_u, int *sm, int n_ops, const int32_t *deg,
                                                       int32_t *uniq, int32_t *seg, int32_t *chunk_pref,
                                                       int32_t *n_uniq_out, int32_t *n_chunks_out) {
  const int t0 = threadIdx.x * ITEMS;
  int h[ITEMS], cnt = 0;
#pragma unroll
  for (int k = 0; k < ITEMS; k++) {
    int i = t0 + k;
    h[k] = i < n_ops && (i == 0 || S.sk[i] != S.sk[i - 1]);
    cnt += h[k];
  }
  int n_uniq;
  int ex = block_excl_scan<THREADS>(cnt, sm, &n_uniq);
#pragma unroll
  for (int k = 0; k < ITEMS; k++) {
    int i = t0 + k;
    if (h[k]) { uniq[ex] = (int32_t)S.sk[i]; seg[ex] = i; s_u[ex] = (int)S.sk[i]; ex++; }
  }
  if (threadIdx.x == 0) seg[n_uniq] = n_ops;
  __syncthreads();
  int ch[ITEMS];
  cnt = 0;
#pragma unroll
  for (int k = 0; k < ITEMS; k++) {
    int i = t0 + k;
    ch[k] = i < n_uniq ? (deg[s_u[i]] + kChunk - 1) / kChunk : 0;
    cnt += ch[k];
  }
  int n_chunks;
  ex = block_excl_scan<THREADS>(cnt, sm, &n_chunks);
#pragma unroll
  for (int k = 0; k < ITEMS; k++) {
    int i = t0 + k;
    if (i < n_uniq) chunk_pref[i] = ex;
    ex += ch[k];
  }
  if (threadIdx.x == 0) { *n_uniq_out = n_uniq; *n_chunks_out = n_chunks; }
}

// In side: validate, order by (dst, src, position), keep the final op per edge, build the op
// lists of the touched destinations.
template <int THREADS, int ITEMS>
__global__ __launch_bounds__(THREADS) void k_small_in(const RawUpdate *raw, int n, int n_nodes, int passes,
                                                            SmallSide o, const int32_t *deg, Counters *cnt) {
  __shared__ SmallSortLds<THREADS, ITEMS> S;
  __shared__ int s_src[THREADS * ITEMS], s_dst[THREADS * ITEMS];
  __shared__ uint8_t s_op[THREADS * ITEMS];
  __shared__ int sm[THREADS / kWave + 1];
  // the stripes and the slots that later kernels fill start from zero; the slots before them
  // are written below, the error flag is sticky
  {
    int32_t *z = &cnt->v[C_TMP2];
    const int words = (int)((sizeof(Counters) - C_TMP2 * sizeof(int32_t)) / sizeof(int32_t));
    for (int i = threadIdx.x; i < words; i += THREADS) z[i] = 0;
  }
  int bad = 0;
  for (int i = threadIdx.x; i < n; i += THREADS) {
    RawUpdate a = raw[i];
    bad |= entry_error(a, n_nodes);
    s_src[i] = a.src; s_dst[i] = a.dst; s_op[i] = a.op;
    S.sk[i] = (uint32_t)a.src; S.sv[i] = (uint32_t)i;
  }
  int any_bad = __syncthreads_or(bad);
  if (any_bad) {              // drop the batch: nothing below uses an id as an index
    if (bad) atomicOr(&cnt->v[C_ERR], bad);
    if (threadIdx.x == 0) { cnt->v[C_NOPS] = 0; cnt->v[C_TMP0] = 0; cnt->v[C_TMP1] = 0; o.seg[0] = 0; }
    return;
  }
  small_sort_lds<THREADS, ITEMS>(S, n, passes);
  for (int i = threadIdx.x; i < n; i += THREADS) S.sk[i] = (uint32_t)s_dst[S.sv[i]];
  small_sort_lds<THREADS, ITEMS>(S, n, passes);
  // the last entry of each run of equal (dst, src) is the edge's final op; self loops never count
  const int t0 = threadIdx.x * ITEMS;
  int keep[ITEMS], c = 0;
#pragma unroll
  for (int k = 0; k < ITEMS; k++) {
    int j = t0 + k;
    keep[k] = 0;
    if (j < n) {
      int a = (int)S.sv[j];
      bool last = true;
      if (j + 1 < n) { int b = (int)S.sv[j + 1]; last = s_src[a] != s_src[b] || s_dst[a] != s_dst[b]; }
      keep[k] = last && s_src[a] != s_dst[a];
    }
    c += keep[k];
  }
  int n_ops;
  int ex = block_excl_scan<THREADS>(c, sm, &n_ops);
#pragma unroll
  for (int k = 0; k < ITEMS; k++) {
    if (keep[k]) {
      int a = (int)S.sv[t0 + k];
      o.node[ex] = (uint32_t)s_dst[a]; o.other[ex] = s_src[a]; o.op[ex] = s_op[a]; o.pos[ex] = -1;
      S.sk[ex] = (uint32_t)s_dst[a];       // sk is not read in this phase
      ex++;
    }
  }
  __syncthreads();
  if (threadIdx.x == 0) cnt->v[C_NOPS] = n_ops;
  // the permutation in sv is used up: its space serves as scratch
  small_heads_and_chunks<THREADS, ITEMS>(S, (int *)S.sv, sm, n_ops, deg, o.uniq, o.seg, o.chunk_pref, &cnt->v[C_TMP0], &cnt->v[C_TMP1]);
}

// Out side, after the in side's k_effect: the effective ops become Delta E (inserted and removed
// edges, each in (dst, src) order) and, stably re-ordered by source, the op lists of the touched
// sources.
template <int THREADS, int ITEMS>
__global__ __launch_bounds__(THREADS) void k_small_out(SmallSide in, int passes, int32_t *ins_s, int32_t *ins_d,
                                                             int32_t *del_s, int32_t *del_d, SmallSide o,
                                                             const int32_t *deg, Counters *cnt) {
  __shared__ SmallSortLds<THREADS, ITEMS> S;
  __shared__ int sm[THREADS / kWave + 1];
  const int n_ops = cnt->v[C_NOPS];
  const int t0 = threadIdx.x * ITEMS;
  int e[ITEMS], packed = 0;       // inserts in the low half, deletes in the high half
#pragma unroll
  for (int k = 0; k < ITEMS; k++) {
    int j = t0 + k;
    e[k] = j < n_ops ? in.eff[j] : 0;
    packed += (e[k] == 1) + ((e[k] == 2) << 16);
  }
  int tot;
  int ex = block_excl_scan<THREADS>(packed, sm, &tot);
  int xi = ex & 0xFFFF, xd = ex >> 16;
  const int n_ins = tot & 0xFFFF, n_del = tot >> 16;
#pragma unroll
  for (int k = 0; k < ITEMS; k++) {
    int j = t0 + k;
    if (e[k] == 0) continue;
    int src = in.other[j], dst = (int)in.node[j];
    S.sk[xi + xd] = (uint32_t)src; S.sv[xi + xd] = (uint32_t)j;
    if (e[k] == 1) { ins_s[xi] = src; ins_d[xi] = dst; xi++; }
    else { del_s[xd] = src; del_d[xd] = dst; xd++; }
  }
  const int m = n_ins + n_del;
  small_sort_lds<THREADS, ITEMS>(S, m, passes);
  for (int p = threadIdx.x; p < m; p += THREADS) {
    int j = (int)S.sv[p];
    o.node[p] = S.sk[p]; o.other[p] = (int)in.node[j]; o.op[p] = in.eff[j] == 2 ? 1 : 0; o.pos[p] = -1;
  }
  if (threadIdx.x == 0) { cnt->v[C_TMP2] = n_ins; cnt->v[C_TMP3] = n_del; }
  __syncthreads();            // sv has been read by everyone: its space serves as scratch
  small_heads_and_chunks<THREADS, ITEMS>(S, (int *)S.sv, sm, m, deg, o.uniq, o.seg, o.chunk_pref, &cnt->v[C_OT], &cnt->v[C_OCH]);
}

static ink_status graph_apply_small(ink_ctx *c, int64_t n, int64_t *n_ins_out, int64_t *n_del_out) {
  hipStream_t s = c->stream;
  const size_t per = ((size_t)(n + 64) * 4 + 255) & ~(size_t)255;
  INK_TRYS(c->b_misc.reserve(per * 28));
  INK_TRYS(c->b_del_s.reserve(per)); INK_TRYS(c->b_del_d.reserve(per));
  INK_TRYS(c->b_ins_s.reserve(per)); INK_TRYS(c->b_ins_d.reserve(per));
  INK_TRYS(c->b_touch_in.reserve(per)); INK_TRYS(c->b_uniq.reserve(per));
  Arena ar(c->b_misc);
  SmallSide sd[2];
  for (int k = 0; k < 2; k++) {
    SmallSide &b = sd[k];
    b.node = ar.get<uint32_t>(n); b.other = ar.get<int32_t>(n); b.op = ar.get<uint8_t>(n + 64);
    b.pos = ar.get<int32_t>(n); b.eff = ar.get<uint8_t>(n + 64);
    b.seg = ar.get<int32_t>(n + 2); b.chunk_pref = ar.get<int32_t>(n + 1);
    b.nd_ins = ar.get<int32_t>(n + 1); b.nd_del = ar.get<int32_t>(n + 1); b.fill = ar.get<int32_t>(n + 1);
  }
  sd[0].uniq = c->b_touch_in.as<int32_t>();     // the touched lists are written in place
  sd[1].uniq = c->b_uniq.as<int32_t>();
  Counters *dc = c->d_cnt;
  const int passes = (c->id_bits + kRadixBits - 1) / kRadixBits;
  c->del_src = c->b_del_s.as<int32_t>(); c->del_dst = c->b_del_d.as<int32_t>();
  c->ins_src = c->b_ins_s.as<int32_t>(); c->ins_dst = c->b_ins_d.as<int32_t>();
  const int st[2][3] = {{ST_REGATHER, ST_EXPOSED, ST_ACHG}, {ST_NODEL, ST_NOEFFECT, ST_COVERED}};
  const int slot_n[2] = {C_TMP0, C_OT}, slot_ch[2] = {C_TMP1, C_OCH};
  GraphSide *gs[2] = {&c->gin, &c->gout};
  for (int k = 0; k < 2; k++) {
    SmallSide &b = sd[k];
    GraphSide &g = *gs[k];
#define INK_SMALL_LAUNCH(T, I)                                                                                      \
  do {                                                                                                             \
    if (k == 0)                                                                                                    \
      hipLaunchKernelGGL((k_small_in<T, I>), dim3(1), dim3(T), 0, s, c->b_raw.as<RawUpdate>(), (int)n, c->n,       \
                         passes, b, (const int32_t *)g.deg, dc);                                                   \
    else                                                                                                           \
      hipLaunchKernelGGL((k_small_out<T, I>), dim3(1), dim3(T), 0, s, sd[0], passes, c->ins_src, c->ins_dst,       \
                         c->del_src, c->del_dst, b, (const int32_t *)g.deg, dc);                                   \
  } while (0)
    // fewer waves make every barrier of the sort cheaper
    if (n <= 256) INK_SMALL_LAUNCH(256, 1);
    else if (n <= 1024) INK_SMALL_LAUNCH(256, 4);
    else INK_SMALL_LAUNCH(1024, 4);
#undef INK_SMALL_LAUNCH
    hipLaunchKernelGGL(k_classify, dim3(256), dim3(256), 0, s, (const int32_t *)b.uniq,
                       (const int32_t *)&dc->v[slot_n[k]], (const int32_t *)b.seg, (const int32_t *)b.chunk_pref,
                       (const int32_t *)&dc->v[slot_ch[k]], (const int64_t *)g.off, (const int32_t *)g.deg, g.ids,
                       (const int32_t *)b.other, (const uint8_t *)b.op, b.pos);
    hipLaunchKernelGGL(k_effect, grid1(n * kWave), dim3(256), 0, s, (const int32_t *)b.uniq,
                       (const int32_t *)&dc->v[slot_n[k]], (const int32_t *)b.seg, (const uint8_t *)b.op,
                       (const int32_t *)b.pos, b.eff, (const int32_t *)g.deg, (const int32_t *)g.cap, b.nd_ins, b.nd_del,
                       c->slack, dc, st[k][0], st[k][1], st[k][2]);
  }
  INK_TRYS(read_counters(c));
  if (c->h_cnt->v[C_ERR]) return batch_error(c);
  const int64_t ti = (int64_t)c->h_cnt->sum(st[0][1]), td = (int64_t)c->h_cnt->sum(st[0][2]);
  if ((int64_t)c->h_cnt->sum(st[1][1]) != ti || (int64_t)c->h_cnt->sum(st[1][2]) != td) {
    c->err = "graph store inconsistent: in- and out-adjacency disagree";
    return INK_E_DEVICE;
  }
  c->n_ins = ti; c->n_del = td;
  *n_ins_out = ti; *n_del_out = td;
  c->n_touched_in = c->h_cnt->v[C_TMP0];
  c->n_touched_src = c->h_cnt->v[C_OT];
  if (ti + td == 0) { c->n_touched_src = 0; return INK_OK; }
  const int slot_top[2] = {C_TOP64, C_TOP64B};
  for (int k = 0; k < 2; k++) {
    SmallSide &b = sd[k];
    GraphSide &g = *gs[k];
    const int64_t need = (int64_t)c->h_cnt->sum(st[k][0]);
    const int n_touched = c->h_cnt->v[slot_n[k]];
    if (g.pool_top + need > g.pool_cap) {
      hipError_t e = grow_pool(c, g, need);
      if (e == hipErrorOutOfMemory) { c->err = "out of device memory while growing the edge pool"; return INK_E_OOM; }
      INK_TRYS(e);
    }
    unsigned long long *d_used = (unsigned long long *)&dc->v[slot_top[k]];     // zero since k_small_in
    if (n_touched > 0)
      hipLaunchKernelGGL(k_apply, dim3(n_touched), dim3(256), 0, s, (const int32_t *)b.uniq, (const int32_t *)b.seg,
                         (const int32_t *)b.other, (const uint8_t *)b.eff, (const int32_t *)b.pos,
                         (const int32_t *)b.nd_ins, (const int32_t *)b.nd_del, g.off, g.deg, g.cap, g.ids, d_used,
                         (unsigned long long)g.pool_top, c->slack, b.fill, k == 1 ? c->new_out : nullptr, g.asc);
    INK_TRYS(hipGetLastError());
    g.pool_top += need;
  }
  return INK_OK;
}

ink_status graph_apply_batch(ink_ctx *c, int64_t n, int64_t *n_ins_out, int64_t *n_del_out) {
  hipStream_t s = c->stream;
  *n_ins_out = *n_del_out = 0;
  c->n_ins = c->n_del = 0;
  c->n_touched_in = 0;
  if (n == 0) return INK_OK;
  if (n <= c->small_batch && n <= kSmallBatch) return graph_apply_small(c, n, n_ins_out, n_del_out);
  const RawUpdate *raw = c->b_raw.as<RawUpdate>();
  size_t per = ((size_t)(n + 64) * 4 + 255) & ~(size_t)255;
  INK_TRYS(c->b_misc.reserve(per * 28));
  INK_TRYS(c->b_del_s.reserve(per)); INK_TRYS(c->b_del_d.reserve(per));
  INK_TRYS(c->b_ins_s.reserve(per)); INK_TRYS(c->b_ins_d.reserve(per));
  Arena ar(c->b_misc);
  uint32_t *k0 = ar.get<uint32_t>(n), *v0 = ar.get<uint32_t>(n), *k1 = ar.get<uint32_t>(n);
  uint32_t *srcv = ar.get<uint32_t>(n), *dstv = ar.get<uint32_t>(n);
  uint8_t *flag = ar.get<uint8_t>(n + 64);
  int32_t *idx = ar.get<int32_t>(n), *idx2 = ar.get<int32_t>(n);
  SideBufs b;
  b.node = ar.get<uint32_t>(n); b.other = ar.get<int32_t>(n); b.op = ar.get<uint8_t>(n + 64);
  b.pos = ar.get<int32_t>(n); b.eff = ar.get<uint8_t>(n + 64);
  b.uniq = ar.get<int32_t>(n + 1); b.seg = ar.get<int32_t>(n + 2); b.chunks = ar.get<int32_t>(n + 1);
  b.chunk_pref = ar.get<int32_t>(n + 1); b.nd_ins = ar.get<int32_t>(n + 1); b.nd_del = ar.get<int32_t>(n + 1);
  b.fill = ar.get<int32_t>(n + 1);
  Counters *dc = c->d_cnt;
  int32_t *n_ops_d = &dc->v[C_NOPS];

  // (dst, src, position) order through two stable sorts
  hipLaunchKernelGGL(k_unpack, grid1(n), dim3(256), 0, s, raw, n, c->n, srcv, dstv, v0, &dc->v[C_ERR]);
  INK_TRYS(hipMemcpyAsync(k0, srcv, (size_t)n * 4, hipMemcpyDeviceToDevice, s));
  INK_TRYS(radix_sort_pairs(c->ws, k0, v0, n, c->id_bits, s));
  hipLaunchKernelGGL(k_gather_u32, grid1(n), dim3(256), 0, s, (const uint32_t *)dstv, (const uint32_t *)v0, n, k1);
  INK_TRYS(radix_sort_pairs(c->ws, k1, v0, n, c->id_bits, s));
  // final op per distinct edge; their number stays on the device (n bounds it)
  hipLaunchKernelGGL(k_mark_last, grid1(n), dim3(256), 0, s, raw, (const uint32_t *)v0, n, flag,
                     (const int32_t *)&dc->v[C_ERR]);
  INK_TRYS(compact_flags_u8(c->ws, flag, n, idx, n_ops_d, s));
  hipLaunchKernelGGL(k_take_ops, grid1(n), dim3(256), 0, s, raw, (const uint32_t *)v0, (const int32_t *)idx,
                     (const int32_t *)n_ops_d, b.node, b.other, b.op, b.pos);

  int n_touched = 0;
  int64_t ti = 0, td = 0;
  ink_status st = apply_side(c, c->gin, b, n, n_ops_d, nullptr, &n_touched, &ti, &td);
  if (st != INK_OK) return st;
  c->n_ins = ti; c->n_del = td;
  *n_ins_out = ti; *n_del_out = td;
  c->n_touched_in = n_touched;
  if (ti + td == 0) return INK_OK;
  INK_TRYS(c->b_touch_in.reserve((size_t)(n_touched + 1) * 4));
  INK_TRYS(hipMemcpyAsync(c->b_touch_in.p, b.uniq, (size_t)n_touched * 4, hipMemcpyDeviceToDevice, s));

  // Delta E lists, (dst, src) order
  hipLaunchKernelGGL(k_flag_eq, grid1(n), dim3(256), 0, s, (const uint8_t *)b.eff, (const int32_t *)n_ops_d, n,
                     (uint8_t)1, flag);
  INK_TRYS(compact_flags_u8(c->ws, flag, n, idx, &dc->v[C_TMP2], s));
  hipLaunchKernelGGL(k_flag_eq, grid1(n), dim3(256), 0, s, (const uint8_t *)b.eff, (const int32_t *)n_ops_d, n,
                     (uint8_t)2, flag);
  INK_TRYS(compact_flags_u8(c->ws, flag, n, idx2, &dc->v[C_TMP3], s));
  c->del_src = c->b_del_s.as<int32_t>(); c->del_dst = c->b_del_d.as<int32_t>();
  c->ins_src = c->b_ins_s.as<int32_t>(); c->ins_dst = c->b_ins_d.as<int32_t>();
  hipLaunchKernelGGL(k_split_ops, grid1(n), dim3(256), 0, s, (const uint32_t *)b.node, (const int32_t *)b.other,
                     (const uint8_t *)b.eff, (const int32_t *)n_ops_d, (const int32_t *)idx, (const int32_t *)idx2,
                     c->ins_src, c->ins_dst, c->del_src, c->del_dst, (const int32_t *)&dc->v[C_TMP2],
                     (const int32_t *)&dc->v[C_TMP3]);

  // out side: the effective ops in (src, dst) order
  int64_t m = ti + td;
  hipLaunchKernelGGL(k_out_dst_key, grid1(m), dim3(256), 0, s, (const int32_t *)c->del_dst, (const int32_t *)c->ins_dst,
                     (int)td, (int)ti, k0, v0);
  INK_TRYS(radix_sort_pairs(c->ws, k0, v0, m, c->id_bits, s));
  // key <- source of the permuted entries
  hipLaunchKernelGGL(k_out_ops, grid1(m), dim3(256), 0, s, (const int32_t *)c->del_src, (const int32_t *)c->del_dst,
                     (const int32_t *)c->ins_src, (const int32_t *)c->ins_dst, (int)td, (int)ti, srcv, dstv);
  hipLaunchKernelGGL(k_gather_u32, grid1(m), dim3(256), 0, s, (const uint32_t *)srcv, (const uint32_t *)v0, m, k1);
  INK_TRYS(radix_sort_pairs(c->ws, k1, v0, m, c->id_bits, s));
  hipLaunchKernelGGL(k_out_take, grid1(m), dim3(256), 0, s, (const uint32_t *)v0, (const int32_t *)c->del_src,
                     (const int32_t *)c->del_dst, (const int32_t *)c->ins_src, (const int32_t *)c->ins_dst, (int)td,
                     (int)ti, b.node, b.other, b.op, b.pos);
  int64_t oi = 0, od = 0;
  st = apply_side(c, c->gout, b, m, nullptr, c->new_out, &n_touched, &oi, &od);
  if (st != INK_OK) return st;
  if (oi != ti || od != td) {
    c->err = "graph store inconsistent: in- and out-adjacency disagree";
    return INK_E_DEVICE;
  }
  // remember the touched sources so that the per-batch marks can be cleared
  INK_TRYS(c->b_uniq.reserve((size_t)(n_touched + 1) * 4));
  INK_TRYS(hipMemcpyAsync(c->b_uniq.p, b.uniq, (size_t)n_touched * 4, hipMemcpyDeviceToDevice, s));
  c->n_touched_src = n_touched;
  return INK_OK;
}

hipError_t graph_end_batch(ink_ctx *c) {
  if (c->n_touched_src > 0)
    hipLaunchKernelGGL(k_zero_at, grid1(c->n_touched_src), dim3(256), 0, c->stream, (const int32_t *)c->b_uniq.p,
                       (int)c->n_touched_src, c->new_out);
  c->n_touched_src = 0;
  return hipGetLastError();
}

}  // namespace ink
