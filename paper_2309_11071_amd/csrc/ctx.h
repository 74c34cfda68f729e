// Internal context of the library: device-resident graph store, cached per-layer tables and
// the work buffers of the per-layer event pipeline.  Not part of the C ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string>
#include <vector>

#include "../../include/ink.h"
#include "prim.h"

namespace ink {

#ifndef INK_BIG_DEG
#define INK_BIG_DEG 256
#endif
// neighbour rows in flight per lane group while gathering, by aggregator family and lanes per row
#ifndef INK_U_SEL16
#define INK_U_SEL16 4
#endif
#ifndef INK_U_SEL32
#define INK_U_SEL32 4
#endif
#ifndef INK_U_SEL64
#define INK_U_SEL64 4
#endif
#ifndef INK_U_SUM16
#define INK_U_SUM16 8       // narrow rows are cheap in registers: 8 loads in flight measured 3.5 % faster than 4
#endif
#ifndef INK_U_SUM32
#define INK_U_SUM32 4
#endif
#ifndef INK_U_SUM64
#define INK_U_SUM64 4
#endif
#ifndef INK_BIG_CHUNK
#define INK_BIG_CHUNK 1024
#endif
constexpr int kBigChunk = INK_BIG_CHUNK;  // neighbours per chunk of such a row
#ifndef INK_BIG_DEG_SUM
#define INK_BIG_DEG_SUM 1024
#endif
// rows with more in-neighbours are re-gathered cooperatively (bigrows.h): kBigDeg for max / min,
// whose per-neighbour work is heavier, kBigDegSum for the sum-type aggregators (both measured)
constexpr int kBigDeg = INK_BIG_DEG;
constexpr int kBigDegSum = INK_BIG_DEG_SUM;
static_assert(kBigDeg <= kBigDegSum, "buffer bounds of the long-row path use the smaller threshold");
constexpr uint32_t kEvKindShift = 30;
constexpr uint32_t kEvIdMask = (1u << kEvKindShift) - 1;
enum : uint32_t { EV_DEL = 0, EV_ADD = 1, EV_CHG = 2 };   // removed edge / inserted edge / changed source

// One direction of the graph store: per-node edge blocks with slack inside one id pool.
struct GraphSide {
  int64_t *off = nullptr;    // [n] first slot of the node's block
  int32_t *deg = nullptr;    // [n] used slots
  int32_t *cap = nullptr;    // [n] block capacity
  uint8_t *asc = nullptr;    // [n] 1 while the block's ids are ascending (true until the node's first applied op)
  int32_t *ids = nullptr;    // pool
  int64_t pool_cap = 0;      // slots in the pool
  int64_t pool_top = 0;      // first free slot (host mirror, exact)
};

struct Table {               // N x d float (or int) table with row stride ld (multiple of 4)
  void *p = nullptr;
  int d = 0, ld = 0;
  float *f() const { return (float *)p; }
  int32_t *i() const { return (int32_t *)p; }
};

struct DevLayer {
  int in_dim = 0, out_dim = 0, hidden = 0, act = 0;
  // first (or only) linear map: rows = K (padded to a multiple of 32), cols = ldw (multiple of 32)
  float *W1 = nullptr; int K1 = 0, K1p = 0, N1 = 0, N1p = 0; float *b1 = nullptr;
  float *W2 = nullptr; int K2 = 0, K2p = 0, N2 = 0, N2p = 0; float *b2 = nullptr;   // GIN second linear
};

constexpr int kStripes = 64;
enum { ST_EXPOSED = 0, ST_REGATHER, ST_ACHG, ST_NODEL, ST_NOEFFECT, ST_COVERED, ST_REGATHER_LONG, ST_PAD7, ST_N };
struct Counters {            // device-written, host-read through pinned memory
  int32_t v[32];
  // statistics that many waves bump: striped by workgroup so that no single address is contended
  unsigned long long stripe[kStripes][ST_N];
  unsigned long long sum(int which) const {
    unsigned long long t = 0;
    for (int i = 0; i < kStripes; i++) t += stripe[i][which];
    return t;
  }
};
// what the host sees of them: the slots and the stripe totals (192 bytes through pinned memory)
struct HostCounters {
  int32_t v[32];
  unsigned long long total[ST_N];
  unsigned long long sum(int which) const { return total[which]; }
};
// slots of Counters::v: event count of the next layer, unique targets, long rows listed, rows to
// transform, rows changed, chunks of long rows, distinct ops of a batch, scratch of the graph stage,
// (C_NEXP: exposed rows of moderate length listed for the recompute, next to the long ones in C_NBIG)
// touched nodes and block chunks of the out side (single-workgroup graph stage), and two 64-bit
// slots (pool tops handed to the apply kernels).  Slot 0 flags a malformed update batch.
enum { C_ERR = 0, C_NEV = 1, C_NT, C_NBIG, C_NEXP, C_NC, C_NEXT, C_NCHUNK, C_NOPS, C_TMP0, C_TMP1, C_TMP2, C_TMP3,
       C_OT, C_OCH, C_TOP64 = 16, C_TOP64B = 18 };

}  // namespace ink

struct ink_ctx {
  int n = 0;
  int64_t n_edges = 0, n_edges_now = 0;
  int64_t pool_reserve = 0;
  int64_t n_cap = 0;          // node capacity: every per-node array has this many entries (>= n)
  int64_t big_hint[INK_MAX_LAYERS + 1] = {0};   // chunks of long rows seen by the last update at each layer
  double dense_frac = 0.75;          // events / edges above which a layer re-aggregates every node
  int id_bits = 1;
  int kind = 0, agg = 0, n_layers = 0, mem = 0, profile = 0;
  float eps = 0.f, slack = 0.25f;
  bool batch_dev = false;
  bool affected_mode = false;        // current call is the affected-area recompute baseline
  bool is_select = true, is_min = false, inferred = false, own_stream = false;
  bool broken = false;               // an updating call failed on the device side: state may be half-written
  hipStream_t stream = nullptr;
  int device = 0;                    // HIP device the context lives on
  void *scratch = nullptr;           // that device's copy of the static work array of ink_full_infer_noalloc
  std::string err;

  ink::GraphSide gin, gout;
  int32_t *new_out = nullptr;        // [n] out-edges appended by the current batch (tail of the block)
  std::vector<ink::DevLayer> layers;
  // tables: H[0..k]; A[1..k] aggregated (sum-type: plain sums); ARG[1..k]
  std::vector<ink::Table> H, A, ARG, UB, ARG2;   // UB / ARG2: max/min only, bound on the runner-up value and its holder when known
  // GCN only: XW[l] = unscaled transformed messages h_{l-1} W_l, H-like scaled copies live in Msc[l]
  std::vector<ink::Table> XW, Msc;
  float *cnorm = nullptr;            // GCN: (indeg + 1)^(-1/2) per node
  std::vector<ink::Table> USER;      // per layer: the term of user-defined events (allocated by the first event of the layer)
  ink::DevBuf u_ev, u_rows, u_key, u_val, u_uniq, u_seg, u_flag, u_idx, u_list;   // work buffers of ink_apply_user_events

  ink::PrimWorkspace ws;
  ink::Counters *d_cnt = nullptr;    // device counters
  ink::HostCounters *h_cnt = nullptr;   // pinned host mirror, written by the publish kernel
  uint32_t *h_seq = nullptr;         // (same allocation) sequence number of the last published copy
  uint32_t pub_seq = 0;
  int64_t small_batch = 4096;        // batches up to this size take the single-workgroup graph stage
  uint64_t *bm_a = nullptr;          // node bitmaps (n bits each)

  // batch buffers (grown on demand)
  int64_t n_touched_src = 0;         // sources whose out-block got new ids in the current batch
  ink::DevBuf b_raw, b_uniq, b_misc;
  int32_t *del_src = nullptr, *del_dst = nullptr, *ins_src = nullptr, *ins_dst = nullptr;  // Delta E lists
  ink::DevBuf b_del_s, b_del_d, b_ins_s, b_ins_d;
  int64_t n_del = 0, n_ins = 0;

  // per-layer pipeline buffers
  ink::DevBuf f_list[2];             // F_l (ascending node ids), ping-pong between layers
  ink::DevBuf f_old[2];              // old message rows of F_l (sum-type aggregators)
  ink::DevBuf f_pref;                // prefix of out-degrees over F_l
  ink::DevBuf f_delta;               // new - old message rows of F_l (sum-type aggregators)
  ink::DevBuf ev_key, ev_val;        // events
  ink::DevBuf t_list, t_seg;         // unique targets, segment offsets
  ink::DevBuf c_list, c_flag, c_idx; // rows to transform, per-row changed flag, compacted positions
  ink::DevBuf c_old;                 // previous table rows of the transformed rows (sum-type)
  ink::DevBuf b_touch_in;            // destinations touched by the current batch
  int64_t n_touched_in = 0;
  ink::DevBuf exp_list;              // exposed rows of moderate length, listed by the event kernel
  ink::DevBuf big_list, big_part_v, big_part_i, big_part_s, big_part_j, big_pref;   // cooperative re-gather of long rows
  ink::DevBuf stage0, stage1;        // transform staging
  ink::DevBuf res_ids, res_emb;      // result of the last batch

  ink_stats stats;
  struct Pending { int cls, layer, kern; hipEvent_t a, b; };
  std::vector<hipEvent_t> ev_free;
  std::vector<Pending> ev_pending;
};

namespace ink {

// Times what is launched during its life with a pair of HIP events on the context's stream (only
// while profiling is on): into the class total `cls` (>= 0) and / or into kernel slot `kern` of
// layer `layer` (1-based).  Launch counts per class are always kept.
struct Prof {
  ink_ctx *c; int cls, layer, kern; hipEvent_t a = nullptr, b = nullptr;
  Prof(ink_ctx *c_, int cls_, int layer_ = 0, int kern_ = -1) : c(c_), cls(cls_), layer(layer_), kern(kern_) {
    if (cls >= 0) c->stats.launches[cls]++;
    if (!c->profile) return;
    while (c->ev_free.size() < 2) { hipEvent_t e; if (hipEventCreate(&e) != hipSuccess) return; c->ev_free.push_back(e); }
    a = c->ev_free.back(); c->ev_free.pop_back();
    b = c->ev_free.back(); c->ev_free.pop_back();
    (void)hipEventRecord(a, c->stream);
  }
  ~Prof() {
    if (!a) return;
    (void)hipEventRecord(b, c->stream);
    c->ev_pending.push_back({cls, layer, kern, a, b});
  }
};
struct KernelTimer : Prof {
  KernelTimer(ink_ctx *c_, int layer_, int kern_) : Prof(c_, -1, layer_, kern_) {}
};

// ---- graph store (graph.hip)
hipError_t graph_build(ink_ctx *c, const int64_t *rowptr_h, const int32_t *col_h);
// applies a validated batch already on the device in c->b_raw; fills Delta E lists and counts
ink_status graph_apply_batch(ink_ctx *c, int64_t n, int64_t *n_ins, int64_t *n_del);
ink_status graph_add_nodes(ink_ctx *c, int64_t n_new);   // empty edge blocks for nodes n .. n + n_new - 1 (before n grows)
hipError_t read_counters(ink_ctx *c);        // device counters -> c->h_cnt, waits for them
hipError_t graph_end_batch(ink_ctx *c);     // clears per-batch marks (new_out)
hipError_t graph_export(ink_ctx *c, int64_t *rowptr_h, int32_t *col_h);

// ---- aggregation (agg.hip)
struct AggArgs {
  int n;
  const int64_t *in_off; const int32_t *in_deg; const int32_t *in_ids;
  const float *M; int ldm;          // message table
  float *A; int32_t *ARG; int ld;   // aggregated table and argument table (row stride ld)
  float *UB;                        // max/min: bound on the best value among the non-holders (same layout)
  const uint8_t *in_asc;            // per node: in-list ascending by id (lets ties go to the first seen)
  int32_t *ARG2;                    // max/min: the non-holder that has exactly that value (lowest id), or -1 if not known
  int d;                            // columns handled by this launch (<= 256; wider rows go block by block)
  int wd;                           // d rounded up to 4
  bool is_min;
  int big_deg;                      // rows with more in-neighbours go to the chunked cooperative path
  int64_t big_grid;                 // workgroups to launch for the chunk kernel (it strides if there are more chunks)
  int layer;                        // 1-based layer the launch belongs to (per-kernel timing)
  int count_cond;                   // tally the per-target condition counters (only the first 256-column block of a wide row does)
};
// full re-aggregation of every node (targets == nullptr) or of a target list; flags rows whose
// alpha changed in bitmap `chg` (may be null); big rows go through the cooperative path
hipError_t agg_select_full(ink_ctx *c, const AggArgs &a, const int32_t *targets, int64_t n_targets,
                           uint64_t *chg);
// n_targets may be an upper bound of the device-side count *n_targets_dev
hipError_t agg_select_events(ink_ctx *c, const AggArgs &a, const int32_t *targets, const int32_t *seg,
                             int64_t n_targets, const int32_t *n_targets_dev, const uint32_t *ev_val, uint64_t *chg);
// sum-type aggregators (agg_sum.hip): A holds the plain sum of message rows.  F (ascending ids)
// and f_old (their previous message rows, row stride ld_old) describe the changed sources.
hipError_t agg_sum_full(ink_ctx *c, const AggArgs &a, const int32_t *targets, int64_t n_targets, uint64_t *chg);
hipError_t agg_sum_events(ink_ctx *c, const AggArgs &a, const int32_t *targets, const int32_t *seg,
                          int64_t n_targets, const int32_t *n_targets_dev, const uint32_t *ev_val, const int32_t *F,
                          int nF, const float *f_old, const float *f_delta, int ld_old, uint64_t *chg);
// f_delta[i] = M[F[i]] - f_old[i] (row stride ld_old): what a kept edge of changed source i adds
hipError_t agg_sum_delta_rows(ink_ctx *c, const AggArgs &a, const int32_t *F, int nF, const float *f_old,
                              float *f_delta, int ld_old);

// ---- dense transform (xform.hip)
struct XformArgs {
  int mode;                 // 0 SAGE concat [A | Hprev], 1 GIN (1+eps) Hprev + A, 2 dense rows,
                            // 3 GCN: x = act(c_v (A + Hp) + in_bias), with A = neighbour sums, Hp = own scaled message
  const int32_t *rows;      // row ids (null: identity)
  int64_t n_rows;           // rows to transform; an upper bound when n_rows_dev is set
  const int32_t *n_rows_dev;   // optional device-side row count (<= n_rows)
  const float *A; int lda;  // aggregated table
  const float *Hp; int ldh; // previous-layer table (or dense input for mode 2)
  int d_in;
  float eps;
  const float *W; int Kp; int Np; const float *bias; int n_out; int relu;
  // output: either staging (dense [n_rows][ld_out]) or table rows with compare-and-emit
  float *out; int ld_out; int to_table;
  uint8_t *row_changed;     // [n_rows] set to 1 if the table row changed bitwise (to_table)
  float *old_rows; int ld_old;   // optional copy of the previous table rows ([n_rows][ld_old])
  const int32_t *out_rows;  // table row ids for to_table when the input is dense (mode 2); null: identity
  const int32_t *mean_deg;  // modes 0/1 with mean aggregation: A is divided by max(deg, 1)
  const float *cnorm;       // mode 3: per-node c_v
  const float *in_bias; int in_relu;   // mode 3
  const float *in_user; int ld_in_user;   // mode 3: per-node term added after in_bias, before the activation; null: none
  float *h_store; int ld_hs;           // mode 3: where x (= h_l) is written, one row per node
  const float *out_scale;   // per-node factor applied to the output row (after bias), null: none
  const float *user; int ld_user;      // per-node term added after the bias, before the activation (to_table only), null: none
};
hipError_t xform_run(ink_ctx *c, const XformArgs &x);
// position of W[k][col] in the padded device copy: k-chunks of 32, inside a chunk one row of 32 per
// column holding first the 16 even then the 16 odd k (the order the MFMA steps consume them)
inline size_t xform_weight_index(int k, int col, int Np) {
  return (size_t)(k / 32) * 32 * Np + (size_t)col * 32 + (size_t)(k & 1) * 16 + (size_t)((k % 32) >> 1);
}

}  // namespace ink
