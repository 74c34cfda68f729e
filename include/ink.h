/*
 * ink.h -- C ABI of the MI355X (gfx950) incremental GNN-inference library.
 *
 * The library keeps, on one GPU, the cached state of a k-layer message-passing GNN
 * (per layer: the messages m_l, the aggregated neighbourhoods alpha_l and, for min/max,
 * the per-dimension argmax/argmin neighbour ids) and updates it after a batch of edge
 * insertions and deletions by the event-driven incremental method of the paper
 * (Sec. 2.3 workflow; Sec. 2.4 events, grouping and propagation; Sec. 2.5 incremental
 * update, reset conditions and recompute).  The result equals plain inference on the
 * post-update snapshot (Abstract; Sec. 1, "No Accuracy Loss").
 *
 * Conventions for every entry point
 *   - Plain C types only.  Pointers are HOST pointers unless `ink_options.mem` says
 *     INK_MEM_DEVICE, in which case caller arrays (graph, features, weights, update
 *     batches) are device pointers on the current HIP device (`ink_options.batch_mem`
 *     can place only the update batches on the device).
 *   - The caller keeps ownership of everything it passes in; the library copies what it
 *     needs.  Buffers returned by the library are library-owned DEVICE memory, valid until
 *     the next ink_apply_updates / ink_full_infer / ink_destroy on the same context.
 *   - Every call returns an ink_status.  On an argument / range / state error nothing in
 *     the context has been modified.  INK_E_OOM or INK_E_DEVICE from a call that updates the
 *     context (ink_apply_updates, ink_apply_updates_affected, ink_update_features,
 *     ink_add_nodes) may leave the graph store or the cache half-written: the context is then
 *     unusable, every later call on it returns INK_E_STATE, and it must be destroyed.
 *     ink_last_error() gives a readable message.
 *   - One context = one HIP stream; calls on one context must not overlap.  All calls are
 *     synchronous: on return the work is complete.
 *   - Node ids are int32 in [0, n_nodes); the graph is a simple directed graph without self
 *     loops.  Edge batches never change n_nodes (the paper's update stream holds edges only,
 *     Sec. 2.1); it grows only through ink_add_nodes, up to ink_options.node_capacity.
 *     Edge (u -> v) makes u an in-neighbour of v: v aggregates m_u.
 *   - At most 2^31 - 2^30 - 1 edges (event offsets are 32-bit); a batch that could take the graph
 *     past that is refused.
 *   - All matrices are row-major float32.  Layer outputs are at most INK_MAX_OUT_DIM wide, layer
 *     inputs (the feature width in particular) at most INK_MAX_IN_DIM.
 */
#ifndef INK_H
#define INK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define INK_MAX_OUT_DIM 256
#define INK_MAX_IN_DIM 16384
#define INK_MAX_LAYERS 8

typedef struct ink_ctx ink_ctx; /* opaque; owns all device state */

typedef enum {
  INK_OK = 0,
  INK_E_ARG = 1,    /* null pointer, bad dimension, malformed CSR, unsupported combination */
  INK_E_STATE = 2,  /* ink_apply_updates / ink_get_layer before ink_full_infer */
  INK_E_OOM = 3,    /* device or host allocation failed; from an updating call: destroy the context */
  INK_E_DEVICE = 4, /* a HIP call failed; the context must be destroyed */
  INK_E_RANGE = 5   /* node id or layer index out of range */
} ink_status;

/* Model families of Sec. 3 (eqs. (1)-(6)). */
typedef enum { INK_MODEL_SAGE = 0, INK_MODEL_GCN = 1, INK_MODEL_GIN = 2 } ink_model_kind;

/* Aggregation function A of Sec. 2.1.  MAX / MIN are the paper's monotonic selections
 * (Sec. 2.2 item 1).  SUM / MEAN / GCN_SYM use the delta-accumulative update the paper names
 * as its extension (Sec. 7).  GCN_SYM = symmetric degree normalisation with self loop:
 * a_v = sum_{u in N(v)+{v}} h_u / sqrt(dhat_u dhat_v), dhat_x = indeg(x) + 1. */
typedef enum {
  INK_AGG_MAX = 0, INK_AGG_MIN = 1, INK_AGG_SUM = 2, INK_AGG_MEAN = 3, INK_AGG_GCN_SYM = 4
} ink_agg;

typedef enum { INK_ACT_NONE = 0, INK_ACT_RELU = 1 } ink_act;
typedef enum { INK_MEM_HOST = 0, INK_MEM_DEVICE = 1 } ink_mem;

/* In-neighbour CSR of the initial snapshot: row v lists the sources u of edges u -> v,
 * strictly ascending within a row (no duplicates), no self loops. */
typedef struct {
  int32_t n_nodes;
  int64_t n_edges;
  const int64_t *rowptr; /* [n_nodes + 1], rowptr[0] = 0, rowptr[n_nodes] = n_edges */
  const int32_t *col;    /* [n_edges] */
} ink_csr;

/* One GNN layer.  Weights are row-major [in][out]; a NULL pointer means "absent".
 *   SAGE: h' = act(W_neigh^T a + W_self^T h + bias)                          (eq. (4))
 *   GCN : h' = act(W_neigh^T a + bias)                                       (eq. (2))
 *   GIN : h' = act(W_mlp2^T relu(W_neigh^T ((1+eps) h + a) + bias) + bias_mlp2)  (eq. (6));
 *         W_neigh is [in_dim][mlp_hidden], W_mlp2 is [mlp_hidden][out_dim]. */
typedef struct {
  int32_t in_dim, out_dim, mlp_hidden;
  const float *W_neigh, *W_self, *bias;
  const float *W_mlp2, *bias_mlp2;
  int32_t act; /* ink_act applied at the end of the layer (Sec. 2.1) */
} ink_layer;

typedef struct {
  int32_t kind;    /* ink_model_kind */
  int32_t agg;     /* ink_agg; SAGE: MAX|MIN|SUM|MEAN, GIN: SUM|MAX|MIN|MEAN, GCN: GCN_SYM */
  float gin_eps;
  int32_t n_layers; /* 1 .. INK_MAX_LAYERS */
  const ink_layer *layers;
} ink_model;

typedef struct {
  int32_t mem;        /* ink_mem: where the caller's arrays live, for every call on the context */
  void *hip_stream;   /* hipStream_t to run on, or NULL for a stream the library creates */
  float slack_factor; /* extra capacity per edge block, as a fraction of its degree (default 0.25) */
  int32_t max_batch;  /* hint: largest update batch expected (sizes buffers up front); 0 = default */
  int32_t profile;    /* non-zero: time each kernel class with HIP events (see ink_stats) */
  float dense_threshold; /* a layer whose event count exceeds this fraction of the edge count
                            re-aggregates every node instead of grouping events (the dense
                            fallback Sec. 5.1 argues for when updates are not sparse);
                            0 = default 0.75, negative = never */
  int32_t batch_mem;     /* ink_mem of the `updates` array of ink_apply_updates when it differs from
                            `mem` (e.g. host-built graph, device-resident update stream): the
                            effective location is device if either field says INK_MEM_DEVICE */
  int32_t small_batch_limit; /* update batches of at most this many entries take the single-workgroup
                                form of the graph-store update (same result, fewer launches, one
                                host read-back instead of two); 0 = default 4096, which is also the
                                largest value; negative = never */
  int64_t pool_reserve;  /* free id slots kept behind the edge blocks of each direction for blocks
                            that outgrow their slack; when they run out the pool is re-allocated
                            at twice the size.  0 = default max(25 % of the pool, 2^20) */
  int64_t node_capacity; /* largest node count the context can grow to with ink_add_nodes; every
                            per-node table is allocated for it.  0 (or less than the graph's
                            node count) = the graph's node count, i.e. no growth */
} ink_options;

/* One streaming update (Sec. 2.1: Delta E holds inserted and removed edges). */
typedef struct {
  uint8_t op; /* 0 = insert, 1 = delete */
  uint8_t pad_[3];
  int32_t src, dst;
} ink_edge_update;

/* Result of one update batch (library-owned device buffers, see top comment). */
typedef struct {
  int64_t n_changed;          /* nodes whose final embedding h_k changed bitwise            */
  const int32_t *changed_ids; /* DEVICE [n_changed], ascending                                */
  const float *embeddings;    /* DEVICE [n_changed][out_dim of last layer], new h_k rows      */
  int64_t n_applied_ins, n_applied_del; /* edges whose presence differs between the snapshots */
  int64_t n_noop; /* list entries without net effect: duplicate insert, delete of an absent
                     edge, self loop, or an insert/delete pair that cancels within the batch */
} ink_update_result;

/* Kernels of a layer that are timed one by one (ink_layer_stats.ms_kernel). */
enum { INK_K_AGG_EVENTS = 0, /* incremental aggregation over the grouped events (Sec. 2.5)          */
       INK_K_AGG_EXPOSED,    /* recompute of the exposed rows of moderate length, one wave per row  */
       INK_K_AGG_LONG,       /* recompute of long rows: plan, chunk partials, combine               */
       INK_K_AGG_FULL,       /* recompute of every row (full inference, dense fallback), short rows */
       INK_K_SORT,           /* grouping: radix sort of the events by target                        */
       INK_K_XFORM,          /* dense combination (all linear maps of the layer)                    */
       INK_K_NKERNEL = 8 };

/* Per-layer counters and timings of the LAST ink_apply_updates (or ink_full_infer). */
typedef struct {
  int64_t n_sources;     /* |F_l|: nodes whose message m_l changed                         */
  int64_t n_events;      /* event records created (changed edges + propagated)   Sec. 2.4.2 */
  int64_t n_targets;     /* unique target nodes after grouping                    Sec. 2.4.1 */
  int64_t n_exposed;     /* targets recomputed from their whole neighbourhood    Sec. 2.5.1 */
  int64_t n_regather_nb; /* neighbour rows fetched by those recomputes                       */
  int64_t n_alpha_changed; /* targets whose alpha changed (not resilient)         Sec. 2.5.2 */
  int64_t n_transformed; /* rows through the dense combination                              */
  int64_t n_changed;     /* rows whose layer output changed: next layer's sources           */
  /* MAX / MIN only: how the targets that were NOT recomputed split over the conditions of
   * Sec. 2.5.1 (the distribution of Sec. 5.2); together with n_exposed they sum to n_targets.
   * Aggregated rows wider than 256 columns are processed in 256-column blocks: the condition
   * counters, n_exposed and n_alpha_changed then describe the first block of each target,
   * n_regather_nb counts the neighbour rows of every block. */
  int64_t n_no_deletion;        /* only additions arrived                                    */
  int64_t n_deletion_no_effect; /* something was cancelled but no dimension needed a reset   */
  int64_t n_covered;            /* resets, all covered by added messages                     */
  int32_t dense;         /* 1 if the layer fell back to re-aggregating every node           */
  int32_t pad_;
  int64_t n_regather_nb_long; /* the part of n_regather_nb fetched by the chunked long-row kernels */
  float ms_kernel[INK_K_NKERNEL]; /* GPU time of single kernels of this layer, HIP events (profile != 0) */
} ink_layer_stats;

enum { INK_T_GRAPH = 0, INK_T_EVENTS, INK_T_GROUP, INK_T_AGG, INK_T_COMPACT, INK_T_TRANSFORM,
       INK_T_NCLASS };

typedef struct {
  int32_t n_layers, pad_;
  ink_layer_stats layer[INK_MAX_LAYERS];
  float ms[INK_T_NCLASS];       /* GPU time per kernel class, HIP events (profile != 0), else 0 */
  int32_t launches[INK_T_NCLASS];
  float ms_total;               /* wall time of the call measured on the host                   */
  float pad2_;
} ink_stats;

/* Builds a context: copies graph, features ([n_nodes][feat_dim]) and weights to the device and
 * builds the device graph store (per-node in- and out-edge blocks with slack).  The method's
 * input is a completed full inference of the initial snapshot (Sec. 2): call ink_full_infer next.  Errors: INK_E_ARG (malformed input), INK_E_RANGE (column id outside
 * [0, n)), INK_E_OOM. */
ink_status ink_create(const ink_csr *graph, const float *features, int32_t feat_dim,
                      const ink_model *model, const ink_options *opts, ink_ctx **out);

/* Initial full-graph inference with caching (Sec. 2: the embedding before and after the
 * aggregation is saved for every node in every layer).  May be called again at any time to
 * rebuild the cache from the current graph. */
ink_status ink_full_infer(ink_ctx *ctx);

/* ink_full_infer for callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid it): same arguments, same result, bit for bit, but
 * the call makes no hipMalloc / hipFree (nor any other allocating call).  The work memory that
 * ink_full_infer takes from the allocator -- the list of long rows, the plan and the partial
 * rows of their chunks, GIN's staging rows -- lies in one static device array of
 * INK_NOALLOC_SCRATCH_BYTES bytes per GPU, which that GPU holds until the process ends; the
 * per-kernel-class timing of ink_stats is off during the call.  Every context on a GPU shares
 * the array: calls of this entry point that overlap on one GPU race (calls on one context never
 * overlap anyway).  Nothing in the array is expected to be zero between calls.
 * Errors: INK_E_RANGE if the graph and model need more than the array holds -- the need is
 * 4 (R + 1) + 4 (R + 2) + p w (E / 1024 + R) 4 bytes plus, for GIN, 4 n_nodes hidden, with
 * E the edge count, R = min(node capacity, max(E / 256, 8192)) + 1 the bound on long rows, w the
 * widest aggregated row (at most 256) and p = 4 tables for MAX / MIN, 1 otherwise; then use
 * ink_full_infer.  Otherwise as ink_full_infer. */
#define INK_NOALLOC_SCRATCH_BYTES (64u << 20)
ink_status ink_full_infer_noalloc(ink_ctx *ctx);

/* Applies an ordered list of n updates and incrementally refreshes every layer (Sec. 2.3).
 * The post-update snapshot is the net effect of the list on the edge set.  `updates` is a host
 * or device array according to ink_options.mem.  n = 0 is allowed (empty result).
 * Errors: INK_E_STATE before ink_full_infer; INK_E_RANGE for an id outside [0, n_nodes);
 * INK_E_ARG for op > 1 or n < 0.  On error the graph and the cache are unchanged. */
ink_status ink_apply_updates(ink_ctx *ctx, const ink_edge_update *updates, int64_t n,
                             ink_update_result *out);

/* Baseline for comparison, same arguments and result as ink_apply_updates: the "Affected" method
 * of Sec. 4.1 (inference on the theoretically affected area; Fig. "Inference on a streaming graph"
 * (b)).  Every node reached by a changed edge or by an affected node of the previous layer is
 * recomputed from its whole neighbourhood and re-transformed, and propagates whether or not it
 * changed.  The cache ends in the same state as after ink_apply_updates. */
ink_status ink_apply_updates_affected(ink_ctx *ctx, const ink_edge_update *updates, int64_t n,
                                      ink_update_result *out);

/* Vertex feature update (the input-side counterpart of an edge update; Sec. 2.6 lets callers
 * create and propagate events of their own next to the built-in ones, and this is the one such
 * event a fixed-function library can offer): x_v <- rows[i] for v = node_ids[i], then the same
 * layer-wise propagation as ink_apply_updates with F_1 = the nodes whose feature row changed
 * bitwise (Sec. 2.4: a node whose message changed sends its old and new message to its
 * out-neighbours; Sec. 3.2: its own next embedding depends on it too).  The graph is unchanged.
 *   node_ids : [n] distinct ids in [0, n_nodes), any order
 *   rows     : [n][feat_dim] fp32, row i belongs to node_ids[i]
 * Both arrays are host or device memory like the update batches (ink_options.batch_mem, else
 * ink_options.mem).  The result has the layout of ink_apply_updates' (n_applied_* are 0).
 * Errors: INK_E_STATE before ink_full_infer; INK_E_RANGE for an id outside [0, n_nodes);
 * INK_E_ARG for a repeated id, n < 0 or NULL arrays.  On error nothing is changed. */
ink_status ink_update_features(ink_ctx *ctx, const int32_t *node_ids, const float *rows, int64_t n,
                               ink_update_result *out);

/* User-defined events (Sec. 2.6: callers may create, group and apply events of their own next
 * to the built-in ones, and these are managed apart from them; Sec. 3.2 shows the use: a user_apply
 * step adds a caller-supplied per-node term to the tensor between the linear map and the
 * activation).  Every layer l has a user term u_l[v] of out_dim_l floats per node, zero until an
 * event touches it, and the layer computes h_l[v] = act(T_l(alpha_l[v], h_{l-1}[v]) + u_l[v])
 * (added to the fp32 result of the linear map and its bias, before the activation).  An event
 * names a layer (1 .. n_layers), a target node and an operation on that node's term. */
typedef enum { INK_USER_SET = 0,   /* u <- row          */
               INK_USER_ADD = 1,   /* u <- u + row, one fp32 addition per event */
               INK_USER_CLEAR = 2  /* u <- 0 (row ignored) */ } ink_user_op;
typedef struct {
  int32_t layer, target;
  int32_t op;      /* ink_user_op */
  int32_t pad_;
} ink_user_event;

/* Applies an ordered list of n user events: they are grouped by (layer, target), each group is
 * applied in list order to its node's term, and every node whose term changed bitwise is
 * re-transformed at its layer and, if its embedding changed, propagates to the deeper layers
 * like any changed node (Sec. 2.4.2).  The graph is unchanged; the terms stay in force for every
 * later call, ink_full_infer included.
 *   events : HOST array [n]
 *   rows   : HOST array [n][row_stride]; the first out_dim_layer floats of row i belong to event i
 * (both always host memory: user events are control input, not a data stream).  The first event
 * on a layer allocates that layer's term table (n_nodes capacity x out_dim floats).
 * The result has the layout of ink_apply_updates' (n_applied_* are 0).  Every model kind takes
 * them; for GCN the term joins the bias: h_l = act(normalised sum of layer l + b_l + u_l).
 * Errors: INK_E_STATE before ink_full_infer; INK_E_RANGE for a layer outside 1 .. n_layers or a
 * target outside [0, n_nodes); INK_E_ARG for an unknown op, row_stride below the width of a named
 * layer, n < 0 or NULL arrays.  On these errors nothing is changed. */
ink_status ink_apply_user_events(ink_ctx *ctx, const ink_user_event *events, const float *rows, int32_t row_stride,
                                 int64_t n, ink_update_result *out);

/* Node arrival (Sec. 1 names newly arriving nodes as one source of change; Sec. 2.1 defines the
 * update stream over edges only, so a node arrives without edges and its edges follow through
 * ink_apply_updates).  Appends n_new nodes with ids n_nodes .. n_nodes + n_new - 1 and the given
 * feature rows ([n_new][feat_dim], host or device like the update batches).  Their cached state
 * is that of a node with an empty neighbourhood (alpha = 0, argument -1; GCN: d-hat = 1) and
 * their embeddings are computed layer by layer from it; no other node changes.  The result lists
 * the new ids with their final embeddings.
 * Errors: INK_E_STATE before ink_full_infer; INK_E_RANGE if the node count would exceed
 * ink_options.node_capacity; INK_E_ARG for n_new < 0 or NULL features.  On error nothing changes. */
ink_status ink_add_nodes(ink_ctx *ctx, const float *features, int64_t n_new, ink_update_result *out);

/* Inspection for tests: copies rows [row0, row0 + nrows) of a cached table to dst (host or
 * device per dst_mem), densely packed [nrows][width].  layer in 0..n_layers.
 *   which = 0: h_layer, the output of layer `layer` (layer 0 = input features); it is the
 *              message m_{layer+1} of the aggregate-first models (Sec. 2.1).
 *   which = 1: alpha_layer, the aggregated neighbourhood of layer `layer` >= 1.  For SUM / MEAN
 *              it is the cached plain sum of the neighbours' messages; for GCN_SYM the cached
 *              sum over in-neighbours u of c_u (h_{layer-1} W_layer)_u with c = dhat^(-1/2)
 *              (the row-local factor c_v and the self term are applied when h is formed).
 *   which = 2: int32 argmax/argmin neighbour ids of layer `layer` >= 1 (MAX / MIN only).
 *   which = 3: MAX / MIN only: the cached bound on the best value among the neighbours other
 *              than the holder (>= it for MAX, <= it for MIN; -inf / +inf if there is none).  It is
 *              exact after a recompute and may be loose afterwards; it never affects results.
 *   which = 4: MAX / MIN only, int32: the neighbour other than the holder that has exactly the
 *              value of which = 3 (the lowest such id), or -1 where that is not known.
 *   which = 5: the user term u_layer of ink_apply_user_events (INK_E_ARG if no event ever named the layer).
 * width is returned in *width_out if not NULL. */
ink_status ink_get_layer(ink_ctx *ctx, int32_t layer, int32_t which, int64_t row0, int64_t nrows,
                         void *dst, int32_t dst_mem, int32_t *width_out);

/* Copies the current in-neighbour lists into caller HOST arrays: rowptr [n_nodes + 1] and, if
 * col is not NULL, col [n_edges] (each row ascending).  Pass col = NULL first to size it. */
ink_status ink_get_graph(ink_ctx *ctx, int64_t *rowptr, int32_t *col);

/* Turns the per-kernel-class HIP-event timing of ink_stats on or off (it costs a few event
 * records per layer, which matters for the latency of tiny batches). */
ink_status ink_set_profiling(ink_ctx *ctx, int32_t on);

/* Copies min(bytes, sizeof(ink_stats)) bytes of the last call's statistics. */
ink_status ink_get_stats(ink_ctx *ctx, void *stats_out, size_t bytes);

/* Message of the last failing call on this context ("" if none).  ctx may be NULL: then the
 * message of the last failing ink_create on this thread. */
const char *ink_last_error(const ink_ctx *ctx);

void ink_destroy(ink_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* INK_H */
