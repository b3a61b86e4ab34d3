/*
 * streamtgn.h -- C ABI of the MI355X (gfx950) incremental TGN / TGAT inference step.
 *
 * The library keeps the whole serving state of a temporal graph network resident in
 * device memory (paper Sec. 3.2: temporal adjacency list, per-node recent-neighbour
 * lists, node memory, one embedding cache per attention layer) and exposes the calls of
 * the paper's problem statement: create the state, ingest a batch of timestamped edges
 * (Sec. 3.3 / Algorithm 1, in the order of the "global index refresh" of Sec. 4: apply
 * edges, GRU memory update, dirty-flag propagation, recompute the affected set), read
 * cached embeddings, and rebuild every embedding from scratch (Sec. 3.5, full rebuild).
 *
 * Conventions
 *  - Every function returns STGN_OK (0) or a negative STGN_E_* code; nothing throws.
 *  - All matrices are fp32, row-major, laid out [inputs x outputs] (y = x * W).
 *  - Node ids and edge ids are uint32; timestamps are fp64; features and embeddings fp32.
 *  - "host" / "device" in a comment says where a pointer must point.  The caller owns
 *    every buffer it passes in.  Host inputs are consumed before the call returns.
 *    Device inputs must stay valid until the stream has executed the call (stgn_sync).
 *  - The device workspace is allocated by the caller (stgn_query_workspace tells the
 *    size) and must outlive the context; the library itself allocates no device memory
 *    after stgn_create has returned.
 *  - Work is enqueued on the HIP stream given at creation.  stgn_ingest_batch and
 *    stgn_full_rebuild are asynchronous unless a statistics struct is requested.
 *  - A context is not thread-safe.
 */
#ifndef STREAMTGN_H
#define STREAMTGN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define STGN_MAX_LAYERS 4
#define STGN_MAX_BATCH  8192   /* edges per ingest call (the batch sort runs in one workgroup) */

enum {
  STGN_OK = 0,
  STGN_E_INVALID_ARG       = -1,  /* NULL pointer, unsupported dimension, bad size             */
  STGN_E_NODE_OUT_OF_RANGE = -2,  /* an endpoint id >= num_nodes                               */
  STGN_E_TIME_ORDER        = -3,  /* a timestamp below its predecessor (Definition 1: the edge
                                     stream is chronological) or not a number                  */
  STGN_E_SELF_LOOP         = -4,  /* src == dst                                                */
  STGN_E_BATCH_TOO_LARGE   = -5,  /* n > max_batch                                             */
  STGN_E_EDGE_CAPACITY     = -6,  /* more than max_edges edges in total                        */
  STGN_E_DEVICE            = -7,  /* a HIP call failed or no gfx950 device is present          */
  STGN_E_WORKSPACE         = -8   /* workspace missing, misaligned or too small                */
};

enum { STGN_AGG_LAST = 0, STGN_AGG_MEAN = 1, STGN_AGG_SUM = 2 };

typedef struct stgn_ctx stgn_ctx;

/* Model and capacity description (paper Sec. 2.2 for the dimensions).
 * d_mem = 0 selects a memoryless (TGAT-style) model: no message/GRU stage, layer-0 rows
 * are the static node features.  Layer-0 width is d_mem + d_node and must be > 0.
 * heads is 1, 2 or 4 and divides d_emb; heads * ceil(d_emb / heads / 64) <= 4 (so d_emb <= 256);
 * d_time <= 128; d_mem + d_node <= 512; d_edge <= 1024; layers <= STGN_MAX_LAYERS;
 * max_batch <= STGN_MAX_BATCH; max_edges < 2^31.
 * Keys and values of Eq. attn_detail are linear in [h_u | e | phi(dt)]; their node and edge parts
 * are kept as cached rows (per node and layer, per edge and layer: 2 * 64 * heads * ceil(d_emb /
 * heads / 64) floats each), so the workspace grows by layers * max_edges such rows.  Edge features
 * of at most 64 floats are kept as they are instead (exact mode: max_edges rows of 64 floats, no
 * cached edge rows). */
typedef struct {
  uint32_t num_nodes;
  uint64_t max_edges;
  uint32_t max_batch;
  uint32_t d_mem, d_node, d_edge, d_time, d_emb, d_msg;
  uint32_t k;        /* most recent neighbours kept per node (Sec. 3.3.2)   */
  uint32_t heads;    /* attention heads                                    */
  uint32_t layers;   /* attention layers = hops of dirty-flag propagation   */
  double   window;   /* temporal window T_w of the neighbour cache (Sec. 3.3.2, "Invalidate"): a recent-
                        neighbour entry older than the query time minus T_w is not attended to;
                        <= 0: no expiry.  The affected set does not depend on it (a sound superset). */
  uint32_t aggregator; /* Eq. agg_functions, how a node's messages of one batch become one: STGN_AGG_LAST
                        (the latest), STGN_AGG_MEAN, STGN_AGG_SUM (added in batch order).  Ignored when d_mem = 0. */
  uint32_t delta_mode; /* 0: every affected row is recomputed exactly (results identical to a full recomputation).
                        1: the approximate mode of Sec. 3.3 "Stage 4" / Eq. delta_embedding (see stgn_maintain). */
  double   drift_gamma; /* delta mode: decay of the drift estimator per batch (Sec. 3.5), in (0, 1]; else ignored */
} stgn_config;

/* Parameters, host pointers, copied (and re-packed) by stgn_create.
 *   time encoding (Sec. 2.2.1):  phi_i(x) = sqrt(1/d_time) * cos(omega_i * x + phase_i)
 *   message (Eq. msg_linear):    m = [s_self | s_other | e | phi(t - t_self_last)] W_msg + b_msg
 *   GRU (Eq. gru_detail):        W_*: [d_msg x d_mem], U_*: [d_mem x d_mem], b_*: [d_mem]
 *   attention layer l (Eq. attn_detail), d_in = (l == 0 ? d_mem + d_node : d_emb):
 *       W_Q[l]: [(d_in + d_time) x d_emb]           input [h_v | phi(0)]
 *       W_K[l], W_V[l]: [(d_in + d_edge + d_time) x d_emb]   input [h_u | e | phi(dt)]
 *       W_O[l]: [d_emb x d_emb], b_O[l]: [d_emb]    applied to the concatenated heads
 * The message/GRU pointers are ignored when d_mem == 0. */
typedef struct {
  const float *omega, *phase;
  const float *W_msg, *b_msg;
  const float *W_z, *U_z, *b_z, *W_r, *U_r, *b_r, *W_h, *U_h, *b_h;
  const float *const *W_Q, *const *W_K, *const *W_V, *const *W_O, *const *b_O; /* [layers] each */
} stgn_weights;

/* Per-batch report; requesting it makes stgn_ingest_batch synchronise the stream. */
typedef struct {
  uint32_t n_edges;
  uint32_t n_direct;                       /* |V_direct|: distinct endpoints of the batch     */
  uint32_t n_affected;                     /* |V_aff| (Eq. affected_set)                      */
  uint32_t frontier[STGN_MAX_LAYERS + 1];  /* nodes first reached at hop h (frontier[0]=|D|)   */
  uint64_t entries_scanned;                /* adjacency entries (push hops) and ring slots    */
                                           /* (pull hops) read by the propagation             */
  uint32_t pull_hops;                      /* bit h set: hop h pulled through the rings of the
                                              clean nodes instead of pushing along the logs of
                                              the frontier (chosen on the device, same flags) */
  uint32_t reserved;
  float    us_stage[6];                    /* sort | memory update | apply | propagate+compact
                                              | embed | total; microseconds from HIP events    */
} stgn_batch_stats;

/* Device bytes stgn_create needs for this configuration (host computation only): the whole
 * device-resident state, dominated by the per-edge tables (adjacency, cached key|value rows of
 * every edge and layer).  From 32,768 nodes (k <= 32) the library also keeps, per node, the query
 * vectors of the first layer (of every layer for a model without memory), 64 * (ks + heads * nt)
 * floats each (ks = heads * ceil(d_emb / heads / 64), nt = ceil(d_time / 64)); delta_mode adds the
 * attention cache described at stgn_maintain. */
int stgn_query_workspace(const stgn_config *cfg, size_t *device_bytes);

/* Builds the state on the current device: zero memory (Sec. 2.2.4), empty adjacency, every
 * cached row equal to the empty-neighbourhood embedding.  node_feat: host [num_nodes x d_node]
 * or NULL (zeros).  workspace: device, 256-byte aligned, >= the queried size.  hip_stream: a
 * hipStream_t (NULL = the default stream).  Synchronises before returning. */
int stgn_create(const stgn_config *cfg, const stgn_weights *w, const float *node_feat,
                void *device_workspace, size_t device_bytes, void *hip_stream, stgn_ctx **out);

void stgn_destroy(stgn_ctx *ctx);

/* One incremental step (Sec. 3.3, Algorithm 1; order of Sec. 4 "Global index refresh"):
 * messages + aggregation (stgn_config.aggregator) + GRU on the batch endpoints from pre-batch
 * state, append the edges, propagate dirty flags `layers` hops, recompute all layers for the
 * affected set.
 * src, dst: [n]; ts: [n] non-decreasing and >= the last ingested timestamp; efeat: [n x d_edge]
 * (may be NULL when d_edge == 0).  All four live on the host (inputs_on_device = 0) or all on
 * the device (1).  Errors found on the host are returned at once and leave the state untouched;
 * with device inputs the check runs on the device, a failing batch is skipped as a whole and
 * its code is returned by the next synchronising call (stgn_sync, stgn_get_*, or this call with
 * stats != NULL).
 * The call is asynchronous.  A batch with stats == NULL that follows another asynchronous call
 * without a synchronising call in between runs its front part (the copy of host inputs,
 * validation, endpoint sort, memory update and, on small graphs, the propagation) on a stream of
 * the library's own so that it overlaps the previous batch's attention layers; the rest runs on
 * hip_stream, and work enqueued on hip_stream after the call is ordered after the whole batch.
 * Device inputs must therefore hold their final contents when the call is made (they are not
 * ordered after work still pending on hip_stream) and must stay unchanged until the batch has
 * completed.  Host inputs are copied before the call returns.  With stats != NULL the call
 * synchronises. */
int stgn_ingest_batch(stgn_ctx *ctx, uint32_t n, const uint32_t *src, const uint32_t *dst,
                      const double *ts, const float *efeat, int inputs_on_device,
                      stgn_batch_stats *stats /* host, nullable */);

/* Cached final-layer rows (Sec. 3.2.3, O(1) lookup per node).  layer: 1..layers, or 0 for the
 * last one.  nodes/out on host (on_device = 0, synchronises) or device (1, asynchronous).
 * out: [n x d_emb].  Host ids >= num_nodes return STGN_E_NODE_OUT_OF_RANGE; a device-resident id
 * >= num_nodes gives that row NaN in every column. */
int stgn_get_embeddings(stgn_ctx *ctx, uint32_t layer, uint32_t n, const uint32_t *nodes,
                        float *out, int on_device);

/* Recompute every layer for every node from the current state (Sec. 3.5, full rebuild); in delta mode every
 * attention cache is refreshed and the drift estimators restart. */
int stgn_full_rebuild(stgn_ctx *ctx);

/* ---- Delta mode (Sec. 3.3 "Stage 4", Eq. delta_embedding; Sec. 3.5, drift-aware rebuild scheduling) ----
 * With delta_mode = 1 the library keeps, per layer and node, an attention cache: per recent-neighbour entry the
 * score, the attention weight in effect and the neighbour|edge part of the value, and per row the weighted sums,
 * the softmax denominator and its reference score.  After a batch a listed row whose own input row and query
 * time are unchanged (it is in the affected set only because neighbours changed) is not recomputed: each entry j
 * whose neighbour's input row changed gets its new score s', the denominator becomes Z' = Z - e^(s_j) + e^(s'),
 * the entry's weight e^(s') / Z', and the sums are corrected by (new weight x new value) - (old weight x old
 * value); the other entries keep the weight they have, so the weights no longer sum to one exactly.  The
 * row's deviation from the exact row is at most
 *     (attention mass of the unchanged entries) x max |V_unchanged| x |1 - Z / Z'| x ||W_O||_2
 * per update.  Endpoints of the batch, rows whose own input changed, and every row touched by a rebuild are
 * recomputed exactly and refresh their cache.  stgn_predict_batch(at_edge_time = 1) always computes exactly.
 * Costs layers x num_nodes x k x (64 ks + 2 heads) floats of workspace on top of the exact mode
 * (ks = heads x ceil(d_emb / heads / 64)), and always keeps the cached edge rows.
 *
 * Drift estimator: per node the decayed sum, over the batches since the node's final-layer row was last
 * exact, of (changed entries / entries) of its delta updates: est_v <- gamma est_v per batch.  The global metric
 * is the mean estimate over the nodes updated since the last rebuild (Eq. global_drift).
 *
 * stgn_drift_status: synchronises; global_drift, n_tracked (size of that node set) and per_node (host
 * [num_nodes], the decayed estimates) are each nullable. */
int stgn_drift_status(stgn_ctx *ctx, double *global_drift, uint32_t *n_tracked, float *per_node);

/* Adaptive rebuild policy (Eq. rebuild_trigger).  Synchronises.  While the global metric is at most delta_max:
 * nothing (STGN_MAINTAIN_NONE).  Otherwise V_drift = nodes whose own estimate exceeds delta_max; if
 * |V_drift| < alpha * num_nodes their rows are recomputed exactly at every layer (STGN_MAINTAIN_PARTIAL; rows
 * outside V_drift keep what they hold), else every row is (STGN_MAINTAIN_FULL, = stgn_full_rebuild); either way
 * all estimators restart at zero.  action, n_drift (|V_drift|): host, nullable.  The rebuild itself is
 * enqueued, not awaited. */
#define STGN_MAINTAIN_NONE 0
#define STGN_MAINTAIN_PARTIAL 1
#define STGN_MAINTAIN_FULL 2
int stgn_maintain(stgn_ctx *ctx, double delta_max, double alpha, int *action, uint32_t *n_drift);

/* Link-prediction head (Algorithm 1, "Link prediction").  The paper's error analysis (Sec. 3.6.3)
 * takes the score as a linear function of the concatenated source and destination embeddings:
 *     y = [h_u | h_v] . w + b.
 * w: host [2 * d_emb], source half first; copied.  May be called again at any time. */
int stgn_set_predictor(stgn_ctx *ctx, const float *w, float b);

/* Per-batch root-node inference (Algorithm 1: embed, predict, THEN update; Sec. 3.6.2,
 * Eq. parallel_embed): link scores of n edges (u_i, v_i, t_i) that have NOT been ingested yet,
 * from the current (pre-batch) state.  Call it before stgn_ingest_batch of the same edges.
 *   at_edge_time = 0: h_u, h_v are the cached final-layer rows (two O(1) lookups per edge: the
 *       caches are exact after every batch, so no root is ever dirty at this point);
 *   at_edge_time = 1: the final layer is evaluated for the 2n roots at the edge's own time (time
 *       gaps t_i - t_j to the root's recent neighbours, query side phi(0)); the layers below are
 *       the cached rows.  With one layer this is Eq. parallel_embed evaluated at t_i.
 * src, dst, ts, scores: [n], all on the host (inputs_on_device = 0; synchronises) or all on the
 * device (1; asynchronous on hip_stream).  n <= max_batch.  Needs stgn_set_predictor.  Host
 * inputs with an id >= num_nodes return STGN_E_NODE_OUT_OF_RANGE; device inputs give that edge
 * the score NaN.  Changes no state. */
int stgn_predict_batch(stgn_ctx *ctx, uint32_t n, const uint32_t *src, const uint32_t *dst,
                       const double *ts, int at_edge_time, int inputs_on_device, float *scores);

/* stgn_predict_batch for callers that cannot allocate (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): device inputs and outputs only, asynchronous on hip_stream,
 * and no allocation of any kind inside the call.  The scratch its kernels need -- the 2n roots, their
 * query times and their final-layer rows -- lives in a file-scope device array of the library instead
 * of the workspace: STGN_STATIC_SCRATCH_BYTES per GPU the library has been used on, held until the
 * process ends.  n edges of d_emb-wide rows need 2n (4 + 8 + 4 d_emb) bytes (each of the three lists
 * rounded up to 256); a larger n returns STGN_E_BATCH_TOO_LARGE and enqueues nothing.  Nothing in the
 * array has to start at zero (every entry read is written first by the same call).  All contexts on a
 * GPU share the array: calls that overlap on one GPU (two streams, two contexts) race; calls on one
 * stream follow each other.  Same results as stgn_predict_batch with inputs_on_device = 1. */
#define STGN_STATIC_SCRATCH_BYTES (4u << 20)
int stgn_predict_batch_static(stgn_ctx *ctx, uint32_t n, const uint32_t *src, const uint32_t *dst,
                              const double *ts, int at_edge_time, float *scores);

/* Waits for the stream; returns the code of the first skipped device-side batch (and clears it). */
int stgn_sync(stgn_ctx *ctx);

/* ---- inspection hooks used by the parity tests (all synchronise, host outputs) ---- */

/* Affected set of the last ingested batch, ascending.  count receives |V_aff|; at most cap ids
 * are written. */
int stgn_get_affected(stgn_ctx *ctx, uint32_t *out, uint32_t cap, uint32_t *count);

/* Most recent <= k neighbours of a node, most recent first (Sec. 3.3.2).  Arrays of length k. */
int stgn_get_neighbors(stgn_ctx *ctx, uint32_t node, uint32_t *nbr, uint32_t *eid, double *ts,
                       uint32_t *count);

/* `count` entries of a node's full temporal adjacency starting at position `first` (arrival
 * order; Sec. 3.2.2 GetNeighbors).  degree receives the node's total entry count. */
int stgn_get_history(stgn_ctx *ctx, uint32_t node, uint32_t first, uint32_t count,
                     uint32_t *nbr, uint32_t *eid, uint32_t *degree);

/* Memory rows [n x d_mem] (nullable) and last-interaction times [n] (nullable). */
int stgn_get_memory(stgn_ctx *ctx, uint32_t n, const uint32_t *nodes, float *mem, double *t_last);

/* Totals since creation: edges ingested, sum of |V_direct|, sum of |V_aff|, adjacency entries
 * scanned by the propagation, recent-neighbour entries gathered and rows recomputed by the
 * attention kernels (both summed over layers; both include full rebuilds).  Layer l of a batch
 * recomputes only the affected nodes whose layer-l inputs changed (the endpoints and the first l
 * hops; one hop less for a memoryless model, whose layer-0 rows never change), so `rows` can be
 * smaller than layers * sum of |V_aff|.  Synchronises.  Any pointer may be NULL. */
int stgn_get_totals(stgn_ctx *ctx, uint64_t *edges, uint64_t *direct, uint64_t *affected,
                    uint64_t *scanned, uint64_t *gathered, uint64_t *rows);

/* Microseconds (HIP events on the context's stream) spent in each kernel class since the last
 * call with reset != 0, and launch counts.  Collection is off until enabled; while it is on,
 * every kernel launch is bracketed by two events.  names: static strings owned by the library.
 * Returns the number of classes written (<= cap) or a negative code. */
int stgn_kernel_times(stgn_ctx *ctx, int enable, int reset, uint32_t cap,
                      const char **names, double *usec, uint64_t *launches);

/* Diagnostic, no context: one launch of a bare gather on hip_stream, for pricing the layer kernel's
 * gathers against what the memory system delivers to that access pattern alone.  table: device,
 * n_rows rows of row_bytes (256 or 1024: a raw edge row, a cached key|value row of two slots per
 * half) each, 256-byte aligned; idx: device, n_groups * per_group row numbers < n_rows (not
 * checked: the caller's); every group of 16 lanes sums its per_group rows, one row in flight, and
 * writes 16 floats to out (device, n_groups * 16 floats).  Asynchronous; the caller times it.
 * STGN_E_INVALID_ARG for a NULL pointer, another row size or an empty launch. */
int stgn_probe_gather(const float *table, uint64_t n_rows, uint32_t row_bytes, const uint32_t *idx,
                      uint32_t n_groups, uint32_t per_group, float *out, void *hip_stream);

const char *stgn_last_error(const stgn_ctx *ctx);   /* NULL ctx: message of the last failed create */
const char *stgn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* STREAMTGN_H */
