// Internal declarations shared by the translation units of libstreamtgn (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include <stddef.h>

#include "streamtgn.h"

namespace stgn {

constexpr uint32_t kLogChunk = 128;    // adjacency entries per propagation work item
constexpr uint32_t kMinBlock = 8;      // entries in the first adjacency block of a node
constexpr uint32_t kMarkPad = 4096;    // the dirty-flag array is padded to whole compaction blocks
inline __host__ __device__ size_t mark_bytes(uint32_t N) { return ((size_t)N + kMarkPad - 1) / kMarkPad * kMarkPad; }

// 16-byte recent-neighbour record (Sec. 3.3.2): slot (pos mod k) of node v at ring[v*k + slot]
struct __align__(16) RingEntry {
  uint32_t nbr;
  uint32_t eid;
  double   t;
};

// Device-resident control block: every size the kernels need lives here so that a whole batch
// can be enqueued without reading anything back.  The fields of one batch are kept twice and the
// batches alternate between the copies (as they do between two sets of the per-batch scratch lists),
// so that the next batch can be staged while kernels of the current one still read theirs.
// Per-batch state (batch fields of the control block, sorted endpoint lists, striped counters, work
// items) is held kSets times: a batch's staging kernel may run while the previous batch's main part
// is still at work and the one before that has only just finished.
constexpr int kSets = 3;

struct BatchCtl {
  uint32_t skip;                 // 1: the batch failed validation, all its kernels exit
  uint32_t n_edges;              // edges of the batch
  uint32_t nD;                   // |V_direct| of the batch
  uint32_t nA;                   // |V_aff| of the batch
  uint32_t n_front[STGN_MAX_LAYERS + 2];  // frontier sizes per hop (n_front[0] = nD)
  uint32_t n_items[STGN_MAX_LAYERS + 1];  // propagation work items per hop
  uint32_t nR[STGN_MAX_LAYERS];  // rows layer l recomputes in the batch
  uint32_t pulled[STGN_MAX_LAYERS + 1];   // bit 0: hop h ran in pull mode; bit 1: its frontier preferred pulling
  uint64_t scanned;              // adjacency entries scanned in the batch (summed up by the compaction)
  uint64_t E_base;               // edges ingested before the batch
};
// Counters that every workgroup of a kernel adds to are STRIPED: same-address atomic updates from
// thousands of workgroups serialise (measured: about 5 ns each, 60 us for the two counters of one
// propagation hop on a million nodes), so a counter is kStripes values in cache lines of their own,
// a workgroup adds to the stripe of its index and readers sum the stripes.  Per batch (held twice, by
// batch parity): counter h = adjacency entries the frontier of hop h owns (exact for hop 0 and after a
// pull hop, an upper estimate after a push hop; decides between pushing along the frontier's logs and
// pulling through the rings of the clean nodes), counter kScannedCounter = adjacency entries scanned.
constexpr uint32_t kStripes = 32;
constexpr uint32_t kStripeWords = 16;                        // uint64 per 128-byte line
constexpr uint32_t kScannedCounter = STGN_MAX_LAYERS + 1;
constexpr uint32_t kStripedCounters = STGN_MAX_LAYERS + 2;
constexpr uint32_t kStatSlots = 1024;                        // per-workgroup statistic slots of the layer kernel (its grid never exceeds this)

struct Ctrl {
  int32_t  err_code;             // first device-side error (sticky until read by the host)
  uint32_t err_batch;
  uint32_t batch_seq;            // batches seen
  uint32_t pad0;
  uint64_t E;                    // edges ingested including the last staged batch
  uint64_t pool_units;           // adjacency pool cursor, in units of kMinBlock entries
  double   t_stream;             // last ingested timestamp
  uint64_t tot_direct, tot_affected, tot_scanned;
  uint64_t tot_rows;             // rows the attention kernels recomputed (all layers)
  BatchCtl b[kSets];
};

// Drift estimator of the delta mode (Sec. 3.5, Definition "Drift Estimator", Eq. global_drift): the sum of the
// per-node estimates, the size of the cumulative affected set since the last rebuild, the batch counter the
// per-node values decay against, and the length of the list of drifted nodes (stgn_maintain).
struct DriftCtl {
  double   G;
  uint32_t count, tau, n_list, pad;
};

// Row-table descriptor: row v starts at base + v * ld (floats)
struct Table {
  float*   base;
  uint32_t ld;
};

// Packed parameters of one attention layer (device pointers).
//
// Keys and values are linear in the attention input z_j = [h_{u_j} | e_j | phi(dt)], so they split by
// input block (paper Eq. attn_detail):  K_j = h_{u_j} W_K[node rows] + e_j W_K[edge rows] + phi W_K[time rows].
// The first term depends on the neighbour alone and the second on the edge alone; both are kept as
// cached rows (KV tables below: per node and layer, refreshed whenever the node's input row changes;
// per edge and layer, written once when the edge arrives).  Only the time term depends on the pair and
// is evaluated re-associated:  q_h . (phi W_K,h) = (W_K,h[time] q_h) . phi  and
// sum_j a_j (phi_j W_V,h) = (sum_j a_j phi_j) W_V,h[time], so every dense product runs over rows, not
// over (row, neighbour) pairs.
//
// A cached row holds [keys | values]; each head occupies whole slots of 64 floats (one slot = 16
// lanes x float4), columns past dk are exact zeros: ld_kv = 2 * 64 * ks floats, ks = heads * ceil(dk / 64).
//
// Narrow edge features (d_edge <= 64, exact mode) are not projected at all: the raw feature row, padded to
// one slot, is kept once per edge and rides through the layer kernel as one more slot of the time encoding,
//   q_h . (f W_K,h[edge]) = (W_K,h[edge] q_h) . f   and   sum_j a_j (f_j W_V,h[edge]) = (sum_j a_j f_j) W_V,h[edge],
// i.e. the vector z_j = [phi(dt_j) | f_j] takes the place of phi in the re-associated products above.  A
// gathered entry then reads 256 bytes for its edge instead of a cached row per layer.
constexpr uint32_t kSlot = 64;
constexpr uint32_t kMaxKeySlots = 4;     // ks
constexpr uint32_t kMaxTimeSlots = 2;    // ceil(d_time / 64)
struct LayerDev {
  uint32_t d_in;                 // input width
  const float* WQn;              // [d_in x d_emb]            node block of W_Q / sqrt(dk)
  const float* cQ;               // [d_emb]                   phi(0) * (time block of W_Q) / sqrt(dk)
  const float* WKT;              // [dk x heads * 64 nz]      (time rows of W_K, head block)^T * sqrt(1/d_t), then, with raw
                                 //                           edge rows, (edge rows of W_K, head block)^T in slot nt
  const float* WV;               // [64 nz x heads * R16(dk)] time rows of W_V, head block, * sqrt(1/d_t); edge rows in slot nt
  const float* WO;               // [64 ks x d_emb]           rows in the padded-head layout of the head outputs
  const float* bO;               // [d_emb]
  const float* WKVn;             // [d_in x 128 ks]           node rows of [W_K | W_V] in the cached-row layout
  const float* WKVe;             // [d_edge x 128 ks]         edge rows of [W_K | W_V] (null without edge features or with raw edge rows)
};

struct Dev {
  // configuration
  uint32_t N, k, heads, layers, d_mem, d_node, d0, d_edge, d_time, d_emb, d_msg, dk;
  uint32_t max_batch, maxb;      // maxb: adjacency blocks per node in the block table
  double   window;               // temporal window of the neighbour cache (+inf: no expiry)
  uint32_t aggregator;           // Eq. agg_functions: 0 Last, 1 Mean, 2 Sum
  uint32_t num_cu;               // compute units of the device the context lives on
  uint64_t max_edges, pool_cap_units;
  // persistent state
  Table    H[STGN_MAX_LAYERS + 1];   // H[0] = [memory | node features]; H[l] = layer-l cache
  double*  t_last;                   // [N]
  uint32_t* deg;                     // [N] adjacency entries per node
  uint32_t* ring_nbr;                // [N x k] neighbour ids of the ring slots alone (4 B per slot, for the pull hop)
  RingEntry* ring;                   // [N x k]
  uint2*   pool_nt;                  // adjacency pool: (neighbour, position of the twin entry)
  uint32_t* pool_eid;                // adjacency pool: edge id
  uint32_t* blk;                     // [N x maxb] block bases in units of kMinBlock entries
  // cached key|value rows (see LayerDev): KV[l] of the rows of H[l], KVE[l] of the edge features
  Table    KV[STGN_MAX_LAYERS];      // [N x ld_kv]
  Table    KVE[STGN_MAX_LAYERS];     // [max_edges x ld_kv]; one zero row (ld 0) without edge features; with raw edge
                                     // rows every layer names the one table [max_edges x 64] of padded feature rows
  uint32_t sh, ks, nt, ld_kv;        // slots per head, key slots, time slots, floats per cached row
  uint32_t es, nz;                   // es = 1: raw edge rows; nz = nt + es slots of the vector z = [phi | f]
  // per-batch scratch: two sets, the batches alternate (bind_batch points the plain fields at one of them)
  struct Scratch {
    uint32_t *D, *seg_start, *last_slot, *deg_new, *slot_pos, *slot_d, *slot_sorted;
    float* mem_new;
  } scr[kSets];
  Ctrl*    ctrl;
  BatchCtl* bc;                      // the current batch's copy of the batch fields (set per batch by the host)
  char*    stage[2];                 // staging blocks for host inputs (batches alternate)
  uint32_t* D;                       // [2*max_batch] sorted distinct endpoints
  uint32_t* seg_start;               // [2*max_batch + 1]
  uint32_t* last_slot;               // [2*max_batch] per D entry: slot (2*i + side) of its last edge
  uint32_t* deg_new;                 // [2*max_batch] per D entry: degree after the batch
  uint32_t* slot_pos;                // [2*max_batch] per slot: position in its node's adjacency
  uint32_t* slot_d;                  // [2*max_batch] per slot: index into D
  uint32_t* slot_sorted;             // [2*max_batch] slots ordered by (node, slot): D entry x owns [seg_start[x], seg_start[x+1])
  float*   mem_new;                  // [2*max_batch x d_mem]
  uint8_t* mark;                     // [mark_bytes(N)] dirty flags, one byte per node (of the bound batch)
  // Small flag arrays are held twice, by batch parity: a batch's one-launch compaction leaves its own
  // flags alone (other workgroups may still be counting them) and clears the other array, which the
  // next batch uses.  Large arrays are one array (both entries equal), cleared by the compaction's second launch.
  uint8_t* mark_set[2];
  uint8_t* mark_other;               // the array of the other parity (bound batch)
  uint64_t* stripes_set[kSets];          // [kStripedCounters][kStripes] lines of kStripeWords words, per batch parity
  uint64_t* stripes;                 // ... of the bound batch
  uint64_t* gathered_slots;          // [kStatSlots] ring entries gathered by the layer kernel, one slot per workgroup index
  uint64_t* items;                   // propagation work items (node, chunk)
  uint64_t* items_set[kSets];            // ... held twice, by batch parity: a batch's first hop may run beside the previous batch's last
  uint64_t items_cap;
  uint32_t* blocksum;                // compaction partial sums
  uint32_t* A;                       // [N] affected set, ascending
  // Layer l only has to recompute the nodes whose inputs changed: flag <= thr[l] (the endpoints plus
  // the first l hops with a memory, one hop less without one, where layer-0 inputs never change).
  // R[l] is that ascending sub-list of A (A itself where the threshold covers every flag).
  uint32_t* R[STGN_MAX_LAYERS];
  // RS[l]: R[l] regrouped by recent-neighbour entry count (bucket_rows_kernel), what the layer launches walk on
  // graphs large enough for it to pay (bucketed); layers that share a list share the copy
  uint32_t* RS[STGN_MAX_LAYERS];
  uint32_t bucketed;
  // Query cache (with the regrouped lists, exact mode): per layer and node the query vector q and its time part
  // qt (Eq. attn_detail: q = [h_v | phi(0)] W_Q; qt_h = q_h W_K,h[time rows]^T), which depend on the node's own
  // input row only, in the layout of the layer kernel's q and qt tiles.  A listed row whose input row did not
  // change in the batch reads them back instead of projecting again; the regrouping puts such rows together
  // and says per tile of 16 list positions whether all of its rows are of that kind (tile_clean).
  uint32_t qcache;
  uint32_t ld_qc;                    // floats per cached row: 64 (ks + heads nz)
  float*   QC[STGN_MAX_LAYERS];      // [N x ld_qc]
  uint8_t* tile_clean[STGN_MAX_LAYERS];   // [ceil(N / 16)]
  uint32_t thr[STGN_MAX_LAYERS];
  uint32_t n_lists;                  // separate lists (layers whose threshold does not cover every flag)
  // delta mode (Sec. 3.3 "Stage 4", Eq. delta_embedding; null / 0 when it is off): the attention cache per layer
  // and node -- the sums in effect S (head outputs before the time part, a row of the head-output tile) and
  // pb (a row of the time tile), the softmax denominator and its reference score per head, and per
  // recent-neighbour entry (index = recency at the row's last exact recomputation) score and weight in effect per
  // head and the neighbour|edge part of the value -- the flags of the last batch where the compaction clears
  // them, and the drift estimator (per node: running sum with lazy decay, batch of the last update, member of
  // the cumulative affected set)
  uint32_t delta;
  float    gamma;
  float*   ac_S[STGN_MAX_LAYERS];    // [N x 64 ks]
  float*   ac_P[STGN_MAX_LAYERS];    // [N x 64 nt heads]
  float*   ac_ZM[STGN_MAX_LAYERS];   // [N x 2 heads]     Z_h at 2h, m_h at 2h + 1
  float*   ac_W[STGN_MAX_LAYERS];    // [N x k x 2 heads] s_h at 2h, a_h at 2h + 1
  float*   ac_V[STGN_MAX_LAYERS];    // [N x k x 64 ks]
  uint8_t* flags_kept;               // [mark_bytes(N)] (also kept for the query cache)
  DriftCtl* drift;
  float*   dsum; uint32_t* dlast; uint8_t* dseen;   // [N] each
  uint32_t* dlist;                   // [N] nodes whose estimate exceeds the threshold (stgn_maintain)
  // root-node inference (stgn_predict_batch): the 2n roots (source, destination of edge i at 2i, 2i+1),
  // their query times, their final-layer rows, staging for host inputs / outputs, and the head [w | b]
  uint32_t* pred_rows; double* pred_tq; float* pred_out;
  uint32_t* pred_src; uint32_t* pred_dst; double* pred_ts; float* pred_scores;
  float*   pred_w;
  uint32_t* qnodes; float* qout;     // staging for host-side get_embeddings
  uint32_t q_cap;
  // parameters
  const double* om_rev; const double* ph_rev;   // omega/(2 pi), phase/(2 pi)
  uint32_t Kmsg;                                // message input width 2 d_mem + d_edge + d_time
  const float* Wmsg; const float* bmsg;         // matrices in the group-major packing of mfma16.h
  const float* Wzr;  const float* Uzr;          // [d_msg x 2 R16(d_mem)], [d_mem x 2 R16(d_mem)]: update | reset gate
  const float* Wh;   const float* Uh;           // [d_msg x d_mem], [d_mem x d_mem]
  const float* bz; const float* br; const float* bh;
  LayerDev L[STGN_MAX_LAYERS];
};

inline __host__ __device__ uint32_t round_up(uint32_t x, uint32_t m) { return (x + m - 1) / m * m; }

// the device description a batch of the given parity is enqueued with
// set: which copy of the per-batch state (0 .. kSets - 1); flag_par: which dirty-flag array (0 / 1)
inline Dev bind_batch(const Dev& base, int set, int flag_par) {
  Dev d = base;
  const Dev::Scratch& s = base.scr[set];
  d.D = s.D; d.seg_start = s.seg_start; d.last_slot = s.last_slot; d.deg_new = s.deg_new;
  d.slot_pos = s.slot_pos; d.slot_d = s.slot_d; d.slot_sorted = s.slot_sorted; d.mem_new = s.mem_new;
  d.bc = base.ctrl ? &base.ctrl->b[set] : nullptr;
  d.mark = base.mark_set[flag_par]; d.mark_other = base.mark_set[flag_par ^ 1];
  d.stripes = base.stripes_set[set];
  d.items = base.items_set[set];
  return d;
}

__device__ inline unsigned long long* stripe(const Dev& d, uint32_t counter, uint32_t index) {
  return reinterpret_cast<unsigned long long*>(d.stripes) + ((size_t)counter * kStripes + (index & (kStripes - 1u))) * kStripeWords;
}
// sum of a striped counter; every lane of the calling wave must be active, all receive the sum
__device__ inline unsigned long long stripes_sum_wave(const Dev& d, uint32_t counter) {
  const uint32_t lane = threadIdx.x & 63u;
  unsigned long long v = lane < kStripes ? *stripe(d, counter, lane) : 0ull;
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
  return v;
}
// ... by a single thread
__device__ inline unsigned long long stripes_sum_thread(const Dev& d, uint32_t counter) {
  unsigned long long v = 0;
  for (uint32_t s = 0; s < kStripes; ++s) v += *stripe(d, counter, s);
  return v;
}

// Kernel classes for the optional event timing
enum KernelClass { KC_SORT = 0, KC_MEMORY, KC_APPLY, KC_PLAN, KC_EXPAND, KC_COMPACT, KC_LAYER,
                   KC_GATHER, KC_NOOP, KC_PROJECT, KC_PREDICT, KC_BUCKET, KC_COUNT };

// A launch whose completion is an event (`done`, may be null): the event rides on the kernel's own
// completion signal instead of a marker of its own behind it, which costs the stream a microsecond or
// two less than hipEventRecord after the launch.  Waits on such an event were checked to be ordered
// behind the kernel's last store (400 producer / consumer pairs on two streams).
template <class K, class... Args>
inline void launch_done(K kernel, dim3 grid, dim3 block, size_t lds, hipStream_t s, hipEvent_t done, Args... args) {
  if (done) hipExtLaunchKernelGGL(kernel, grid, block, lds, s, nullptr, done, 0, args...);
  else hipLaunchKernelGGL(kernel, grid, block, lds, s, args...);
}

// ---- launch wrappers (one per kernel family), defined in the .hip files ----
void launch_stage_sort(const Dev& d, hipStream_t s, uint32_t n, const uint32_t* src, const uint32_t* dst,
                       const double* ts);
void launch_place(const Dev& d, hipStream_t s, uint32_t n, hipEvent_t done = nullptr);
// with_place: the launch also places the batch's endpoint slots (no launch_place then)
void launch_memory_update(const Dev& d, hipStream_t s, const uint32_t* src, const uint32_t* dst, const double* ts,
                          const float* ef, bool with_place, hipEvent_t done = nullptr);
void launch_apply(const Dev& d, hipStream_t s, const uint32_t* src, const uint32_t* dst, const double* ts,
                  const float* ef, bool with_compaction, hipEvent_t done = nullptr);   // with_compaction: only for compact_in_one(d), after the propagation
void launch_plan(const Dev& d, hipStream_t s, uint32_t hop);
void launch_expand(const Dev& d, hipStream_t s, uint32_t hop, bool planned, hipEvent_t done = nullptr);
void launch_compact(const Dev& d, hipStream_t s, int phase);
void launch_bucket_rows(const Dev& d, hipStream_t s, bool all_rows);   // regroups the layers' row lists by entry count (Dev::RS)
bool compact_in_one(const Dev& d);   // the compaction is a single launch (phase 0) for this node count
// force_exact: recompute every listed row exactly (initial state, rebuilds); otherwise, in delta mode, a row
// whose own input row and query time are unchanged takes the delta update
void launch_layer(const Dev& d, hipStream_t s, uint32_t layer, const uint32_t* rows, const uint32_t* count_ptr,
                  uint32_t count_max, bool force_exact = true);
// drift estimator: clear it; list the nodes whose estimate exceeds `threshold` (Dev::dlist, DriftCtl::n_list)
void launch_drift_reset(const Dev& d, hipStream_t s);
void launch_drift_list(const Dev& d, hipStream_t s, float threshold);
void launch_drift_values(const Dev& d, hipStream_t s, float* out);   // every node's decayed estimate, [N]
void launch_gather_rows(const Dev& d, hipStream_t s, uint32_t layer, uint32_t n, const uint32_t* nodes, float* out);
void launch_gather_times(const Dev& d, hipStream_t s, uint32_t n, const uint32_t* nodes, double* out);   // last-interaction times
// root-node inference: roots and query times of n edges; the final layer for the 2n roots; the linear head
void launch_predict_prep(const Dev& d, hipStream_t s, uint32_t n, const uint32_t* src, const uint32_t* dst, const double* ts);
void launch_layer_roots(const Dev& d, hipStream_t s, uint32_t nroots);
void launch_predict_head(const Dev& d, hipStream_t s, uint32_t n, const uint32_t* src, const uint32_t* dst,
                         int at_edge_time, float* scores);
void launch_init_state(const Dev& d, hipStream_t s);
void launch_zero(float* p, size_t n, hipStream_t s);
void launch_noop(hipStream_t s);
int  attn_supported(uint32_t d_emb, uint32_t d_time, uint32_t heads);
// cached key|value rows of all nodes for layer 0 (those of a batch's endpoints and edges are computed by launch_apply)
void launch_project_nodes(const Dev& d, hipStream_t s);
constexpr size_t kMaxLds = 160 * 1024;   // LDS per workgroup on gfx950
int  setup_ingest_attributes(const Dev& d);
void launch_gather_probe(hipStream_t s, const float* table, uint32_t slots, const uint32_t* idx, uint32_t n_groups,
                         uint32_t per, float* out);
int  setup_embed_attributes(const Dev& d);
int  layer_tiles_fit(const Dev& d, uint32_t nz);   // the layer kernel's LDS tiles with nz slots of z = [phi | raw edge row]
int  setup_memory_attributes(const Dev& d);

}  // namespace stgn
