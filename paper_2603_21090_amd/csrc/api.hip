// extern "C" boundary and host orchestration: argument checks, workspace layout, parameter
// packing, launch order of one incremental step.  No arithmetic of the method runs here.
#include <cmath>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

#include "stgn_internal.h"
#include "mfma16.h"

using namespace stgn;

namespace {

const char* const kClassNames[KC_COUNT] = {"stage_sort", "memory_update", "apply", "plan", "expand", "compact",
                                           "layer", "gather_rows", "noop", "project", "predict", "bucket_rows"};

std::string g_create_error;

// Scratch of the entry point that allocates nothing (stgn_predict_batch_static): the root list, the
// roots' query times and their final-layer rows live in this array instead of the caller's workspace.
// Every device the library runs on holds its own copy at its own address; the name below is only a
// host-side handle, the address kernels may use is looked up once per device (static_scratch()).
constexpr size_t kStaticScratchBytes = STGN_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};

// address of the current device's copy of `scratch`; resolved once per device, with that device current
hipError_t static_scratch(int dev, void** out) {
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

struct TimedLaunch { int cls; hipEvent_t a, b; };

}  // namespace

struct stgn_ctx {
  stgn_config cfg;
  Dev d;
  hipStream_t stream = nullptr;
  // A batch's front part (staging, placement, memory update and, for small flag arrays, the propagation
  // hops) can run on a second stream beside the previous batch's main part.  The staging kernel needs only
  // the batch and writes the batch's own state set (held kSets times): it runs a batch ahead.  The rest
  // reads the degrees, memory, rings and logs the previous apply step left and waits for it (ev_apply[],
  // recorded on `stream`); nothing in the previous batch's main part writes what the front part reads or
  // reads what it writes.  The batch's own apply step on `stream` waits for the front part (ev_front,
  // recorded on `front`).  Only batches with device inputs that find `stream` busy take this path; calls
  // that ask for per-stage statistics, calls with host inputs, and all calls while per-kernel timing is
  // on, run everything on `stream`.
  hipStream_t front = nullptr;
  hipEvent_t ev_apply[kSets] = {}, ev_front = nullptr;   // ev_apply cycles with the batches' state sets
  bool recorded[kSets] = {};        // ev_apply of that set has been recorded
  bool prev_on_front = false;       // the previous batch's front part ran on `front`
  int set = 0;                      // state set (scratch lists, batch fields, counters, work items, apply event) of the next batch
  int parity = 0;                   // staging block and dirty-flag array of the next batch
  int last_par = 0;                 // state set of the batch enqueued last
  bool idle = true;                 // nothing was enqueued since the library last synchronised `stream`
  bool have_predictor = false;      // stgn_set_predictor was called
  unsigned char* static_scratch = nullptr;   // this device's copy of the static scratch array
  std::string err;
  uint64_t host_edges = 0;          // upper bound of edges enqueued so far
  bool host_t_known = true;         // host knows the last ingested timestamp
  // Per hop: the last batch whose statistics the host has seen preferred the pull direction.  Such a
  // hop is enqueued without its plan kernel and told to pull; a stale hint costs speed, never correctness.
  bool pull_hint[STGN_MAX_LAYERS + 1] = {};
  bool any_edges = false;
  double host_t_last = 0.0;
  // pinned staging for host inputs, double buffered
  char* pin[2] = {nullptr, nullptr};
  hipEvent_t pin_ev[2] = {nullptr, nullptr};
  bool pin_used[2] = {false, false};
  size_t pin_bytes = 0;
  int pin_next = 0;
  Ctrl* ctrl_host = nullptr;        // pinned read-back of the control block
  hipEvent_t stage_ev[7] = {};
  // optional per-kernel timing
  bool timing = false;
  std::vector<TimedLaunch> pending;
  std::vector<hipEvent_t> free_events;
  double k_usec[KC_COUNT] = {};
  uint64_t k_launches[KC_COUNT] = {};
};

namespace {

int fail(stgn_ctx* c, int code, const std::string& msg) {
  if (c) c->err = msg; else g_create_error = msg;
  return code;
}

#define HIPCHK(ctx, call)                                                                      \
  do {                                                                                         \
    hipError_t e_ = (call);                                                                    \
    if (e_ != hipSuccess)                                                                      \
      return fail(ctx, STGN_E_DEVICE, std::string(#call) + ": " + hipGetErrorString(e_));      \
  } while (0)

uint32_t row_ld(uint32_t width) { return width ? round_up(width, kSlot) : 0; }   // whole 64-float slots: gathers never need a mask

struct Bump {
  char* base;
  size_t off = 0;
  template <class T>
  T* take(size_t count) {
    off = (off + 255) & ~(size_t)255;
    T* p = base ? reinterpret_cast<T*>(base + off) : nullptr;
    off += count * sizeof(T);
    return p;
  }
};

int check_config(const stgn_config* c, std::string* why) {
  auto bad = [&](const char* m) { *why = m; return STGN_E_INVALID_ARG; };
  if (!c) return bad("config is NULL");
  if (c->num_nodes == 0 || c->num_nodes > 0x7FFFFFFFu) return bad("num_nodes out of range");
  if (c->max_edges == 0 || c->max_edges >= (1ull << 31)) return bad("max_edges out of range");
  if (c->max_batch == 0 || c->max_batch > STGN_MAX_BATCH) return bad("max_batch out of range");
  if (c->layers == 0 || c->layers > STGN_MAX_LAYERS) return bad("layers out of range");
  if (c->k == 0 || c->k > 1024) return bad("k out of range");
  if (c->d_emb == 0 || c->d_emb > 512 || c->d_time == 0 || c->d_time > 512 || c->d_edge > 1024) return bad("dimension out of range");
  if (c->d_mem + c->d_node == 0 || c->d_mem + c->d_node > 512) return bad("layer-0 width (d_mem + d_node) out of range");
  if (c->d_mem && (c->d_msg == 0 || c->d_msg > 512)) return bad("d_msg out of range");
  if (c->heads == 0 || c->d_emb % c->heads != 0) return bad("heads must divide d_emb");
  if (c->aggregator > STGN_AGG_SUM) return bad("aggregator must be STGN_AGG_LAST, STGN_AGG_MEAN or STGN_AGG_SUM");
  if (c->delta_mode > 1) return bad("delta_mode must be 0 or 1");
  if (c->delta_mode && !(c->drift_gamma > 0.0 && c->drift_gamma <= 1.0)) return bad("drift_gamma must lie in (0, 1]");
  if (!attn_supported(c->d_emb, c->d_time, c->heads))
    return bad("unsupported attention shape: heads in {1,2,4}, d_time <= 128, and heads * ceil(d_emb / heads / 64) <= 4 "
               "(every head takes whole 64-float slots of a cached key row)");
  return STGN_OK;
}

// Group-major packing of a [K x N] weight matrix for 16x16x4 matrix instructions (mfma16.h): for
// column tile n = j / 16 and group g = k / 16 a block of 64 lanes x 4 floats, lane (i, col) =
// ((k % 16) / 4, j % 16) holding the four k-steps u = k % 4 side by side; K zero padded to whole
// chunks of four groups.
size_t tiled_size(uint32_t K, uint32_t N) {
  return (size_t)((N + 15) / 16) * groups_of(K) * kGrpFloats;
}
void put_tiled(std::vector<float>& dst, uint32_t K, uint32_t k, uint32_t j, double v) {
  const size_t block = (size_t)(j / 16) * groups_of(K) + k / kGrpK;
  dst[block * kGrpFloats + (((k % kGrpK) / 4) * 16 + j % 16) * 4 + k % 4] = (float)v;
}

// Host inputs travel as one block: src at 0, dst at 4 B, ts at 8 B, edge features at 16 B per edge of the largest batch.
size_t stage_bytes(const stgn_config& c) { return (size_t)c.max_batch * (16 + (size_t)c.d_edge * sizeof(float)); }

// Lays the whole device state out in one workspace; base == nullptr only measures.
size_t layout(const stgn_config& c, char* base, Dev* d) {
  Bump b{base};
  const uint32_t N = c.num_nodes, B2 = 2 * c.max_batch;
  d->N = N; d->k = c.k; d->heads = c.heads; d->layers = c.layers;
  d->d_mem = c.d_mem; d->d_node = c.d_node; d->d0 = c.d_mem + c.d_node; d->d_edge = c.d_edge;
  d->d_time = c.d_time; d->d_emb = c.d_emb; d->d_msg = c.d_msg; d->dk = c.d_emb / c.heads;
  d->max_batch = c.max_batch; d->max_edges = c.max_edges;
  d->window = c.window > 0.0 ? c.window : (double)INFINITY;
  d->aggregator = c.aggregator;
  d->num_cu = 0;
  // adjacency blocks of 8, 16, 32, ... entries: capacity after b blocks is 8 (2^b - 1)
  uint32_t maxb = 1;
  while (8ull * ((1ull << maxb) - 1) < 2 * c.max_edges) ++maxb;
  d->maxb = maxb;
  const uint64_t active = std::min<uint64_t>(N, 2 * c.max_edges);
  d->pool_cap_units = active + (4 * c.max_edges + kMinBlock - 1) / kMinBlock + 1;   // sum(2 deg + 8) / 8

  d->H[0].ld = row_ld(d->d0);
  d->H[0].base = b.take<float>((size_t)N * d->H[0].ld);
  for (uint32_t l = 1; l <= c.layers; ++l) {
    d->H[l].ld = row_ld(c.d_emb);
    d->H[l].base = b.take<float>((size_t)N * d->H[l].ld);
  }
  d->t_last = b.take<double>(N);
  d->deg = b.take<uint32_t>(N);
  d->ring = b.take<RingEntry>((size_t)N * c.k);
  d->ring_nbr = b.take<uint32_t>((size_t)N * c.k);
  d->pool_nt = b.take<uint2>(d->pool_cap_units * kMinBlock);
  d->pool_eid = b.take<uint32_t>(d->pool_cap_units * kMinBlock);
  d->blk = b.take<uint32_t>((size_t)N * maxb);
  d->sh = (d->dk + kSlot - 1) / kSlot;
  if (d->sh == 3) d->sh = 4;                                  // kernel variants exist for 1, 2 and 4 slots per head
  d->ks = c.heads * d->sh;
  d->nt = (c.d_time + kSlot - 1) / kSlot;
  // edge features of at most one slot stay raw rows (stgn_internal.h); the delta mode caches per-entry values
  // that hold the edge part, and keeps the projected edge rows
  d->es = c.d_edge && c.d_edge <= kSlot && !c.delta_mode ? 1u : 0u;
  if (d->es && !layer_tiles_fit(*d, d->nt + 1)) d->es = 0;   // (shapes whose tiles fill the LDS as they are)
  d->nz = d->nt + d->es;
  d->ld_kv = 2 * kSlot * d->ks;
  float* raw_rows = d->es ? b.take<float>((size_t)c.max_edges * kSlot) : nullptr;
  for (uint32_t l = 0; l < c.layers; ++l) {
    d->KV[l].ld = d->ld_kv;
    d->KV[l].base = b.take<float>((size_t)N * d->ld_kv);
    if (d->es) { d->KVE[l].ld = kSlot; d->KVE[l].base = raw_rows; continue; }
    d->KVE[l].ld = c.d_edge ? d->ld_kv : 0;                   // without edge features every edge reads one zero row
    d->KVE[l].base = b.take<float>((size_t)(c.d_edge ? c.max_edges : 1) * d->ld_kv);
  }
  d->ctrl = b.take<Ctrl>(1);
  // staging for host inputs: two blocks (batches alternate), each laid out like the pinned host block
  // [src | dst | ts | efeat] so that one copy moves a batch
  for (int i = 0; i < 2; ++i) d->stage[i] = b.take<char>(stage_bytes(c));
  for (Dev::Scratch& s : d->scr) {
    s.D = b.take<uint32_t>(B2);
    s.seg_start = b.take<uint32_t>(B2 + 1);
    s.last_slot = b.take<uint32_t>(B2);
    s.deg_new = b.take<uint32_t>(B2);
    s.slot_pos = b.take<uint32_t>(B2);
    s.slot_d = b.take<uint32_t>(B2);
    s.slot_sorted = b.take<uint32_t>(B2);
    s.mem_new = b.take<float>((size_t)B2 * c.d_mem);
  }
  *d = bind_batch(*d, 0, 0);
  d->mark_set[0] = b.take<uint8_t>(mark_bytes(N));
  d->mark_set[1] = compact_in_one(*d) ? b.take<uint8_t>(mark_bytes(N)) : d->mark_set[0];
  d->mark = d->mark_set[0];
  d->mark_other = d->mark_set[1];
  for (int i = 0; i < kSets; ++i) d->stripes_set[i] = b.take<uint64_t>((size_t)kStripedCounters * kStripes * kStripeWords);
  d->stripes = d->stripes_set[0];
  d->gathered_slots = b.take<uint64_t>(kStatSlots);
  d->items_cap = (uint64_t)N + 2 * c.max_edges / kLogChunk + 1024;
  for (int i = 0; i < kSets; ++i) d->items_set[i] = b.take<uint64_t>(d->items_cap);
  d->items = d->items_set[0];
  d->blocksum = b.take<uint32_t>((size_t)(c.layers + 1) * (mark_bytes(N) / kMarkPad + 2));
  d->A = b.take<uint32_t>(N);
  d->n_lists = 0;
  for (uint32_t l = 0; l < c.layers; ++l) {
    d->thr[l] = c.d_mem ? l + 2 : l + 1;                      // flags are 1 (endpoint) and h + 2 (hop h)
    if (d->thr[l] >= c.layers + 1) { d->R[l] = d->A; d->thr[l] = 0xFFu; }
    else { d->R[l] = b.take<uint32_t>(N); ++d->n_lists; }
  }
  // row lists regrouped by entry count: worth a launch once a layer has thousands of tiles
  d->bucketed = N >= 32768u && c.k <= 64u ? 1u : 0u;          // (the regrouping kernel has bins for up to 64 entries)
  // query cache: shapes whose tiles are staged a tile ahead (layer_kernel.h: two staged items per thread)
  // Memoryless models: every layer (the first layer's inputs never change and layer l's only within l - 1 hops
  // of an endpoint, so nearly every listed row reads its query back; config 5: layer launch 9 % shorter).  With
  // a memory only the first layer, whose inputs change for the batch's endpoints alone: at the later layers the
  // endpoints' first hop projects again, most of the affected set on graphs with hubs, and storing those
  // queries costs what the other rows save (measured with every layer cached: config 3 4 % slower).
  d->qcache = d->bucketed && !c.delta_mode && 16u * c.k <= 512u &&
              4u * round_up(std::max(d->d0, c.d_emb), 16u) <= 512u ? 1u : 0u;
  d->ld_qc = kSlot * (d->ks + c.heads * d->nz);
  for (uint32_t l = 0; l < STGN_MAX_LAYERS; ++l) {
    if (l >= c.layers || !d->bucketed) d->RS[l] = nullptr;
    else if (l && !d->qcache && d->thr[l] == 0xFFu && d->thr[l - 1] == 0xFFu) d->RS[l] = d->RS[l - 1];   // both walk A (pointers are null while measuring)
    else d->RS[l] = b.take<uint32_t>(N);
    const bool qc = d->qcache && l < c.layers && (c.d_mem == 0 || l == 0);
    d->QC[l] = qc ? b.take<float>((size_t)N * d->ld_qc) : nullptr;
    d->tile_clean[l] = qc ? b.take<uint8_t>(round_up(N / 16u + 1u, 256u)) : nullptr;
  }
  // delta mode: attention cache per layer, the kept flags, the drift estimator
  d->delta = c.delta_mode;
  d->gamma = (float)c.drift_gamma;
  for (uint32_t l = 0; l < STGN_MAX_LAYERS; ++l) {
    const bool on = c.delta_mode && l < c.layers;
    d->ac_S[l] = on ? b.take<float>((size_t)N * kSlot * d->ks) : nullptr;
    d->ac_P[l] = on ? b.take<float>((size_t)N * kSlot * d->nt * c.heads) : nullptr;
    d->ac_ZM[l] = on ? b.take<float>((size_t)N * 2 * c.heads) : nullptr;
    d->ac_W[l] = on ? b.take<float>((size_t)N * c.k * 2 * c.heads) : nullptr;
    d->ac_V[l] = on ? b.take<float>((size_t)N * c.k * kSlot * d->ks) : nullptr;
  }
  d->flags_kept = c.delta_mode || d->qcache ? b.take<uint8_t>(mark_bytes(N)) : nullptr;
  d->drift = c.delta_mode ? b.take<DriftCtl>(1) : nullptr;
  d->dsum = c.delta_mode ? b.take<float>(N) : nullptr;
  d->dlast = c.delta_mode ? b.take<uint32_t>(N) : nullptr;
  d->dseen = c.delta_mode ? b.take<uint8_t>(N) : nullptr;
  d->dlist = c.delta_mode ? b.take<uint32_t>(N) : nullptr;
  for (uint32_t l = 0; l < c.layers; ++l) d->L[l].d_in = l == 0 ? d->d0 : c.d_emb;
  d->pred_rows = b.take<uint32_t>(B2);
  d->pred_tq = b.take<double>(B2);
  d->pred_out = b.take<float>((size_t)B2 * c.d_emb);
  d->pred_src = b.take<uint32_t>(c.max_batch);
  d->pred_dst = b.take<uint32_t>(c.max_batch);
  d->pred_ts = b.take<double>(c.max_batch);
  d->pred_scores = b.take<float>(c.max_batch);
  d->pred_w = b.take<float>(2 * c.d_emb + 1);
  d->q_cap = 65536;
  d->qnodes = b.take<uint32_t>(d->q_cap);
  d->qout = b.take<float>((size_t)d->q_cap * std::max(d->d0, c.d_emb));
  // parameters
  d->om_rev = b.take<double>(c.d_time);
  d->ph_rev = b.take<double>(c.d_time);
  if (c.d_mem) {
    d->Kmsg = 2 * c.d_mem + c.d_edge + c.d_time;
    d->Wmsg = b.take<float>(tiled_size(d->Kmsg, c.d_msg));
    d->bmsg = b.take<float>(c.d_msg);
    d->Wzr = b.take<float>(tiled_size(c.d_msg, 2 * round_up(c.d_mem, 16)));
    d->Uzr = b.take<float>(tiled_size(c.d_mem, 2 * round_up(c.d_mem, 16)));
    d->Wh = b.take<float>(tiled_size(c.d_msg, c.d_mem));
    d->Uh = b.take<float>(tiled_size(c.d_mem, c.d_mem));
    d->bz = b.take<float>(c.d_mem);
    d->br = b.take<float>(c.d_mem);
    d->bh = b.take<float>(c.d_mem);
  } else {
    d->Kmsg = 0;
    d->Wmsg = d->bmsg = d->Wzr = d->Uzr = d->Wh = d->Uh = d->bz = d->br = d->bh = nullptr;
  }
  for (uint32_t l = 0; l < c.layers; ++l) {
    LayerDev& L = d->L[l];
    L.WQn = b.take<float>(tiled_size(L.d_in, c.d_emb));
    L.cQ = b.take<float>(c.d_emb);
    L.WKT = b.take<float>(tiled_size(kSlot * d->sh, c.heads * kSlot * d->nz));
    L.WV = b.take<float>(tiled_size(kSlot * d->nz, c.heads * round_up(d->dk, 16)));
    L.WO = b.take<float>(tiled_size(kSlot * d->ks, c.d_emb));
    L.bO = b.take<float>(c.d_emb);
    L.WKVn = b.take<float>(tiled_size(L.d_in, d->ld_kv));
    L.WKVe = c.d_edge && !d->es ? b.take<float>(tiled_size(c.d_edge, d->ld_kv)) : nullptr;
  }
  return (b.off + 255) & ~(size_t)255;
}

template <class T>
int upload(stgn_ctx* ctx, const T* dst, const std::vector<T>& v) {
  if (v.empty()) return STGN_OK;
  HIPCHK(ctx, hipMemcpy(const_cast<T*>(dst), v.data(), v.size() * sizeof(T), hipMemcpyHostToDevice));
  return STGN_OK;
}

int pack_parameters(stgn_ctx* ctx, const stgn_weights* w) {
  const stgn_config& c = ctx->cfg;
  const Dev& d = ctx->d;
  const double two_pi = 6.283185307179586476925286766559;
  const double tscale = std::sqrt(1.0 / (double)c.d_time);
  std::vector<double> om(c.d_time), ph(c.d_time);
  for (uint32_t i = 0; i < c.d_time; ++i) { om[i] = (double)w->omega[i] / two_pi; ph[i] = (double)w->phase[i] / two_pi; }
  int rc;
  if ((rc = upload(ctx, d.om_rev, om))) return rc;
  if ((rc = upload(ctx, d.ph_rev, ph))) return rc;
  auto vec = [](const float* p, uint32_t n) { return std::vector<float>(p, p + n); };
  if (c.d_mem) {
    // memory weights feed 16x16x4 matrix instructions: group-major packing (see tiled_size); the
    // update and reset gates share one matrix, the reset gate's column tiles behind the update gate's
    const uint32_t npm = round_up(c.d_mem, 16);
    std::vector<float> Wm(tiled_size(d.Kmsg, c.d_msg), 0.0f);
    for (uint32_t i = 0; i < d.Kmsg; ++i) {
      const double rs = i >= 2 * c.d_mem + c.d_edge ? tscale : 1.0;             // phi carries sqrt(1/d_t)
      for (uint32_t col = 0; col < c.d_msg; ++col) put_tiled(Wm, d.Kmsg, i, col, (double)w->W_msg[(size_t)i * c.d_msg + col] * rs);
    }
    std::vector<float> Wzr(tiled_size(c.d_msg, 2 * npm), 0.0f), Uzr(tiled_size(c.d_mem, 2 * npm), 0.0f);
    std::vector<float> Wh(tiled_size(c.d_msg, c.d_mem), 0.0f), Uh(tiled_size(c.d_mem, c.d_mem), 0.0f);
    for (uint32_t col = 0; col < c.d_mem; ++col) {
      for (uint32_t i = 0; i < c.d_msg; ++i) {
        put_tiled(Wzr, c.d_msg, i, col, w->W_z[(size_t)i * c.d_mem + col]);
        put_tiled(Wzr, c.d_msg, i, npm + col, w->W_r[(size_t)i * c.d_mem + col]);
        put_tiled(Wh, c.d_msg, i, col, w->W_h[(size_t)i * c.d_mem + col]);
      }
      for (uint32_t i = 0; i < c.d_mem; ++i) {
        put_tiled(Uzr, c.d_mem, i, col, w->U_z[(size_t)i * c.d_mem + col]);
        put_tiled(Uzr, c.d_mem, i, npm + col, w->U_r[(size_t)i * c.d_mem + col]);
        put_tiled(Uh, c.d_mem, i, col, w->U_h[(size_t)i * c.d_mem + col]);
      }
    }
    if ((rc = upload(ctx, d.Wmsg, Wm)) || (rc = upload(ctx, d.bmsg, vec(w->b_msg, c.d_msg))) ||
        (rc = upload(ctx, d.Wzr, Wzr)) || (rc = upload(ctx, d.Uzr, Uzr)) || (rc = upload(ctx, d.Wh, Wh)) ||
        (rc = upload(ctx, d.Uh, Uh)) || (rc = upload(ctx, d.bz, vec(w->b_z, c.d_mem))) ||
        (rc = upload(ctx, d.br, vec(w->b_r, c.d_mem))) || (rc = upload(ctx, d.bh, vec(w->b_h, c.d_mem))))
      return rc;
  }
  // attention weights feed 16x16x4 matrix instructions: group-major packing (see tiled_size).
  // Row z of W_K / W_V belongs to the node block (z < d_in), the edge block or the time block of the
  // attention input; column h dk + cc to head h.  In a cached row and in the head-output tile head h
  // starts at float 64 sh h (padded-head layout).
  const uint32_t dk = d.dk, npk = round_up(dk, 16), hp = kSlot * d.sh, Ztp = kSlot * d.nz;
  const double inv_sqrt_dk = 1.0 / std::sqrt((double)dk);
  for (uint32_t l = 0; l < c.layers; ++l) {
    const LayerDev& L = d.L[l];
    const float *WQ = w->W_Q[l], *WK = w->W_K[l], *WV = w->W_V[l], *WOs = w->W_O[l];
    const uint32_t e0 = L.d_in, t0 = L.d_in + c.d_edge;       // first edge row, first time row
    // the query carries the 1 / sqrt(dk) of the scores
    std::vector<float> WQn(tiled_size(L.d_in, c.d_emb), 0.0f);
    for (uint32_t i = 0; i < L.d_in; ++i)
      for (uint32_t col = 0; col < c.d_emb; ++col)
        put_tiled(WQn, L.d_in, i, col, (double)WQ[(size_t)i * c.d_emb + col] * inv_sqrt_dk);
    std::vector<float> cQ(c.d_emb);
    for (uint32_t col = 0; col < c.d_emb; ++col) {
      double acc = 0.0;
      for (uint32_t i = 0; i < c.d_time; ++i)
        acc += tscale * std::cos((double)w->phase[i]) * (double)WQ[(size_t)(L.d_in + i) * c.d_emb + col];
      cQ[col] = (float)(acc * inv_sqrt_dk);
    }
    // time rows of W_K, head blocks transposed: K = column inside the head, columns = (head, index in z);
    // time rows of W_V, head blocks: K = index in z, columns = (head, column inside the head padded to 16).
    // z = [phi | f]: time index i at i, and with raw edge rows feature i at 64 nt + i.
    std::vector<float> WKT(tiled_size(hp, c.heads * Ztp), 0.0f);
    std::vector<float> WVp(tiled_size(Ztp, c.heads * npk), 0.0f);
    for (uint32_t h = 0; h < c.heads; ++h)
      for (uint32_t cc = 0; cc < dk; ++cc) {
        for (uint32_t i = 0; i < c.d_time; ++i) {
          put_tiled(WKT, hp, cc, h * Ztp + i, (double)WK[(size_t)(t0 + i) * c.d_emb + h * dk + cc] * tscale);
          put_tiled(WVp, Ztp, i, h * npk + cc, (double)WV[(size_t)(t0 + i) * c.d_emb + h * dk + cc] * tscale);
        }
        for (uint32_t i = 0; i < (d.es ? c.d_edge : 0u); ++i) {
          put_tiled(WKT, hp, cc, h * Ztp + kSlot * d.nt + i, WK[(size_t)(e0 + i) * c.d_emb + h * dk + cc]);
          put_tiled(WVp, Ztp, kSlot * d.nt + i, h * npk + cc, WV[(size_t)(e0 + i) * c.d_emb + h * dk + cc]);
        }
      }
    // W_O with its rows moved to the padded-head layout of the head outputs
    std::vector<float> WO(tiled_size(kSlot * d.ks, c.d_emb), 0.0f);
    for (uint32_t h = 0; h < c.heads; ++h)
      for (uint32_t cc = 0; cc < dk; ++cc)
        for (uint32_t col = 0; col < c.d_emb; ++col)
          put_tiled(WO, kSlot * d.ks, h * hp + cc, col, WOs[(size_t)(h * dk + cc) * c.d_emb + col]);
    // node and edge rows of [W_K | W_V] in the cached-row layout: keys in floats [0, 64 ks), values behind
    std::vector<float> WKVn(tiled_size(L.d_in, d.ld_kv), 0.0f);
    std::vector<float> WKVe(c.d_edge && !d.es ? tiled_size(c.d_edge, d.ld_kv) : 0, 0.0f);
    for (uint32_t h = 0; h < c.heads; ++h)
      for (uint32_t cc = 0; cc < dk; ++cc) {
        const uint32_t kc = h * hp + cc, vc = kSlot * d.ks + h * hp + cc;
        const size_t wc = (size_t)h * dk + cc;
        for (uint32_t i = 0; i < L.d_in; ++i) {
          put_tiled(WKVn, L.d_in, i, kc, WK[(size_t)i * c.d_emb + wc]);
          put_tiled(WKVn, L.d_in, i, vc, WV[(size_t)i * c.d_emb + wc]);
        }
        for (uint32_t i = 0; i < (d.es ? 0u : c.d_edge); ++i) {
          put_tiled(WKVe, c.d_edge, i, kc, WK[(size_t)(e0 + i) * c.d_emb + wc]);
          put_tiled(WKVe, c.d_edge, i, vc, WV[(size_t)(e0 + i) * c.d_emb + wc]);
        }
      }
    if ((rc = upload(ctx, L.WQn, WQn)) || (rc = upload(ctx, L.cQ, cQ)) || (rc = upload(ctx, L.WKT, WKT)) ||
        (rc = upload(ctx, L.WV, WVp)) || (rc = upload(ctx, L.WO, WO)) || (rc = upload(ctx, L.bO, vec(w->b_O[l], c.d_emb))) ||
        (rc = upload(ctx, L.WKVn, WKVn)) || (rc = upload(ctx, L.WKVe, WKVe)))
      return rc;
  }
  return STGN_OK;
}

// ---- optional per-kernel event timing
hipEvent_t get_event(stgn_ctx* ctx) {
  if (!ctx->free_events.empty()) { hipEvent_t e = ctx->free_events.back(); ctx->free_events.pop_back(); return e; }
  // timing-only events: no system-scope cache write-back / invalidate around the measured kernel
  hipEvent_t e = nullptr;
  if (hipEventCreateWithFlags(&e, hipEventDisableSystemFence) != hipSuccess) return nullptr;
  return e;
}

struct Scope {
  stgn_ctx* ctx; int cls; hipStream_t st; hipEvent_t a = nullptr, b = nullptr;
  Scope(stgn_ctx* c, int k, hipStream_t on = nullptr) : ctx(c), cls(k), st(on ? on : c->stream) {
    if (ctx->timing) { a = get_event(ctx); b = get_event(ctx); if (a) hipEventRecord(a, st); }
  }
  ~Scope() {
    if (ctx->timing && a && b) { hipEventRecord(b, st); ctx->pending.push_back({cls, a, b}); }
  }
};

void drain_timing(stgn_ctx* ctx) {
  for (const TimedLaunch& t : ctx->pending) {
    float ms = 0.0f;
    if (hipEventElapsedTime(&ms, t.a, t.b) == hipSuccess) { ctx->k_usec[t.cls] += 1000.0 * ms; ctx->k_launches[t.cls] += 1; }
    ctx->free_events.push_back(t.a);
    ctx->free_events.push_back(t.b);
  }
  ctx->pending.clear();
}

// every layer over all rows (initial state, full rebuild) or over the per-layer lists of the last batch
void run_layers(stgn_ctx* ctx, const Dev& d, bool all_rows) {
  if (all_rows) { Scope s(ctx, KC_PROJECT); launch_project_nodes(d, ctx->stream); }   // cached keys|values of the layer-0 rows
  if (d.bucketed) { Scope s(ctx, KC_BUCKET); launch_bucket_rows(d, ctx->stream, all_rows); }
  for (uint32_t l = 0; l < d.layers; ++l) {
    Scope s(ctx, KC_LAYER);
    if (all_rows) launch_layer(d, ctx->stream, l, d.bucketed ? d.RS[0] : nullptr, nullptr, d.N);
    else launch_layer(d, ctx->stream, l, d.bucketed ? d.RS[l] : d.R[l], &d.bc->nR[l], d.N, /*force_exact=*/false);
  }
}

int read_ctrl(stgn_ctx* ctx) {
  HIPCHK(ctx, hipMemcpyAsync(ctx->ctrl_host, ctx->d.ctrl, sizeof(Ctrl), hipMemcpyDeviceToHost, ctx->stream));
  HIPCHK(ctx, hipStreamSynchronize(ctx->stream));
  ctx->idle = true;
  return STGN_OK;
}

// synchronise, fetch the control block, report and clear a pending device-side error
int sync_and_poll(stgn_ctx* ctx) {
  int rc = read_ctrl(ctx);
  if (rc) return rc;
  if (ctx->timing) drain_timing(ctx);
  const BatchCtl& lb = ctx->ctrl_host->b[ctx->last_par];          // the batch enqueued last
  if (!lb.skip && lb.n_edges)
    for (uint32_t h = 0; h < ctx->cfg.layers; ++h) ctx->pull_hint[h] = (lb.pulled[h] & 2u) != 0;
  const int code = ctx->ctrl_host->err_code;
  if (code != 0) {
    const int32_t zero = 0;
    HIPCHK(ctx, hipMemcpy(&ctx->d.ctrl->err_code, &zero, sizeof(zero), hipMemcpyHostToDevice));
    char buf[128];
    snprintf(buf, sizeof buf, "batch %u rejected on the device with code %d; it was skipped as a whole",
             ctx->ctrl_host->err_batch, code);
    ctx->err = buf;
    ctx->host_t_known = false;
    return code;
  }
  return STGN_OK;
}

}  // namespace

extern "C" {

const char* stgn_version(void) { return "streamtgn-gfx950 0.1"; }

int stgn_probe_gather(const float* table, uint64_t n_rows, uint32_t row_bytes, const uint32_t* idx, uint32_t n_groups,
                      uint32_t per_group, float* out, void* hip_stream) {
  if (!table || !idx || !out || !n_rows || !n_groups || !per_group || n_groups > (1u << 27)) return STGN_E_INVALID_ARG;
  if (row_bytes != 256 && row_bytes != 1024) return STGN_E_INVALID_ARG;
  launch_gather_probe((hipStream_t)hip_stream, table, row_bytes / 256, idx, n_groups, per_group, out);
  return hipGetLastError() == hipSuccess ? STGN_OK : STGN_E_DEVICE;
}

const char* stgn_last_error(const stgn_ctx* ctx) { return ctx ? ctx->err.c_str() : g_create_error.c_str(); }

int stgn_query_workspace(const stgn_config* cfg, size_t* device_bytes) {
  std::string why;
  int rc = check_config(cfg, &why);
  if (rc) return fail(nullptr, rc, why);
  if (!device_bytes) return fail(nullptr, STGN_E_INVALID_ARG, "device_bytes is NULL");
  Dev tmp;
  memset(&tmp, 0, sizeof tmp);
  *device_bytes = layout(*cfg, nullptr, &tmp);
  return STGN_OK;
}

int stgn_create(const stgn_config* cfg, const stgn_weights* w, const float* node_feat, void* device_workspace,
                size_t device_bytes, void* hip_stream, stgn_ctx** out) {
  std::string why;
  int rc = check_config(cfg, &why);
  if (rc) return fail(nullptr, rc, why);
  if (!w || !out) return fail(nullptr, STGN_E_INVALID_ARG, "weights or out pointer is NULL");
  if (!w->omega || !w->phase || !w->W_Q || !w->W_K || !w->W_V || !w->W_O || !w->b_O)
    return fail(nullptr, STGN_E_INVALID_ARG, "a time-encoding or attention parameter pointer is NULL");
  for (uint32_t l = 0; l < cfg->layers; ++l)
    if (!w->W_Q[l] || !w->W_K[l] || !w->W_V[l] || !w->W_O[l] || !w->b_O[l])
      return fail(nullptr, STGN_E_INVALID_ARG, "an attention layer parameter pointer is NULL");
  if (cfg->d_mem && (!w->W_msg || !w->b_msg || !w->W_z || !w->U_z || !w->b_z || !w->W_r || !w->U_r || !w->b_r ||
                     !w->W_h || !w->U_h || !w->b_h))
    return fail(nullptr, STGN_E_INVALID_ARG, "a message/GRU parameter pointer is NULL");
  Dev tmp;
  memset(&tmp, 0, sizeof tmp);
  const size_t need = layout(*cfg, nullptr, &tmp);
  if (!device_workspace || ((uintptr_t)device_workspace & 255) || device_bytes < need)
    return fail(nullptr, STGN_E_WORKSPACE, "workspace is NULL, not 256-byte aligned or smaller than stgn_query_workspace reports");
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || ndev == 0) return fail(nullptr, STGN_E_DEVICE, "no HIP device");
  int dev = 0;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess)
    return fail(nullptr, STGN_E_DEVICE, "cannot query the current device");
  if (strncmp(prop.gcnArchName, "gfx950", 6) != 0)
    return fail(nullptr, STGN_E_DEVICE, std::string("built for gfx950, current device is ") + prop.gcnArchName);

  void* sscratch = nullptr;
  {
    const hipError_t e = static_scratch(dev, &sscratch);
    if (e != hipSuccess) return fail(nullptr, STGN_E_DEVICE, std::string("static scratch lookup: ") + hipGetErrorString(e));
  }
  stgn_ctx* ctx = new stgn_ctx();
  ctx->cfg = *cfg;
  ctx->static_scratch = static_cast<unsigned char*>(sscratch);
  memset(&ctx->d, 0, sizeof(Dev));
  layout(*cfg, (char*)device_workspace, &ctx->d);
  ctx->stream = (hipStream_t)hip_stream;
  auto bail = [&](int code) { g_create_error = ctx->err; stgn_destroy(ctx); return code; };

  ctx->pin_bytes = stage_bytes(*cfg);
  for (int i = 0; i < 2; ++i) {
    if (hipHostMalloc((void**)&ctx->pin[i], ctx->pin_bytes, hipHostMallocDefault) != hipSuccess ||
        hipEventCreateWithFlags(&ctx->pin_ev[i], hipEventDisableTiming) != hipSuccess) {
      ctx->err = "pinned staging allocation failed";
      return bail(STGN_E_DEVICE);
    }
  }
  if (hipHostMalloc((void**)&ctx->ctrl_host, sizeof(Ctrl), hipHostMallocDefault) != hipSuccess) {
    ctx->err = "pinned control block allocation failed";
    return bail(STGN_E_DEVICE);
  }
  for (auto& e : ctx->stage_ev)
    if (hipEventCreate(&e) != hipSuccess) { ctx->err = "event creation failed"; return bail(STGN_E_DEVICE); }
  if (hipStreamCreateWithFlags(&ctx->front, hipStreamNonBlocking) != hipSuccess ||
      hipEventCreateWithFlags(&ctx->ev_apply[0], hipEventDisableTiming) != hipSuccess ||
      hipEventCreateWithFlags(&ctx->ev_apply[1], hipEventDisableTiming) != hipSuccess ||
      hipEventCreateWithFlags(&ctx->ev_apply[2], hipEventDisableTiming) != hipSuccess ||
      hipEventCreateWithFlags(&ctx->ev_front, hipEventDisableTiming) != hipSuccess) {
    ctx->err = "second stream or its events could not be created";
    return bail(STGN_E_DEVICE);
  }
  {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0)
      ctx->d.num_cu = (uint32_t)cus;
  }
  if (setup_ingest_attributes(ctx->d) || setup_embed_attributes(ctx->d) || setup_memory_attributes(ctx->d)) {
    ctx->err = "a kernel needs more LDS than one gfx950 workgroup has for these dimensions";
    return bail(STGN_E_INVALID_ARG);
  }
  if ((rc = pack_parameters(ctx, w))) return bail(rc);
  launch_init_state(ctx->d, ctx->stream);
  for (uint32_t l = 1; l <= cfg->layers; ++l)     // padding columns of the layer caches are read by 16-byte gathers
    launch_zero(ctx->d.H[l].base, (size_t)cfg->num_nodes * ctx->d.H[l].ld, ctx->stream);
  if (hipStreamSynchronize(ctx->stream) != hipSuccess) { ctx->err = "state initialisation failed"; return bail(STGN_E_DEVICE); }
  if (node_feat && cfg->d_node) {
    hipError_t e = hipMemcpy2D(ctx->d.H[0].base + cfg->d_mem, (size_t)ctx->d.H[0].ld * sizeof(float), node_feat,
                               (size_t)cfg->d_node * sizeof(float), (size_t)cfg->d_node * sizeof(float), cfg->num_nodes,
                               hipMemcpyHostToDevice);
    if (e != hipSuccess) { ctx->err = std::string("node feature upload: ") + hipGetErrorString(e); return bail(STGN_E_DEVICE); }
  }
  // ring places past a row's entry count read edge 0: its rows must be finite before the first edge arrives
  for (uint32_t l = 0; l < cfg->layers; ++l) launch_zero(ctx->d.KVE[l].base, ctx->d.es ? kSlot : ctx->d.ld_kv, ctx->stream);
  if (ctx->d.flags_kept) launch_zero(reinterpret_cast<float*>(ctx->d.flags_kept), mark_bytes(cfg->num_nodes) / sizeof(float), ctx->stream);
  if (cfg->delta_mode) {            // no flag set, estimator at rest
    launch_zero(reinterpret_cast<float*>(ctx->d.drift), sizeof(DriftCtl) / sizeof(float), ctx->stream);
    launch_drift_reset(ctx->d, ctx->stream);
  }
  run_layers(ctx, ctx->d, true);    // every cache row = empty-neighbourhood embedding
  if (cfg->delta_mode) launch_drift_reset(ctx->d, ctx->stream);
  hipError_t e = hipStreamSynchronize(ctx->stream);
  if (e == hipSuccess) e = hipGetLastError();
  if (e != hipSuccess) { ctx->err = std::string("initial rebuild: ") + hipGetErrorString(e); return bail(STGN_E_DEVICE); }
  *out = ctx;
  return STGN_OK;
}

void stgn_destroy(stgn_ctx* ctx) {
  if (!ctx) return;
  if (ctx->front) hipStreamSynchronize(ctx->front);
  if (ctx->stream || ctx->ctrl_host) hipStreamSynchronize(ctx->stream);
  if (ctx->front) hipStreamDestroy(ctx->front);
  for (auto& e : ctx->ev_apply) if (e) hipEventDestroy(e);
  if (ctx->ev_front) hipEventDestroy(ctx->ev_front);
  for (int i = 0; i < 2; ++i) {
    if (ctx->pin[i]) hipHostFree(ctx->pin[i]);
    if (ctx->pin_ev[i]) hipEventDestroy(ctx->pin_ev[i]);
  }
  if (ctx->ctrl_host) hipHostFree(ctx->ctrl_host);
  for (auto& e : ctx->stage_ev) if (e) hipEventDestroy(e);
  for (const TimedLaunch& t : ctx->pending) { hipEventDestroy(t.a); hipEventDestroy(t.b); }
  for (hipEvent_t e : ctx->free_events) hipEventDestroy(e);
  delete ctx;
}

int stgn_ingest_batch(stgn_ctx* ctx, uint32_t n, const uint32_t* src, const uint32_t* dst, const double* ts,
                      const float* efeat, int inputs_on_device, stgn_batch_stats* stats) {
  if (!ctx) return STGN_E_INVALID_ARG;
  const stgn_config& c = ctx->cfg;
  const int par = ctx->parity;                 // the batch's staging block and dirty-flag array
  const int set = ctx->set;                    // ... and its state set
  const int prev = (set + kSets - 1) % kSets, prev2 = (set + kSets - 2) % kSets;   // the state sets of the two batches before
  const Dev d = bind_batch(ctx->d, set, par);
  if (n > c.max_batch) return fail(ctx, STGN_E_BATCH_TOO_LARGE, "batch larger than max_batch");
  if (n && (!src || !dst || !ts || (c.d_edge && !efeat))) return fail(ctx, STGN_E_INVALID_ARG, "NULL batch array");
  if (ctx->host_edges + n > c.max_edges) return fail(ctx, STGN_E_EDGE_CAPACITY, "max_edges exceeded");

  const uint32_t *dsrc = src, *ddst = dst;
  const double* dts = ts;
  const float* def = efeat;
  // stream of the front part (see stgn_ctx::front)
  // Only worth it, and only used, when there is something to overlap with (work was enqueued on
  // hip_stream since the library last synchronised it).  Host inputs are copied on the same stream,
  // ahead of the staging kernel: like it, the copy runs a batch ahead.
  const bool overlapped = stats == nullptr && !ctx->timing && !ctx->idle;
  ctx->idle = false;
  hipStream_t sf = overlapped ? ctx->front : ctx->stream;
  const bool prev_on_front = ctx->prev_on_front;
  // The batch's state set and staging block were last used three / two batches ago: whatever the front
  // part writes first is ordered behind the apply step of the batch before the previous one, whose
  // stream position is behind everything that used them.  (When the previous batch's front part ran
  // on `front` too, its own wait for that event already stands in front in stream order.)
  // A previous batch whose front part ran on `stream` has its staging kernel there, possibly still
  // queued behind work of the caller's: both staging kernels update the running edge count, the stream
  // time and the batch counter, so this one must not overtake it.  Its apply step follows it in stream
  // order and is also behind the batch before it, so that one event orders both (once per
  // synchronising call; the steady state never takes this branch).
  if (overlapped && !prev_on_front) {
    if (ctx->recorded[prev]) HIPCHK(ctx, hipStreamWaitEvent(sf, ctx->ev_apply[prev], 0));
    else if (ctx->recorded[prev2]) HIPCHK(ctx, hipStreamWaitEvent(sf, ctx->ev_apply[prev2], 0));
  }
  if (!inputs_on_device) {
    // host-side validation: nothing is enqueued for a bad batch
    double t_before = (ctx->any_edges && ctx->host_t_known) ? ctx->host_t_last : -INFINITY;
    for (uint32_t i = 0; i < n; ++i) {
      if (src[i] >= c.num_nodes || dst[i] >= c.num_nodes) return fail(ctx, STGN_E_NODE_OUT_OF_RANGE, "endpoint id >= num_nodes");
      if (src[i] == dst[i]) return fail(ctx, STGN_E_SELF_LOOP, "self loop");
      if (!(ts[i] >= t_before)) return fail(ctx, STGN_E_TIME_ORDER, "timestamps must be non-decreasing");
      t_before = ts[i];
    }
    if (n) {
      const int pb = ctx->pin_next;
      ctx->pin_next ^= 1;
      if (ctx->pin_used[pb]) HIPCHK(ctx, hipEventSynchronize(ctx->pin_ev[pb]));
      char* p = ctx->pin[pb];
      const size_t o_dst = (size_t)c.max_batch * 4, o_ts = (size_t)c.max_batch * 8, o_ef = (size_t)c.max_batch * 16;
      memcpy(p, src, (size_t)n * 4);
      memcpy(p + o_dst, dst, (size_t)n * 4);
      memcpy(p + o_ts, ts, (size_t)n * 8);
      if (c.d_edge) memcpy(p + o_ef, efeat, (size_t)n * c.d_edge * 4);
      // one copy moves the batch
      HIPCHK(ctx, hipMemcpyAsync(d.stage[par], p, o_ef + (size_t)n * c.d_edge * 4, hipMemcpyHostToDevice, sf));
      HIPCHK(ctx, hipEventRecord(ctx->pin_ev[pb], sf));
      ctx->pin_used[pb] = true;
      ctx->host_t_last = ts[n - 1];
      ctx->host_t_known = true;
      ctx->any_edges = true;
    }
    char* st = d.stage[par];
    dsrc = reinterpret_cast<const uint32_t*>(st);
    ddst = reinterpret_cast<const uint32_t*>(st + (size_t)c.max_batch * 4);
    dts = reinterpret_cast<const double*>(st + (size_t)c.max_batch * 8);
    def = reinterpret_cast<const float*>(st + (size_t)c.max_batch * 16);
  } else if (n) {
    ctx->host_t_known = false;
    ctx->any_edges = true;
  }
  ctx->host_edges += n;
  ctx->parity ^= 1;                            // from here on the batch is enqueued
  ctx->set = (set + 1) % kSets;
  ctx->last_par = set;
  ctx->prev_on_front = overlapped;
  hipStream_t s = ctx->stream;
  // The staging kernel looks only at the batch and the running edge count and writes the batch's own
  // state set: it may run beside the previous batch's main part, a batch ahead of the rest of the front part.
  hipEvent_t* ev = stats ? ctx->stage_ev : nullptr;
  if (ev) hipEventRecord(ev[0], s);
  { Scope t(ctx, KC_SORT, sf); launch_stage_sort(d, sf, n, dsrc, ddst, dts); }
  // degrees and memory as the previous apply step left them
  if (overlapped && ctx->recorded[prev]) HIPCHK(ctx, hipStreamWaitEvent(sf, ctx->ev_apply[prev], 0));
  // (calls that ask for statistics keep the plain order, so that their stage times mean what they say)
  const uint32_t first_main_hop = !stats && !ctx->timing && compact_in_one(d) && (c.layers >= 2 || !overlapped) ? c.layers : 0u;
  // the front part's last kernel carries the event the apply step waits for
  hipEvent_t front_done = overlapped ? ctx->ev_front : nullptr;
  const int last_front = first_main_hop ? 2 : c.d_mem ? 1 : 0;          // hops / memory update / placement
  // (the placement rides in the memory update's launch when there is one)
  const bool place_in_memory = c.d_mem != 0;
  if (!place_in_memory) { Scope t(ctx, KC_SORT, sf); launch_place(d, sf, n, last_front == 0 ? front_done : nullptr); }
  if (ev) hipEventRecord(ev[1], s);
  if (c.d_mem) { Scope t(ctx, KC_MEMORY, sf); launch_memory_update(d, sf, dsrc, ddst, dts, def, place_in_memory, last_front == 1 ? front_done : nullptr); }
  if (ev) hipEventRecord(ev[2], s);
  // With two flag arrays the placement kernel has seeded the dirty flags, and the propagation hops may
  // run in the front part, ahead of the apply step: a node that is not an endpoint of the batch keeps
  // its ring, degree and log through the apply step and endpoints are dirty from the start, so a hop
  // sets the same flags before the apply step as after it.  They follow the memory update: that
  // kernel's few large workgroups need CUs of their own and find them while the previous batch's
  // first layer launch (fewer rows than the last) leaves some free, whereas the hops' small
  // workgroups fit beside the layer kernel's on any CU.  (Measured on C2, per batch: hops on the
  // caller's stream 112 us; first hop in front of the memory update 110; behind it 105; both hops
  // behind it 103; both in front of it 117.)  Only beside at least two layer launches: the single
  // launch of a one-layer model is shorter than the front part (C1: 82 instead of 72 us).
  for (uint32_t hop = 0; hop < first_main_hop; ++hop) {
    const bool planned = !ctx->pull_hint[hop];
    if (planned) { Scope t(ctx, KC_PLAN, sf); launch_plan(d, sf, hop); }
    { Scope t(ctx, KC_EXPAND, sf); launch_expand(d, sf, hop, planned, hop + 1 == first_main_hop ? front_done : nullptr); }
  }
  if (overlapped) HIPCHK(ctx, hipStreamWaitEvent(s, ctx->ev_front, 0));
  // the propagation is done: the compaction depends on the flags alone and shares the apply step's launch
  const bool fused_compaction = first_main_hop != 0;
  // ... and its own completion is the event the next batch's front part waits for
  { Scope t(ctx, KC_APPLY); launch_apply(d, s, dsrc, ddst, dts, def, fused_compaction, ctx->ev_apply[set]); }
  ctx->recorded[set] = true;
  if (ev) hipEventRecord(ev[3], s);
  for (uint32_t hop = first_main_hop; hop < c.layers; ++hop) {
    const bool planned = !ctx->pull_hint[hop];
    if (planned) { Scope t(ctx, KC_PLAN); launch_plan(d, s, hop); }
    { Scope t(ctx, KC_EXPAND); launch_expand(d, s, hop, planned); }
  }
  if (!fused_compaction) {
    { Scope t(ctx, KC_COMPACT); launch_compact(d, s, 0); }
    if (!compact_in_one(d)) { Scope t(ctx, KC_COMPACT); launch_compact(d, s, 1); }
  }
  if (ev) hipEventRecord(ev[4], s);
  run_layers(ctx, d, false);
  if (ctx->timing) { Scope t(ctx, KC_NOOP); launch_noop(s); }   // event-pair overhead, for calibration
  if (ev) hipEventRecord(ev[5], s);
  HIPCHK(ctx, hipGetLastError());

  if (stats) {
    int rc = sync_and_poll(ctx);
    const BatchCtl& h = ctx->ctrl_host->b[set];
    memset(stats, 0, sizeof *stats);
    stats->n_edges = h.n_edges;
    stats->n_direct = h.nD;
    stats->n_affected = h.nA;
    for (int i = 0; i <= STGN_MAX_LAYERS; ++i) stats->frontier[i] = h.n_front[i];
    stats->entries_scanned = h.scanned;
    stats->pull_hops = 0;
    stats->reserved = 0;
    for (uint32_t i = 0; i < ctx->cfg.layers; ++i) stats->pull_hops |= (h.pulled[i] & 1u) << i;
    for (int i = 0; i < 5; ++i) {
      float ms = 0.0f;
      hipEventElapsedTime(&ms, ev[i], ev[i + 1]);
      stats->us_stage[i] = 1000.0f * ms;
    }
    float ms = 0.0f;
    hipEventElapsedTime(&ms, ev[0], ev[5]);
    stats->us_stage[5] = 1000.0f * ms;
    return rc;
  }
  return STGN_OK;
}

int stgn_full_rebuild(stgn_ctx* ctx) {
  if (!ctx) return STGN_E_INVALID_ARG;
  ctx->idle = false;
  run_layers(ctx, ctx->d, true);
  if (ctx->cfg.delta_mode) launch_drift_reset(ctx->d, ctx->stream);   // every row is exact again
  HIPCHK(ctx, hipGetLastError());
  return STGN_OK;
}

int stgn_drift_status(stgn_ctx* ctx, double* global_drift, uint32_t* n_tracked, float* per_node) {
  if (!ctx) return STGN_E_INVALID_ARG;
  if (!ctx->cfg.delta_mode) return fail(ctx, STGN_E_INVALID_ARG, "the context was not created in delta mode");
  const Dev& d = ctx->d;
  if (per_node) launch_drift_values(d, ctx->stream, reinterpret_cast<float*>(d.dlist));
  DriftCtl h{};
  HIPCHK(ctx, hipMemcpyAsync(&h, d.drift, sizeof h, hipMemcpyDeviceToHost, ctx->stream));
  if (per_node)
    HIPCHK(ctx, hipMemcpyAsync(per_node, d.dlist, (size_t)d.N * sizeof(float), hipMemcpyDeviceToHost, ctx->stream));
  int rc = sync_and_poll(ctx);
  if (global_drift) *global_drift = h.count ? h.G / (double)h.count : 0.0;
  if (n_tracked) *n_tracked = h.count;
  return rc;
}

int stgn_maintain(stgn_ctx* ctx, double delta_max, double alpha, int* action, uint32_t* n_drift) {
  if (!ctx) return STGN_E_INVALID_ARG;
  if (!ctx->cfg.delta_mode) return fail(ctx, STGN_E_INVALID_ARG, "the context was not created in delta mode");
  const Dev& d = ctx->d;
  if (action) *action = STGN_MAINTAIN_NONE;
  if (n_drift) *n_drift = 0;
  DriftCtl h{};
  HIPCHK(ctx, hipMemcpyAsync(&h, d.drift, sizeof h, hipMemcpyDeviceToHost, ctx->stream));
  int rc = sync_and_poll(ctx);
  if (rc) return rc;
  const double global = h.count ? h.G / (double)h.count : 0.0;
  if (!(global > delta_max)) return STGN_OK;
  ctx->idle = false;
  const uint32_t zero = 0;
  HIPCHK(ctx, hipMemcpyAsync(&d.drift->n_list, &zero, sizeof zero, hipMemcpyHostToDevice, ctx->stream));
  launch_drift_list(d, ctx->stream, (float)delta_max);
  uint32_t n_list = 0;
  HIPCHK(ctx, hipMemcpyAsync(&n_list, &d.drift->n_list, sizeof n_list, hipMemcpyDeviceToHost, ctx->stream));
  HIPCHK(ctx, hipStreamSynchronize(ctx->stream));
  if (n_drift) *n_drift = n_list;
  if ((double)n_list < alpha * (double)d.N) {
    // partial rebuild: the drifted rows, layer by layer, exactly (the other rows keep what they hold)
    for (uint32_t l = 0; l < d.layers; ++l) {
      Scope s(ctx, KC_LAYER);
      launch_layer(d, ctx->stream, l, d.dlist, &d.drift->n_list, d.N);
    }
    if (action) *action = STGN_MAINTAIN_PARTIAL;
  } else {
    run_layers(ctx, d, true);
    if (action) *action = STGN_MAINTAIN_FULL;
  }
  launch_drift_reset(d, ctx->stream);
  HIPCHK(ctx, hipGetLastError());
  return STGN_OK;
}

int stgn_set_predictor(stgn_ctx* ctx, const float* w, float b) {
  if (!ctx) return STGN_E_INVALID_ARG;
  if (!w) return fail(ctx, STGN_E_INVALID_ARG, "NULL weights");
  const uint32_t d2 = 2 * ctx->cfg.d_emb;
  std::vector<float> wb(w, w + d2);
  wb.push_back(b);
  // ordered after predictions already enqueued, before those that follow
  HIPCHK(ctx, hipStreamSynchronize(ctx->stream));
  HIPCHK(ctx, hipMemcpy(ctx->d.pred_w, wb.data(), wb.size() * sizeof(float), hipMemcpyHostToDevice));
  ctx->have_predictor = true;
  return STGN_OK;
}

int stgn_predict_batch(stgn_ctx* ctx, uint32_t n, const uint32_t* src, const uint32_t* dst, const double* ts,
                       int at_edge_time, int inputs_on_device, float* scores) {
  if (!ctx) return STGN_E_INVALID_ARG;
  const stgn_config& c = ctx->cfg;
  const Dev& d = ctx->d;
  if (!ctx->have_predictor) return fail(ctx, STGN_E_INVALID_ARG, "stgn_set_predictor has not been called");
  if (n > c.max_batch) return fail(ctx, STGN_E_BATCH_TOO_LARGE, "more edges than max_batch");
  if (n == 0) return inputs_on_device ? STGN_OK : sync_and_poll(ctx);
  if (!src || !dst || !ts || !scores) return fail(ctx, STGN_E_INVALID_ARG, "NULL array");
  hipStream_t s = ctx->stream;
  const uint32_t *dsrc = src, *ddst = dst;
  const double* dts = ts;
  float* dout = scores;
  if (!inputs_on_device) {
    for (uint32_t i = 0; i < n; ++i)
      if (src[i] >= c.num_nodes || dst[i] >= c.num_nodes) return fail(ctx, STGN_E_NODE_OUT_OF_RANGE, "endpoint id >= num_nodes");
    HIPCHK(ctx, hipMemcpyAsync(d.pred_src, src, (size_t)n * 4, hipMemcpyHostToDevice, s));
    HIPCHK(ctx, hipMemcpyAsync(d.pred_dst, dst, (size_t)n * 4, hipMemcpyHostToDevice, s));
    HIPCHK(ctx, hipMemcpyAsync(d.pred_ts, ts, (size_t)n * 8, hipMemcpyHostToDevice, s));
    dsrc = d.pred_src; ddst = d.pred_dst; dts = d.pred_ts; dout = d.pred_scores;
  }
  ctx->idle = false;
  {
    Scope t(ctx, KC_PREDICT);
    if (at_edge_time) {
      launch_predict_prep(d, s, n, dsrc, ddst, dts);
      launch_layer_roots(d, s, 2 * n);
    }
    launch_predict_head(d, s, n, dsrc, ddst, at_edge_time, dout);
  }
  HIPCHK(ctx, hipGetLastError());
  if (!inputs_on_device) {
    HIPCHK(ctx, hipMemcpyAsync(scores, d.pred_scores, (size_t)n * sizeof(float), hipMemcpyDeviceToHost, s));
    return sync_and_poll(ctx);
  }
  return STGN_OK;
}

// Device bytes of static scratch a prediction of n edges needs: the 2n roots, their query times, their rows.
static size_t static_predict_bytes(uint32_t n, uint32_t d_emb) {
  auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
  return up((size_t)2 * n * sizeof(uint32_t)) + up((size_t)2 * n * sizeof(double)) + up((size_t)2 * n * d_emb * sizeof(float));
}

int stgn_predict_batch_static(stgn_ctx* ctx, uint32_t n, const uint32_t* src, const uint32_t* dst, const double* ts,
                              int at_edge_time, float* scores) {
  if (!ctx) return STGN_E_INVALID_ARG;
  const stgn_config& c = ctx->cfg;
  if (!ctx->have_predictor) return fail(ctx, STGN_E_INVALID_ARG, "stgn_set_predictor has not been called");
  if (n > c.max_batch) return fail(ctx, STGN_E_BATCH_TOO_LARGE, "more edges than max_batch");
  if (static_predict_bytes(n, c.d_emb) > kStaticScratchBytes) {
    char buf[160];
    snprintf(buf, sizeof buf, "%u edges of %u-wide rows need %zu bytes of static scratch, the array holds %zu",
             n, c.d_emb, static_predict_bytes(n, c.d_emb), kStaticScratchBytes);
    return fail(ctx, STGN_E_BATCH_TOO_LARGE, buf);
  }
  if (n == 0) return STGN_OK;
  if (!src || !dst || !ts || !scores) return fail(ctx, STGN_E_INVALID_ARG, "NULL array");
  if (!ctx->static_scratch) return fail(ctx, STGN_E_DEVICE, "static scratch was not resolved for this device");
  // the same kernels as stgn_predict_batch, their scratch lists pointed at the static array
  Dev d = ctx->d;
  auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
  unsigned char* p = ctx->static_scratch;
  d.pred_rows = reinterpret_cast<uint32_t*>(p);
  d.pred_tq = reinterpret_cast<double*>(p + up((size_t)2 * n * sizeof(uint32_t)));
  d.pred_out = reinterpret_cast<float*>(p + up((size_t)2 * n * sizeof(uint32_t)) + up((size_t)2 * n * sizeof(double)));
  hipStream_t s = ctx->stream;
  ctx->idle = false;
  if (at_edge_time) {
    launch_predict_prep(d, s, n, src, dst, ts);
    launch_layer_roots(d, s, 2 * n);
  }
  launch_predict_head(d, s, n, src, dst, at_edge_time, scores);
  HIPCHK(ctx, hipGetLastError());
  return STGN_OK;
}

int stgn_sync(stgn_ctx* ctx) {
  if (!ctx) return STGN_E_INVALID_ARG;
  return sync_and_poll(ctx);
}

int stgn_get_embeddings(stgn_ctx* ctx, uint32_t layer, uint32_t n, const uint32_t* nodes, float* out, int on_device) {
  if (!ctx) return STGN_E_INVALID_ARG;
  const stgn_config& c = ctx->cfg;
  const Dev& d = ctx->d;
  if (layer == 0) layer = c.layers;
  if (layer > c.layers) return fail(ctx, STGN_E_INVALID_ARG, "layer out of range");
  if (n == 0) return on_device ? STGN_OK : sync_and_poll(ctx);
  if (!nodes || !out) return fail(ctx, STGN_E_INVALID_ARG, "NULL nodes or out");
  if (on_device) {
    ctx->idle = false;
    Scope t(ctx, KC_GATHER);
    launch_gather_rows(d, ctx->stream, layer, n, nodes, out);
    return STGN_OK;
  }
  for (uint32_t i = 0; i < n; ++i)
    if (nodes[i] >= c.num_nodes) return fail(ctx, STGN_E_NODE_OUT_OF_RANGE, "node id >= num_nodes");
  for (uint32_t lo = 0; lo < n; lo += d.q_cap) {
    const uint32_t m = std::min(d.q_cap, n - lo);
    HIPCHK(ctx, hipMemcpyAsync(d.qnodes, nodes + lo, (size_t)m * 4, hipMemcpyHostToDevice, ctx->stream));
    launch_gather_rows(d, ctx->stream, layer, m, d.qnodes, d.qout);
    HIPCHK(ctx, hipMemcpyAsync(out + (size_t)lo * c.d_emb, d.qout, (size_t)m * c.d_emb * 4, hipMemcpyDeviceToHost, ctx->stream));
    HIPCHK(ctx, hipStreamSynchronize(ctx->stream));
  }
  return sync_and_poll(ctx);
}

int stgn_get_affected(stgn_ctx* ctx, uint32_t* out, uint32_t cap, uint32_t* count) {
  if (!ctx || !count) return STGN_E_INVALID_ARG;
  int rc = sync_and_poll(ctx);
  const uint32_t nA = ctx->ctrl_host->b[ctx->last_par].nA;
  *count = nA;
  const uint32_t m = std::min(nA, cap);
  if (m && out) HIPCHK(ctx, hipMemcpy(out, ctx->d.A, (size_t)m * 4, hipMemcpyDeviceToHost));
  return rc;
}

int stgn_get_neighbors(stgn_ctx* ctx, uint32_t node, uint32_t* nbr, uint32_t* eid, double* ts, uint32_t* count) {
  if (!ctx || !count) return STGN_E_INVALID_ARG;
  if (node >= ctx->cfg.num_nodes) return fail(ctx, STGN_E_NODE_OUT_OF_RANGE, "node id >= num_nodes");
  int rc = sync_and_poll(ctx);
  const uint32_t k = ctx->cfg.k;
  uint32_t dg = 0;
  HIPCHK(ctx, hipMemcpy(&dg, ctx->d.deg + node, 4, hipMemcpyDeviceToHost));
  std::vector<RingEntry> r(k);
  HIPCHK(ctx, hipMemcpy(r.data(), ctx->d.ring + (size_t)node * k, (size_t)k * sizeof(RingEntry), hipMemcpyDeviceToHost));
  const uint32_t cnt = std::min(dg, k);
  for (uint32_t j = 0; j < cnt; ++j) {
    const RingEntry& e = r[(dg - 1 - j) % k];
    if (nbr) nbr[j] = e.nbr;
    if (eid) eid[j] = e.eid;
    if (ts) ts[j] = e.t;
  }
  *count = cnt;
  return rc;
}

int stgn_get_history(stgn_ctx* ctx, uint32_t node, uint32_t first, uint32_t count, uint32_t* nbr, uint32_t* eid,
                     uint32_t* degree) {
  if (!ctx) return STGN_E_INVALID_ARG;
  if (node >= ctx->cfg.num_nodes) return fail(ctx, STGN_E_NODE_OUT_OF_RANGE, "node id >= num_nodes");
  int rc = sync_and_poll(ctx);
  const Dev& d = ctx->d;
  uint32_t dg = 0;
  HIPCHK(ctx, hipMemcpy(&dg, d.deg + node, 4, hipMemcpyDeviceToHost));
  if (degree) *degree = dg;
  if (count == 0) return rc;
  if ((uint64_t)first + count > dg) return fail(ctx, STGN_E_INVALID_ARG, "history range beyond the node's degree");
  std::vector<uint32_t> blk(d.maxb);
  HIPCHK(ctx, hipMemcpy(blk.data(), d.blk + (size_t)node * d.maxb, (size_t)d.maxb * 4, hipMemcpyDeviceToHost));
  std::vector<uint2> tmp;
  uint32_t p = first;
  while (p < first + count) {
    uint32_t b = 0;
    while (kMinBlock * ((2u << b) - 1u) <= p) ++b;                 // block holding position p
    const uint32_t bstart = kMinBlock * ((1u << b) - 1u), bend = kMinBlock * ((2u << b) - 1u);
    const uint32_t m = std::min(bend, first + count) - p;
    const uint64_t a = (uint64_t)blk[b] * kMinBlock + (p - bstart);
    if (nbr) {
      tmp.resize(m);
      HIPCHK(ctx, hipMemcpy(tmp.data(), d.pool_nt + a, (size_t)m * sizeof(uint2), hipMemcpyDeviceToHost));
      for (uint32_t i = 0; i < m; ++i) nbr[p - first + i] = tmp[i].x;
    }
    if (eid) HIPCHK(ctx, hipMemcpy(eid + (p - first), d.pool_eid + a, (size_t)m * 4, hipMemcpyDeviceToHost));
    p += m;
  }
  return rc;
}

int stgn_get_memory(stgn_ctx* ctx, uint32_t n, const uint32_t* nodes, float* mem, double* t_last) {
  if (!ctx || (n && !nodes)) return STGN_E_INVALID_ARG;
  const stgn_config& c = ctx->cfg;
  const Dev& d = ctx->d;
  for (uint32_t i = 0; i < n; ++i)
    if (nodes[i] >= c.num_nodes) return fail(ctx, STGN_E_NODE_OUT_OF_RANGE, "node id >= num_nodes");
  int rc = sync_and_poll(ctx);
  if (mem && c.d_mem) {
    std::vector<float> rowbuf;
    for (uint32_t lo = 0; lo < n; lo += d.q_cap) {
      const uint32_t m = std::min(d.q_cap, n - lo);
      rowbuf.resize((size_t)m * d.d0);
      HIPCHK(ctx, hipMemcpyAsync(d.qnodes, nodes + lo, (size_t)m * 4, hipMemcpyHostToDevice, ctx->stream));
      launch_gather_rows(d, ctx->stream, 0, m, d.qnodes, d.qout);
      HIPCHK(ctx, hipMemcpyAsync(rowbuf.data(), d.qout, rowbuf.size() * 4, hipMemcpyDeviceToHost, ctx->stream));
      HIPCHK(ctx, hipStreamSynchronize(ctx->stream));
      for (uint32_t i = 0; i < m; ++i)
        memcpy(mem + (size_t)(lo + i) * c.d_mem, rowbuf.data() + (size_t)i * d.d0, (size_t)c.d_mem * 4);
    }
  }
  if (t_last) {
    // the row staging block holds at least q_cap floats per column, i.e. q_cap / 2 doubles per column
    const uint32_t cap = d.q_cap / 2;
    for (uint32_t lo = 0; lo < n; lo += cap) {
      const uint32_t m = std::min(cap, n - lo);
      HIPCHK(ctx, hipMemcpyAsync(d.qnodes, nodes + lo, (size_t)m * 4, hipMemcpyHostToDevice, ctx->stream));
      launch_gather_times(d, ctx->stream, m, d.qnodes, reinterpret_cast<double*>(d.qout));
      HIPCHK(ctx, hipMemcpyAsync(t_last + lo, d.qout, (size_t)m * 8, hipMemcpyDeviceToHost, ctx->stream));
      HIPCHK(ctx, hipStreamSynchronize(ctx->stream));
    }
  }
  return rc;
}

int stgn_get_totals(stgn_ctx* ctx, uint64_t* edges, uint64_t* direct, uint64_t* affected, uint64_t* scanned,
                    uint64_t* gathered, uint64_t* rows) {
  if (!ctx) return STGN_E_INVALID_ARG;
  int rc = sync_and_poll(ctx);
  const Ctrl& h = *ctx->ctrl_host;
  if (edges) *edges = h.E;
  if (direct) *direct = h.tot_direct;
  if (affected) *affected = h.tot_affected;
  if (scanned) *scanned = h.tot_scanned;
  if (gathered) {
    // the layer kernel keeps one plain counter per workgroup index (no atomic updates)
    std::vector<uint64_t> slots(kStatSlots);
    HIPCHK(ctx, hipMemcpy(slots.data(), ctx->d.gathered_slots, kStatSlots * sizeof(uint64_t), hipMemcpyDeviceToHost));
    uint64_t sum = 0;
    for (uint64_t v : slots) sum += v;
    *gathered = sum;
  }
  if (rows) *rows = h.tot_rows;
  return rc;
}

int stgn_kernel_times(stgn_ctx* ctx, int enable, int reset, uint32_t cap, const char** names, double* usec,
                      uint64_t* launches) {
  if (!ctx) return STGN_E_INVALID_ARG;
  HIPCHK(ctx, hipStreamSynchronize(ctx->stream));
  drain_timing(ctx);
  const uint32_t m = std::min<uint32_t>(cap, KC_COUNT);
  for (uint32_t i = 0; i < m; ++i) {
    if (names) names[i] = kClassNames[i];
    if (usec) usec[i] = ctx->k_usec[i];
    if (launches) launches[i] = ctx->k_launches[i];
  }
  if (reset) for (int i = 0; i < KC_COUNT; ++i) { ctx->k_usec[i] = 0.0; ctx->k_launches[i] = 0; }
  ctx->timing = enable != 0;
  return (int)m;
}

}  // extern "C"
