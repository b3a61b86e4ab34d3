// Launch plumbing of the fused attention-layer kernel (defined in layer_kernel.h, instantiated per
// head count in layer_h*.hip) and the cached-row gather behind stgn_get_embeddings.
#include "layer_kernel.h"

namespace stgn {

extern template void layer_entry<1>(layer_impl::LaunchArgs&);
extern template void layer_entry<2>(layer_impl::LaunchArgs&);
extern template void layer_entry<4>(layer_impl::LaunchArgs&);

namespace {

using layer_impl::LaunchArgs;
using layer_impl::LayerArgs;

// Rows of a table for a list of node ids; an id past the node count (device-resident lists are not
// checked on the host) yields a row of NaN instead of a read outside the table.
__global__ void gather_rows_kernel(Table T, uint32_t N, uint32_t width, uint32_t n, const uint32_t* __restrict__ nodes,
                                   float* __restrict__ out) {
  const size_t tot = (size_t)n * width;
  for (size_t x = (size_t)blockIdx.x * blockDim.x + threadIdx.x; x < tot; x += (size_t)gridDim.x * blockDim.x) {
    const size_t i = x / width, c = x - i * width;
    const uint32_t v = nodes[i];
    out[x] = v < N ? T.base[(size_t)v * T.ld + c] : __builtin_nanf("");
  }
}

__global__ void gather_times_kernel(const double* __restrict__ t, uint32_t N, uint32_t n, const uint32_t* __restrict__ nodes,
                                    double* __restrict__ out) {
  for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) {
    const uint32_t v = nodes[i];
    out[i] = v < N ? t[v] : __builtin_nan("");
  }
}

// Roots of n edges for stgn_predict_batch: source and destination of edge i at list positions 2i and
// 2i + 1, both queried at the edge's time.  An id past the node count becomes a dead row.
__global__ void predict_prep_kernel(Dev d, uint32_t n, const uint32_t* __restrict__ src, const uint32_t* __restrict__ dst,
                                    const double* __restrict__ ts) {
  for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) {
    const uint32_t u = src[i], v = dst[i];
    d.pred_rows[2 * i] = u < d.N ? u : 0xFFFFFFFFu;
    d.pred_rows[2 * i + 1] = v < d.N ? v : 0xFFFFFFFFu;
    d.pred_tq[2 * i] = ts[i];
    d.pred_tq[2 * i + 1] = ts[i];
  }
}

// Linear link score (Algorithm 1, "Link prediction"): one 64-lane wave per edge,
// y = h_u . w[0 : d) + h_v . w[d : 2d) + b, the two rows either cached final-layer rows or the rows
// the final layer just produced for the roots.
__global__ __launch_bounds__(256) void predict_head_kernel(Dev d, uint32_t n, const uint32_t* __restrict__ src,
                                                           const uint32_t* __restrict__ dst, int at_edge_time,
                                                           float* __restrict__ scores) {
  const uint32_t lane = threadIdx.x & 63u;
  const uint32_t wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6, nwaves = (gridDim.x * blockDim.x) >> 6;
  const uint32_t de = d.d_emb;
  const Table HL = d.H[d.layers];
  for (uint32_t i = wave; i < n; i += nwaves) {
    const uint32_t u = src[i], v = dst[i];
    const bool ok = u < d.N && v < d.N;
    const float* hu = at_edge_time ? d.pred_out + (size_t)(2 * i) * de : HL.base + (size_t)(ok ? u : 0u) * HL.ld;
    const float* hv = at_edge_time ? d.pred_out + (size_t)(2 * i + 1) * de : HL.base + (size_t)(ok ? v : 0u) * HL.ld;
    float acc = 0.0f;
    for (uint32_t c = lane; c < de; c += 64) acc = fmaf(hu[c], d.pred_w[c], fmaf(hv[c], d.pred_w[de + c], acc));
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
    if (lane == 0) scores[i] = ok ? acc + d.pred_w[2 * de] : __builtin_nanf("");
  }
}

LaunchArgs make_args(const Dev& d, uint32_t layer) {
  const LayerDev& L = d.L[layer];
  LaunchArgs a{};
  LayerArgs& k = a.k;
  k.Hin = d.H[layer].base; k.Hout = d.H[layer + 1].base;
  k.KVn = d.KV[layer].base; k.KVe = d.KVE[layer].base;
  k.KVout = layer + 1 < d.layers ? d.KV[layer + 1].base : nullptr;
  k.WKVnext = layer + 1 < d.layers ? d.L[layer + 1].WKVn : nullptr;
  k.ring = d.ring; k.deg = d.deg; k.t_last = d.t_last;
  k.om_rev = d.om_rev; k.ph_rev = d.ph_rev; k.ctrl = d.ctrl; k.gathered_slots = d.gathered_slots;
  k.WQ = L.WQn; k.cQ = L.cQ; k.WKT = L.WKT; k.WV = L.WV; k.WO = L.WO; k.bO = L.bO;
  k.ld_in = d.H[layer].ld; k.ld_out = d.H[layer + 1].ld; k.ld_kv = d.ld_kv; k.ld_kve = d.KVE[layer].ld;
  k.window = d.window;
  k.k = d.k; k.d_in = L.d_in; k.d_emb = d.d_emb; k.dk = d.dk; k.d_time = d.d_time; k.d_edge = d.d_edge;
  if (d.delta) {
    k.flags = d.flags_kept;
    k.thr_in = d.d_mem ? layer + 1u : layer;                  // flags at or below: the owner's input row of this layer changed
    k.force_exact = 1u; k.is_final = layer + 1 == d.layers ? 1u : 0u;
    k.gamma = d.gamma;
    k.ac_S = d.ac_S[layer]; k.ac_P = d.ac_P[layer]; k.ac_ZM = d.ac_ZM[layer]; k.ac_W = d.ac_W[layer]; k.ac_V = d.ac_V[layer];
    k.drift = d.drift; k.dsum = d.dsum; k.dlast = d.dlast; k.dseen = d.dseen;
  }
  k.QC = d.qcache ? d.QC[layer] : nullptr;                     // (null for the layers that keep none)
  k.tile_clean = d.qcache ? d.tile_clean[layer] : nullptr;
  a.delta = d.delta != 0;
  a.es = d.es != 0;
  a.ks = d.ks; a.nt = d.nt; a.heads = d.heads;
  a.num_cu = d.num_cu;
  a.lds = (size_t)layer_impl::layer_lds(L.d_in, d.heads, d.ks, d.nz, d.k, d.delta != 0).total * sizeof(float);
  a.err = hipSuccess;
  return a;
}

void go_heads(LaunchArgs& a) {
  switch (a.heads) {
    case 1: layer_entry<1>(a); break;
    case 2: layer_entry<2>(a); break;
    default: layer_entry<4>(a); break;
  }
}

}  // namespace

// heads in {1, 2, 4}; every head takes whole 64-float slots of a cached row, at most four in total;
// the time encoding takes at most two
int attn_supported(uint32_t d_emb, uint32_t d_time, uint32_t heads) {
  if (!(heads == 1 || heads == 2 || heads == 4) || d_emb == 0 || d_emb % heads) return 0;
  uint32_t sh = (d_emb / heads + kSlot - 1) / kSlot;
  if (sh == 3) sh = 4;
  return d_time >= 1 && d_time <= kMaxTimeSlots * kSlot && heads * sh <= kMaxKeySlots;
}

void launch_layer(const Dev& d, hipStream_t s, uint32_t layer, const uint32_t* rows, const uint32_t* cp, uint32_t cm,
                  bool force_exact) {
  LaunchArgs a = make_args(d, layer);
  a.k.force_exact = force_exact ? 1u : 0u;
  if (force_exact) a.k.tile_clean = nullptr;                   // every row projects its query again (and refreshes the cache)
  a.s = s; a.rows = rows; a.cp = cp; a.cm = cm; a.set_attr = false;
  go_heads(a);
}

void launch_predict_prep(const Dev& d, hipStream_t s, uint32_t n, const uint32_t* src, const uint32_t* dst, const double* ts) {
  hipLaunchKernelGGL(predict_prep_kernel, dim3((n + 255) / 256), dim3(256), 0, s, d, n, src, dst, ts);
}

// the final layer for the roots listed in pred_rows, at the times in pred_tq, into pred_out
void launch_layer_roots(const Dev& d, hipStream_t s, uint32_t nroots) {
  LaunchArgs a = make_args(d, d.layers - 1);
  a.delta = false;                                            // root rows are computed at their own times, from nothing cached
  a.k.tile_clean = nullptr;                                   // the cached rows are current, hence every root's q and qt
  a.k.all_clean = a.k.QC ? 1u : 0u;
  a.k.tq_rows = d.pred_tq;
  a.k.out_rows = d.pred_out;
  a.s = s; a.rows = d.pred_rows; a.cp = nullptr; a.cm = nroots; a.set_attr = false;
  go_heads(a);
}

void launch_predict_head(const Dev& d, hipStream_t s, uint32_t n, const uint32_t* src, const uint32_t* dst,
                         int at_edge_time, float* scores) {
  hipLaunchKernelGGL(predict_head_kernel, dim3((n + 3) / 4), dim3(256), 0, s, d, n, src, dst, at_edge_time, scores);
}

void launch_gather_rows(const Dev& d, hipStream_t s, uint32_t layer, uint32_t n, const uint32_t* nodes, float* out) {
  const uint32_t width = layer == 0 ? d.d0 : d.d_emb;
  uint64_t blocks = ((uint64_t)n * width + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(gather_rows_kernel, dim3((uint32_t)blocks), dim3(256), 0, s, d.H[layer], d.N, width, n, nodes, out);
}

void launch_gather_times(const Dev& d, hipStream_t s, uint32_t n, const uint32_t* nodes, double* out) {
  uint32_t blocks = (n + 255) / 256;
  if (blocks > 1024) blocks = 1024;
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(gather_times_kernel, dim3(blocks), dim3(256), 0, s, d.t_last, d.N, n, nodes, out);
}

// ---- drift estimator (Sec. 3.5)
__global__ __launch_bounds__(256) void drift_reset_kernel(Dev d) {
  const uint32_t nth = gridDim.x * blockDim.x, tid = blockIdx.x * blockDim.x + threadIdx.x;
  for (uint32_t v = tid; v < d.N; v += nth) { d.dsum[v] = 0.0f; d.dlast[v] = 0u; d.dseen[v] = 0; }
  if (tid == 0) { d.drift->G = 0.0; d.drift->count = 0u; d.drift->n_list = 0u; }
}

// nodes whose decayed estimate exceeds the threshold, in no particular order
__global__ __launch_bounds__(256) void drift_list_kernel(Dev d, float threshold) {
  const uint32_t nth = gridDim.x * blockDim.x, tid = blockIdx.x * blockDim.x + threadIdx.x;
  const uint32_t tau = d.drift->tau;
  // (grid-stride with a uniform trip count: every lane of a wave takes part in the ballots; one reservation
  // of list places per wave and round)
  const uint32_t lane = threadIdx.x & 63u;
  for (uint32_t v0 = tid - lane; v0 < d.N; v0 += nth) {
    const uint32_t v = v0 + lane;
    bool hit = false;
    if (v < d.N && d.dseen[v]) hit = d.dsum[v] * __powf(d.gamma, (float)(tau - d.dlast[v])) > threshold;
    const uint64_t m = __ballot(hit);
    if (m == 0ull) continue;
    uint32_t base = 0;
    if (lane == 0) base = atomicAdd(&d.drift->n_list, (uint32_t)__popcll(m));
    base = (uint32_t)__builtin_amdgcn_readfirstlane((int)base);
    if (hit) d.dlist[base + (uint32_t)__popcll(m & ((1ull << lane) - 1ull))] = v;
  }
}

// every node's decayed estimate (0 for nodes outside the cumulative affected set)
__global__ __launch_bounds__(256) void drift_values_kernel(Dev d, float* out) {
  const uint32_t nth = gridDim.x * blockDim.x, tid = blockIdx.x * blockDim.x + threadIdx.x;
  const uint32_t tau = d.drift->tau;
  for (uint32_t v = tid; v < d.N; v += nth)
    out[v] = d.dseen[v] ? d.dsum[v] * __powf(d.gamma, (float)(tau - d.dlast[v])) : 0.0f;
}

void launch_drift_values(const Dev& d, hipStream_t s, float* out) {
  uint32_t blocks = (d.N + 255) / 256;
  if (blocks > 2048) blocks = 2048;
  hipLaunchKernelGGL(drift_values_kernel, dim3(blocks ? blocks : 1), dim3(256), 0, s, d, out);
}

void launch_drift_reset(const Dev& d, hipStream_t s) {
  uint32_t blocks = (d.N + 255) / 256;
  if (blocks > 2048) blocks = 2048;
  hipLaunchKernelGGL(drift_reset_kernel, dim3(blocks ? blocks : 1), dim3(256), 0, s, d);
}

void launch_drift_list(const Dev& d, hipStream_t s, float threshold) {
  uint32_t blocks = (d.N + 255) / 256;
  if (blocks > 2048) blocks = 2048;
  hipLaunchKernelGGL(drift_list_kernel, dim3(blocks ? blocks : 1), dim3(256), 0, s, d, threshold);
}

// Whether the layer kernel's tiles fit its share of the LDS at every layer with nz slots of z (d: the
// configuration fields and ks, nt).
int layer_tiles_fit(const Dev& d, uint32_t nz) {
  LaunchArgs a{};
  a.ks = d.ks; a.nt = d.nt; a.heads = d.heads; a.query_wgs = 1;
  go_heads(a);
  if (a.wgs == 0) return 0;
  for (uint32_t l = 0; l < d.layers; ++l) {
    const size_t lds = (size_t)layer_impl::layer_lds(l ? d.d_emb : d.d0, d.heads, d.ks, nz, d.k, false).total * sizeof(float);
    if (lds + 3072 > kMaxLds / a.wgs) return 0;
  }
  return 1;
}

// ---- bare gather (diagnostic): 16 lanes per row piece of 256 B, as in the layer kernel's entry loop, and
// nothing else -- few registers, full occupancy
template <int SLOTS>
__global__ __launch_bounds__(256) void gather_probe_kernel(const float* __restrict__ table, const uint32_t* __restrict__ idx,
                                                           uint32_t n_groups, uint32_t per, float* __restrict__ out) {
  const uint32_t g = (blockIdx.x * 256u + threadIdx.x) >> 4, sub = threadIdx.x & 15u;
  if (g >= n_groups) return;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  const uint32_t* ip = idx + (size_t)g * per;
  for (uint32_t j = 0; j < per; ++j) {
    const float* row = table + (size_t)ip[j] * (SLOTS * kSlot) + 4u * sub;
#pragma unroll
    for (int s = 0; s < SLOTS; ++s) {
      const float4 v = *reinterpret_cast<const float4*>(row + s * kSlot);
      acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
  }
  out[(size_t)g * 16u + sub] = acc.x + acc.y + acc.z + acc.w;
}

void launch_gather_probe(hipStream_t s, const float* table, uint32_t slots, const uint32_t* idx, uint32_t n_groups,
                         uint32_t per, float* out) {
  const dim3 grid((uint32_t)(((uint64_t)n_groups * 16u + 255u) / 256u)), blk(256);
  if (slots == 1) hipLaunchKernelGGL(gather_probe_kernel<1>, grid, blk, 0, s, table, idx, n_groups, per, out);
  else hipLaunchKernelGGL(gather_probe_kernel<4>, grid, blk, 0, s, table, idx, n_groups, per, out);
}

int setup_embed_attributes(const Dev& d) {
  for (uint32_t l = 0; l < d.layers; ++l) {
    LaunchArgs a = make_args(d, l);
    a.query_wgs = 1;
    go_heads(a);
    if (a.wgs == 0) return -1;                                    // no kernel variant for this shape
    if (a.lds + 3072 > kMaxLds / a.wgs) return -1;                // that many workgroups per CU, plus the static arrays
    a.query_wgs = 0;
    a.set_attr = true;
    go_heads(a);
    if (a.err != hipSuccess) return -1;
    if (a.delta) {                                                // the exact variant serves the root rows
      a.delta = false;
      go_heads(a);
      if (a.err != hipSuccess) return -1;
    }
  }
  return 0;
}

}  // namespace stgn
