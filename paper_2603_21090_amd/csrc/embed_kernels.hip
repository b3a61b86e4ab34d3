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

__global__ void gather_rows_kernel(Table T, uint32_t width, uint32_t n, const uint32_t* __restrict__ nodes,
                                   float* __restrict__ out) {
  const size_t tot = (size_t)n * width;
  for (size_t x = (size_t)blockIdx.x * blockDim.x + threadIdx.x; x < tot; x += (size_t)gridDim.x * blockDim.x) {
    const size_t i = x / width, c = x - i * width;
    out[x] = T.base[(size_t)nodes[i] * T.ld + c];
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
  k.om_rev = d.om_rev; k.ph_rev = d.ph_rev; k.ctrl = d.ctrl;
  k.WQ = L.WQn; k.cQ = L.cQ; k.WKT = L.WKT; k.WV = L.WV; k.WO = L.WO; k.bO = L.bO;
  k.ld_in = d.H[layer].ld; k.ld_out = d.H[layer + 1].ld; k.ld_kv = d.ld_kv; k.ld_kve = d.KVE[layer].ld;
  k.k = d.k; k.d_in = L.d_in; k.d_emb = d.d_emb; k.dk = d.dk; k.d_time = d.d_time;
  a.ks = d.ks; a.nt = d.nt; a.heads = d.heads;
  a.num_cu = d.num_cu;
  a.lds = (size_t)layer_impl::layer_lds(L.d_in, d.heads, d.ks, d.nt, d.k).total * sizeof(float);
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

void launch_layer(const Dev& d, hipStream_t s, uint32_t layer, const uint32_t* rows, const uint32_t* cp, uint32_t cm) {
  LaunchArgs a = make_args(d, layer);
  a.s = s; a.rows = rows; a.cp = cp; a.cm = cm; a.set_attr = false;
  go_heads(a);
}

void launch_gather_rows(const Dev& d, hipStream_t s, uint32_t layer, uint32_t n, const uint32_t* nodes, float* out) {
  const uint32_t width = layer == 0 ? d.d0 : d.d_emb;
  uint64_t blocks = ((uint64_t)n * width + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(gather_rows_kernel, dim3((uint32_t)blocks), dim3(256), 0, s, d.H[layer], width, n, nodes, out);
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
  }
  return 0;
}

}  // namespace stgn
