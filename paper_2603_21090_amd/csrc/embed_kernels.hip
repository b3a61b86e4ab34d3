// Launch plumbing of the fused attention-layer kernel (defined in layer_kernel.h, instantiated per
// slot count in layer_ns*.hip) and the cached-row gather behind stgn_get_embeddings.
#include "layer_kernel.h"

namespace stgn {

#define STGN_DECL_ENTRY(NS) extern template void layer_entry<NS>(layer_impl::LaunchArgs&);
STGN_DECL_ENTRY(2) STGN_DECL_ENTRY(3) STGN_DECL_ENTRY(4) STGN_DECL_ENTRY(5)
STGN_DECL_ENTRY(6) STGN_DECL_ENTRY(7) STGN_DECL_ENTRY(8)
#undef STGN_DECL_ENTRY

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
  k.Hin = d.H[layer].base; k.Hout = d.H[layer + 1].base; k.efeat = d.efeat.base;
  k.ring = d.ring; k.deg = d.deg; k.t_last = d.t_last;
  k.om_rev = d.om_rev; k.ph_rev = d.ph_rev; k.ctrl = d.ctrl;
  k.WQ = L.WQn; k.cQ = L.cQ; k.WKT = L.WKT; k.WV = L.WV; k.WO = L.WO; k.bO = L.bO;
  k.ld_in = d.H[layer].ld; k.ld_out = d.H[layer + 1].ld; k.ld_ef = d.efeat.ld;
  k.k = d.k; k.heads = d.heads; k.d_in = L.d_in; k.d_emb = d.d_emb; k.dk = d.dk; k.d_time = d.d_time; k.Zp = L.Zp;
  for (uint32_t s = 0; s < kMaxSlots; ++s) {
    k.valid[s] = s < L.ns ? L.valid[s] : 0;
    k.segoff[s] = s < L.ns ? L.segoff[s] : 0;
    k.kind[s] = s < L.ns ? L.kind[s] : 3;
  }
  a.nt = L.nt;
  a.grid_cap = 2u * (d.num_cu ? d.num_cu : 256u);
  a.lds = (size_t)layer_impl::layer_lds(L.d_in, d.d_emb, d.heads, L.Zp, d.k).total * sizeof(float);
  a.err = hipSuccess;
  return a;
}

void go_ns(LaunchArgs& a, uint32_t ns) {
  switch (ns) {
    case 2: layer_entry<2>(a); break;
    case 3: layer_entry<3>(a); break;
    case 4: layer_entry<4>(a); break;
    case 5: layer_entry<5>(a); break;
    case 6: layer_entry<6>(a); break;
    case 7: layer_entry<7>(a); break;
    default: layer_entry<8>(a); break;
  }
}

}  // namespace

int attn_supported(uint32_t d_in, uint32_t d_edge, uint32_t d_time, uint32_t heads) {
  const uint32_t ns = (d_in + kSlot - 1) / kSlot + (d_edge + kSlot - 1) / kSlot + (d_time + kSlot - 1) / kSlot;
  return d_in >= 1 && d_time >= 1 && d_time <= 2 * kSlot && ns <= kMaxSlots && (heads == 1 || heads == 2 || heads == 4);
}

void launch_layer(const Dev& d, hipStream_t s, uint32_t layer, const uint32_t* rows, const uint32_t* cp, uint32_t cm) {
  LaunchArgs a = make_args(d, layer);
  a.s = s; a.rows = rows; a.cp = cp; a.cm = cm; a.set_attr = false;
  go_ns(a, d.L[layer].ns);
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
    if (a.lds + 4096 > kMaxLds / 2) return -1;     // two workgroups per CU, plus the static arrays
    a.set_attr = true;
    go_ns(a, d.L[l].ns);
    if (a.err != hipSuccess) return -1;
  }
  return 0;
}

}  // namespace stgn
