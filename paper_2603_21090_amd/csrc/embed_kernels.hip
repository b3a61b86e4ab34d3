// Launch plumbing of the fused attention-layer kernel (defined in layer_kernel.h, instantiated per
// head count in layer_h*.hip), the projection kernel that fills the cached key|value rows outside the
// layer kernel, and the cached-row gather behind stgn_get_embeddings.
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

// Cached key|value rows that do not come out of a layer kernel (see LayerDev):
//   all_nodes = 0, once per batch:  KV[0][v] = H[0][v] [W_K | W_V](node rows of layer 0) for the batch's
//       endpoints v (their memory just changed; skipped without a memory), and for every layer l
//       KVE[l][e] = feat_e [W_K | W_V](edge rows of layer l) for the batch's edges e;
//   all_nodes = 1 (initial state, full rebuild):  KV[0][v] for every node.
// One workgroup (four waves) per 16 rows: the rows go through LDS as the A operand, wave w computes
// the column tiles w + 8 i and w + 8 i + 4 of the 128 ks output columns.
constexpr uint32_t kProjRows = 16;
__global__ __launch_bounds__(256) void project_kernel(Dev d, const float* __restrict__ ef, uint32_t all_nodes) {
  extern __shared__ __align__(16) float lds[];
  const Ctrl* c = d.ctrl;
  if (!all_nodes && c->skip) return;
  const uint32_t nD = all_nodes ? d.N : (d.d_mem ? c->nD : 0u);
  const uint32_t nE = (all_nodes || !d.d_edge) ? 0u : c->n_edges;
  const uint64_t E0 = c->E_base;
  const uint32_t tD = (nD + kProjRows - 1) / kProjRows, tE = (nE + kProjRows - 1) / kProjRows;
  const uint32_t ntiles = tD + d.layers * tE;
  const uint32_t kmax = d.d0 > d.d_edge ? d.d0 : d.d_edge;
  const uint32_t lda = round_up(kmax, kGrpK) + 4;
  const uint32_t lane = threadIdx.x & 63u;
  const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const uint32_t a_off = a16_lane_off(lda);
  const uint32_t ntkv = 8u * d.ks;
  // operand padding must be finite: clear the tile once (one chunk of slack behind the last row)
  for (uint32_t x = threadIdx.x; x < kProjRows * lda + 4 * kGrpK; x += 256) lds[x] = 0.0f;
  __syncthreads();
  for (uint32_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
    const bool node_job = tile < tD;
    const uint32_t layer = node_job ? 0u : (tile - tD) / tE;
    const uint32_t r0 = (node_job ? tile : (tile - tD) - layer * tE) * kProjRows;
    const uint32_t nrows = node_job ? nD : nE;
    const uint32_t K = node_job ? d.d0 : d.d_edge;
    const float* W = node_job ? d.L[0].WKVn : d.L[layer].WKVe;
    float* out = node_job ? d.KV[0].base : d.KVE[layer].base;
    // stage the rows (columns K .. lda keep their zeros or finite leftovers of a wider job: they meet zero weights)
    for (uint32_t x = threadIdx.x; x < kProjRows * K; x += 256) {
      const uint32_t r = x / K, col = x - r * K;
      float v = 0.0f;
      if (r0 + r < nrows) {
        if (node_job) v = d.H[0].base[(size_t)(all_nodes ? r0 + r : d.D[r0 + r]) * d.H[0].ld + col];
        else v = ef[(size_t)(r0 + r) * d.d_edge + col];
      }
      lds[r * lda + col] = v;
    }
    __syncthreads();
    const uint32_t ck = chunks_of(K), gk = kCG * ck;
    for (uint32_t nt = wave; nt < ntkv; nt += 8) {
      const float* const Bt[2] = {W + (size_t)nt * gk * kGrpFloats, W + (size_t)(nt + 4) * gk * kGrpFloats};
      floatx4 acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
      mfma16_gemm<2>(lds + a_off, ck, Bt, acc);
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const uint32_t col = (nt + 4 * t) * 16 + m16_col(lane);     // every column is written: padding columns get exact zeros
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const uint32_t row = r0 + m16_row(lane, r);
          if (row < nrows) {
            const size_t orow = node_job ? (size_t)(all_nodes ? row : d.D[row]) : (size_t)(E0 + row);
            out[orow * d.ld_kv + col] = acc[t][r];
          }
        }
      }
    }
    __syncthreads();
  }
}

size_t project_lds(const Dev& d) {
  const uint32_t kmax = d.d0 > d.d_edge ? d.d0 : d.d_edge;
  return ((size_t)kProjRows * (round_up(kmax, kGrpK) + 4) + 4 * kGrpK) * sizeof(float);
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

void launch_project_batch(const Dev& d, hipStream_t s, const float* ef) {
  if (!d.d_mem && !d.d_edge) return;
  const uint32_t per = (d.max_batch + kProjRows - 1) / kProjRows;
  uint32_t blocks = (d.d_mem ? 2 * per : 0) + (d.d_edge ? d.layers * per : 0);
  if (blocks > 2048) blocks = 2048;
  hipLaunchKernelGGL(project_kernel, dim3(blocks), dim3(256), project_lds(d), s, d, ef, 0u);
}

void launch_project_nodes(const Dev& d, hipStream_t s) {
  uint32_t blocks = (d.N + kProjRows - 1) / kProjRows;
  const uint32_t cap = 8u * (d.num_cu ? d.num_cu : 256u);
  if (blocks > cap) blocks = cap;
  hipLaunchKernelGGL(project_kernel, dim3(blocks), dim3(256), project_lds(d), s, d, (const float*)nullptr, 1u);
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
  if (project_lds(d) + 1024 > kMaxLds) return -1;
  return hipFuncSetAttribute((const void*)project_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                             (int)project_lds(d)) == hipSuccess ? 0 : -1;
}

}  // namespace stgn
