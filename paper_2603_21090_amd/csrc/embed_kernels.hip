// Temporal-attention layer for a list of target rows (paper Eq. attn_detail, Sec. 3.3.4 exact
// mode, Sec. 3.6.2 "single batched kernel" over the affected set).
//
// The layer is evaluated in an algebraically re-associated form so that every dense product runs
// over |rows| instead of |rows| * k:
//     score_{h,j} = q_h . (z_j W_K,h) / sqrt(dk)      =  (W_K,h q_h / sqrt(dk)) . z_j  =  qt_h . z_j
//     o_h         = sum_j alpha_{h,j} (z_j W_V,h)     =  (sum_j alpha_{h,j} z_j) W_V,h =  zb_h W_V,h
// with z_j = [h_{u_j} | e_j | phi(t_v - t_j)] the raw gathered neighbour row.  Three kernels:
//   qproj : q = h_v W_Q(node block) + phi(0) W_Q(time block);  qt_h = q_h W_K,h^T / sqrt(dk)   (MFMA)
//   attn  : gather z_j (node row, edge row, time encoding), scores, softmax, zb_h          (HBM bound)
//   oproj : o_h = zb_h W_V,h;  h_v' = [o_1 | .. | o_H] W_O + b_O, written into the layer cache (MFMA)
#include "stgn_internal.h"
#include "mfma_gemm.h"

namespace stgn {

namespace {

constexpr uint32_t kTileRows = 64;

__device__ inline uint32_t row_count(const Dev& d, const uint32_t* count_ptr, uint32_t count_max) {
  if (!count_ptr) return count_max;
  const uint32_t n = *count_ptr;
  return n < count_max ? n : count_max;
}

// ------------------------------------------------------------------------------------------ qproj
__global__ __launch_bounds__(256) void qproj_kernel(Dev d, uint32_t layer, const uint32_t* __restrict__ rows,
                                                    const uint32_t* count_ptr, uint32_t count_max) {
  extern __shared__ float lds[];
  if (count_ptr && d.ctrl->skip) return;
  const LayerDev& L = d.L[layer];
  const Table Hin = d.H[layer];
  const uint32_t n = row_count(d, count_ptr, count_max);
  const uint32_t ntiles = (n + kTileRows - 1) / kTileRows;
  const uint32_t ldx = L.d_in2 + 1;                    // odd stride: conflict-free column reads
  const uint32_t ldq = (d.d_emb + 2) | 1u;
  float* Xs = lds;
  float* Qs = lds + kTileRows * ldx;
  const uint32_t npd = round_up(d.d_emb, 32);
  const uint32_t dk2 = round_up(d.dk, 2);
  const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
  const uint32_t rowstride = d.heads * L.Zp;

  for (uint32_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
    const uint32_t r0 = tile * kTileRows;
    // stage the input rows (zero rows past the end, zero pad column)
    for (uint32_t x = threadIdx.x; x < kTileRows * L.d_in2; x += 256) {
      const uint32_t r = x / L.d_in2, cidx = x - r * L.d_in2;
      float v = 0.0f;
      if (r0 + r < n && cidx < L.d_in) {
        const uint32_t node = rows ? rows[r0 + r] : r0 + r;
        v = Hin.base[(size_t)node * Hin.ld + cidx];
      }
      Xs[r * ldx + cidx] = v;
    }
    for (uint32_t x = threadIdx.x; x < kTileRows * (ldq - d.d_emb); x += 256) {
      const uint32_t r = x / (ldq - d.d_emb), cidx = d.d_emb + x % (ldq - d.d_emb);
      Qs[r * ldq + cidx] = 0.0f;
    }
    __syncthreads();
    // q = x W_Q(node) + c_Q
    for (uint32_t nt = wave; nt < npd / 32; nt += 4) {
      floatx16 acc[2];
      zero_acc(acc);
      mfma_tile<2>(Xs, ldx, L.d_in2, L.WQn, npd, nt * 32, acc);
      const uint32_t col = nt * 32 + mfma_col(lane);
      if (col < d.d_emb) {
        const float cq = L.cQ[col];
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
          for (int j = 0; j < 16; ++j) Qs[(rb * 32 + mfma_row(lane, j)) * ldq + col] = acc[rb][j] + cq;
      }
    }
    __syncthreads();
    // qt_h = q_h W_K,h^T / sqrt(dk)  (scale folded into the packed matrix)
    for (uint32_t h = 0; h < d.heads; ++h) {
      const float* B = L.WKT + (size_t)h * dk2 * L.Zp;
      for (uint32_t nt = wave; nt < L.Zp / 32; nt += 4) {
        floatx16 acc[2];
        zero_acc(acc);
        mfma_tile<2>(Qs + h * d.dk, ldq, dk2, B, L.Zp, nt * 32, acc);
        const uint32_t col = nt * 32 + mfma_col(lane);
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
          for (int j = 0; j < 16; ++j) {
            const uint32_t r = r0 + rb * 32 + mfma_row(lane, j);
            if (r < n) d.QT[(size_t)r * rowstride + h * L.Zp + col] = acc[rb][j];
          }
      }
    }
    __syncthreads();
  }
}

// ------------------------------------------------------------------------------------------- attn
template <int CTRL>
__device__ inline float dpp_mov(float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xF, 0xF, false));
}

// sum over the 64 lanes, result uniform
__device__ inline float wave_sum(float x) {
  x += dpp_mov<0xB1>(x);    // quad_perm [1,0,3,2]
  x += dpp_mov<0x4E>(x);    // quad_perm [2,3,0,1]
  x += dpp_mov<0x141>(x);   // row_half_mirror
  x += dpp_mov<0x140>(x);   // row_mirror: every lane of a 16-lane row holds the row sum
  const float a = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 0));
  const float b = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 16));
  const float c = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 32));
  const float e = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 48));
  return (a + b) + (c + e);
}

// cos(2 pi frac(x)) with the argument reduced in fp64: timestamps reach 1e7 and beyond
__device__ inline float cos_rev(double x) {
  const double f = __builtin_amdgcn_fract(x);
  return __builtin_amdgcn_cosf((float)f);
}

constexpr int kJC = 5;   // ring entries fetched together

template <int NI, int H>
__global__ __launch_bounds__(256) void attn_kernel(Dev d, uint32_t layer, const uint32_t* __restrict__ rows,
                                                   const uint32_t* count_ptr, uint32_t count_max) {
  if (count_ptr && d.ctrl->skip) return;
  const LayerDev& L = d.L[layer];
  const Table Hin = d.H[layer];
  const uint32_t n = row_count(d, count_ptr, count_max);
  const uint32_t lane = threadIdx.x & 63u;
  const uint32_t wave0 = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const uint32_t nwaves = (gridDim.x * blockDim.x) >> 6;
  const uint32_t d_in = L.d_in, d_e = d.d_edge, Zdim = L.Zdim, Zp = L.Zp;
  const uint32_t rowstride = d.heads * Zp;

  // per-lane column roles: 0 node row, 1 edge row, 2 time encoding, 3 padding
  int kind[NI];
  uint32_t off[NI];
  double om[NI], ph[NI];
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const uint32_t c = lane + 64u * i;
    om[i] = 0.0; ph[i] = 0.0;
    if (c < d_in) { kind[i] = 0; off[i] = c; }
    else if (c < d_in + d_e) { kind[i] = 1; off[i] = c - d_in; }
    else if (c < Zdim) { kind[i] = 2; off[i] = c - d_in - d_e; om[i] = d.om_rev[off[i]]; ph[i] = d.ph_rev[off[i]]; }
    else { kind[i] = 3; off[i] = 0; }
  }

  for (uint32_t idx = wave0; idx < n; idx += nwaves) {
    const uint32_t v = rows ? rows[idx] : idx;
    const uint32_t dg = d.deg[v];
    const uint32_t cnt = dg < d.k ? dg : d.k;
    const double tq = d.t_last[v];
    const float* qrow = d.QT + (size_t)idx * rowstride;
    float* zrow = d.ZB + (size_t)idx * rowstride;
    float qt[H][NI], acc[H][NI];
#pragma unroll
    for (int h = 0; h < H; ++h)
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        const uint32_t c = lane + 64u * i;
        qt[h][i] = (c < Zp) ? qrow[h * Zp + c] : 0.0f;
        acc[h][i] = 0.0f;
      }
    float mrun[H], lrun[H];
#pragma unroll
    for (int h = 0; h < H; ++h) { mrun[h] = -INFINITY; lrun[h] = 0.0f; }

    const RingEntry* ring = d.ring + (size_t)v * d.k;
    for (uint32_t j0 = 0; j0 < cnt; j0 += kJC) {
      float z[kJC][NI];
      float s[kJC][H];
#pragma unroll
      for (int jc = 0; jc < kJC; ++jc) {
        const uint32_t j = j0 + jc;
        const bool valid = j < cnt;
        uint32_t nbr = 0, eid = 0;
        double dt = 0.0;
        if (valid) {
          const uint32_t pos = dg - 1u - j;           // most recent first
          const RingEntry e = ring[pos % d.k];
          nbr = __builtin_amdgcn_readfirstlane(e.nbr);
          eid = __builtin_amdgcn_readfirstlane(e.eid);
          dt = tq - e.t;
        }
        const float* hrow = Hin.base + (size_t)nbr * Hin.ld;
        const float* erow = d.efeat.base + (size_t)eid * d.efeat.ld;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
          float zz = 0.0f;
          if (valid) {
            if (kind[i] == 0) zz = hrow[off[i]];
            else if (kind[i] == 1) zz = erow[off[i]];
            else if (kind[i] == 2) zz = cos_rev(om[i] * dt + ph[i]);
          }
          z[jc][i] = zz;
        }
      }
#pragma unroll
      for (int jc = 0; jc < kJC; ++jc)
#pragma unroll
        for (int h = 0; h < H; ++h) {
          float p = 0.0f;
#pragma unroll
          for (int i = 0; i < NI; ++i) p = fmaf(qt[h][i], z[jc][i], p);
          p = wave_sum(p);
          s[jc][h] = (j0 + jc < cnt) ? p : -INFINITY;
        }
#pragma unroll
      for (int h = 0; h < H; ++h) {
        float mnew = mrun[h];
#pragma unroll
        for (int jc = 0; jc < kJC; ++jc) mnew = fmaxf(mnew, s[jc][h]);
        const float scale = __expf(mrun[h] - mnew);
        float lsum = lrun[h] * scale;
#pragma unroll
        for (int i = 0; i < NI; ++i) acc[h][i] *= scale;
#pragma unroll
        for (int jc = 0; jc < kJC; ++jc) {
          const float p = __expf(s[jc][h] - mnew);
          lsum += p;
#pragma unroll
          for (int i = 0; i < NI; ++i) acc[h][i] = fmaf(p, z[jc][i], acc[h][i]);
        }
        mrun[h] = mnew;
        lrun[h] = lsum;
      }
    }
#pragma unroll
    for (int h = 0; h < H; ++h) {
      const float inv = cnt ? 1.0f / lrun[h] : 0.0f;
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        const uint32_t c = lane + 64u * i;
        if (c < Zp) zrow[h * Zp + c] = acc[h][i] * inv;
      }
    }
  }
}

// ------------------------------------------------------------------------------------------ oproj
constexpr uint32_t kKC = 64;     // K chunk staged through LDS

__global__ __launch_bounds__(256) void oproj_kernel(Dev d, uint32_t layer, const uint32_t* __restrict__ rows,
                                                    const uint32_t* count_ptr, uint32_t count_max) {
  extern __shared__ float lds[];
  if (count_ptr && d.ctrl->skip) return;
  const LayerDev& L = d.L[layer];
  const Table Hout = d.H[layer + 1];
  const uint32_t n = row_count(d, count_ptr, count_max);
  const uint32_t ntiles = (n + kTileRows - 1) / kTileRows;
  const uint32_t ldz = kKC + 1;
  const uint32_t ldo = (d.d_emb + 2) | 1u;
  float* Zs = lds;
  float* Os = lds + kTileRows * ldz;
  const uint32_t npk = round_up(d.dk, 32), npd = round_up(d.d_emb, 32);
  const uint32_t NT = npk / 32;
  const uint32_t Zdim2 = round_up(L.Zdim, 2);
  const uint32_t d2 = round_up(d.d_emb, 2);
  const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
  const uint32_t rowstride = d.heads * L.Zp;

  for (uint32_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
    const uint32_t r0 = tile * kTileRows;
    for (uint32_t x = threadIdx.x; x < kTileRows * (ldo - d.d_emb); x += 256) {
      const uint32_t r = x / (ldo - d.d_emb), cidx = d.d_emb + x % (ldo - d.d_emb);
      Os[r * ldo + cidx] = 0.0f;
    }
    for (uint32_t h = 0; h < d.heads; ++h) {
      // (row block, column tile) pairs of the 64 x npk head output, two per wave at most
      floatx16 acc[2][1];
      zero_acc(acc[0]);
      zero_acc(acc[1]);
      const float* B = L.WV + (size_t)h * Zdim2 * npk;
      for (uint32_t kc0 = 0; kc0 < Zdim2; kc0 += kKC) {
        const uint32_t kc = (Zdim2 - kc0) < kKC ? (Zdim2 - kc0) : kKC;
        for (uint32_t x = threadIdx.x; x < kTileRows * kKC; x += 256) {
          const uint32_t r = x / kKC, cidx = x - r * kKC;
          float v = 0.0f;
          if (r0 + r < n && cidx < kc) v = d.ZB[(size_t)(r0 + r) * rowstride + h * L.Zp + kc0 + cidx];
          Zs[r * ldz + cidx] = v;
        }
        __syncthreads();
#pragma unroll
        for (int pi = 0; pi < 2; ++pi) {
          const uint32_t p = wave + 4u * pi;
          if (p < 2 * NT) {
            const uint32_t rb = p / NT, nt = p - rb * NT;
            mfma_tile<1>(Zs + rb * 32 * ldz, ldz, kc, B + (size_t)kc0 * npk, npk, nt * 32, acc[pi]);
          }
        }
        __syncthreads();
      }
#pragma unroll
      for (int pi = 0; pi < 2; ++pi) {
        const uint32_t p = wave + 4u * pi;
        if (p < 2 * NT) {
          const uint32_t rb = p / NT, nt = p - rb * NT;
          const uint32_t col = nt * 32 + mfma_col(lane);
          if (col < d.dk) {
#pragma unroll
            for (int j = 0; j < 16; ++j) Os[(rb * 32 + mfma_row(lane, j)) * ldo + h * d.dk + col] = acc[pi][0][j];
          }
        }
      }
    }
    __syncthreads();
    // h' = o W_O + b_O, written into the layer cache
    for (uint32_t nt = wave; nt < npd / 32; nt += 4) {
      floatx16 acc[2];
      zero_acc(acc);
      mfma_tile<2>(Os, ldo, d2, L.WO, npd, nt * 32, acc);
      const uint32_t col = nt * 32 + mfma_col(lane);
      if (col < d.d_emb) {
        const float b = L.bO[col];
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
          for (int j = 0; j < 16; ++j) {
            const uint32_t r = r0 + rb * 32 + mfma_row(lane, j);
            if (r < n) {
              const uint32_t node = rows ? rows[r] : r;
              Hout.base[(size_t)node * Hout.ld + col] = acc[rb][j] + b;
            }
          }
      }
    }
    __syncthreads();
  }
}

__global__ void gather_rows_kernel(Table T, uint32_t width, uint32_t n, const uint32_t* __restrict__ nodes,
                                   float* __restrict__ out) {
  const size_t tot = (size_t)n * width;
  for (size_t x = (size_t)blockIdx.x * blockDim.x + threadIdx.x; x < tot; x += (size_t)gridDim.x * blockDim.x) {
    const size_t i = x / width, c = x - i * width;
    out[x] = T.base[(size_t)nodes[i] * T.ld + c];
  }
}

uint32_t persistent_blocks(uint32_t count_max, uint32_t per_block) {
  uint64_t b = ((uint64_t)count_max + per_block - 1) / per_block;
  if (b < 1) b = 1;
  return b > 2048 ? 2048u : (uint32_t)b;
}

template <int NI>
void launch_attn_h(const Dev& d, hipStream_t s, uint32_t layer, const uint32_t* rows, const uint32_t* cp, uint32_t cm) {
  const uint32_t blocks = persistent_blocks(cm, 4);   // one wave per row, 4 waves per block
  switch (d.heads) {
    case 1: hipLaunchKernelGGL((attn_kernel<NI, 1>), dim3(blocks), dim3(256), 0, s, d, layer, rows, cp, cm); break;
    case 2: hipLaunchKernelGGL((attn_kernel<NI, 2>), dim3(blocks), dim3(256), 0, s, d, layer, rows, cp, cm); break;
    default: hipLaunchKernelGGL((attn_kernel<NI, 4>), dim3(blocks), dim3(256), 0, s, d, layer, rows, cp, cm); break;
  }
}

size_t qproj_lds(const Dev& d, uint32_t layer) {
  const uint32_t ldx = d.L[layer].d_in2 + 1, ldq = (d.d_emb + 2) | 1u;
  return (size_t)kTileRows * (ldx + ldq) * sizeof(float);
}
size_t oproj_lds(const Dev& d) {
  const uint32_t ldz = kKC + 1, ldo = (d.d_emb + 2) | 1u;
  return (size_t)kTileRows * (ldz + ldo) * sizeof(float);
}

}  // namespace

int attn_supported(uint32_t Zdim, uint32_t heads) {
  const uint32_t ni = (Zdim + 63) / 64;
  return ni >= 1 && ni <= 8 && (heads == 1 || heads == 2 || heads == 4);
}

void launch_qproj(const Dev& d, hipStream_t s, uint32_t layer, const uint32_t* rows, const uint32_t* cp, uint32_t cm) {
  hipLaunchKernelGGL(qproj_kernel, dim3(persistent_blocks(cm, kTileRows)), dim3(256), qproj_lds(d, layer), s, d, layer,
                     rows, cp, cm);
}

void launch_attn(const Dev& d, hipStream_t s, uint32_t layer, const uint32_t* rows, const uint32_t* cp, uint32_t cm) {
  switch ((d.L[layer].Zdim + 63) / 64) {
    case 1: launch_attn_h<1>(d, s, layer, rows, cp, cm); break;
    case 2: launch_attn_h<2>(d, s, layer, rows, cp, cm); break;
    case 3: launch_attn_h<3>(d, s, layer, rows, cp, cm); break;
    case 4: launch_attn_h<4>(d, s, layer, rows, cp, cm); break;
    case 5: launch_attn_h<5>(d, s, layer, rows, cp, cm); break;
    case 6: launch_attn_h<6>(d, s, layer, rows, cp, cm); break;
    case 7: launch_attn_h<7>(d, s, layer, rows, cp, cm); break;
    default: launch_attn_h<8>(d, s, layer, rows, cp, cm); break;
  }
}

void launch_oproj(const Dev& d, hipStream_t s, uint32_t layer, const uint32_t* rows, const uint32_t* cp, uint32_t cm) {
  hipLaunchKernelGGL(oproj_kernel, dim3(persistent_blocks(cm, kTileRows)), dim3(256), oproj_lds(d), s, d, layer, rows,
                     cp, cm);
}

void launch_gather_rows(const Dev& d, hipStream_t s, uint32_t layer, uint32_t n, const uint32_t* nodes, float* out) {
  const uint32_t width = layer == 0 ? d.d0 : d.d_emb;
  uint64_t blocks = ((uint64_t)n * width + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(gather_rows_kernel, dim3((uint32_t)blocks), dim3(256), 0, s, d.H[layer], width, n, nodes, out);
}

int setup_embed_attributes(const Dev& d) {
  size_t q = 0;
  for (uint32_t l = 0; l < d.layers; ++l) q = qproj_lds(d, l) > q ? qproj_lds(d, l) : q;
  const size_t o = oproj_lds(d);
  if (q > kMaxLds || o > kMaxLds) return -1;
  hipError_t e1 = hipFuncSetAttribute((const void*)qproj_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)q);
  hipError_t e2 = hipFuncSetAttribute((const void*)oproj_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)o);
  return (e1 == hipSuccess && e2 == hipSuccess) ? 0 : -1;
}

}  // namespace stgn
