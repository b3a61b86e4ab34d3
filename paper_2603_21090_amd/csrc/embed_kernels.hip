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
// qt and zb rows use the slot layout of LayerDev (segments padded to 64 floats).
#include "stgn_internal.h"
#include "mfma_gemm.h"

namespace stgn {

namespace {

__device__ inline uint32_t row_count(const Dev& d, const uint32_t* count_ptr, uint32_t count_max) {
  if (!count_ptr) return count_max;
  const uint32_t n = *count_ptr;
  return n < count_max ? n : count_max;
}

// Cooperative load of TM rows x `width` floats (row r from table T at node rows[r0 + r]) into LDS
// with stride lds_ld; rows past n and columns in [width, width_pad) are zero.  Loads are issued in
// batches of 4 per thread so their latencies overlap.
// The row ids go through LDS first (s_node, TM entries), then every thread issues four
// unconditional 16-byte loads back to back (table rows are 128-byte aligned and zero padded).
// Ends with a barrier.
template <uint32_t TM>
__device__ inline void stage_rows(float* dst, uint32_t lds_ld, uint32_t* s_node, const Table T,
                                  const uint32_t* __restrict__ rows, uint32_t r0, uint32_t n, uint32_t width,
                                  uint32_t width_pad) {
  if (threadIdx.x < TM) {
    const uint32_t r = r0 + threadIdx.x;
    s_node[threadIdx.x] = r < n ? (rows ? rows[r] : r) : 0xFFFFFFFFu;
  }
  __syncthreads();
  const uint32_t qpr = (width + 3) / 4;              // 16-byte quads per row
  const uint32_t total = TM * qpr;
  for (uint32_t x0 = threadIdx.x; x0 < total; x0 += 256u * 4u) {
    float4 v[4];
    uint32_t rr[4], cc[4];
    bool ok[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      uint32_t x = x0 + 256u * e;
      ok[e] = x < total;
      x = ok[e] ? x : 0u;
      const uint32_t r = x / qpr, q = x - r * qpr;
      const uint32_t node = s_node[r];
      rr[e] = r; cc[e] = 4u * q;
      const bool live = node != 0xFFFFFFFFu;
      v[e] = *reinterpret_cast<const float4*>(T.base + (size_t)(live ? node : 0u) * T.ld + 4u * q);
      if (!live) v[e] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (ok[e]) {
        float* p = dst + rr[e] * lds_ld + cc[e];
        const uint32_t c = cc[e];
        if (c + 0 < width_pad) p[0] = v[e].x;
        if (c + 1 < width_pad) p[1] = v[e].y;
        if (c + 2 < width_pad) p[2] = v[e].z;
        if (c + 3 < width_pad) p[3] = v[e].w;
      }
  }
  __syncthreads();
}

// ------------------------------------------------------------------------------------------ qproj
template <int RB>
__global__ __launch_bounds__(256) void qproj_kernel(Dev d, uint32_t layer, const uint32_t* __restrict__ rows,
                                                    const uint32_t* count_ptr, uint32_t count_max) {
  extern __shared__ float lds[];
  __shared__ uint32_t s_node[64];
  if (count_ptr && d.ctrl->skip) return;
  constexpr uint32_t TM = 32u * RB;
  const LayerDev& L = d.L[layer];
  const Table Hin = d.H[layer];
  const uint32_t n = row_count(d, count_ptr, count_max);
  const uint32_t ntiles = (n + TM - 1) / TM;
  const uint32_t ldx = L.d_in2 + 1;                    // odd stride: conflict-free column reads
  const uint32_t ldq = (d.d_emb + 2) | 1u;
  float* Xs = lds;
  float* Qs = lds + TM * ldx;
  const uint32_t npd = round_up(d.d_emb, 32);
  const uint32_t dk2 = round_up(d.dk, 2);
  const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
  const uint32_t rowstride = d.heads * L.Zp;

  const uint32_t ksteps = dk2 >> 1;                    // k-steps of one qt tile
  const uint32_t nqt = L.nqt;
  // one qt tile: B chunk(s) `bq` already in flight for k-steps [0, kBU)
  auto qt_tile = [&](uint32_t ti, float (&bq)[kBU], uint32_t r0) {
    const uint32_t h = L.qt_h[ti], nt = L.qt_nt[ti];
    floatx16 acc[RB];
    zero_acc(acc);
    mfma_tile_pre<RB>(Qs + h * d.dk, ldq, dk2, L.WKT + (size_t)h * dk2 * L.Zp, L.Zp, nt * 32, acc, bq);
    const uint32_t col = nt * 32 + mfma_col(lane);
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        const uint32_t r = r0 + rb * 32 + mfma_row(lane, j);
        if (r < n) d.QT[(size_t)r * rowstride + h * L.Zp + col] = acc[rb][j];
      }
  };
  auto qt_prefetch = [&](uint32_t ti, float (&bq)[kBU]) {
    const uint32_t h = L.qt_h[ti], nt = L.qt_nt[ti];
    load_b<kBU>(b_lane_ptr(L.WKT + (size_t)h * dk2 * L.Zp, L.Zp, nt * 32), L.Zp, 0, ksteps, bq);
  };

  for (uint32_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
    const uint32_t r0 = tile * TM;
    // weights of the first product are requested before the rows are staged
    float b1[kBU];
    const bool has1 = wave < npd / 32;
    if (has1) load_b<kBU>(b_lane_ptr(L.WQn, npd, wave * 32), npd, 0, L.d_in2 >> 1, b1);
    for (uint32_t x = threadIdx.x; x < TM * (ldq - d.d_emb); x += 256) {
      const uint32_t r = x / (ldq - d.d_emb), cidx = d.d_emb + x % (ldq - d.d_emb);
      Qs[r * ldq + cidx] = 0.0f;
    }
    stage_rows<TM>(Xs, ldx, s_node, Hin, rows, r0, n, L.d_in, L.d_in2);
    // q = x W_Q(node) + c_Q
    float bA[kBU], bB[kBU];
    if (wave < nqt) qt_prefetch(wave, bA);
    for (uint32_t nt = wave; nt < npd / 32; nt += 4) {
      floatx16 acc[RB];
      zero_acc(acc);
      if (nt == wave) mfma_tile_pre<RB>(Xs, ldx, L.d_in2, L.WQn, npd, nt * 32, acc, b1);
      else mfma_tile<RB>(Xs, ldx, L.d_in2, L.WQn, npd, nt * 32, acc);
      const uint32_t col = nt * 32 + mfma_col(lane);
      if (col < d.d_emb) {
        const float cq = L.cQ[col];
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
          for (int j = 0; j < 16; ++j) Qs[(rb * 32 + mfma_row(lane, j)) * ldq + col] = acc[rb][j] + cq;
      }
    }
    __syncthreads();
    // qt_h = q_h W_K,h^T / sqrt(dk)  (scale folded into the packed matrix).  Tiles that lie wholly
    // in slot padding are not in the list -- the attention kernel never reads them.  The weights of
    // the next tile are in flight while the current one is multiplied.
    for (uint32_t ti = wave; ti < nqt; ti += 8) {
      if (ti + 4 < nqt) qt_prefetch(ti + 4, bB);
      qt_tile(ti, bA, r0);
      if (ti + 4 >= nqt) break;
      if (ti + 8 < nqt) qt_prefetch(ti + 8, bA);
      qt_tile(ti + 4, bB, r0);
    }
    __syncthreads();
  }
}

// ------------------------------------------------------------------------------------------- attn
template <int CTRL>
__device__ inline float dpp_mov(float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xF, 0xF, false));
}

// sum over each 16-lane row; every lane of a row receives its row's sum
__device__ inline float row16_sum(float x) {
  x += dpp_mov<0xB1>(x);    // quad_perm [1,0,3,2]
  x += dpp_mov<0x4E>(x);    // quad_perm [2,3,0,1]
  x += dpp_mov<0x141>(x);   // row_half_mirror
  x += dpp_mov<0x140>(x);   // row_mirror
  return x;
}

// cos(2 pi frac(x)) with the argument reduced in fp64: timestamps reach 1e7 and beyond
__device__ inline float cos_rev(double x) {
  const double f = __builtin_amdgcn_fract(x);
  return __builtin_amdgcn_cosf((float)f);
}

__device__ inline float dot4(const float4 a, const float4 b, float acc) {
  acc = fmaf(a.x, b.x, acc);
  acc = fmaf(a.y, b.y, acc);
  acc = fmaf(a.z, b.z, acc);
  return fmaf(a.w, b.w, acc);
}

// One wave serves four target rows: 16 lanes per row, each lane owns one float4 of every slot.
// NS slots in total, the last NT of them time-encoding slots; JC ring entries are fetched together.
template <int NS, int NT, int H, int JC>
__global__ __launch_bounds__(256) void attn_kernel(Dev d, uint32_t layer, const uint32_t* __restrict__ rows,
                                                   const uint32_t* count_ptr, uint32_t count_max) {
  if (count_ptr && d.ctrl->skip) return;
  const LayerDev& L = d.L[layer];
  const Table Hin = d.H[layer];
  const uint32_t n = row_count(d, count_ptr, count_max);
  const uint32_t lane = threadIdx.x & 63u, sub = lane & 15u, grp = lane >> 4;
  const uint32_t wave0 = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const uint32_t nwaves = (gridDim.x * blockDim.x) >> 6;
  const uint32_t Zp = L.Zp, rowstride = d.heads * Zp;
  const uint32_t k = d.k;
  constexpr int NG = NS - NT;                 // gathered (node / edge) slots

  bool lane_ok[NS];
#pragma unroll
  for (int s = 0; s < NS; ++s) lane_ok[s] = 4u * sub < L.valid[s];
  // time-encoding parameters of this lane's four columns in each time slot (omega, phase in revolutions)
  double om[NT][4], ph[NT][4];
  bool tok[NT][4];
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const uint32_t q = (uint32_t)t * kSlot + 4u * sub + c;
      tok[t][c] = q < d.d_time;
      om[t][c] = tok[t][c] ? d.om_rev[q] : 0.0;
      ph[t][c] = tok[t][c] ? d.ph_rev[q] : 0.0;
    }

  for (uint32_t base = wave0 * 4u; base < n; base += nwaves * 4u) {
    const uint32_t idx = base + grp;
    const bool act = idx < n;
    const uint32_t v = act ? (rows ? rows[idx] : idx) : 0u;
    const uint32_t dg = act ? d.deg[v] : 0u;
    const uint32_t cnt = dg < k ? dg : k;
    const double tq = d.t_last[v];
    const float* qrow = d.QT + (size_t)idx * rowstride;
    float4 qt[H][NS], acc[H][NS];
#pragma unroll
    for (int h = 0; h < H; ++h)
#pragma unroll
      for (int s = 0; s < NS; ++s) {
        qt[h][s] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (act && lane_ok[s]) qt[h][s] = *reinterpret_cast<const float4*>(qrow + h * Zp + s * kSlot + 4u * sub);
        acc[h][s] = make_float4(0.f, 0.f, 0.f, 0.f);
      }
    float mrun[H], lrun[H];
#pragma unroll
    for (int h = 0; h < H; ++h) { mrun[h] = -INFINITY; lrun[h] = 0.0f; }

    // largest entry count among the wave's four rows (uniform loop bound)
    uint32_t cmax = (uint32_t)__builtin_amdgcn_readlane((int)cnt, 0);
    cmax = max(cmax, (uint32_t)__builtin_amdgcn_readlane((int)cnt, 16));
    cmax = max(cmax, (uint32_t)__builtin_amdgcn_readlane((int)cnt, 32));
    cmax = max(cmax, (uint32_t)__builtin_amdgcn_readlane((int)cnt, 48));

    const RingEntry* ring = d.ring + (size_t)v * k;
    int slot = cnt ? (int)((dg - 1u) % k) : 0;            // ring slot of the most recent entry
    for (uint32_t j0 = 0; j0 < cmax; j0 += JC) {
      float4 z[JC][NS];
      bool vj[JC];
#pragma unroll
      for (int jc = 0; jc < JC; ++jc) {
        vj[jc] = j0 + jc < cnt;
        uint32_t nbr = 0, eid = 0;
        double dt = 0.0;
        if (vj[jc]) {
          const RingEntry e = ring[slot];
          nbr = e.nbr; eid = e.eid; dt = tq - e.t;
          slot = slot == 0 ? (int)k - 1 : slot - 1;
        }
        const float* hrow = Hin.base + (size_t)nbr * Hin.ld + 4u * sub;
        const float* erow = d.efeat.base + (size_t)eid * d.efeat.ld + 4u * sub;
#pragma unroll
        for (int s = 0; s < NG; ++s) {
          float4 zz = make_float4(0.f, 0.f, 0.f, 0.f);
          if (vj[jc] && lane_ok[s]) {
            const float* p = (L.kind[s] == 0 ? hrow : erow) + L.segoff[s];
            zz = *reinterpret_cast<const float4*>(p);
          }
          z[jc][s] = zz;
        }
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          float4 zz;
          zz.x = (vj[jc] && tok[t][0]) ? cos_rev(om[t][0] * dt + ph[t][0]) : 0.0f;
          zz.y = (vj[jc] && tok[t][1]) ? cos_rev(om[t][1] * dt + ph[t][1]) : 0.0f;
          zz.z = (vj[jc] && tok[t][2]) ? cos_rev(om[t][2] * dt + ph[t][2]) : 0.0f;
          zz.w = (vj[jc] && tok[t][3]) ? cos_rev(om[t][3] * dt + ph[t][3]) : 0.0f;
          z[jc][NG + t] = zz;
        }
      }
      float sc[JC][H];
#pragma unroll
      for (int jc = 0; jc < JC; ++jc)
#pragma unroll
        for (int h = 0; h < H; ++h) {
          float p = 0.0f;
#pragma unroll
          for (int s = 0; s < NS; ++s) p = dot4(qt[h][s], z[jc][s], p);
          p = row16_sum(p);
          sc[jc][h] = vj[jc] ? p : -INFINITY;
        }
#pragma unroll
      for (int h = 0; h < H; ++h) {
        float mnew = mrun[h];
#pragma unroll
        for (int jc = 0; jc < JC; ++jc) mnew = fmaxf(mnew, sc[jc][h]);
        // rows with no entry in this chunk keep their state (mnew may still be -inf for them)
        const float scale = (mnew == -INFINITY) ? 1.0f : __expf(mrun[h] - mnew);
        float lsum = lrun[h] * scale;
#pragma unroll
        for (int s = 0; s < NS; ++s) {
          acc[h][s].x *= scale; acc[h][s].y *= scale; acc[h][s].z *= scale; acc[h][s].w *= scale;
        }
#pragma unroll
        for (int jc = 0; jc < JC; ++jc) {
          const float p = vj[jc] ? __expf(sc[jc][h] - mnew) : 0.0f;
          lsum += p;
#pragma unroll
          for (int s = 0; s < NS; ++s) {
            acc[h][s].x = fmaf(p, z[jc][s].x, acc[h][s].x);
            acc[h][s].y = fmaf(p, z[jc][s].y, acc[h][s].y);
            acc[h][s].z = fmaf(p, z[jc][s].z, acc[h][s].z);
            acc[h][s].w = fmaf(p, z[jc][s].w, acc[h][s].w);
          }
        }
        mrun[h] = mnew;
        lrun[h] = lsum;
      }
    }
    if (act) {
      float* zrow = d.ZB + (size_t)idx * rowstride;
#pragma unroll
      for (int h = 0; h < H; ++h) {
        const float inv = cnt ? 1.0f / lrun[h] : 0.0f;
#pragma unroll
        for (int s = 0; s < NS; ++s)
          if (lane_ok[s]) {
            float4 o = acc[h][s];
            o.x *= inv; o.y *= inv; o.z *= inv; o.w *= inv;
            *reinterpret_cast<float4*>(zrow + h * Zp + s * kSlot + 4u * sub) = o;
          }
      }
    }
  }
}

// ------------------------------------------------------------------------------------------ oproj
constexpr int kMaxPairsCap = 4;  // (head, column tile) accumulator groups per wave, at most

// Wave w owns the (head, 32-column tile) pairs w, w + 4, ...; each pair accumulates RB row blocks.
// The zb rows of the tile are staged through LDS one slot (64 k values) at a time, double buffered;
// with one pair per wave (PP == 1) the weights of the next slot are also kept in flight.
template <int RB, int H, int PP>
__global__ __launch_bounds__(256) void oproj_kernel(Dev d, uint32_t layer, const uint32_t* __restrict__ rows,
                                                    const uint32_t* count_ptr, uint32_t count_max) {
  extern __shared__ float lds[];
  __shared__ uint32_t s_node[64];
  if (count_ptr && d.ctrl->skip) return;
  constexpr uint32_t TM = 32u * RB;
  constexpr uint32_t ldz = kSlot + 1;
  constexpr uint32_t kStage = H * TM * kSlot / 256;   // staged elements per thread and slot
  const LayerDev& L = d.L[layer];
  const Table Hout = d.H[layer + 1];
  const uint32_t n = row_count(d, count_ptr, count_max);
  const uint32_t ntiles = (n + TM - 1) / TM;
  const uint32_t ldo = (d.d_emb + 2) | 1u;
  float* Zs = lds;                                   // [2][H][TM][ldz]
  float* Os = lds + 2 * H * TM * ldz;                // [TM][ldo]
  const uint32_t npk = round_up(d.dk, 32), npd = round_up(d.d_emb, 32);
  const uint32_t NT = npk / 32;
  const uint32_t npairs = H * NT;
  const uint32_t d2 = round_up(d.d_emb, 2);
  const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
  const uint32_t rowstride = d.heads * L.Zp;
  const uint32_t nchunks = L.ns;                     // one K chunk per slot

  float stage[kStage];
  uint32_t r0 = 0;
  auto load_chunk = [&](uint32_t c) {
    const uint32_t kc = round_up(L.valid[c], 2);
#pragma unroll
    for (uint32_t e = 0; e < kStage; ++e) {
      const uint32_t x = threadIdx.x + 256u * e;
      const uint32_t cidx = x % kSlot, r = (x / kSlot) % TM, h = x / (kSlot * TM);
      float v = 0.0f;
      if (r0 + r < n && cidx < kc) v = d.ZB[(size_t)(r0 + r) * rowstride + h * L.Zp + c * kSlot + cidx];
      stage[e] = v;
    }
  };
  auto store_chunk = [&](uint32_t buf) {
#pragma unroll
    for (uint32_t e = 0; e < kStage; ++e) {
      const uint32_t x = threadIdx.x + 256u * e;
      const uint32_t cidx = x % kSlot, r = (x / kSlot) % TM, h = x / (kSlot * TM);
      Zs[((buf * H + h) * TM + r) * ldz + cidx] = stage[e];
    }
  };
  // B pointer of pair p at slot c, and the A tile it multiplies
  auto pair_b = [&](uint32_t p, uint32_t c) {
    const uint32_t h = p / NT, nt = p - h * NT;
    return b_lane_ptr(L.WV + ((size_t)h * L.Zp + c * kSlot) * npk, npk, nt * 32);
  };
  auto pair_a = [&](uint32_t p, uint32_t c) {
    const uint32_t h = p / NT;
    return a_lane_ptr(Zs + (((c & 1u) * H + h) * TM) * ldz, ldz);
  };

  for (uint32_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
    r0 = tile * TM;
    if (threadIdx.x < TM) {
      const uint32_t r = r0 + threadIdx.x;
      s_node[threadIdx.x] = r < n ? (rows ? rows[r] : r) : 0u;
    }
    for (uint32_t x = threadIdx.x; x < TM * (ldo - d.d_emb); x += 256) {
      const uint32_t r = x / (ldo - d.d_emb), cidx = d.d_emb + x % (ldo - d.d_emb);
      Os[r * ldo + cidx] = 0.0f;
    }
    floatx16 acc[PP][RB];
#pragma unroll
    for (int pi = 0; pi < PP; ++pi) zero_acc(acc[pi]);
    load_chunk(0);
    store_chunk(0);
    if constexpr (PP == 1) {
      float bA[kBU], bB[kBU];
      const bool mine = wave < npairs;
      if (mine) load_b<kBU>(pair_b(wave, 0), npk, 0, round_up(L.valid[0], 2) >> 1, bA);
      __syncthreads();
      for (uint32_t c = 0; c < nchunks; c += 2) {
        const uint32_t st0 = round_up(L.valid[c], 2) >> 1;
        if (c + 1 < nchunks) {
          load_chunk(c + 1);
          if (mine) load_b<kBU>(pair_b(wave, c + 1), npk, 0, round_up(L.valid[c + 1], 2) >> 1, bB);
        }
        if (mine) mfma_steps<RB, kBU>(pair_a(wave, c), ldz, 0, st0, bA, acc[0]);
        if (c + 1 < nchunks) store_chunk((c + 1) & 1u);
        __syncthreads();
        if (c + 1 >= nchunks) break;
        const uint32_t st1 = round_up(L.valid[c + 1], 2) >> 1;
        if (c + 2 < nchunks) {
          load_chunk(c + 2);
          if (mine) load_b<kBU>(pair_b(wave, c + 2), npk, 0, round_up(L.valid[c + 2], 2) >> 1, bA);
        }
        if (mine) mfma_steps<RB, kBU>(pair_a(wave, c + 1), ldz, 0, st1, bB, acc[0]);
        if (c + 2 < nchunks) store_chunk(c & 1u);
        __syncthreads();
      }
    } else {
      __syncthreads();
      for (uint32_t c = 0; c < nchunks; ++c) {
        if (c + 1 < nchunks) load_chunk(c + 1);
        const uint32_t kc = round_up(L.valid[c], 2);
#pragma unroll
        for (int pi = 0; pi < PP; ++pi) {
          const uint32_t p = wave + 4u * pi;
          if (p < npairs) {
            const uint32_t h = p / NT, nt = p - h * NT;
            mfma_tile<RB>(Zs + (((c & 1u) * H + h) * TM) * ldz, ldz, kc, L.WV + ((size_t)h * L.Zp + c * kSlot) * npk, npk,
                          nt * 32, acc[pi]);
          }
        }
        if (c + 1 < nchunks) store_chunk((c + 1) & 1u);
        __syncthreads();
      }
    }
    // weights of the output projection are requested before the head outputs are exchanged
    float bo[kBU];
    const bool haso = wave < npd / 32;
    if (haso) load_b<kBU>(b_lane_ptr(L.WO, npd, wave * 32), npd, 0, d2 >> 1, bo);
#pragma unroll
    for (int pi = 0; pi < PP; ++pi) {
      const uint32_t p = wave + 4u * pi;
      if (p < npairs) {
        const uint32_t h = p / NT, nt = p - h * NT;
        const uint32_t col = nt * 32 + mfma_col(lane);
        if (col < d.dk) {
#pragma unroll
          for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int j = 0; j < 16; ++j) Os[(rb * 32 + mfma_row(lane, j)) * ldo + h * d.dk + col] = acc[pi][rb][j];
        }
      }
    }
    __syncthreads();
    // h' = o W_O + b_O, written into the layer cache
    for (uint32_t nt = wave; nt < npd / 32; nt += 4) {
      floatx16 acc2[RB];
      zero_acc(acc2);
      if (nt == wave) mfma_tile_pre<RB>(Os, ldo, d2, L.WO, npd, nt * 32, acc2, bo);
      else mfma_tile<RB>(Os, ldo, d2, L.WO, npd, nt * 32, acc2);
      const uint32_t col = nt * 32 + mfma_col(lane);
      if (col < d.d_emb) {
        const float b = L.bO[col];
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
          for (int j = 0; j < 16; ++j) {
            const uint32_t r = r0 + rb * 32 + mfma_row(lane, j);
            if (r < n) {
              const uint32_t node = s_node[rb * 32 + mfma_row(lane, j)];
              Hout.base[(size_t)node * Hout.ld + col] = acc2[rb][j] + b;
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

// ---- attn dispatch: (slots, time slots, heads, chunk)
template <int NS, int NT, int JC>
void launch_attn_h(const Dev& d, hipStream_t s, uint32_t layer, const uint32_t* rows, const uint32_t* cp, uint32_t cm) {
  const uint32_t blocks = persistent_blocks(cm, 16);   // four rows per wave, four waves per block
  switch (d.heads) {
    case 1: hipLaunchKernelGGL((attn_kernel<NS, NT, 1, JC>), dim3(blocks), dim3(256), 0, s, d, layer, rows, cp, cm); break;
    case 2: hipLaunchKernelGGL((attn_kernel<NS, NT, 2, JC>), dim3(blocks), dim3(256), 0, s, d, layer, rows, cp, cm); break;
    default: hipLaunchKernelGGL((attn_kernel<NS, NT, 4, JC>), dim3(blocks), dim3(256), 0, s, d, layer, rows, cp, cm); break;
  }
}

template <int NS, int NT>
void launch_attn_nt(const Dev& d, hipStream_t s, uint32_t layer, const uint32_t* rows, const uint32_t* cp, uint32_t cm) {
  // entries in flight per row: bounded by registers (JC * NS float4 per lane)
  if (NS * d.heads <= 10) launch_attn_h<NS, NT, 4>(d, s, layer, rows, cp, cm);
  else launch_attn_h<NS, NT, 2>(d, s, layer, rows, cp, cm);
}

template <int NS>
void launch_attn_ns(const Dev& d, hipStream_t s, uint32_t layer, const uint32_t* rows, const uint32_t* cp, uint32_t cm) {
  if constexpr (NS >= 3) {
    if (d.L[layer].nt == 2) { launch_attn_nt<NS, 2>(d, s, layer, rows, cp, cm); return; }
  }
  launch_attn_nt<NS, 1>(d, s, layer, rows, cp, cm);
}

// rows per workgroup tile: small graphs get 32-row tiles so that the chip still sees enough workgroups
uint32_t tile_rb(const Dev& d) { return d.N < 65536u ? 1u : 2u; }

size_t qproj_lds(const Dev& d, uint32_t layer, uint32_t rb) {
  const uint32_t ldx = d.L[layer].d_in2 + 1, ldq = (d.d_emb + 2) | 1u;
  return (size_t)32 * rb * (ldx + ldq) * sizeof(float);
}
size_t oproj_lds(const Dev& d, uint32_t rb) {
  const uint32_t ldz = kSlot + 1, ldo = (d.d_emb + 2) | 1u;
  return (size_t)32 * rb * (2 * d.heads * ldz + ldo) * sizeof(float);
}

uint32_t oproj_pairs_per_wave(const Dev& d) {
  const uint32_t pairs = d.heads * (round_up(d.dk, 32) / 32);
  const uint32_t need = (pairs + 3) / 4;
  return need <= 1 ? 1 : need <= 2 ? 2 : 4;
}

// applies `f` to the oproj instantiation selected by (heads, pairs per wave)
template <int RB, class F>
void with_oproj(const Dev& d, F f) {
  const uint32_t pp = oproj_pairs_per_wave(d);
#define STGN_OPROJ_CASE(HH)                                              \
  switch (pp) {                                                          \
    case 1: f(oproj_kernel<RB, HH, 1>); break;                           \
    case 2: f(oproj_kernel<RB, HH, 2>); break;                           \
    default: f(oproj_kernel<RB, HH, 4>); break;                          \
  }
  switch (d.heads) {
    case 1: STGN_OPROJ_CASE(1) break;
    case 2: STGN_OPROJ_CASE(2) break;
    default: STGN_OPROJ_CASE(4) break;
  }
#undef STGN_OPROJ_CASE
}

template <int RB>
hipError_t set_oproj_attr(const Dev& d, int bytes) {
  hipError_t e = hipSuccess;
  with_oproj<RB>(d, [&](auto kern) {
    e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  });
  return e;
}

template <int RB>
void launch_oproj_rb(const Dev& d, hipStream_t s, uint32_t layer, const uint32_t* rows, const uint32_t* cp, uint32_t cm) {
  const dim3 grid(persistent_blocks(cm, 32 * RB)), block(256);
  const size_t lds = oproj_lds(d, RB);
  with_oproj<RB>(d, [&](auto kern) { hipLaunchKernelGGL(kern, grid, block, lds, s, d, layer, rows, cp, cm); });
}

}  // namespace

int attn_supported(uint32_t d_in, uint32_t d_edge, uint32_t d_time, uint32_t heads) {
  const uint32_t ns = (d_in + kSlot - 1) / kSlot + (d_edge + kSlot - 1) / kSlot + (d_time + kSlot - 1) / kSlot;
  return d_in >= 1 && d_time >= 1 && d_time <= 2 * kSlot && ns <= kMaxSlots && (heads == 1 || heads == 2 || heads == 4);
}

void launch_qproj(const Dev& d, hipStream_t s, uint32_t layer, const uint32_t* rows, const uint32_t* cp, uint32_t cm) {
  if (tile_rb(d) == 1)
    hipLaunchKernelGGL(qproj_kernel<1>, dim3(persistent_blocks(cm, 32)), dim3(256), qproj_lds(d, layer, 1), s, d, layer,
                       rows, cp, cm);
  else
    hipLaunchKernelGGL(qproj_kernel<2>, dim3(persistent_blocks(cm, 64)), dim3(256), qproj_lds(d, layer, 2), s, d, layer,
                       rows, cp, cm);
}

void launch_attn(const Dev& d, hipStream_t s, uint32_t layer, const uint32_t* rows, const uint32_t* cp, uint32_t cm) {
  switch (d.L[layer].ns) {
    case 2: launch_attn_ns<2>(d, s, layer, rows, cp, cm); break;
    case 3: launch_attn_ns<3>(d, s, layer, rows, cp, cm); break;
    case 4: launch_attn_ns<4>(d, s, layer, rows, cp, cm); break;
    case 5: launch_attn_ns<5>(d, s, layer, rows, cp, cm); break;
    case 6: launch_attn_ns<6>(d, s, layer, rows, cp, cm); break;
    case 7: launch_attn_ns<7>(d, s, layer, rows, cp, cm); break;
    default: launch_attn_ns<8>(d, s, layer, rows, cp, cm); break;
  }
}

void launch_oproj(const Dev& d, hipStream_t s, uint32_t layer, const uint32_t* rows, const uint32_t* cp, uint32_t cm) {
  if (tile_rb(d) == 1) launch_oproj_rb<1>(d, s, layer, rows, cp, cm);
  else launch_oproj_rb<2>(d, s, layer, rows, cp, cm);
}

void launch_gather_rows(const Dev& d, hipStream_t s, uint32_t layer, uint32_t n, const uint32_t* nodes, float* out) {
  const uint32_t width = layer == 0 ? d.d0 : d.d_emb;
  uint64_t blocks = ((uint64_t)n * width + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(gather_rows_kernel, dim3((uint32_t)blocks), dim3(256), 0, s, d.H[layer], width, n, nodes, out);
}

int setup_embed_attributes(const Dev& d) {
  const uint32_t rb = tile_rb(d);
  size_t q = 0;
  for (uint32_t l = 0; l < d.layers; ++l) q = qproj_lds(d, l, rb) > q ? qproj_lds(d, l, rb) : q;
  const size_t o = oproj_lds(d, rb);
  if (q > kMaxLds || o > kMaxLds) return -1;
  if (d.heads * (round_up(d.dk, 32) / 32) > 4 * kMaxPairsCap) return -1;
  hipError_t e1 = rb == 1 ? hipFuncSetAttribute((const void*)qproj_kernel<1>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)q)
                          : hipFuncSetAttribute((const void*)qproj_kernel<2>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)q);
  hipError_t e2 = rb == 1 ? set_oproj_attr<1>(d, (int)o) : set_oproj_attr<2>(d, (int)o);
  return (e1 == hipSuccess && e2 == hipSuccess) ? 0 : -1;
}

}  // namespace stgn
