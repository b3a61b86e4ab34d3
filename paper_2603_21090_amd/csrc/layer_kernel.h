// Temporal-attention layer for a list of target rows (paper Eq. attn_detail, Sec. 3.3.4 exact
// mode, Sec. 3.6.2 "single batched kernel" over the affected set), one fused kernel per layer.
//
// The layer is evaluated in an algebraically re-associated form so that every dense product runs
// over |rows| instead of |rows| * k:
//     score_{h,j} = q_h . (z_j W_K,h) / sqrt(dk)      =  (W_K,h q_h / sqrt(dk)) . z_j  =  qt_h . z_j
//     o_h         = sum_j alpha_{h,j} (z_j W_V,h)     =  (sum_j alpha_{h,j} z_j) W_V,h =  zb_h W_V,h
// with z_j = [h_{u_j} | e_j | phi(t_v - t_j)] the raw gathered neighbour row.  A workgroup of four
// waves owns 16 target rows and runs five phases without leaving the CU:
//   1. q  = h_v W_Q(node block) + phi(0) W_Q(time block)                         (MFMA 16x16x4)
//   2. qt_h = q_h W_K,h^T / sqrt(dk), kept in LDS in the slot layout               (MFMA)
//   3. gather z_j (node row, edge-feature row, time encoding), scores, softmax, zb_h; one wave
//      serves four rows, 16 lanes x float4 per 64-float slot; zb overwrites qt in LDS   (HBM bound)
//   4. o_h = zb_h W_V,h                                                          (MFMA)
//   5. h_v' = [o_1 | .. | o_H] W_O + b_O, written into the layer cache             (MFMA)
// Weights stream from L2 (tile-major packing, see mfma16.h); two workgroups per CU overlap one's
// gather with the other's products.
#pragma once
#include "stgn_internal.h"
#include "mfma16.h"

namespace stgn {

namespace layer_impl {

constexpr uint32_t kTM = 16;   // target rows per workgroup

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

struct LayerLds {
  uint32_t ldx, ldq, ldz;        // strides (floats) of the X, Q/O and qt/zb tiles
  uint32_t off_q, off_z, off_o, total;
};

__host__ __device__ inline LayerLds layer_lds(uint32_t d_in, uint32_t d_emb, uint32_t heads, uint32_t Zp) {
  LayerLds l;
  l.ldx = round_up(d_in, 4) + 1;
  l.ldq = (round_up(d_emb, 4) + 4) | 1u;          // room for the K padding of the last head
  l.ldz = heads * Zp + 4;                         // 16-byte aligned rows, banks staggered by 4
  l.off_q = kTM * l.ldx;
  l.off_z = round_up(l.off_q + kTM * l.ldq, 4);
  l.off_o = l.off_z + kTM * l.ldz;
  l.total = l.off_o + kTM * l.ldq;
  return l;
}

// Everything the kernel needs, and nothing else (keeps the scalar register file uncrowded).
struct LayerArgs {
  const float* Hin; float* Hout; const float* efeat;
  const RingEntry* ring; const uint32_t* deg; const double* t_last;
  const double* om_rev; const double* ph_rev;
  Ctrl* ctrl;
  const float *WQ, *cQ, *WKT, *WV, *WO, *bO;        // WQ, WKT, WV, WO tile-major (mfma16.h)
  uint32_t ld_in, ld_out, ld_ef;
  uint32_t k, heads, d_in, d_emb, dk, d_time, Zp;
  uint16_t valid[kMaxSlots];     // valid floats per slot
  uint16_t segoff[kMaxSlots];    // offset of the slot inside its source row
  uint8_t  kind[kMaxSlots];      // 0 node row, 1 edge-feature row, 2 time encoding
};

// NS slots in total, the last NT of them time-encoding slots; JC ring entries fetched together.
template <int NS, int NT, int H, int JC>
__global__ __launch_bounds__(256, 2) void layer_kernel(LayerArgs a, const uint32_t* __restrict__ rows,
                                                       const uint32_t* count_ptr, uint32_t count_max) {
  extern __shared__ __align__(16) float lds[];
  __shared__ uint32_t s_node[kTM];
  __shared__ double s_om[2 * kSlot], s_ph[2 * kSlot];
  if (count_ptr && a.ctrl->skip) return;
  uint32_t n = count_max;
  if (count_ptr) { const uint32_t c = *count_ptr; n = c < count_max ? c : count_max; }
  const uint32_t ntiles = (n + kTM - 1) / kTM;
  const uint32_t lane = threadIdx.x & 63u, sub = lane & 15u, grp = lane >> 4;
  // wave index, made provably uniform so that tile indices and weight addresses stay in scalar registers
  const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const uint32_t Zp = a.Zp, k = a.k, dk = a.dk;
  const uint32_t s_in = round_up(a.d_in, 4) >> 2, s_de = round_up(a.d_emb, 4) >> 2, s_dk = round_up(dk, 4) >> 2;  // k-steps
  const uint32_t ntd = round_up(a.d_emb, 16) >> 4, ntk = round_up(dk, 16) >> 4, ntz = Zp >> 4;               // column tiles
  const LayerLds ll = layer_lds(a.d_in, a.d_emb, a.heads, Zp);
  float* Xs = lds;
  float* Qs = lds + ll.off_q;
  float* Zs = lds + ll.off_z;
  float* Os = lds + ll.off_o;
  constexpr int NG = NS - NT;                 // gathered (node / edge) slots

  // ---- per-lane constants
  bool lane_ok[NS];
#pragma unroll
  for (int s = 0; s < NS; ++s) lane_ok[s] = 4u * sub < a.valid[s];
  // time-encoding parameters (omega, phase in revolutions) live in LDS, zero past d_time
  for (uint32_t q = threadIdx.x; q < 2 * kSlot; q += 256) {
    s_om[q] = q < a.d_time ? a.om_rev[q] : 0.0;
    s_ph[q] = q < a.d_time ? a.ph_rev[q] : 0.0;
  }
  bool tok[NT][4];
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int c = 0; c < 4; ++c) tok[t][c] = (uint32_t)t * kSlot + 4u * sub + c < a.d_time;
  uint32_t gathered = 0;
  const uint32_t a_x = a16_lane_off(ll.ldx), a_q = a16_lane_off(ll.ldq), a_z = a16_lane_off(ll.ldz);
  const uint32_t c_off_q = m16_row(lane, 0) * ll.ldq + m16_col(lane);
  const uint32_t c_off_z = m16_row(lane, 0) * ll.ldz + m16_col(lane);

  // ---- phase-2 tile cursor: (head, 16-column tile); this wave owns tiles wave, wave + 4, ... of
  // every head; tiles that lie wholly in slot padding are skipped (nobody reads them)
  struct Cur { uint32_t h, t; };
  auto cur_skip = [&](Cur& c) {
    while (c.h < a.heads) {
      if (c.t >= ntz) { ++c.h; c.t = wave; continue; }
      if ((c.t & 3u) * 16u < a.valid[c.t >> 2]) break;
      c.t += 4;
    }
  };
  auto cur_next = [&](Cur c) { c.t += 4; cur_skip(c); return c; };
  auto qt_weights = [&](const Cur& c) { return a.WKT + (size_t)(c.h * ntz + c.t) * s_dk * kBlk16; };
  auto qt_tile = [&](const Cur& c, float (&b)[kU16]) {
    floatx4 acc = {0.f, 0.f, 0.f, 0.f};
    mfma16_tile_pre<kU16>(Qs + c.h * dk, a_q, s_dk, qt_weights(c), acc, b);
    float* zp = Zs + c.h * Zp + c.t * 16 + c_off_z;
#pragma unroll
    for (int r = 0; r < 4; ++r) zp[r * ll.ldz] = acc[r];
  };

  for (uint32_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
    const uint32_t r0 = tile * kTM;
    // ================================================================ phase 0: stage the tile
    float b1[kU16];
    const bool has1 = wave < ntd;
    if (has1) load_b16<kU16>(a.WQ + (size_t)wave * s_in * kBlk16, 0, b1);
    if (threadIdx.x < kTM) {
      const uint32_t r = r0 + threadIdx.x;
      s_node[threadIdx.x] = r < n ? (rows ? rows[r] : r) : 0xFFFFFFFFu;
    }
    for (uint32_t x = threadIdx.x; x < kTM * (ll.ldq - a.d_emb); x += 256) {
      const uint32_t r = x / (ll.ldq - a.d_emb), c = a.d_emb + x % (ll.ldq - a.d_emb);
      Qs[r * ll.ldq + c] = 0.0f;
      Os[r * ll.ldq + c] = 0.0f;
    }
    __syncthreads();
    {
      const uint32_t qpr = s_in, total = kTM * qpr;            // 16-byte quads per row / per tile
      for (uint32_t x0 = threadIdx.x; x0 < total; x0 += 512u) {
        float4 v[2];
        uint32_t rr[2], cc[2];
        bool ok[2];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
          uint32_t x = x0 + 256u * e;
          ok[e] = x < total;
          x = ok[e] ? x : 0u;
          const uint32_t r = x / qpr, q = x - r * qpr;
          const uint32_t node = s_node[r];
          rr[e] = r; cc[e] = 4u * q;
          const bool live = node != 0xFFFFFFFFu;
          v[e] = *reinterpret_cast<const float4*>(a.Hin + (size_t)(live ? node : 0u) * a.ld_in + 4u * q);
          if (!live) v[e] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int e = 0; e < 2; ++e)
          if (ok[e]) {
            float* p = Xs + rr[e] * ll.ldx + cc[e];
            p[0] = v[e].x; p[1] = v[e].y; p[2] = v[e].z; p[3] = v[e].w;
          }
      }
    }
    __syncthreads();
    // ================================================================ phase 1: q = x W_Q + c_Q
    float bA[kU16], bB[kU16];
    Cur f{0u, wave};
    cur_skip(f);
    if (f.h < a.heads) load_b16<kU16>(qt_weights(f), 0, bA);
    for (uint32_t nt = wave; nt < ntd; nt += 4) {
      floatx4 acc = {0.f, 0.f, 0.f, 0.f};
      const float* Wt = a.WQ + (size_t)nt * s_in * kBlk16;
      if (nt == wave) mfma16_tile_pre<kU16>(Xs, a_x, s_in, Wt, acc, b1);
      else mfma16_tile<kU16>(Xs, a_x, s_in, Wt, acc);
      const uint32_t col = nt * 16 + m16_col(lane);
      if (col < a.d_emb) {
        const float cq = a.cQ[col];
        float* qp = Qs + nt * 16 + c_off_q;
#pragma unroll
        for (int r = 0; r < 4; ++r) qp[r * ll.ldq] = acc[r] + cq;
      }
    }
    __syncthreads();
    // ================================================================ phase 2: qt_h = q_h W_K,h^T / sqrt(dk)
    while (f.h < a.heads) {
      const Cur g = cur_next(f);
      if (g.h < a.heads) load_b16<kU16>(qt_weights(g), 0, bB);
      qt_tile(f, bA);
      if (g.h >= a.heads) break;
      f = cur_next(g);
      if (f.h < a.heads) load_b16<kU16>(qt_weights(f), 0, bA);
      qt_tile(g, bB);
    }
    __syncthreads();
    // ================================================================ phase 3: gather + attention
    {
      const uint32_t local = wave * 4u + grp;
      const uint32_t v = s_node[local];
      const bool act = v != 0xFFFFFFFFu;
      const uint32_t vv = act ? v : 0u;
      const uint32_t dg = act ? a.deg[vv] : 0u;
      const uint32_t cnt = dg < k ? dg : k;
      gathered += cnt;
      const double tq = a.t_last[vv];
      float* zrow = Zs + local * ll.ldz + 4u * sub;          // this lane's float4 of slot s, head h: + h Zp + 64 s
      float4 acc[H][NS];
#pragma unroll
      for (int h = 0; h < H; ++h)
#pragma unroll
        for (int s = 0; s < NS; ++s) acc[h][s] = make_float4(0.f, 0.f, 0.f, 0.f);
      float mrun[H], lrun[H];
#pragma unroll
      for (int h = 0; h < H; ++h) { mrun[h] = -INFINITY; lrun[h] = 0.0f; }
      uint32_t cmax = (uint32_t)__builtin_amdgcn_readlane((int)cnt, 0);
      cmax = max(cmax, (uint32_t)__builtin_amdgcn_readlane((int)cnt, 16));
      cmax = max(cmax, (uint32_t)__builtin_amdgcn_readlane((int)cnt, 32));
      cmax = max(cmax, (uint32_t)__builtin_amdgcn_readlane((int)cnt, 48));
      const RingEntry* ring = a.ring + (size_t)vv * k;
      int slot = cnt ? (int)((dg - 1u) % k) : 0;            // ring slot of the most recent entry
      for (uint32_t j0 = 0; j0 < cmax; j0 += JC) {
        // ring records of the whole chunk first, then every row load of the chunk
        RingEntry re[JC];
        bool vj[JC];
#pragma unroll
        for (int jc = 0; jc < JC; ++jc) {
          vj[jc] = j0 + jc < cnt;
          re[jc] = ring[vj[jc] ? slot : 0];
          if (vj[jc]) slot = slot == 0 ? (int)k - 1 : slot - 1;
        }
        float4 z[JC][NS];
#pragma unroll
        for (int jc = 0; jc < JC; ++jc) {
          const uint32_t nbr = vj[jc] ? re[jc].nbr : 0u, eid = vj[jc] ? re[jc].eid : 0u;
          const double dt = tq - re[jc].t;
          const float* hrow = a.Hin + (size_t)nbr * a.ld_in + 4u * sub;
          const float* erow = a.efeat + (size_t)eid * a.ld_ef + 4u * sub;
#pragma unroll
          for (int s = 0; s < NG; ++s) {
            float4 zz = make_float4(0.f, 0.f, 0.f, 0.f);
            if (vj[jc] && lane_ok[s]) zz = *reinterpret_cast<const float4*>((a.kind[s] == 0 ? hrow : erow) + a.segoff[s]);
            z[jc][s] = zz;
          }
#pragma unroll
          for (int t = 0; t < NT; ++t) {
            float4 zz;
            const double* om = s_om + t * kSlot + 4u * sub;
            const double* ph = s_ph + t * kSlot + 4u * sub;
            zz.x = (vj[jc] && tok[t][0]) ? cos_rev(om[0] * dt + ph[0]) : 0.0f;
            zz.y = (vj[jc] && tok[t][1]) ? cos_rev(om[1] * dt + ph[1]) : 0.0f;
            zz.z = (vj[jc] && tok[t][2]) ? cos_rev(om[2] * dt + ph[2]) : 0.0f;
            zz.w = (vj[jc] && tok[t][3]) ? cos_rev(om[3] * dt + ph[3]) : 0.0f;
            z[jc][NG + t] = zz;
          }
        }
        float sc[JC][H];
#pragma unroll
        for (int h = 0; h < H; ++h) {
          float p[JC];
#pragma unroll
          for (int jc = 0; jc < JC; ++jc) p[jc] = 0.0f;
#pragma unroll
          for (int s = 0; s < NS; ++s) {
            float4 qv = make_float4(0.f, 0.f, 0.f, 0.f);
            if (lane_ok[s]) qv = *reinterpret_cast<const float4*>(zrow + h * Zp + s * kSlot);
#pragma unroll
            for (int jc = 0; jc < JC; ++jc) p[jc] = dot4(qv, z[jc][s], p[jc]);
          }
#pragma unroll
          for (int jc = 0; jc < JC; ++jc) {
            const float t = row16_sum(p[jc]);
            sc[jc][h] = vj[jc] ? t : -INFINITY;
          }
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
      // zb overwrites qt (each lane owns its float4s; padding lanes write zeros)
#pragma unroll
      for (int h = 0; h < H; ++h) {
        const float inv = cnt ? 1.0f / lrun[h] : 0.0f;
#pragma unroll
        for (int s = 0; s < NS; ++s) {
          float4 o = acc[h][s];
          o.x *= inv; o.y *= inv; o.z *= inv; o.w *= inv;
          *reinterpret_cast<float4*>(zrow + h * Zp + s * kSlot) = o;
        }
      }
    }
    __syncthreads();
    // ================================================================ phase 4: o_h = zb_h W_V,h
    {
      // wave w owns the (head, 16-column tile) pairs w, w + 4, ...; K runs over the slots, one chunk
      // of 16 k-steps per slot; the weights of the next slot are in flight during the current one
      const uint32_t npairs = a.heads * ntk;
      bool first = true;
      for (uint32_t p = wave; p < npairs; p += 4) {
        const uint32_t h = p / ntk, nt = p - h * ntk;
        const float* Wt = a.WV + (size_t)p * (Zp >> 2) * kBlk16;          // column tile p = h * ntk + nt
        const float* Ap = Zs + h * Zp;
        floatx4 acc = {0.f, 0.f, 0.f, 0.f};
        float bc[kU16], bn[kU16];
        load_b16<kU16>(Wt, 0, bc);
#pragma unroll
        for (int c = 0; c < NS; ++c) {
          if (c + 1 < NS) load_b16<kU16>(Wt, (c + 1) * kU16, bn);
          mfma16_steps<kU16>(Ap + c * kSlot, a_z, 0, (uint32_t)(a.valid[c] + 3u) >> 2, bc, acc);
#pragma unroll
          for (int u = 0; u < kU16; ++u) bc[u] = bn[u];
        }
        // weights of the output projection are requested before the head outputs are exchanged
        if (first && has1) load_b16<kU16>(a.WO + (size_t)wave * s_de * kBlk16, 0, b1);
        first = false;
        const uint32_t col = nt * 16 + m16_col(lane);
        if (col < dk) {
          float* op = Os + h * dk + nt * 16 + c_off_q;
#pragma unroll
          for (int r = 0; r < 4; ++r) op[r * ll.ldq] = acc[r];
        }
      }
      if (first && has1) load_b16<kU16>(a.WO + (size_t)wave * s_de * kBlk16, 0, b1);
    }
    __syncthreads();
    // ================================================================ phase 5: h' = o W_O + b_O
    for (uint32_t nt = wave; nt < ntd; nt += 4) {
      floatx4 acc = {0.f, 0.f, 0.f, 0.f};
      const float* Wt = a.WO + (size_t)nt * s_de * kBlk16;
      if (nt == wave) mfma16_tile_pre<kU16>(Os, a_q, s_de, Wt, acc, b1);
      else mfma16_tile<kU16>(Os, a_q, s_de, Wt, acc);
      const uint32_t col = nt * 16 + m16_col(lane);
      if (col < a.d_emb) {
        const float b = a.bO[col];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const uint32_t node = s_node[m16_row(lane, r)];
          if (node != 0xFFFFFFFFu) a.Hout[(size_t)node * a.ld_out + col] = acc[r] + b;
        }
      }
    }
    __syncthreads();
  }
  // statistics: one atomic per wave
  const uint32_t gsum = (uint32_t)__builtin_amdgcn_readlane((int)gathered, 0) +
                        (uint32_t)__builtin_amdgcn_readlane((int)gathered, 16) +
                        (uint32_t)__builtin_amdgcn_readlane((int)gathered, 32) +
                        (uint32_t)__builtin_amdgcn_readlane((int)gathered, 48);
  if (lane == 0 && gsum) atomicAdd((unsigned long long*)&a.ctrl->tot_gathered, (unsigned long long)gsum);
}

// ---- dispatch over (slots, time slots, heads, chunk)
struct LaunchArgs {
  LayerArgs k;
  hipStream_t s; const uint32_t* rows; const uint32_t* cp; uint32_t cm;
  uint32_t nt;                      // time slots of this layer
  bool set_attr; size_t lds; hipError_t err;
};

template <int NS, int NT, int H, int JC>
void go(LaunchArgs& a) {
  auto kern = layer_kernel<NS, NT, H, JC>;
  if (a.set_attr) {
    a.err = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)a.lds);
    return;
  }
  uint64_t blocks = ((uint64_t)a.cm + kTM - 1) / kTM;
  if (blocks > 4096) blocks = 4096;          // persistent: each workgroup strides over the tiles
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(kern, dim3((uint32_t)blocks), dim3(256), a.lds, a.s, a.k, a.rows, a.cp, a.cm);
}

template <int NS, int NT>
void go_h(LaunchArgs& a) {
  // ring entries in flight per row are bounded by registers (JC * NS float4 per lane)
  switch (a.k.heads) {
    case 1: go<NS, NT, 1, (NS <= 4 ? 5 : NS == 5 ? 3 : 2)>(a); break;
    case 2: go<NS, NT, 2, (NS <= 4 ? 5 : NS == 5 ? 3 : 2)>(a); break;
    default: go<NS, NT, 4, (NS <= 4 ? 3 : 2)>(a); break;
  }
}

template <int NS>
void go_nt(LaunchArgs& a) {
  if constexpr (NS >= 3) {
    if (a.nt == 2) { go_h<NS, 2>(a); return; }
  }
  go_h<NS, 1>(a);
}

}  // namespace layer_impl

// one translation unit per slot count instantiates this (keeps the build parallel)
template <int NS>
void layer_entry(layer_impl::LaunchArgs& a) { layer_impl::go_nt<NS>(a); }

}  // namespace stgn
