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
// Weights stream from L2 (group-major packing, see mfma16.h); two workgroups per CU overlap one's
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
  uint32_t ldx, ldq, ldz;        // strides (floats) of the X / O tile, the Q tile and the qt / zb tile
  uint32_t dkp;                  // floats reserved per head in a Q row (dk rounded up to a group)
  uint32_t off_q, off_z, off_r, total;
};

// Every stride is 4 (mod 8) floats: rows stay 16-byte aligned and the 16 rows of an operand read
// fall into distinct banks.
__host__ __device__ inline LayerLds layer_lds(uint32_t d_in, uint32_t d_emb, uint32_t heads, uint32_t Zp, uint32_t k) {
  LayerLds l;
  const uint32_t wx = round_up(d_in, kGrpK), wo = round_up(d_emb, kGrpK);
  l.ldx = (wx > wo ? wx : wo) + 4;                // the input tile and the head-output tile share storage
  l.dkp = round_up(d_emb / heads, kGrpK);
  l.ldq = heads * l.dkp + 4;
  l.ldz = heads * Zp + 4;
  l.off_q = kTM * l.ldx;
  l.off_z = l.off_q + kTM * l.ldq;
  l.off_r = l.off_z + kTM * l.ldz + 4 * kGrpK;    // operand reads may run one chunk past the last row
  l.total = l.off_r + kTM * k * 4;                // the ring records of the tile's rows, 16 bytes each
  return l;
}

// Everything the kernel needs, and nothing else (keeps the scalar register file uncrowded).
struct LayerArgs {
  const float* Hin; float* Hout; const float* efeat;
  const RingEntry* ring; const uint32_t* deg; const double* t_last;
  const double* om_rev; const double* ph_rev;
  Ctrl* ctrl;
  const float *WQ, *cQ, *WKT, *WV, *WO, *bO;        // WQ, WKT, WV, WO group-major (mfma16.h)
  uint32_t ld_in, ld_out, ld_ef;
  uint32_t k, heads, d_in, d_emb, dk, d_time, Zp;
  uint16_t valid[kMaxSlots];     // valid floats per slot
  uint16_t segoff[kMaxSlots];    // offset of the slot inside its source row
  uint8_t  kind[kMaxSlots];      // 0 node row, 1 edge-feature row, 2 time encoding
};

// gathered (node / edge) slots of one chunk of JC ring entries, one float4 per lane and slot
template <int JC, int NG>
struct GatherBuf {
  float4 g[JC][NG];
};

// NS slots in total, the last NT of them time-encoding slots; JC ring entries fetched together.
template <int NS, int NT, int H, int JC>
__global__ __launch_bounds__(256, 2) void layer_kernel(LayerArgs a, const uint32_t* __restrict__ rows,
                                                       const uint32_t* count_ptr, uint32_t count_max) {
  extern __shared__ __align__(16) float lds[];
  __shared__ uint32_t s_node[kTM], s_cnt[kTM], s_next[kTM];
  __shared__ double s_tq[kTM];
  __shared__ uint32_t s_zt[4 * kMaxSlots];     // 16-column tiles of a qt row that hold valid columns
  __shared__ __align__(16) double s_om[2 * kSlot], s_ph[2 * kSlot];
  if (count_ptr && a.ctrl->skip) return;
  uint32_t n = count_max;
  if (count_ptr) { const uint32_t c = *count_ptr; n = c < count_max ? c : count_max; }
  const uint32_t ntiles = (n + kTM - 1) / kTM;
  const uint32_t lane = threadIdx.x & 63u, sub = lane & 15u, grp = lane >> 4;
  // wave index, made provably uniform so that tile indices and weight addresses stay in scalar registers
  const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const uint32_t Zp = a.Zp, k = a.k, dk = a.dk;
  const uint32_t c_in = chunks_of(a.d_in), c_de = chunks_of(a.d_emb), c_dk = chunks_of(dk);                    // chunks of K
  const uint32_t g_in = kCG * c_in, g_de = kCG * c_de, g_dk = kCG * c_dk, g_z = Zp / kGrpK;                   // groups of K
  const uint32_t ntd = round_up(a.d_emb, 16) >> 4, ntk = round_up(dk, 16) >> 4, ntz = Zp >> 4;                // column tiles
  const LayerLds ll = layer_lds(a.d_in, a.d_emb, a.heads, Zp, k);
  float* Xs = lds;                            // input rows (phases 0-1), then head outputs (phases 4-5)
  float* Qs = lds + ll.off_q;
  float* Zs = lds + ll.off_z;
  RingEntry* Rs = reinterpret_cast<RingEntry*>(lds + ll.off_r);   // [row][j], j = 0 the most recent entry
  constexpr int NG = NS - NT;                 // gathered (node / edge) slots
  using ZBuf = GatherBuf<JC, NG>;

  // ---- per-lane constants
  // time-encoding parameters (omega, phase in revolutions) live in LDS, zero past d_time
  for (uint32_t q = threadIdx.x; q < 2 * kSlot; q += 256) {
    s_om[q] = q < a.d_time ? a.om_rev[q] : 0.0;
    s_ph[q] = q < a.d_time ? a.ph_rev[q] : 0.0;
  }
  // operand padding (columns nobody writes) must be finite: clear the tiles once
  for (uint32_t x = threadIdx.x; x < ll.off_r; x += 256) lds[x] = 0.0f;
  // list of the qt column tiles that are not wholly slot padding
  uint32_t nzt;
  {
    uint32_t vq = 0;
#pragma unroll
    for (int s = 0; s < NS; ++s)
      if ((lane >> 2) == (uint32_t)s) vq = a.valid[s];
    const bool tv = lane < ntz && (lane & 3u) * 16u < vq;
    const uint64_t m = __ballot(tv);
    nzt = (uint32_t)__popcll(m);
    if (wave == 0 && tv) s_zt[__popcll(m & ((1ull << lane) - 1ull))] = lane;
  }
  bool tok[NT][4];
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int c = 0; c < 4; ++c) tok[t][c] = (uint32_t)t * kSlot + 4u * sub + c < a.d_time;
  uint32_t gathered = 0;
  const uint32_t a_x = a16_lane_off(ll.ldx), a_q = a16_lane_off(ll.ldq), a_z = a16_lane_off(ll.ldz);
  const uint32_t c_off_x = m16_row(lane, 0) * ll.ldx + m16_col(lane);
  const uint32_t c_off_z = m16_row(lane, 0) * ll.ldz + m16_col(lane);

  // ---- phase-2 work units: (head, pair of valid qt column tiles); wave w owns units w, w + 4, ...
  // Lane i of `udesc` holds the description of the wave's i-th unit (head, the two tiles, whether the
  // second tile is real), worked out once; inside the tile loop a unit costs one cross-lane read.
  const uint32_t npr = (nzt + 1u) >> 1, nunits2 = a.heads * npr;
  const uint32_t nu2 = wave < nunits2 ? (nunits2 - wave + 3u) >> 2 : 0u;     // units of this wave
  struct Unit2 { uint32_t h, t0, t1; bool two; };
  __syncthreads();                                                           // s_zt is complete
  uint32_t udesc = 0;
  if (lane < nu2) {
    const uint32_t x = wave + 4u * lane, h = x / npr, i0 = 2u * (x - h * npr);
    const uint32_t two = i0 + 1u < nzt ? 1u : 0u;
    udesc = h | (s_zt[i0] << 8) | (s_zt[i0 + two] << 16) | (two << 24);
  }
  auto decode2 = [&](uint32_t i) {
    const uint32_t dsc = (uint32_t)__builtin_amdgcn_readlane((int)udesc, (int)i);
    Unit2 u;
    u.h = dsc & 0xFFu; u.t0 = (dsc >> 8) & 0xFFu; u.t1 = (dsc >> 16) & 0xFFu; u.two = (dsc >> 24) != 0u;
    return u;
  };
  auto wkt = [&](uint32_t h, uint32_t t) { return a.WKT + (size_t)(h * ntz + t) * g_dk * kGrpFloats; };
  auto store2 = [&](const Unit2& u, const floatx4 (&acc)[2]) {
    float* zp = Zs + u.h * Zp + c_off_z;
#pragma unroll
    for (int r = 0; r < 4; ++r) zp[u.t0 * 16 + r * ll.ldz] = acc[0][r];
    if (u.two) {
#pragma unroll
      for (int r = 0; r < 4; ++r) zp[u.t1 * 16 + r * ll.ldz] = acc[1][r];
    }
  };
  // ---- phase-4 work units: (head, pair of head-output column tiles)
  const uint32_t np4 = (ntk + 1u) >> 1, nunits4 = a.heads * np4;
  // ---- phases 1 and 5: column tiles nt and nt + 4 of the d_emb outputs form a unit
  __syncthreads();

  // ---- staging of a tile, one tile ahead.  Stage A reads the tile's row ids into s_next; stage B
  // (issued while the previous tile's last products run) fetches, into registers, this thread's
  // share of the rows' ring slots, degrees, query times and own input rows; the tile's phase 0 then
  // only moves registers into LDS.  A workgroup strides over many tiles, so all but its first tile
  // start without waiting for memory.  Shapes whose share does not fit two items per thread stage
  // inside phase 0 instead.
  const uint32_t qpr = round_up(a.d_in, kGrpK) >> 2;          // 16-byte quads per staged input row
  const bool pf_ok = kTM * k <= 512u && kTM * qpr <= 512u;
  RingEntry p_ring[2];
  uint32_t p_deg[2];
  double p_tl[2];
  float4 p_x[2];
  auto stage_a = [&](uint32_t t) {
    if (threadIdx.x < kTM) {
      const uint32_t r = t * kTM + threadIdx.x;
      s_next[threadIdx.x] = (t < ntiles && r < n) ? (rows ? rows[r] : r) : 0xFFFFFFFFu;
    }
  };
  auto stage_b = [&]() {
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      const uint32_t x = threadIdx.x + 256u * e;
      {
        const uint32_t xc = x < kTM * k ? x : 0u;
        const uint32_t r = xc / k, sl = xc - r * k;
        const uint32_t node = s_next[r];
        const uint32_t nn = node != 0xFFFFFFFFu ? node : 0u;
        p_ring[e] = a.ring[(size_t)nn * k + sl];
        p_deg[e] = a.deg[nn];
        p_tl[e] = a.t_last[nn];
      }
      {
        const uint32_t xc = x < kTM * qpr ? x : 0u;
        const uint32_t r = xc / qpr, q = xc - r * qpr;
        const uint32_t node = s_next[r];
        // columns past d_in are row padding of the table (zero)
        p_x[e] = *reinterpret_cast<const float4*>(a.Hin + (size_t)(node != 0xFFFFFFFFu ? node : 0u) * a.ld_in + 4u * q);
      }
    }
  };
  // the record of adjacency position p sits in ring slot p mod k; with the row's degree known, slot
  // sl holds the j-th most recent entry, j = (newest - sl) mod k; places past the row's entry count
  // name node 0 / edge 0 (finite rows that later meet a zero weight)
  auto place_ring = [&](uint32_t r, uint32_t sl, bool live, RingEntry e, uint32_t dg_in, double tl) {
    const uint32_t dg = live ? dg_in : 0u;
    const uint32_t cnt = dg < k ? dg : k;
    const uint32_t newest = dg ? (dg - 1u) % k : 0u;
    const uint32_t j = newest >= sl ? newest - sl : newest + k - sl;
    if (j >= cnt) { e.nbr = 0u; e.eid = 0u; e.t = 0.0; }
    Rs[r * k + j] = e;
    if (sl == 0) { s_cnt[r] = cnt; s_tq[r] = tl; }
  };
  stage_a(blockIdx.x);
  __syncthreads();
  auto stage_none = [&]() {                                   // keeps the registers defined on every path
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      p_ring[e].nbr = 0u; p_ring[e].eid = 0u; p_ring[e].t = 0.0; p_deg[e] = 0u; p_tl[e] = 0.0;
      p_x[e] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
  };
  if (pf_ok) stage_b(); else stage_none();

  for (uint32_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
    // ================================================================ phase 0: stage the tile
    Ops16<2> oq;                                              // first weight chunk of this wave's first unit
    const uint32_t w1 = wave < ntd ? wave : 0u;              // loads are unconditional (clamped), products are not
    load_b16(a.WQ + (size_t)w1 * g_in * kGrpFloats, 0, oq.b[0]);
    load_b16(a.WQ + (size_t)(w1 + 4 < ntd ? w1 + 4 : w1) * g_in * kGrpFloats, 0, oq.b[1]);
    if (threadIdx.x < kTM) s_node[threadIdx.x] = s_next[threadIdx.x];
    if (pf_ok) {
      // everything was fetched a tile ago: registers -> LDS
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        const uint32_t x = threadIdx.x + 256u * e;
        if (x < kTM * k) {
          const uint32_t r = x / k, sl = x - r * k;
          place_ring(r, sl, s_next[r] != 0xFFFFFFFFu, p_ring[e], p_deg[e], p_tl[e]);
        }
        if (x < kTM * qpr) {
          const uint32_t r = x / qpr, q = x - r * qpr;
          const float4 v = s_next[r] != 0xFFFFFFFFu ? p_x[e] : make_float4(0.f, 0.f, 0.f, 0.f);
          *reinterpret_cast<float4*>(Xs + r * ll.ldx + 4u * q) = v;
        }
      }
    }
    __syncthreads();
    if (!pf_ok) {
      // thread (row, slot) fetches its slot without waiting for the row's degree (both loads leave together)
      for (uint32_t x = threadIdx.x; x < kTM * k; x += 256) {
        const uint32_t r = x / k, sl = x - r * k;
        const uint32_t node = s_node[r];
        const bool live = node != 0xFFFFFFFFu;
        const uint32_t nn = live ? node : 0u;
        place_ring(r, sl, live, a.ring[(size_t)nn * k + sl], a.deg[nn], a.t_last[nn]);
      }
      const uint32_t total = kTM * qpr;
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
          // columns past d_in are row padding of the table (zero)
          v[e] = *reinterpret_cast<const float4*>(a.Hin + (size_t)(live ? node : 0u) * a.ld_in + 4u * q);
          if (!live) v[e] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int e = 0; e < 2; ++e)
          if (ok[e]) *reinterpret_cast<float4*>(Xs + rr[e] * ll.ldx + cc[e]) = v[e];
      }
      __syncthreads();
    }
    stage_a(tile + gridDim.x);                               // row ids of this workgroup's next tile
    // ---- this lane group's row: entry count, query time, ring records; the first chunk of neighbour
    // rows is requested now and arrives while the projections below run
    const uint32_t local = wave * 4u + grp;
    const uint32_t cnt = s_cnt[local];
    const double tq = s_tq[local];
    const RingEntry* rrow = Rs + local * k;
    gathered += cnt;
    uint32_t cmax = (uint32_t)__builtin_amdgcn_readlane((int)cnt, 0);
    cmax = max(cmax, (uint32_t)__builtin_amdgcn_readlane((int)cnt, 16));
    cmax = max(cmax, (uint32_t)__builtin_amdgcn_readlane((int)cnt, 32));
    cmax = max(cmax, (uint32_t)__builtin_amdgcn_readlane((int)cnt, 48));
    const uint32_t nchunk3 = (cmax + JC - 1) / JC;
    auto gather = [&](uint32_t c, ZBuf& zb) {
#pragma unroll
      for (int jc = 0; jc < JC; ++jc) {
        const uint32_t j = c * JC + jc;
        const RingEntry e = rrow[j < k ? j : k - 1u];
        const float* hrow = a.Hin + (size_t)e.nbr * a.ld_in + 4u * sub;
        const float* erow = a.efeat + (size_t)e.eid * a.ld_ef + 4u * sub;
#pragma unroll
        for (int s = 0; s < NG; ++s)
          zb.g[jc][s] = *reinterpret_cast<const float4*>((a.kind[s] == 0 ? hrow : erow) + a.segoff[s]);
      }
    };
    ZBuf z0;
    gather(0, z0);
    // ================================================================ phase 1: q = x W_Q + c_Q
    for (uint32_t nt = wave; nt < ntd; nt += 8) {
      const bool two = nt + 4 < ntd;
      const float* const Bt[2] = {a.WQ + (size_t)nt * g_in * kGrpFloats, a.WQ + (size_t)(two ? nt + 4 : nt) * g_in * kGrpFloats};
      floatx4 acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
      if (nt != wave) { load_b16(Bt[0], 0, oq.b[0]); load_b16(Bt[1], 0, oq.b[1]); }
      mfma16_gemm_pre<2>(Xs + a_x, c_in, Bt, acc, oq);
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const uint32_t col = (nt + 4 * t) * 16 + m16_col(lane);
        if ((t == 0 || two) && col < a.d_emb) {
          const float cq = a.cQ[col];
          const uint32_t h = col / dk;
          float* qp = Qs + m16_row(lane, 0) * ll.ldq + h * ll.dkp + (col - h * dk);
#pragma unroll
          for (int r = 0; r < 4; ++r) qp[r * ll.ldq] = acc[t][r] + cq;
        }
      }
    }
    // ================================================================ phase 2: qt_h = q_h W_K,h^T / sqrt(dk)
    {
      Ops16<2> o2;
      Unit2 ua = decode2(0);                                  // weights of the first unit are requested
      load_b16(wkt(ua.h, ua.t0), 0, o2.b[0]);                 // ahead of the barrier (unit 0 of an idle wave: head 0, tile 0)
      load_b16(wkt(ua.h, ua.t1), 0, o2.b[1]);
      __syncthreads();
      if (c_dk == 1) {
        // one chunk per unit: the operands of the next unit are in flight during this unit's products
        load_a16(Qs + ua.h * ll.dkp + a_q, 0, o2.a);
        if (nu2) pingpong_peeled<Ops16<2>>(
            nu2, o2,
            [&](uint32_t i, Ops16<2>& o) {
              const Unit2 u = decode2(i);
              load_a16(Qs + u.h * ll.dkp + a_q, 0, o.a);
              load_b16(wkt(u.h, u.t0), 0, o.b[0]);
              load_b16(wkt(u.h, u.t1), 0, o.b[1]);
            },
            [&](uint32_t i, const Ops16<2>& o) {
              const Unit2 u = decode2(i);
              floatx4 acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
              mfma16_chunk<2>(o, acc);
              store2(u, acc);
            });
      } else {
        for (uint32_t i = 0; i < nu2; ++i) {
          ua = decode2(i);
          const float* const Bt[2] = {wkt(ua.h, ua.t0), wkt(ua.h, ua.t1)};
          floatx4 acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
          mfma16_gemm<2>(Qs + ua.h * ll.dkp + a_q, c_dk, Bt, acc);
          store2(ua, acc);
        }
      }
    }
    __syncthreads();
    // ================================================================ phase 3: gather + attention
    {
      float4 acc[H][NS];
#pragma unroll
      for (int h = 0; h < H; ++h)
#pragma unroll
        for (int s = 0; s < NS; ++s) acc[h][s] = make_float4(0.f, 0.f, 0.f, 0.f);
      float mref[H], lrun[H];
#pragma unroll
      for (int h = 0; h < H; ++h) { mref[h] = -INFINITY; lrun[h] = 0.0f; }
      // this lane's share of the row's qt vectors stays in registers for the whole phase
      const float* zq = Zs + local * ll.ldz + 4u * sub;       // float4 of slot s, head h: + h Zp + 64 s
      constexpr bool QREG = H * NS <= 16;                     // otherwise the registers go to the accumulators
      float4 qt[QREG ? H : 1][QREG ? NS : 1];
      if constexpr (QREG) {
#pragma unroll
        for (int h = 0; h < H; ++h)
#pragma unroll
          for (int s = 0; s < NS; ++s) qt[h][s] = *reinterpret_cast<const float4*>(zq + h * Zp + s * kSlot);
      }
      auto attend = [&](uint32_t c, const ZBuf& zb) {
        // time encodings of the chunk's entries (computed for every lane, then masked: no branches)
        float4 zt[JC][NT];
        bool vj[JC];
        double2 om[NT][2], ph[NT][2];
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
          for (int q = 0; q < 2; ++q) {
            om[t][q] = *reinterpret_cast<const double2*>(s_om + t * kSlot + 4u * sub + 2 * q);
            ph[t][q] = *reinterpret_cast<const double2*>(s_ph + t * kSlot + 4u * sub + 2 * q);
          }
#pragma unroll
        for (int jc = 0; jc < JC; ++jc) {
          const uint32_t j = c * JC + jc;
          vj[jc] = j < cnt;
          const double dt = tq - rrow[j < k ? j : k - 1u].t;
#pragma unroll
          for (int t = 0; t < NT; ++t) {
            const float c0 = cos_rev(om[t][0].x * dt + ph[t][0].x), c1 = cos_rev(om[t][0].y * dt + ph[t][0].y);
            const float c2 = cos_rev(om[t][1].x * dt + ph[t][1].x), c3 = cos_rev(om[t][1].y * dt + ph[t][1].y);
            float4 zz;
            zz.x = tok[t][0] ? c0 : 0.0f;
            zz.y = tok[t][1] ? c1 : 0.0f;
            zz.z = tok[t][2] ? c2 : 0.0f;
            zz.w = tok[t][3] ? c3 : 0.0f;
            zt[jc][t] = zz;
          }
        }
        // scores
        float sc[JC][H];
#pragma unroll
        for (int h = 0; h < H; ++h) {
          float p[JC];
#pragma unroll
          for (int jc = 0; jc < JC; ++jc) p[jc] = 0.0f;
#pragma unroll
          for (int s = 0; s < NS; ++s) {
            float4 qv;
            if constexpr (QREG) qv = qt[h][s];
            else qv = *reinterpret_cast<const float4*>(zq + h * Zp + s * kSlot);
#pragma unroll
            for (int jc = 0; jc < JC; ++jc)
              p[jc] = dot4(qv, s < NG ? zb.g[jc][s < NG ? s : 0] : zt[jc][s < NG ? 0 : s - NG], p[jc]);
          }
#pragma unroll
          for (int jc = 0; jc < JC; ++jc) {
            const float t = row16_sum(p[jc]);
            sc[jc][h] = vj[jc] ? t : -INFINITY;
          }
        }
        // softmax against a reference score that only moves when a score exceeds it by a wide
        // margin (any reference gives the same quotient; the margin keeps exp() in range)
        bool need = false;
        float smax[H];
#pragma unroll
        for (int h = 0; h < H; ++h) {
          smax[h] = sc[0][h];
#pragma unroll
          for (int jc = 1; jc < JC; ++jc) smax[h] = fmaxf(smax[h], sc[jc][h]);
          need = need || smax[h] > mref[h] + 30.0f;
        }
        if (__any(need)) {
#pragma unroll
          for (int h = 0; h < H; ++h) {
            const bool mv = smax[h] > mref[h] + 30.0f;
            const float mnew = mv ? smax[h] : mref[h];
            const float scale = mv ? __expf(mref[h] - mnew) : 1.0f;     // exp(-inf) = 0 on the first move
            lrun[h] *= scale;
#pragma unroll
            for (int s = 0; s < NS; ++s) {
              acc[h][s].x *= scale; acc[h][s].y *= scale; acc[h][s].z *= scale; acc[h][s].w *= scale;
            }
            mref[h] = mnew;
          }
        }
#pragma unroll
        for (int h = 0; h < H; ++h) {
#pragma unroll
          for (int jc = 0; jc < JC; ++jc) {
            const float p = vj[jc] ? __expf(sc[jc][h] - mref[h]) : 0.0f;
            lrun[h] += p;
#pragma unroll
            for (int s = 0; s < NS; ++s) {
              const float4 zv = s < NG ? zb.g[jc][s < NG ? s : 0] : zt[jc][s < NG ? 0 : s - NG];
              acc[h][s].x = fmaf(p, zv.x, acc[h][s].x);
              acc[h][s].y = fmaf(p, zv.y, acc[h][s].y);
              acc[h][s].z = fmaf(p, zv.z, acc[h][s].z);
              acc[h][s].w = fmaf(p, zv.w, acc[h][s].w);
            }
          }
        }
      };
      if (nchunk3) pingpong_clamped<ZBuf>(nchunk3, z0, gather, attend);
      // zb overwrites qt (each lane owns its float4s; padding lanes hold zeros)
      float* zw = Zs + local * ll.ldz + 4u * sub;
#pragma unroll
      for (int h = 0; h < H; ++h) {
        const float inv = cnt ? 1.0f / lrun[h] : 0.0f;
#pragma unroll
        for (int s = 0; s < NS; ++s) {
          float4 o = acc[h][s];
          o.x *= inv; o.y *= inv; o.z *= inv; o.w *= inv;
          *reinterpret_cast<float4*>(zw + h * Zp + s * kSlot) = o;
        }
      }
    }
    // ================================================================ phase 4: o_h = zb_h W_V,h
    {
      // K runs over the slots, one chunk per slot; the operands of the next slot are in flight
      // during the current one.  The weights of the first slot are requested ahead of the barrier.
      Ops16<2> ov[2];
      uint32_t x = wave;
      auto wv = [&](uint32_t h, uint32_t nt) { return a.WV + (size_t)(h * ntk + nt) * g_z * kGrpFloats; };
      uint32_t h4 = 0, n0 = 0, n1 = 0;
      bool two4 = false;
      auto decode4 = [&](uint32_t xx) {
        h4 = xx / np4;
        n0 = 2u * (xx - h4 * np4);
        two4 = n0 + 1u < ntk;
        n1 = two4 ? n0 + 1u : n0;
      };
      decode4(x < nunits4 ? x : nunits4 - 1u);
      load_b16(wv(h4, n0), 0, ov[0].b[0]);
      load_b16(wv(h4, n1), 0, ov[0].b[1]);
      __syncthreads();
      if (pf_ok) stage_b(); else stage_none();                // next tile's rows, in flight during phases 4 and 5
      for (; x < nunits4; x += 4) {
        if (x != wave) {
          decode4(x);
          load_b16(wv(h4, n0), 0, ov[0].b[0]);
          load_b16(wv(h4, n1), 0, ov[0].b[1]);
        }
        const float* Ap = Zs + h4 * Zp + a_z;
        const float* B0 = wv(h4, n0);
        const float* B1 = wv(h4, n1);
        load_a16(Ap, 0, ov[0].a);
        floatx4 acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
#pragma unroll
        for (int c = 0; c < NS; ++c) {
          if (c + 1 < NS) {
            load_a16(Ap, (c + 1) * kCG, ov[(c + 1) & 1].a);
            load_b16(B0, (c + 1) * kCG, ov[(c + 1) & 1].b[0]);
            load_b16(B1, (c + 1) * kCG, ov[(c + 1) & 1].b[1]);
          }
          __builtin_amdgcn_sched_barrier(0);      // requests stay ahead of the products they overlap
          mfma16_chunk<2>(ov[c & 1], acc);
          __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          const uint32_t col = (t ? n1 : n0) * 16 + m16_col(lane);
          if ((t == 0 || two4) && col < dk) {
            float* op = Xs + c_off_x - m16_col(lane) + h4 * dk + col;
#pragma unroll
            for (int r = 0; r < 4; ++r) op[r * ll.ldx] = acc[t][r];
          }
        }
      }
    }
    // ================================================================ phase 5: h' = o W_O + b_O
    {
      Ops16<2> oo;
      load_b16(a.WO + (size_t)w1 * g_de * kGrpFloats, 0, oo.b[0]);
      load_b16(a.WO + (size_t)(w1 + 4 < ntd ? w1 + 4 : w1) * g_de * kGrpFloats, 0, oo.b[1]);
      __syncthreads();
      for (uint32_t nt = wave; nt < ntd; nt += 8) {
        const bool two = nt + 4 < ntd;
        const float* const Bt[2] = {a.WO + (size_t)nt * g_de * kGrpFloats, a.WO + (size_t)(two ? nt + 4 : nt) * g_de * kGrpFloats};
        floatx4 acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
        if (nt != wave) { load_b16(Bt[0], 0, oo.b[0]); load_b16(Bt[1], 0, oo.b[1]); }
        mfma16_gemm_pre<2>(Xs + a_x, c_de, Bt, acc, oo);
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          const uint32_t col = (nt + 4 * t) * 16 + m16_col(lane);
          if ((t == 0 || two) && col < a.d_emb) {
            const float b = a.bO[col];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              const uint32_t node = s_node[m16_row(lane, r)];
              if (node != 0xFFFFFFFFu) a.Hout[(size_t)node * a.ld_out + col] = acc[t][r] + b;
            }
          }
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
  if (blockIdx.x == 0 && threadIdx.x == 0 && n) atomicAdd((unsigned long long*)&a.ctrl->tot_rows, (unsigned long long)n);
}

// ---- dispatch over (slots, time slots, heads, chunk)
struct LaunchArgs {
  LayerArgs k;
  hipStream_t s; const uint32_t* rows; const uint32_t* cp; uint32_t cm;
  uint32_t nt;                      // time slots of this layer
  uint32_t grid_cap;                // workgroups that are resident at once (two per CU)
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
  if (blocks > a.grid_cap) blocks = a.grid_cap;   // persistent: each workgroup strides over the tiles, staging one tile ahead
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(kern, dim3((uint32_t)blocks), dim3(256), a.lds, a.s, a.k, a.rows, a.cp, a.cm);
}

template <int NS, int NT>
void go_h(LaunchArgs& a) {
  // ring entries per chunk are bounded by registers (two chunks of JC * NS float4 per lane in flight,
  // beside 2 * H * NS float4 of accumulators and qt values)
  switch (a.k.heads) {
    case 1: go<NS, NT, 1, (NS <= 4 ? 4 : NS == 5 ? 2 : 1)>(a); break;
    case 2: go<NS, NT, 2, (NS <= 4 ? 2 : 1)>(a); break;
    default: go<NS, NT, 4, 1>(a); break;
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
