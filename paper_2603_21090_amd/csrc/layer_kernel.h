// Temporal-attention layer for a list of target rows (paper Eq. attn_detail; Sec. 3.3 "Stage 4:
// Incremental Embedding Generation", exact recomputation of the affected rows; Sec. 3.6 "Parallel
// Batch Processing", one batched kernel over the affected set), one fused kernel per layer.
//
// Keys and values are linear in z_j = [h_{u_j} | e_j | phi(t_v - t_j)].  Their node and edge terms are
// cached rows (per node / per edge, [keys | values], see LayerDev); the time term is re-associated so
// that its dense products run over rows instead of (row, neighbour) pairs:
//     score_{h,j} = q_h . (kn_{u_j} + ke_j)_h + qt_h . phi_j ,     qt_h = W_K,h[time] q_h      (q carries 1/sqrt(dk))
//     o_h         = sum_j a_{h,j} (vn_{u_j} + ve_j)_h + pb_h W_V,h[time] ,   pb_h = sum_j a_{h,j} phi_j
// Edge features of at most one 64-float slot are not cached at all (ES variants): the raw row rides with the
// time encoding, z_j = [phi_j | e_j] in place of phi_j and W[time | edge] in place of W[time] above, and the
// cached rows hold the node terms alone.
// A workgroup of four waves owns 16 target rows and runs its phases without leaving the CU:
//   1. q  = h_v W_Q(node block) + phi(0) W_Q(time block)                           (MFMA 16x16x4)
//   2. qt_h = q_h W_K,h[time]^T, kept in LDS                                        (MFMA)
//   3. gather the cached rows of the ring entries, time encodings, scores, softmax, weighted sums;
//      one wave serves four rows, 16 lanes x float4 per 64-float slot                (HBM / vector ALU)
//   4. o_h += pb_h W_V,h[time]                                                       (MFMA)
//   5. h_v' = [o_1 | .. | o_H] W_O + b_O, written into the layer cache               (MFMA)
//   6. unless this is the last layer: the row's own cached keys|values for the next layer,
//      h_v' [W_K | W_V](node rows of layer l + 1)                                     (MFMA)
// Weights stream from L2 (group-major packing, see mfma16.h); several workgroups per CU overlap one's
// gather with another's products.
#pragma once
#include <mutex>
#include <type_traits>
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

// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>): register arrays indexed by constants
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (N > 0) {
    static_for<N - 1>(f);
    f(std::integral_constant<int, N - 1>{});
  }
}

struct LayerLds {
  uint32_t ldx, ldq, ldz;        // strides (floats) of the X / O tile, the Q / H' tile and the qt / pb tile
  uint32_t off_q, off_z, off_r, off_sc, total;
};

// Every stride is 4 (mod 8) floats: rows stay 16-byte aligned and the 16 rows of an operand read
// fall into distinct banks.  ks = key slots (heads * slots per head), nz = slots of z = [phi | raw edge row].
__host__ __device__ inline LayerLds layer_lds(uint32_t d_in, uint32_t heads, uint32_t ks, uint32_t nz, uint32_t k, bool delta) {
  LayerLds l;
  const uint32_t wx = round_up(d_in, kGrpK), wo = kSlot * ks;
  l.ldx = (wx > wo ? wx : wo) + 4;                // the input tile and the head-output tile share storage
  l.ldq = wo + 4;                                 // q in the padded-head layout, later the output rows h'
  l.ldz = heads * kSlot * nz + 4;
  l.off_q = kTM * l.ldx;
  l.off_z = l.off_q + kTM * l.ldq;
  l.off_r = l.off_z + kTM * l.ldz + 4 * kGrpK;    // operand reads may run one chunk past the last row
  l.off_sc = l.off_r + kTM * k * 4;               // the ring records of the tile's rows, 16 bytes each
  l.total = l.off_sc + (delta ? kTM * k * heads : 0u);       // delta mode: the scores of a row's entries until its weights are known
  return l;
}

// Everything the kernel needs, and nothing else (keeps the scalar register file uncrowded).
struct LayerArgs {
  const float* Hin; float* Hout;
  const float* KVn; const float* KVe;              // cached key|value rows of the input table's nodes / of the edges
                                                   // (ES variants: KVe holds the raw feature rows, one slot each)
  float* KVout;                                    // the next layer's node table (null for the last layer)
  // root-node inference: query time per list row instead of the node's last-interaction time, and the
  // output rows go to out_rows[list position] instead of the layer cache (both null otherwise)
  const double* tq_rows; float* out_rows;
  double window;                                   // ring entries older than the query time minus this are ignored (+inf: none)
  const RingEntry* ring; const uint32_t* deg; const double* t_last;
  const double* om_rev; const double* ph_rev;
  Ctrl* ctrl;
  uint64_t* gathered_slots;                        // statistic: ring entries gathered, one plain counter per workgroup index
  const float *WQ, *cQ, *WKT, *WV, *WO, *bO, *WKVnext;   // matrices group-major (mfma16.h)
  uint32_t ld_in, ld_out, ld_kv, ld_kve;           // ld_kve = 0 without edge features (every edge reads one zero row)
  uint32_t k, d_in, d_emb, dk, d_time, d_edge;
  // query cache (both null: off): this layer's cached q | qt rows, [node][64 (KS + H NZ)], and per tile of the
  // row list whether every row's input row is unchanged (then q and qt are read back, not projected); a
  // launch that must recompute everything passes tile_clean = null and still refreshes QC
  float* QC; const uint8_t* tile_clean;
  uint32_t all_clean;                              // every listed row reads q | qt back (root-node inference: nothing changed)
  // delta mode (read by the delta variant only): the batch's dirty flags and the highest flag whose owner's
  // input row of this layer changed (a row at or below it, or an endpoint, is recomputed exactly; an entry whose
  // neighbour is at or below it is a changed entry); the attention cache of this layer; the drift estimator
  const uint8_t* flags;
  uint32_t thr_in, force_exact, is_final;
  float gamma;
  float *ac_S, *ac_P, *ac_ZM, *ac_W, *ac_V;
  DriftCtl* drift; float* dsum; uint32_t* dlast; uint8_t* dseen;
};

// cached rows (node and edge, keys and values) of one chunk of JC ring entries, one float4 per lane and slot;
// ES: the edge's raw feature row (one slot) instead of its cached row
template <int JC, int KS, int ES>
struct GatherBuf {
  float4 n[JC][2 * KS];
  float4 e[JC][ES ? 1 : 2 * KS];
};

// KS key slots in total (heads x slots per head), NT time slots; JC ring entries fetched together.
// ES = 1: raw edge rows.  The vector z_j = [phi(dt_j) | f_j] of NZ = NT + 1 slots takes the place of phi(dt_j)
// in the re-associated time products (scores: (W_K,h[time | edge] q_h) . z_j; values: (sum_j a_j z_j)
// W_V,h[time | edge]), and the cached rows hold the node parts alone.
// DELTA: the approximate mode of Sec. 3.3 "Stage 4" (attention cache, delta update of changed entries).
// QCACHE: the query cache is in use (rows may read q and qt back, rows that project store theirs).
template <int KS, int NT, int ES, int H, int JC, int WGS, bool DELTA, bool QCACHE>
__global__ __launch_bounds__(256, WGS) void layer_kernel(LayerArgs a, const uint32_t* __restrict__ rows,
                                                         const uint32_t* count_ptr, uint32_t count_max) {
  extern __shared__ __align__(16) float lds[];
  __shared__ uint32_t s_node[kTM], s_cnt[kTM], s_next[kTM], s_ex[kTM], s_cleann;
  __shared__ double s_tq[kTM], s_tqn[kTM];
  __shared__ __align__(16) double s_om[NT * kSlot], s_ph[NT * kSlot];
  static_assert(KS % H == 0, "whole slots per head");
  static_assert(!(DELTA && ES), "the delta mode keeps projected edge rows");
  constexpr int SH = KS / H;                  // slots per head
  constexpr int NZ = NT + ES;                 // slots of z
  constexpr uint32_t Ztp = NZ * kSlot;        // floats of one head's qt / pb vector
  // (a batch that failed validation leaves every per-layer count at zero: nothing to test here, and the
  // control block's batch fields may already belong to the next batch, whose front part runs concurrently)
  uint32_t n = count_max;
  if (count_ptr) { const uint32_t c = *count_ptr; n = c < count_max ? c : count_max; }
  const uint32_t ntiles = (n + kTM - 1) / kTM;
  // Per-lane indices and everything derived from them are re-derived at the top of every tile from an
  // opaque copy of the thread index: otherwise the compiler hoists dozens of loop-invariant address
  // registers out of the persistent tile loop and keeps them alive (or spilled) across all phases.
  uint32_t tid = threadIdx.x, lane = tid & 63u, sub = lane & 15u, grp = lane >> 4;
  // wave index, made provably uniform so that tile indices and weight addresses stay in scalar registers
  const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const uint32_t k = a.k, dk = a.dk;
  const uint32_t c_in = chunks_of(a.d_in), c_de = chunks_of(a.d_emb);                                     // chunks of K
  const uint32_t g_in = kCG * c_in, g_de = kCG * c_de, g_dk = kCG * SH, g_zt = kCG * NZ, g_o = kCG * KS;  // groups of K
  const uint32_t ntd = round_up(a.d_emb, 16) >> 4, ntk = round_up(dk, 16) >> 4;                           // column tiles
  constexpr uint32_t ntz = Ztp >> 4;                                                                       // tiles of a qt vector
  const uint32_t nzt_t = (a.d_time + 15u) >> 4, nzt = nzt_t + (ES ? (a.d_edge + 15u) >> 4 : 0u);           // ... that hold valid columns
  const LayerLds ll = layer_lds(a.d_in, H, KS, NZ, k, DELTA);
  float* Xs = lds;                            // input rows (phases 0-1), then head outputs (phases 3-5)
  float* Qs = lds + ll.off_q;                 // q (phases 1-3), then the output rows (phases 5-6)
  float* Zs = lds + ll.off_z;                 // qt (phases 2-3), then pb (phases 3-4)
  RingEntry* Rs = reinterpret_cast<RingEntry*>(lds + ll.off_r);   // [row][j], j = 0 the most recent entry
  using ZBuf = GatherBuf<JC, KS, ES>;

  // ---- per-lane constants
  // time-encoding parameters (omega, phase in revolutions) live in LDS, zero past d_time
  for (uint32_t q = threadIdx.x; q < NT * kSlot; q += 256) {
    s_om[q] = q < a.d_time ? a.om_rev[q] : 0.0;
    s_ph[q] = q < a.d_time ? a.ph_rev[q] : 0.0;
  }
  // operand padding (columns nobody writes) must be finite: clear the tiles once
  for (uint32_t x = threadIdx.x; x < ll.off_r; x += 256) lds[x] = 0.0f;
  uint32_t gathered = 0;
  double drift_sum = 0.0;                     // delta mode: this wave's share of the drift estimator's sum and member count
  uint32_t drift_new = 0;
  uint32_t a_x, a_q, a_z, c_off_x, c_off_q, c_off_z;
  auto derive_lane = [&]() {
    asm volatile("" : "+v"(tid));
    lane = tid & 63u; sub = lane & 15u; grp = lane >> 4;
    a_x = (lane & 15u) * ll.ldx + 4u * (lane >> 4);
    a_q = (lane & 15u) * ll.ldq + 4u * (lane >> 4);
    a_z = (lane & 15u) * ll.ldz + 4u * (lane >> 4);
    c_off_x = (4u * (lane >> 4)) * ll.ldx + (lane & 15u);
    c_off_q = (4u * (lane >> 4)) * ll.ldq + (lane & 15u);
    c_off_z = (4u * (lane >> 4)) * ll.ldz + (lane & 15u);
  };
  derive_lane();

  // ---- phase-2 work units: (head, pair of valid qt column tiles); wave w owns units w, w + 4, ...
  // Lane i of `udesc` holds the description of the wave's i-th unit (head, first tile, whether a
  // second tile follows), worked out once; inside the tile loop a unit costs one cross-lane read.
  const uint32_t npr = (nzt + 1u) >> 1, nunits2 = H * npr;
  const uint32_t nu2 = wave < nunits2 ? (nunits2 - wave + 3u) >> 2 : 0u;     // units of this wave
  struct Unit2 { uint32_t h, t0, t1; bool two; };
  uint32_t udesc = 0;
  if (lane < nu2) {
    // the i-th valid tile: time tiles first, then (raw edge rows) the tiles of slot NT
    auto vt = [&](uint32_t i) { return i < nzt_t ? i : 4u * NT + (i - nzt_t); };
    const uint32_t x = wave + 4u * lane, h = x / npr, i0 = 2u * (x - h * npr);
    const uint32_t two = i0 + 1u < nzt ? 1u : 0u;
    udesc = h | (vt(i0) << 8) | (vt(i0 + two) << 16) | (two << 24);
  }
  auto decode2 = [&](uint32_t i) {
    const uint32_t dsc = (uint32_t)__builtin_amdgcn_readlane((int)udesc, (int)i);
    Unit2 u;
    u.h = dsc & 0xFFu; u.t0 = (dsc >> 8) & 0xFFu; u.t1 = (dsc >> 16) & 0xFFu; u.two = (dsc >> 24) != 0u;
    return u;
  };
  auto wkt = [&](uint32_t h, uint32_t t) { return a.WKT + (size_t)(h * ntz + t) * g_dk * kGrpFloats; };
  auto store2 = [&](const Unit2& u, const floatx4 (&acc)[2]) {
    float* zp = Zs + u.h * Ztp + c_off_z;
#pragma unroll
    for (int r = 0; r < 4; ++r) zp[u.t0 * 16 + r * ll.ldz] = acc[0][r];
    if (u.two) {
#pragma unroll
      for (int r = 0; r < 4; ++r) zp[u.t1 * 16 + r * ll.ldz] = acc[1][r];
    }
  };
  // ---- phase-4 work units: (head, pair of head-output column tiles)
  const uint32_t np4 = (ntk + 1u) >> 1, nunits4 = H * np4;
  // ---- phases 1 and 5: column tiles nt and nt + 4 of the d_emb outputs form a unit; the bias values of
  // a wave's first unit stay in registers (further units, d_emb > 128, read theirs when they get there)
  float cq_r[2], bo_r[2];
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    const uint32_t col = (wave + 4 * t) * 16 + m16_col(lane);
    cq_r[t] = col < a.d_emb ? a.cQ[col] : 0.0f;
    bo_r[t] = col < a.d_emb ? a.bO[col] : 0.0f;
  }
  __syncthreads();

  // ---- staging of a tile, one tile ahead.  Stage A requests the tile's row ids (ahead of phase 1) and
  // puts them into s_next once they are there (end of phase 2); stage B (issued with the first gathers of
  // phase 3, whose waits cover it: a later wait for a weight chunk would stall on it, loads return in
  // order) fetches, into registers, this thread's
  // share of the rows' ring slots, degrees, query times and own input rows; the tile's phase 0 then
  // only moves registers into LDS.  A workgroup strides over many tiles, so all but its first tile
  // start without waiting for memory.  Shapes whose share does not fit two items per thread stage
  // inside phase 0 instead.
  const uint32_t qpr = round_up(a.d_in, kGrpK) >> 2;          // 16-byte quads per staged input row
  const bool pf_ok = kTM * k <= 512u && kTM * qpr <= 512u;
  RingEntry p_ring[2];
  uint32_t p_deg[2];
  double p_tl[2];
  float4 p_x[2];                                              // own input rows (not fetched for a tile that reads q | qt back)
  constexpr int NQ = KS + H * NZ;                             // quads per thread of a tile's cached q | qt rows
  constexpr uint32_t QW4 = 16u * NQ;                          // quads per cached row
  uint32_t p_row = 0xFFFFFFFFu, p_clean = 0u;
  double p_tqn = 0.0;
  auto stage_a = [&](uint32_t t) {                            // requests only: nothing waits for the values here
    if (tid < kTM) {
      const uint32_t r = t * kTM + tid;
      p_row = (t < ntiles && r < n) ? (rows ? rows[r] : r) : 0xFFFFFFFFu;
      p_tqn = (a.tq_rows && t < ntiles && r < n) ? a.tq_rows[r] : 0.0;
      if constexpr (QCACHE) { if (tid == 0) p_clean = t < ntiles ? (a.all_clean ? 1u : a.tile_clean ? a.tile_clean[t] : 0u) : 0u; }
    }
  };
  auto stage_a_commit = [&]() {
    if (tid < kTM) { s_next[tid] = p_row; s_tqn[tid] = p_tqn; }
    if constexpr (QCACHE) { if (tid == 0) s_cleann = p_clean; }
  };
  auto stage_b = [&]() {
    const bool cl = QCACHE && __builtin_amdgcn_readfirstlane((int)s_cleann) != 0;
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      const uint32_t x = tid + 256u * e;
      {
        const uint32_t xc = x < kTM * k ? x : 0u;
        const uint32_t r = xc / k, sl = xc - r * k;
        const uint32_t node = s_next[r];
        const uint32_t nn = node != 0xFFFFFFFFu ? node : 0u;
        p_ring[e] = a.ring[(size_t)nn * k + sl];
        p_deg[e] = a.deg[nn];
        p_tl[e] = a.t_last[nn];
      }
      if (!cl) {
        const uint32_t xc = x < kTM * qpr ? x : 0u;
        const uint32_t r = xc / qpr, q = xc - r * qpr;
        const uint32_t node = s_next[r];
        // columns past d_in are row padding of the table (zero)
        p_x[e] = *reinterpret_cast<const float4*>(a.Hin + (size_t)(node != 0xFFFFFFFFu ? node : 0u) * a.ld_in + 4u * q);
      } else {
        p_x[e] = make_float4(0.f, 0.f, 0.f, 0.f);
      }
    }
  };
  // the record of adjacency position p sits in ring slot p mod k; with the row's degree known, slot
  // sl holds the j-th most recent entry, j = (newest - sl) mod k; places past the row's entry count
  // name node 0 / edge 0 (finite cached rows whose weight in every sum is zero)
  auto place_ring = [&](uint32_t r, uint32_t sl, bool live, RingEntry e, uint32_t dg_in, double tl) {
    const uint32_t dg = live ? dg_in : 0u;
    const uint32_t cnt = dg < k ? dg : k;
    const uint32_t newest = dg ? (dg - 1u) % k : 0u;
    const uint32_t j = newest >= sl ? newest - sl : newest + k - sl;
    if (j >= cnt) { e.nbr = 0u; e.eid = 0u; e.t = 0.0; }
    Rs[r * k + j] = e;
    if (sl == 0) { s_cnt[r] = cnt; s_tq[r] = a.tq_rows ? s_tqn[r] : tl; }
  };
  stage_a(blockIdx.x);
  stage_a_commit();
  __syncthreads();
  auto stage_none = [&]() {                                   // keeps the registers defined on every path
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      p_ring[e].nbr = 0u; p_ring[e].eid = 0u; p_ring[e].t = 0.0; p_deg[e] = 0u; p_tl[e] = 0.0;
    }
    p_x[0] = p_x[1] = make_float4(0.f, 0.f, 0.f, 0.f);
  };
  if (pf_ok) stage_b(); else stage_none();

  // Round i gives workgroup b the tile i G + (b + 37 i) mod G (G workgroups): every round is a permutation of
  // its G tiles, and a workgroup's position inside the round moves from round to round.  The row list may
  // be regrouped by entry count in windows of 256 tiles (long rows first), so a fixed position would hand
  // the same workgroups every long tile.
  const uint32_t G = gridDim.x;
  auto tile_of = [&](uint32_t i) { return i * G + (blockIdx.x + 37u * i) % G; };
  for (uint32_t round = 0;; ++round) {
    const uint32_t tile = tile_of(round);
    if (tile >= ntiles) break;                                // wave-uniform; only in a workgroup's last round
    derive_lane();
    // every row of the tile has its q and qt in the query cache (set by the staging of a tile ago; uniform)
    const bool clean = QCACHE && __builtin_amdgcn_readfirstlane((int)s_cleann) != 0;
    // ================================================================ phase 0: stage the tile
    Ops16<2> oq;                                              // first weight chunk of this wave's first unit
    const uint32_t w1 = wave < ntd ? wave : 0u;              // loads are unconditional (clamped), products are not
    if (!clean) {
      load_b16(a.WQ + (size_t)w1 * g_in * kGrpFloats, 0, oq.b[0]);
      load_b16(a.WQ + (size_t)(w1 + 4 < ntd ? w1 + 4 : w1) * g_in * kGrpFloats, 0, oq.b[1]);
    }
    if (tid < kTM) {
      s_node[tid] = s_next[tid];
      if constexpr (DELTA) {
        // exact recomputation for endpoints of the batch (query time and entries moved), for rows whose own
        // input row changed (every score moves), and whenever the caller asks for it
        const uint32_t node = s_next[tid];
        const uint32_t fl = node != 0xFFFFFFFFu ? a.flags[node] : 0u;
        s_ex[tid] = (a.force_exact || fl == 1u || (fl != 0u && fl <= a.thr_in)) ? 1u : 0u;
      }
    }
    if (pf_ok) {
      // everything was fetched a tile ago: registers -> LDS
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        const uint32_t x = tid + 256u * e;
        if (x < kTM * k) {
          const uint32_t r = x / k, sl = x - r * k;
          place_ring(r, sl, s_next[r] != 0xFFFFFFFFu, p_ring[e], p_deg[e], p_tl[e]);
        }
        if (!clean && x < kTM * qpr) {
          const uint32_t r = x / qpr, q = x - r * qpr;
          const float4 v = s_next[r] != 0xFFFFFFFFu ? p_x[e] : make_float4(0.f, 0.f, 0.f, 0.f);
          *reinterpret_cast<float4*>(Xs + r * ll.ldx + 4u * q) = v;
        }
      }
    }
    __syncthreads();
    if (!pf_ok) {
      // thread (row, slot) fetches its slot without waiting for the row's degree (both loads leave together)
      for (uint32_t x = tid; x < kTM * k; x += 256) {
        const uint32_t r = x / k, sl = x - r * k;
        const uint32_t node = s_node[r];
        const bool live = node != 0xFFFFFFFFu;
        const uint32_t nn = live ? node : 0u;
        place_ring(r, sl, live, a.ring[(size_t)nn * k + sl], a.deg[nn], a.t_last[nn]);
      }
      const uint32_t total = kTM * qpr;
      for (uint32_t x0 = tid; x0 < total; x0 += 512u) {
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
    stage_a(tile_of(round + 1u));                            // row ids of this workgroup's next tile
    // ---- this lane group's row: entry count, query time, ring records; the first chunk of cached
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
        const float* nrow = a.KVn + (size_t)e.nbr * a.ld_kv + 4u * sub;
        const float* erow = a.KVe + (size_t)e.eid * a.ld_kve + 4u * sub;
#pragma unroll
        for (int s = 0; s < 2 * KS; ++s) {
          zb.n[jc][s] = *reinterpret_cast<const float4*>(nrow + s * kSlot);
          if constexpr (!ES) zb.e[jc][s] = *reinterpret_cast<const float4*>(erow + s * kSlot);
        }
        if constexpr (ES) zb.e[jc][0] = *reinterpret_cast<const float4*>(erow);
      }
    };
    ZBuf z0;
    if (clean) {
      // the rows' q and qt from the query cache, requested together with the first gather (whose wait at
      // the start of phase 3 is there in any case), then into their tiles
      float4 qv[NQ];
      static_for<NQ>([&](auto E) {
        constexpr int e = decltype(E)::value;
        const uint32_t x = tid + 256u * e, r = x / QW4, q4 = x - r * QW4;
        const uint32_t node = s_node[r];
        qv[e] = *reinterpret_cast<const float4*>(a.QC + (size_t)(node != 0xFFFFFFFFu ? node : 0u) * (4u * QW4) + 4u * q4);
      });
      if constexpr (!DELTA) gather(0, z0);
      static_for<NQ>([&](auto E) {
        constexpr int e = decltype(E)::value;
        const uint32_t x = tid + 256u * e, r = x / QW4, q4 = x - r * QW4;
        const float4 v = s_node[r] != 0xFFFFFFFFu ? qv[e] : make_float4(0.f, 0.f, 0.f, 0.f);
        float* dst = q4 < 16u * KS ? Qs + r * ll.ldq + 4u * q4 : Zs + r * ll.ldz + 4u * (q4 - 16u * KS);
        *reinterpret_cast<float4*>(dst) = v;
      });
    } else {
    if constexpr (!DELTA) gather(0, z0);
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
          const float cq = nt == wave ? cq_r[t] : a.cQ[col];
          const uint32_t h = col / dk;
          float* qp = Qs + m16_row(lane, 0) * ll.ldq + h * (SH * kSlot) + (col - h * dk);
#pragma unroll
          for (int r = 0; r < 4; ++r) qp[r * ll.ldq] = acc[t][r] + cq;
        }
      }
    }
    // ================================================================ phase 2: qt_h = q_h W_K,h[time]^T
    {
      Ops16<2> o2;
      Unit2 ua = decode2(0);                                  // weights of the first unit are requested
      load_b16(wkt(ua.h, ua.t0), 0, o2.b[0]);                 // ahead of the barrier (unit 0 of an idle wave: head 0, tile 0)
      load_b16(wkt(ua.h, ua.t1), 0, o2.b[1]);
      __syncthreads();
      if constexpr (SH == 1) {
        // one chunk per unit: the operands of the next unit are in flight during this unit's products
        load_a16(Qs + ua.h * kSlot + a_q, 0, o2.a);
        if (nu2) pingpong_peeled<Ops16<2>>(
            nu2, o2,
            [&](uint32_t i, Ops16<2>& o) {
              const Unit2 u = decode2(i);
              load_a16(Qs + u.h * kSlot + a_q, 0, o.a);
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
          if (i) { load_b16(Bt[0], 0, o2.b[0]); load_b16(Bt[1], 0, o2.b[1]); }
          mfma16_gemm_pre<2>(Qs + ua.h * (SH * kSlot) + a_q, SH, Bt, acc, o2);
          store2(ua, acc);
        }
      }
    }
    }  // q and qt: read back, or projected
    stage_a_commit();                                         // requested ahead of the loads waited for above: here by now
    __syncthreads();
    // next tile's rows, in flight among the gathers of phase 3 (four-slot shapes have no registers to
    // spare in phase 3: theirs are requested behind it)
    if constexpr (KS <= 2) { if (pf_ok) stage_b(); else stage_none(); }
    if (QCACHE && !clean && !a.out_rows) {                    // the rows' q | qt for later batches
      static_for<NQ>([&](auto E) {
        constexpr int e = decltype(E)::value;
        const uint32_t x = tid + 256u * e, r = x / QW4, q4 = x - r * QW4;
        const uint32_t node = s_node[r];
        const float* src = q4 < 16u * KS ? Qs + r * ll.ldq + 4u * q4 : Zs + r * ll.ldz + 4u * (q4 - 16u * KS);
        if (node != 0xFFFFFFFFu) *reinterpret_cast<float4*>(a.QC + (size_t)node * (4u * QW4) + 4u * q4) = *reinterpret_cast<const float4*>(src);
      });
      __syncthreads();                                        // phase 3 puts pb where qt is: not before every thread has read its share
    }
    // ================================================================ phase 3: gather + attention
    // The time encodings are not masked per entry: a column past d_time has omega = phase = 0 and comes out as
    // cos(0) = 1.  In the scores it meets an exact zero of qt (zero weight columns; tiles phase 2 does not
    // write hold what the previous tile's pb left there, hence the zeros written here), and its share of pb
    // is cleared once per row, when pb goes into its tile.
    auto clear_past_d_time = [&](float4& o, int t) {
      const uint32_t c0 = (uint32_t)t * kSlot + 4u * sub;
      o.x = c0 < a.d_time ? o.x : 0.0f;
      o.y = c0 + 1u < a.d_time ? o.y : 0.0f;
      o.z = c0 + 2u < a.d_time ? o.z : 0.0f;
      o.w = c0 + 3u < a.d_time ? o.w : 0.0f;
    };
    if constexpr (DELTA) {
      // ---- delta mode.  An exact row runs the same online softmax as the exact mode and leaves its attention
      // cache behind: per entry score, weight and the neighbour|edge part of the value, per row the sums S and
      // pb, the denominator and its reference score.  A delta row starts from its cached sums and visits only
      // the entries whose neighbour's input row changed: new score, denominator Z' = Z - e_old + e_new, new
      // weight e_new / Z', sums corrected by (new weight x new value) - (old weight x old value); the
      // other entries keep the weight they have (Eq. delta_embedding, "updated neighbours").
      float* Sc = lds + ll.off_sc;
      const uint32_t node = s_node[local];
      const bool live = node != 0xFFFFFFFFu;
      const uint32_t nn = live ? node : 0u;
      const bool ex = s_ex[local] != 0u;
      float* acS = a.ac_S + (size_t)nn * (kSlot * KS) + 4u * sub;
      float* acP = a.ac_P + (size_t)nn * (kSlot * NT * H) + 4u * sub;
      float* acZM = a.ac_ZM + (size_t)nn * (2 * H);
      // (first, and behind a fence of its own: a fence further down would wait for the cache reads below)
      for (uint32_t j = sub; j < cnt; j += 16)
#pragma unroll
        for (int h = 0; h < H; ++h) Sc[(local * k + j) * H + h] = -INFINITY;
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      float4 accv[KS], accp[H][NT];
      float mref[H], lrun[H];                                 // exact row: running reference and denominator; delta row: m and Z
#pragma unroll
      for (int s = 0; s < KS; ++s) accv[s] = ex ? make_float4(0.f, 0.f, 0.f, 0.f) : *reinterpret_cast<const float4*>(acS + s * kSlot);
#pragma unroll
      for (int h = 0; h < H; ++h) {
#pragma unroll
        for (int t = 0; t < NT; ++t)
          accp[h][t] = ex ? make_float4(0.f, 0.f, 0.f, 0.f) : *reinterpret_cast<const float4*>(acP + (h * NT + t) * kSlot);
        mref[h] = ex ? -INFINITY : acZM[2 * h + 1];
        lrun[h] = ex ? 0.0f : acZM[2 * h];
      }
      float4 qk[KS];
#pragma unroll
      for (int s = 0; s < KS; ++s) qk[s] = *reinterpret_cast<const float4*>(Qs + local * ll.ldq + s * kSlot + 4u * sub);
      const float* zq = Zs + local * ll.ldz + 4u * sub;
      uint32_t nch = 0, nvalid = 0;
      const bool any_delta = __any(!ex);                      // (exact rows take every entry: no flags needed)
      struct DBuf { float4 n[2 * KS], e[2 * KS]; uint32_t j; };
      for (uint32_t jb = 0; jb < cmax; jb += 32u) {
        // Which of the entries jb .. jb + 31 each row takes, worked out at once (lane s of a row looks at entries
        // jb + s and jb + 16 + s: their window test and the flag of their neighbour), instead of one dependent
        // flag read per entry: an exact row takes its valid entries, a delta row the valid ones whose
        // neighbour's input row changed.
        uint32_t vmask = 0, cmask = 0;
#pragma unroll
        for (uint32_t half = 0; half < 2; ++half) {
          const uint32_t jj = jb + 16u * half + sub;
          bool v = false, c = false;
          if (jj < cnt) {
            const RingEntry e = rrow[jj];
            v = tq - e.t <= a.window;
            if (any_delta) { const uint32_t fl = a.flags[e.nbr]; c = fl != 0u && fl <= a.thr_in; }
          }
          const uint64_t bv = __ballot(v), bc = __ballot(c);
          vmask |= ((uint32_t)(bv >> (16u * grp)) & 0xFFFFu) << (16u * half);
          cmask |= ((uint32_t)(bc >> (16u * grp)) & 0xFFFFu) << (16u * half);
        }
        const uint32_t amask = ex ? vmask : (vmask & cmask);
        nvalid += (uint32_t)__popc(vmask);
        if (!ex) nch += (uint32_t)__popc(amask);
        // entries some row of the wave takes, in entry order; the cached rows of the next one are in flight
        // while the current one is worked on
        const uint32_t wmask = (uint32_t)__builtin_amdgcn_readlane((int)amask, 0) | (uint32_t)__builtin_amdgcn_readlane((int)amask, 16) |
                               (uint32_t)__builtin_amdgcn_readlane((int)amask, 32) | (uint32_t)__builtin_amdgcn_readlane((int)amask, 48);
        const uint32_t n_items = (uint32_t)__popc(wmask);
        if (n_items == 0u) continue;
        uint32_t cur_idx = 0, cur_mask = wmask;               // item c = the c-th set bit (requests come in ascending c)
        auto fetch = [&](uint32_t c, DBuf& bf) {
          while (cur_idx < c) { cur_mask &= cur_mask - 1u; ++cur_idx; }
          const uint32_t j = jb + (uint32_t)__builtin_ctz(cur_mask);
          bf.j = j;
          const RingEntry e = rrow[j];
          const bool act = (amask >> (j - jb)) & 1u;
          const float* nrow = a.KVn + (size_t)(act ? e.nbr : 0u) * a.ld_kv + 4u * sub;
          const float* erow = a.KVe + (size_t)(act ? e.eid : 0u) * a.ld_kve + 4u * sub;
#pragma unroll
          for (int s = 0; s < 2 * KS; ++s) {
            bf.n[s] = *reinterpret_cast<const float4*>(nrow + s * kSlot);
            bf.e[s] = *reinterpret_cast<const float4*>(erow + s * kSlot);
          }
        };
        auto work = [&](uint32_t, const DBuf& bf) {
        const uint32_t j = bf.j;
        const RingEntry e = rrow[j];
        const bool act = (amask >> (j - jb)) & 1u;
        const double dt = tq - e.t;
        float4 kk[KS], vv[KS];
#pragma unroll
        for (int s = 0; s < KS; ++s) {
          kk[s] = make_float4(bf.n[s].x + bf.e[s].x, bf.n[s].y + bf.e[s].y, bf.n[s].z + bf.e[s].z, bf.n[s].w + bf.e[s].w);
          vv[s] = make_float4(bf.n[KS + s].x + bf.e[KS + s].x, bf.n[KS + s].y + bf.e[KS + s].y,
                              bf.n[KS + s].z + bf.e[KS + s].z, bf.n[KS + s].w + bf.e[KS + s].w);
        }
        float4 zt[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          const double2 oa = *reinterpret_cast<const double2*>(s_om + t * kSlot + 4u * sub), ob = *reinterpret_cast<const double2*>(s_om + t * kSlot + 4u * sub + 2);
          const double2 pa = *reinterpret_cast<const double2*>(s_ph + t * kSlot + 4u * sub), pb = *reinterpret_cast<const double2*>(s_ph + t * kSlot + 4u * sub + 2);
          const float c0 = cos_rev(oa.x * dt + pa.x), c1 = cos_rev(oa.y * dt + pa.y);
          const float c2 = cos_rev(ob.x * dt + pb.x), c3 = cos_rev(ob.y * dt + pb.y);
          zt[t] = make_float4(c0, c1, c2, c3);           // (columns past d_time: see the exact variant)
        }
        float sc[H];
#pragma unroll
        for (int h = 0; h < H; ++h) {
          float p = 0.0f;
#pragma unroll
          for (int s = h * SH; s < (h + 1) * SH; ++s) p = dot4(qk[s], kk[s], p);
#pragma unroll
          for (int t = 0; t < NT; ++t) p = dot4(*reinterpret_cast<const float4*>(zq + h * Ztp + t * kSlot), zt[t], p);
          sc[h] = row16_sum(p);
        }
        if (act && live) {
          float* w = a.ac_W + ((size_t)nn * k + j) * (2 * H);
          float* vc = a.ac_V + ((size_t)nn * k + j) * (kSlot * KS) + 4u * sub;
          if (ex) {
#pragma unroll
            for (int h = 0; h < H; ++h) {
              const bool mv = sc[h] > mref[h] + 30.0f;
              const float mnew = mv ? sc[h] : mref[h];
              const float scale = mv ? __expf(mref[h] - mnew) : 1.0f;     // exp(-inf) = 0 on the first move
              mref[h] = mnew;
              const float p = __expf(sc[h] - mnew);
              lrun[h] = fmaf(lrun[h], scale, p);
#pragma unroll
              for (int s = h * SH; s < (h + 1) * SH; ++s) {
                accv[s].x = fmaf(accv[s].x, scale, p * vv[s].x); accv[s].y = fmaf(accv[s].y, scale, p * vv[s].y);
                accv[s].z = fmaf(accv[s].z, scale, p * vv[s].z); accv[s].w = fmaf(accv[s].w, scale, p * vv[s].w);
              }
#pragma unroll
              for (int t = 0; t < NT; ++t) {
                accp[h][t].x = fmaf(accp[h][t].x, scale, p * zt[t].x); accp[h][t].y = fmaf(accp[h][t].y, scale, p * zt[t].y);
                accp[h][t].z = fmaf(accp[h][t].z, scale, p * zt[t].z); accp[h][t].w = fmaf(accp[h][t].w, scale, p * zt[t].w);
              }
              if (sub == 0) Sc[(local * k + j) * H + h] = sc[h];
            }
          } else {
#pragma unroll
            for (int h = 0; h < H; ++h) {
              const float s_old = w[2 * h], a_old = w[2 * h + 1];
              const float e_old = __expf(s_old - mref[h]), e_new = __expf(sc[h] - mref[h]);
              const float Zn = lrun[h] - e_old + e_new;
              const float a_new = e_new / Zn;
              lrun[h] = Zn;
#pragma unroll
              for (int s = h * SH; s < (h + 1) * SH; ++s) {
                const float4 vo = *reinterpret_cast<const float4*>(vc + s * kSlot);
                accv[s].x += a_new * vv[s].x - a_old * vo.x; accv[s].y += a_new * vv[s].y - a_old * vo.y;
                accv[s].z += a_new * vv[s].z - a_old * vo.z; accv[s].w += a_new * vv[s].w - a_old * vo.w;
              }
              const float da = a_new - a_old;
#pragma unroll
              for (int t = 0; t < NT; ++t) {
                accp[h][t].x = fmaf(da, zt[t].x, accp[h][t].x); accp[h][t].y = fmaf(da, zt[t].y, accp[h][t].y);
                accp[h][t].z = fmaf(da, zt[t].z, accp[h][t].z); accp[h][t].w = fmaf(da, zt[t].w, accp[h][t].w);
              }
              if (sub == 0) { w[2 * h] = sc[h]; w[2 * h + 1] = a_new; }
            }
          }
#pragma unroll
          for (int s = 0; s < KS; ++s) *reinterpret_cast<float4*>(vc + s * kSlot) = vv[s];
        }
        };
        DBuf b0;
        fetch(0u, b0);
        pingpong_clamped<DBuf>(n_items, b0, fetch, work);
      }
      // ---- the row's sums: normalised by the denominator after an exact recomputation, as they stand after a delta update
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
      for (int h = 0; h < H; ++h) {
        const float inv = ex ? (lrun[h] > 0.0f ? 1.0f / lrun[h] : 0.0f) : 1.0f;
#pragma unroll
        for (int s = h * SH; s < (h + 1) * SH; ++s) {
          float4 o = accv[s];
          o.x *= inv; o.y *= inv; o.z *= inv; o.w *= inv;
          *reinterpret_cast<float4*>(Xs + local * ll.ldx + s * kSlot + 4u * sub) = o;
          if (live) *reinterpret_cast<float4*>(acS + s * kSlot) = o;
        }
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          float4 o = accp[h][t];
          o.x *= inv; o.y *= inv; o.z *= inv; o.w *= inv;
          clear_past_d_time(o, t);
          *reinterpret_cast<float4*>(Zs + local * ll.ldz + h * Ztp + t * kSlot + 4u * sub) = o;
          if (live) *reinterpret_cast<float4*>(acP + (h * NT + t) * kSlot) = o;
        }
        if (live && sub == 0) { acZM[2 * h] = lrun[h]; acZM[2 * h + 1] = mref[h]; }
        if (ex && live)
          for (uint32_t j = sub; j < cnt; j += 16) {          // the weights in effect after the exact recomputation
            const float sj = Sc[(local * k + j) * H + h];
            float* w = a.ac_W + ((size_t)nn * k + j) * (2 * H);
            w[2 * h] = sj;
            w[2 * h + 1] = lrun[h] > 0.0f ? __expf(sj - mref[h]) * inv : 0.0f;
          }
      }
      // ---- drift estimator (Sec. 3.5), final layer: an exact recomputation restarts the node's estimate, a
      // delta update adds the changed fraction of its entries to the decayed estimate
      // (the changes of the sum and of the member count are collected per wave and added once, at the end of
      // the launch: one update of the same word per row serialises -- 860 K of them took half of a launch)
      float dg = 0.0f;
      uint32_t dc = 0u;
      if (a.is_final && live && sub == 0 && !a.out_rows) {
        const uint32_t tau = a.drift->tau;
        const float old = a.dseen[nn] ? a.dsum[nn] * __powf(a.gamma, (float)(tau - a.dlast[nn])) : 0.0f;
        const float nw = ex ? 0.0f : old + (nvalid ? (float)nch / (float)nvalid : 0.0f);
        if (!a.dseen[nn]) { a.dseen[nn] = 1; dc = 1u; }
        a.dsum[nn] = nw; a.dlast[nn] = tau;
        dg = nw - old;
      }
      drift_sum += (double)__int_as_float(__builtin_amdgcn_readlane(__float_as_int(dg), 0)) +
                   (double)__int_as_float(__builtin_amdgcn_readlane(__float_as_int(dg), 16)) +
                   (double)__int_as_float(__builtin_amdgcn_readlane(__float_as_int(dg), 32)) +
                   (double)__int_as_float(__builtin_amdgcn_readlane(__float_as_int(dg), 48));
      drift_new += (uint32_t)__builtin_amdgcn_readlane((int)dc, 0) + (uint32_t)__builtin_amdgcn_readlane((int)dc, 16) +
                   (uint32_t)__builtin_amdgcn_readlane((int)dc, 32) + (uint32_t)__builtin_amdgcn_readlane((int)dc, 48);
    } else
    {
      float4 accv[KS], accp[H][NZ];
#pragma unroll
      for (int s = 0; s < KS; ++s) accv[s] = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
      for (int h = 0; h < H; ++h)
#pragma unroll
        for (int t = 0; t < NZ; ++t) accp[h][t] = make_float4(0.f, 0.f, 0.f, 0.f);
      float mref[H], lrun[H];
#pragma unroll
      for (int h = 0; h < H; ++h) { mref[h] = -INFINITY; lrun[h] = 0.0f; }
      // this lane's share of the row's q and qt vectors stays in registers for the whole phase
      float4 qk[KS];
#pragma unroll
      for (int s = 0; s < KS; ++s) qk[s] = *reinterpret_cast<const float4*>(Qs + local * ll.ldq + s * kSlot + 4u * sub);
      const float* zq = Zs + local * ll.ldz + 4u * sub;       // qt of head h, time slot t: + h Ztp + 64 t (read per chunk)
      auto attend = [&](uint32_t c, const ZBuf& zb) {
        // time encodings of the chunk's entries (computed for every lane, then masked: no branches)
        float4 zt[JC][NZ];
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
          const double dt = tq - rrow[j < k ? j : k - 1u].t;
          vj[jc] = j < cnt && dt <= a.window;          // inside the temporal window [tq - T_w, tq] (Sec. 3.3.2)
#pragma unroll
          for (int t = 0; t < NT; ++t) {
            const float c0 = cos_rev(om[t][0].x * dt + ph[t][0].x), c1 = cos_rev(om[t][0].y * dt + ph[t][0].y);
            const float c2 = cos_rev(om[t][1].x * dt + ph[t][1].x), c3 = cos_rev(om[t][1].y * dt + ph[t][1].y);
            // columns past d_time come out as cos(0) = 1 and need no mask: qt is exactly zero there (zero
            // weight columns), and what they add to pb meets zero weight rows in phase 4
            zt[jc][t] = make_float4(c0, c1, c2, c3);
          }
          if constexpr (ES) zt[jc][NT] = zb.e[jc][0];
        }
        // scores: q . (cached node keys + cached edge keys) + qt . phi  (raw edge rows: q . node keys + qt . z)
        float sc[JC][H];
#pragma unroll
        for (int h = 0; h < H; ++h) {
#pragma unroll
          for (int jc = 0; jc < JC; ++jc) {
            float p = 0.0f;
#pragma unroll
            for (int s = h * SH; s < (h + 1) * SH; ++s) {
              float4 kk = zb.n[jc][s];
              if constexpr (!ES) {
                kk.x += zb.e[jc][s].x; kk.y += zb.e[jc][s].y; kk.z += zb.e[jc][s].z; kk.w += zb.e[jc][s].w;
              }
              p = dot4(qk[s], kk, p);
            }
#pragma unroll
            for (int t = 0; t < NZ; ++t) p = dot4(*reinterpret_cast<const float4*>(zq + h * Ztp + t * kSlot), zt[jc][t], p);
            const float tsum = row16_sum(p);
            sc[jc][h] = vj[jc] ? tsum : -INFINITY;
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
            for (int s = h * SH; s < (h + 1) * SH; ++s) {
              accv[s].x *= scale; accv[s].y *= scale; accv[s].z *= scale; accv[s].w *= scale;
            }
#pragma unroll
            for (int t = 0; t < NZ; ++t) {
              accp[h][t].x *= scale; accp[h][t].y *= scale; accp[h][t].z *= scale; accp[h][t].w *= scale;
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
            for (int s = h * SH; s < (h + 1) * SH; ++s) {
              float4 vv = zb.n[jc][KS + s];
              if constexpr (!ES) {
                const float4 ve = zb.e[jc][KS + s];
                vv.x += ve.x; vv.y += ve.y; vv.z += ve.z; vv.w += ve.w;
              }
              accv[s].x = fmaf(p, vv.x, accv[s].x);
              accv[s].y = fmaf(p, vv.y, accv[s].y);
              accv[s].z = fmaf(p, vv.z, accv[s].z);
              accv[s].w = fmaf(p, vv.w, accv[s].w);
            }
#pragma unroll
            for (int t = 0; t < NZ; ++t) {
              const float4 zv = zt[jc][t];
              accp[h][t].x = fmaf(p, zv.x, accp[h][t].x);
              accp[h][t].y = fmaf(p, zv.y, accp[h][t].y);
              accp[h][t].z = fmaf(p, zv.z, accp[h][t].z);
              accp[h][t].w = fmaf(p, zv.w, accp[h][t].w);
            }
          }
        }
      };
      if (nchunk3) pingpong_clamped<ZBuf>(nchunk3, z0, gather, attend);
      // the cached-value part of the head outputs goes into the O tile (padded-head layout; the
      // padding lanes hold exact zeros), pb overwrites qt (each lane owns its float4s)
#pragma unroll
      for (int h = 0; h < H; ++h) {
        const float inv = lrun[h] > 0.0f ? 1.0f / lrun[h] : 0.0f;    // no entry, or none inside the window: b_O alone
#pragma unroll
        for (int s = h * SH; s < (h + 1) * SH; ++s) {
          float4 o = accv[s];
          o.x *= inv; o.y *= inv; o.z *= inv; o.w *= inv;
          *reinterpret_cast<float4*>(Xs + local * ll.ldx + s * kSlot + 4u * sub) = o;
        }
#pragma unroll
        for (int t = 0; t < NZ; ++t) {
          float4 o = accp[h][t];
          o.x *= inv; o.y *= inv; o.z *= inv; o.w *= inv;
          if (t < NT) clear_past_d_time(o, t);                 // (a raw edge row's padding is zero, and so are its sums)
          *reinterpret_cast<float4*>(Zs + local * ll.ldz + h * Ztp + t * kSlot + 4u * sub) = o;
        }
      }
    }
    // ================================================================ phase 4: o_h += pb_h W_V,h[time | raw edge]
    {
      // K runs over the slots of z, one chunk per slot; the operands of the next slot are in flight
      // during the current one.  The weights of the first slot are requested ahead of the barrier.
      Ops16<2> ov[2];
      uint32_t x = wave;
      auto wv = [&](uint32_t h, uint32_t nt) { return a.WV + (size_t)(h * ntk + nt) * g_zt * kGrpFloats; };
      uint32_t h4 = 0, n0 = 0, n1 = 0;
      bool two4 = false;
      auto decode4 = [&](uint32_t xx) {
        h4 = xx / np4;
        n0 = 2u * (xx - h4 * np4);
        two4 = n0 + 1u < ntk;
        n1 = two4 ? n0 + 1u : n0;
      };
      decode4(x < nunits4 ? x : nunits4 - 1u);
      // every weight chunk of the wave's first unit is requested ahead of the barrier: one memory latency
      // for the unit, most of it spent waiting for the slowest wave of phase 3 anyway
      Upfront16<2, NZ> u4;
      {
        const float* const B4[2] = {wv(h4, n0), wv(h4, n1)};
        u4.request(B4, NZ);
      }
      __syncthreads();
      if constexpr (KS > 2) { if (pf_ok) stage_b(); else stage_none(); }
      for (; x < nunits4; x += 4) {
        floatx4 acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
        if (x == wave) {
          u4.multiply(Zs + h4 * Ztp + a_z, NZ, acc);
        } else {
          decode4(x);
          load_b16(wv(h4, n0), 0, ov[0].b[0]);
          load_b16(wv(h4, n1), 0, ov[0].b[1]);
          const float* Ap = Zs + h4 * Ztp + a_z;
          const float* B0 = wv(h4, n0);
          const float* B1 = wv(h4, n1);
          load_a16(Ap, 0, ov[0].a);
#pragma unroll
          for (int c = 0; c < NZ; ++c) {
            if (c + 1 < NZ) {
              load_a16(Ap, (c + 1) * kCG, ov[(c + 1) & 1].a);
              load_b16(B0, (c + 1) * kCG, ov[(c + 1) & 1].b[0]);
              load_b16(B1, (c + 1) * kCG, ov[(c + 1) & 1].b[1]);
            }
            __builtin_amdgcn_sched_barrier(0);      // requests stay ahead of the products they overlap
            mfma16_chunk<2>(ov[c & 1], acc);
            __builtin_amdgcn_sched_barrier(0);
          }
        }
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          const uint32_t col = (t ? n1 : n0) * 16 + m16_col(lane);
          if ((t == 0 || two4) && col < dk) {
            float* op = Xs + c_off_x - m16_col(lane) + h4 * (SH * kSlot) + col;    // one lane per (row, column)
#pragma unroll
            for (int r = 0; r < 4; ++r) op[r * ll.ldx] += acc[t][r];
          }
        }
      }
    }
    // ================================================================ phase 5: h' = o W_O + b_O
    {
      Ops16<2> oo;
      constexpr int U5 = KS <= 2 ? KS : 1;                    // weight chunks of the first unit requested up front
      Upfront16<2, U5> u5;
      {
        const float* const B5[2] = {a.WO + (size_t)w1 * g_o * kGrpFloats, a.WO + (size_t)(w1 + 4 < ntd ? w1 + 4 : w1) * g_o * kGrpFloats};
        if constexpr (KS <= 2) u5.request(B5, KS);
        else { load_b16(B5[0], 0, oo.b[0]); load_b16(B5[1], 0, oo.b[1]); }
      }
      __syncthreads();
      for (uint32_t nt = wave; nt < ntd; nt += 8) {
        const bool two = nt + 4 < ntd;
        const float* const Bt[2] = {a.WO + (size_t)nt * g_o * kGrpFloats, a.WO + (size_t)(two ? nt + 4 : nt) * g_o * kGrpFloats};
        floatx4 acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
        if (KS <= 2 && nt == wave) {
          u5.multiply(Xs + a_x, KS, acc);
        } else {
          if (nt != wave) { load_b16(Bt[0], 0, oo.b[0]); load_b16(Bt[1], 0, oo.b[1]); }
          mfma16_gemm_pre<2>(Xs + a_x, KS, Bt, acc, oo);
        }
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          const uint32_t col = (nt + 4 * t) * 16 + m16_col(lane);
          if ((t == 0 || two) && col < a.d_emb) {
            const float b = nt == wave ? bo_r[t] : a.bO[col];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              const uint32_t node = s_node[m16_row(lane, r)];
              const float v = acc[t][r] + b;
              if (a.out_rows) {
                const uint32_t lr = tile * kTM + m16_row(lane, r);
                if (lr < n) a.out_rows[(size_t)lr * a.d_emb + col] = v;
              } else if (node != 0xFFFFFFFFu) {
                a.Hout[(size_t)node * a.ld_out + col] = v;
              }
              Qs[c_off_q - m16_col(lane) + r * ll.ldq + col] = v;     // operand of phase 6 (q is no longer needed)
            }
          }
        }
      }
    }
    // ================================================================ phase 6: next layer's cached keys | values of these rows
    if (a.KVout) {
      constexpr uint32_t ntkv = 8u * KS;                      // column tiles of a cached row; a wave takes tiles w + 8 i, w + 8 i + 4
      Ops16<2> ok;
      load_b16(a.WKVnext + (size_t)wave * g_de * kGrpFloats, 0, ok.b[0]);
      load_b16(a.WKVnext + (size_t)(wave + 4) * g_de * kGrpFloats, 0, ok.b[1]);
      __syncthreads();
      for (uint32_t nt = wave; nt < ntkv; nt += 8) {
        const float* const Bt[2] = {a.WKVnext + (size_t)nt * g_de * kGrpFloats, a.WKVnext + (size_t)(nt + 4) * g_de * kGrpFloats};
        floatx4 acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
        if (nt != wave) { load_b16(Bt[0], 0, ok.b[0]); load_b16(Bt[1], 0, ok.b[1]); }
        mfma16_gemm_pre<2>(Qs + a_q, c_de, Bt, acc, ok);
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          const uint32_t col = (nt + 4 * t) * 16 + m16_col(lane);   // every column is written: padding columns get exact zeros
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const uint32_t node = s_node[m16_row(lane, r)];
            if (node != 0xFFFFFFFFu) a.KVout[(size_t)node * a.ld_kv + col] = acc[t][r];
          }
        }
      }
    }
    __syncthreads();
  }
  if constexpr (DELTA) {
    if (lane == 0 && a.is_final && !a.out_rows) {
      if (drift_sum != 0.0) atomicAdd(&a.drift->G, drift_sum);
      if (drift_new) atomicAdd(&a.drift->count, drift_new);
    }
  }
  // statistics: the workgroup's count goes into the slot of its index with a plain update (launches
  // on one stream follow each other, and no other workgroup of a launch has this index); thousands of
  // same-address atomic updates at the end of a launch were measured to cost a third of its duration
  const uint32_t gsum = (uint32_t)__builtin_amdgcn_readlane((int)gathered, 0) +
                        (uint32_t)__builtin_amdgcn_readlane((int)gathered, 16) +
                        (uint32_t)__builtin_amdgcn_readlane((int)gathered, 32) +
                        (uint32_t)__builtin_amdgcn_readlane((int)gathered, 48);
  if (!a.out_rows) {
    if (lane == 0) s_cnt[wave] = gsum;
    __syncthreads();
    if (threadIdx.x == 0) {
      const uint32_t tot = s_cnt[0] + s_cnt[1] + s_cnt[2] + s_cnt[3];
      if (tot) a.gathered_slots[blockIdx.x] += tot;
      if (blockIdx.x == 0 && n) a.ctrl->tot_rows += n;
    }
  }
}

// ---- dispatch over (heads, key slots, time slots)
struct LaunchArgs {
  LayerArgs k;
  hipStream_t s; const uint32_t* rows; const uint32_t* cp; uint32_t cm;
  uint32_t ks, nt, heads;
  bool es;                          // raw edge rows (never together with delta)
  bool delta;                       // the delta-mode variant of the kernel
  uint32_t num_cu;                  // compute units of the device
  bool set_attr; size_t lds; hipError_t err;
  int query_wgs; uint32_t wgs;      // query_wgs: only report the workgroups per CU of the variant in `wgs`
};

template <int KS, int NT, int ES, int H, int JC, int WGS, bool DELTA, bool QCACHE>
void go_k(LaunchArgs& a) {
  auto kern = layer_kernel<KS, NT, ES, H, JC, WGS, DELTA, QCACHE>;
  if (a.query_wgs) { a.wgs = WGS; return; }
  if (a.set_attr) {
    // never lowered: other layers of this context and other contexts of the process may launch the same variant
    static std::mutex mu;
    static size_t granted = 0;
    std::lock_guard<std::mutex> lock(mu);
    a.err = hipSuccess;
    if (a.lds > granted) {
      a.err = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)a.lds);
      if (a.err == hipSuccess) granted = a.lds;
    }
    return;
  }
  uint64_t blocks = ((uint64_t)a.cm + kTM - 1) / kTM;
  uint64_t cap = (uint64_t)WGS * (a.num_cu ? a.num_cu : 256u);         // persistent: each workgroup strides over the tiles,
  if (cap > kStatSlots) cap = kStatSlots;                              // staging one tile ahead
  if (blocks > cap) blocks = cap;
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(kern, dim3((uint32_t)blocks), dim3(256), a.lds, a.s, a.k, a.rows, a.cp, a.cm);
}

template <int KS, int NT, int H, int JC, int WGS>
void go(LaunchArgs& a) {
  if (a.delta) { go_k<KS, NT, 0, H, 1, WGS, true, false>(a); return; }
  if (a.es) {
    if (a.k.QC) go_k<KS, NT, 1, H, JC, WGS, false, true>(a); else go_k<KS, NT, 1, H, JC, WGS, false, false>(a);
    return;
  }
  if (a.k.QC) { go_k<KS, NT, 0, H, JC, WGS, false, true>(a); return; }
  go_k<KS, NT, 0, H, JC, WGS, false, false>(a);
}

// Ring entries per chunk and workgroups per CU are bounded by registers: two chunks of JC * 4 KS
// float4 per lane are in flight beside 2 (KS + H NT) float4 of accumulators and query values.
template <int KS, int NT, int H>
void go_jc(LaunchArgs& a) {
  if constexpr (KS == 1) go<KS, NT, H, 2, 3>(a);
  else if constexpr (KS == 2) go<KS, NT, H, 1, 2>(a);
  else go<KS, NT, H, 1, 2>(a);
}

template <int H>
void go_h(LaunchArgs& a) {
  const uint32_t sh = a.ks / H;
  if (a.nt == 1) {
    if (sh == 1) go_jc<H, 1, H>(a);
    else if constexpr (H <= 2) { if (sh == 2) go_jc<2 * H, 1, H>(a); else if constexpr (H == 1) go_jc<4, 1, 1>(a); }
  } else {
    if (sh == 1) go_jc<H, 2, H>(a);
    else if constexpr (H <= 2) { if (sh == 2) go_jc<2 * H, 2, H>(a); else if constexpr (H == 1) go_jc<4, 2, 1>(a); }
  }
}

}  // namespace layer_impl

// one translation unit per head count instantiates this (keeps the build parallel)
template <int H>
void layer_entry(layer_impl::LaunchArgs& a) { layer_impl::go_h<H>(a); }

}  // namespace stgn
