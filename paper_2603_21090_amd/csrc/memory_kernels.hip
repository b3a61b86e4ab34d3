// Message + "Last" aggregation + GRU memory update on the distinct endpoints of a batch
// (paper Eq. msg_linear, Eq. agg_functions "Last", Eq. gru_detail; Sec. 3.6.2: every read sees the
// pre-batch state and each node makes one transition per batch).  One workgroup of eight waves
// handles 16 rows: the message input rows are gathered into LDS (two memory rows, the edge-feature
// row of the node's last edge in the batch, the time encoding of t_edge - t_last), then three
// chained stages of 16x16x4 matrix-core products run without leaving the CU, each wave owning one
// 16-column tile of the stage's output.  A batch has few rows (at most two per edge), so the work is
// spread over columns rather than rows.  New rows go to a scratch table; the apply kernel commits
// them once every read of the old rows is done.
#include "stgn_internal.h"
#include "mfma16.h"
#include "placement.h"

namespace stgn {

namespace {

constexpr uint32_t kRows = 16;
constexpr uint32_t kThreads = 512;
constexpr uint32_t kWaves = kThreads / 64;

__device__ inline float sigmoidf_(float x) { return 1.0f / (1.0f + expf(-x)); }

__device__ inline float cos_rev64(double x) {
  const double f = __builtin_amdgcn_fract(x);
  return __builtin_amdgcn_cosf((float)f);
}

struct MemLds {
  uint32_t ldx, ldm, ldr;      // strides of the input, message and (z | r.s) tiles, all 4 (mod 8)
  uint32_t off_m, off_z, off_r, total;
};

__host__ __device__ inline MemLds memory_lds_layout(uint32_t Kmsg, uint32_t d_msg, uint32_t d_mem) {
  MemLds l;
  l.ldx = round_up(Kmsg, kGrpK) + 4;
  l.ldm = round_up(d_msg, kGrpK) + 4;
  l.ldr = round_up(d_mem, kGrpK) + 4;
  l.off_m = kRows * l.ldx;
  l.off_z = l.off_m + kRows * l.ldm;
  l.off_r = l.off_z + kRows * l.ldr;
  l.total = l.off_r + kRows * l.ldr + 4 * kGrpK;      // operand reads may run one chunk past the last row
  return l;
}

template <bool UP>
__global__ __launch_bounds__(kThreads) void memory_update_kernel(Dev d, const uint32_t* __restrict__ src,
                                                                 const uint32_t* __restrict__ dst,
                                                                 const double* __restrict__ ts,
                                                                 const float* __restrict__ ef, uint32_t with_place) {
  extern __shared__ __align__(16) float lds[];
  __shared__ uint32_t s_self[kRows], s_oth[kRows], s_ef[kRows], s_live[kRows];
  __shared__ double s_dt[kRows];
  // Mean / Sum aggregation: the row's slots in sorted order [s_seg, s_seg + s_n), its last-interaction time,
  // and the factor of the aggregated message (the slot count for Sum, 1 otherwise)
  __shared__ uint32_t s_seg[kRows], s_n[kRows];
  __shared__ double s_tl[kRows];
  __shared__ float s_scale[kRows];
  // The last workgroup places the batch's endpoint slots in the adjacency logs instead (placement.h):
  // that step depends on the same staging kernel and the same apply step as the memory update and on
  // nothing in it, and riding along saves its launch.
  __shared__ uint32_t s_place[17];
  if (with_place && blockIdx.x == gridDim.x - 1) {
    place_batch(d, s_place, s_place + 16);
    return;
  }
  const uint32_t nblk = gridDim.x - (with_place ? 1u : 0u);     // workgroups that update memory rows
  const BatchCtl* c = d.bc;
  if (c->skip) return;
  const uint32_t nD = c->nD;
  const uint32_t ntiles = (nD + kRows - 1) / kRows;
  const uint32_t dm = d.d_mem, dg = d.d_msg, de = d.d_edge, Kmsg = d.Kmsg;
  const MemLds ll = memory_lds_layout(Kmsg, dg, dm);
  float* Xs = lds;                       // [16 x Kmsg]  message input rows; first dm columns = s
  float* Ms = lds + ll.off_m;            // [16 x dg]    messages
  float* Zs = lds + ll.off_z;            // [16 x dm]    update gate
  float* Rs = lds + ll.off_r;            // [16 x dm]    r . s
  const uint32_t lane = threadIdx.x & 63u;
  // wave index, made provably uniform so that tile indices and weight addresses stay in scalar registers
  const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const uint32_t c_x = chunks_of(Kmsg), c_g = chunks_of(dg), c_m = chunks_of(dm);
  const uint32_t ntg = round_up(dg, 16) >> 4, ntm = round_up(dm, 16) >> 4;
  const uint32_t a_x = a16_lane_off(ll.ldx), a_m = a16_lane_off(ll.ldm), a_r = a16_lane_off(ll.ldr);
  const uint32_t row0 = m16_row(lane, 0), colL = m16_col(lane);
  const Table H0 = d.H[0];
  // operand padding (columns nobody writes) must be finite: clear the tiles once
  for (uint32_t x = threadIdx.x; x < ll.total; x += kThreads) lds[x] = 0.0f;

  for (uint32_t tile = blockIdx.x; tile < ntiles; tile += nblk) {
    const uint32_t r0 = tile * kRows;
    Upfront16<1, 8> um;      // message weights: requested before anything else of the tile
    if constexpr (UP) {
      const float* const B0[1] = {d.Wmsg + (size_t)(wave < ntg ? wave : 0u) * kCG * c_x * kGrpFloats};
      um.request(B0, c_x);
    }
    // per-row metadata first (one thread per row: node, partner, edge, time gap), through LDS
    if (threadIdx.x < kRows) {
      const uint32_t r = threadIdx.x;
      uint32_t so = 0, oo = 0, eo = 0, live = 0, seg = 0, cnt = 0;
      double dtv = 0.0, tl = 0.0;
      if (r0 + r < nD) {
        const uint32_t node = d.D[r0 + r];
        seg = d.seg_start[r0 + r]; cnt = d.seg_start[r0 + r + 1] - seg;
        tl = d.t_last[node];
        const uint32_t slot = d.last_slot[r0 + r];
        const uint32_t i = slot >> 1;
        const uint32_t other = (slot & 1) ? src[i] : dst[i];
        so = node; oo = other; eo = i * de; live = 1;          // node ids: row offsets are formed in 64 bits at the use
        dtv = ts[i] - d.t_last[node];
      }
      s_self[r] = so; s_oth[r] = oo; s_ef[r] = eo; s_live[r] = live; s_dt[r] = dtv;
      s_seg[r] = seg; s_n[r] = cnt; s_tl[r] = tl;
      s_scale[r] = d.aggregator == 2u ? (float)cnt : 1.0f;
    }
    __syncthreads();
    if (!UP && d.aggregator != 0u) {       // (the all-weights-up-front variant is only launched for Last)
      // Mean / Sum (Eq. agg_functions).  The message is linear in its input, so the node's inputs are
      // averaged instead of its messages (added in slot order = batch order, a fixed order): the mean
      // message is mean(x) W_msg + b_msg and the sum is the slot count times that.  The node's own
      // memory is the same in every one of its inputs and is staged as it is.
      const uint32_t total = kRows * Kmsg;
      for (uint32_t x = threadIdx.x; x < total; x += kThreads) {
        const uint32_t r = x / Kmsg, col = x - r * Kmsg;
        float val = 0.0f;
        if (s_live[r]) {
          if (col < dm) {
            val = H0.base[(size_t)s_self[r] * H0.ld + col];
          } else {
            const uint32_t n = s_n[r];
            float acc = 0.0f;
            for (uint32_t j = 0; j < n; ++j) {
              const uint32_t slot = d.slot_sorted[s_seg[r] + j], i = slot >> 1;
              if (col < 2 * dm) {
                const uint32_t other = (slot & 1) ? src[i] : dst[i];
                acc += H0.base[(size_t)other * H0.ld + (col - dm)];
              } else if (col < 2 * dm + de) {
                acc += ef[(size_t)i * de + (col - 2 * dm)];
              } else {
                const uint32_t q = col - 2 * dm - de;
                acc += cos_rev64(d.om_rev[q] * (ts[i] - s_tl[r]) + d.ph_rev[q]);
              }
            }
            val = acc / (float)n;
          }
        }
        Xs[r * ll.ldx + col] = val;
      }
    } else
    // then every thread issues its loads in batches of sixteen, unconditionally (dead elements read a
    // valid dummy address and are zeroed afterwards), so the latencies overlap
    {
      const uint32_t total = kRows * Kmsg;
      const float* efp = ef ? ef : H0.base;
      constexpr int kInFlight = UP ? 8 : 16;
      for (uint32_t x0 = threadIdx.x; x0 < total; x0 += kThreads * kInFlight) {
        float v[kInFlight];
        uint32_t rr[kInFlight], cc[kInFlight];
        bool ok[kInFlight];
#pragma unroll
        for (int e = 0; e < kInFlight; ++e) {
          uint32_t x = x0 + kThreads * e;
          ok[e] = x < total;
          x = ok[e] ? x : 0u;
          const uint32_t r = x / Kmsg, col = x - r * Kmsg;
          rr[e] = r; cc[e] = col;
          const float* p = H0.base;
          if (col < dm) p = H0.base + (size_t)s_self[r] * H0.ld + col;
          else if (col < 2 * dm) p = H0.base + (size_t)s_oth[r] * H0.ld + (col - dm);
          else if (col < 2 * dm + de) p = efp + s_ef[r] + (col - 2 * dm);
          v[e] = *p;
        }
#pragma unroll
        for (int e = 0; e < kInFlight; ++e) {
          const uint32_t r = rr[e], col = cc[e];
          float val = v[e];
          if (col >= 2 * dm + de) {
            const uint32_t q = col - 2 * dm - de;
            val = cos_rev64(d.om_rev[q] * s_dt[r] + d.ph_rev[q]);
          }
          if (!s_live[r]) val = 0.0f;
          if (ok[e]) Xs[r * ll.ldx + col] = val;
        }
      }
    }
    // A workgroup of this kernel has a CU to itself and nothing to overlap a memory latency with, so
    // each stage requests ALL its weights at once, ahead of the barrier that completes its input
    // (kernel variant UP, for short products only: up to 8 chunks of K for the message, 2 for the gates,
    // one column tile per wave; other shapes run the chunk-by-chunk pipeline).
    constexpr bool up_ok = UP;
    const uint32_t wt = wave < ntm ? wave : 0u;
    // ---- m = x W_msg + b_msg
    {
      __syncthreads();
      for (uint32_t nt = wave, it = 0; nt < ntg && !(UP && it); nt += kWaves, ++it) {
        const float* const Bt[1] = {d.Wmsg + (size_t)nt * kCG * c_x * kGrpFloats};
        floatx4 acc[1] = {{0.f, 0.f, 0.f, 0.f}};
        if constexpr (up_ok) {
          um.multiply(Xs + a_x, c_x, acc);
        } else {
          mfma16_gemm<1>(Xs + a_x, c_x, Bt, acc);
        }
        const uint32_t col = nt * 16 + colL;
        if (col < dg) {
          const float b = d.bmsg[col];
#pragma unroll
          for (int r = 0; r < 4; ++r) Ms[(row0 + r) * ll.ldm + col] = (acc[0][r] + b) * s_scale[row0 + r];
        }
      }
    }
    // ---- z = sigma(m W_z + s U_z + b_z), r = sigma(m W_r + s U_r + b_r): one wave, one column tile of both
    {
      Upfront16<2, 2> uw, uu;
      {
        const float* const Bw[2] = {d.Wzr + (size_t)wt * kCG * c_g * kGrpFloats, d.Wzr + (size_t)(ntm + wt) * kCG * c_g * kGrpFloats};
        const float* const Bu[2] = {d.Uzr + (size_t)wt * kCG * c_m * kGrpFloats, d.Uzr + (size_t)(ntm + wt) * kCG * c_m * kGrpFloats};
        if constexpr (up_ok) { uw.request(Bw, c_g); uu.request(Bu, c_m); }
      }
      __syncthreads();
      for (uint32_t nt = wave, it = 0; nt < ntm && !(UP && it); nt += kWaves, ++it) {
        const float* const Bw[2] = {d.Wzr + (size_t)nt * kCG * c_g * kGrpFloats, d.Wzr + (size_t)(ntm + nt) * kCG * c_g * kGrpFloats};
        const float* const Bu[2] = {d.Uzr + (size_t)nt * kCG * c_m * kGrpFloats, d.Uzr + (size_t)(ntm + nt) * kCG * c_m * kGrpFloats};
        floatx4 acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
        if constexpr (up_ok) {
          uw.multiply(Ms + a_m, c_g, acc);
          uu.multiply(Xs + a_x, c_m, acc);
        } else {
          mfma16_gemm<2>(Ms + a_m, c_g, Bw, acc);
          mfma16_gemm<2>(Xs + a_x, c_m, Bu, acc);
        }
        const uint32_t col = nt * 16 + colL;
        if (col < dm) {
          const float bz = d.bz[col], br = d.br[col];
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const uint32_t row = row0 + r;
            Zs[row * ll.ldr + col] = sigmoidf_(acc[0][r] + bz);
            Rs[row * ll.ldr + col] = sigmoidf_(acc[1][r] + br) * Xs[row * ll.ldx + col];
          }
        }
      }
    }
    // ---- candidate = tanh(m W_h + (r . s) U_h + b_h);  s' = (1 - z) candidate + z s
    {
      Upfront16<1, 2> uw, uu;
      {
        const float* const Bw[1] = {d.Wh + (size_t)wt * kCG * c_g * kGrpFloats};
        const float* const Bu[1] = {d.Uh + (size_t)wt * kCG * c_m * kGrpFloats};
        if constexpr (up_ok) { uw.request(Bw, c_g); uu.request(Bu, c_m); }
      }
      __syncthreads();
      for (uint32_t nt = wave, it = 0; nt < ntm && !(UP && it); nt += kWaves, ++it) {
        const float* const Bw[1] = {d.Wh + (size_t)nt * kCG * c_g * kGrpFloats};
        const float* const Bu[1] = {d.Uh + (size_t)nt * kCG * c_m * kGrpFloats};
        floatx4 acc[1] = {{0.f, 0.f, 0.f, 0.f}};
        if constexpr (up_ok) {
          uw.multiply(Ms + a_m, c_g, acc);
          uu.multiply(Rs + a_r, c_m, acc);
        } else {
          mfma16_gemm<1>(Ms + a_m, c_g, Bw, acc);
          mfma16_gemm<1>(Rs + a_r, c_m, Bu, acc);
        }
        const uint32_t col = nt * 16 + colL;
        if (col < dm) {
          const float b = d.bh[col];
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const uint32_t row = row0 + r;
            if (r0 + row < nD) {
              const float cand = tanhf(acc[0][r] + b);
              const float z = Zs[row * ll.ldr + col], s = Xs[row * ll.ldx + col];
              d.mem_new[(size_t)(r0 + row) * dm + col] = (1.0f - z) * cand + z * s;
            }
          }
        }
      }
    }
    __syncthreads();
  }
}

// shapes the all-weights-up-front variant covers: every stage one column tile per wave, the products
// short enough for their whole B operand to sit in registers
bool memory_upfront(const Dev& d) {
  return d.aggregator == 0u && chunks_of(d.Kmsg) <= 8u && chunks_of(d.d_msg) <= 2u && chunks_of(d.d_mem) <= 2u &&
         round_up(d.d_msg, 16) / 16 <= kWaves && round_up(d.d_mem, 16) / 16 <= kWaves;
}

size_t memory_lds(const Dev& d) { return (size_t)memory_lds_layout(d.Kmsg, d.d_msg, d.d_mem).total * sizeof(float); }

}  // namespace

void launch_memory_update(const Dev& d, hipStream_t s, const uint32_t* src, const uint32_t* dst, const double* ts,
                          const float* ef, bool with_place, hipEvent_t done) {
  uint32_t blocks = (2 * d.max_batch + kRows - 1) / kRows;
  if (blocks > 1024) blocks = 1024;
  const uint32_t wp = with_place ? 1u : 0u;
  blocks += wp;
  if (memory_upfront(d))
    launch_done(memory_update_kernel<true>, dim3(blocks), dim3(kThreads), memory_lds(d), s, done, d, src, dst, ts, ef, wp);
  else
    launch_done(memory_update_kernel<false>, dim3(blocks), dim3(kThreads), memory_lds(d), s, done, d, src, dst, ts, ef, wp);
}

int setup_memory_attributes(const Dev& d) {
  if (d.d_mem == 0) return 0;
  const size_t need = memory_lds(d);
  if (need + 1024 > kMaxLds) return -1;
  const void* f = memory_upfront(d) ? (const void*)memory_update_kernel<true> : (const void*)memory_update_kernel<false>;
  return hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, (int)need) == hipSuccess ? 0 : -1;
}

}  // namespace stgn
