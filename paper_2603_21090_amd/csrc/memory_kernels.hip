// Message + "Last" aggregation + GRU memory update on the distinct endpoints of a batch
// (paper Eq. msg_linear, Eq. agg_functions "Last", Eq. gru_detail; Sec. 3.6.2: every read sees the
// pre-batch state and each node makes one transition per batch).  One workgroup handles 32 rows:
// the message input rows are gathered into LDS (two memory rows, the edge-feature row of the
// node's last edge in the batch, the time encoding of t_edge - t_last), then four chained
// matrix-core products run without leaving the CU.  New rows go to a scratch table; the apply
// kernel commits them once every read of the old rows is done.
#include "stgn_internal.h"
#include "mfma_gemm.h"

namespace stgn {

namespace {

constexpr uint32_t kRows = 32;

__device__ inline float sigmoidf_(float x) { return 1.0f / (1.0f + expf(-x)); }

__device__ inline float cos_rev64(double x) {
  const double f = __builtin_amdgcn_fract(x);
  return __builtin_amdgcn_cosf((float)f);
}

__global__ __launch_bounds__(256) void memory_update_kernel(Dev d, const uint32_t* __restrict__ src,
                                                            const uint32_t* __restrict__ dst,
                                                            const double* __restrict__ ts,
                                                            const float* __restrict__ ef) {
  extern __shared__ float lds[];
  __shared__ uint32_t s_self[kRows], s_oth[kRows], s_ef[kRows], s_live[kRows];
  __shared__ double s_dt[kRows];
  const Ctrl* c = d.ctrl;
  if (c->skip) return;
  const uint32_t nD = c->nD;
  const uint32_t ntiles = (nD + kRows - 1) / kRows;
  const uint32_t dm = d.d_mem, dg = d.d_msg, de = d.d_edge;
  const uint32_t dm2 = round_up(dm, 2), dg2 = round_up(dg, 2);
  const uint32_t ldx = d.Kmsg2 + 1, ldm = dg2 + 1, ldg = dm2 + 1;
  float* Xs = lds;                       // [32 x Kmsg2]  message input rows; first dm columns = s
  float* Ms = Xs + kRows * ldx;          // [32 x dg2]    messages
  float* Zg = Ms + kRows * ldm;          // [32 x dm2]    update gate
  float* Rs = Zg + kRows * ldg;          // [32 x dm2]    r . s
  const uint32_t npg = round_up(dg, 32), npm = round_up(dm, 32);
  const uint32_t lane = threadIdx.x & 63u;
  // wave index, made provably uniform so that tile indices and weight addresses stay in scalar registers
  const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const Table H0 = d.H[0];

  for (uint32_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
    const uint32_t r0 = tile * kRows;
    // per-row metadata first (one thread per row: node, partner, edge, time gap), through LDS
    if (threadIdx.x < kRows) {
      const uint32_t r = threadIdx.x;
      uint32_t so = 0, oo = 0, eo = 0, live = 0;
      double dtv = 0.0;
      if (r0 + r < nD) {
        const uint32_t node = d.D[r0 + r];
        const uint32_t slot = d.last_slot[r0 + r];
        const uint32_t i = slot >> 1;
        const uint32_t other = (slot & 1) ? src[i] : dst[i];
        so = node * H0.ld; oo = other * H0.ld; eo = i * de; live = 1;
        dtv = ts[i] - d.t_last[node];
      }
      s_self[r] = so; s_oth[r] = oo; s_ef[r] = eo; s_live[r] = live; s_dt[r] = dtv;
    }
    __syncthreads();
    // then every thread issues its loads in batches of four, unconditionally (dead elements read a
    // valid dummy address and are zeroed afterwards), so the latencies overlap
    {
      const uint32_t total = kRows * d.Kmsg2;
      const float* efp = ef ? ef : H0.base;
      for (uint32_t x0 = threadIdx.x; x0 < total; x0 += 256u * 4u) {
        float v[4];
        uint32_t rr[4], cc[4];
        bool ok[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          uint32_t x = x0 + 256u * e;
          ok[e] = x < total;
          x = ok[e] ? x : 0u;
          const uint32_t r = x / d.Kmsg2, col = x - r * d.Kmsg2;
          rr[e] = r; cc[e] = col;
          const float* p = H0.base;
          if (col < dm) p = H0.base + s_self[r] + col;
          else if (col < 2 * dm) p = H0.base + s_oth[r] + (col - dm);
          else if (col < 2 * dm + de) p = efp + s_ef[r] + (col - 2 * dm);
          v[e] = *p;
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const uint32_t r = rr[e], col = cc[e];
          float val = v[e];
          if (col >= 2 * dm + de && col < d.Kmsg) {
            const uint32_t q = col - 2 * dm - de;
            val = cos_rev64(d.om_rev[q] * s_dt[r] + d.ph_rev[q]);
          }
          if (!s_live[r] || col >= d.Kmsg) val = 0.0f;
          if (ok[e]) Xs[r * ldx + col] = val;
        }
      }
    }
    for (uint32_t x = threadIdx.x; x < kRows; x += 256) {
      Ms[x * ldm + dg2 - 1] = 0.0f;
      Rs[x * ldg + dm2 - 1] = 0.0f;
    }
    __syncthreads();
    // m = x W_msg + b_msg
    for (uint32_t nt = wave; nt < npg / 32; nt += 4) {
      floatx16 acc[1];
      zero_acc(acc);
      mfma_tile<1>(Xs, ldx, d.Kmsg2, d.Wmsg, npg, nt * 32, acc);
      const uint32_t col = nt * 32 + mfma_col(lane);
      if (col < dg) {
        const float b = d.bmsg[col];
#pragma unroll
        for (int j = 0; j < 16; ++j) Ms[mfma_row(lane, j) * ldm + col] = acc[0][j] + b;
      }
    }
    __syncthreads();
    // z = sigma(m W_z + s U_z + b_z) | r = sigma(m W_r + s U_r + b_r)
    for (uint32_t nt = wave; nt < 2 * npm / 32; nt += 4) {
      floatx16 acc[1];
      zero_acc(acc);
      mfma_tile<1>(Ms, ldm, dg2, d.Wzr, 2 * npm, nt * 32, acc);
      mfma_tile<1>(Xs, ldx, dm2, d.Uzr, 2 * npm, nt * 32, acc);
      const uint32_t gcol = nt * 32 + mfma_col(lane);
      if (gcol < npm) {
        if (gcol < dm) {
          const float b = d.bz[gcol];
#pragma unroll
          for (int j = 0; j < 16; ++j) Zg[mfma_row(lane, j) * ldg + gcol] = sigmoidf_(acc[0][j] + b);
        }
      } else {
        const uint32_t col = gcol - npm;
        if (col < dm) {
          const float b = d.br[col];
#pragma unroll
          for (int j = 0; j < 16; ++j) {
            const uint32_t r = mfma_row(lane, j);
            Rs[r * ldg + col] = sigmoidf_(acc[0][j] + b) * Xs[r * ldx + col];
          }
        }
      }
    }
    __syncthreads();
    // candidate = tanh(m W_h + (r . s) U_h + b_h);  s' = (1 - z) candidate + z s
    for (uint32_t nt = wave; nt < npm / 32; nt += 4) {
      floatx16 acc[1];
      zero_acc(acc);
      mfma_tile<1>(Ms, ldm, dg2, d.Wh, npm, nt * 32, acc);
      mfma_tile<1>(Rs, ldg, dm2, d.Uh, npm, nt * 32, acc);
      const uint32_t col = nt * 32 + mfma_col(lane);
      if (col < dm) {
        const float b = d.bh[col];
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          const uint32_t r = mfma_row(lane, j);
          if (r0 + r < nD) {
            const float cand = tanhf(acc[0][j] + b);
            const float z = Zg[r * ldg + col], s = Xs[r * ldx + col];
            d.mem_new[(size_t)(r0 + r) * dm + col] = (1.0f - z) * cand + z * s;
          }
        }
      }
    }
    __syncthreads();
  }
}

size_t memory_lds(const Dev& d) {
  const uint32_t dm2 = round_up(d.d_mem, 2), dg2 = round_up(d.d_msg, 2);
  return (size_t)kRows * ((d.Kmsg2 + 1) + (dg2 + 1) + 2 * (dm2 + 1)) * sizeof(float);
}

}  // namespace

void launch_memory_update(const Dev& d, hipStream_t s, const uint32_t* src, const uint32_t* dst, const double* ts,
                          const float* ef) {
  uint32_t blocks = (2 * d.max_batch + kRows - 1) / kRows;
  if (blocks > 1024) blocks = 1024;
  hipLaunchKernelGGL(memory_update_kernel, dim3(blocks), dim3(256), memory_lds(d), s, d, src, dst, ts, ef);
}

int setup_memory_attributes(const Dev& d) {
  if (d.d_mem == 0) return 0;
  const size_t need = memory_lds(d);
  if (need > kMaxLds) return -1;
  return hipFuncSetAttribute((const void*)memory_update_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                             (int)need) == hipSuccess ? 0 : -1;
}

}  // namespace stgn
