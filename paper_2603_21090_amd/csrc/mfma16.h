// fp32 matrix-core tiles for gfx950 with 16-row operands: C[16 x 16] += A[16 x K] * B[K x 16]
// using v_mfma_f32_16x16x4_f32 (K advances by 4 per instruction, one "k-step").
//
// K is cut into GROUPS of 16 elements = four k-steps.  Inside a group the four lane groups
// (lane / 16 = i) own the elements 16 g + 4 i + u, u = 0..3 being the k-step: the matrix
// instruction does not care which element of K a lane group contributes as long as A and B agree,
// and this assignment makes both operands of four consecutive k-steps one 16-byte value per lane:
//   A (LDS, row-major, stride lda = 4 mod 8 floats):  one ds_read_b128 at row * lda + 16 g + 4 i
//   B (weights, global): packed GROUP-MAJOR per 16-column tile at create time -- for column tile n
//     and group g, 64 lanes x 4 floats, lane (i, col) holding B[16 g + 4 i + u][16 n + col] for
//     u = 0..3; the groups of one column tile follow each other.  A wave's load of one group is one
//     contiguous 1 KiB read at an immediate offset.
// Four groups (64 elements of K) form a CHUNK, the unit of register double buffering: while the
// matrix pipe works on one chunk the operands of the next one are in flight.  K is padded to whole
// chunks with zero weights.  Two column tiles
// that share the A operand are multiplied together (independent accumulators, so consecutive
// matrix instructions never wait for each other).
#pragma once
#include <hip/hip_runtime.h>

namespace stgn {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr uint32_t kGrpK = 16;            // elements of K per group
constexpr uint32_t kGrpFloats = 256;      // floats of one (column tile, group) block of packed B
constexpr int kCG = 4;                    // groups per chunk
constexpr uint32_t kChunkSteps = 4 * kCG; // k-steps per chunk

// number of groups that cover K elements, rounded up to whole chunks
__host__ __device__ inline uint32_t chunks_of(uint32_t K) { return (K + kGrpK * kCG - 1) / (kGrpK * kCG); }
__host__ __device__ inline uint32_t groups_of(uint32_t K) { return kCG * chunks_of(K); }

// Operand layout of v_mfma_f32_16x16x4_f32 for lane l:
//   A element: row l % 16, lane group l / 16        B element: lane group l / 16, column l % 16
//   accumulator register r (0..3): row 4 * (l / 16) + r, column l % 16
__device__ inline uint32_t m16_row(uint32_t lane, uint32_t r) { return 4u * (lane >> 4) + r; }
__device__ inline uint32_t m16_col(uint32_t lane) { return lane & 15u; }

// per-lane element offset into an A tile in LDS with stride lda
__device__ inline uint32_t a16_lane_off(uint32_t lda) {
  const uint32_t lane = threadIdx.x & 63u;
  return (lane & 15u) * lda + 4u * (lane >> 4);
}

template <int U>
__device__ inline float comp4(const float4& v) {
  if constexpr (U == 0) return v.x;
  else if constexpr (U == 1) return v.y;
  else if constexpr (U == 2) return v.z;
  else return v.w;
}

// A operands of groups [g0, g0 + kCG) of the tile row range this lane serves (Ap = tile + lane offset).
// Reads past the last element of K land in neighbouring (finite) LDS data and meet zero weights.
__device__ inline void load_a16(const float* Ap, uint32_t g0, float4 (&a)[kCG]) {
#pragma unroll
  for (int c = 0; c < kCG; ++c) a[c] = *reinterpret_cast<const float4*>(Ap + kGrpK * (g0 + c));
}

// B operands of groups [g0, g0 + kCG) of the column tile whose group 0 is Bt (wave-uniform).
__device__ inline void load_b16(const float* __restrict__ Bt, uint32_t g0, float4 (&b)[kCG]) {
  const float4* p = reinterpret_cast<const float4*>(Bt) + (size_t)g0 * 64u + (threadIdx.x & 63u);
#pragma unroll
  for (int c = 0; c < kCG; ++c) b[c] = p[c * 64];
}

template <int U, int NTL>
__device__ inline void mfma16_one(const float4& a, const float4 (&b)[NTL][kCG], int c, floatx4 (&acc)[NTL]) {
#pragma unroll
  for (int t = 0; t < NTL; ++t)
    acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(comp4<U>(a), comp4<U>(b[t][c]), acc[t], 0, 0, 0);
}

// all 16 k-steps of one chunk, for NTL column tiles sharing the A operand.  Straight-line code: K is
// padded to whole chunks (zero weights, finite A), which costs a few surplus products and buys a
// loop body without branches that the compiler can schedule around the outstanding loads.
template <int NTL>
__device__ inline void mfma16_chunk(const float4 (&a)[kCG], const float4 (&b)[NTL][kCG], floatx4 (&acc)[NTL]) {
#pragma unroll
  for (int c = 0; c < kCG; ++c) {
    mfma16_one<0, NTL>(a[c], b, c, acc);
    mfma16_one<1, NTL>(a[c], b, c, acc);
    mfma16_one<2, NTL>(a[c], b, c, acc);
    mfma16_one<3, NTL>(a[c], b, c, acc);
  }
}

// Operands of one chunk for NTL column tiles.
template <int NTL>
struct Ops16 {
  float4 a[kCG];
  float4 b[NTL][kCG];
};

template <int NTL>
__device__ inline void mfma16_chunk(const Ops16<NTL>& o, floatx4 (&acc)[NTL]) { mfma16_chunk<NTL>(o.a, o.b, acc); }

// Runs compute(i, buf) for i = 0 .. n - 1 (n >= 1) with two operand buffers: the operands of item
// i + 1 are requested (load(i + 1, buf)) before the work on item i is issued, so every load has one
// whole item of work to arrive.  P already holds item 0.  Scheduling fences keep the requests ahead
// of the work they are meant to overlap.
//
// Loads inside the steady-state loop are never conditional: the memory counter a wave waits on
// counts requests in issue order, and after a branch that may or may not have issued requests the
// compiler must wait for the youngest of them -- which would drain the prefetch it was meant to hide.
//
// Peeled form: the tail is written out, so no request is wasted (three more copies of `compute`).
template <class Buf, class LoadF, class ComputeF>
__device__ __forceinline__ void pingpong_peeled(uint32_t n, Buf& P, LoadF load, ComputeF compute) {
  Buf Q;
  uint32_t i = 0;
  for (; i + 2 < n; i += 2) {
    load(i + 1, Q);
    __builtin_amdgcn_sched_barrier(0);
    compute(i, P);
    __builtin_amdgcn_sched_barrier(0);
    load(i + 2, P);
    __builtin_amdgcn_sched_barrier(0);
    compute(i + 1, Q);
    __builtin_amdgcn_sched_barrier(0);
  }
  if (i + 1 < n) {
    load(i + 1, Q);
    __builtin_amdgcn_sched_barrier(0);
    compute(i, P);
    __builtin_amdgcn_sched_barrier(0);
    compute(i + 1, Q);
  } else {
    compute(i, P);
  }
}

// Clamped form: two copies of `compute` only; past the end the last item is requested again (a
// cache hit) and ignored.
template <class Buf, class LoadF, class ComputeF>
__device__ __forceinline__ void pingpong_clamped(uint32_t n, Buf& P, LoadF load, ComputeF compute) {
  Buf Q;
  for (uint32_t i = 0; i < n; i += 2) {
    load(i + 1 < n ? i + 1 : n - 1, Q);
    __builtin_amdgcn_sched_barrier(0);
    compute(i, P);
    __builtin_amdgcn_sched_barrier(0);
    load(i + 2 < n ? i + 2 : n - 1, P);
    __builtin_amdgcn_sched_barrier(0);
    if (i + 1 < n) compute(i + 1, Q);
    __builtin_amdgcn_sched_barrier(0);
  }
}

// acc[t] += A[16 x 64 nchunks] * (column tile Bt[t]), nchunks >= 1; the weights of the first chunk are
// already in P.b -- callers request them ahead of the barrier that makes A valid.
template <int NTL>
__device__ __forceinline__ void mfma16_gemm_pre(const float* Ap, uint32_t nchunks, const float* const (&Bt)[NTL],
                                                floatx4 (&acc)[NTL], Ops16<NTL>& P) {
  load_a16(Ap, 0, P.a);
  pingpong_peeled<Ops16<NTL>>(
      nchunks, P,
      [&](uint32_t ch, Ops16<NTL>& o) {
        load_a16(Ap, ch * kCG, o.a);
#pragma unroll
        for (int t = 0; t < NTL; ++t) load_b16(Bt[t], ch * kCG, o.b[t]);
      },
      [&](uint32_t, const Ops16<NTL>& o) { mfma16_chunk<NTL>(o, acc); });
}

template <int NTL>
__device__ __forceinline__ void mfma16_gemm(const float* Ap, uint32_t nchunks, const float* const (&Bt)[NTL],
                                            floatx4 (&acc)[NTL]) {
  Ops16<NTL> P;
#pragma unroll
  for (int t = 0; t < NTL; ++t) load_b16(Bt[t], 0, P.b[t]);
  mfma16_gemm_pre<NTL>(Ap, nchunks, Bt, acc, P);
}

// All weight chunks of a short product at once: for K of at most MAXC chunks the whole B operand of
// NTL column tiles is requested in one go (MAXC * NTL * 16 registers), typically ahead of the barrier
// that completes A, and the products then run as the chunks arrive -- one memory latency per product
// instead of one per chunk.  For workgroups that run alone on a CU and cannot hide latencies.
template <int NTL, int MAXC>
struct Upfront16 {
  float4 b[MAXC][NTL][kCG];
  // requests are unconditional: chunks past the end repeat the last one and are never multiplied
  __device__ __forceinline__ void request(const float* const (&Bt)[NTL], uint32_t nchunks) {
#pragma unroll
    for (int ch = 0; ch < MAXC; ++ch) {
      const uint32_t c = (uint32_t)ch < nchunks ? (uint32_t)ch : nchunks - 1u;
#pragma unroll
      for (int t = 0; t < NTL; ++t) load_b16(Bt[t], c * kCG, b[ch][t]);
    }
  }
  __device__ __forceinline__ void multiply(const float* Ap, uint32_t nchunks, floatx4 (&acc)[NTL]) {
#pragma unroll
    for (int ch = 0; ch < MAXC; ++ch) {
      if ((uint32_t)ch < nchunks) {                  // wave-uniform; only LDS reads and products inside
        float4 a[kCG];
        load_a16(Ap, ch * kCG, a);
        mfma16_chunk<NTL>(a, b[ch], acc);
      }
    }
  }
};

}  // namespace stgn
