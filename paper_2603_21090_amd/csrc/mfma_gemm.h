// fp32 matrix-core tiles for gfx950: C[32 x 32] += A[32 x K] * B[K x 32] with
// v_mfma_f32_32x32x2_f32.  A comes from LDS (row-major, any stride), B from global memory in the
// packed layout [K2 x ldb] (K padded to even with zero rows, columns padded to a multiple of 32).
// B is streamed straight from L2 into registers in chunks of kBU k-steps; callers keep the next
// chunk's loads in flight while the matrix instructions of the current chunk run.  Inside a chunk
// the code is branch-free in groups of kBG k-steps so that the LDS reads of a whole group are
// issued ahead of its matrix instructions.
#pragma once
#include <hip/hip_runtime.h>

namespace stgn {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kBU = 32;   // k-steps (of 2) per register chunk of B
constexpr int kBG = 8;    // k-steps per branch-free group

// Operand layout of v_mfma_f32_32x32x2_f32 for lane l (64 lanes):
//   A element: row l % 32, k index l / 32        B element: k index l / 32, column l % 32
//   accumulator register j (0..15): row 8 * (j / 4) + 4 * (l / 32) + j % 4, column l % 32
__device__ inline uint32_t mfma_row(uint32_t lane, uint32_t j) { return 8u * (j >> 2) + 4u * (lane >> 5) + (j & 3u); }
__device__ inline uint32_t mfma_col(uint32_t lane) { return lane & 31u; }

// this lane's B pointer for column tile n0: k-step s reads bp[2 s ldb]
__device__ inline const float* b_lane_ptr(const float* __restrict__ B, uint32_t ldb, uint32_t n0) {
  const uint32_t lane = threadIdx.x & 63u;
  return B + (size_t)(lane >> 5) * ldb + n0 + (lane & 31u);
}
// this lane's A pointer: k-step s of row block rb reads ap[rb 32 lda + 2 s]
__device__ inline const float* a_lane_ptr(const float* As, uint32_t lda) {
  const uint32_t lane = threadIdx.x & 63u;
  return As + (size_t)(lane & 31u) * lda + (lane >> 5);
}

// issue the loads of k-steps [s0, s0 + U) (clamped to the last step; steps >= 1)
template <int U>
__device__ inline void load_b(const float* __restrict__ bp, uint32_t ldb, uint32_t s0, uint32_t steps, float (&b)[U]) {
  const uint32_t last = steps - 1;
#pragma unroll
  for (int u = 0; u < U; ++u) {
    uint32_t s = s0 + u;
    s = s < steps ? s : last;
    b[u] = bp[(size_t)2 * s * ldb];
  }
}

// matrix instructions of k-steps [s0, min(s0 + U, steps)).  A k-step past `steps` inside the last
// group multiplies a zero A operand (its B value is a clamped, finite weight).
template <int RB, int U>
__device__ inline void mfma_steps(const float* ap, uint32_t lda, uint32_t s0, uint32_t steps, const float (&b)[U],
                                  floatx16 (&acc)[RB]) {
  const uint32_t last = steps - 1;
#pragma unroll
  for (int g = 0; g < U / kBG; ++g) {
    const uint32_t sg = s0 + g * kBG;
    if (sg < steps) {                      // wave-uniform, one branch per group
      float a[RB][kBG];
#pragma unroll
      for (int u = 0; u < kBG; ++u) {
        const uint32_t s = sg + u;
        const uint32_t sc = s < steps ? s : last;
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
          const float v = ap[(size_t)rb * 32u * lda + 2u * sc];
          a[rb][u] = s < steps ? v : 0.0f;
        }
      }
#pragma unroll
      for (int u = 0; u < kBG; ++u)
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
          acc[rb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[rb][u], b[g * kBG + u], acc[rb], 0, 0, 0);
    }
  }
}

// acc[rb] += As[rb*32 .. rb*32+31][0..K2) * B[0..K2)[n0 .. n0+31]; `bcur` already holds chunk 0
template <int RB, int U = kBU>
__device__ inline void mfma_tile_pre(const float* As, uint32_t lda, uint32_t K2, const float* __restrict__ B,
                                     uint32_t ldb, uint32_t n0, floatx16 (&acc)[RB], float (&bcur)[U]) {
  const uint32_t steps = K2 >> 1;
  if (steps == 0) return;
  const float* bp = b_lane_ptr(B, ldb, n0);
  const float* ap = a_lane_ptr(As, lda);
  float bnext[U];
  for (uint32_t s0 = 0; s0 < steps; s0 += U) {
    if (s0 + U < steps) load_b<U>(bp, ldb, s0 + U, steps, bnext);
    mfma_steps<RB, U>(ap, lda, s0, steps, bcur, acc);
    if (s0 + U < steps) {
#pragma unroll
      for (int u = 0; u < U; ++u) bcur[u] = bnext[u];
    }
  }
}

template <int RB, int U = kBU>
__device__ inline void mfma_tile(const float* As, uint32_t lda, uint32_t K2, const float* __restrict__ B,
                                 uint32_t ldb, uint32_t n0, floatx16 (&acc)[RB]) {
  if ((K2 >> 1) == 0) return;
  float bcur[U];
  load_b<U>(b_lane_ptr(B, ldb, n0), ldb, 0, K2 >> 1, bcur);
  mfma_tile_pre<RB, U>(As, lda, K2, B, ldb, n0, acc, bcur);
}

template <int RB>
__device__ inline void zero_acc(floatx16 (&acc)[RB]) {
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[rb][j] = 0.0f;
}

}  // namespace stgn
