// fp32 matrix-core tiles for gfx950: C[32 x 32] += A[32 x K] * B[K x 32] with
// v_mfma_f32_32x32x2_f32.  A comes from LDS (row-major, any stride), B from global memory in the
// packed layout [K2 x ldb] (K padded to even with zero rows, columns padded to a multiple of 32).
#pragma once
#include <hip/hip_runtime.h>

namespace stgn {

typedef float floatx16 __attribute__((ext_vector_type(16)));

// Operand layout of v_mfma_f32_32x32x2_f32 for lane l (64 lanes):
//   A element: row l % 32, k index l / 32        B element: k index l / 32, column l % 32
//   accumulator register j (0..15): row 8 * (j / 4) + 4 * (l / 32) + j % 4, column l % 32
__device__ inline uint32_t mfma_row(uint32_t lane, uint32_t j) { return 8u * (j >> 2) + 4u * (lane >> 5) + (j & 3u); }
__device__ inline uint32_t mfma_col(uint32_t lane) { return lane & 31u; }

// acc[rb] += As[rb*32 .. rb*32+31][0..K2) * B[0..K2)[n0 .. n0+31]
template <int RB>
__device__ inline void mfma_tile(const float* As, uint32_t lda, uint32_t K2, const float* __restrict__ B,
                                 uint32_t ldb, uint32_t n0, floatx16 (&acc)[RB]) {
  const uint32_t lane = threadIdx.x & 63u;
  const uint32_t r = lane & 31u, kk = lane >> 5;
  const float* bp = B + (size_t)kk * ldb + n0 + r;
  const float* ap = As + (size_t)r * lda + kk;
#pragma unroll 4
  for (uint32_t k0 = 0; k0 < K2; k0 += 2) {
    const float b = bp[(size_t)k0 * ldb];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      const float a = ap[(size_t)rb * 32u * lda + k0];
      acc[rb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[rb], 0, 0, 0);
    }
  }
}

template <int RB>
__device__ inline void zero_acc(floatx16 (&acc)[RB]) {
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[rb][j] = 0.0f;
}

}  // namespace stgn
