// fp32 matrix-core tiles for gfx950 with 16-row operands: C[16 x 16] += A[16 x K] * B[K x 16]
// using v_mfma_f32_16x16x4_f32 (K advances by 4 per instruction, one "k-step").
//
// A comes from LDS.  B (weights) comes from global memory in a TILE-MAJOR packing: for a column
// tile n and k-step s the 4 x 16 operand block is stored as 64 consecutive floats [kk][col], and
// the blocks of one column tile follow each other in k order.  A wave's B load is then one
// contiguous 256-byte read, consecutive k-steps are 256 bytes apart (immediate offsets, no address
// arithmetic), and reading a few blocks past the end of a tile is harmless (the packing is padded
// and the surplus products are never issued).  B is streamed from L2 into registers one chunk of
// kU16 k-steps at a time; callers keep the next chunk in flight while the current one is multiplied.
#pragma once
#include <hip/hip_runtime.h>

namespace stgn {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kU16 = 16;            // k-steps per register chunk of B
constexpr int kG16 = 4;             // k-steps per branch-free group
constexpr uint32_t kBlk16 = 64;     // floats in one (column tile, k-step) block
constexpr uint32_t kPadBlocks = 2 * kU16;   // blocks of zero padding behind every packed matrix

// Operand layout of v_mfma_f32_16x16x4_f32 for lane l:
//   A element: row l % 16, k index l / 16        B element: k index l / 16, column l % 16
//   accumulator register r (0..3): row 4 * (l / 16) + r, column l % 16
__device__ inline uint32_t m16_row(uint32_t lane, uint32_t r) { return 4u * (lane >> 4) + r; }
__device__ inline uint32_t m16_col(uint32_t lane) { return lane & 15u; }

// per-lane element offset into an A tile in LDS with stride lda: row * lda + k index
__device__ inline uint32_t a16_lane_off(uint32_t lda) {
  const uint32_t lane = threadIdx.x & 63u;
  return (lane & 15u) * lda + (lane >> 4);
}

// Issue the loads of k-steps [s0, s0 + U) of the column tile whose block 0 is Bt (wave-uniform).
template <int U>
__device__ inline void load_b16(const float* __restrict__ Bt, uint32_t s0, float (&b)[U]) {
  const float* base = Bt + (size_t)s0 * kBlk16;          // uniform
  const uint32_t lane = threadIdx.x & 63u;
#pragma unroll
  for (int u = 0; u < U; ++u) b[u] = base[lane + u * kBlk16];
}

// Matrix instructions of k-steps [s0, min(s0 + U, steps)) with A tile `At` (LDS, this lane's
// element offset aoff).
template <int U>
__device__ inline void mfma16_steps(const float* At, uint32_t aoff, uint32_t s0, uint32_t steps, const float (&b)[U],
                                    floatx4& acc) {
  const float* ap = At + aoff;
#pragma unroll
  for (int g = 0; g < U / kG16; ++g) {
    const uint32_t sg = s0 + g * kG16;
    if (sg + kG16 <= steps) {              // wave-uniform: a full group
      float a[kG16];
#pragma unroll
      for (int u = 0; u < kG16; ++u) a[u] = ap[4u * (sg + u)];
#pragma unroll
      for (int u = 0; u < kG16; ++u) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[u], b[g * kG16 + u], acc, 0, 0, 0);
    } else if (sg < steps) {               // ragged tail
#pragma unroll
      for (int u = 0; u < kG16; ++u) {
        if (sg + u < steps) {
          const float a = ap[4u * (sg + u)];
          acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b[g * kG16 + u], acc, 0, 0, 0);
        }
      }
    }
  }
}

// acc += At[0..15][0 .. 4 steps) * (column tile Bt); `bcur` already holds k-steps [0, U)
template <int U = kU16>
__device__ inline void mfma16_tile_pre(const float* At, uint32_t aoff, uint32_t steps, const float* __restrict__ Bt,
                                       floatx4& acc, float (&bcur)[U]) {
  float bnext[U];
  for (uint32_t s0 = 0; s0 < steps; s0 += U) {
    if (s0 + U < steps) load_b16<U>(Bt, s0 + U, bnext);
    mfma16_steps<U>(At, aoff, s0, steps, bcur, acc);
    if (s0 + U < steps) {
#pragma unroll
      for (int u = 0; u < U; ++u) bcur[u] = bnext[u];
    }
  }
}

template <int U = kU16>
__device__ inline void mfma16_tile(const float* At, uint32_t aoff, uint32_t steps, const float* __restrict__ Bt,
                                   floatx4& acc) {
  if (steps == 0) return;
  float bcur[U];
  load_b16<U>(Bt, 0, bcur);
  mfma16_tile_pre<U>(At, aoff, steps, Bt, acc, bcur);
}

}  // namespace stgn
