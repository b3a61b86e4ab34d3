// Compaction of the dirty flags into ascending lists: helpers shared by the compaction kernels and
// by the apply kernel, which carries the one-launch compaction of small flag arrays as extra
// workgroups when the propagation has already run (paper Sec. 3.3.1, Eq. affected_set).
#pragma once
#include "stgn_internal.h"

namespace stgn {

// inclusive scan over the 64 lanes of a wave
__device__ inline uint32_t wave_incl_scan(uint32_t v) {
  const uint32_t lane = threadIdx.x & 63u;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const uint32_t o = __shfl_up(v, off);
    if (lane >= (uint32_t)off) v += o;
  }
  return v;
}

// exclusive scan of one value per thread of a 256-thread workgroup (s: at least 4 words of LDS);
// returns the total.  Lane shuffles inside each wave, one exchange of the four wave totals.
__device__ inline uint32_t block_scan_256(uint32_t v, uint32_t* s, uint32_t* excl) {
  const uint32_t lane = threadIdx.x & 63u, w = threadIdx.x >> 6;
  const uint32_t incl = wave_incl_scan(v);
  if (lane == 63) s[w] = incl;
  __syncthreads();
  const uint32_t t0 = s[0], t1 = s[1], t2 = s[2], t3 = s[3];
  __syncthreads();
  const uint32_t before = w == 0 ? 0u : w == 1 ? t0 : w == 2 ? t0 + t1 : t0 + t1 + t2;
  *excl = before + incl - v;
  return t0 + t1 + t2 + t3;
}

constexpr uint32_t kFlagsPerThread = 16;
constexpr uint32_t kFlagsPerBlock = 256 * kFlagsPerThread;

// bit j set iff byte j of the 16 flags lies in [1, thr]
__device__ inline uint32_t bytes_upto(const uint4 m, uint32_t thr) {
  uint32_t bits = 0;
  const uint32_t w[4] = {m.x, m.y, m.z, m.w};
  for (int q = 0; q < 4; ++q)
    for (int j = 0; j < 4; ++j) {
      const uint32_t f = (w[q] >> (8 * j)) & 0xFFu;
      if (f != 0u && f <= thr) bits |= 1u << (4 * q + j);
    }
  return bits;
}
__device__ inline uint32_t bytes_equal(const uint4 m, uint32_t value) {
  uint32_t n = 0;
  const uint32_t w[4] = {m.x, m.y, m.z, m.w};
  for (int q = 0; q < 4; ++q)
    for (int j = 0; j < 4; ++j) n += ((w[q] >> (8 * j)) & 0xFFu) == value ? 1u : 0u;
  return n;
}

// list 0 is A (every non-zero flag); list 1 + l is R[l] for the layers that need their own list.
// Block sums are stored list-major: blocksum[list * nblocks + block].
__device__ inline uint32_t list_threshold(const Dev& d, uint32_t list) {
  if (list == 0) return 0xFFu;
  uint32_t seen = 0;
  for (uint32_t l = 0; l < d.layers; ++l)
    if (d.R[l] != d.A && ++seen == list) return d.thr[l];
  return 0xFFu;
}
__device__ inline uint32_t* list_base(const Dev& d, uint32_t list) {
  if (list == 0) return d.A;
  uint32_t seen = 0;
  for (uint32_t l = 0; l < d.layers; ++l)
    if (d.R[l] != d.A && ++seen == list) return d.R[l];
  return d.A;
}

// Last step of a batch's compaction, by one thread: list sizes and running totals.
__device__ inline void finish_batch(const Dev& d, const uint32_t (&total)[STGN_MAX_LAYERS + 1]) {
  Ctrl* c = d.ctrl;
  BatchCtl* bc = d.bc;
  bc->nA = total[0];
  uint32_t seen = 0;
  for (uint32_t l = 0; l < d.layers; ++l) bc->nR[l] = d.R[l] != d.A ? total[++seen] : total[0];
  c->tot_affected += total[0];
  c->tot_direct += bc->nD;
  bc->scanned = stripes_sum_thread(d, kScannedCounter);
  c->tot_scanned += bc->scanned;
  // delta mode: one more batch for the drift estimator (every per-node estimate, hence their sum, decays by gamma)
  if (d.delta && !bc->skip) { d.drift->tau += 1u; d.drift->G *= (double)d.gamma; }
}

// Count and write in one launch, for flag arrays of at most kSmallBlocks blocks: a workgroup counts
// the flags of the blocks before its own instead of waiting for their sums (at most 124 KiB of reads
// that hit L2), so no workgroup depends on another.  The batch's flags stay as they are (other workgroups
// may still be counting them): small flag arrays are held twice, by batch parity, and the next
// batch's apply step clears this one.
constexpr uint32_t kSmallBlocks = 32;
// bid / nblk: the workgroup's index and count among those that compact; s: 256 words of LDS.
__device__ inline void compact_small_block(const Dev& d, uint32_t last_value, uint32_t bid, uint32_t nblk, uint32_t* s) {
  const uint32_t t = threadIdx.x;
  const uint32_t v0 = bid * kFlagsPerBlock + t * kFlagsPerThread;
  const uint32_t nl = d.n_lists + 1u;
  uint32_t thr[STGN_MAX_LAYERS + 1], part[STGN_MAX_LAYERS + 1], total[STGN_MAX_LAYERS + 1];
#pragma unroll
  for (uint32_t list = 0; list <= STGN_MAX_LAYERS; ++list) {
    thr[list] = list < nl ? list_threshold(d, list) : 0u;
    part[list] = 0u; total[list] = 0u;
  }
  // statistics: nodes first reached by hop h carry the flag h + 2; the last workgroup has seen every block
  uint32_t eq[STGN_MAX_LAYERS + 1];
#pragma unroll
  for (uint32_t i = 0; i <= STGN_MAX_LAYERS; ++i) eq[i] = 0u;
  const bool last_block = bid == nblk - 1;
  for (uint32_t b = 0; b < bid; ++b) {
    const uint4 pm = *reinterpret_cast<const uint4*>(d.mark + b * kFlagsPerBlock + t * kFlagsPerThread);
#pragma unroll
    for (uint32_t list = 0; list <= STGN_MAX_LAYERS; ++list)
      if (list < nl) part[list] += (uint32_t)__popc(bytes_upto(pm, thr[list]));
    if (last_block) {
#pragma unroll
      for (uint32_t i = 0; i <= STGN_MAX_LAYERS; ++i)
        if (i + 2u <= last_value) eq[i] += bytes_equal(pm, i + 2u);
    }
  }
  uint4 m = make_uint4(0u, 0u, 0u, 0u);
  if (v0 < d.N) m = *reinterpret_cast<const uint4*>(d.mark + v0);     // the flag array is padded to whole blocks
  if (d.flags_kept && v0 < d.N) *reinterpret_cast<uint4*>(d.flags_kept + v0) = m;   // delta mode reads the batch's flags in the layer launches
  uint32_t excl;
#pragma unroll
  for (uint32_t list = 0; list <= STGN_MAX_LAYERS; ++list) {
    if (list < nl) {                                                   // uniform
      const uint32_t before = block_scan_256(part[list], s, &excl);
      uint32_t bits = bytes_upto(m, thr[list]);
      const uint32_t block_total = block_scan_256((uint32_t)__popc(bits), s, &excl);
      uint32_t* out = list_base(d, list) + before + excl;
      while (bits) {
        const uint32_t bit = (uint32_t)__ffs((int)bits) - 1u;
        *out++ = v0 + bit;
        bits &= bits - 1u;
      }
      total[list] = before + block_total;
    }
  }
  if (last_block) {                                                    // uniform
    uint32_t reached[STGN_MAX_LAYERS + 1];
#pragma unroll
    for (uint32_t i = 0; i <= STGN_MAX_LAYERS; ++i) {
      reached[i] = 0u;
      if (i + 2u <= last_value) reached[i] = block_scan_256(eq[i] + bytes_equal(m, i + 2u), s, &excl);
    }
    if (t == 0) {
      BatchCtl* bc = d.bc;
#pragma unroll
      for (uint32_t i = 0; i <= STGN_MAX_LAYERS; ++i)
        if (i + 2u <= last_value) bc->n_front[i + 1u] = reached[i];
      finish_batch(d, total);
    }
  }
}


inline __host__ __device__ uint32_t compact_blocks_of(uint32_t N) { return (N + kFlagsPerBlock - 1) / kFlagsPerBlock; }

}  // namespace stgn
