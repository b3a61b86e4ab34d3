// Placement of a batch's endpoint slots in the adjacency logs: the degree-dependent second half of the
// staging (paper Sec. 3.2.2, append-only temporal adjacency).  Shared by the placement kernel and by
// the memory-update launch, which carries it as one extra workgroup.
#pragma once
#include "stgn_internal.h"

namespace stgn {

// Exclusive scan of one value per thread of the (whole-wave multiple, at most 1024 threads) workgroup:
// lane shuffles inside each wave, one exchange of the wave totals through s_buf (16 words).  Returns
// the exclusive prefix and writes the workgroup total to *total.
__device__ inline uint32_t block_excl_scan(uint32_t v, uint32_t* s_buf, uint32_t* total) {
  const uint32_t lane = threadIdx.x & 63u, w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  uint32_t incl = v;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const uint32_t o = __shfl_up(incl, off);
    if (lane >= (uint32_t)off) incl += o;
  }
  if (lane == 63) s_buf[w] = incl;
  __syncthreads();
  uint32_t before = 0, all = 0;
  for (uint32_t i = 0; i < nw; ++i) {
    const uint32_t ti = s_buf[i];
    before += i < w ? ti : 0u;
    all += ti;
  }
  if (total && threadIdx.x == 0) *total = all;
  __syncthreads();
  return before + incl - v;
}

// number of adjacency blocks (sizes 8, 16, 32, ...) needed to hold x entries
__device__ inline uint32_t blocks_for(uint32_t x) {
  const uint32_t units = (x + kMinBlock - 1) / kMinBlock;
  return units ? 32u - (uint32_t)__clz((int)units) : 0u;
}

// Second half of the staging, the part that depends on the degrees the previous batch's apply step
// left behind (the first half only looks at the batch itself): position of every endpoint slot in its
// node's adjacency log, the endpoints' new degrees, the adjacency blocks they need (allocated in
// endpoint order, so the placement is deterministic) and the number of adjacency entries the
// endpoints own, which the first propagation hop plans with.  Called by the whole workgroup once the
// sorted lists are visible to it; returns (to thread 0, through *units_total) the pool units taken.
__device__ inline void place_rows(const Dev& d, uint32_t n, uint32_t nD, uint32_t* s_buf, uint32_t* units_total) {
  const Ctrl* c = d.ctrl;
  const uint32_t t = threadIdx.x, nth = blockDim.x;
  const uint32_t m = 2 * n;
  for (uint32_t i = t; i < m; i += nth) {
    const uint32_t slot = d.slot_sorted[i];
    const uint32_t di = d.slot_d[slot];
    d.slot_pos[slot] = d.deg[d.D[di]] + (i - d.seg_start[di]);
  }
  // dirty seeds of the propagation.  With two flag arrays (small node counts) this batch's array is
  // clean already -- the previous batch's apply step cleared it -- and seeding here lets the first hop
  // run ahead of the apply step; a single array is still being compacted by the previous batch now,
  // and the apply step seeds it.
  if (d.mark_other != d.mark)
    for (uint32_t x = t; x < nD; x += nth) d.mark[d.D[x]] = 1;
  const uint32_t eptd = (nD + nth - 1) / nth;     // contiguous endpoints per thread
  const uint32_t dlo = min(t * eptd, nD), dhi = min(dlo + eptd, nD);
  uint32_t units = 0;
  unsigned long long fdeg = 0;              // adjacency entries the endpoints own after this batch
  for (uint32_t x = dlo; x < dhi; ++x) {
    const uint32_t dp = d.deg[d.D[x]], dn = dp + (d.seg_start[x + 1] - d.seg_start[x]);
    d.deg_new[x] = dn;
    fdeg += dn;
    units += (1u << blocks_for(dn)) - (1u << blocks_for(dp));
  }
  const uint32_t uexcl = block_excl_scan(units, s_buf, units_total);
  {
    uint64_t base = c->pool_units + uexcl;
    for (uint32_t x = dlo; x < dhi; ++x) {
      const uint32_t node = d.D[x];
      const uint32_t b0 = blocks_for(d.deg[node]), b1 = blocks_for(d.deg_new[x]);
      for (uint32_t b = b0; b < b1; ++b) {
        d.blk[(size_t)node * d.maxb + b] = (uint32_t)base;
        base += 1u << b;
      }
    }
  }
  for (int off = 32; off > 0; off >>= 1) fdeg += __shfl_xor(fdeg, off);
  if ((t & 63) == 0 && fdeg) atomicAdd(stripe(d, 0, t >> 6), fdeg);
  __syncthreads();                          // every thread has read pool_units
}

// the whole step for one workgroup of any whole-wave size; s_buf: 16 words, s_units: one word of LDS
__device__ inline void place_batch(const Dev& d, uint32_t* s_buf, uint32_t* s_units) {
  const BatchCtl* bc = d.bc;
  if (bc->skip) return;
  place_rows(d, bc->n_edges, bc->nD, s_buf, s_units);
  if (threadIdx.x == 0) d.ctrl->pool_units += *s_units;
}

}  // namespace stgn
