// Dirty-flag propagation over the temporal adjacency and compaction of the flags into the
// ascending affected-set list (paper Sec. 3.3.1, Eq. affected_set; invalidation rule Sec. 3.2.3).
//
// A frontier node u scans its whole adjacency log.  An entry (w, twin) names the neighbour and the
// position the same edge has in w's own log; the edge is still one of w's most recent k entries --
// so w's embedding reads u's row -- exactly when twin + k >= deg[w].
//
// Flags are one BYTE per node: 0 = clean, 1 = endpoint of the batch, h + 2 = first reached by hop h.
// A byte can be set with a plain store: every writer of one hop stores the same value, a stale read
// of 0 only repeats that store, and neighbouring bytes are never touched -- the expansion needs no
// atomic operation at all.  The frontier of the next hop is simply "all nodes whose flag equals
// h + 2", found by a scan of the flag array that also cuts the nodes' logs into work items of
// kLogChunk entries (one wavefront each), so that a hub's log is spread over the whole chip.
#include "stgn_internal.h"

namespace stgn {

namespace {

constexpr uint32_t kPlanThreads = 256;
constexpr uint32_t kPlanNodes = 1024;      // candidate nodes per workgroup (4 flags per thread)

// exclusive scan of one value per thread of a 256-thread workgroup; returns the total
__device__ inline uint32_t block_scan_256(uint32_t v, uint32_t* s, uint32_t* excl) {
  const uint32_t t = threadIdx.x;
  s[t] = v;
  __syncthreads();
  for (uint32_t off = 1; off < 256; off <<= 1) {
    const uint32_t add = t >= off ? s[t - off] : 0u;
    __syncthreads();
    s[t] += add;
    __syncthreads();
  }
  *excl = s[t] - v;
  const uint32_t total = s[255];
  __syncthreads();
  return total;
}

// Work items of hop `hop`: from the list D (hop 0) or from the flags that equal hop + 1.
__global__ __launch_bounds__(kPlanThreads) void plan_kernel(Dev d, uint32_t hop) {
  __shared__ uint32_t s_scan[256], s_list[kPlanNodes], s_off[256], s_v[256];
  __shared__ uint32_t s_base;
  Ctrl* c = d.ctrl;
  if (c->skip) return;
  const uint32_t t = threadIdx.x;
  // ---- candidates of this workgroup, compacted into s_list
  uint32_t cand[4], nc = 0;
  if (hop == 0) {
    const uint32_t nD = c->nD;
    for (uint32_t j = 0; j < 4; ++j) {
      const uint32_t x = blockIdx.x * kPlanNodes + 4 * t + j;
      if (x < nD) cand[nc++] = d.D[x];
    }
  } else {
    const uint32_t v0 = blockIdx.x * kPlanNodes + 4 * t;
    if (v0 < d.N) {                                          // the flag array is padded to whole words
      const uint32_t m = *reinterpret_cast<const uint32_t*>(d.mark + v0);
      for (uint32_t j = 0; j < 4; ++j)
        if (((m >> (8 * j)) & 0xFFu) == hop + 1u) cand[nc++] = v0 + j;
    }
  }
  uint32_t excl;
  const uint32_t ncand = block_scan_256(nc, s_scan, &excl);
  if (ncand == 0) return;
  for (uint32_t j = 0; j < nc; ++j) s_list[excl + j] = cand[j];
  __syncthreads();
  // ---- rounds of 256 candidates: chunk counts, one counter update per round, cooperative fill
  unsigned long long scanned = 0;
  for (uint32_t r0 = 0; r0 < ncand; r0 += 256) {
    const uint32_t v = r0 + t < ncand ? s_list[r0 + t] : 0u;
    const uint32_t dg = r0 + t < ncand ? d.deg[v] : 0u;
    const uint32_t nch = (dg + kLogChunk - 1) / kLogChunk;
    scanned += dg;
    uint32_t off;
    const uint32_t total = block_scan_256(nch, s_scan, &off);
    s_off[t] = off;
    s_v[t] = v;
    if (t == 0) s_base = total ? atomicAdd(&c->n_items[hop], total) : 0u;
    __syncthreads();
    const uint32_t base = s_base;
    for (uint32_t i = t; i < total; i += 256) {
      uint32_t lo = 0, hi = 255;                             // last thread whose offset is <= i
      while (lo < hi) {
        const uint32_t mid = (lo + hi + 1) >> 1;
        if (s_off[mid] <= i) lo = mid; else hi = mid - 1;
      }
      d.items[base + i] = ((uint64_t)s_v[lo] << 32) | (i - s_off[lo]);
    }
    __syncthreads();
  }
  // statistics: frontier size and entries the expansion of this hop will read
  for (int off = 32; off > 0; off >>= 1) scanned += __shfl_xor(scanned, off);
  if ((t & 63) == 0 && scanned) atomicAdd((unsigned long long*)&c->scanned, scanned);
  if (t == 0 && hop > 0) atomicAdd(&c->n_front[hop], ncand);
}

__global__ __launch_bounds__(256) void expand_kernel(Dev d, uint32_t hop) {
  const Ctrl* c = d.ctrl;
  if (c->skip) return;
  const uint32_t n_items = c->n_items[hop];
  const uint32_t lane = threadIdx.x & 63;
  const uint8_t value = (uint8_t)(hop + 2u);
  // wave index, made provably uniform so that everything derived from it stays in scalar registers
  const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)((blockIdx.x * blockDim.x + threadIdx.x) >> 6));
  const uint32_t nwaves = (gridDim.x * blockDim.x) >> 6;
  for (uint32_t it = wave; it < n_items; it += nwaves) {
    const uint64_t item = d.items[it];
    const uint32_t u = (uint32_t)(item >> 32), ch = (uint32_t)item;
    const uint32_t dg = d.deg[u];
    const uint32_t lo = ch * kLogChunk, hi = min(dg, lo + kLogChunk);
    const uint32_t* blk = d.blk + (size_t)u * d.maxb;
    for (uint32_t p0 = lo; p0 < hi; p0 += 64) {
      const uint32_t p = p0 + lane;
      if (p < hi) {
        const uint32_t b = 31u - (uint32_t)__clz((int)((p >> 3) + 1u));
        const uint32_t off = p - kMinBlock * ((1u << b) - 1u);
        const uint2 e = d.pool_nt[(uint64_t)blk[b] * kMinBlock + off];
        const uint32_t w = e.x;
        if ((uint64_t)e.y + d.k >= d.deg[w] && d.mark[w] == 0) d.mark[w] = value;
      }
    }
  }
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

__global__ __launch_bounds__(256) void compact_count_kernel(Dev d, uint32_t last_value) {
  __shared__ uint32_t s[256];
  const uint32_t v0 = blockIdx.x * kFlagsPerBlock + threadIdx.x * kFlagsPerThread;
  uint4 m = make_uint4(0u, 0u, 0u, 0u);
  if (v0 < d.N) m = *reinterpret_cast<const uint4*>(d.mark + v0);     // the flag array is padded to whole blocks
  uint32_t excl;
  for (uint32_t list = 0; list <= d.n_lists; ++list) {
    const uint32_t cnt = (uint32_t)__popc(bytes_upto(m, list_threshold(d, list)));
    const uint32_t tot = block_scan_256(cnt, s, &excl);
    if (threadIdx.x == 0) d.blocksum[list * gridDim.x + blockIdx.x] = tot;
  }
  const uint32_t tot_reached = block_scan_256(bytes_equal(m, last_value), s, &excl);
  if (threadIdx.x == 0 && tot_reached) atomicAdd(&d.ctrl->n_front[last_value - 1u], tot_reached);   // first reached by the last hop
}

__global__ __launch_bounds__(256) void compact_write_kernel(Dev d) {
  __shared__ uint32_t s[256];
  const uint32_t t = threadIdx.x;
  const uint32_t v0 = blockIdx.x * kFlagsPerBlock + t * kFlagsPerThread;
  uint4 m = make_uint4(0u, 0u, 0u, 0u);
  if (v0 < d.N) m = *reinterpret_cast<const uint4*>(d.mark + v0);
  uint32_t excl, total[STGN_MAX_LAYERS + 1];
  for (uint32_t list = 0; list <= d.n_lists; ++list) {
    // ids before this block
    uint32_t part = 0;
    for (uint32_t b = t; b < blockIdx.x; b += 256) part += d.blocksum[list * gridDim.x + b];
    const uint32_t before = block_scan_256(part, s, &excl);
    // scan inside the block
    uint32_t bits = bytes_upto(m, list_threshold(d, list));
    const uint32_t cnt = (uint32_t)__popc(bits);
    const uint32_t block_total = block_scan_256(cnt, s, &excl);
    uint32_t* out = list_base(d, list) + before + excl;
    while (bits) {
      const uint32_t bit = (uint32_t)__ffs((int)bits) - 1u;
      *out++ = v0 + bit;
      bits &= bits - 1u;
    }
    total[list] = before + block_total;
  }
  if (m.x | m.y | m.z | m.w) *reinterpret_cast<uint4*>(d.mark + v0) = make_uint4(0u, 0u, 0u, 0u);   // ready for the next batch
  if (blockIdx.x == gridDim.x - 1 && t == 0) {
    Ctrl* c = d.ctrl;
    c->nA = total[0];
    uint32_t seen = 0;
    for (uint32_t l = 0; l < d.layers; ++l) c->nR[l] = d.R[l] != d.A ? total[++seen] : total[0];
    c->tot_affected += total[0];
    c->tot_direct += c->nD;
    c->tot_scanned += c->scanned;
  }
}

}  // namespace

void launch_plan(const Dev& d, hipStream_t s, uint32_t hop) {
  const uint32_t span = hop == 0 ? 2 * d.max_batch : d.N;
  const uint32_t blocks = (span + kPlanNodes - 1) / kPlanNodes;
  hipLaunchKernelGGL(plan_kernel, dim3(blocks), dim3(kPlanThreads), 0, s, d, hop);
}

void launch_expand(const Dev& d, hipStream_t s, uint32_t hop) {
  // one wave per work item, grid-stride; enough waves to fill the chip without a long empty tail
  uint64_t want = ((uint64_t)d.N + 3) / 4;
  uint32_t blocks = want > 4096 ? 4096u : (uint32_t)(want ? want : 1);
  hipLaunchKernelGGL(expand_kernel, dim3(blocks), dim3(256), 0, s, d, hop);
}

void launch_compact(const Dev& d, hipStream_t s, int phase) {
  const uint32_t blocks = (d.N + kFlagsPerBlock - 1) / kFlagsPerBlock;
  if (phase == 0) hipLaunchKernelGGL(compact_count_kernel, dim3(blocks), dim3(256), 0, s, d, d.layers + 1u);
  else hipLaunchKernelGGL(compact_write_kernel, dim3(blocks), dim3(256), 0, s, d);
}

}  // namespace stgn
