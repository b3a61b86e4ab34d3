// Dirty-flag propagation over the temporal adjacency and compaction of the dirty bitmap into the
// ascending affected-set list (paper Sec. 3.3.1, Eq. affected_set; invalidation rule Sec. 3.2.3).
//
// A frontier node u scans its whole adjacency log.  An entry (w, twin) names the neighbour and the
// position the same edge has in w's own log; the edge is still one of w's most recent k entries --
// so w's embedding reads u's row -- exactly when twin + k >= deg[w].  Such w are flagged with an
// atomic OR into an N-bit bitmap; the returned word tells which lane set the bit first, and those
// lanes append w to the next frontier (one atomic add per wave, ballot-compacted).
#include "stgn_internal.h"

namespace stgn {

namespace {

__global__ __launch_bounds__(256) void plan_kernel(Dev d, uint32_t hop) {
  Ctrl* c = d.ctrl;
  if (c->skip) return;
  const uint32_t nf = c->n_front[hop];
  const uint32_t* list = hop == 0 ? d.D : d.front[hop & 1];
  const uint32_t tid = blockIdx.x * blockDim.x + threadIdx.x, nth = gridDim.x * blockDim.x;
  unsigned long long scanned = 0;
  for (uint32_t x = tid; x < nf; x += nth) {
    const uint32_t u = list[x];
    const uint32_t dg = d.deg[u];
    const uint32_t nch = (dg + kLogChunk - 1) / kLogChunk;
    if (nch == 0) continue;
    scanned += dg;
    const uint32_t base = atomicAdd(&c->n_items[hop], nch);
    for (uint32_t ch = 0; ch < nch; ++ch) d.items[base + ch] = ((uint64_t)u << 32) | ch;
  }
  // entries the expansion of this hop will read: one atomic per wave
  for (int off = 32; off > 0; off >>= 1) scanned += __shfl_xor(scanned, off);
  if ((threadIdx.x & 63) == 0 && scanned) atomicAdd((unsigned long long*)&c->scanned, scanned);
}

__global__ __launch_bounds__(256) void expand_kernel(Dev d, uint32_t hop, int write_next) {
  Ctrl* c = d.ctrl;
  if (c->skip) return;
  const uint32_t n_items = c->n_items[hop];
  uint32_t* next = d.front[(hop + 1) & 1];
  const uint32_t lane = threadIdx.x & 63;
  // wave index, made provably uniform so that everything derived from it stays in scalar registers
  const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)((blockIdx.x * blockDim.x + threadIdx.x) >> 6));
  const uint32_t nwaves = (gridDim.x * blockDim.x) >> 6;
  const uint64_t lt_mask = (1ull << lane) - 1ull;
  for (uint32_t it = wave; it < n_items; it += nwaves) {
    const uint64_t item = d.items[it];
    const uint32_t u = (uint32_t)(item >> 32), ch = (uint32_t)item;
    const uint32_t dg = d.deg[u];
    const uint32_t lo = ch * kLogChunk, hi = min(dg, lo + kLogChunk);
    const uint32_t* blk = d.blk + (size_t)u * d.maxb;
    for (uint32_t p0 = lo; p0 < hi; p0 += 64) {
      const uint32_t p = p0 + lane;
      bool isnew = false;
      uint32_t w = 0;
      if (p < hi) {
        const uint32_t b = 31u - (uint32_t)__clz((int)((p >> 3) + 1u));
        const uint32_t off = p - kMinBlock * ((1u << b) - 1u);
        const uint2 e = d.pool_nt[(uint64_t)blk[b] * kMinBlock + off];
        w = e.x;
        if ((uint64_t)e.y + d.k >= d.deg[w]) {
          const uint32_t bit = 1u << (w & 31);
          uint32_t* word = d.bitmap + (w >> 5);
          // coherent (L2) read first: most flags are already set, and a stale L1 line would turn
          // every one of those into an atomic on a handful of hot cache lines
          const uint32_t cur = __hip_atomic_load(word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          if (!(cur & bit)) isnew = !(atomicOr(word, bit) & bit);
        }
      }
      const uint64_t m = __ballot(isnew);
      if (m) {
        uint32_t base = 0;
        if (lane == (uint32_t)__ffsll((long long)m) - 1) base = atomicAdd(&c->n_front[hop + 1], (uint32_t)__popcll(m));
        base = __shfl(base, __ffsll((long long)m) - 1);
        if (isnew && write_next) next[base + (uint32_t)__popcll(m & lt_mask)] = w;
      }
    }
  }
}

constexpr uint32_t kWordsPerThread = 4;
constexpr uint32_t kWordsPerBlock = 256 * kWordsPerThread;

__device__ inline uint32_t block_sum_256(uint32_t v, uint32_t* s) {
  const uint32_t t = threadIdx.x;
  s[t] = v;
  __syncthreads();
  for (uint32_t off = 128; off > 0; off >>= 1) {
    if (t < off) s[t] += s[t + off];
    __syncthreads();
  }
  const uint32_t r = s[0];
  __syncthreads();
  return r;
}

__global__ __launch_bounds__(256) void compact_count_kernel(Dev d, uint32_t nwords) {
  __shared__ uint32_t s[256];
  const uint32_t w0 = blockIdx.x * kWordsPerBlock + threadIdx.x * kWordsPerThread;
  uint32_t cnt = 0;
  for (uint32_t j = 0; j < kWordsPerThread; ++j)
    if (w0 + j < nwords) cnt += (uint32_t)__popc(d.bitmap[w0 + j]);
  const uint32_t tot = block_sum_256(cnt, s);
  if (threadIdx.x == 0) d.blocksum[blockIdx.x] = tot;
}

__global__ __launch_bounds__(256) void compact_write_kernel(Dev d, uint32_t nwords) {
  __shared__ uint32_t s[256];
  const uint32_t t = threadIdx.x;
  // ids before this block
  uint32_t part = 0;
  for (uint32_t b = t; b < blockIdx.x; b += 256) part += d.blocksum[b];
  const uint32_t before = block_sum_256(part, s);
  // scan inside the block
  const uint32_t w0 = blockIdx.x * kWordsPerBlock + t * kWordsPerThread;
  uint32_t words[kWordsPerThread];
  uint32_t cnt = 0;
  for (uint32_t j = 0; j < kWordsPerThread; ++j) {
    words[j] = (w0 + j < nwords) ? d.bitmap[w0 + j] : 0u;
    cnt += (uint32_t)__popc(words[j]);
  }
  s[t] = cnt;
  __syncthreads();
  for (uint32_t off = 1; off < 256; off <<= 1) {
    const uint32_t add = t >= off ? s[t - off] : 0u;
    __syncthreads();
    s[t] += add;
    __syncthreads();
  }
  uint32_t out = before + s[t] - cnt;
  const uint32_t block_total = s[255];
  for (uint32_t j = 0; j < kWordsPerThread; ++j) {
    uint32_t wv = words[j];
    while (wv) {
      const uint32_t bit = (uint32_t)__ffs((int)wv) - 1u;
      d.A[out++] = (w0 + j) * 32u + bit;
      wv &= wv - 1u;
    }
    if (w0 + j < nwords && words[j]) d.bitmap[w0 + j] = 0u;   // ready for the next batch
  }
  if (blockIdx.x == gridDim.x - 1 && t == 0) {
    Ctrl* c = d.ctrl;
    const uint32_t nA = before + block_total;
    c->nA = nA;
    c->tot_affected += nA;
    c->tot_direct += c->nD;
    c->tot_scanned += c->scanned;
  }
}

}  // namespace

void launch_plan(const Dev& d, hipStream_t s, uint32_t hop) {
  uint32_t blocks = (d.N + 255) / 256;
  if (blocks > 1024) blocks = 1024;
  hipLaunchKernelGGL(plan_kernel, dim3(blocks), dim3(256), 0, s, d, hop);
}

void launch_expand(const Dev& d, hipStream_t s, uint32_t hop, bool last) {
  // one wave per work item, grid-stride; enough waves to fill the chip without a long empty tail
  uint64_t want = ((uint64_t)d.N + 3) / 4;
  uint32_t blocks = want > 4096 ? 4096u : (uint32_t)(want ? want : 1);
  hipLaunchKernelGGL(expand_kernel, dim3(blocks), dim3(256), 0, s, d, hop, last ? 0 : 1);
}

void launch_compact(const Dev& d, hipStream_t s, int phase) {
  const uint32_t nwords = (d.N + 31) / 32;
  const uint32_t blocks = (nwords + kWordsPerBlock - 1) / kWordsPerBlock;
  if (phase == 0) hipLaunchKernelGGL(compact_count_kernel, dim3(blocks), dim3(256), 0, s, d, nwords);
  else hipLaunchKernelGGL(compact_write_kernel, dim3(blocks), dim3(256), 0, s, d, nwords);
}

}  // namespace stgn
