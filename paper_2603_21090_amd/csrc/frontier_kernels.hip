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
//
// Direction.  Pushing costs one coalesced 8-byte read per entry of the frontier's logs plus a random
// 4-byte degree lookup each (a 64-byte sector from L2 or HBM).  When the frontier owns more log
// entries than half the node count -- every batch that touches a hub -- it is cheaper to PULL: every
// clean node with at least one edge walks the neighbour ids of its own ring (k sequential 4-byte
// reads) and asks whether any of them carries the frontier's flag (byte reads that hit L2).  Both
// give the same flags: u is in w's ring exactly when w's ring holds u.  The choice is made on the
// device from a running count of the frontier's log entries, identically by every workgroup.
#include "stgn_internal.h"
#include "compaction.h"

namespace stgn {

namespace {

constexpr uint32_t kPlanThreads = 256;
constexpr uint32_t kPlanWaves = kPlanThreads / 64;
constexpr uint32_t kRoundFlags = 256;      // flags one wave looks at per round (hop >= 1): 4 per lane
constexpr uint32_t kRoundList = 64;        // entries of D one wave looks at per round (hop 0)
constexpr uint32_t kMaxRounds = 16;        // rounds per chunk: a chunk costs one update of the item counter
constexpr uint32_t kPlanWavesWanted = 2048;

// Work items of hop `hop`: from the list D (hop 0) or from the flags that equal hop + 1.  Every wave
// plans whole chunks on its own -- no workgroup barrier anywhere: a first pass over the chunk counts
// its items (one counter update per chunk), a second pass writes them, the 64 lanes filling the
// items of up to 64 frontier nodes together so that a hub's thousands of items do not land on one lane.
// (wave-collective: every lane of the calling wave must be active)
__device__ inline bool pull_hop(const Dev& d, uint32_t hop) { return stripes_sum_wave(d, hop) >= (unsigned long long)(d.N / 2u); }
// pulled[hop]: bit 0 the hop ran in pull mode, bit 1 the frontier was large enough to prefer pulling
constexpr uint32_t kRanPull = 1u, kWantsPull = 2u;

__global__ __launch_bounds__(kPlanThreads) void plan_kernel(Dev d, uint32_t hop, uint32_t rounds) {
  __shared__ uint32_t s_off[kPlanWaves][64], s_v[kPlanWaves][64];
  BatchCtl* c = d.bc;
  if (c->skip || pull_hop(d, hop)) return;               // a pull hop needs no work items
  const uint32_t lane = threadIdx.x & 63u;
  const uint32_t wib = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const uint32_t gw = blockIdx.x * kPlanWaves + wib, nw = gridDim.x * kPlanWaves;
  const uint32_t span = hop == 0 ? c->nD : d.N;
  const uint32_t per_round = hop == 0 ? kRoundList : kRoundFlags;
  const uint32_t chunk = rounds * per_round;
  const uint32_t want = hop + 1u;
  uint32_t* my_off = s_off[wib];
  uint32_t* my_v = s_v[wib];
  for (uint32_t base0 = gw * chunk; base0 < span; base0 += nw * chunk) {
    // candidates of round r held by this lane: up to 4 (flags) or 1 (list)
    auto candidates = [&](uint32_t r, uint32_t (&v)[4]) {
      uint32_t n = 0;
      const uint32_t x0 = base0 + r * per_round;
      if (hop == 0) {
        if (x0 + lane < span) v[n++] = d.D[x0 + lane];
      } else {
        const uint32_t f0 = x0 + 4u * lane;
        if (f0 < d.N) {                                        // the flag array is padded to whole words
          const uint32_t m = *reinterpret_cast<const uint32_t*>(d.mark + f0);
#pragma unroll
          for (uint32_t j = 0; j < 4; ++j)
            if (((m >> (8 * j)) & 0xFFu) == want) v[n++] = f0 + j;
        }
      }
      return n;
    };
    // ---- pass 1: items and scanned entries of the chunk
    uint32_t items = 0;
    unsigned long long scanned = 0;
    for (uint32_t r = 0; r < rounds; ++r) {
      uint32_t v[4] = {0u, 0u, 0u, 0u};
      const uint32_t n = candidates(r, v);
      uint32_t dg[4];
#pragma unroll
      for (uint32_t j = 0; j < 4; ++j) dg[j] = d.deg[v[j]];     // independent loads (dummy node 0 past n)
#pragma unroll
      for (uint32_t j = 0; j < 4; ++j)
        if (j < n) { items += (dg[j] + kLogChunk - 1) / kLogChunk; scanned += dg[j]; }
    }
    for (int off = 32; off > 0; off >>= 1) { items += __shfl_xor(items, off); scanned += __shfl_xor(scanned, off); }
    if (items == 0) continue;                                  // wave-uniform
    uint32_t out = 0;
    if (lane == 0) {
      out = atomicAdd(&c->n_items[hop], items);
      atomicAdd(stripe(d, kScannedCounter, gw), scanned);
    }
    out = (uint32_t)__builtin_amdgcn_readfirstlane((int)out);
    // ---- pass 2: write the items, up to 64 frontier nodes per step
    for (uint32_t r = 0; r < rounds; ++r) {
      uint32_t v[4] = {0u, 0u, 0u, 0u};
      const uint32_t n = candidates(r, v);
      uint32_t dg[4];
#pragma unroll
      for (uint32_t j = 0; j < 4; ++j) dg[j] = d.deg[v[j]];
      const uint32_t nmax = hop == 0 ? 1u : 4u;
#pragma unroll
      for (uint32_t j = 0; j < 4; ++j) {
        if (j >= nmax) break;
        const bool have = j < n;
        if (!__any(have)) break;                               // lanes fill v[] from the front
        const uint32_t node = have ? v[j] : 0u;
        const uint32_t nch = have ? (dg[j] + kLogChunk - 1) / kLogChunk : 0u;
        const uint32_t incl = wave_incl_scan(nch);
        const uint32_t total = (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
        if (total == 0) continue;
        my_off[lane] = incl - nch;
        my_v[lane] = node;
        for (uint32_t i = lane; i < total; i += 64) {
          uint32_t lo = 0, hi = 63;                            // last lane whose offset is <= i
          while (lo < hi) {
            const uint32_t mid = (lo + hi + 1) >> 1;
            if (my_off[mid] <= i) lo = mid; else hi = mid - 1;
          }
          d.items[out + i] = ((uint64_t)my_v[lo] << 32) | (i - my_off[lo]);
        }
        out += total;
      }
    }
  }
}

// planned = 0: the host launched no plan kernel for this hop (its last look at the statistics said the
// hop pulls), so there are no work items and the hop pulls whatever the frontier's size: both modes
// flag the same nodes.
__global__ __launch_bounds__(256) void expand_kernel(Dev d, uint32_t hop, uint32_t planned) {
  __shared__ unsigned long long s_deg[4], s_scan[4];
  BatchCtl* c = d.bc;
  if (c->skip) return;
  const uint32_t lane = threadIdx.x & 63;
  const uint8_t value = (uint8_t)(hop + 2u);
  unsigned long long newdeg = 0;                 // log entries owned by the nodes this thread flags
  unsigned long long looked = 0;                 // ring slots a pull hop examined
  const bool wants_pull = pull_hop(d, hop);
  if (wants_pull || !planned) {
    // ---- pull: one clean node per lane
    const uint8_t want = (uint8_t)(hop + 1u);
    const uint32_t k = d.k;
    for (uint32_t w = blockIdx.x * blockDim.x + threadIdx.x; w < d.N; w += gridDim.x * blockDim.x) {
      if (d.mark[w] != 0) continue;
      const uint32_t dg = d.deg[w];
      if (dg == 0) continue;
      const uint32_t cnt = dg < k ? dg : k;      // a ring that is not full yet fills slots 0 .. deg - 1
      const uint32_t* nb = d.ring_nbr + (size_t)w * k;
      bool hit = false;
      for (uint32_t j0 = 0; j0 < cnt && !hit; j0 += 4) {
        uint32_t u[4];
#pragma unroll
        for (uint32_t j = 0; j < 4; ++j) u[j] = nb[j0 + j < cnt ? j0 + j : j0];
        uint8_t f[4];
#pragma unroll
        for (uint32_t j = 0; j < 4; ++j) f[j] = d.mark[u[j]];
        hit = f[0] == want || f[1] == want || f[2] == want || f[3] == want;
        looked += cnt - j0 < 4u ? cnt - j0 : 4u;
      }
      if (hit) { d.mark[w] = value; newdeg += dg; }
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) c->pulled[hop] = kRanPull | (wants_pull ? kWantsPull : 0u);
  } else {
    // ---- push: one wavefront per work item of the frontier's logs
    const uint32_t n_items = c->n_items[hop];
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
          const uint32_t dw = d.deg[w];
          if ((uint64_t)e.y + d.k >= dw && d.mark[w] == 0) { d.mark[w] = value; newdeg += dw; }   // may count a node twice
        }
      }
    }
  }
  // the next hop's frontier owns this many log entries: one counter update per workgroup
  for (int off = 32; off > 0; off >>= 1) { newdeg += __shfl_xor(newdeg, off); looked += __shfl_xor(looked, off); }
  if (lane == 0) { s_deg[threadIdx.x >> 6] = newdeg; s_scan[threadIdx.x >> 6] = looked; }
  __syncthreads();
  if (threadIdx.x == 0) {
    const unsigned long long tot = s_deg[0] + s_deg[1] + s_deg[2] + s_deg[3];
    if (tot) atomicAdd(stripe(d, hop + 1, blockIdx.x), tot);
    const unsigned long long sc = s_scan[0] + s_scan[1] + s_scan[2] + s_scan[3];
    if (sc) atomicAdd(stripe(d, kScannedCounter, blockIdx.x), sc);
  }
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
  // statistics: nodes first reached by hop h carry the flag h + 2
  for (uint32_t value = 2; value <= last_value; ++value) {
    const uint32_t reached = block_scan_256(bytes_equal(m, value), s, &excl);
    if (threadIdx.x == 0 && reached) atomicAdd(&d.bc->n_front[value - 1u], reached);
  }
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
  if (d.flags_kept && v0 < d.N) *reinterpret_cast<uint4*>(d.flags_kept + v0) = m;   // delta mode reads the batch's flags in the layer launches
  if (m.x | m.y | m.z | m.w) *reinterpret_cast<uint4*>(d.mark + v0) = make_uint4(0u, 0u, 0u, 0u);   // ready for the next batch
  if (blockIdx.x == gridDim.x - 1 && t == 0) finish_batch(d, total);
}

// Orders a layer's row list so that rows with equally many recent-neighbour entries sit together.  The
// attention kernel serves four rows per wave in lockstep and sixteen per workgroup, so a tile costs what
// its LONGEST row costs: on skewed graphs a tile of sixteen consecutive ids runs to nearly k entries while
// the mean row holds a few.  Within every window of 4,096 list positions the rows are regrouped by
// descending entry count min(deg, k) (a counting sort, stable: ids stay ascending inside a group, and the
// order is the same on every run); tiles cut from the regrouped list are homogeneous.  With the query cache
// the rows whose own input row changed in the batch (flag at most thr_in) come first, grouped the same way,
// then the others, and every tile of the window is marked: 1 when none of its rows changed.  A row's result
// does not depend on which rows share its tile, so only the cost changes.  grid.y = list.
constexpr uint32_t kBucketWindow = 4096;
constexpr uint32_t kMaxBins = 2 * 65;                        // entry counts 0 .. k, k <= 64; changed | unchanged input
struct BucketJob { const uint32_t* in; const uint32_t* count; uint32_t* out; uint32_t count_max; uint8_t* tile_clean; uint32_t thr_in; };
struct BucketJobs { BucketJob j[STGN_MAX_LAYERS]; };
__global__ __launch_bounds__(256) void bucket_rows_kernel(Dev d, BucketJobs jobs) {
  __shared__ uint32_t s[4];
  __shared__ uint32_t s_hist[kMaxBins], s_base[kMaxBins];
  __shared__ uint32_t s_changed[kBucketWindow / 16];
  const BucketJob job = jobs.j[blockIdx.y];
  uint32_t n = job.count_max;
  if (job.count) { const uint32_t c = *job.count; n = c < n ? c : n; }
  const uint32_t w0 = blockIdx.x * kBucketWindow;
  if (w0 >= n) return;
  const uint32_t t = threadIdx.x, p0 = w0 + t * 16u;
  const uint32_t nbk = d.k + 1u, nb = job.tile_clean ? 2u * nbk : nbk;
  if (t < nb) s_hist[t] = 0u;
  s_changed[t] = 0u;
  __syncthreads();
  uint32_t id[16], bin[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const uint32_t p = p0 + i;
    id[i] = p < n ? (job.in ? job.in[p] : p) : 0xFFFFFFFFu;
    uint32_t b = 0xFFFFu;                                    // no row
    if (p < n) {
      const uint32_t dg = d.deg[id[i]];
      b = d.k - (dg < d.k ? dg : d.k);                       // bin 0 = full rings: longest rows first
      if (job.tile_clean && d.flags_kept[id[i]] > job.thr_in) b += nbk;
    }
    bin[i] = b;
    if (b != 0xFFFFu) atomicAdd(&s_hist[b], 1u);
  }
  __syncthreads();
  if (t == 0) {
    uint32_t run = 0;
    for (uint32_t b = 0; b < nb; ++b) { s_base[b] = run; run += s_hist[b]; }
  }
  __syncthreads();
  for (uint32_t b = 0; b < nb; ++b) {
    if (s_hist[b] == 0u) continue;                           // the same for every thread
    uint32_t mine = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) mine += bin[i] == b ? 1u : 0u;
    uint32_t excl;
    block_scan_256(mine, s, &excl);
    uint32_t o = w0 + s_base[b] + excl;
#pragma unroll
    for (int i = 0; i < 16; ++i)
      if (bin[i] == b) {
        if (b < nbk) s_changed[(o - w0) >> 4] = 1u;          // (every writer stores the same value)
        job.out[o++] = id[i];
      }
  }
  if (job.tile_clean) {
    __syncthreads();
    if (p0 < n) job.tile_clean[p0 >> 4] = s_changed[t] ? 0 : 1;
  }
}

__global__ __launch_bounds__(256) void compact_small_kernel(Dev d, uint32_t last_value) {
  __shared__ uint32_t s[256];
  compact_small_block(d, last_value, blockIdx.x, gridDim.x, s);
}

}  // namespace

void launch_plan(const Dev& d, hipStream_t s, uint32_t hop) {
  const uint32_t span = hop == 0 ? 2 * d.max_batch : d.N;
  const uint32_t per_round = hop == 0 ? kRoundList : kRoundFlags;
  // as many waves as the span allows, up to kPlanWavesWanted; beyond that, more rounds per chunk
  uint32_t rounds = (span + per_round * kPlanWavesWanted - 1) / (per_round * kPlanWavesWanted);
  rounds = rounds < 1 ? 1 : rounds > kMaxRounds ? kMaxRounds : rounds;
  const uint32_t chunk = rounds * per_round;
  uint32_t blocks = ((span + chunk - 1) / chunk + kPlanWaves - 1) / kPlanWaves;
  if (blocks > 2048) blocks = 2048;
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(plan_kernel, dim3(blocks), dim3(kPlanThreads), 0, s, d, hop, rounds);
}

void launch_expand(const Dev& d, hipStream_t s, uint32_t hop, bool planned, hipEvent_t done) {
  // one wave per work item (push) or one lane per node (pull), grid-stride.  A node per lane four
  // times over: small graphs get few workgroups, which all find room at once beside another kernel's.
  uint64_t want = ((uint64_t)d.N + 63) / 64;
  uint32_t blocks = want > 4096 ? 4096u : (uint32_t)(want ? want : 1);
  launch_done(expand_kernel, dim3(blocks), dim3(256), 0, s, done, d, hop, planned ? 1u : 0u);
}

// the lists the layers of a batch (all_rows = false) or of a rebuild (true) walk, regrouped by entry count
void launch_bucket_rows(const Dev& d, hipStream_t s, bool all_rows) {
  BucketJobs jobs{};
  uint32_t nj = 0;
  if (all_rows) {
    jobs.j[nj++] = BucketJob{nullptr, nullptr, d.RS[0], d.N, nullptr, 0u};
  } else {
    for (uint32_t l = 0; l < d.layers; ++l) {
      if (l && d.RS[l] == d.RS[l - 1]) continue;             // the same list: ordered once (its copy is shared)
      // flags at or below thr_in: the owner's input row of this layer changed in the batch
      jobs.j[nj++] = BucketJob{d.R[l], &d.bc->nR[l], d.RS[l], d.N, d.tile_clean[l], d.d_mem ? l + 1u : l};
    }
  }
  const uint32_t blocks = (d.N + kBucketWindow - 1) / kBucketWindow;
  hipLaunchKernelGGL(bucket_rows_kernel, dim3(blocks, nj), dim3(256), 0, s, d, jobs);
}

bool compact_in_one(const Dev& d) { return (d.N + kFlagsPerBlock - 1) / kFlagsPerBlock <= kSmallBlocks; }

void launch_compact(const Dev& d, hipStream_t s, int phase) {
  const uint32_t blocks = (d.N + kFlagsPerBlock - 1) / kFlagsPerBlock;
  if (compact_in_one(d)) {
    if (phase == 0) hipLaunchKernelGGL(compact_small_kernel, dim3(blocks), dim3(256), 0, s, d, d.layers + 1u);
    return;
  }
  if (phase == 0) hipLaunchKernelGGL(compact_count_kernel, dim3(blocks), dim3(256), 0, s, d, d.layers + 1u);
  else hipLaunchKernelGGL(compact_write_kernel, dim3(blocks), dim3(256), 0, s, d);
}

}  // namespace stgn
