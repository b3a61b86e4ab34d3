// Batch staging (validate + endpoint sort + dedupe + adjacency block allocation) and the apply
// step (append to the temporal adjacency, recent-neighbour rings, edge-feature table, memory
// commit).  Paper Sec. 3.2 "Edge Queue" and "Temporal Adjacency List", Sec. 3.3 "Stage 1:
// Incremental Neighborhood Sampling" (the neighbour cache) and "Stage 5: Incremental Memory Update"
// (adjacency append, in-place memory write-back).
#include "stgn_internal.h"
#include "mfma16.h"
#include "compaction.h"
#include "placement.h"

namespace stgn {

namespace {

constexpr int kSortThreads = 1024;   // largest workgroup of the staging kernel; small batches launch fewer waves

// orders the LDS traffic of one wave: what its lanes stored before is visible to its lanes after
__device__ inline void wave_sync_lds() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// One workgroup.  keys: (node << 32 | slot), slot = 2*i (source side) or 2*i + 1 (destination).
__global__ __launch_bounds__(kSortThreads) void place_kernel(Dev d) {
  __shared__ uint32_t s_buf[kSortThreads / 64];
  __shared__ uint32_t s_units;
  place_batch(d, s_buf, &s_units);
}

__global__ __launch_bounds__(kSortThreads) void stage_sort_kernel(Dev d, uint32_t n, const uint32_t* __restrict__ src,
                                                                  const uint32_t* __restrict__ dst,
                                                                  const double* __restrict__ ts, uint32_t P) {
  extern __shared__ uint64_t keys[];
  __shared__ uint32_t s_buf[kSortThreads / 64];
  __shared__ uint32_t s_err, s_nD;
  const uint32_t t = threadIdx.x;
  Ctrl* c = d.ctrl;
  BatchCtl* bc = d.bc;
  if (t == 0) s_err = 0xFFFFFFFFu;
  // the batch's striped counters start at zero (nothing else touches this parity's set now)
  if (t < kStripedCounters * kStripes) *stripe(d, t / kStripes, t % kStripes) = 0ull;
  __syncthreads();

  // ---- validation: first offending edge decides the code (ids, self loop, time order)
  const double t_prev_stream = c->t_stream;
  const bool have_prev = c->E > 0;
  for (uint32_t i = t; i < n; i += blockDim.x) {
    uint32_t code = 0;
    const uint32_t u = src[i], v = dst[i];
    const double ti = ts[i];
    if (u >= d.N || v >= d.N) code = 2;                       // STGN_E_NODE_OUT_OF_RANGE
    else if (u == v) code = 4;                                // STGN_E_SELF_LOOP
    else {
      bool ok;
      if (i > 0) ok = ti >= ts[i - 1];
      else ok = have_prev ? (ti >= t_prev_stream) : (ti == ti);
      if (!ok) code = 3;                                      // STGN_E_TIME_ORDER
    }
    if (code) atomicMin(&s_err, (i << 4) | code);
  }
  if (t == 0 && c->E + n > d.max_edges) atomicMin(&s_err, 6u);   // STGN_E_EDGE_CAPACITY
  __syncthreads();
  if (s_err != 0xFFFFFFFFu) {
    if (t == 0) {
      bc->skip = 1;
      if (c->err_code == 0) { c->err_code = -(int32_t)(s_err & 15u); c->err_batch = c->batch_seq; }
      c->batch_seq += 1;
      bc->n_edges = 0; bc->nD = 0; bc->scanned = 0;
      for (int h = 0; h < STGN_MAX_LAYERS + 2; ++h) bc->n_front[h] = 0;
      for (int h = 0; h < STGN_MAX_LAYERS + 1; ++h) { bc->n_items[h] = 0; bc->pulled[h] = 0; }
    }
    return;
  }

  // ---- keys + bitonic sort in LDS
  const uint32_t m = 2 * n;
  for (uint32_t s = t; s < P; s += blockDim.x) {
    uint64_t key = ~0ull;
    if (s < m) {
      const uint32_t node = (s & 1) ? dst[s >> 1] : src[s >> 1];
      key = ((uint64_t)node << 32) | s;
    }
    keys[s] = key;
  }
  __syncthreads();
  // Compare-exchange stage (k2, j): thread x owns the pair whose lower index is x with a zero bit
  // inserted at position log2 j.  For j <= 64 the 64 pairs of a wave lie in one aligned block of 128
  // keys, so those stages only need the wave's own LDS traffic ordered; a workgroup barrier is needed
  // only around the wider strides.
  const uint32_t nth = blockDim.x;
  for (uint32_t k2 = 2; k2 <= P; k2 <<= 1) {
    for (uint32_t j = k2 >> 1; j > 0; j >>= 1) {
      for (uint32_t x = t; x < (P >> 1); x += nth) {
        const uint32_t i = ((x & ~(j - 1)) << 1) | (x & (j - 1));
        const uint32_t ij = i + j;
        const bool up = (i & k2) == 0;
        const uint64_t a = keys[i], b = keys[ij];
        if ((a > b) == up) { keys[i] = b; keys[ij] = a; }
      }
      // the next stage (j / 2, or the first of the next k2, j' = k2) is wave-local iff its stride is <= 64
      // and so was this one
      const uint32_t jn = j > 1 ? (j >> 1) : k2;
      if (j <= 64 && jn <= 64) wave_sync_lds(); else __syncthreads();
    }
  }
  __syncthreads();

  // ---- segment heads -> D, seg_start
  const uint32_t ept = (P + nth - 1) / nth;   // contiguous elements per thread
  const uint32_t lo = t * ept, hi = min(lo + ept, m);
  uint32_t heads = 0;
  for (uint32_t i = lo; i < hi; ++i) {
    const uint32_t node = (uint32_t)(keys[i] >> 32);
    heads += (i == 0 || node != (uint32_t)(keys[i - 1] >> 32)) ? 1u : 0u;
  }
  uint32_t* totp = &s_nD;
  uint32_t excl = block_excl_scan(heads, s_buf, totp);
  const uint32_t nD = s_nD;
  {
    uint32_t dcur = excl;          // number of heads before element lo
    for (uint32_t i = lo; i < hi; ++i) {
      const uint64_t key = keys[i];
      const uint32_t node = (uint32_t)(key >> 32), slot = (uint32_t)key;
      if (i == 0 || node != (uint32_t)(keys[i - 1] >> 32)) {
        d.D[dcur] = node;
        d.seg_start[dcur] = i;
        ++dcur;
      }
      const uint32_t di = dcur - 1;
      d.slot_d[slot] = di;
      d.slot_sorted[i] = slot;
      if (i + 1 == m || (uint32_t)(keys[i + 1] >> 32) != node) d.last_slot[di] = slot;
    }
    if (t == 0) d.seg_start[nD] = m;
  }
  if (t == 0) {
    bc->skip = 0;
    c->batch_seq += 1;
    bc->n_edges = n;
    bc->nD = nD;
    bc->scanned = 0;
    for (int h = 0; h < STGN_MAX_LAYERS + 2; ++h) bc->n_front[h] = 0;
    for (int h = 0; h < STGN_MAX_LAYERS + 1; ++h) { bc->n_items[h] = 0; bc->pulled[h] = 0; }
    bc->n_front[0] = nD;
    bc->E_base = c->E;
    c->E += n;
    if (n) c->t_stream = ts[n - 1];
  }
}

__device__ inline uint64_t log_addr(const Dev& d, uint32_t node, uint32_t pos) {
  const uint32_t b = 31u - (uint32_t)__clz((int)((pos >> 3) + 1u));
  const uint32_t off = pos - kMinBlock * ((1u << b) - 1u);
  return (uint64_t)d.blk[(size_t)node * d.maxb + b] * kMinBlock + off;
}

// Cached key|value rows that do not come out of a layer kernel (see LayerDev):
//   per batch:  KV[0][v] = [memory'(v) | features(v)] [W_K | W_V](node rows of layer 0) for the batch's
//       endpoints v (their memory just changed; skipped without a memory), and for every layer l
//       KVE[l][e] = feat_e [W_K | W_V](edge rows of layer l) for the batch's edges e (not with raw edge rows:
//       those are copied by the appending workgroups of the launch);
//   all_nodes (initial state, full rebuild):  KV[0][v] for every node.
// One workgroup (four waves) per 16 rows and 128 of the 128 ks output columns: the rows go through
// LDS as the A operand, wave w computes the column tiles w and w + 4 of the workgroup's column group
// (these launches are small and latency-bound: more, shorter workgroups finish sooner).  `bid` / `nblk`
// are the workgroup's index and count among the workgroups that project.
constexpr uint32_t kProjRows = 16;
__device__ void project_rows(const Dev& d, const float* __restrict__ ef, uint32_t all_nodes, uint32_t bid, uint32_t nblk,
                             float* lds) {
  const BatchCtl* c = d.bc;
  const uint32_t nD = all_nodes ? d.N : (d.d_mem ? c->nD : 0u);
  const uint32_t nE = (all_nodes || !d.d_edge || d.es) ? 0u : c->n_edges;
  const uint64_t E0 = c->E_base;
  const uint32_t tD = (nD + kProjRows - 1) / kProjRows, tE = (nE + kProjRows - 1) / kProjRows;
  // work items: (row tile, column group); for all nodes one item per row tile, which takes every column group
  // in turn (the rows are staged once, with 16-byte loads)
  const uint32_t groups_per_item = all_nodes ? d.ks : 1u;
  const uint32_t ntiles = (tD + d.layers * tE) * (all_nodes ? 1u : d.ks);
  const uint32_t kmax = d.d0 > d.d_edge ? d.d0 : d.d_edge;
  const uint32_t lda = round_up(kmax, kGrpK) + 4;
  const uint32_t lane = threadIdx.x & 63u;
  const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const uint32_t a_off = a16_lane_off(lda);
  // operand padding must be finite: clear the tile once (one chunk of slack behind the last row)
  for (uint32_t x = threadIdx.x; x < kProjRows * lda + 4 * kGrpK; x += 256) lds[x] = 0.0f;
  __syncthreads();
  for (uint32_t item = bid; item < ntiles; item += nblk) {
    const uint32_t tile = all_nodes ? item : item / d.ks;
    uint32_t nt = all_nodes ? wave : wave + 8u * (item - tile * d.ks);
    const bool node_job = tile < tD;
    const uint32_t layer = node_job ? 0u : (tile - tD) / tE;
    const uint32_t r0 = (node_job ? tile : (tile - tD) - layer * tE) * kProjRows;
    const uint32_t nrows = node_job ? nD : nE;
    const uint32_t K = node_job ? d.d0 : d.d_edge;
    const float* W = node_job ? d.L[0].WKVn : d.L[layer].WKVe;
    float* out = node_job ? d.KV[0].base : d.KVE[layer].base;
    const uint32_t ck = chunks_of(K), gk = kCG * ck;
    Ops16<2> P;                                               // first weight chunk, requested ahead of the staging
    load_b16(W + (size_t)nt * gk * kGrpFloats, 0, P.b[0]);
    load_b16(W + (size_t)(nt + 4) * gk * kGrpFloats, 0, P.b[1]);
    // stage the rows (columns K .. lda keep zeros or finite leftovers of a wider job: they meet zero weights).
    // A batch endpoint's new memory is read from the batch's scratch rows: the write-back into the
    // memory table runs in the same launch.
    if (all_nodes) {
      // whole table rows (stride and row padding are multiples of four floats; padding columns are zero)
      const uint32_t q4 = round_up(K, 4u) >> 2;
      for (uint32_t x = threadIdx.x; x < kProjRows * q4; x += 256) {
        const uint32_t r = x / q4, q = x - r * q4;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (r0 + r < nrows) v = *reinterpret_cast<const float4*>(d.H[0].base + (size_t)(r0 + r) * d.H[0].ld + 4u * q);
        *reinterpret_cast<float4*>(lds + r * lda + 4u * q) = v;
      }
    } else
    for (uint32_t x = threadIdx.x; x < kProjRows * K; x += 256) {
      const uint32_t r = x / K, col = x - r * K;
      float v = 0.0f;
      if (r0 + r < nrows) {
        if (!node_job) v = ef[(size_t)(r0 + r) * d.d_edge + col];
        else if (all_nodes) v = d.H[0].base[(size_t)(r0 + r) * d.H[0].ld + col];
        else if (col < d.d_mem) v = d.mem_new[(size_t)(r0 + r) * d.d_mem + col];
        else v = d.H[0].base[(size_t)d.D[r0 + r] * d.H[0].ld + col];
      }
      lds[r * lda + col] = v;
    }
    __syncthreads();
    for (uint32_t cg = 0; cg < groups_per_item; ++cg, nt += 8u) {
      const float* const Bt[2] = {W + (size_t)nt * gk * kGrpFloats, W + (size_t)(nt + 4) * gk * kGrpFloats};
      if (cg) { load_b16(Bt[0], 0, P.b[0]); load_b16(Bt[1], 0, P.b[1]); }
      floatx4 acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
      mfma16_gemm_pre<2>(lds + a_off, ck, Bt, acc, P);
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const uint32_t col = (nt + 4 * t) * 16 + m16_col(lane);     // every column is written: padding columns get exact zeros
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const uint32_t row = r0 + m16_row(lane, r);
          if (row < nrows) {
            const size_t orow = node_job ? (size_t)(all_nodes ? row : d.D[row]) : (size_t)(E0 + row);
            out[orow * d.ld_kv + col] = acc[t][r];
          }
        }
      }
    }
    __syncthreads();
  }
}

size_t project_lds(const Dev& d) {
  const uint32_t kmax = d.d0 > d.d_edge ? d.d0 : d.d_edge;
  return ((size_t)kProjRows * (round_up(kmax, kGrpK) + 4) + 4 * kGrpK) * sizeof(float);
}

__global__ __launch_bounds__(256) void project_nodes_kernel(Dev d) {
  extern __shared__ __align__(16) float lds[];
  project_rows(d, nullptr, 1u, blockIdx.x, gridDim.x, lds);
}

// The first `proj_blocks` workgroups compute the batch's cached key|value rows (project_rows: the
// longer job, so it is dispatched first); the next `compact_blocks` compact the dirty flags when the
// propagation has already run in the front part (one-launch compaction of small flag arrays: it
// depends on the flags alone, not on the apply step); the others append the batch to the graph
// state.  No group reads what another writes.
__global__ __launch_bounds__(256) void apply_kernel(Dev d, const uint32_t* __restrict__ src,
                                                    const uint32_t* __restrict__ dst,
                                                    const double* __restrict__ ts, const float* __restrict__ ef,
                                                    uint32_t proj_blocks, uint32_t compact_blocks) {
  extern __shared__ __align__(16) float lds[];
  __shared__ uint32_t s_scan[256];
  const BatchCtl* c = d.bc;
  if (blockIdx.x >= proj_blocks && blockIdx.x < proj_blocks + compact_blocks) {
    // (also for a batch that failed validation: its flags are all clear and its lists come out empty)
    compact_small_block(d, d.layers + 1u, blockIdx.x - proj_blocks, compact_blocks, s_scan);
    return;
  }
  const uint32_t first = proj_blocks + compact_blocks;      // first workgroup of the append group
  const uint32_t tid = (blockIdx.x - first) * blockDim.x + threadIdx.x, nth = (gridDim.x - first) * blockDim.x;
  // Two flag arrays: the other one was last read by the previous batch's compaction and is seeded
  // next by the next batch's placement kernel, which waits for this kernel -- cleared here, skipped batch or not.
  if (blockIdx.x >= proj_blocks && d.mark_other != d.mark) {
    const uint32_t words = (uint32_t)(mark_bytes(d.N) / 16);
    for (uint32_t x = tid; x < words; x += nth) reinterpret_cast<uint4*>(d.mark_other)[x] = make_uint4(0u, 0u, 0u, 0u);
  }
  if (c->skip) return;
  if (blockIdx.x < proj_blocks) {
    project_rows(d, ef, 0u, blockIdx.x, proj_blocks, lds);
    return;
  }
  const uint32_t n = c->n_edges, nD = c->nD;
  const uint64_t E0 = c->E_base;

  // adjacency entries and ring slots, one thread per (edge, side)
  for (uint32_t s = tid; s < 2 * n; s += nth) {
    const uint32_t i = s >> 1;
    const uint32_t u = src[i], v = dst[i];
    const uint32_t node = (s & 1) ? v : u, other = (s & 1) ? u : v;
    const uint32_t pos = d.slot_pos[s], twin = d.slot_pos[s ^ 1];
    const uint32_t eid = (uint32_t)(E0 + i);
    const uint64_t a = log_addr(d, node, pos);
    d.pool_nt[a] = make_uint2(other, twin);
    d.pool_eid[a] = eid;
    // only the last k entries a node receives in this batch reach its ring (no slot is written twice)
    if ((uint64_t)pos + d.k >= d.deg_new[d.slot_d[s]]) {
      RingEntry r; r.nbr = other; r.eid = eid; r.t = ts[i];
      d.ring[(size_t)node * d.k + pos % d.k] = r;
      d.ring_nbr[(size_t)node * d.k + pos % d.k] = other;
    }
  }
  // per distinct endpoint: degree, last interaction time, dirty seed
  for (uint32_t x = tid; x < nD; x += nth) {
    const uint32_t v = d.D[x];
    d.deg[v] = d.deg_new[x];
    d.t_last[v] = ts[d.last_slot[x] >> 1];
    if (d.mark_other == d.mark) d.mark[v] = 1;
  }
  // in-place memory write-back (all reads of the old rows happened in the previous kernel)
  if (d.d_mem) {
    const uint32_t tot = nD * d.d_mem;
    for (uint32_t x = tid; x < tot; x += nth) {
      const uint32_t dd = x / d.d_mem, col = x - dd * d.d_mem;
      d.H[0].base[(size_t)d.D[dd] * d.H[0].ld + col] = d.mem_new[(size_t)dd * d.d_mem + col];
    }
  }
  // An edge's features live on in its cached key|value rows, written by the projecting workgroups of this
  // launch, or (narrow features) as the raw row padded with zeros to one slot; its time in the ring records.
  if (d.es) {
    float4* rows = reinterpret_cast<float4*>(d.KVE[0].base + (size_t)E0 * kSlot);
    for (uint32_t x = tid; x < n * (kSlot / 4); x += nth) {       // one 16-byte piece of a padded row per thread
      const uint32_t i = x / (kSlot / 4), col = 4u * (x - i * (kSlot / 4));
      const float* f = ef + (size_t)i * d.d_edge;
      float4 v;
      v.x = col < d.d_edge ? f[col] : 0.0f;
      v.y = col + 1 < d.d_edge ? f[col + 1] : 0.0f;
      v.z = col + 2 < d.d_edge ? f[col + 2] : 0.0f;
      v.w = col + 3 < d.d_edge ? f[col + 3] : 0.0f;
      rows[x] = v;
    }
  }
}

__global__ void zero_kernel(float* p, size_t n) {
  for (size_t x = (size_t)blockIdx.x * blockDim.x + threadIdx.x; x < n; x += (size_t)gridDim.x * blockDim.x) p[x] = 0.0f;
}

// initial state: zero memory, node features copied by the host afterwards, empty graph
__global__ void init_state_kernel(Dev d) {
  const size_t tid = (size_t)blockIdx.x * blockDim.x + threadIdx.x, nth = (size_t)gridDim.x * blockDim.x;
  for (size_t x = tid; x < (size_t)d.N; x += nth) { d.deg[x] = 0; d.t_last[x] = 0.0; }
  const size_t h0 = (size_t)d.N * d.H[0].ld;
  for (size_t x = tid; x < h0; x += nth) d.H[0].base[x] = 0.0f;
  const size_t nw = mark_bytes(d.N) / 4;
  for (size_t x = tid; x < nw; x += nth) { reinterpret_cast<uint32_t*>(d.mark_set[0])[x] = 0; reinterpret_cast<uint32_t*>(d.mark_set[1])[x] = 0; }
  const size_t nr = (size_t)d.N * d.k;
  for (size_t x = tid; x < nr; x += nth) { RingEntry r; r.nbr = 0; r.eid = 0; r.t = 0.0; d.ring[x] = r; d.ring_nbr[x] = 0; }
  for (size_t x = tid; x < (size_t)kStripedCounters * kStripes * kStripeWords; x += nth)
    for (int i = 0; i < kSets; ++i) d.stripes_set[i][x] = 0;
  for (size_t x = tid; x < kStatSlots; x += nth) d.gathered_slots[x] = 0;
  if (tid == 0) {
    Ctrl z = {};
    *d.ctrl = z;
  }
}

}  // namespace

void launch_stage_sort(const Dev& d, hipStream_t s, uint32_t n, const uint32_t* src, const uint32_t* dst,
                       const double* ts) {
  uint32_t P = 2;
  while (P < 2 * n) P <<= 1;
  // one thread per compared pair, within 256 .. 1024: idle waves would only lengthen the barriers
  uint32_t threads = P / 2;
  threads = threads < 256 ? 256 : threads > (uint32_t)kSortThreads ? (uint32_t)kSortThreads : threads;
  hipLaunchKernelGGL(stage_sort_kernel, dim3(1), dim3(threads), P * sizeof(uint64_t), s, d, n, src, dst, ts, P);
}

void launch_place(const Dev& d, hipStream_t s, uint32_t n, hipEvent_t done) {
  uint32_t threads = (2 * n + 63u) & ~63u;     // one endpoint slot per thread where the batch allows
  threads = threads < 64 ? 64 : threads > (uint32_t)kSortThreads ? (uint32_t)kSortThreads : threads;
  launch_done(place_kernel, dim3(1), dim3(threads), 0, s, done, d);
}

void launch_apply(const Dev& d, hipStream_t s, const uint32_t* src, const uint32_t* dst, const double* ts,
                  const float* ef, bool with_compaction, hipEvent_t done) {
  // sized for the largest section (memory rows of a full batch's endpoints), grid-stride inside
  uint32_t work = 2 * d.max_batch * (d.d_mem > 1 ? d.d_mem : 1);
  if (d.es && work < d.max_batch * (kSlot / 4)) work = d.max_batch * (kSlot / 4);
  uint32_t blocks = (work + 255) / 256;
  if (blocks > 2048) blocks = 2048;
  if (blocks < 1) blocks = 1;
  // workgroups that project: one per 16-row tile of the largest batch (endpoints, and edges per layer)
  const uint32_t per = (d.max_batch + kProjRows - 1) / kProjRows;
  uint32_t pblocks = ((d.d_mem ? 2 * per : 0) + (d.d_edge && !d.es ? d.layers * per : 0)) * d.ks;
  if (pblocks > 2048) pblocks = 2048;
  const uint32_t cblocks = with_compaction ? compact_blocks_of(d.N) : 0u;
  launch_done(apply_kernel, dim3(blocks + pblocks + cblocks), dim3(256), pblocks ? project_lds(d) : 0, s, done, d, src, dst,
              ts, ef, pblocks, cblocks);
}

void launch_project_nodes(const Dev& d, hipStream_t s) {
  uint64_t blocks = (uint64_t)((d.N + kProjRows - 1) / kProjRows);
  const uint32_t cap = 8u * (d.num_cu ? d.num_cu : 256u);
  if (blocks > cap) blocks = cap;
  hipLaunchKernelGGL(project_nodes_kernel, dim3((uint32_t)blocks), dim3(256), project_lds(d), s, d);
}

void launch_init_state(const Dev& d, hipStream_t s) {
  hipLaunchKernelGGL(init_state_kernel, dim3(2048), dim3(256), 0, s, d);
}

__global__ void noop_kernel() {}
void launch_noop(hipStream_t s) { hipLaunchKernelGGL(noop_kernel, dim3(1), dim3(64), 0, s); }

void launch_zero(float* p, size_t n, hipStream_t s) {
  hipLaunchKernelGGL(zero_kernel, dim3(2048), dim3(256), 0, s, p, n);
}

int setup_ingest_attributes(const Dev& d) {
  if (hipFuncSetAttribute((const void*)stage_sort_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                          2 * STGN_MAX_BATCH * (int)sizeof(uint64_t)) != hipSuccess) return -1;
  if (project_lds(d) + 1024 > kMaxLds) return -1;
  if (hipFuncSetAttribute((const void*)apply_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                          (int)project_lds(d)) != hipSuccess) return -1;
  return hipFuncSetAttribute((const void*)project_nodes_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                             (int)project_lds(d)) == hipSuccess ? 0 : -1;
}

}  // namespace stgn
