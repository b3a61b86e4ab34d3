// CPU ORACLE -- TEST INFRASTRUCTURE ONLY.
//
// A plain, single-threaded, full-recompute implementation of the TGN / TGAT
// forward pass and of the affected-set rule, written from the paper's equations.
// Nothing in the product path may include, link or call this file; only the
// tests, the smoke check and the benchmark's CPU-baseline leg do.  It shares no
// code, header, table or constant with the HIP library.
//
// Precision: parameters, edge features, node memory and every stored embedding
// row are fp32 (the precision the method stores its state in); all arithmetic on
// them is carried out in fp64 and rounded to fp32 once per stored row.
// Timestamps are fp64 throughout.
//
// What it follows (sections / equations of the paper):
//   time encoding ............ Sec. 2.2.1 (Stage 1: Time Encoding)
//   message .................. Eq. (msg), Eq. (msg_linear)
//   aggregation "Last" ....... Eq. (agg_functions)
//   GRU memory update ........ Eq. (gru_detail)
//   temporal attention ....... Eq. (emb_multihead), Eq. (attn_detail)
//   most-recent-k neighbours . Sec. 3.3.2 (Stage 1: Incremental Neighborhood Sampling)
//   affected set ............. Sec. 3.3.1, Eq. (affected_set); Theorem "Equivalence of
//                              Incremental Computation" is the property it must give
//   batching ................. Sec. 3.6.2 (pre-batch memory for all reads, one GRU
//                              transition per node per batch)
//   root inference + score ... Algorithm 1 (embed, predict, then update), Eq. (parallel_embed)
//   delta mode ............... Sec. 3.3 "Stage 4: Incremental Embedding Generation" (Eq. delta_embedding, the
//                              attention cache), Sec. 3.4 "Correctness of Incremental Computation" (delta mode);
//                              an approximation: the algorithm's steps in the paper's order
//   drift estimator, rebuild . Sec. 3.5 (Definition "Drift Estimator", Eq. global_drift, Eq. rebuild_trigger,
//                              partial / full rebuild)
//
// Pins (tests/test_oracle_*.py): closed forms for the time encoding and the GRU,
// library GRU cell and library scaled-dot-product attention as cross-checks,
// brute-force neighbour lists, brute-force affected set (row-by-row diff of two
// full recomputes, and an independent ring scan), hand-computed 2x2 GRU case.
// The numeric level of a whole embedding row is not printed anywhere in the
// paper: that part is "parity unpinned" by the paper and pinned only by the
// special cases and library cross-checks above.

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>

namespace {

struct Entry { uint32_t nbr; uint32_t eid; };

struct Layer {
  uint32_t d_in;
  std::vector<float> WQ, WK, WV, WO, bO;
};

// ---- delta mode (approximate; Sec. 3.3 Stage 4, "Delta embedding" and "Attention score caching")
// AttnCache of one (layer, node): per recent-neighbour entry the score, the weight currently in effect in
// the cached sums, and the part of the value that depends on the neighbour and the edge; per row the sums
// themselves.  The value of entry j is V_j = Vc_j + phi_j W_V[time rows]; the head output is kept as
// o_h = S_h + pb_h W_V,h[time rows] with S = sum_j a_j Vc_j and pb_h = sum_j a_{h,j} phi_j.
struct AttnRow {
  bool valid = false;
  std::vector<uint32_t> eid;            // the entries the row was built on, most recent first
  std::vector<double> s, a;             // [n x heads] scores, weights in effect
  std::vector<double> vc;               // [n x d_emb]
  std::vector<double> S, pb, Z, m;      // [d_emb], [heads x d_time], [heads], [heads] (softmax denominator and its reference score)
};
struct Delta {
  bool on = false;
  double gamma = 0.9;
  std::vector<std::vector<float>> H;            // [layers][N x d_emb] cached rows (fp32, as the method stores them)
  std::vector<std::vector<AttnRow>> ac;         // [layers][N]
  // drift estimator (Sec. 3.5): per node a running sum with lazy decay, globally their sum and the
  // size of the cumulative affected set since the last rebuild
  std::vector<double> dsum;
  std::vector<uint32_t> dlast;
  std::vector<char> seen;
  double G = 0.0;
  uint32_t count = 0, tau = 0;
  std::vector<float> last_frac;                 // per node: changed fraction in the last batch (final layer); -1 exact, -2 untouched
};

struct Oracle {
  Delta dl;
  double window = 0.0;               // T_w; <= 0: no expiry
  uint32_t aggregator = 0;           // 0 Last, 1 Mean, 2 Sum
  uint32_t N, d_mem, d_node, d_edge, d_time, d_emb, d_msg, k, heads, layers;
  std::vector<float> omega, phase;
  std::vector<float> W_msg, b_msg, W_z, U_z, b_z, W_r, U_r, b_r, W_h, U_h, b_h;
  std::vector<Layer> L;
  std::vector<float> xfeat;                 // N x d_node (zeros if none given)
  // raw state
  std::vector<uint32_t> src, dst;           // arrival order; eid = index
  std::vector<double> ts;
  std::vector<float> efeat;                 // E x d_edge
  std::vector<std::vector<Entry>> log;      // per node, arrival order
  std::vector<float> mem;                   // N x d_mem
  std::vector<double> t_last;               // N
  double t_stream = 0.0;                    // last ingested timestamp
  bool any_edge = false;
};

double sigmoid(double x) { return 1.0 / (1.0 + std::exp(-x)); }

// phi_i(x) = sqrt(1/d_t) * cos(omega_i * x + phase_i)    (Sec. 2.2.1; the printed
// cos/sin pairs are the instance omega_{2j}=omega_{2j+1}, phase = 0, -pi/2)
void time_encode(uint32_t d_time, const float* omega, const float* phase, double x, double* out) {
  const double scale = std::sqrt(1.0 / (double)d_time);
  for (uint32_t i = 0; i < d_time; ++i)
    out[i] = scale * std::cos((double)omega[i] * x + (double)phase[i]);
}

// y[n_out] = x[n_in] * W[n_in x n_out] (+ b)
void vecmat(const double* x, const float* W, const float* b, uint32_t n_in, uint32_t n_out, double* y) {
  for (uint32_t o = 0; o < n_out; ++o) {
    double acc = b ? (double)b[o] : 0.0;
    for (uint32_t i = 0; i < n_in; ++i) acc += x[i] * (double)W[(size_t)i * n_out + o];
    y[o] = acc;
  }
}

// Eq. (msg_linear): m = [s_self || s_other || e || phi(dt)] W_m + b_m
void message(const Oracle& o, const float* s_self, const float* s_other, const float* e, double dt, double* m) {
  std::vector<double> x(2 * o.d_mem + o.d_edge + o.d_time);
  size_t p = 0;
  for (uint32_t i = 0; i < o.d_mem; ++i) x[p++] = s_self[i];
  for (uint32_t i = 0; i < o.d_mem; ++i) x[p++] = s_other[i];
  for (uint32_t i = 0; i < o.d_edge; ++i) x[p++] = e[i];
  time_encode(o.d_time, o.omega.data(), o.phase.data(), dt, x.data() + p);
  vecmat(x.data(), o.W_msg.data(), o.b_msg.data(), (uint32_t)x.size(), o.d_msg, m);
}

// Eq. (gru_detail), reset gate applied inside the recurrent product U_h (r . s)
void gru(uint32_t d_msg, uint32_t d_mem,
         const float* W_z, const float* U_z, const float* b_z,
         const float* W_r, const float* U_r, const float* b_r,
         const float* W_h, const float* U_h, const float* b_h,
         const double* m, const double* s, double* s_new) {
  std::vector<double> a(d_mem), c(d_mem), z(d_mem), r(d_mem), rs(d_mem), cand(d_mem);
  vecmat(m, W_z, b_z, d_msg, d_mem, a.data());
  vecmat(s, U_z, nullptr, d_mem, d_mem, c.data());
  for (uint32_t i = 0; i < d_mem; ++i) z[i] = sigmoid(a[i] + c[i]);
  vecmat(m, W_r, b_r, d_msg, d_mem, a.data());
  vecmat(s, U_r, nullptr, d_mem, d_mem, c.data());
  for (uint32_t i = 0; i < d_mem; ++i) r[i] = sigmoid(a[i] + c[i]);
  for (uint32_t i = 0; i < d_mem; ++i) rs[i] = r[i] * s[i];
  vecmat(m, W_h, b_h, d_msg, d_mem, a.data());
  vecmat(rs.data(), U_h, nullptr, d_mem, d_mem, c.data());
  for (uint32_t i = 0; i < d_mem; ++i) cand[i] = std::tanh(a[i] + c[i]);
  for (uint32_t i = 0; i < d_mem; ++i) s_new[i] = (1.0 - z[i]) * cand[i] + z[i] * s[i];
}

// Eq. (attn_detail) for one target: q [d], K,V [n x d]; per head softmax of q.k/sqrt(d_k);
// heads concatenated, then W_O, b_O.  n == 0 gives b_O.
void attention(uint32_t d, uint32_t heads, uint32_t n, const double* q, const double* K, const double* V,
               const float* WO, const float* bO, double* out) {
  const uint32_t dk = d / heads;
  std::vector<double> o(d, 0.0), sc(n);
  for (uint32_t h = 0; h < heads; ++h) {
    if (n == 0) break;
    double mx = -INFINITY;
    for (uint32_t j = 0; j < n; ++j) {
      double acc = 0.0;
      for (uint32_t c = 0; c < dk; ++c) acc += q[h * dk + c] * K[(size_t)j * d + h * dk + c];
      sc[j] = acc / std::sqrt((double)dk);
      mx = std::max(mx, sc[j]);
    }
    double den = 0.0;
    for (uint32_t j = 0; j < n; ++j) { sc[j] = std::exp(sc[j] - mx); den += sc[j]; }
    for (uint32_t j = 0; j < n; ++j) {
      const double alpha = sc[j] / den;
      for (uint32_t c = 0; c < dk; ++c) o[h * dk + c] += alpha * V[(size_t)j * d + h * dk + c];
    }
  }
  vecmat(o.data(), WO, bO, d, d, out);
}

// most recent min(k, deg) entries of v, most recent first (Sec. 3.3.2)
std::vector<Entry> recent(const Oracle& o, uint32_t v) {
  const std::vector<Entry>& lg = o.log[v];
  std::vector<Entry> out;
  for (size_t i = lg.size(); i > 0 && out.size() < o.k; --i) out.push_back(lg[i - 1]);
  return out;
}

// is edge `eid` one of the most recent k entries of w's log?
bool held_by(const Oracle& o, uint32_t w, uint32_t eid) {
  const std::vector<Entry>& lg = o.log[w];
  size_t seen = 0;
  for (size_t i = lg.size(); i > 0 && seen < o.k; --i, ++seen)
    if (lg[i - 1].eid == eid) return true;
  return false;
}

// layer-0 row: [mem[v] || x[v]]
void h0_row(const Oracle& o, uint32_t v, float* row) {
  for (uint32_t i = 0; i < o.d_mem; ++i) row[i] = o.mem[(size_t)v * o.d_mem + i];
  for (uint32_t i = 0; i < o.d_node; ++i) row[o.d_mem + i] = o.xfeat[(size_t)v * o.d_node + i];
}

// One target row of layer l (1-based) at query time tq, given a callback that yields layer l-1 rows.
template <class PrevRow>
void embed_row_at(const Oracle& o, uint32_t l, uint32_t v, double tq, PrevRow prev, float* out_row) {
  const Layer& Ly = o.L[l - 1];
  const uint32_t din = Ly.d_in, d = o.d_emb, dt = o.d_time, de = o.d_edge;
  std::vector<double> qin(din + dt), q(d);
  std::vector<float> hrow(din);
  prev(v, hrow.data());
  for (uint32_t i = 0; i < din; ++i) qin[i] = hrow[i];
  time_encode(dt, o.omega.data(), o.phase.data(), 0.0, qin.data() + din);
  vecmat(qin.data(), Ly.WQ.data(), nullptr, din + dt, d, q.data());
  // the most recent entries, without those that fall outside the temporal window [tq - T_w, tq]
  std::vector<Entry> nb = recent(o, v);
  if (o.window > 0.0)
    nb.erase(std::remove_if(nb.begin(), nb.end(), [&](const Entry& e) { return tq - o.ts[e.eid] > o.window; }), nb.end());
  const uint32_t n = (uint32_t)nb.size();
  std::vector<double> K((size_t)n * d), V((size_t)n * d), z(din + de + dt);
  for (uint32_t j = 0; j < n; ++j) {
    prev(nb[j].nbr, hrow.data());
    for (uint32_t i = 0; i < din; ++i) z[i] = hrow[i];
    for (uint32_t i = 0; i < de; ++i) z[din + i] = o.efeat[(size_t)nb[j].eid * de + i];
    time_encode(dt, o.omega.data(), o.phase.data(), tq - o.ts[nb[j].eid], z.data() + din + de);
    vecmat(z.data(), Ly.WK.data(), nullptr, din + de + dt, d, K.data() + (size_t)j * d);
    vecmat(z.data(), Ly.WV.data(), nullptr, din + de + dt, d, V.data() + (size_t)j * d);
  }
  std::vector<double> res(d);
  attention(d, o.heads, n, q.data(), K.data(), V.data(), Ly.WO.data(), Ly.bO.data(), res.data());
  for (uint32_t i = 0; i < d; ++i) out_row[i] = (float)res[i];
}

// The row a refreshed cache holds: query time = time of the node's latest edge.
template <class PrevRow>
void embed_row(const Oracle& o, uint32_t l, uint32_t v, PrevRow prev, float* out_row) {
  embed_row_at(o, l, v, o.t_last[v], prev, out_row);
}

// ---------------------------------------------------------------------------------------------------
// Delta mode.  Layer l (1-based) reads the CACHED rows of layer l - 1 (layer 0: memory | features).

void delta_prev_row(const Oracle& o, uint32_t l, uint32_t u, float* row) {
  if (l == 1) { h0_row(o, u, row); return; }
  std::memcpy(row, &o.dl.H[l - 2][(size_t)u * o.d_emb], o.d_emb * sizeof(float));
}

// q of row v at layer l (Eq. attn_detail, query side [h_v || phi(0)] W_Q)
void delta_query(const Oracle& o, uint32_t l, uint32_t v, double* q) {
  const Layer& Ly = o.L[l - 1];
  std::vector<double> qin(Ly.d_in + o.d_time);
  std::vector<float> hrow(Ly.d_in);
  delta_prev_row(o, l, v, hrow.data());
  for (uint32_t i = 0; i < Ly.d_in; ++i) qin[i] = hrow[i];
  time_encode(o.d_time, o.omega.data(), o.phase.data(), 0.0, qin.data() + Ly.d_in);
  vecmat(qin.data(), Ly.WQ.data(), nullptr, Ly.d_in + o.d_time, o.d_emb, q);
}

// One entry (neighbour u, edge e) of row v at layer l, query time tq: per-head score, the neighbour|edge
// part of the value, and the time encoding of the gap.
void delta_entry(const Oracle& o, uint32_t l, const double* q, const Entry& en, double tq,
                 double* score, double* vc, double* phi) {
  const Layer& Ly = o.L[l - 1];
  const uint32_t din = Ly.d_in, d = o.d_emb, dt = o.d_time, de = o.d_edge, dk = d / o.heads;
  std::vector<double> z(din + de + dt), K(d);
  std::vector<float> hrow(din);
  delta_prev_row(o, l, en.nbr, hrow.data());
  for (uint32_t i = 0; i < din; ++i) z[i] = hrow[i];
  for (uint32_t i = 0; i < de; ++i) z[din + i] = o.efeat[(size_t)en.eid * de + i];
  time_encode(dt, o.omega.data(), o.phase.data(), tq - o.ts[en.eid], phi);
  for (uint32_t i = 0; i < dt; ++i) z[din + de + i] = phi[i];
  vecmat(z.data(), Ly.WK.data(), nullptr, din + de + dt, d, K.data());
  for (uint32_t h = 0; h < o.heads; ++h) {
    double acc = 0.0;
    for (uint32_t c = 0; c < dk; ++c) acc += q[h * dk + c] * K[h * dk + c];
    score[h] = acc / std::sqrt((double)dk);
  }
  vecmat(z.data(), Ly.WV.data(), nullptr, din + de, d, vc);       // node and edge rows of W_V only
}

// the cached row from the cached sums: o_h = S_h + pb_h W_V,h[time rows]; row = o W_O + b_O
void delta_emit(Oracle& o, uint32_t l, uint32_t v) {
  const Layer& Ly = o.L[l - 1];
  const AttnRow& r = o.dl.ac[l - 1][v];
  const uint32_t d = o.d_emb, dt = o.d_time, dk = d / o.heads, t0 = Ly.d_in + o.d_edge;
  std::vector<double> oh(r.S), res(d);
  for (uint32_t h = 0; h < o.heads; ++h)
    for (uint32_t c = 0; c < dk; ++c) {
      double acc = 0.0;
      for (uint32_t i = 0; i < dt; ++i) acc += r.pb[h * dt + i] * (double)Ly.WV[(size_t)(t0 + i) * d + h * dk + c];
      oh[h * dk + c] += acc;
    }
  vecmat(oh.data(), Ly.WO.data(), Ly.bO.data(), d, d, res.data());
  float* out = &o.dl.H[l - 1][(size_t)v * d];
  for (uint32_t i = 0; i < d; ++i) out[i] = (float)res[i];
}

// Exact recomputation of row v at layer l; refreshes its attention cache.
void delta_exact_row(Oracle& o, uint32_t l, uint32_t v) {
  const uint32_t d = o.d_emb, dt = o.d_time, H = o.heads, dk = d / H;
  const double tq = o.t_last[v];
  std::vector<Entry> nb = recent(o, v);
  if (o.window > 0.0)
    nb.erase(std::remove_if(nb.begin(), nb.end(), [&](const Entry& e) { return tq - o.ts[e.eid] > o.window; }), nb.end());
  const uint32_t n = (uint32_t)nb.size();
  AttnRow& r = o.dl.ac[l - 1][v];
  r.valid = true;
  r.eid.resize(n);
  r.s.assign((size_t)n * H, 0.0); r.a.assign((size_t)n * H, 0.0); r.vc.assign((size_t)n * d, 0.0);
  r.S.assign(d, 0.0); r.pb.assign((size_t)H * dt, 0.0); r.Z.assign(H, 0.0); r.m.assign(H, 0.0);
  std::vector<double> q(d), phi((size_t)n * dt);
  delta_query(o, l, v, q.data());
  for (uint32_t j = 0; j < n; ++j) {
    r.eid[j] = nb[j].eid;
    delta_entry(o, l, q.data(), nb[j], tq, &r.s[(size_t)j * H], &r.vc[(size_t)j * d], &phi[(size_t)j * dt]);
  }
  for (uint32_t h = 0; h < H && n; ++h) {
    double mx = -INFINITY;
    for (uint32_t j = 0; j < n; ++j) mx = std::max(mx, r.s[(size_t)j * H + h]);
    double den = 0.0;
    for (uint32_t j = 0; j < n; ++j) den += std::exp(r.s[(size_t)j * H + h] - mx);
    r.m[h] = mx; r.Z[h] = den;
    for (uint32_t j = 0; j < n; ++j) {
      const double a = std::exp(r.s[(size_t)j * H + h] - mx) / den;
      r.a[(size_t)j * H + h] = a;
      for (uint32_t c = 0; c < dk; ++c) r.S[h * dk + c] += a * r.vc[(size_t)j * d + h * dk + c];
      for (uint32_t i = 0; i < dt; ++i) r.pb[h * dt + i] += a * phi[(size_t)j * dt + i];
    }
  }
  delta_emit(o, l, v);
}

// Delta update of row v at layer l (Eq. delta_embedding, "updated neighbours"): the row itself, its query
// time and its entries are unchanged; entries whose neighbour's input row changed get a new score, a new
// weight from the updated denominator and a new value part, the other entries keep the weight they have.
// Returns the number of changed entries.
template <class Changed>
uint32_t delta_update_row(Oracle& o, uint32_t l, uint32_t v, Changed changed) {
  const uint32_t d = o.d_emb, dt = o.d_time, H = o.heads, dk = d / H;
  AttnRow& r = o.dl.ac[l - 1][v];
  const uint32_t n = (uint32_t)r.eid.size();
  const double tq = o.t_last[v];
  std::vector<double> q(d), sc(H), vc(d), phi(dt);
  delta_query(o, l, v, q.data());
  uint32_t nch = 0;
  for (uint32_t j = 0; j < n; ++j) {
    const uint32_t e = r.eid[j];
    const Entry en{o.src[e] == v ? o.dst[e] : o.src[e], e};
    if (!changed(en.nbr)) continue;
    ++nch;
    delta_entry(o, l, q.data(), en, tq, sc.data(), vc.data(), phi.data());
    for (uint32_t h = 0; h < H; ++h) {
      const double e_old = std::exp(r.s[(size_t)j * H + h] - r.m[h]), e_new = std::exp(sc[h] - r.m[h]);
      const double Zn = r.Z[h] - e_old + e_new;
      const double a_old = r.a[(size_t)j * H + h], a_new = e_new / Zn;
      for (uint32_t c = 0; c < dk; ++c)
        r.S[h * dk + c] += a_new * vc[h * dk + c] - a_old * r.vc[(size_t)j * d + h * dk + c];
      for (uint32_t i = 0; i < dt; ++i) r.pb[h * dt + i] += (a_new - a_old) * phi[i];
      r.s[(size_t)j * H + h] = sc[h];
      r.a[(size_t)j * H + h] = a_new;
      r.Z[h] = Zn;
    }
    for (uint32_t c = 0; c < d; ++c) r.vc[(size_t)j * d + c] = vc[c];
  }
  delta_emit(o, l, v);
  return nch;
}

double drift_now(const Delta& dl, uint32_t v) {
  return dl.seen[v] ? dl.dsum[v] * std::pow(dl.gamma, (double)(dl.tau - dl.dlast[v])) : 0.0;
}
void drift_set(Delta& dl, uint32_t v, double value) {
  const double old = drift_now(dl, v);
  if (!dl.seen[v]) { dl.seen[v] = 1; dl.count += 1; }
  dl.dsum[v] = value; dl.dlast[v] = dl.tau;
  dl.G += value - old;
}
void drift_reset_all(Delta& dl) {
  std::fill(dl.dsum.begin(), dl.dsum.end(), 0.0);
  std::fill(dl.seen.begin(), dl.seen.end(), 0);
  dl.G = 0.0; dl.count = 0;
}

// Refresh of the caches after a batch.  flag[v]: 0 untouched, 1 endpoint of the batch, h + 2 first reached
// by hop h.  Layer l recomputes the rows whose inputs changed (flags up to thr_l); of those, a row whose
// own input row or query time changed is recomputed exactly, the others take the delta update.
void delta_refresh(Oracle& o, const std::vector<uint32_t>& flag) {
  Delta& dl = o.dl;
  dl.tau += 1;
  dl.G *= dl.gamma;
  std::fill(dl.last_frac.begin(), dl.last_frac.end(), -2.0f);
  auto thr = [&](uint32_t l) { return o.d_mem ? l + 1 : l; };         // rows layer l (1-based) recomputes: flags 1 .. thr(l)
  for (uint32_t l = 1; l <= o.layers; ++l) {
    auto input_changed = [&](uint32_t u) {                             // u's layer-(l-1) row changed in this batch
      if (flag[u] == 0) return false;
      return l == 1 ? (o.d_mem != 0 && flag[u] == 1) : flag[u] <= thr(l - 1);
    };
    for (uint32_t v = 0; v < o.N; ++v) {
      if (flag[v] == 0 || flag[v] > thr(l)) continue;
      const bool exact = flag[v] == 1 || input_changed(v) || !dl.ac[l - 1][v].valid;
      if (exact) {
        delta_exact_row(o, l, v);
        if (l == o.layers) { drift_set(dl, v, 0.0); dl.last_frac[v] = -1.0f; }
      } else {
        const uint32_t n = (uint32_t)dl.ac[l - 1][v].eid.size();
        const uint32_t nch = delta_update_row(o, l, v, input_changed);
        if (l == o.layers) {
          const double frac = n ? (double)nch / (double)n : 0.0;
          drift_set(dl, v, drift_now(dl, v) + frac);
          dl.last_frac[v] = (float)frac;
        }
      }
    }
  }
}

void delta_rebuild_rows(Oracle& o, uint32_t n, const uint32_t* nodes) {
  for (uint32_t l = 1; l <= o.layers; ++l)
    for (uint32_t i = 0; i < n; ++i) delta_exact_row(o, l, nodes ? nodes[i] : i);
}

void copyf(std::vector<float>& dst, const float* src, size_t n) {
  dst.assign(n, 0.0f);
  if (src && n) std::memcpy(dst.data(), src, n * sizeof(float));
}

}  // namespace

extern "C" {

struct orc_config {
  uint32_t num_nodes, d_mem, d_node, d_edge, d_time, d_emb, d_msg, k, heads, layers;
  double window;     // temporal window T_w of the neighbour cache (Sec. 3.3.2, "Invalidate"); <= 0: none
  uint32_t aggregator;   // Eq. (agg_functions): 0 Last, 1 Mean, 2 Sum
  uint32_t reserved;
};

struct orc_weights {
  const float *omega, *phase;
  const float *W_msg, *b_msg;
  const float *W_z, *U_z, *b_z, *W_r, *U_r, *b_r, *W_h, *U_h, *b_h;
  const float *const *W_Q, *const *W_K, *const *W_V, *const *W_O, *const *b_O;
};

void* orc_create(const orc_config* c, const orc_weights* w, const float* node_feat) {
  if (!c || !w || c->heads == 0 || c->d_emb % c->heads != 0 || c->layers == 0 || c->k == 0) return nullptr;
  Oracle* o = new Oracle();
  o->N = c->num_nodes; o->d_mem = c->d_mem; o->d_node = c->d_node; o->d_edge = c->d_edge;
  o->d_time = c->d_time; o->d_emb = c->d_emb; o->d_msg = c->d_msg; o->k = c->k;
  o->heads = c->heads; o->layers = c->layers;
  o->window = c->window;
  if (c->aggregator > 2) { delete o; return nullptr; }
  o->aggregator = c->aggregator;
  copyf(o->omega, w->omega, o->d_time);
  copyf(o->phase, w->phase, o->d_time);
  if (o->d_mem) {
    const size_t kin = 2 * (size_t)o->d_mem + o->d_edge + o->d_time;
    copyf(o->W_msg, w->W_msg, kin * o->d_msg); copyf(o->b_msg, w->b_msg, o->d_msg);
    copyf(o->W_z, w->W_z, (size_t)o->d_msg * o->d_mem); copyf(o->U_z, w->U_z, (size_t)o->d_mem * o->d_mem); copyf(o->b_z, w->b_z, o->d_mem);
    copyf(o->W_r, w->W_r, (size_t)o->d_msg * o->d_mem); copyf(o->U_r, w->U_r, (size_t)o->d_mem * o->d_mem); copyf(o->b_r, w->b_r, o->d_mem);
    copyf(o->W_h, w->W_h, (size_t)o->d_msg * o->d_mem); copyf(o->U_h, w->U_h, (size_t)o->d_mem * o->d_mem); copyf(o->b_h, w->b_h, o->d_mem);
  }
  o->L.resize(o->layers);
  for (uint32_t l = 0; l < o->layers; ++l) {
    Layer& Ly = o->L[l];
    Ly.d_in = (l == 0) ? o->d_mem + o->d_node : o->d_emb;
    copyf(Ly.WQ, w->W_Q[l], (size_t)(Ly.d_in + o->d_time) * o->d_emb);
    copyf(Ly.WK, w->W_K[l], (size_t)(Ly.d_in + o->d_edge + o->d_time) * o->d_emb);
    copyf(Ly.WV, w->W_V[l], (size_t)(Ly.d_in + o->d_edge + o->d_time) * o->d_emb);
    copyf(Ly.WO, w->W_O[l], (size_t)o->d_emb * o->d_emb);
    copyf(Ly.bO, w->b_O[l], o->d_emb);
  }
  copyf(o->xfeat, node_feat, (size_t)o->N * o->d_node);
  o->log.resize(o->N);
  o->mem.assign((size_t)o->N * o->d_mem, 0.0f);   // s_v(0) = 0  (Sec. 2.2.4)
  o->t_last.assign(o->N, 0.0);
  return o;
}

void orc_destroy(void* h) { delete (Oracle*)h; }

// Error codes of orc_ingest (nothing is changed when one is returned).
enum { ORC_OK = 0, ORC_E_NODE = -2, ORC_E_TIME = -3, ORC_E_SELF = -4 };

// Apply one batch: memory update from pre-batch state, append, affected set.
// direct_out / affected_out: ascending node ids, capacity num_nodes each (nullable).
int orc_ingest(void* h, uint32_t n, const uint32_t* src, const uint32_t* dst, const double* ts,
               const float* ef, uint32_t* direct_out, uint32_t* n_direct,
               uint32_t* affected_out, uint32_t* n_affected) {
  Oracle& o = *(Oracle*)h;
  // 1. validate (chronological stream, Definition "Temporal Graph")
  double prev = o.any_edge ? o.t_stream : -INFINITY;
  for (uint32_t i = 0; i < n; ++i) {
    if (src[i] >= o.N || dst[i] >= o.N) return ORC_E_NODE;
    if (src[i] == dst[i]) return ORC_E_SELF;
    if (!(ts[i] >= prev)) return ORC_E_TIME;
    prev = ts[i];
  }
  // V_direct
  std::vector<char> isd(o.N, 0);
  for (uint32_t i = 0; i < n; ++i) { isd[src[i]] = 1; isd[dst[i]] = 1; }
  std::vector<uint32_t> D;
  for (uint32_t v = 0; v < o.N; ++v) if (isd[v]) D.push_back(v);

  // 2. messages for every edge and both roles from PRE-batch memory and t_last, aggregated per node
  //    (Eq. agg_functions: the message of the highest batch index, "Last"; or the mean / the sum of the
  //    node's messages, added in batch order), one GRU transition per node.
  if (o.d_mem) {
    std::vector<int64_t> last_edge(o.N, -1);
    std::vector<uint32_t> n_msg(D.size(), 0);
    std::vector<double> last_msg((size_t)D.size() * o.d_msg, 0.0);
    std::vector<uint32_t> slot_of(o.N, 0);
    for (size_t d = 0; d < D.size(); ++d) slot_of[D[d]] = (uint32_t)d;
    std::vector<double> m(o.d_msg);
    for (uint32_t i = 0; i < n; ++i) {
      for (int role = 0; role < 2; ++role) {
        const uint32_t self = role ? dst[i] : src[i], other = role ? src[i] : dst[i];
        message(o, &o.mem[(size_t)self * o.d_mem], &o.mem[(size_t)other * o.d_mem],
                ef + (size_t)i * o.d_edge, ts[i] - o.t_last[self], m.data());
        double* agg = &last_msg[(size_t)slot_of[self] * o.d_msg];
        n_msg[slot_of[self]] += 1;
        if (o.aggregator == 0) {
          if ((int64_t)i >= last_edge[self]) {
            last_edge[self] = i;
            std::copy(m.begin(), m.end(), agg);
          }
        } else {
          for (uint32_t c = 0; c < o.d_msg; ++c) agg[c] += m[c];
        }
      }
    }
    if (o.aggregator == 1)
      for (size_t d = 0; d < D.size(); ++d)
        for (uint32_t c = 0; c < o.d_msg; ++c) last_msg[d * o.d_msg + c] /= (double)n_msg[d];
    std::vector<float> new_mem((size_t)D.size() * o.d_mem);
    std::vector<double> s(o.d_mem), sn(o.d_mem);
    for (size_t d = 0; d < D.size(); ++d) {
      const uint32_t v = D[d];
      for (uint32_t i = 0; i < o.d_mem; ++i) s[i] = o.mem[(size_t)v * o.d_mem + i];
      gru(o.d_msg, o.d_mem, o.W_z.data(), o.U_z.data(), o.b_z.data(), o.W_r.data(), o.U_r.data(), o.b_r.data(),
          o.W_h.data(), o.U_h.data(), o.b_h.data(), &last_msg[d * o.d_msg], s.data(), sn.data());
      for (uint32_t i = 0; i < o.d_mem; ++i) new_mem[d * o.d_mem + i] = (float)sn[i];
    }
    for (size_t d = 0; d < D.size(); ++d)      // write only after every read
      std::copy(new_mem.begin() + d * o.d_mem, new_mem.begin() + (d + 1) * o.d_mem,
                o.mem.begin() + (size_t)D[d] * o.d_mem);
  }

  // 3. append in arrival order, source side first
  for (uint32_t i = 0; i < n; ++i) {
    const uint32_t eid = (uint32_t)o.src.size();
    o.src.push_back(src[i]); o.dst.push_back(dst[i]); o.ts.push_back(ts[i]);
    o.efeat.insert(o.efeat.end(), ef + (size_t)i * o.d_edge, ef + (size_t)(i + 1) * o.d_edge);
    o.log[src[i]].push_back({dst[i], eid});
    o.log[dst[i]].push_back({src[i], eid});
    o.t_last[src[i]] = ts[i];
    o.t_last[dst[i]] = ts[i];
  }
  if (n) { o.t_stream = ts[n - 1]; o.any_edge = true; }

  // 4. affected set from the post-batch logs.  w depends on u iff an edge between them is
  //    still among w's most recent k entries; a changed u therefore dirties exactly those w.
  std::vector<char> inA(o.N, 0);
  std::vector<uint32_t> flag(o.N, 0);                 // 1: endpoint, h + 2: first reached by hop h
  std::vector<uint32_t> frontier = D;
  for (uint32_t v : D) { inA[v] = 1; flag[v] = 1; }
  for (uint32_t hop = 0; hop < o.layers; ++hop) {
    std::vector<uint32_t> next;
    for (uint32_t u : frontier) {
      for (const Entry& en : o.log[u]) {
        const uint32_t w = en.nbr;
        if (inA[w]) continue;
        if (held_by(o, w, en.eid)) { inA[w] = 1; flag[w] = hop + 2; next.push_back(w); }
      }
    }
    frontier.swap(next);
  }
  if (o.dl.on) delta_refresh(o, flag);
  uint32_t na = 0;
  for (uint32_t v = 0; v < o.N; ++v) if (inA[v]) { if (affected_out) affected_out[na] = v; ++na; }
  if (n_affected) *n_affected = na;
  if (direct_out) std::copy(D.begin(), D.end(), direct_out);
  if (n_direct) *n_direct = (uint32_t)D.size();
  return ORC_OK;
}

// Full recompute, layer by layer over all nodes.  out: [layers][N][d_emb] fp32.
void orc_embed_all(void* h, float* out) {
  Oracle& o = *(Oracle*)h;
  const uint32_t d0 = o.d_mem + o.d_node;
  std::vector<float> H0((size_t)o.N * d0);
  for (uint32_t v = 0; v < o.N; ++v) h0_row(o, v, &H0[(size_t)v * d0]);
  const float* prev = H0.data();
  uint32_t dprev = d0;
  for (uint32_t l = 1; l <= o.layers; ++l) {
    float* cur = out + (size_t)(l - 1) * o.N * o.d_emb;
    for (uint32_t v = 0; v < o.N; ++v)
      embed_row(o, l, v, [&](uint32_t u, float* row) { std::memcpy(row, prev + (size_t)u * dprev, dprev * sizeof(float)); },
                cur + (size_t)v * o.d_emb);
    prev = cur; dprev = o.d_emb;
  }
}

// Final-layer rows of the given nodes by plain recursion (no table of all nodes).
static void embed_rec(const Oracle& o, uint32_t l, uint32_t v, float* row) {
  if (l == 0) { h0_row(o, v, row); return; }
  embed_row(o, l, v, [&](uint32_t u, float* r) { embed_rec(o, l - 1, u, r); }, row);
}
void orc_embed_nodes(void* h, uint32_t layer, uint32_t n, const uint32_t* nodes, float* out) {
  Oracle& o = *(Oracle*)h;
  for (uint32_t i = 0; i < n; ++i) embed_rec(o, layer, nodes[i], out + (size_t)i * o.d_emb);
}

// Per-batch root-node inference (Algorithm 1, "Link prediction"; Sec. 3.6.2, Eq. parallel_embed): for every
// edge (u, v, t) of a batch that has NOT been ingested yet, the embeddings of u and v from the current
// (pre-batch) state and the link score, which the paper's error analysis takes as a linear function of the
// concatenated embeddings:  y = [h_u || h_v] . w + b.
//   at_edge_time = 0: h = the refreshed cache row (query time = the node's latest edge);
//   at_edge_time = 1: the final layer is evaluated at the edge's own time t (time gaps t - t_j, query side
//                     phi(0)); the layers below it are the refreshed rows (layered snapshot).
// w: [2 d_emb] (source half first).  out: [n] fp64.
void orc_predict(void* h, uint32_t n, const uint32_t* src, const uint32_t* dst, const double* ts, int at_edge_time,
                 const float* w, float b, double* out) {
  Oracle& o = *(Oracle*)h;
  const uint32_t d = o.d_emb;
  std::vector<float> hu(d), hv(d);
  auto root = [&](uint32_t v, double t, float* row) {
    if (!at_edge_time) { embed_rec(o, o.layers, v, row); return; }
    embed_row_at(o, o.layers, v, t, [&](uint32_t u, float* r) { embed_rec(o, o.layers - 1, u, r); }, row);
  };
  for (uint32_t i = 0; i < n; ++i) {
    root(src[i], ts[i], hu.data());
    root(dst[i], ts[i], hv.data());
    double y = (double)b;
    for (uint32_t c = 0; c < d; ++c) y += (double)hu[c] * (double)w[c] + (double)hv[c] * (double)w[d + c];
    out[i] = y;
  }
}

// most recent <= k neighbours of `node`, most recent first; returns the count
uint32_t orc_neighbors(void* h, uint32_t node, uint32_t* nbr, uint32_t* eid, double* ts) {
  Oracle& o = *(Oracle*)h;
  const std::vector<Entry> r = recent(o, node);
  for (size_t j = 0; j < r.size(); ++j) { nbr[j] = r[j].nbr; eid[j] = r[j].eid; ts[j] = o.ts[r[j].eid]; }
  return (uint32_t)r.size();
}

uint32_t orc_degree(void* h, uint32_t node) { return (uint32_t)((Oracle*)h)->log[node].size(); }

void orc_memory(void* h, uint32_t n, const uint32_t* nodes, float* mem, double* t_last) {
  Oracle& o = *(Oracle*)h;
  for (uint32_t i = 0; i < n; ++i) {
    if (mem) for (uint32_t c = 0; c < o.d_mem; ++c) mem[(size_t)i * o.d_mem + c] = o.mem[(size_t)nodes[i] * o.d_mem + c];
    if (t_last) t_last[i] = o.t_last[nodes[i]];
  }
}

// test hook: overwrite memory rows / t_last (to start a unit case from a chosen state)
void orc_set_memory(void* h, uint32_t n, const uint32_t* nodes, const float* mem, const double* t_last) {
  Oracle& o = *(Oracle*)h;
  for (uint32_t i = 0; i < n; ++i) {
    if (mem) for (uint32_t c = 0; c < o.d_mem; ++c) o.mem[(size_t)nodes[i] * o.d_mem + c] = mem[(size_t)i * o.d_mem + c];
    if (t_last) o.t_last[nodes[i]] = t_last[i];
  }
}

// ---- the individual equations, exposed so that each can be pinned on its own ----

void orc_time_encode(uint32_t d_time, const float* omega, const float* phase, double x, double* out) {
  time_encode(d_time, omega, phase, x, out);
}

void orc_message(void* h, const float* s_self, const float* s_other, const float* e, double dt, double* m) {
  message(*(Oracle*)h, s_self, s_other, e, dt, m);
}

void orc_gru(uint32_t d_msg, uint32_t d_mem,
             const float* W_z, const float* U_z, const float* b_z,
             const float* W_r, const float* U_r, const float* b_r,
             const float* W_h, const float* U_h, const float* b_h,
             const double* m, const double* s, double* s_new) {
  gru(d_msg, d_mem, W_z, U_z, b_z, W_r, U_r, b_r, W_h, U_h, b_h, m, s, s_new);
}

void orc_attention(uint32_t d, uint32_t heads, uint32_t n, const double* q, const double* K, const double* V,
                   const float* WO, const float* bO, double* out) {
  attention(d, heads, n, q, K, V, WO, bO, out);
}

// ---- delta mode and drift-aware rebuild scheduling (approximate; see the header) ----

// Switches the delta mode on (gamma: decay of the drift estimator) and rebuilds every cache exactly.
void orc_delta_enable(void* h, double gamma) {
  Oracle& o = *(Oracle*)h;
  Delta& dl = o.dl;
  dl.on = true; dl.gamma = gamma;
  dl.H.assign(o.layers, std::vector<float>((size_t)o.N * o.d_emb, 0.0f));
  dl.ac.assign(o.layers, std::vector<AttnRow>(o.N));
  dl.dsum.assign(o.N, 0.0); dl.dlast.assign(o.N, 0); dl.seen.assign(o.N, 0); dl.last_frac.assign(o.N, -2.0f);
  dl.G = 0.0; dl.count = 0; dl.tau = 0;
  delta_rebuild_rows(o, o.N, nullptr);
}

// cached rows of the given nodes at a layer (1-based)
void orc_delta_rows(void* h, uint32_t layer, uint32_t n, const uint32_t* nodes, float* out) {
  Oracle& o = *(Oracle*)h;
  for (uint32_t i = 0; i < n; ++i)
    std::memcpy(out + (size_t)i * o.d_emb, &o.dl.H[layer - 1][(size_t)nodes[i] * o.d_emb], o.d_emb * sizeof(float));
}

// attention cache of one row: entry count; weights in effect [n x heads]; scores [n x heads] (nullable)
uint32_t orc_delta_attn(void* h, uint32_t layer, uint32_t v, double* a, double* s) {
  Oracle& o = *(Oracle*)h;
  const AttnRow& r = o.dl.ac[layer - 1][v];
  if (a) std::copy(r.a.begin(), r.a.end(), a);
  if (s) std::copy(r.s.begin(), r.s.end(), s);
  return (uint32_t)r.eid.size();
}

// per node: fraction of changed entries in the last batch at the final layer (-1: recomputed exactly, -2: untouched)
void orc_delta_last_fractions(void* h, float* out) {
  Oracle& o = *(Oracle*)h;
  std::copy(o.dl.last_frac.begin(), o.dl.last_frac.end(), out);
}

// drift estimator: the global metric (Eq. global_drift), the size of the cumulative affected set, and per node (nullable, [N])
void orc_drift_status(void* h, double* global, uint32_t* count, double* per_node) {
  Oracle& o = *(Oracle*)h;
  if (global) *global = o.dl.count ? o.dl.G / (double)o.dl.count : 0.0;
  if (count) *count = o.dl.count;
  if (per_node) for (uint32_t v = 0; v < o.N; ++v) per_node[v] = drift_now(o.dl, v);
}

// Adaptive rebuild policy (Eq. rebuild_trigger): nothing (0) while the global metric is at most delta_max;
// otherwise the nodes whose own estimate exceeds delta_max are recomputed exactly (1, partial rebuild) when
// they are fewer than alpha * N, else every row is (2, full rebuild); either way all estimators restart.
int orc_maintain(void* h, double delta_max, double alpha, uint32_t* n_drift) {
  Oracle& o = *(Oracle*)h;
  Delta& dl = o.dl;
  if (n_drift) *n_drift = 0;
  const double global = dl.count ? dl.G / (double)dl.count : 0.0;
  if (!(global > delta_max)) return 0;
  std::vector<uint32_t> drifted;
  for (uint32_t v = 0; v < o.N; ++v) if (drift_now(dl, v) > delta_max) drifted.push_back(v);
  if (n_drift) *n_drift = (uint32_t)drifted.size();
  int action;
  if ((double)drifted.size() < alpha * (double)o.N) { delta_rebuild_rows(o, (uint32_t)drifted.size(), drifted.data()); action = 1; }
  else { delta_rebuild_rows(o, o.N, nullptr); action = 2; }
  drift_reset_all(dl);
  return action;
}

void orc_delta_full_rebuild(void* h) {
  Oracle& o = *(Oracle*)h;
  delta_rebuild_rows(o, o.N, nullptr);
  drift_reset_all(o.dl);
}

}  // extern "C"
