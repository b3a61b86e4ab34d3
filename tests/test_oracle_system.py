"""System-level pins of the oracle on tiny graphs: neighbour lists and affected sets by brute
force, the invariants of the paper's equivalence theorem, and an independent vectorised
PyTorch (fp64) evaluation of the memory update and of the layered embeddings."""
import math

import numpy as np
import pytest
import torch

from oracle import oracle as orc
from paper_2603_21090_amd import synth
from tests.helpers import brute_affected, brute_rings, tiny_workload


def stream_and_oracle(w, node_feat=None, weights=None):
    st = synth.EdgeStream(w)
    weights = synth.make_weights(w) if weights is None else weights
    return st, weights, orc.Oracle.from_workload(w, weights, node_feat)


# ------------------------------------------------------------------ neighbour lists, D, t_last

@pytest.mark.parametrize("k,batch", [(3, 20), (2, 50), (5, 7)])
def test_neighbour_lists_match_brute_force(k, batch):
    w = tiny_workload(k=k, batch=batch, num_nodes=25, num_edges=300, zipf_s=1.3)
    st, _, o = stream_and_oracle(w)
    for b in range(w.num_batches):
        s, d, t, ef = st.batch(b)
        rc, D, A = o.ingest(s, d, t, ef)
        assert rc == 0
        assert np.array_equal(D, np.unique(np.concatenate([s, d])))
        hi = min((b + 1) * batch, w.num_edges)
        rings = brute_rings(st.src, st.dst, hi, w.num_nodes, k)
        for v in range(w.num_nodes):
            nbr, eid, ts = o.neighbors(v)
            assert [(int(a), int(e)) for a, e in zip(nbr, eid)] == rings[v]
            assert np.array_equal(ts, st.ts[eid])
            _, tl = o.memory([v])
            inc = [e for e in range(hi) if st.src[e] == v or st.dst[e] == v]
            assert tl[0] == (st.ts[inc[-1]] if inc else 0.0)
            assert o.degree(v) == len(inc)


def test_hub_receiving_more_than_k_edges_in_one_batch_and_multi_edges():
    w = tiny_workload(k=3, num_nodes=6, layers=1)
    _, _, o = stream_and_oracle(w)
    src = np.array([0, 1, 0, 2, 0, 0, 3], dtype=np.uint32)
    dst = np.array([1, 0, 1, 0, 4, 5, 0], dtype=np.uint32)   # node 0 gets 7 entries, pair (0,1) three times
    ts = np.arange(1, 8, dtype=np.float64)
    rc, D, A = o.ingest(src, dst, ts, np.zeros((7, w.d_edge), np.float32))
    assert rc == 0
    nbr, eid, _ = o.neighbors(0)
    assert list(nbr) == [3, 5, 4] and list(eid) == [6, 5, 4]
    nbr, eid, _ = o.neighbors(1)
    assert list(nbr) == [0, 0, 0] and list(eid) == [2, 1, 0]


# ------------------------------------------------------------------ affected set

@pytest.mark.parametrize("layers,d_mem,d_node", [(1, 8, 0), (2, 8, 0), (3, 8, 0), (2, 0, 8)])
def test_affected_set_brute_force_and_theorem_invariants(layers, d_mem, d_node):
    w = tiny_workload(layers=layers, d_mem=d_mem, d_node=d_node, num_nodes=40, num_edges=360, batch=12, k=3,
                      zipf_s=0.9)
    nf = synth.node_features(w)
    st, _, o = stream_and_oracle(w, nf)
    before = o.embed_all()
    mem_before, _ = o.memory(np.arange(w.num_nodes)) if d_mem else (None, None)
    n_strict = 0
    for b in range(w.num_batches):
        s, d, t, ef = st.batch(b)
        rc, D, A = o.ingest(s, d, t, ef)
        assert rc == 0
        hi = (b + 1) * w.batch
        rings = brute_rings(st.src, st.dst, hi, w.num_nodes, w.k)
        # independent derivation (scan every ring instead of the logs)
        assert np.array_equal(A, brute_affected(rings, D, layers))
        # superset check: all-time undirected ball of radius `layers`
        adj = [set() for _ in range(w.num_nodes)]
        for e in range(hi):
            adj[int(st.src[e])].add(int(st.dst[e])); adj[int(st.dst[e])].add(int(st.src[e]))
        ball, fr = set(map(int, D)), set(map(int, D))
        for _ in range(layers):
            fr = set().union(*[adj[u] for u in fr]) - ball if fr else set()
            ball |= fr
        assert set(map(int, A)) <= ball
        # theorem: rows outside A are bit-identical to the previous full recompute;
        after = o.embed_all()
        changed = np.nonzero((after != before).any(axis=(0, 2)))[0]
        assert set(changed) <= set(map(int, A))
        inA = np.zeros(w.num_nodes, bool); inA[A] = True
        assert np.array_equal(after[:, ~inA], before[:, ~inA])
        if d_mem:   # generic weights: every affected node really changes (minimality)
            n_strict += int(set(changed) == set(map(int, A)))
            mem_after, _ = o.memory(np.arange(w.num_nodes))
            moved = np.nonzero((mem_after != mem_before).any(axis=1))[0]
            assert set(moved) <= set(map(int, D))          # memory changes only on V_direct
            mem_before = mem_after
        before = after
    if d_mem:
        assert n_strict == w.num_batches


def test_expanding_through_a_dirty_nodes_own_ring_misses_a_changed_row():
    """The other reading of the propagation rule -- a dirty node u dirties the members of ITS OWN ring --
    is not sound.  Hand-built stream: w meets hub u once; u then meets k other nodes, so w has left u's
    ring while u is still the only entry of w's ring.  A batch that touches u changes u's memory, hence
    w's row (w attends to u), but walking u's own ring never reaches w.  The rule the oracle follows
    (w is dirty when a changed node sits in w's ring) does."""
    k = 3
    w_ = tiny_workload(num_nodes=10, k=k, layers=1)
    _, _, o = stream_and_oracle(w_)
    u, wn, y = 0, 1, 9
    others = [2, 3, 4]
    ef = lambda n: np.full((n, w_.d_edge), 0.25, np.float32)
    assert o.ingest(np.array([wn], np.uint32), np.array([u], np.uint32), np.array([1.0]), ef(1))[0] == 0
    src = np.array(others, np.uint32)
    assert o.ingest(src, np.full(len(others), u, np.uint32), np.array([2.0, 3.0, 4.0]), ef(3))[0] == 0
    assert wn not in o.neighbors(u)[0] and list(o.neighbors(wn)[0]) == [u]
    before = o.embed_all()
    rc, D, A = o.ingest(np.array([u], np.uint32), np.array([y], np.uint32), np.array([5.0]), ef(1))
    assert rc == 0 and set(map(int, D)) == {u, y}
    after = o.embed_all()
    changed = set(np.nonzero((after != before).any(axis=(0, 2)))[0].tolist())
    assert wn in changed                                   # w's row moved ...
    own_ring_rule = set(map(int, D))
    for v in map(int, D):
        own_ring_rule |= set(map(int, o.neighbors(v)[0]))
    assert wn not in own_ring_rule                         # ... the own-ring walk leaves it outside
    assert changed <= set(map(int, A)) and wn in set(map(int, A))   # the reverse-membership rule covers it


def test_embed_nodes_recursion_equals_layered_table():
    w = tiny_workload(layers=2)
    st, _, o = stream_and_oracle(w)
    for b in range(6):
        o.ingest(*st.batch(b))
    allrows = o.embed_all()
    nodes = np.arange(w.num_nodes, dtype=np.uint32)
    assert np.array_equal(o.embed_nodes(nodes, 2), allrows[1])
    assert np.array_equal(o.embed_nodes(nodes, 1), allrows[0])


def test_validation_errors_leave_state_untouched():
    w = tiny_workload()
    st, _, o = stream_and_oracle(w)
    o.ingest(*st.batch(0))
    ref = o.embed_all()
    s, d, t, ef = [a.copy() for a in st.batch(1)]
    bad = s.copy(); bad[3] = w.num_nodes
    assert o.ingest(bad, d, t, ef)[0] == -2
    loop = d.copy(); loop[5] = s[5]
    assert o.ingest(s, loop, t, ef)[0] == -4
    tt = t.copy(); tt[7] = tt[6] - 1.0
    assert o.ingest(s, d, tt, ef)[0] == -3
    tt = t.copy(); tt[0] = st.ts[w.batch - 1] - 0.5         # earlier than the previous batch's end
    assert o.ingest(s, d, tt, ef)[0] == -3
    assert np.array_equal(o.embed_all(), ref)
    assert o.ingest(s, d, t, ef)[0] == 0


# ------------------------------------------------------------------ independent vectorised evaluation

def torch_phi(omega, phase, x):
    om = torch.tensor(omega, dtype=torch.float64)
    ph = torch.tensor(phase, dtype=torch.float64)
    return torch.cos(x[..., None] * om + ph) / math.sqrt(len(omega))


def torch_embed_all(w, W, rings, ts_all, efeat_all, H0, t_last, t_final=None, window=None):
    """Layered embeddings with padded neighbour tensors and library attention (fp64).  t_final: query
    times of the LAST layer (default: t_last, like every other layer).  window: entries older than
    (query time - window) are masked out."""
    N, k, H = w.num_nodes, w.k, w.heads
    nbr = torch.zeros((N, k), dtype=torch.long)
    eid = torch.zeros((N, k), dtype=torch.long)
    valid = torch.zeros((N, k), dtype=torch.bool)
    for v, r in enumerate(rings):
        for j, (u, e) in enumerate(r):
            nbr[v, j], eid[v, j], valid[v, j] = u, e, True
    tl = torch.tensor(t_last)
    dt = tl[:, None] - torch.tensor(ts_all)[eid]
    phi = torch_phi(W["omega"], W["phase"], dt)                                   # [N,k,dt]
    phi0 = torch_phi(W["omega"], W["phase"], torch.zeros(N, dtype=torch.float64))  # [N,dt]
    E = torch.tensor(efeat_all, dtype=torch.float64)[eid]                          # [N,k,de]
    Hprev = torch.tensor(H0, dtype=torch.float64)
    outs = []
    for l in range(w.layers):
        T = lambda a: torch.tensor(a[l], dtype=torch.float64)
        q = torch.cat([Hprev, phi0], 1) @ T(W["W_Q"])
        if t_final is not None and l == w.layers - 1:
            dt = torch.tensor(t_final)[:, None] - torch.tensor(ts_all)[eid]
            phi = torch_phi(W["omega"], W["phase"], dt)
        live = valid if window is None else valid & (dt <= window)
        z = torch.cat([Hprev[nbr], E, phi], 2)
        K, V = z @ T(W["W_K"]), z @ T(W["W_V"])
        dk = w.d_emb // H
        qh = q.reshape(N, H, 1, dk)
        Kh = K.reshape(N, k, H, dk).permute(0, 2, 1, 3)
        Vh = V.reshape(N, k, H, dk).permute(0, 2, 1, 3)
        mask = live[:, None, None, :].expand(N, H, 1, k).clone()
        empty = ~live.any(1)
        mask[empty] = True                                    # avoid NaN rows; zeroed below
        o = torch.nn.functional.scaled_dot_product_attention(qh, Kh, Vh, attn_mask=mask).reshape(N, w.d_emb)
        o[empty] = 0.0
        Hl = (o @ T(W["W_O"]) + T(W["b_O"])).to(torch.float32)   # stored rows are fp32
        outs.append(Hl.numpy())
        Hprev = Hl.to(torch.float64)
    return np.stack(outs)


@pytest.mark.parametrize("d_mem,d_node", [(8, 0), (0, 6), (8, 4)])
def test_full_pipeline_against_vectorised_torch(d_mem, d_node):
    w = tiny_workload(d_mem=d_mem, d_node=d_node, layers=2, heads=2, k=4, num_nodes=30, num_edges=240, batch=16)
    nf = synth.node_features(w)
    W = synth.make_weights(w)
    if d_mem:   # diagonal U_h lets the library GRU cell stand in for the printed GRU
        W["U_h"] = np.diag(np.diag(W["U_h"])).astype(np.float32)
    st, _, o = stream_and_oracle(w, nf, W)
    mem = np.zeros((w.num_nodes, d_mem), np.float32)
    t_last = np.zeros(w.num_nodes)
    if d_mem:
        cell = torch.nn.GRUCell(w.d_msg, d_mem, dtype=torch.float64)
        with torch.no_grad():
            cell.weight_ih.copy_(torch.tensor(np.concatenate([W["W_r"].T, W["W_z"].T, W["W_h"].T]), dtype=torch.float64))
            cell.weight_hh.copy_(torch.tensor(np.concatenate([W["U_r"].T, W["U_z"].T, W["U_h"].T]), dtype=torch.float64))
            cell.bias_ih.copy_(torch.tensor(np.concatenate([W["b_r"], W["b_z"], W["b_h"]]), dtype=torch.float64))
            cell.bias_hh.zero_()
    for b in range(w.num_batches):
        s, d, t, ef = st.batch(b)
        assert o.ingest(s, d, t, ef)[0] == 0
        if d_mem:
            # last incident edge of each endpoint, both roles, all from pre-batch state
            last = {}
            for i in range(len(s)):
                last[int(s[i])] = (i, int(d[i])); last[int(d[i])] = (i, int(s[i]))
            nodes = sorted(last)
            idx = [last[v][0] for v in nodes]
            oth = [last[v][1] for v in nodes]
            tt = torch.tensor(t[idx]) - torch.tensor(t_last[nodes])
            x = torch.cat([torch.tensor(mem[nodes], dtype=torch.float64), torch.tensor(mem[oth], dtype=torch.float64),
                           torch.tensor(ef[idx], dtype=torch.float64), torch_phi(W["omega"], W["phase"], tt)], 1)
            m = x @ torch.tensor(W["W_msg"], dtype=torch.float64) + torch.tensor(W["b_msg"], dtype=torch.float64)
            with torch.no_grad():
                new = cell(m, torch.tensor(mem[nodes], dtype=torch.float64)).to(torch.float32).numpy()
            mem[nodes] = new
        t_last[s] = t; t_last[d] = t     # ascending timestamps: the last write is the latest
        for i in range(len(s)):
            t_last[s[i]] = t[i]; t_last[d[i]] = t[i]
        if d_mem:
            got, gtl = o.memory(np.arange(w.num_nodes))
            assert np.array_equal(gtl, t_last)
            assert np.abs(got.astype(np.float64) - mem).max() <= 2e-7   # at most one fp32 ulp of drift
            mem = got.copy()                                         # follow the oracle's rounding
    hi = w.num_edges
    rings = brute_rings(st.src, st.dst, hi, w.num_nodes, w.k)
    H0 = np.concatenate([mem, nf if nf is not None else np.zeros((w.num_nodes, 0), np.float32)], 1)
    want = torch_embed_all(w, W, rings, st.ts, st.edge_features(0, hi), H0, t_last)
    got = o.embed_all()
    assert np.abs(got.astype(np.float64) - want).max() < 5e-7


# ------------------------------------------------------------------ temporal window of the neighbour cache

def _windowed(window, layers=2, d_mem=8):
    w = tiny_workload(d_mem=d_mem, layers=layers, heads=2, k=4, num_nodes=30, num_edges=240, batch=16, window=window)
    W = synth.make_weights(w)
    st, _, o = stream_and_oracle(w, None, W)
    for b in range(w.num_batches):
        assert o.ingest(*st.batch(b))[0] == 0
    return w, W, st, o


def test_window_special_cases():
    """A window wider than the stream changes nothing; a window narrower than every gap leaves a node
    only the entries that carry its own last timestamp (gap 0), i.e. exactly its latest edge here."""
    w0, W, st, o0 = _windowed(0.0)
    ref = o0.embed_all()
    assert np.array_equal(_windowed(1e9)[3].embed_all(), ref)
    # synthetic timestamps are strictly increasing: with a tiny window every node sees one entry, which is
    # what a ring of capacity k = 1 holds
    _, W1, st1, ot = _windowed(1e-9, layers=1)
    tiny = ot.embed_all()
    w1 = tiny_workload(d_mem=8, layers=1, heads=2, k=1, num_nodes=30, num_edges=240, batch=16)
    o1 = orc.Oracle.from_workload(w1, W1)
    for b in range(w1.num_batches):
        assert o1.ingest(*st1.batch(b))[0] == 0
    assert np.array_equal(tiny, o1.embed_all())
    assert not np.array_equal(tiny, _windowed(0.0, layers=1)[3].embed_all())


@pytest.mark.parametrize("window", [3.0, 12.0, 40.0])
def test_window_against_vectorised_torch(window):
    w, W, st, o = _windowed(window)
    nodes = np.arange(w.num_nodes, dtype=np.uint32)
    mem, t_last = o.memory(nodes)
    rings = brute_rings(st.src, st.dst, w.num_edges, w.num_nodes, w.k)
    want = torch_embed_all(w, W, rings, st.ts, st.edge_features(0, w.num_edges), mem, t_last, window=window)
    got = o.embed_all()
    assert np.abs(got.astype(np.float64) - want).max() < 5e-7
    full = torch_embed_all(w, W, rings, st.ts, st.edge_features(0, w.num_edges), mem, t_last)
    assert np.abs(want - full).max() > 1e-3, "this window expires nothing: the case tests nothing"


# ------------------------------------------------------------------ Mean / Sum message aggregation

def test_aggregators_coincide_when_every_node_has_one_message_per_batch():
    """Eq. agg_functions: with one edge per batch a node never has two messages, so the mean, the sum and
    the last message are the same vector."""
    ref = None
    for agg in (0, 1, 2):
        w = tiny_workload(d_mem=8, layers=1, num_nodes=30, num_edges=60, batch=1, aggregator=agg)
        st, _, o = stream_and_oracle(w)
        for b in range(w.num_batches):
            assert o.ingest(*st.batch(b))[0] == 0
        mem = o.memory(np.arange(w.num_nodes))[0]
        if ref is None:
            ref = mem
        assert np.array_equal(mem, ref)


@pytest.mark.parametrize("agg", [1, 2])
def test_mean_and_sum_aggregators_against_vectorised_torch(agg):
    """Every (edge, role) message from pre-batch state with a library matmul, summed per node with
    index_add (divided by the count for the mean), then the library GRU cell (diagonal U_h)."""
    w = tiny_workload(d_mem=8, layers=1, heads=2, k=4, num_nodes=12, num_edges=240, batch=16, zipf_s=1.3, aggregator=agg)
    W = synth.make_weights(w)
    W["U_h"] = np.diag(np.diag(W["U_h"])).astype(np.float32)
    st, _, o = stream_and_oracle(w, None, W)
    d_mem = w.d_mem
    mem = np.zeros((w.num_nodes, d_mem), np.float32)
    t_last = np.zeros(w.num_nodes)
    cell = torch.nn.GRUCell(w.d_msg, d_mem, dtype=torch.float64)
    with torch.no_grad():
        cell.weight_ih.copy_(torch.tensor(np.concatenate([W["W_r"].T, W["W_z"].T, W["W_h"].T]), dtype=torch.float64))
        cell.weight_hh.copy_(torch.tensor(np.concatenate([W["U_r"].T, W["U_z"].T, W["U_h"].T]), dtype=torch.float64))
        cell.bias_ih.copy_(torch.tensor(np.concatenate([W["b_r"], W["b_z"], W["b_h"]]), dtype=torch.float64))
        cell.bias_hh.zero_()
    multi = 0
    for b in range(w.num_batches):
        s, d, t, ef = st.batch(b)
        assert o.ingest(s, d, t, ef)[0] == 0
        self_ = np.concatenate([s, d]).astype(np.int64)            # one row per (edge, role)
        oth = np.concatenate([d, s]).astype(np.int64)
        idx = np.concatenate([np.arange(len(s)), np.arange(len(s))])
        T64 = lambda a: torch.tensor(a, dtype=torch.float64)
        x = torch.cat([T64(mem[self_]), T64(mem[oth]), T64(ef[idx]),
                       torch_phi(W["omega"], W["phase"], torch.tensor(t[idx]) - torch.tensor(t_last[self_]))], 1)
        m = x @ T64(W["W_msg"]) + T64(W["b_msg"])
        nodes, inv, cnt = np.unique(self_, return_inverse=True, return_counts=True)
        multi += int((cnt > 1).sum())
        acc = torch.zeros((len(nodes), w.d_msg), dtype=torch.float64).index_add_(0, torch.tensor(inv), m)
        if agg == 1:
            acc = acc / torch.tensor(cnt, dtype=torch.float64)[:, None]
        with torch.no_grad():
            new = cell(acc, T64(mem[nodes])).to(torch.float32).numpy()
        mem[nodes] = new
        for i in range(len(s)):
            t_last[s[i]] = t[i]; t_last[d[i]] = t[i]
        got = o.memory(np.arange(w.num_nodes))[0]
        assert np.abs(got.astype(np.float64) - mem).max() <= 5e-7
        mem = got.copy()                                             # follow the oracle's rounding
    assert multi > 50, "the stream has no node with several messages in one batch: the case tests nothing"


def test_vectorised_ring_table_matches_the_brute_force_lists():
    """`rings_matrix` (used by the full-size GPU tests) against the per-node Python lists."""
    from tests.helpers import affected_from_rings, rings_matrix
    w = tiny_workload(num_nodes=30, num_edges=500, k=4, zipf_s=1.2)
    st = synth.EdgeStream(w)
    for hi in (0, 1, 37, 500):
        nbr_m, eid_m, deg = rings_matrix(st.src, st.dst, hi, w.num_nodes, w.k)
        rings = brute_rings(st.src, st.dst, hi, w.num_nodes, w.k)
        for v in range(w.num_nodes):
            c = min(int(deg[v]), w.k)
            assert [(int(a), int(e)) for a, e in zip(nbr_m[v, :c], eid_m[v, :c])] == rings[v]
            assert (nbr_m[v, c:] == -1).all()
        D = np.unique(np.concatenate([st.src[max(hi - 20, 0):hi], st.dst[max(hi - 20, 0):hi]])).astype(np.uint32)
        if len(D):
            assert np.array_equal(affected_from_rings(nbr_m, D, 2), brute_affected(rings, D, 2))
