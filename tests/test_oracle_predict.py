"""Pins of the oracle's per-batch root-node inference and link score (Algorithm 1, "Link
prediction"; Sec. 3.6.2, Eq. parallel_embed): the linear score by closed-form special cases, the
cached-row mode against the layered table, the edge-time mode against its special case (edge time =
the node's own last time) and against an independent vectorised PyTorch evaluation."""
import numpy as np
import pytest

from oracle import oracle as orc
from paper_2603_21090_amd import synth
from tests.helpers import brute_rings, tiny_workload
from tests.test_oracle_system import torch_embed_all


def build(layers, d_mem=8, d_node=0, batches=10):
    w = tiny_workload(d_mem=d_mem, d_node=d_node, layers=layers, heads=2, k=4, num_nodes=40, num_edges=320, batch=16)
    nf = synth.node_features(w)
    W = synth.make_weights(w)
    st = synth.EdgeStream(w)
    o = orc.Oracle.from_workload(w, W, nf)
    for b in range(batches):
        assert o.ingest(*st.batch(b))[0] == 0
    return w, W, nf, st, o


@pytest.mark.parametrize("layers", [1, 2])
def test_score_is_the_linear_form_of_the_two_root_rows(layers):
    w, W, nf, st, o = build(layers)
    s, d, t, _ = st.batch(10)                       # the next batch: not ingested
    table = o.embed_all()[-1].astype(np.float64)
    zero = np.zeros(2 * w.d_emb, np.float32)
    # a one-hot weight picks one coordinate of the source (first half) or destination (second half) row
    for c in (0, 3, w.d_emb - 1):
        e = zero.copy(); e[c] = 1.0
        assert np.array_equal(o.predict(s, d, t, e, 0.0), table[s, c])
        e = zero.copy(); e[w.d_emb + c] = 1.0
        assert np.array_equal(o.predict(s, d, t, e, 0.0), table[d, c])
    # bias alone, and additivity in the weights
    assert np.array_equal(o.predict(s, d, t, zero, 0.75), np.full(len(s), 0.75))
    rng = np.random.default_rng(5)
    w1, w2 = rng.standard_normal(2 * w.d_emb).astype(np.float32), rng.standard_normal(2 * w.d_emb).astype(np.float32)
    # w1 + w2 is rounded to fp32 before the oracle sees it: use weights whose sum is exact
    w1 = np.round(w1 * 64) / 64; w2 = np.round(w2 * 64) / 64
    y = o.predict(s, d, t, (w1 + w2).astype(np.float32), 0.0)
    assert np.allclose(y, o.predict(s, d, t, w1.astype(np.float32), 0.0) + o.predict(s, d, t, w2.astype(np.float32), 0.0),
                       rtol=0, atol=1e-12)
    # prediction reads the state, it does not change it
    assert np.array_equal(o.embed_all()[-1].astype(np.float64), table)


@pytest.mark.parametrize("layers", [1, 2])
def test_edge_time_mode_at_the_nodes_own_last_time_is_the_cached_row(layers):
    w, W, nf, st, o = build(layers)
    nodes = np.arange(w.num_nodes, dtype=np.uint32)
    _, t_last = o.memory(nodes)
    rng = np.random.default_rng(7)
    wu = np.concatenate([rng.standard_normal(w.d_emb), np.zeros(w.d_emb)]).astype(np.float32)   # source half only
    other = np.roll(nodes, 1)
    got = o.predict(nodes, other, t_last, wu, 0.0, at_edge_time=True)
    want = o.predict(nodes, other, t_last, wu, 0.0, at_edge_time=False)
    assert np.array_equal(got, want)


@pytest.mark.parametrize("layers,d_mem,d_node", [(1, 8, 0), (2, 8, 0), (2, 0, 6)])
def test_edge_time_mode_against_vectorised_torch(layers, d_mem, d_node):
    w, W, nf, st, o = build(layers, d_mem, d_node)
    nodes = np.arange(w.num_nodes, dtype=np.uint32)
    mem, t_last = o.memory(nodes) if d_mem else (np.zeros((w.num_nodes, 0), np.float32), None)
    if t_last is None:
        t_last = np.zeros(w.num_nodes)
        for i in range(10 * w.batch):
            t_last[st.src[i]] = st.ts[i]; t_last[st.dst[i]] = st.ts[i]
    hi = 10 * w.batch
    rings = brute_rings(st.src, st.dst, hi, w.num_nodes, w.k)
    H0 = np.concatenate([mem, nf if nf is not None else np.zeros((w.num_nodes, 0), np.float32)], 1)
    s, d, t, _ = st.batch(10)
    rng = np.random.default_rng(11)
    wp = rng.standard_normal(2 * w.d_emb).astype(np.float32)
    got = o.predict(s, d, t, wp, 0.25, at_edge_time=True)
    for i in range(len(s)):
        tf = t_last.copy()
        tf[s[i]] = t[i]; tf[d[i]] = t[i]              # only the two roots' final-layer rows are read below
        H = torch_embed_all(w, W, rings, st.ts, st.edge_features(0, hi), H0, t_last, t_final=tf)[-1].astype(np.float64)
        want = H[s[i]] @ wp[:w.d_emb].astype(np.float64) + H[d[i]] @ wp[w.d_emb:].astype(np.float64) + 0.25
        assert abs(got[i] - want) <= 2e-6 * (1.0 + abs(want)), (i, got[i], want)
    # the edge time matters: the cached-row mode gives different scores for nodes whose last edge is older
    assert np.abs(got - o.predict(s, d, t, wp, 0.25, at_edge_time=False)).max() > 1e-4
