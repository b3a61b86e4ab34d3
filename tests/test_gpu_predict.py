"""Parity of per-batch root-node inference and the linear link score (stgn_predict_batch, through
the C ABI) against the CPU oracle.  A score is a dot product of two embedding rows with the head's
weights: with rows within 1e-4 relative of the oracle's (the embedding bar), the score must satisfy
|y_g - y_r| <= 1e-4 (||h_u|| ||w_u|| + ||h_v|| ||w_v||) + 1e-6."""
import numpy as np
import pytest

from oracle import oracle as orc
from paper_2603_21090_amd import synth
from tests.helpers import tiny_workload

pytestmark = pytest.mark.gpu

REL = 1e-4


@pytest.fixture(scope="module")
def binding():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a device"
    from paper_2603_21090_amd import binding as b
    b.load_library()
    return b


def score_bound(o, w, wp, s, d):
    H = o.embed_all()[-1].astype(np.float64)
    de = w.d_emb
    return REL * (np.linalg.norm(H[s], axis=1) * np.linalg.norm(wp[:de]) +
                  np.linalg.norm(H[d], axis=1) * np.linalg.norm(wp[de:])) + 1e-6


@pytest.mark.parametrize("kw", [
    dict(layers=1, d_mem=16, d_edge=12, d_time=16, d_emb=16, d_msg=16, heads=2, k=4),
    dict(layers=2, d_mem=16, d_edge=12, d_time=16, d_emb=16, d_msg=16, heads=2, k=4),
    dict(layers=2, d_mem=0, d_node=12, d_edge=6, d_time=8, d_emb=16, heads=1, k=5),            # memoryless
    dict(layers=2, d_mem=100, d_edge=172, d_time=100, d_emb=100, d_msg=100, heads=2, k=10),    # the paper's widths
    # enough nodes for the regrouped row lists and the query cache (the roots read their q back)
    dict(layers=2, d_mem=16, d_edge=12, d_time=16, d_emb=16, d_msg=16, heads=2, k=4, num_nodes=40000, num_edges=2000, zipf_s=0.7),
    dict(layers=2, d_mem=0, d_node=12, d_edge=6, d_time=8, d_emb=16, heads=1, k=5, num_nodes=40000, num_edges=2000, zipf_s=0.7),
])
def test_scores_match_the_oracle_before_every_batch(binding, kw):
    import torch
    w = tiny_workload(**{**dict(num_nodes=300, num_edges=3000, batch=100, zipf_s=1.0), **kw})
    nf = synth.node_features(w)
    st = synth.EdgeStream(w)
    W = synth.make_weights(w)
    o = orc.Oracle.from_workload(w, W, nf)
    g = binding.StreamTGN.from_workload(w, W, nf)
    rng = np.random.default_rng(3)
    wp = (rng.standard_normal(2 * w.d_emb) / np.sqrt(w.d_emb)).astype(np.float32)
    g.set_predictor(wp, 0.125)
    allnodes = np.arange(w.num_nodes, dtype=np.uint32)
    for b in range(w.num_batches):
        s, d, t, ef = st.batch(b)
        if b % 5 == 0 or b == w.num_batches - 1:
            before = g.get_embeddings(allnodes)
            bound = score_bound(o, w, wp, s, d)
            for mode in (False, True):
                want = o.predict(s, d, t, wp, 0.125, at_edge_time=mode)
                got = g.predict_batch(s, d, t, at_edge_time=mode)
                assert (np.abs(got - want) <= bound).all(), f"batch {b} mode {mode}: worst {np.abs(got - want).max():.3e}"
                dev = g.predict_batch(torch.from_numpy(s.astype(np.int32)).cuda(), torch.from_numpy(d.astype(np.int32)).cuda(),
                                      torch.from_numpy(t).cuda(), at_edge_time=mode)
                assert np.array_equal(dev.cpu().numpy(), got), "device inputs give the same bits as host inputs"
            assert np.array_equal(g.get_embeddings(allnodes), before), "prediction changed a cached row"
        assert o.ingest(s, d, t, ef)[0] == 0
        g.ingest_batch(s, d, t, ef)
    g.close()


@pytest.mark.parametrize("num_nodes,d_mem,d_node", [(200, 16, 0), (40000, 0, 12)])
def test_edge_time_mode_at_a_nodes_own_last_time_reproduces_the_cached_row_bit_for_bit(binding, num_nodes, d_mem, d_node):
    """The roots go through the same layer kernel as the cache refresh, only with the query time taken
    from the edge: asked at the node's own last-interaction time it must give the cached row's bits
    (the memoryless model of 40,000 nodes keeps a query cache, which its roots read)."""
    w = tiny_workload(num_nodes=num_nodes, num_edges=2000, batch=100, layers=2, k=4, d_mem=d_mem, d_node=d_node, d_edge=12,
                      d_time=16, d_emb=16, d_msg=16, heads=2)
    st = synth.EdgeStream(w)
    W = synth.make_weights(w)
    g = binding.StreamTGN.from_workload(w, W, synth.node_features(w))
    t_last = np.zeros(w.num_nodes)
    for b in range(10):
        s, d, t, ef = st.batch(b)
        g.ingest_batch(s, d, t, ef)
        np.maximum.at(t_last, s, t)
        np.maximum.at(t_last, d, t)
    nodes = np.arange(w.num_nodes, dtype=np.uint32)
    H = g.get_embeddings(nodes)
    for c in (0, 7, w.d_emb - 1):
        e = np.zeros(2 * w.d_emb, np.float32); e[c] = 1.0           # score = coordinate c of the source row
        g.set_predictor(e, 0.0)
        n = 100                                                      # max_batch
        for lo in range(0, min(w.num_nodes, 2000), n):
            u = nodes[lo:lo + n]
            got = g.predict_batch(u, np.roll(u, 1), t_last[lo:lo + n], at_edge_time=True)
            assert np.array_equal(got, H[u, c])
            assert np.array_equal(g.predict_batch(u, np.roll(u, 1), t_last[lo:lo + n]), H[u, c])
    g.close()


def test_predict_argument_errors_and_dead_rows(binding):
    import torch
    w = tiny_workload(num_nodes=50, num_edges=200, batch=40, d_mem=8, d_edge=6, d_time=8, d_emb=8, d_msg=8)
    st = synth.EdgeStream(w)
    g = binding.StreamTGN.from_workload(w, synth.make_weights(w))
    g.ingest_batch(*st.batch(0))
    s, d, t, _ = st.batch(1)
    with pytest.raises(binding.StgnError) as e:
        g.predict_batch(s, d, t)                                     # no head yet
    assert e.value.code == -1
    g.set_predictor(np.ones(2 * w.d_emb, np.float32), 0.0)
    assert len(g.predict_batch(s[:0], d[:0], t[:0])) == 0            # empty batch
    bad = s.copy(); bad[3] = w.num_nodes
    with pytest.raises(binding.StgnError) as e:
        g.predict_batch(bad, d, t)
    assert e.value.code == -2
    with pytest.raises(binding.StgnError) as e:
        g.predict_batch(np.zeros(41, np.uint32), np.ones(41, np.uint32), np.zeros(41))
    assert e.value.code == -5
    for mode in (False, True):                                       # device inputs: that edge alone gets NaN
        ref = g.predict_batch(s, d, t, at_edge_time=mode)
        dev = g.predict_batch(torch.from_numpy(bad.astype(np.int64).astype(np.int32)).cuda(),
                              torch.from_numpy(d.astype(np.int32)).cuda(), torch.from_numpy(t).cuda(), at_edge_time=mode)
        got = dev.cpu().numpy()
        assert np.isnan(got[3]) and np.array_equal(np.delete(got, 3), np.delete(ref, 3))
    g.sync()
    g.close()
