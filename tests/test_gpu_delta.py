"""Delta mode on the GPU against the oracle's delta mode (paper Sec. 3.3 "Stage 4: Incremental Embedding
Generation", Eq. delta_embedding; Sec. 3.5, drift estimator and adaptive rebuild policy).

The mode is an approximation, so parity is with the oracle taking the same steps: after every compared
batch the cached rows of every layer and node, the per-node drift estimates, the global metric and the
size of the cumulative affected set; the policy's decisions (none / partial / full) and the number of
drifted nodes; and the rows after each rebuild.  The oracle works in fp64 and stores rows in fp32, the
library keeps its sums in fp32, so rows are compared to the tolerance of the exact mode."""
import numpy as np
import pytest

from oracle import oracle as orc
from paper_2603_21090_amd import synth
from tests.helpers import rows_close, tiny_workload

pytestmark = pytest.mark.gpu

GAMMA = 0.9


@pytest.fixture(scope="module")
def binding():
    import torch
    assert torch.cuda.is_available()
    from paper_2603_21090_amd import binding as b
    b.load_library()
    return b


def compare(g, o, w, what):
    nodes = np.arange(w.num_nodes, dtype=np.uint32)
    for l in range(1, w.layers + 1):
        got, ref = g.get_embeddings(nodes, layer=l), o.delta_rows(nodes, l)
        ok = rows_close(got, ref, 1e-4)
        if not ok.all():
            bad = np.nonzero(~ok)[0]
            e = np.linalg.norm(got[bad].astype(np.float64) - ref[bad], axis=1) / (np.linalg.norm(ref[bad], axis=1) + 1e-30)
            raise AssertionError(f"{what}, layer {l}: {len(bad)} rows out of tolerance (first {bad[:5]}), worst rel {e.max():.3e}")
    gg, gc, gper = g.drift_status(per_node=True)
    og, oc, oper = o.drift_status()
    assert gc == oc, f"{what}: cumulative affected set {gc} vs {oc}"
    assert np.allclose(gper, oper, rtol=1e-4, atol=1e-6), f"{what}: per-node drift estimates"
    assert abs(gg - og) <= 1e-4 * abs(og) + 1e-6, f"{what}: global drift {gg} vs {og}"


def run(binding, w, delta_max, alpha, every=1, maintain_every=7, batches=None):
    st = synth.EdgeStream(w)
    W = synth.make_weights(w)
    nf = synth.node_features(w)
    g = binding.StreamTGN.from_workload(w, W, nf, delta_mode=1, drift_gamma=GAMMA)
    o = orc.Oracle.from_workload(w, W, nf)
    o.delta_enable(GAMMA)
    compare(g, o, w, "initial state")
    actions = {0: 0, 1: 0, 2: 0}
    n_delta_rows = 0
    nb = w.num_batches if batches is None else batches
    for b in range(nb):
        s, d, t, ef = st.batch(b)
        rc, D, A = o.ingest(s, d, t, ef)
        assert rc == 0
        g.ingest_batch(s, d, t, ef)
        assert np.array_equal(g.get_affected(), A), f"batch {b}"
        n_delta_rows += int((o.delta_last_fractions() >= 0).sum())
        if b % every == 0:
            compare(g, o, w, f"batch {b}")
        if b % maintain_every == maintain_every - 1:
            ga, gn = g.maintain(delta_max, alpha)
            oa, on = o.maintain(delta_max, alpha)
            assert (ga, gn) == (oa, on), f"batch {b}: policy decided {(ga, gn)}, oracle {(oa, on)}"
            actions[ga] += 1
            compare(g, o, w, f"after maintenance at batch {b} (action {ga})")
    return g, o, actions, n_delta_rows


@pytest.mark.parametrize("kw", [
    dict(layers=2, d_mem=16, d_edge=6, d_time=8, d_emb=16, d_msg=16, heads=2, k=4),
    dict(layers=3, d_mem=16, d_edge=6, d_time=8, d_emb=16, d_msg=16, heads=2, k=3),
    dict(layers=1, d_mem=8, d_edge=6, d_time=8, d_emb=8, d_msg=8, heads=2, k=3),
    dict(layers=2, d_mem=0, d_node=12, d_edge=6, d_time=8, d_emb=16, heads=2, k=5),           # memoryless
    dict(layers=2, d_mem=16, d_edge=0, d_time=8, d_emb=16, d_msg=16, heads=1, k=2),           # no edge features
    dict(layers=2, d_mem=100, d_edge=172, d_time=100, d_emb=100, d_msg=100, heads=2, k=10),   # the paper's widths
    dict(layers=2, d_mem=12, d_edge=9, d_time=70, d_emb=130, d_msg=16, heads=1, k=3),         # one wide head, two time slots
    dict(layers=2, d_mem=10, d_edge=7, d_time=6, d_emb=12, d_msg=9, heads=4, k=3),            # four heads
])
def test_delta_mode_follows_the_oracle_step_by_step(binding, kw):
    w = tiny_workload(num_nodes=600, num_edges=2400, batch=30, zipf_s=0.6, **kw)
    g, o, actions, n_delta_rows = run(binding, w, delta_max=0.12, alpha=0.12, every=1)
    if w.layers >= 2:
        assert n_delta_rows > 50, "the delta update hardly ran"
    # full rebuild: onto the exact rows, estimators at rest
    g.full_rebuild()
    o.delta_full_rebuild()
    compare(g, o, w, "after a full rebuild")
    nodes = np.arange(w.num_nodes, dtype=np.uint32)
    exact = o.embed_all()
    for l in range(1, w.layers + 1):
        assert rows_close(g.get_embeddings(nodes, layer=l), exact[l - 1], 1e-4).all()
    assert g.drift_status()[:2] == (0.0, 0)
    g.close()


def test_policy_takes_each_of_its_three_branches(binding):
    w = tiny_workload(num_nodes=300, num_edges=6000, batch=40, zipf_s=0.8, layers=2, d_mem=16, d_edge=6, d_time=8,
                      d_emb=16, d_msg=16, heads=2, k=5)
    seen = {0: 0, 1: 0, 2: 0}
    for delta_max, alpha in [(5.0, 0.5), (0.12, 0.9), (0.12, 0.01)]:
        g, o, actions, _ = run(binding, w, delta_max, alpha, every=5, maintain_every=5, batches=60)
        for a, c in actions.items():
            seen[a] += c
        g.close()
    assert seen[0] and seen[1] and seen[2], seen


def test_delta_mode_with_lists_longer_than_one_flag_fetch(binding):
    """k = 40: the kernel fetches the flags of 32 entries at a time, a hub's list takes two fetches."""
    w = tiny_workload(num_nodes=300, num_edges=3000, batch=40, zipf_s=1.2, layers=2, k=40, d_mem=8, d_edge=6, d_time=8,
                      d_emb=16, d_msg=8, heads=2)
    g, o, _, n_delta_rows = run(binding, w, delta_max=0.3, alpha=0.2, every=3)
    assert n_delta_rows > 50
    g.close()


def test_delta_mode_with_a_temporal_window(binding):
    w = tiny_workload(num_nodes=300, num_edges=3000, batch=40, layers=2, k=5, d_mem=16, d_edge=6, d_time=16, d_emb=16,
                      d_msg=16, heads=2, zipf_s=0.8, window=15.0)
    g, o, _, n_delta_rows = run(binding, w, delta_max=0.2, alpha=0.2, every=2)
    assert n_delta_rows > 50
    g.close()


def test_delta_mode_on_the_two_launch_compaction_and_regrouped_row_lists(binding):
    """More than 32 blocks of 4,096 flags: the flags are kept by the second compaction launch, and the row
    lists are regrouped by entry count."""
    w = tiny_workload(num_nodes=140000, num_edges=6000, batch=300, zipf_s=0.6, k=3, layers=2)
    st = synth.EdgeStream(w)
    W = synth.make_weights(w)
    g = binding.StreamTGN.from_workload(w, W, None, delta_mode=1, drift_gamma=GAMMA)
    o = orc.Oracle.from_workload(w, W, None)
    o.delta_enable(GAMMA)
    for b in range(w.num_batches):
        s, d, t, ef = st.batch(b)
        rc, D, A = o.ingest(s, d, t, ef)
        g.ingest_batch(s, d, t, ef)
        assert np.array_equal(g.get_affected(), A), f"batch {b}"
        if b % 5 == 4:
            compare(g, o, w, f"batch {b}")
    ga, gn = g.maintain(0.05, 0.5)
    assert (ga, gn) == o.maintain(0.05, 0.5)
    compare(g, o, w, "after maintenance")
    g.close()


def test_exact_mode_rejects_the_delta_calls(binding):
    w = tiny_workload()
    g = binding.StreamTGN.from_workload(w, synth.make_weights(w), None)
    with pytest.raises(binding.StgnError):
        g.drift_status()
    with pytest.raises(binding.StgnError):
        g.maintain(0.1, 0.1)
    g.close()
