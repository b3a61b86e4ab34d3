"""The prediction entry point that allocates nothing (static device scratch) against the ordinary one:
same kernels, so the scores must agree bit for bit -- on two calls in a row, the second with a smaller
input, so that whatever the first call left in the shared scratch array would show."""
import numpy as np
import pytest

from paper_2603_21090_amd import synth
from tests.helpers import tiny_workload

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def binding():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a device"
    from paper_2603_21090_amd import binding as b
    b.load_library()
    return b


@pytest.mark.parametrize("kw", [
    dict(layers=2, d_mem=16, d_edge=12, d_time=16, d_emb=16, d_msg=16, heads=2, k=4),
    dict(layers=2, d_mem=100, d_edge=172, d_time=100, d_emb=100, d_msg=100, heads=2, k=10),    # the paper's widths
    dict(layers=2, d_mem=0, d_node=12, d_edge=6, d_time=8, d_emb=16, heads=1, k=5),            # memoryless
])
def test_static_scratch_prediction_matches_the_ordinary_entry_point(binding, kw):
    import torch
    w = tiny_workload(num_nodes=200, num_edges=2400, batch=120, zipf_s=1.0, **kw)
    st = synth.EdgeStream(w)
    g = binding.StreamTGN.from_workload(w, synth.make_weights(w), synth.node_features(w))
    rng = np.random.default_rng(9)
    g.set_predictor((rng.standard_normal(2 * w.d_emb) / np.sqrt(w.d_emb)).astype(np.float32), 0.125)
    for b in range(12):
        g.ingest_batch(*st.batch(b))
    g.sync()

    def dev(b, n):
        s, d, t, _ = st.batch(b)
        return (torch.from_numpy(s[:n].astype(np.int32)).cuda(), torch.from_numpy(d[:n].astype(np.int32)).cuda(),
                torch.from_numpy(t[:n] + 3.0).cuda())

    for mode in (True, False):
        big, small = dev(12, 120), dev(13, 37)           # second call smaller than the first
        torch.cuda.synchronize()
        for args in (big, small):
            want = g.predict_batch(*args, at_edge_time=mode)
            out = torch.full((args[0].shape[0],), float("nan"), dtype=torch.float32, device="cuda")
            got = g.predict_batch_static(*args, at_edge_time=mode, out=out)
            assert g.sync() == 0
            want, got = want.cpu().numpy(), got.cpu().numpy()
            assert np.isfinite(want).all()
            assert np.array_equal(got, want), f"mode {mode}, n {len(want)}: worst {np.abs(got - want).max():.3e}"
    # an id past the node count scores NaN, as in the ordinary call; the others are unaffected
    s, d, t = dev(14, 50)
    s2 = s.clone(); s2[7] = w.num_nodes + 5
    torch.cuda.synchronize()
    got = g.predict_batch_static(s2, d, t, at_edge_time=True).cpu().numpy()
    ref = g.predict_batch(s, d, t, at_edge_time=True).cpu().numpy()
    assert np.isnan(got[7]) and np.array_equal(np.delete(got, 7), np.delete(ref, 7))
    g.close()


def test_static_scratch_limit_is_enforced(binding):
    """More roots than the static array holds: a clear error, nothing enqueued."""
    import torch
    w = tiny_workload(num_nodes=64, num_edges=256, batch=64, layers=1, d_mem=8, d_edge=4, d_time=8, d_emb=256, d_msg=8,
                      heads=4, k=2)
    g = binding.StreamTGN.from_workload(w, synth.make_weights(w), max_batch=4096)
    g.set_predictor(np.zeros(2 * w.d_emb, np.float32), 0.0)
    n = 4096                                              # 2 n (4 + 8 + 4 * 256) bytes > 4 MiB
    z = torch.zeros(n, dtype=torch.int32, device="cuda")
    o = torch.ones(n, dtype=torch.int32, device="cuda")
    t = torch.zeros(n, dtype=torch.float64, device="cuda")
    rc = g.predict_batch_static(z, o, t, at_edge_time=True, check=False)
    assert rc == -5 and "static scratch" in g.last_error()
    ok = g.predict_batch_static(z[:100], o[:100], t[:100], at_edge_time=True)
    assert g.sync() == 0 and np.isfinite(ok.cpu().numpy()).all()
    g.close()
