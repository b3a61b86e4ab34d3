"""Pins of the oracle's delta mode (paper Sec. 3.3 "Stage 4: Incremental Embedding Generation",
Eq. delta_embedding and the attention cache; Sec. 3.4 "Correctness of Incremental Computation", delta mode)
and of its drift estimator and rebuild policy (Sec. 3.5).

The delta mode is an approximation, so its oracle is the algorithm step by step.  What pins it from
outside: a case in which the approximation is exact (neighbours are flagged as changed but their keys and
values are not), a hand-evaluated update of one changed neighbour written with NumPy from the weights,
the error bound that follows from the update rule against the exact oracle, an exact rebuild that must
land on the exact oracle's rows, and the estimator's definition evaluated by brute force."""
import numpy as np
import pytest

from oracle import oracle as orc
from paper_2603_21090_amd import synth
from tests.helpers import tiny_workload


def both(w, weights=None, gamma=0.9):
    st = synth.EdgeStream(w)
    W = synth.make_weights(w) if weights is None else weights
    nf = synth.node_features(w)
    exact, delta = orc.Oracle.from_workload(w, W, nf), orc.Oracle.from_workload(w, W, nf)
    delta.delta_enable(gamma)
    return st, W, exact, delta


def rel(a, b):
    return np.linalg.norm(a.astype(np.float64) - b, axis=-1) / (np.linalg.norm(b, axis=-1) + 1e-30)


@pytest.mark.parametrize("layers", [1, 2])
def test_delta_update_with_unchanged_keys_and_values_reproduces_the_exact_rows(layers):
    """With a saturated update gate the GRU returns the old memory: every endpoint is flagged as changed,
    rows around them take the delta update, but no key or value really moved -- the update must leave every
    row where the exact recomputation puts it."""
    w = tiny_workload(layers=layers, num_nodes=40, num_edges=400, batch=10, k=4)
    W = synth.make_weights(w)
    W["b_z"] = np.full_like(W["b_z"], 40.0)
    st, _, exact, delta = both(w, W)
    nodes = np.arange(w.num_nodes, dtype=np.uint32)
    n_delta = 0
    for b in range(w.num_batches):
        exact.ingest(*st.batch(b)); delta.ingest(*st.batch(b))
        n_delta += int((delta.delta_last_fractions() >= 0).sum())
        ref = exact.embed_all()
        for l in range(1, layers + 1):
            assert rel(delta.delta_rows(nodes, l), ref[l - 1]).max() < 1e-6, f"batch {b}, layer {l}"
    assert n_delta > 20                       # the delta update really ran


def test_one_changed_neighbour_hand_evaluated_and_within_the_error_bound():
    """One layer, one head.  Node v holds u1, u2, u3; a batch then touches u2 only.  NumPy evaluates the
    attention of v before the batch from the weights, then the update rule for the one changed entry: new
    score, new denominator Z' = Z - e_old + e_new, new weight e_new / Z', the other two weights as they
    were.  The oracle's delta row must be that row; and its distance from the exact row stays below
    (1 - a_old) * max ||V_unchanged|| * |1 - Z / Z'| * ||W_O||_2, the bound the update rule implies (the
    printed bound has the changed fraction |dN| / |N| in place of the unchanged attention mass)."""
    w = tiny_workload(layers=1, heads=1, num_nodes=12, k=4, d_mem=6, d_edge=3, d_time=4, d_emb=6, d_msg=6)
    W = synth.make_weights(w)
    nf = None
    exact, delta = orc.Oracle.from_workload(w, W, nf), orc.Oracle.from_workload(w, W, nf)
    rng = np.random.default_rng(3)
    v, u1, u2, u3, x = 0, 1, 2, 3, 9
    ef = lambda n: rng.standard_normal((n, w.d_edge)).astype(np.float32)
    first = (np.array([v, v, v, 5], np.uint32), np.array([u1, u2, u3, 6], np.uint32), np.array([1.0, 2.5, 4.0, 4.5]), ef(4))
    second = (np.array([7], np.uint32), np.array([8], np.uint32), np.array([6.0]), ef(1))       # moves memories a little first
    third = (np.array([u2], np.uint32), np.array([x], np.uint32), np.array([9.0]), ef(1))
    for o in (exact, delta):
        assert o.ingest(*first)[0] == 0
    delta.delta_enable(0.9)
    for o in (exact, delta):
        assert o.ingest(*second)[0] == 0

    d, dt, de, dm = w.d_emb, w.d_time, w.d_edge, w.d_mem
    WQ, WK, WV, WO, bO = [np.asarray(W[n][0], np.float64) for n in ("W_Q", "W_K", "W_V", "W_O", "b_O")]
    om, ph = W["omega"].astype(np.float64), W["phase"].astype(np.float64)
    phi = lambda x_: np.sqrt(1.0 / dt) * np.cos(om * x_ + ph)

    def attention_inputs(o):
        nbr, eid, ts = o.neighbors(v)
        mem, tl = o.memory(np.arange(w.num_nodes))
        q = np.concatenate([mem[v].astype(np.float64), phi(0.0)]) @ WQ
        Z = np.stack([np.concatenate([mem[u].astype(np.float64), first[3][int(e)].astype(np.float64), phi(tl[v] - t)])
                      for u, e, t in zip(nbr, eid, ts)])
        return nbr, q, Z @ WK, Z @ WV

    nbr0, q0, K0, V0 = attention_inputs(exact)
    assert list(nbr0) == [u3, u2, u1]
    s0 = K0 @ q0 / np.sqrt(d)
    m = s0.max(); e0 = np.exp(s0 - m); Zold = e0.sum(); a0 = e0 / Zold
    assert np.abs(delta.delta_attn(v)[0][:, 0] - a0).max() < 1e-12            # the cache after the exact refresh

    for o in (exact, delta):
        rc, D, A = o.ingest(*third)
        assert rc == 0 and v in A and v not in D
    nbr1, q1, K1, V1 = attention_inputs(exact)
    assert np.array_equal(nbr1, nbr0) and np.allclose(q1, q0) and np.allclose(K1[[0, 2]], K0[[0, 2]])
    assert np.abs(K1[1] - K0[1]).max() > 1e-4                                  # u2's memory really moved
    s_new = K1[1] @ q1 / np.sqrt(d)
    e_new = np.exp(s_new - m)
    Znew = Zold - e0[1] + e_new
    a_new = e_new / Znew
    o_delta = a0[0] * V1[0] + a_new * V1[1] + a0[2] * V1[2]
    want = o_delta @ WO + bO
    got = delta.delta_rows([v])[0].astype(np.float64)
    assert np.abs(got - want).max() < 1e-6 * np.abs(want).max() + 1e-7
    a_cache = delta.delta_attn(v)[0][:, 0]
    assert np.abs(a_cache - np.array([a0[0], a_new, a0[2]])).max() < 1e-12
    assert abs(a_cache.sum() - 1.0) > 1e-6                                     # the kept weights are not renormalised
    # against the exact row
    h_exact = exact.embed_nodes([v])[0].astype(np.float64)
    err = np.linalg.norm(got - h_exact)
    bound = (1.0 - a0[1]) * max(np.linalg.norm(V1[0]), np.linalg.norm(V1[2])) * abs(1.0 - Zold / Znew) * np.linalg.norm(WO, 2)
    assert 1e-9 < err <= bound * (1 + 1e-5) + 1e-6
    printed = (1.0 / 3.0) * np.linalg.norm(V1, axis=1).max() * abs(1.0 - Zold / Znew)   # Eq. delta_error as printed
    assert printed > 0


@pytest.mark.parametrize("d_mem,d_node", [(8, 0), (0, 8)])
def test_delta_rows_stay_near_the_exact_rows_and_a_rebuild_lands_on_them(d_mem, d_node):
    w = tiny_workload(layers=2, d_mem=d_mem, d_node=d_node, num_nodes=60, num_edges=900, batch=15, k=4, zipf_s=0.8)
    st, W, exact, delta = both(w)
    nodes = np.arange(w.num_nodes, dtype=np.uint32)
    worst, moved = 0.0, 0
    for b in range(w.num_batches):
        rc, D, A = exact.ingest(*st.batch(b))
        rc2, D2, A2 = delta.ingest(*st.batch(b))
        assert np.array_equal(A, A2)
        ref = exact.embed_all()[-1]
        got = delta.delta_rows(nodes)
        fr = delta.delta_last_fractions()
        outside = np.setdiff1d(nodes, A)
        assert (fr[outside] == -2).all() and (fr[D] == -1).all()              # untouched / recomputed exactly
        exact_rows = nodes[fr == -1]
        if d_mem == 0:
            # memoryless, layer 2: an endpoint's row is exact only if its neighbours' layer-1 rows are; they are
            # (layer-1 rows change on endpoints only, and those are recomputed exactly)
            assert rel(got[exact_rows], ref[exact_rows]).max() < 1e-6
        e = rel(got, ref)
        worst = max(worst, e.max()); moved += int((e > 1e-6).sum())
    assert moved > 0 and worst < 0.5          # an approximation, but not a different model
    delta.delta_full_rebuild()
    ref = exact.embed_all()
    for l in (1, 2):
        assert rel(delta.delta_rows(nodes, l), ref[l - 1]).max() < 1e-6
    g, c, per = delta.drift_status()
    assert g == 0.0 and c == 0 and not per.any()


def test_drift_estimator_by_brute_force_and_the_rebuild_policy():
    """Definition "Drift Estimator": delta_hat_v(tau) = sum_j (|dN_v^(j)| / |N_v|) gamma^(tau - j) over the
    batches since the node's row was last exact; global metric = mean over the cumulative affected set
    (Eq. global_drift); rebuild when it exceeds delta_max, partially when fewer than alpha * n nodes exceed
    it themselves (Sec. 3.5, "Adaptive Rebuild Policy")."""
    gamma, delta_max, alpha = 0.8, 0.12, 0.12
    w = tiny_workload(layers=2, num_nodes=50, num_edges=1000, batch=10, k=4, zipf_s=0.7)
    st, W, exact, delta = both(w, gamma=gamma)
    nodes = np.arange(w.num_nodes, dtype=np.uint32)
    events = [[] for _ in nodes]              # per node: (batch, fraction) since its last exact recomputation
    seen = np.zeros(w.num_nodes, bool)
    actions = []
    for b in range(w.num_batches):
        exact.ingest(*st.batch(b)); delta.ingest(*st.batch(b))
        tau = b + 1
        fr = delta.delta_last_fractions()
        for v in nodes:
            if fr[v] == -1:
                events[v] = []; seen[v] = True
            elif fr[v] >= 0:
                events[v].append((tau, float(fr[v]))); seen[v] = True
        want = np.array([sum(f * gamma ** (tau - j) for j, f in ev) for ev in events])
        g, c, per = delta.drift_status()
        assert np.abs(per - want).max() < 1e-6          # the fractions are read back as fp32
        assert c == int(seen.sum())
        assert abs(g - (want[seen].sum() / max(c, 1))) < 1e-6
        over = int((per > delta_max).sum())
        expect = 0 if not g > delta_max else (1 if over < alpha * w.num_nodes else 2)
        act, n_drift = delta.maintain(delta_max, alpha)
        assert act == expect and (act == 0 or n_drift == over)
        actions.append(act)
        if act:
            events = [[] for _ in nodes]; seen[:] = False
            g, c, per = delta.drift_status()
            assert g == 0.0 and c == 0 and not per.any()
            if act == 2:
                ref = exact.embed_all()[-1]
                assert rel(delta.delta_rows(nodes), ref).max() < 1e-6
    assert 1 in actions and 2 in actions      # both kinds of rebuild fired on this stream
