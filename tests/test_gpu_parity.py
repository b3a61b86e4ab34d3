"""Parity of the HIP path (through the C ABI) against the CPU oracle.

Integer results (batch endpoints, affected set, neighbour lists, degrees, adjacency history,
last-interaction times) must be bit-exact.  Memory rows and embedding rows must satisfy, per
row, ||g - r||_2 <= 1e-4 ||r||_2 + 1e-6 and the same in max-norm (r = oracle row, fp64
arithmetic rounded once to fp32; g = fp32 arithmetic on the GPU)."""
import numpy as np
import pytest

from oracle import oracle as orc
from paper_2603_21090_amd import synth
from tests.helpers import rows_close, tiny_workload

pytestmark = pytest.mark.gpu

REL = 1e-4


@pytest.fixture(scope="module")
def binding():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a device"
    from paper_2603_21090_amd import binding as b
    b.load_library()          # no fallback: a missing library fails here
    return b


def check_rows(got, ref, what):
    ok = rows_close(got, ref, REL)
    if not ok.all():
        bad = np.nonzero(~ok)[0]
        e = np.linalg.norm(got[bad].astype(np.float64) - ref[bad], axis=1) / (np.linalg.norm(ref[bad], axis=1) + 1e-30)
        raise AssertionError(f"{what}: {len(bad)} rows out of tolerance, worst rel {e.max():.3e} (row {bad[e.argmax()]})")


def check_neighbours(g, o, nodes):
    for v in nodes:
        gn, ge, gt = g.get_neighbors(v)
        on, oe, ot = o.neighbors(v)
        assert np.array_equal(gn, on) and np.array_equal(ge, oe) and np.array_equal(gt, ot), f"ring of node {v}"
        assert g.get_degree(v) == o.degree(v)


def run_stream(binding, w, *, batches=None, check_every=1, full_check_at=(), nodes_for_rings=None, node_feat=None,
               device_inputs=False, weights=None, ts_shift=0.0):
    import torch
    st = synth.EdgeStream(w)
    if ts_shift:
        st.ts = st.ts + ts_shift                 # the whole stream moved along the time axis (both sides read st)
    W = synth.make_weights(w) if weights is None else weights
    o = orc.Oracle.from_workload(w, W, node_feat)
    g = binding.StreamTGN.from_workload(w, W, node_feat)
    nb = w.num_batches if batches is None else batches
    allnodes = np.arange(w.num_nodes, dtype=np.uint32)
    for b in range(nb):
        s, d, t, ef = st.batch(b)
        rc, D, A = o.ingest(s, d, t, ef)
        assert rc == 0
        if device_inputs:
            args = (torch.from_numpy(s.astype(np.int32)).cuda(), torch.from_numpy(d.astype(np.int32)).cuda(),
                    torch.from_numpy(t).cuda(), torch.from_numpy(ef).cuda())
            stats = g.ingest_batch(*args, stats=True)
        else:
            stats = g.ingest_batch(s, d, t, ef, stats=True)
        assert stats["n_direct"] == len(D), f"batch {b}: |D| {stats['n_direct']} != {len(D)}"
        if b % check_every == 0 or b == nb - 1:
            assert np.array_equal(g.get_affected(), A), f"batch {b}: affected set differs"
        else:
            assert stats["n_affected"] == len(A), f"batch {b}: |A|"
        if b in full_check_at or b == nb - 1:
            if w.d_mem:
                gm, gt = g.get_memory(allnodes)
                om, ot = o.memory(allnodes)
                assert np.array_equal(gt, ot), f"batch {b}: t_last"
                check_rows(gm, om, f"batch {b}: memory")
            ref = o.embed_all()
            for l in range(1, w.layers + 1):
                check_rows(g.get_embeddings(allnodes, layer=l), ref[l - 1], f"batch {b}: layer {l}")
            check_neighbours(g, o, allnodes if nodes_for_rings is None else nodes_for_rings)
    return g, o, st


def test_c1_full_stream(binding):
    """Config 1 as specified: every batch's affected set, full state at ten checkpoints."""
    w = synth.WORKLOADS["C1"]
    g, o, st = run_stream(binding, w, full_check_at=set(range(0, 100, 10)))
    tot = g.totals()
    assert tot["edges"] == w.num_edges
    # adjacency history of the busiest node, in arrival order
    deg = np.bincount(np.concatenate([st.src, st.dst]), minlength=w.num_nodes)
    hub = int(deg.argmax())
    nbr, eid = g.get_history(hub)
    inc = np.nonzero((st.src == hub) | (st.dst == hub))[0]
    assert np.array_equal(eid, inc.astype(np.uint32))
    assert np.array_equal(nbr, np.where(st.src[inc] == hub, st.dst[inc], st.src[inc]))
    g.close()


@pytest.mark.parametrize("kw", [
    dict(layers=1, d_mem=8, d_edge=6, d_time=8, d_emb=8, d_msg=8, heads=2, k=3),
    dict(layers=2, d_mem=10, d_edge=7, d_time=6, d_emb=12, d_msg=9, heads=4, k=3),          # odd widths
    dict(layers=3, d_mem=33, d_edge=5, d_time=31, d_emb=66, d_msg=35, heads=2, k=4),          # ragged tiles
    dict(layers=2, d_mem=16, d_edge=0, d_time=8, d_emb=16, d_msg=16, heads=1, k=2),           # no edge features
    dict(layers=2, d_mem=0, d_node=12, d_edge=6, d_time=8, d_emb=16, heads=2, k=5),           # memoryless
    dict(layers=2, d_mem=8, d_node=5, d_edge=6, d_time=8, d_emb=16, d_msg=8, heads=2, k=3),   # memory + features
    dict(layers=2, d_mem=100, d_edge=172, d_time=100, d_emb=100, d_msg=100, heads=2, k=10),   # the paper's widths
    dict(layers=2, d_mem=0, d_node=100, d_edge=64, d_time=100, d_emb=100, heads=2, k=20),     # config-5 widths
    dict(layers=1, d_mem=136, d_edge=20, d_time=24, d_emb=32, d_msg=140, heads=2, k=3),       # wide memory: chunked GRU path
    dict(layers=2, d_mem=12, d_edge=9, d_time=70, d_emb=130, d_msg=16, heads=1, k=3),         # one wide head: three key slots rounded to four
    dict(layers=2, d_mem=0, d_node=20, d_edge=0, d_time=16, d_emb=140, heads=2, k=4),         # two slots per head, no edge features
    dict(layers=3, d_mem=16, d_edge=5, d_time=100, d_emb=100, d_msg=16, heads=1, k=3),        # one 100-wide head (two key slots), two time slots
    # edge features on both sides of one 64-float slot (kept as raw rows up to it, projected past it)
    dict(layers=2, d_mem=12, d_edge=64, d_time=20, d_emb=32, d_msg=12, heads=4, k=3),         # a full slot, four heads
    dict(layers=2, d_mem=0, d_node=10, d_edge=63, d_time=70, d_emb=16, heads=2, k=4),         # one float short of a slot, two time slots
    dict(layers=2, d_mem=0, d_node=10, d_edge=65, d_time=8, d_emb=16, heads=2, k=4),          # one float past a slot
    dict(layers=1, d_mem=8, d_edge=1, d_time=8, d_emb=8, d_msg=8, heads=1, k=3),              # a single feature
    dict(layers=2, d_mem=12, d_edge=40, d_time=100, d_emb=64, d_msg=12, heads=4, k=3),        # four heads and two time slots: no room for the edge slot in the LDS tiles
    # the first layer's tiles are much larger than the second's (74 KB against 50 KB of LDS per workgroup):
    # both layers launch one kernel variant, which must be allowed the larger of the two
    dict(layers=2, d_mem=0, d_node=512, d_edge=6, d_time=8, d_emb=100, heads=2, k=64),
])
def test_small_graphs_all_shapes(binding, kw):
    w = tiny_workload(num_nodes=150, num_edges=1500, batch=50, zipf_s=1.0, **kw)
    nf = synth.node_features(w)
    g, o, st = run_stream(binding, w, node_feat=nf, full_check_at=set(range(0, 30, 5)))
    g.close()


@pytest.mark.parametrize("shift", [1e7, 1e9])
@pytest.mark.parametrize("kw", [
    dict(layers=2, d_mem=16, d_edge=6, d_time=16, d_emb=16, d_msg=16, heads=2, k=4),
    dict(layers=2, d_mem=100, d_edge=172, d_time=100, d_emb=100, d_msg=100, heads=2, k=10),   # the paper's widths
])
def test_timestamps_of_large_magnitude(binding, kw, shift):
    """Every timestamp moved by 1e7 and by 1e9 (the paper's largest streams reach such values).  A node's
    first message then encodes a gap of that size (its last-interaction time starts at 0), where the
    argument omega * dt + phase only makes sense reduced in fp64; attention gaps stay differences of
    fp64 times.  Memory and both layers against the oracle, which evaluates cos of the fp64 argument."""
    w = tiny_workload(num_nodes=150, num_edges=1500, batch=50, zipf_s=1.0, **kw)
    g, o, st = run_stream(binding, w, full_check_at=set(range(0, 30, 5)), ts_shift=shift)
    assert st.ts[0] > 0.99 * shift
    g.close()


@pytest.mark.parametrize("kw", [
    dict(num_nodes=300, k=40),                                  # more ring slots than a tile stages ahead: staged inside the tile
    dict(num_nodes=300, k=70, d_mem=0, d_node=12),
    dict(num_nodes=40000, k=40),                                # regrouped row lists; no query cache at this k
    dict(num_nodes=40000, k=70),                                # more entries than the regrouping has bins for: plain lists
    dict(num_nodes=40000, k=70, d_mem=0, d_node=12),
    dict(num_nodes=40000, k=30, d_mem=0, d_node=12),            # regrouped lists and query cache with nearly full staging
])
def test_long_recent_neighbour_lists(binding, kw):
    """Recent-neighbour lists of 30 to 70 entries, filled by the hubs of a skewed stream, on both sides of
    the node count from which the row lists are regrouped."""
    w = tiny_workload(**{**dict(num_edges=3000, batch=100, zipf_s=1.2, layers=2, d_mem=8, d_edge=6, d_time=8, d_emb=16,
                                d_msg=8, heads=2), **kw})
    rng = np.random.default_rng(4)
    some = np.sort(rng.choice(w.num_nodes, 300, replace=False)).astype(np.uint32)
    g, o, st = run_stream(binding, w, node_feat=synth.node_features(w), full_check_at={3, 11, 19}, nodes_for_rings=some)
    deg = np.bincount(np.concatenate([st.src, st.dst]), minlength=w.num_nodes)
    assert (deg >= w.k).sum() >= 3, "no list was filled"
    g.full_rebuild()
    ref = o.embed_all()
    allnodes = np.arange(w.num_nodes, dtype=np.uint32)
    for l in range(1, w.layers + 1):
        check_rows(g.get_embeddings(allnodes, layer=l), ref[l - 1], f"after a rebuild: layer {l}")
    g.close()


@pytest.mark.parametrize("d_mem,d_node", [(16, 0), (0, 12)])
def test_layers_recompute_only_rows_whose_inputs_changed(binding, d_mem, d_node):
    """Layer l of a batch recomputes the endpoints plus the first l hops (one hop less without a
    memory, whose layer-0 rows never change); the skipped rows of A are exactly those a recomputation
    would leave bit-identical, so every layer cache must still equal the oracle's full recompute."""
    w = tiny_workload(num_nodes=600, num_edges=2400, batch=30, layers=3, d_mem=d_mem, d_node=d_node, d_edge=6,
                      d_time=8, d_emb=16, d_msg=16, heads=2, k=3, zipf_s=0.6)
    nf = synth.node_features(w)
    g, o, st = run_stream(binding, w, node_feat=nf, full_check_at=set(range(0, 80, 8)))
    t = g.totals()
    assert t["affected"] > 0 and t["direct"] > 0
    initial = w.layers * w.num_nodes                         # the rebuild at creation
    rows = t["rows"] - initial
    assert rows < w.layers * t["affected"]                  # some layer skipped part of A
    if d_mem == 0:
        assert rows >= t["direct"]                           # layer 1 of a memoryless model: the endpoints only
        assert rows <= t["direct"] + (w.layers - 1) * t["affected"]
    g.close()


@pytest.mark.parametrize("num_nodes", [61000, 131072, 131073, 140000])
def test_compaction_on_both_sides_of_the_one_launch_limit(binding, num_nodes):
    """Flag arrays of at most 32 blocks of 4096 nodes are compacted in one launch (every workgroup
    counts the blocks before its own, the flags are held twice), larger ones in two; the affected
    sets, the per-layer lists (through the embeddings) and the frontier statistics must come out
    the same on both sides of the limit, and through many batches (the flag arrays alternate)."""
    w = tiny_workload(num_nodes=num_nodes, num_edges=6000, batch=300, zipf_s=0.6, k=3, layers=2)
    st = synth.EdgeStream(w)
    W = synth.make_weights(w)
    o = orc.Oracle.from_workload(w, W, None)
    g = binding.StreamTGN.from_workload(w, W, None)
    for b in range(w.num_batches):
        s, d, t, ef = st.batch(b)
        rc, D, A = o.ingest(s, d, t, ef)
        assert rc == 0
        stats = g.ingest_batch(s, d, t, ef, stats=True)
        assert stats["n_direct"] == len(D)
        assert np.array_equal(g.get_affected(), A), f"batch {b}: affected set differs"
        assert sum(stats["frontier"][: w.layers + 1]) == len(A), f"batch {b}: frontier sizes {stats['frontier']}"
    sample = np.unique(np.concatenate([A[:: max(1, len(A) // 400)], np.arange(0, num_nodes, 997, dtype=np.uint32),
                                       np.array([num_nodes - 1], dtype=np.uint32)])).astype(np.uint32)
    for l in range(1, w.layers + 1):
        check_rows(g.get_embeddings(sample, layer=l), o.embed_nodes(sample, layer=l), f"layer {l}")
    g.close()


def test_push_and_pull_hops_give_the_same_affected_set(binding):
    """The expansion pushes along the frontier's logs while the frontier owns few adjacency entries
    and pulls through the clean nodes' rings once it owns more than half the node count; the flags
    must come out the same.  A large sparse graph with small batches starts in push mode and turns
    to pull mode as degrees grow; the affected set is compared with the oracle on every batch."""
    w = tiny_workload(num_nodes=3000, num_edges=6000, batch=25, layers=2, k=3, d_mem=8, d_edge=4, d_time=8, d_emb=8,
                      d_msg=8, zipf_s=1.1)
    st = synth.EdgeStream(w)
    W = synth.make_weights(w)
    o = orc.Oracle.from_workload(w, W)
    g = binding.StreamTGN.from_workload(w, W)
    seen = set()
    for b in range(w.num_batches):
        s, d, t, ef = st.batch(b)
        rc, D, A = o.ingest(s, d, t, ef)
        stats = g.ingest_batch(s, d, t, ef, stats=True)
        assert np.array_equal(g.get_affected(), A), f"batch {b} (pull hops {stats['pull_hops']:b})"
        seen.add(stats["pull_hops"] & 1)
        seen.add(2 + ((stats["pull_hops"] >> 1) & 1))
    assert {0, 1} <= seen, "hop 0 never ran in both directions"
    allnodes = np.arange(w.num_nodes, dtype=np.uint32)
    check_rows(g.get_embeddings(allnodes), o.embed_all()[-1], "final embeddings")
    g.close()


def test_unplanned_hops_and_stale_direction_hints(binding):
    """The host enqueues a hop without its planning kernel when the last statistics it saw said the
    hop pulls, and the device then pulls whatever the frontier's size; a planned hop may still push
    a frontier that has grown large since.  Both are only slower, never different: batches of very
    different sizes are enqueued back to back without a host read in between (so the hints go stale
    in both directions) and the whole state is compared with the oracle afterwards."""
    w = tiny_workload(num_nodes=2000, num_edges=4000, batch=400, layers=2, k=3, d_mem=8, d_edge=4, d_time=8, d_emb=8,
                      d_msg=8, zipf_s=1.2)
    st = synth.EdgeStream(w)
    W = synth.make_weights(w)
    o = orc.Oracle.from_workload(w, W)
    g = binding.StreamTGN.from_workload(w, W)
    allnodes = np.arange(w.num_nodes, dtype=np.uint32)
    # (edges in the batch, poll the statistics afterwards)
    plan = [(400, True), (1, False), (2, False), (1, False), (400, False), (1, True), (400, False), (300, False),
            (1, False), (400, True), (3, False), (400, False), (1, False)]
    lo, directions = 0, set()
    for n, poll in plan:
        hi = lo + n
        s, d, t, ef = st.src[lo:hi], st.dst[lo:hi], st.ts[lo:hi], st.edge_features(lo, hi)
        rc, D, A = o.ingest(s, d, t, ef)
        assert rc == 0
        if poll:
            stats = g.ingest_batch(s, d, t, ef, stats=True)
            assert stats["n_affected"] == len(A)
            directions.add(stats["pull_hops"] & 1)
        else:
            g.ingest_batch(s, d, t, ef)
        lo = hi
    assert np.array_equal(g.get_affected(), A)
    assert directions == {0, 1}, "the polled batches never disagreed about the direction of hop 0"
    gm, gt = g.get_memory(allnodes)
    om, ot = o.memory(allnodes)
    assert np.array_equal(gt, ot)
    check_rows(gm, om, "memory")
    ref = o.embed_all()
    for l in range(1, w.layers + 1):
        check_rows(g.get_embeddings(allnodes, layer=l), ref[l - 1], f"layer {l}")
    g.close()


@pytest.mark.parametrize("window", [2.0, 15.0])
def test_temporal_window_of_the_neighbour_cache(binding, window):
    """Ring entries older than the query time minus T_w are not attended to (Sec. 3.3.2, Invalidate);
    with the narrow window many nodes are left with no entry at all and hold b_O.  Root-node inference
    at the edge's own time applies the window at that time."""
    w = tiny_workload(num_nodes=150, num_edges=1500, batch=50, layers=2, k=5, d_mem=16, d_edge=6, d_time=16, d_emb=16,
                      d_msg=16, heads=2, zipf_s=1.0, window=window)
    g, o, st = run_stream(binding, w, batches=29, full_check_at=set(range(0, 29, 7)))
    ref_no_window = orc.Oracle.from_workload(w.scaled(window=0.0), synth.make_weights(w))
    for b in range(29):
        ref_no_window.ingest(*st.batch(b))
    assert np.abs(ref_no_window.embed_all()[-1] - o.embed_all()[-1]).max() > 1e-3, "this window expires nothing"
    rng = np.random.default_rng(2)
    wp = (rng.standard_normal(2 * w.d_emb) / 4).astype(np.float32)
    g.set_predictor(wp, 0.0)
    s, d, t, _ = st.batch(29)
    t = t + 5.0                                  # later than any stored edge: more entries have expired by then
    want = o.predict(s, d, t, wp, 0.0, at_edge_time=True)
    got = g.predict_batch(s, d, t, at_edge_time=True)
    H = o.embed_all()[-1].astype(np.float64)
    bound = REL * (np.linalg.norm(H[s], axis=1) + np.linalg.norm(H[d], axis=1)) * np.linalg.norm(wp) + 1e-6
    assert (np.abs(got - want) <= bound).all(), np.abs(got - want).max()
    g.close()


@pytest.mark.parametrize("agg", [1, 2])
def test_mean_and_sum_aggregators(binding, agg):
    """Eq. agg_functions: a node's messages of one batch are averaged / summed in batch order before the
    GRU.  Small node count and large batches, so most endpoints have several messages per batch."""
    w = tiny_workload(num_nodes=60, num_edges=2400, batch=80, layers=2, k=4, d_mem=16, d_edge=12, d_time=16, d_emb=16,
                      d_msg=16, heads=2, zipf_s=1.2, aggregator=agg)
    g, o, st = run_stream(binding, w, full_check_at=set(range(0, 30, 6)))
    last = orc.Oracle.from_workload(w.scaled(aggregator=0), synth.make_weights(w))
    for b in range(w.num_batches):
        last.ingest(*st.batch(b))
    nodes = np.arange(w.num_nodes, dtype=np.uint32)
    assert np.abs(last.memory(nodes)[0] - o.memory(nodes)[0]).max() > 1e-3, "the aggregator made no difference"
    g.close()


def test_device_inputs_match_host_inputs(binding):
    w = tiny_workload(num_nodes=300, num_edges=3000, batch=100, d_mem=16, d_edge=12, d_time=16, d_emb=16, d_msg=16, k=4)
    g, o, st = run_stream(binding, w, device_inputs=True, full_check_at={0, 7, 15})
    g.close()


def test_back_to_back_device_batches_overlap_and_a_skipped_batch(binding):
    """Device batches enqueued back to back without a synchronising call run their validation and
    memory update on the library's second stream, beside the previous batch's attention layers.  The
    whole stream goes in that way, with one invalid batch (skipped on the device) in the middle; the
    final state must equal the oracle's, which never saw the invalid batch."""
    import torch
    w = tiny_workload(num_nodes=400, num_edges=6000, batch=100, layers=2, k=4, d_mem=16, d_edge=12, d_time=16,
                      d_emb=16, d_msg=16, zipf_s=1.1)
    st = synth.EdgeStream(w)
    W = synth.make_weights(w)
    o = orc.Oracle.from_workload(w, W)
    g = binding.StreamTGN.from_workload(w, W)
    allnodes = np.arange(w.num_nodes, dtype=np.uint32)

    def dev(s, d, t, ef):
        return (torch.from_numpy(s.astype(np.int32)).cuda(), torch.from_numpy(d.astype(np.int32)).cuda(),
                torch.from_numpy(t).cuda(), torch.from_numpy(ef).cuda())

    nb = w.num_batches - 1                                           # the skipped batch counts against the edge capacity
    batches = [dev(*st.batch(b)) for b in range(nb)]                 # all inputs resident before the first call
    s, d, t, ef = [a.copy() for a in st.batch(31)]
    t[5] = t[4] - 1.0                                                # out of order: the device rejects the whole batch
    bad = dev(s, d, t, ef)
    torch.cuda.synchronize()
    for b in range(nb):
        rc, D, A = o.ingest(*st.batch(b))
        assert rc == 0
        if b == 20:                                                  # a polled batch in between takes the serial path
            assert g.ingest_batch(*batches[b], stats=True)["n_affected"] == len(A)
            continue
        assert g.ingest_batch(*batches[b], check=False) == 0
        if b == 30:
            assert g.ingest_batch(*bad, check=False) == 0
        if b == 40:                                                  # an empty batch and a rebuild between two overlapped batches
            e = batches[b]
            assert g.ingest_batch(e[0][:0], e[1][:0], e[2][:0], e[3][:0], check=False) == 0
            g.full_rebuild()
    assert g.sync(check=False) == -3                                 # the skipped batch is reported once
    assert g.sync(check=False) == 0
    assert np.array_equal(g.get_affected(), A)
    gm, gt = g.get_memory(allnodes)
    om, ot = o.memory(allnodes)
    assert np.array_equal(gt, ot)
    check_rows(gm, om, "memory")
    ref = o.embed_all()
    for l in range(1, w.layers + 1):
        check_rows(g.get_embeddings(allnodes, layer=l), ref[l - 1], f"layer {l}")
    check_neighbours(g, o, allnodes)
    # the same stream through the serial path (a synchronising call after every batch) gives the same bits
    g2 = binding.StreamTGN.from_workload(w, W)
    for b in range(nb):
        g2.ingest_batch(*st.batch(b))
        g2.sync()
    for l in range(1, w.layers + 1):
        assert np.array_equal(g.get_embeddings(allnodes, layer=l), g2.get_embeddings(allnodes, layer=l))
    g.close(); g2.close()


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_random_mix_of_calls_between_overlapped_batches(binding, seed):
    """A seeded random mix of everything a caller can put between two batches -- device and host
    batches without a synchronising call, polled batches, empty batches, full rebuilds, link scores
    of the next batch (both modes, on the device), embedding look-ups on the device, synchronising
    calls -- with the oracle beside it: every result that comes back is compared when it comes back,
    the whole state at the end."""
    import torch
    rng = np.random.default_rng(seed)
    w = tiny_workload(num_nodes=700, num_edges=9000, batch=90, layers=2, k=4, d_mem=16, d_edge=8, d_time=16,
                      d_emb=16, d_msg=16, zipf_s=0.9)
    st = synth.EdgeStream(w)
    W = synth.make_weights(w)
    o = orc.Oracle.from_workload(w, W)
    g = binding.StreamTGN.from_workload(w, W)
    wp = rng.standard_normal(2 * w.d_emb).astype(np.float32)
    g.set_predictor(wp, 0.25)
    allnodes = np.arange(w.num_nodes, dtype=np.uint32)
    dev_nodes = torch.from_numpy(allnodes.astype(np.int32)).cuda()

    def dev(s, d, t, ef):
        return (torch.from_numpy(s.astype(np.int32)).cuda(), torch.from_numpy(d.astype(np.int32)).cuda(),
                torch.from_numpy(t).cuda(), torch.from_numpy(ef).cuda())

    pending = []                                    # (what, device tensor, expected) of asynchronous results
    A = None
    for b in range(w.num_batches):
        s, d, t, ef = st.batch(b)
        # calls before the batch
        for _ in range(int(rng.integers(0, 3))):
            what = int(rng.integers(0, 5))
            if what == 0:
                g.full_rebuild()
            elif what == 1:
                mode = bool(rng.integers(0, 2))
                ds, dd, dt, _ = dev(s, d, t, ef)
                H = o.embed_all()[-1].astype(np.float64)
                bound = REL * (np.linalg.norm(H[s], axis=1) * np.linalg.norm(wp[:w.d_emb]) +
                               np.linalg.norm(H[d], axis=1) * np.linalg.norm(wp[w.d_emb:])) + 1e-6
                pending.append((f"scores before batch {b}, mode {mode}", g.predict_batch(ds, dd, dt, at_edge_time=mode),
                                o.predict(s, d, t, wp, 0.25, at_edge_time=mode), bound))
            elif what == 2:
                layer = int(rng.integers(1, w.layers + 1))
                pending.append((f"rows of layer {layer} before batch {b}", g.get_embeddings(dev_nodes, layer=layer),
                                o.embed_nodes(allnodes, layer=layer), None))
            elif what == 3:
                assert g.sync() == 0
            else:
                z = dev(s[:0], d[:0], t[:0], ef[:0])
                assert g.ingest_batch(*z, check=False) == 0
        rc, D, A = o.ingest(s, d, t, ef)
        assert rc == 0
        how = int(rng.integers(0, 4))
        if how == 0:
            assert g.ingest_batch(*dev(s, d, t, ef), check=False) == 0
        elif how == 1:
            assert g.ingest_batch(s, d, t, ef, check=False) == 0
        elif how == 2:
            stats = g.ingest_batch(*dev(s, d, t, ef), stats=True)
            assert stats["n_affected"] == len(A) and stats["n_direct"] == len(D)
        else:
            assert g.ingest_batch(s, d, t, ef, check=False) == 0
            assert g.sync() == 0
            assert np.array_equal(g.get_affected(), A), f"batch {b}"
        if len(pending) > 6 or b == w.num_batches - 1:
            assert g.sync() == 0
            for name, got, ref, bound in pending:
                got = got.cpu().numpy()
                if got.ndim == 1:
                    assert (np.abs(got - ref) <= bound).all(), f"{name}: worst {np.abs(got - ref).max():.3e}"
                else:
                    check_rows(got, ref, name)
            pending = []
    assert g.sync() == 0
    assert np.array_equal(g.get_affected(), A)
    gm, gt = g.get_memory(allnodes)
    om, ot = o.memory(allnodes)
    assert np.array_equal(gt, ot)
    check_rows(gm, om, "memory")
    ref = o.embed_all()
    for l in range(1, w.layers + 1):
        check_rows(g.get_embeddings(allnodes, layer=l), ref[l - 1], f"layer {l}")
    check_neighbours(g, o, allnodes)
    g.close()


def test_serial_batch_behind_caller_work_then_overlapped_batch(binding):
    """The first batch after a synchronising call runs wholly on the caller's stream; the next one runs
    its front part on the library's second stream.  Both staging kernels update the running edge count,
    the stream time and the batch counter, so the second must stay behind the first even when the first
    is still queued behind work of the caller's own on that stream.  A few milliseconds of matrix products
    are parked on the stream before the two batches go in; edge ids, rings, affected set and rows must
    come out as the oracle's, and no batch may be rejected (a staging kernel that overtook its
    predecessor would see a stale stream time and refuse it, or hand out edge ids in the wrong order)."""
    import torch
    w = tiny_workload(num_nodes=300, num_edges=3000, batch=100, layers=2, k=4, d_mem=16, d_edge=12, d_time=16,
                      d_emb=16, d_msg=16, zipf_s=0.9)
    st = synth.EdgeStream(w)
    W = synth.make_weights(w)
    o = orc.Oracle.from_workload(w, W)
    g = binding.StreamTGN.from_workload(w, W)
    allnodes = np.arange(w.num_nodes, dtype=np.uint32)

    def dev(b):
        s, d, t, ef = st.batch(b)
        return (torch.from_numpy(s.astype(np.int32)).cuda(), torch.from_numpy(d.astype(np.int32)).cuda(),
                torch.from_numpy(t).cuda(), torch.from_numpy(ef).cuda())

    x = torch.randn(2048, 2048, device="cuda")
    b = 0
    for rnd in range(5):
        for _ in range(2):                                   # some state first, synchronised
            rc, D, A = o.ingest(*st.batch(b))
            g.ingest_batch(*dev(b)); b += 1
        assert g.sync() == 0
        first, second, third = dev(b), dev(b + 1), dev(b + 2)
        torch.cuda.synchronize()                             # device inputs hold their final contents
        y = x
        for _ in range(12):                                  # caller's work, still running when the batches arrive
            y = (y @ x) * 0.01
        g.ingest_batch(*first)                               # serial: everything on the caller's stream, behind the products
        g.ingest_batch(*second)                              # overlapped: front part on the second stream
        g.ingest_batch(*third)
        for i in range(3):
            rc, D, A = o.ingest(*st.batch(b + i))
            assert rc == 0
        b += 3
        assert g.sync(check=False) == 0, f"round {rnd}: a batch was rejected: {g.last_error()}"
        assert np.array_equal(g.get_affected(), A), f"round {rnd}: affected set"
        assert g.totals()["edges"] == b * w.batch
        deg = np.bincount(np.concatenate([st.src[:b * w.batch], st.dst[:b * w.batch]]), minlength=w.num_nodes)
        for v in np.argsort(deg)[-3:]:                       # full adjacency (edge ids in arrival order) of the busiest nodes
            nbr, eid = g.get_history(int(v))
            inc = np.nonzero((st.src[:b * w.batch] == v) | (st.dst[:b * w.batch] == v))[0]
            assert np.array_equal(eid, inc.astype(np.uint32)), f"round {rnd}: edge ids of node {v}"
            assert np.array_equal(nbr, np.where(st.src[inc] == v, st.dst[inc], st.src[inc]))
        check_neighbours(g, o, allnodes)
        gm, gt = g.get_memory(allnodes)
        om, ot = o.memory(allnodes)
        assert np.array_equal(gt, ot)
        check_rows(gm, om, f"round {rnd}: memory")
        ref = o.embed_all()
        for l in range(1, w.layers + 1):
            check_rows(g.get_embeddings(allnodes, layer=l), ref[l - 1], f"round {rnd}: layer {l}")
    g.close()


def test_back_to_back_host_batches(binding):
    """A whole stream of host batches without a synchronising call in between: each batch is copied
    into one of two pinned blocks and from there into one of two device staging blocks on the
    library's second stream, a batch ahead of the kernels that read it.  The final state must equal
    the oracle's and, bit for bit, that of the same stream with a synchronising call after every batch."""
    w = tiny_workload(num_nodes=500, num_edges=8000, batch=80, layers=2, k=4, d_mem=16, d_edge=12, d_time=16,
                      d_emb=16, d_msg=16, zipf_s=0.9)
    st = synth.EdgeStream(w)
    W = synth.make_weights(w)
    o = orc.Oracle.from_workload(w, W)
    g = binding.StreamTGN.from_workload(w, W)
    g2 = binding.StreamTGN.from_workload(w, W)
    allnodes = np.arange(w.num_nodes, dtype=np.uint32)
    for b in range(w.num_batches):
        rc, D, A = o.ingest(*st.batch(b))
        assert rc == 0
        s, d, t, ef = [a.copy() for a in st.batch(b)]
        assert g.ingest_batch(s, d, t, ef, check=False) == 0
        s[:] = 0; d[:] = 0; t[:] = 0.0; ef[:] = 0.0          # host inputs are copied before the call returns
        g2.ingest_batch(*st.batch(b))
        g2.sync()
    assert g.sync() == 0
    assert np.array_equal(g.get_affected(), A)
    gm, gt = g.get_memory(allnodes)
    om, ot = o.memory(allnodes)
    assert np.array_equal(gt, ot)
    check_rows(gm, om, "memory")
    ref = o.embed_all()
    for l in range(1, w.layers + 1):
        got = g.get_embeddings(allnodes, layer=l)
        check_rows(got, ref[l - 1], f"layer {l}")
        assert np.array_equal(got, g2.get_embeddings(allnodes, layer=l))
    check_neighbours(g, o, allnodes)
    g.close(); g2.close()


@pytest.mark.parametrize("host_inputs", [False, True])
@pytest.mark.parametrize("num_nodes,batch,zipf_s,expect_pull,layers",
                         [(400, 100, 1.1, True, 2), (6000, 60, 0.3, False, 2), (400, 100, 1.1, True, 1), (3000, 60, 0.3, False, 3),
                          (401, 100, 1.1, True, 2)])         # 401 nodes: the memoryless variant (placement as a launch of its own)
def test_overlapped_pairs_give_the_oracles_affected_sets(binding, num_nodes, batch, zipf_s, expect_pull, layers, host_inputs):
    """Device batches go in in pairs without a synchronising call in between, so the second batch of
    every pair runs its front part -- staging, the first propagation hop, the memory update -- beside
    the first one's main part.  After each pair the second batch's affected set, frontier sizes and
    direction bits are compared with the oracle.  The dense graph pulls, the sparse one pushes
    (work items planned in the front part while the previous batch's last hop reads its own); a
    one-layer model keeps its hop and its compaction on the caller's stream."""
    import torch
    memoryless = num_nodes == 401
    w = tiny_workload(num_nodes=num_nodes, num_edges=40 * batch, batch=batch, layers=layers, k=4,
                      d_mem=0 if memoryless else 16, d_node=12 if memoryless else 0, d_edge=6,
                      d_time=8, d_emb=16, d_msg=16, zipf_s=zipf_s)
    st = synth.EdgeStream(w)
    W = synth.make_weights(w)
    nf = synth.node_features(w)
    o = orc.Oracle.from_workload(w, W, nf)
    g = binding.StreamTGN.from_workload(w, W, nf)

    def dev(s, d, t, ef):
        return (torch.from_numpy(s.astype(np.int32)).cuda(), torch.from_numpy(d.astype(np.int32)).cuda(),
                torch.from_numpy(t).cuda(), torch.from_numpy(ef).cuda())

    # host inputs take the same path: their copy to the device runs ahead like the staging kernel
    batches = [st.batch(b) if host_inputs else dev(*st.batch(b)) for b in range(w.num_batches)]
    torch.cuda.synchronize()
    for b in range(0, w.num_batches - 2, 2):
        rc, D0, A0 = o.ingest(*st.batch(b))
        rc1, D1, A1 = o.ingest(*st.batch(b + 1))
        assert rc == 0 and rc1 == 0
        assert g.ingest_batch(*batches[b], check=False) == 0
        assert g.ingest_batch(*batches[b + 1], check=False) == 0
        assert g.sync() == 0
        assert np.array_equal(g.get_affected(), A1), f"batch {b + 1}: affected set differs"
    # which direction the hops of this graph take (a polled batch reports it)
    last = w.num_batches - 2                                          # the batch after the last pair
    rc, D, A = o.ingest(*st.batch(last))
    stats = g.ingest_batch(*batches[last], stats=True)
    assert stats["n_affected"] == len(A)
    assert (stats["pull_hops"] != 0) == expect_pull, stats
    allnodes = np.arange(w.num_nodes, dtype=np.uint32)
    ref = o.embed_all()
    for l in range(1, w.layers + 1):
        check_rows(g.get_embeddings(allnodes, layer=l), ref[l - 1], f"layer {l}")
    g.close()


def test_rows_outside_A_untouched_and_rebuild_is_bit_identical(binding):
    """Theorem 'Equivalence of Incremental Computation': cached rows outside the affected set are
    bit-identical before and after a batch; a full rebuild reproduces every cached row bit for bit
    (same kernels, per-row results independent of which rows share a launch)."""
    w = tiny_workload(num_nodes=400, num_edges=4000, batch=40, d_mem=32, d_edge=12, d_time=16, d_emb=32, d_msg=32,
                      k=4, zipf_s=0.8)
    st = synth.EdgeStream(w)
    W = synth.make_weights(w)
    g = binding.StreamTGN.from_workload(w, W)
    allnodes = np.arange(w.num_nodes, dtype=np.uint32)
    before = [g.get_embeddings(allnodes, layer=l) for l in (1, 2)]
    seen_small = 0
    for b in range(40):
        g.ingest_batch(*st.batch(b))
        A = g.get_affected()
        outside = np.setdiff1d(allnodes, A)
        after = [g.get_embeddings(allnodes, layer=l) for l in (1, 2)]
        for l in range(2):
            assert np.array_equal(after[l][outside], before[l][outside]), f"batch {b} layer {l + 1}"
        seen_small += len(outside) > 0
        before = after
    assert seen_small > 0
    g.full_rebuild()
    for l in (1, 2):
        assert np.array_equal(g.get_embeddings(allnodes, layer=l), before[l - 1])
    g.close()


def test_bad_batches_leave_the_state_unchanged(binding):
    import torch
    w = tiny_workload(num_nodes=100, num_edges=1000, batch=50, d_mem=8, d_edge=6, d_time=8, d_emb=8, d_msg=8)
    st = synth.EdgeStream(w)
    W = synth.make_weights(w)
    g = binding.StreamTGN.from_workload(w, W)
    allnodes = np.arange(w.num_nodes, dtype=np.uint32)
    g.ingest_batch(*st.batch(0))
    ref = g.get_embeddings(allnodes)
    refm = g.get_memory(allnodes)
    s, d, t, ef = [a.copy() for a in st.batch(1)]

    def variants():
        x = s.copy(); x[3] = w.num_nodes
        yield (x, d, t, ef), -2
        x = d.copy(); x[5] = s[5]
        yield (s, x, t, ef), -4
        x = t.copy(); x[7] = x[6] - 1.0
        yield (s, d, x, ef), -3
        x = t.copy(); x[0] = st.ts[w.batch - 1] - 0.5
        yield (s, d, x, ef), -3
        x = t.copy(); x[9] = np.nan
        yield (s, d, x, ef), -3

    for args, code in variants():        # host inputs: rejected at once
        assert g.ingest_batch(*args, check=False) == code
        assert np.array_equal(g.get_embeddings(allnodes), ref)
    for args, code in variants():        # device inputs: skipped on the device, reported at the next sync
        dev = (torch.from_numpy(args[0].astype(np.int32)).cuda(), torch.from_numpy(args[1].astype(np.int32)).cuda(),
               torch.from_numpy(args[2]).cuda(), torch.from_numpy(args[3]).cuda())
        assert g.ingest_batch(*dev, check=False) == 0
        assert g.sync(check=False) == code
        assert g.sync(check=False) == 0
        assert np.array_equal(g.get_embeddings(allnodes), ref)
        m = g.get_memory(allnodes)
        assert np.array_equal(m[0], refm[0]) and np.array_equal(m[1], refm[1])
    big = np.zeros(w.batch + 1, dtype=np.uint32)
    assert g.ingest_batch(big, big + 1, np.zeros(w.batch + 1), np.zeros((w.batch + 1, w.d_edge), np.float32),
                          check=False) == -5
    # the stream continues normally afterwards
    o = orc.Oracle.from_workload(w, W)
    o.ingest(*st.batch(0))
    rc, D, A = o.ingest(s, d, t, ef)
    g.ingest_batch(s, d, t, ef)
    assert np.array_equal(g.get_affected(), A)
    check_rows(g.get_embeddings(allnodes), o.embed_all()[-1], "after recovery")
    g.close()


def test_empty_batch_and_ring_overflow_in_one_batch(binding):
    w = tiny_workload(num_nodes=6, num_edges=7, batch=7, layers=1, k=3, d_mem=8, d_edge=6, d_time=8, d_emb=8, d_msg=8)
    W = synth.make_weights(w)
    g = binding.StreamTGN.from_workload(w, W, max_edges=64, max_batch=16)
    o = orc.Oracle.from_workload(w, W)
    e = np.zeros(0, dtype=np.uint32)
    st0 = g.ingest_batch(e, e, np.zeros(0), np.zeros((0, w.d_edge), np.float32), stats=True)
    assert st0["n_direct"] == 0 and st0["n_affected"] == 0 and len(g.get_affected()) == 0
    src = np.array([0, 1, 0, 2, 0, 0, 3], dtype=np.uint32)
    dst = np.array([1, 0, 1, 0, 4, 5, 0], dtype=np.uint32)
    ts = np.arange(1, 8, dtype=np.float64)
    ef = np.random.default_rng(3).standard_normal((7, w.d_edge)).astype(np.float32)
    rc, D, A = o.ingest(src, dst, ts, ef)
    g.ingest_batch(src, dst, ts, ef)
    assert np.array_equal(g.get_affected(), A)
    allnodes = np.arange(6, dtype=np.uint32)
    check_neighbours(g, o, allnodes)
    check_rows(g.get_embeddings(allnodes), o.embed_all()[-1], "overflow batch")
    gm, _ = g.get_memory(allnodes)
    check_rows(gm, o.memory(allnodes)[0], "memory")
    g.close()


def test_equal_timestamps_and_repeated_pairs(binding):
    """Ties: many edges share one timestamp and the same pair repeats inside a batch; arrival order
    (batch index, source side first) is the only order, multi-edges are separate ring entries."""
    w = tiny_workload(num_nodes=12, num_edges=96, batch=24, layers=2, k=4, d_mem=8, d_edge=6, d_time=8, d_emb=8,
                      d_msg=8)
    W = synth.make_weights(w)
    g = binding.StreamTGN.from_workload(w, W)
    o = orc.Oracle.from_workload(w, W)
    rng = np.random.default_rng(11)
    allnodes = np.arange(w.num_nodes, dtype=np.uint32)
    t0 = 0.0
    for b in range(4):
        src = rng.integers(0, 4, size=24).astype(np.uint32)               # few nodes: many repeated pairs
        dst = (src + 1 + rng.integers(0, 3, size=24)).astype(np.uint32) % 12
        dst = np.where(dst == src, (src + 1) % 12, dst).astype(np.uint32)
        ts = np.full(24, t0 + 1.0) if b % 2 == 0 else t0 + np.repeat(np.arange(1, 7, dtype=np.float64), 4)
        t0 = float(ts[-1])
        ef = rng.standard_normal((24, w.d_edge)).astype(np.float32)
        rc, D, A = o.ingest(src, dst, ts, ef)
        assert rc == 0
        g.ingest_batch(src, dst, ts, ef)
        assert np.array_equal(g.get_affected(), A)
        check_neighbours(g, o, allnodes)
        ref = o.embed_all()
        for l in (1, 2):
            check_rows(g.get_embeddings(allnodes, layer=l), ref[l - 1], f"batch {b} layer {l}")
    g.close()


def test_largest_batch_and_four_layers(binding):
    """One batch of STGN_MAX_BATCH edges (the sort runs at its largest size) on a graph deep enough
    for four layers; affected set exact, sampled embeddings against the oracle's recursion."""
    w = tiny_workload(num_nodes=5000, num_edges=2 * 8192, batch=8192, layers=4, k=5, d_mem=16, d_edge=8, d_time=8,
                      d_emb=16, d_msg=16, heads=2, zipf_s=0.9)
    st = synth.EdgeStream(w)
    W = synth.make_weights(w)
    g = binding.StreamTGN.from_workload(w, W)
    o = orc.Oracle.from_workload(w, W)
    rng = np.random.default_rng(5)
    for b in range(2):
        s, d, t, ef = st.batch(b)
        assert len(s) == 8192
        rc, D, A = o.ingest(s, d, t, ef)
        assert rc == 0
        stats = g.ingest_batch(s, d, t, ef, stats=True)
        assert stats["n_direct"] == len(D)
        assert np.array_equal(g.get_affected(), A)
        S = np.unique(np.concatenate([rng.choice(A, size=150), rng.integers(0, w.num_nodes, size=50)])).astype(np.uint32)
        check_neighbours(g, o, S)
        check_rows(g.get_embeddings(S), o.embed_nodes(S), f"batch {b}: sampled embeddings")
    g.close()


def test_edge_capacity_is_enforced(binding):
    w = tiny_workload(num_nodes=50, num_edges=200, batch=40, d_mem=8, d_edge=6, d_time=8, d_emb=8, d_msg=8)
    st = synth.EdgeStream(w)
    g = binding.StreamTGN.from_workload(w, synth.make_weights(w), max_edges=100)
    allnodes = np.arange(w.num_nodes, dtype=np.uint32)
    assert g.ingest_batch(*st.batch(0), check=False) == 0
    assert g.ingest_batch(*st.batch(1), check=False) == 0
    ref = g.get_embeddings(allnodes)
    assert g.ingest_batch(*st.batch(2), check=False) == -6          # 120 > 100: refused, nothing changes
    assert np.array_equal(g.get_embeddings(allnodes), ref)
    g.close()


def test_c2_stream_sampled(binding):
    """Config 2, the WHOLE stream of 1,000 batches with device-resident inputs as the benchmark feeds
    them: exact affected set on every batch; memory of the batch's endpoints and sampled embeddings
    (inside and outside the affected set) at checkpoints that include the span the benchmark times
    (batches 700-850) and the end of the stream; all rows of both layers at the end."""
    import torch
    w = synth.WORKLOADS["C2"]
    st = synth.EdgeStream(w)
    W = synth.make_weights(w)
    o = orc.Oracle.from_workload(w, W)
    g = binding.StreamTGN.from_workload(w, W)
    rng = np.random.default_rng(5)
    allnodes = np.arange(w.num_nodes, dtype=np.uint32)
    nb = w.num_batches
    d_src = torch.from_numpy(st.src.astype(np.int32)).cuda()
    d_dst = torch.from_numpy(st.dst.astype(np.int32)).cuda()
    d_ts = torch.from_numpy(st.ts).cuda()
    d_ef = torch.from_numpy(st.edge_features(0, w.num_edges)).cuda()
    checkpoints = {59, 299, 499, 700, 775, 850, 925, 999}
    for b in range(nb):
        s, d, t, ef = st.batch(b)
        rc, D, A = o.ingest(s, d, t, ef)
        lo, hi = b * w.batch, (b + 1) * w.batch
        g.ingest_batch(d_src[lo:hi], d_dst[lo:hi], d_ts[lo:hi], d_ef[lo:hi])
        assert np.array_equal(g.get_affected(), A), f"batch {b}"
        if b in checkpoints:
            gm, gt = g.get_memory(D)
            om, ot = o.memory(D)
            assert np.array_equal(gt, ot)
            check_rows(gm, om, f"batch {b}: memory of D")
            inA = rng.choice(A, size=60, replace=False)
            out = rng.choice(np.setdiff1d(allnodes, A), size=20, replace=False)
            S = np.concatenate([inA, out]).astype(np.uint32)
            for l in (1, 2):
                check_rows(g.get_embeddings(S, layer=l), o.embed_nodes(S, layer=l), f"batch {b}: sampled rows of layer {l}")
            check_neighbours(g, o, S[:20])
    ref = o.embed_all()
    for l in (1, 2):
        check_rows(g.get_embeddings(allnodes, layer=l), ref[l - 1], f"final layer {l}")
    gm, gt = g.get_memory(allnodes)
    om, ot = o.memory(allnodes)
    assert np.array_equal(gt, ot)
    check_rows(gm, om, "final memory")
    g.close()
