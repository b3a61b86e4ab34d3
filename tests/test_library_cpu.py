"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol, sizes a
workspace and rejects bad arguments.  No kernel runs here."""
import ctypes as C
import os
import re

import pytest

from paper_2603_21090_amd import binding, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2603_21090_amd import build
        build.build_library()
    return binding.load_library()


def test_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "streamtgn.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(stgn_[a-z_]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name
    assert lib.stgn_version().decode().startswith("streamtgn")


def cfg_of(w, **kw):
    base = dict(num_nodes=w.num_nodes, max_edges=w.num_edges, max_batch=w.batch, d_mem=w.d_mem, d_node=w.d_node,
                d_edge=w.d_edge, d_time=w.d_time, d_emb=w.d_emb, d_msg=w.d_msg, k=w.k, heads=w.heads, layers=w.layers)
    base.update(kw)
    return binding.make_config(**base)


def test_workspace_sizes_scale_with_the_configuration():
    sizes = {name: binding.query_workspace(cfg_of(w)) for name, w in synth.WORKLOADS.items()}
    assert sizes["C1"] < sizes["C2"] < sizes["C3"] < sizes["C4"] < sizes["C5"]
    assert sizes["C5"] < 200 * 2**30          # the largest workload fits one MI355X (288 GB)
    # wide edge features (172 floats): one cached key|value row per edge and layer (two heads of 50: 2 x 2 x 64
    # floats) must be inside, the raw edge-feature rows are not kept
    # ... and the query row (q and its time part: 64 x (2 + 2 x 2) floats) per node: of the first layer
    # with a memory, of every layer without
    w = synth.WORKLOADS["C4"]
    qrow = 64 * 6 * 4
    assert w.num_edges * (w.layers * 256 * 4) + w.num_nodes * qrow < sizes["C4"] \
        < w.num_edges * (w.layers * 256 * 4 + 128 * 4) + w.num_nodes * qrow
    # narrow edge features (64 floats): the raw row padded to 64 floats once per edge, no cached edge rows; per
    # node and layer a cached key|value row and a query row of 64 x (2 + 2 x 3) floats (the edge slot rides
    # with the time part)
    w5 = synth.WORKLOADS["C5"]
    per_node = w5.layers * (256 * 4 + 64 * 8 * 4)
    assert w5.num_edges * 64 * 4 + w5.num_nodes * per_node < sizes["C5"] \
        < w5.num_edges * (64 * 4 + 64) + w5.num_nodes * (per_node + 3072)
    # ... the delta mode keeps the cached edge rows
    d5 = binding.query_workspace(cfg_of(w5, delta_mode=1, drift_gamma=0.9))
    assert d5 > w5.num_edges * w5.layers * 256 * 4
    per_node = 0
    # delta mode adds the attention cache: per node, layer and recent-neighbour entry the value part and two floats per head
    d4 = binding.query_workspace(cfg_of(w, delta_mode=1, drift_gamma=0.9))
    assert d4 - sizes["C4"] > w.num_nodes * w.layers * w.k * (128 + 4) * 4 - w.num_nodes * per_node


def test_edge_features_of_one_slot_are_kept_raw():
    """Up to 64 edge features: one 64-float row per edge.  Past that, in the delta mode, and for shapes whose
    layer-kernel tiles leave no room for the edge slot: a cached key|value row per edge and layer."""
    w = synth.WORKLOADS["C5"]
    kv = 2 * 64 * 2 * 4                       # two heads of 50: one slot each, keys and values, fp32
    s64, s65 = (binding.query_workspace(cfg_of(w, d_edge=e)) for e in (64, 65))
    # (with raw rows the cached query of a node is one slot per head longer)
    assert s65 - s64 > w.num_edges * (w.layers * kv - 64 * 4) - w.num_nodes * w.layers * 2 * 64 * 4 - (1 << 24)
    s1 = binding.query_workspace(cfg_of(w, d_edge=1))
    assert abs(s64 - s1) < w.num_edges * 16 + 2 * 8192 * 64 * 4 * 4      # the same rows; staging differs by the batch's features
    wide = dict(heads=4, d_emb=64, d_time=100)                              # four heads x (two time slots + the edge slot)
    t0, t40 = (binding.query_workspace(cfg_of(w, d_edge=e, **wide)) for e in (0, 40))
    assert t40 - t0 > w.num_edges * w.layers * (2 * 64 * 4 * 4) * 0.99
    narrow = dict(heads=4, d_emb=64, d_time=20)                             # one time slot: the edge slot fits
    u0, u40 = (binding.query_workspace(cfg_of(w, d_edge=e, **narrow)) for e in (0, 40))
    assert u40 - u0 < w.num_edges * (64 * 4 + 16) + w.num_nodes * w.layers * 4 * 64 * 4 + (1 << 24)


@pytest.mark.parametrize("ok", [dict(d_emb=256, heads=4), dict(d_emb=256, heads=1), dict(d_emb=130, heads=1),
                                dict(d_emb=128, heads=2, d_time=128)])
def test_widest_supported_attention_shapes(lib, ok):
    n = C.c_size_t(0)
    assert lib.stgn_query_workspace(C.byref(cfg_of(synth.WORKLOADS["C1"], **ok)), C.byref(n)) == 0 and n.value > 0


@pytest.mark.parametrize("bad", [dict(num_nodes=0), dict(max_edges=0), dict(max_batch=0), dict(max_batch=8193),
                                 dict(layers=0), dict(layers=5), dict(k=0), dict(heads=3), dict(heads=0),
                                 dict(d_emb=0), dict(d_time=0), dict(d_mem=0, d_node=0), dict(max_edges=2**31),
                                 dict(d_emb=300, heads=4),      # 75-wide heads: 8 key slots, more than a cached row has
                                 dict(d_emb=260, heads=1), dict(d_time=129), dict(aggregator=3), dict(delta_mode=2),
                                 dict(delta_mode=1, drift_gamma=0.0), dict(delta_mode=1, drift_gamma=1.5)])
def test_bad_configurations_are_rejected(lib, bad):
    w = synth.WORKLOADS["C1"]
    n = C.c_size_t(0)
    assert lib.stgn_query_workspace(C.byref(cfg_of(w, **bad)), C.byref(n)) == -1
    assert lib.stgn_last_error(None)


def test_null_arguments(lib):
    n = C.c_size_t(0)
    assert lib.stgn_query_workspace(None, C.byref(n)) == -1
    assert lib.stgn_query_workspace(C.byref(cfg_of(synth.WORKLOADS["C1"])), None) == -1
    assert lib.stgn_sync(None) == -1
    assert lib.stgn_full_rebuild(None) == -1
    lib.stgn_destroy(None)


def test_create_without_workspace_or_device_fails_cleanly(lib):
    w = synth.WORKLOADS["C1"]
    W = synth.make_weights(w)
    cw, keep = binding._marshal_weights(W, w.layers, True)
    h = C.c_void_p(None)
    rc = lib.stgn_create(C.byref(cfg_of(w)), C.byref(cw), None, None, 0, None, C.byref(h))
    assert rc == -8 and not h.value
    rc = lib.stgn_create(C.byref(cfg_of(w)), None, None, None, 0, None, C.byref(h))
    assert rc == -1


@pytest.mark.parametrize("name", ["C2", "C4", "C5"])
def test_stored_counter_traffic_belongs_to_the_batches_the_benchmark_profiles(name):
    """bench.py reports `roofline.traffic` from the counter summaries under profiles/, which are keyed to a
    batch range: it must be the range of the benchmark's per-kernel pass, or the figure silently turns null."""
    import bench
    w = synth.WORKLOADS[name]
    window = bench.pass_positions(w.num_batches)[5]
    got = bench.stored_traffic(name, window)
    assert got is not None and got > 0, f"profiles/layer_kernel_{name}_hbm_traffic.txt does not cover batches {window}"
