#!/usr/bin/env python3
"""Benchmark of the per-batch incremental inference step on one MI355X.

A step is one batch of the synthetic edge stream through the whole hot path
(stage + sort, message/GRU, apply, dirty-flag propagation, compaction, all attention
layers for the affected set).  Inputs are resident in device memory before the timed
region starts.  The stream is replayed from the empty graph, and every pass sits at a
FIXED position of the stream, whatever --warmup / --steps say:

  state    batches [0, P), P = 70 % of the stream, untimed: builds the graph state
  warmup   W more untimed batches                              (--warmup, default 0)
  timed    K batches enqueued back to back, one sync          -> `value` (edges/s), ms_per_step
           (--steps, default: all of [P + W, Q), Q = 85 % of the stream; a W + K longer than that moves P
           back, down to 20 % of the stream)
  filler   untimed up to batch Q
  latency  from batch Q on, one sync per batch                 -> p50 / p95 batch latency
  host     next batches fed from host memory                   -> PCIe-inclusive rate
  stages   next batches with the library's per-stage events
  kernels  next batches with one HIP event pair per launch     -> per-kernel average duration,
                                                                  roofline of the dominant kernel
  cpu      the CPU oracle on a bounded sample of the same workload, 1 core
  copy     a plain 1 GiB copy and a bare gather of the layer launch's own mix of rows, after the
           library's context is gone                           -> roofline.measured_copy_GBs, roofline.bare_gather

Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_F32_PEAK_TFLOPS = 157.3   # MI355X dense fp32 matrix, published


def algorithmic_bytes(w, rows, entries):
    """Bytes one attention layer must move, by the plain definition of the layer, for `rows` target
    rows that hold `entries` recent-neighbour records in total: per row the own layer-input row, the
    last-interaction time and the output row; per record the 16-byte ring entry, one neighbour row
    and one edge-feature row (fp32).  With full rings (entries = k * rows) this is the
    per-(node, layer) figure 4 d + 8 + 4 d + k (16 + 4 d + 4 d_edge)."""
    d_in = np.mean([(w.d_mem + w.d_node) if l == 0 else w.d_emb for l in range(w.layers)])
    return rows * (4 * d_in + 8 + 4 * w.d_emb) + entries * (16 + 4 * d_in + 4 * w.d_edge)


def cached_row_floats(w):
    """Floats of one cached key|value row: every head takes whole 64-float slots (1, 2 or 4 of them)."""
    sh = -(-(w.d_emb // w.heads) // 64)
    sh = 4 if sh == 3 else sh
    return 2 * 64 * w.heads * sh


def raw_edge_rows(w, delta_mode=False):
    """Whether the library keeps an edge's features as one raw 64-float row (narrow features, exact mode)
    instead of a cached key|value row per layer."""
    return 0 < w.d_edge <= 64 and not delta_mode


def layout_bytes(w, rows, entries, delta_mode=False):
    """Bytes the layer kernel's own data layout moves: per record the ring entry, the neighbour's cached
    key|value row and the edge's (a cached row, or the raw feature row padded to 64 floats) instead of the
    raw rows; per target row its input row, time, output row and, for every layer but the last, its own
    cached row for the next layer."""
    d_in = np.mean([(w.d_mem + w.d_node) if l == 0 else w.d_emb for l in range(w.layers)])
    kv = 4 * cached_row_floats(w)
    per_row = 4 * d_in + 8 + 4 * w.d_emb + kv * (w.layers - 1) / w.layers
    edge = 256 if raw_edge_rows(w, delta_mode) else kv if w.d_edge else 0
    return rows * per_row + entries * (16 + kv + edge)


def projection_flops_per_row(w, layer, delta_mode=False):
    """FLOPs of the dense products the layer kernel executes for one (node, layer), padding not
    counted: the query; the time parts of keys and values, re-associated (with raw edge rows the edge
    parts ride along); the output projection; and, for every layer but the last, the row's cached keys
    and values for the next layer.  (The node parts of keys and values, and the edge parts of wide edge
    features, are cached rows: computed once per changed row / once per edge.)"""
    d_in = (w.d_mem + w.d_node) if layer == 0 else w.d_emb
    d_z = w.d_time + (w.d_edge if raw_edge_rows(w, delta_mode) else 0)
    q = 2 * (d_in * w.d_emb + w.d_emb * d_z)                      # q, then qt_h = W_K,h[time | edge] q_h
    o = 2 * (d_z * w.d_emb + w.d_emb * w.d_emb)                   # pb_h W_V,h[time | edge], then W_O
    if layer + 1 < w.layers:
        o += 2 * (w.d_emb * 2 * w.d_emb)                          # cached keys | values of the next layer
    return q, o


def stored_traffic(workload, batches):
    """HBM bytes per layer-kernel launch from the hardware counters.  Counters cannot be read from
    inside this process; the figure comes from the two counter runs of this same command whose
    summary is kept as text under profiles/, and applies only to the same workload and batch range."""
    path = os.path.join(ROOT, "profiles", f"layer_kernel_{workload}_hbm_traffic.txt")
    try:
        text = open(path).read()
    except OSError:
        return None
    m = re.search(r"^traffic_bytes_per_launch\s*=\s*([0-9.eE+]+)", text, re.M)
    r = re.search(r"^batches\s*=\s*\[(\d+),\s*(\d+)\]", text, re.M)
    if not m or not r or [int(r.group(1)), int(r.group(2))] != list(batches):
        return None
    return float(m.group(1))


def pass_positions(nb, latency_steps=None, host_steps=None, kernel_steps=None):
    """Fixed positions of the passes in a stream of nb batches: (P, Q, LAT, HOST, KER, [first, last) of the
    per-kernel pass) -- the state-building prefix, the start of the diagnostic passes, their lengths, and the
    batches whose layer launches the roofline figures (and the stored counter traffic) refer to."""
    P = int(0.70 * nb)
    Q = int(0.85 * nb)
    rest = nb - Q
    LAT = min(rest * 6 // 15, 160) if latency_steps is None else latency_steps
    HOST = min(rest * 4 // 15, 48) if host_steps is None else host_steps
    KER = min(rest - LAT - HOST, 100) if kernel_steps is None else kernel_steps
    n_stage = min(20, KER)
    first = Q + LAT + HOST + n_stage
    return P, Q, LAT, HOST, KER, [first, first + KER - n_stage]


def cpu_sample_plan(w, st, Q, n_s=120_000):
    """Large graphs: the nodes whose rows the CPU oracle will evaluate (uniform over all nodes) and the
    edges their recent-neighbour lists hold after batch Q (ascending edge ids).  Bookkeeping on the raw
    edge list only."""
    hi = Q * w.batch
    rng = np.random.default_rng(7)
    n_s = min(n_s, w.num_nodes)
    S = np.sort(rng.choice(w.num_nodes, size=n_s, replace=False)).astype(np.int64)
    src, dst = st.src[:hi].astype(np.int64), st.dst[:hi].astype(np.int64)
    inS = np.zeros(w.num_nodes, dtype=bool)
    inS[S] = True
    eids = np.nonzero(inS[src] | inS[dst])[0]
    node = np.concatenate([src[eids], dst[eids]])
    eid2 = np.concatenate([eids, eids])
    keep = inS[node]
    node, eid2 = node[keep], eid2[keep]
    order = np.lexsort((eid2, node))
    node, eid2 = node[order], eid2[order]
    # rank of every entry from the end of its node's list: the last k are the recent-neighbour list
    n_ent = len(node)
    last = np.r_[node[1:] != node[:-1], True] if n_ent else np.zeros(0, bool)
    end_of = np.zeros(n_ent, dtype=np.int64)
    if n_ent:
        ends = np.nonzero(last)[0]
        end_of = ends[np.searchsorted(ends, np.arange(n_ent), side="left")]
    in_ring = (end_of - np.arange(n_ent)) < w.k
    return {"S": S, "ring_e": np.unique(eid2[in_ring]), "entries": int(in_ring.sum()), "Q": Q}


def cpu_baseline(w, st, weights, nf, Q, cpu_steps, note, plan=None, plan_rows=None):
    """The CPU oracle (full recompute of every node after every batch, one core) at the stream position
    the GPU passes are taken at (batch Q).

    Small graphs: the oracle replays the stream up to batch Q, then `cpu_steps` batches are timed, each
    = ingest + full recompute of all rows.  Large graphs (a full recompute alone would take minutes to
    hours): the cost of one row is measured on a uniform sample of nodes -- a fresh oracle is fed exactly
    the edges the sampled nodes' recent-neighbour lists hold after batch Q (`plan`, their feature rows in
    `plan_rows`) and evaluates their first-layer rows (a row's cost depends on how many entries it
    attends to and on the widths, equal for all layers here, not on the values) -- and multiplied out to
    all N nodes and all layers; one real batch is ingested on the same oracle for the message / GRU /
    append part.  Labelled "extrapolated"."""
    from oracle import oracle as orc
    if plan is None:
        o = orc.Oracle.from_workload(w, weights, nf)
        for ob in range(Q):
            o.ingest(*st.batch(ob))
        note("cpu baseline: oracle state built", force=True)
        c0 = time.perf_counter()
        ce = 0
        for i in range(cpu_steps):
            s_, d_, t_, e_ = st.batch(Q + i)
            o.ingest(s_, d_, t_, e_)
            o.embed_all()                                  # the oracle has no cache: full recompute
            ce += len(s_)
        cw = time.perf_counter() - c0
        return {"value": ce / cw, "unit": "edges/s", "cores": 1, "kind": "oracle",
                "sample": f"{cpu_steps} batches of {w.batch} edges after {Q} untimed state-building batches (the "
                          f"position of the GPU passes); each = ingest + full recompute of all {w.num_nodes} nodes, "
                          f"{w.layers} layers; host has {os.cpu_count()} logical cores, oracle uses 1",
                "seconds_per_batch": cw / cpu_steps, "extrapolated": False}
    S, ring_e, entries = plan["S"], plan["ring_e"], plan["entries"]
    o = orc.Oracle.from_workload(w, weights, nf)
    for lo in range(0, len(ring_e), w.batch):
        e = ring_e[lo:lo + w.batch]
        rc, _, _ = o.ingest(st.src[e], st.dst[e], st.ts[e], plan_rows[lo:lo + w.batch])
        assert rc == 0
    note("cpu baseline: sampled neighbourhoods loaded", force=True)
    c0 = time.perf_counter()
    o.embed_nodes(S.astype(np.uint32), layer=1)
    row_s = (time.perf_counter() - c0) / len(S)
    # one real batch for the message / GRU / append / affected-set part (on a graph far smaller than the real one)
    s_, d_, t_, e_ = st.batch(Q)
    if len(ring_e):
        t_ = t_ - t_[0] + st.ts[ring_e[-1]] + 1.0
    c0 = time.perf_counter()
    o.ingest(s_, d_, t_, e_)
    ing_s = time.perf_counter() - c0
    per_batch = w.num_nodes * w.layers * row_s + ing_s
    return {"value": w.batch / per_batch, "unit": "edges/s", "cores": 1, "kind": "oracle",
            "sample": f"extrapolated: first-layer rows of {len(S)} nodes drawn uniformly from all {w.num_nodes} "
                      f"({entries} recent-neighbour entries, as held after batch {Q}) evaluated by the oracle in "
                      f"{row_s * len(S):.1f} s, times N x layers = {w.num_nodes} x {w.layers} rows of a full recompute "
                      f"per batch, plus one batch ingested ({ing_s:.2f} s); host has {os.cpu_count()} logical "
                      f"cores, oracle uses 1",
            "seconds_per_batch": per_batch, "seconds_per_row": row_s, "extrapolated": True}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="C5")
    ap.add_argument("--predict-reps", type=int, default=20, help="timed repetitions of the root-inference call per mode")
    ap.add_argument("--batch", type=int, default=None, help="override the workload's batch size (ablation sweeps)")
    ap.add_argument("--k", type=int, default=None, help="override the workload's recent-neighbour count (ablation sweeps)")
    ap.add_argument("--latency-steps", type=int, default=None)
    ap.add_argument("--kernel-steps", type=int, default=None)
    ap.add_argument("--host-steps", type=int, default=None,
                    help="batches fed from host (pageable numpy) buffers, for the PCIe-inclusive rate")
    ap.add_argument("--rebuilds", type=int, default=3, help="timed full_rebuild() calls at the end")
    ap.add_argument("--cpu-steps", type=int, default=2)
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--delta-mode", action="store_true",
                    help="run the approximate delta-embedding mode instead of the exact one (a diagnostic: the line's "
                         "`mode` says so); reports the drift metric and the deviation from an exact rebuild at the end")
    ap.add_argument("--drift-gamma", type=float, default=0.95)
    ap.add_argument("--maintain-every", type=int, default=0, help="delta mode: call the rebuild policy every this many batches")
    ap.add_argument("--delta-max", type=float, default=0.5)
    ap.add_argument("--alpha", type=float, default=0.1)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="kept for the counter runs' command lines: the plain 1 GiB device copy (5 launches) that scales "
                         "the hardware byte counters is now always run at the end")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(no collectives or sharding in this library)", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2603_21090_amd import binding, synth

    w = synth.WORKLOADS[args.workload]
    if args.batch or args.k:          # a variant of the named workload; stored traffic figures do not apply to it
        w = w.scaled(name=f"{w.name}(B={args.batch or w.batch},k={args.k or w.k})", batch=args.batch or w.batch,
                     k=args.k or w.k)
    nb = w.num_batches
    # state-building prefix and start of the diagnostic passes: the same for every invocation
    P, Q, LAT, HOST, KER, _ = pass_positions(nb, args.latency_steps, args.host_steps, args.kernel_steps)
    W = 0 if args.warmup is None else args.warmup
    K = (Q - P - W) if args.steps is None else args.steps
    rest = nb - Q
    if K > 0 and W >= 0 and P + W + K > Q and Q - W - K >= int(0.20 * nb):
        P = Q - W - K                      # a longer timed span than 15 % of the stream: it starts earlier, and still ends at Q
    if K <= 0 or W < 0 or P + W + K > Q:
        print(f"bench.py: warmup {W} + steps {K} do not fit batches [{int(0.20 * nb)}, {Q}) of the {nb}-batch stream "
              f"(at least the first 20 % build the graph state, the passes from batch {Q} on have fixed positions)",
              file=sys.stderr)
        sys.exit(2)
    if Q + LAT + HOST + KER > nb:
        print(f"bench.py: latency {LAT} + host {HOST} + kernel {KER} batches exceed the last {rest} batches of the stream",
              file=sys.stderr)
        sys.exit(2)

    last_note = [time.perf_counter()]

    def note(msg, force=False):
        """progress on stderr, at most every 20 s (long workloads are otherwise silent for minutes)"""
        now = time.perf_counter()
        if force or now - last_note[0] > 20.0:
            print(f"[bench {w.name}] {msg}", file=sys.stderr, flush=True)
            last_note[0] = now

    dev = torch.device("cuda:0")
    note("generating the edge stream", force=True)
    st = synth.EdgeStream(w)
    weights = synth.make_weights(w)
    nf = synth.node_features(w)
    g = binding.StreamTGN.from_workload(w, weights, nf, delta_mode=1 if args.delta_mode else 0,
                                        drift_gamma=args.drift_gamma if args.delta_mode else 0.0)
    maintained = {0: 0, 1: 0, 2: 0}

    # the whole stream segment that will be used, resident on the device
    used = min((Q + LAT + HOST + KER) * w.batch, w.num_edges)
    d_src = torch.from_numpy(st.src[:used].astype(np.int32)).to(dev)
    d_dst = torch.from_numpy(st.dst[:used].astype(np.int32)).to(dev)
    d_ts = torch.from_numpy(st.ts[:used]).to(dev)
    d_ef = torch.empty((used, w.d_edge), dtype=torch.float32, device=dev)
    # large graphs: which edges the CPU baseline's sampled rows need (their feature rows are picked up below)
    plan, plan_rows = None, None
    if not args.no_cpu and args.cpu_steps > 0 and w.num_nodes > 20_000:
        plan = cpu_sample_plan(w, st, Q)
        plan_rows = np.zeros((len(plan["ring_e"]), w.d_edge), dtype=np.float32)
    CH = 1 << 18
    if w.d_edge:
        # the feature rows are drawn chunk by chunk from independently keyed generators: several host threads
        import concurrent.futures as cf
        with cf.ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as pool:
            spans = [(lo, min(lo + CH, used)) for lo in range(0, used, CH)]
            for (lo, hi), rows in zip(spans, pool.map(lambda sp: st.edge_features(*sp), spans)):
                d_ef[lo:hi] = torch.from_numpy(rows).to(dev)
                if plan is not None:
                    i0, i1 = np.searchsorted(plan["ring_e"], [lo, hi])
                    plan_rows[i0:i1] = rows[plan["ring_e"][i0:i1] - lo]
                note(f"edge features resident: {hi}/{used}")
    torch.cuda.synchronize()
    note("warm-up", force=True)

    def feed(b, stats=False):
        lo, hi = b * w.batch, min((b + 1) * w.batch, used)
        r = g.ingest_batch(d_src[lo:hi], d_dst[lo:hi], d_ts[lo:hi], d_ef[lo:hi], stats=stats)
        if args.delta_mode and args.maintain_every and b % args.maintain_every == args.maintain_every - 1:
            maintained[g.maintain(args.delta_max, args.alpha)[0]] += 1      # (synchronises: part of this mode's cost)
        return r

    b = 0

    def run_untimed(upto, what):
        nonlocal b
        while b < upto:
            feed(b); b += 1
            if b % 256 == 0:
                g.sync()
                note(f"{what}: batch {b}/{upto}")
        g.sync()

    run_untimed(P + W, "state building")
    tot0 = g.totals()
    note("timed region", force=True)

    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(K):
        feed(b); b += 1
    g.sync()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    tot1 = g.totals()
    wall = t1 - t0
    edges = tot1["edges"] - tot0["edges"]
    aff = tot1["affected"] - tot0["affected"]
    direct = tot1["direct"] - tot0["direct"]

    run_untimed(Q, "filler up to the diagnostic passes")
    note("latency / host-input / kernel passes", force=True)
    # per-batch latency: enqueue + wait, one batch at a time
    lat = []
    stage_us = np.zeros(6)
    for _ in range(LAT):
        a = time.perf_counter()
        feed(b); g.sync()
        lat.append(time.perf_counter() - a)
        b += 1
    # the same call with host-resident inputs: pinned staging copy + H2D inside the call
    host_edges, host_wall = 0, 0.0
    if HOST:
        hb = [st.batch(b + i) for i in range(HOST)]
        # untimed: once per process, about ten calls into a run of back-to-back host batches, one call takes 6 ms
        # (the runtime sets something up lazily for copies on a stream that has work queued behind events;
        # copies on the idle stream at create time do not trigger it) -- not part of the steady-state rate
        n_pre = min(16, HOST // 2)
        for s_, d_, t_, e_ in hb[:n_pre]:
            g.ingest_batch(s_, d_, t_, e_)
        g.sync()
        a = time.perf_counter()
        for s_, d_, t_, e_ in hb[n_pre:]:
            g.ingest_batch(s_, d_, t_, e_)
            host_edges += len(s_)
        g.sync()
        host_wall = time.perf_counter() - a
        b += HOST
    for _ in range(min(20, KER)):      # stage split from the library's own events (adds a sync per batch)
        s = feed(b, stats=True); b += 1
        stage_us += np.array([s["us_stage"][k] for k in ("sort", "memory", "apply", "propagate", "embed", "total")])
    n_stage = min(20, KER)
    kernel_pass = [b, b + KER - n_stage]

    # per-kernel durations from HIP events on the library's stream
    g.kernel_times(enable=True, reset=True)
    totk0 = g.totals()
    n_ker = 0
    for _ in range(KER - n_stage):
        feed(b); b += 1; n_ker += 1
    kt = g.kernel_times(enable=False, reset=False)
    totk1 = g.totals()
    n_layer_launches = max(n_ker * w.layers, 1)
    rows_per_launch = (totk1["rows"] - totk0["rows"]) / n_layer_launches              # rows a layer launch recomputes
    entries_per_launch = (totk1["gathered"] - totk0["gathered"]) / n_layer_launches    # ring records per launch

    # An event pair around an empty kernel measures what the bracketing itself costs (the command
    # processor handles two marker packets and one dispatch); it is subtracted from every class.
    overhead_us = kt["noop"]["usec"] / kt["noop"]["launches"] if kt.get("noop", {}).get("launches") else 0.0
    kernels = {}
    for name, v in kt.items():
        if v["launches"] and name != "noop":
            raw = v["usec"] / v["launches"]
            kernels[name] = {"avg_us": max(raw - overhead_us, 0.05), "avg_us_with_event_overhead": raw,
                             "launches": v["launches"]}
            kernels[name]["total_us"] = kernels[name]["avg_us"] * v["launches"]
    roofline = None
    if kernels:
        qf = np.mean([projection_flops_per_row(w, l, args.delta_mode)[0] for l in range(w.layers)])
        of = np.mean([projection_flops_per_row(w, l, args.delta_mode)[1] for l in range(w.layers)])
        layer_bytes = algorithmic_bytes(w, rows_per_launch, entries_per_launch)
        if "layer" in kernels:
            # the fused layer kernel gathers (HBM) and projects (fp32 MFMA); per row the gather is the
            # larger of the two at the published peaks, so HBM is the bounding roof
            s_ = kernels["layer"]["avg_us"] * 1e-6
            kernels["layer"]["algorithmic_GBs"] = layer_bytes / s_ / 1e9
            kernels["layer"]["frac_hbm"] = kernels["layer"]["algorithmic_GBs"] / HBM_PEAK_GBS
            kernels["layer"]["projection_TFLOPs"] = (qf + of) * rows_per_launch / s_ / 1e12
            kernels["layer"]["frac_mfma_f32"] = kernels["layer"]["projection_TFLOPs"] / MFMA_F32_PEAK_TFLOPS
        dom = max(kernels, key=lambda k: kernels[k]["total_us"])
        roofline = {"kernel": "layer", "bound": "hbm", "achieved": kernels["layer"]["algorithmic_GBs"],
                    "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": kernels["layer"]["frac_hbm"], "traffic": None,
                    "mfma_f32_frac": kernels["layer"]["frac_mfma_f32"]}
        if dom != "layer":
            roofline["note"] = f"largest total time is in {dom}, which moves too little data for a roofline"
        # what the kernel's own data layout asks the memory system for (cached key|value rows): more
        # bytes than the plain definition needs, priced separately and never used for `achieved`
        lay = layout_bytes(w, rows_per_launch, entries_per_launch, args.delta_mode)
        roofline["layout_bytes_per_launch"] = lay
        roofline["layout_GBs"] = lay / (kernels["layer"]["avg_us"] * 1e-6) / 1e9
        roofline["layout_frac"] = roofline["layout_GBs"] / HBM_PEAK_GBS
        roofline["rows_per_launch"] = rows_per_launch
        roofline["ring_entries_per_launch"] = entries_per_launch
        roofline["avg_launch_us"] = kernels[roofline["kernel"]]["avg_us"]
        roofline["event_overhead_us"] = overhead_us
        roofline["batches"] = kernel_pass
        roofline["traffic"] = stored_traffic(w.name, kernel_pass)

    # delta mode: how far the cached rows have moved from what an exact recomputation of the same state gives
    delta = None
    if args.delta_mode:
        rng = np.random.default_rng(5)
        probe = rng.choice(w.num_nodes, size=min(w.num_nodes, 200_000), replace=False).astype(np.uint32)
        gdrift, tracked = g.drift_status()
        approx = g.get_embeddings(probe).astype(np.float64)
        g.full_rebuild()
        exact = g.get_embeddings(probe).astype(np.float64)
        dev_ = np.linalg.norm(approx - exact, axis=1) / (np.linalg.norm(exact, axis=1) + 1e-30)
        moved = dev_ > 0
        delta = {"drift_gamma": args.drift_gamma, "global_drift": gdrift, "tracked_nodes": tracked,
                 "maintain_every": args.maintain_every, "delta_max": args.delta_max, "alpha": args.alpha,
                 "maintain_actions": {"none": maintained[0], "partial": maintained[1], "full": maintained[2]},
                 "probe_rows": int(len(probe)), "rows_off_exact": int(moved.sum()),
                 "rel_deviation_p50": float(np.percentile(dev_[moved], 50)) if moved.any() else 0.0,
                 "rel_deviation_p99": float(np.percentile(dev_[moved], 99)) if moved.any() else 0.0,
                 "rel_deviation_max": float(dev_.max())}

    # full_rebuild(): every layer over all N rows, the largest launches this path has
    rebuild = None
    if args.rebuilds > 0:
        g.full_rebuild(); g.sync()
        tr0 = g.totals()
        a = time.perf_counter()
        for _ in range(args.rebuilds):
            g.full_rebuild()
        g.sync()
        rw = (time.perf_counter() - a) / args.rebuilds
        tr1 = g.totals()
        ent = (tr1["gathered"] - tr0["gathered"]) / args.rebuilds          # ring records over all layers
        rb_bytes = w.layers * algorithmic_bytes(w, w.num_nodes, ent / w.layers)        # every row, every layer
        # a rebuild projects every row of every layer and gathers few entries per row (most nodes of a skewed
        # graph hold short lists): at the published peaks its fp32 matrix work takes longer than its bytes
        rb_flops = w.num_nodes * sum(sum(projection_flops_per_row(w, l, args.delta_mode)) for l in range(w.layers))
        rebuild = {"ms": rw * 1e3, "node_layers_per_s": w.num_nodes * w.layers / rw,
                   "algorithmic_GBs": rb_bytes / rw / 1e9, "frac_hbm": rb_bytes / rw / 1e9 / HBM_PEAK_GBS,
                   "projection_TFLOPs": rb_flops / rw / 1e12,
                   "frac_mfma_f32": rb_flops / rw / 1e12 / MFMA_F32_PEAK_TFLOPS,
                   "bound": "mfma" if rb_flops / (MFMA_F32_PEAK_TFLOPS * 1e12) > rb_bytes / (HBM_PEAK_GBS * 1e9) else "hbm",
                   "ring_entries": ent / w.layers}

    # per-batch root-node inference (Algorithm 1: embed and score the batch's endpoints BEFORE the batch is
    # applied): link scores of one batch of edges from the current state, device inputs, call + wait.
    # Prediction changes no state, so the same batch can be scored repeatedly.
    roots = None
    if args.predict_reps > 0:
        rng = np.random.default_rng(1)
        g.set_predictor((rng.standard_normal(2 * w.d_emb) / np.sqrt(w.d_emb)).astype(np.float32), 0.0)
        lo = (b if (b + 1) * w.batch <= used else b - 1) * w.batch
        ps, pd, pt = d_src[lo:lo + w.batch], d_dst[lo:lo + w.batch], d_ts[lo:lo + w.batch]
        roots = {"edges": int(ps.shape[0])}
        for name, mode in (("cached_rows", False), ("edge_time", True)):
            g.predict_batch(ps, pd, pt, at_edge_time=mode); g.sync()
            a = time.perf_counter()
            for _ in range(args.predict_reps):
                g.predict_batch(ps, pd, pt, at_edge_time=mode)
                g.sync()
            dt_ = (time.perf_counter() - a) / args.predict_reps
            roots[name + "_us"] = dt_ * 1e6
            roots[name + "_edges_per_s"] = ps.shape[0] / dt_

    cpu = None
    if not args.no_cpu and args.cpu_steps > 0:
        cpu = cpu_baseline(w, st, weights, nf, Q, args.cpu_steps, note, plan, plan_rows)

    lat_ms = np.array(lat) * 1e3 if lat else np.array([float("nan")])
    out = {
        "metric": "streamed_edges_per_s",
        "value": edges / wall,
        "unit": "edges/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "ms_per_step": 1e3 * wall / K,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "mode": "delta (approximate embeddings; not the headline configuration)" if args.delta_mode else "exact",
        "delta_mode": delta,
        "config": {"workload": f"{w.name}: {w.num_nodes} nodes, {w.num_edges} edges, Zipf s={w.zipf_s}, "
                               f"d_edge={w.d_edge}, d={w.d_emb}, k={w.k}, heads={w.heads}, layers={w.layers}, "
                               f"batch={w.batch}, {'TGN' if w.d_mem else 'TGAT (memoryless)'}",
                   "batch": w.batch, "layers": w.layers, "k": w.k, "timed_batches": [P + W, P + W + K],
                   "state_building_batches": P, "diagnostic_passes_from_batch": Q},
        "p50_batch_latency_ms": float(np.percentile(lat_ms, 50)),
        "p95_batch_latency_ms": float(np.percentile(lat_ms, 95)),
        "affected_embeddings_per_s": aff / wall,
        # the same count over the time of the layer launches alone (per-stage pass, serial path)
        "affected_embeddings_per_s_of_embed_stage": (aff / K) / (stage_us[4] / max(n_stage, 1) * 1e-6) if n_stage and stage_us[4] > 0 else None,
        "mean_affected": aff / K,
        "mean_rows_recomputed_per_layer": (tot1["rows"] - tot0["rows"]) / K / w.layers,
        "mean_direct": direct / K,
        "affected_fraction": aff / K / w.num_nodes,
        "paper_bound_2BLK": binding.paper_affected_bound(w.batch, w.k, w.layers),
        "host_input_edges_per_s": (host_edges / host_wall) if host_wall else None,
        "full_rebuild": rebuild,
        "root_inference": roots,
        "stage_us": dict(zip(("sort", "memory", "apply", "propagate", "embed", "total"),
                             (stage_us / max(n_stage, 1)).round(2).tolist())),
        "kernels": kernels,
        "roofline": roofline,
        "cpu_baseline": cpu,
        "workspace_GiB": g.workspace_bytes / 2**30,
    }
    g.close()
    # a plain elementwise copy (reads 1 GiB, writes 1 GiB per launch): what the memory system delivers to the
    # simplest streaming kernel on this machine, beside the published peak; under a counter run the same launches
    # give the scale of the byte counters (--calibrate-copy keeps that name)
    a_ = torch.empty(1 << 28, dtype=torch.float32, device=dev)
    b_ = torch.zeros(1 << 28, dtype=torch.float32, device=dev)
    torch.mul(b_, 1.0, out=a_)          # the first launch also pages the memory in
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(4):
        torch.mul(b_, 1.0, out=a_)
    e1.record()
    torch.cuda.synchronize()
    copy_gbs = 4 * 2 * (1 << 30) / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del a_, b_
    # a bare gather with the layer launch's own mix (rows recomputed, entries per row, a 1 KiB cached row and
    # a 256-byte or 1 KiB edge row per entry, uniformly random rows of tables of the workload's sizes): what the
    # memory system delivers to the kernel's access pattern when nothing else is asked of the chip
    gather = None
    if out["roofline"] is not None and w.num_nodes >= 32768:
        rows_l = max(int(out["roofline"]["rows_per_launch"]), 1)
        per = max(int(round(out["roofline"]["ring_entries_per_launch"] / rows_l)), 1)
        rows_l = max(int(round(out["roofline"]["ring_entries_per_launch"] / per)), 1)     # groups: the launch's entry count
        edge_floats = 64 if raw_edge_rows(w, args.delta_mode) else 256 if w.d_edge else 0
        g_rows = min(w.num_edges, (8 << 30) // (4 * max(edge_floats, 1)))          # at most 8 GiB of edge rows
        tn = torch.empty((w.num_nodes, 256), dtype=torch.float32, device=dev).normal_()
        te = torch.empty((g_rows, edge_floats), dtype=torch.float32, device=dev).normal_() if edge_floats else None
        gen = torch.Generator(device=dev).manual_seed(7)
        i_n = torch.randint(0, w.num_nodes, (rows_l * per,), device=dev, generator=gen).to(torch.int32)
        i_e = torch.randint(0, g_rows, (rows_l * per,), device=dev, generator=gen).to(torch.int32) if edge_floats else None
        o_ = torch.empty(rows_l * 16, dtype=torch.float32, device=dev)
        cs = torch.cuda.current_stream().cuda_stream
        def one():
            binding.probe_gather(tn, i_n, per, o_, cs)
            if te is not None:
                binding.probe_gather(te, i_e, per, o_, cs)
        one()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(4):
            one()
        e1.record()
        torch.cuda.synchronize()
        g_us = e0.elapsed_time(e1) * 1e3 / 4
        g_bytes = rows_l * per * 4 * (256 + edge_floats)
        gather = {"us": g_us, "GBs": g_bytes / g_us / 1e3, "groups": rows_l, "entries_per_group": per,
                  "bytes_per_entry": 4 * (256 + edge_floats),
                  "layer_launch_over_bare_gather": out["roofline"]["avg_launch_us"] / g_us}
        del tn, te, i_n, i_e, o_
    if out["roofline"] is not None:
        out["roofline"]["bare_gather"] = gather
        out["roofline"]["measured_copy_GBs"] = copy_gbs
        out["roofline"]["frac_of_measured_copy"] = out["roofline"]["achieved"] / copy_gbs
        if out["roofline"]["traffic"]:
            out["roofline"]["traffic_GBs"] = out["roofline"]["traffic"] / (out["roofline"]["avg_launch_us"] * 1e-6) / 1e9
    print(json.dumps(out))


if __name__ == "__main__":
    main()
