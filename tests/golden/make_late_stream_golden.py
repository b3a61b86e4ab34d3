#!/usr/bin/env python3
"""Writes the expected values of the late-stream parity tests (tests/test_gpu_large.py).

The CPU oracle replays a workload's synthetic stream from the empty graph -- every batch, nothing
skipped -- and at each requested checkpoint (a batch index b: the state after batches 0 .. b) stores

  * |V_direct|, |V_aff| and a CRC-32 of the ascending affected set of batch b,
  * memory rows and last-interaction times of sampled endpoints of batch b,
  * layer-1 and final-layer rows (oracle `embed_nodes`, plain recursion) of sampled nodes inside and
    outside the affected set of batch b,

into tests/golden/late_stream_<workload>.npz (one entry group per checkpoint; the file is rewritten
after every checkpoint, so an interrupted replay keeps what it reached).  Only `oracle/` and the seeded
input generators are imported: no value in the file comes from the HIP path.

    python tests/golden/make_late_stream_golden.py C3 850 999
    python tests/golden/make_late_stream_golden.py C4 3500 4250

One core; C3 takes minutes, C4 hours (the oracle scans whole adjacency logs per batch).
"""
from __future__ import annotations

import os
import sys
import time
import zlib

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
sys.path.insert(0, ROOT)

from oracle import oracle as orc                      # noqa: E402
from paper_2603_21090_amd import synth                # noqa: E402

N_IN, N_OUT, N_MEM = 400, 200, 300


def main():
    name = sys.argv[1]
    checkpoints = sorted(int(x) for x in sys.argv[2:])
    w = synth.WORKLOADS[name]
    st = synth.EdgeStream(w)
    W = synth.make_weights(w)
    nf = synth.node_features(w)
    o = orc.Oracle.from_workload(w, W, nf)
    out_path = os.path.join(HERE, f"late_stream_{name}.npz")
    store = {"checkpoints": np.array([], dtype=np.int64)}
    allnodes = np.arange(w.num_nodes, dtype=np.uint32)
    t0 = time.time()
    for b in range(checkpoints[-1] + 1):
        rc, D, A = o.ingest(*st.batch(b))
        assert rc == 0
        if b % 50 == 0:
            print(f"[{name}] batch {b}  |D| {len(D)}  |A| {len(A)}  {time.time() - t0:.0f} s", flush=True)
        if b not in checkpoints:
            continue
        rng = np.random.default_rng(1000 * w.index + b)
        outside = np.setdiff1d(allnodes, A)
        s_in = np.sort(rng.choice(A, size=min(N_IN, len(A)), replace=False)).astype(np.uint32)
        s_out = np.sort(rng.choice(outside, size=min(N_OUT, len(outside)), replace=False)).astype(np.uint32)
        nodes = np.concatenate([s_in, s_out])
        key = f"b{b}_"
        store[key + "n_direct"] = np.int64(len(D))
        store[key + "n_affected"] = np.int64(len(A))
        store[key + "affected_crc32"] = np.int64(zlib.crc32(np.ascontiguousarray(A, dtype=np.uint32).tobytes()))
        store[key + "nodes"] = nodes
        store[key + "n_inside"] = np.int64(len(s_in))
        for layer in range(1, w.layers + 1):
            store[key + f"rows_l{layer}"] = o.embed_nodes(nodes, layer=layer)
        if w.d_mem:
            dm = np.sort(rng.choice(D, size=min(N_MEM, len(D)), replace=False)).astype(np.uint32)
            mem, tl = o.memory(dm)
            store[key + "mem_nodes"], store[key + "mem"], store[key + "t_last"] = dm, mem, tl
        store["checkpoints"] = np.append(store["checkpoints"], b)
        np.savez_compressed(out_path, **store)
        print(f"[{name}] checkpoint {b} written to {out_path}  ({time.time() - t0:.0f} s)", flush=True)


if __name__ == "__main__":
    main()
