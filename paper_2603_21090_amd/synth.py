"""Seeded synthetic temporal-graph streams and random-init weights.

This module only draws random inputs (edge streams, feature rows, weight
matrices); it contains none of the method's arithmetic.  Both the CPU oracle
tests and the HIP library tests/bench read their inputs from here, so the two
sides see byte-identical buffers without sharing any code of the method.

The five workloads mirror the shapes of the paper's datasets (Table of
datasets in the evaluation section): node/edge counts, edge-feature width,
power-law (Zipf) endpoint popularity and chronological timestamps.  None of the
real datasets is used; every stream is generated from a counter-based Philox
generator keyed by (seed, purpose, chunk).
"""
from __future__ import annotations

import dataclasses
import math

import numpy as np

BASE_SEED = 260321000

# purposes for Philox keys (second key word)
_K_ENDPOINTS, _K_PERM, _K_TIME, _K_EFEAT, _K_WEIGHT, _K_NODEFEAT = 1, 2, 3, 4, 5, 6

EFEAT_CHUNK = 4096  # edges per independently keyed feature chunk


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    index: int
    num_nodes: int
    num_edges: int
    zipf_s: float
    d_edge: int
    batch: int
    k: int
    layers: int
    heads: int = 2
    d_mem: int = 100      # 0 => memoryless (TGAT-style)
    d_node: int = 0
    d_time: int = 100
    d_emb: int = 100
    d_msg: int = 100
    bipartite: tuple | None = None   # (n_left, n_right): src from left, dst from right
    window: float = 0.0              # temporal window T_w of the neighbour cache; 0 = no expiry
    aggregator: int = 0              # message aggregation per node and batch: 0 Last, 1 Mean, 2 Sum

    @property
    def seed(self) -> int:
        return BASE_SEED + self.index

    @property
    def num_batches(self) -> int:
        return (self.num_edges + self.batch - 1) // self.batch

    def scaled(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)


WORKLOADS = {
    "C1": Workload("C1", 1, 2_000, 20_000, 1.1, 16, 200, 10, 1),
    "C2": Workload("C2", 2, 10_000, 200_000, 1.2, 172, 200, 10, 2, bipartite=(8_000, 2_000)),
    "C3": Workload("C3", 3, 100_000, 1_000_000, 1.1, 172, 1_000, 10, 2),
    "C4": Workload("C4", 4, 1_000_000, 10_000_000, 1.1, 100, 2_000, 10, 2),
    "C5": Workload("C5", 5, 2_600_000, 30_000_000, 1.05, 64, 2_000, 20, 2, d_mem=0, d_node=100),
}


def _rng(seed: int, purpose: int, chunk: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed & 0xFFFFFFFFFFFFFFFF,
                                                     (purpose << 40) | chunk]))


def _zipf_ranks(rng: np.random.Generator, n_items: int, s: float, count: int) -> np.ndarray:
    """`count` draws of a rank in [0, n_items) with P(rank r) ~ (r+1)^-s (inverse CDF)."""
    w = np.arange(1, n_items + 1, dtype=np.float64) ** (-s)
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    u = rng.random(count)
    return np.minimum(np.searchsorted(cdf, u, side="left"), n_items - 1).astype(np.int64)


class EdgeStream:
    """Chronological edge list (src, dst, ts) plus lazily generated edge-feature rows."""

    def __init__(self, w: Workload):
        self.w = w
        E, N = w.num_edges, w.num_nodes
        rng = _rng(w.seed, _K_ENDPOINTS)
        if w.bipartite is None:
            perm = _rng(w.seed, _K_PERM).permutation(N)
            src = perm[_zipf_ranks(rng, N, w.zipf_s, E)]
            dst = perm[_zipf_ranks(rng, N, w.zipf_s, E)]
            # redraw destinations that collide with their source
            bad = np.nonzero(src == dst)[0]
            while bad.size:
                dst[bad] = perm[_zipf_ranks(rng, N, w.zipf_s, bad.size)]
                bad = bad[src[bad] == dst[bad]]
        else:
            nl, nr = w.bipartite
            assert nl + nr == N
            pl = _rng(w.seed, _K_PERM, 0).permutation(nl)
            pr = _rng(w.seed, _K_PERM, 1).permutation(nr) + nl
            src = pl[_zipf_ranks(rng, nl, w.zipf_s, E)]
            dst = pr[_zipf_ranks(rng, nr, w.zipf_s, E)]
        self.src = np.ascontiguousarray(src, dtype=np.uint32)
        self.dst = np.ascontiguousarray(dst, dtype=np.uint32)
        gaps = _rng(w.seed, _K_TIME).standard_exponential(E)
        self.ts = np.cumsum(gaps, dtype=np.float64)

    def edge_features(self, lo: int, hi: int) -> np.ndarray:
        """fp32 N(0,1) rows for edges [lo, hi); any slice reproduces the same values."""
        de = self.w.d_edge
        out = np.empty((hi - lo, de), dtype=np.float32)
        if de == 0 or hi <= lo:
            return out
        c0, c1 = lo // EFEAT_CHUNK, (hi - 1) // EFEAT_CHUNK
        for c in range(c0, c1 + 1):
            blk = _rng(self.w.seed, _K_EFEAT, c).standard_normal((EFEAT_CHUNK, de), dtype=np.float32)
            a, b = max(lo, c * EFEAT_CHUNK), min(hi, (c + 1) * EFEAT_CHUNK)
            out[a - lo:b - lo] = blk[a - c * EFEAT_CHUNK:b - c * EFEAT_CHUNK]
        return out

    def batch(self, b: int):
        """(src, dst, ts, efeat) of batch index b."""
        lo = b * self.w.batch
        hi = min(lo + self.w.batch, self.w.num_edges)
        return self.src[lo:hi], self.dst[lo:hi], self.ts[lo:hi], self.edge_features(lo, hi)


def node_features(w: Workload) -> np.ndarray | None:
    if w.d_node == 0:
        return None
    return _rng(w.seed, _K_NODEFEAT).standard_normal((w.num_nodes, w.d_node), dtype=np.float32)


def _uniform(rng, fan_in: int, shape) -> np.ndarray:
    b = 1.0 / math.sqrt(fan_in)
    return rng.uniform(-b, b, size=shape).astype(np.float32)


def make_weights(w: Workload, seed: int | None = None) -> dict:
    """Random-init parameters, all fp32, matrices row-major [in x out] (y = x @ W).

    Time encoding uses the paper's paired layout: frequency j drives a cosine
    column (phase 0) and a sine column (phase -pi/2); frequencies form a geometric
    ladder from 1 down to 1e-9 so every scale of the time gaps matters.
    """
    seed = w.seed if seed is None else seed
    rng = _rng(seed, _K_WEIGHT)
    dt, dm, dn, de, d, dmsg = w.d_time, w.d_mem, w.d_node, w.d_edge, w.d_emb, w.d_msg
    half = dt // 2
    lad = 10.0 ** (-9.0 * np.arange(half) / max(half - 1, 1))
    omega = np.repeat(lad, 2)[:dt].astype(np.float32)
    phase = np.tile(np.array([0.0, -math.pi / 2]), half)[:dt].astype(np.float32)
    if dt % 2:
        omega = np.append(omega, np.float32(lad[-1] if half else 1.0)).astype(np.float32)[:dt]
        phase = np.append(phase, np.float32(0.0)).astype(np.float32)[:dt]
    out = {"omega": omega, "phase": phase}
    if dm > 0:
        kin = 2 * dm + de + dt
        out["W_msg"] = _uniform(rng, kin, (kin, dmsg))
        out["b_msg"] = _uniform(rng, kin, (dmsg,))
        for g in "zrh":
            out[f"W_{g}"] = _uniform(rng, dmsg, (dmsg, dm))
            out[f"U_{g}"] = _uniform(rng, dm, (dm, dm))
            out[f"b_{g}"] = _uniform(rng, dm, (dm,))
    for name in ("W_Q", "W_K", "W_V", "W_O", "b_O"):
        out[name] = []
    for l in range(1, w.layers + 1):
        din = (dm + dn) if l == 1 else d
        out["W_Q"].append(_uniform(rng, din + dt, (din + dt, d)))
        out["W_K"].append(_uniform(rng, din + de + dt, (din + de + dt, d)))
        out["W_V"].append(_uniform(rng, din + de + dt, (din + de + dt, d)))
        out["W_O"].append(_uniform(rng, d, (d, d)))
        out["b_O"].append(_uniform(rng, d, (d,)))
    return out
