"""Shared test helpers: tiny workloads and brute-force graph bookkeeping (no model arithmetic)."""
import numpy as np

from paper_2603_21090_amd import synth


def tiny_workload(**kw):
    base = dict(name="T", index=77, num_nodes=40, num_edges=400, zipf_s=1.1, d_edge=6, batch=20, k=3,
                layers=2, heads=2, d_mem=8, d_node=0, d_time=8, d_emb=8, d_msg=8)
    base.update(kw)
    return synth.Workload(**base)


def brute_rings(src, dst, n_edges, num_nodes, k):
    """Most recent k (nbr, eid) per node from the raw edge list, most recent first."""
    rings = [[] for _ in range(num_nodes)]
    for e in range(n_edges):
        rings[int(src[e])].append((int(dst[e]), e))
        rings[int(dst[e])].append((int(src[e]), e))
    return [list(reversed(r[-k:])) for r in rings]


def brute_affected(rings, direct, hops):
    """Pull formulation: w joins when any member of its ring is in the previous frontier."""
    A = set(int(v) for v in direct)
    frontier = set(A)
    for _ in range(hops):
        nxt = set()
        for w, ring in enumerate(rings):
            if w in A:
                continue
            if any(u in frontier for (u, _) in ring):
                nxt.add(w)
        A |= nxt
        frontier = nxt
    return np.array(sorted(A), dtype=np.uint32)


def row_err(got, ref):
    """Per-row relative error: max(||g-r||_2 / (||r||_2 + eps), max-norm ratio)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    d = got - ref
    e2 = np.linalg.norm(d, axis=-1) / (np.linalg.norm(ref, axis=-1) + 1e-30)
    return e2


def rows_close(got, ref, rel=1e-4, abs_=1e-6):
    """||g - r||_2 <= rel*||r||_2 + abs and the same in max-norm, for every row."""
    got = np.asarray(got, dtype=np.float64).reshape(-1, got.shape[-1])
    ref = np.asarray(ref, dtype=np.float64).reshape(-1, ref.shape[-1])
    d = got - ref
    ok2 = np.linalg.norm(d, axis=1) <= rel * np.linalg.norm(ref, axis=1) + abs_
    okm = np.abs(d).max(axis=1) <= rel * np.abs(ref).max(axis=1) + abs_
    return ok2 & okm


def rings_matrix(src, dst, n_edges, num_nodes, k):
    """Vectorised most-recent-k table from the raw edge list: nbr[N,k], eid[N,k] (most recent
    first, -1 padded) and the per-node degree.  Pure bookkeeping on the inputs."""
    s = np.asarray(src[:n_edges], dtype=np.int64)
    d = np.asarray(dst[:n_edges], dtype=np.int64)
    e = np.arange(n_edges, dtype=np.int64)
    node = np.concatenate([s, d])
    other = np.concatenate([d, s])
    eid = np.concatenate([e, e])
    # by node, then arrival: an edge appears once per node (no self loops), so (node, edge id) is a total
    # order and one 64-bit key sorts it
    order = np.argsort(node * np.int64(max(n_edges, 1)) + eid, kind="stable")
    node, other, eid = node[order], other[order], eid[order]
    deg = np.bincount(node, minlength=num_nodes)
    end = np.cumsum(deg)                              # one past the last entry of each node
    nbr_m = np.full((num_nodes, k), -1, dtype=np.int64)
    eid_m = np.full((num_nodes, k), -1, dtype=np.int64)
    for j in range(k):
        has = deg > j
        idx = end[has] - 1 - j
        nbr_m[has, j] = other[idx]
        eid_m[has, j] = eid[idx]
    return nbr_m, eid_m, deg


def affected_from_rings(nbr_m, direct, hops):
    """Pull formulation on the ring table: w joins when a member of its ring joined one hop ago."""
    N = nbr_m.shape[0]
    inA = np.zeros(N, dtype=bool)
    inA[np.asarray(direct, dtype=np.int64)] = True
    front = inA.copy()
    valid = nbr_m >= 0
    safe = np.where(valid, nbr_m, 0)
    for _ in range(hops):
        hit = (front[safe] & valid).any(axis=1) & ~inA
        inA |= hit
        front = hit
    return np.nonzero(inA)[0].astype(np.uint32)
