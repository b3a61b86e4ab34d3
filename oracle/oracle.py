"""ctypes front end of the CPU oracle (test infrastructure only).

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this
module.  It builds `liboracle.so` from `stgn_oracle.cpp` with g++ when the library
is missing and exposes the oracle's C entry points with NumPy arguments.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "stgn_oracle.cpp")
_LIB = os.path.join(_HERE, "liboracle.so")

_f32p = C.POINTER(C.c_float)
_f64p = C.POINTER(C.c_double)
_u32p = C.POINTER(C.c_uint32)


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["g++", "-O2", "-std=c++17", "-Wall", "-shared", "-fPIC", "-o", _LIB, _SRC])
    return _LIB


class _Config(C.Structure):
    _fields_ = [(n, C.c_uint32) for n in
                ("num_nodes", "d_mem", "d_node", "d_edge", "d_time", "d_emb", "d_msg", "k", "heads", "layers")] + \
               [("window", C.c_double), ("aggregator", C.c_uint32), ("reserved", C.c_uint32)]


class _Weights(C.Structure):
    _fields_ = [(n, _f32p) for n in
                ("omega", "phase", "W_msg", "b_msg", "W_z", "U_z", "b_z", "W_r", "U_r", "b_r", "W_h", "U_h", "b_h")] + \
               [(n, C.POINTER(_f32p)) for n in ("W_Q", "W_K", "W_V", "W_O", "b_O")]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_create.restype = C.c_void_p
        _lib.orc_create.argtypes = [C.POINTER(_Config), C.POINTER(_Weights), _f32p]
        _lib.orc_destroy.argtypes = [C.c_void_p]
        _lib.orc_ingest.restype = C.c_int
        _lib.orc_ingest.argtypes = [C.c_void_p, C.c_uint32, _u32p, _u32p, _f64p, _f32p, _u32p, _u32p, _u32p, _u32p]
        _lib.orc_embed_all.argtypes = [C.c_void_p, _f32p]
        _lib.orc_embed_nodes.argtypes = [C.c_void_p, C.c_uint32, C.c_uint32, _u32p, _f32p]
        _lib.orc_predict.argtypes = [C.c_void_p, C.c_uint32, _u32p, _u32p, _f64p, C.c_int, _f32p, C.c_float, _f64p]
        _lib.orc_neighbors.restype = C.c_uint32
        _lib.orc_neighbors.argtypes = [C.c_void_p, C.c_uint32, _u32p, _u32p, _f64p]
        _lib.orc_degree.restype = C.c_uint32
        _lib.orc_degree.argtypes = [C.c_void_p, C.c_uint32]
        _lib.orc_memory.argtypes = [C.c_void_p, C.c_uint32, _u32p, _f32p, _f64p]
        _lib.orc_set_memory.argtypes = [C.c_void_p, C.c_uint32, _u32p, _f32p, _f64p]
        _lib.orc_delta_enable.argtypes = [C.c_void_p, C.c_double]
        _lib.orc_delta_rows.argtypes = [C.c_void_p, C.c_uint32, C.c_uint32, _u32p, _f32p]
        _lib.orc_delta_attn.restype = C.c_uint32
        _lib.orc_delta_attn.argtypes = [C.c_void_p, C.c_uint32, C.c_uint32, _f64p, _f64p]
        _lib.orc_delta_last_fractions.argtypes = [C.c_void_p, _f32p]
        _lib.orc_drift_status.argtypes = [C.c_void_p, _f64p, _u32p, _f64p]
        _lib.orc_maintain.restype = C.c_int
        _lib.orc_maintain.argtypes = [C.c_void_p, C.c_double, C.c_double, _u32p]
        _lib.orc_delta_full_rebuild.argtypes = [C.c_void_p]
        _lib.orc_time_encode.argtypes = [C.c_uint32, _f32p, _f32p, C.c_double, _f64p]
        _lib.orc_message.argtypes = [C.c_void_p, _f32p, _f32p, _f32p, C.c_double, _f64p]
        _lib.orc_gru.argtypes = [C.c_uint32, C.c_uint32] + [_f32p] * 9 + [_f64p] * 3
        _lib.orc_attention.argtypes = [C.c_uint32, C.c_uint32, C.c_uint32, _f64p, _f64p, _f64p, _f32p, _f32p, _f64p]
    return _lib


def _f32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float32)


def _p(a, t):
    return None if a is None else a.ctypes.data_as(t)


class Oracle:
    """Full-recompute TGN/TGAT state machine on the CPU."""

    def __init__(self, *, num_nodes, d_mem, d_node, d_edge, d_time, d_emb, d_msg, k, heads, layers,
                 weights: dict, node_feat=None, window=0.0, aggregator=0):
        L = lib()
        self.cfg = _Config(num_nodes, d_mem, d_node, d_edge, d_time, d_emb, d_msg, k, heads, layers, float(window),
                           int(aggregator), 0)
        self._keep = []
        w = _Weights()
        for name in ("omega", "phase", "W_msg", "b_msg", "W_z", "U_z", "b_z", "W_r", "U_r", "b_r", "W_h", "U_h", "b_h"):
            a = _f32(weights.get(name))
            self._keep.append(a)
            setattr(w, name, _p(a, _f32p))
        for name in ("W_Q", "W_K", "W_V", "W_O", "b_O"):
            arrs = [_f32(a) for a in weights[name]]
            assert len(arrs) == layers
            self._keep.append(arrs)
            ptrs = (_f32p * layers)(*[_p(a, _f32p) for a in arrs])
            self._keep.append(ptrs)
            setattr(w, name, ptrs)
        nf = _f32(node_feat)
        self._h = L.orc_create(C.byref(self.cfg), C.byref(w), _p(nf, _f32p))
        if not self._h:
            raise ValueError("orc_create rejected the configuration")
        self.N, self.d_mem, self.d_emb, self.k, self.layers = num_nodes, d_mem, d_emb, k, layers
        self.d_edge = d_edge

    @classmethod
    def from_workload(cls, w, weights, node_feat=None):
        return cls(num_nodes=w.num_nodes, d_mem=w.d_mem, d_node=w.d_node, d_edge=w.d_edge, d_time=w.d_time,
                   d_emb=w.d_emb, d_msg=w.d_msg, k=w.k, heads=w.heads, layers=w.layers,
                   weights=weights, node_feat=node_feat, window=getattr(w, "window", 0.0),
                   aggregator=getattr(w, "aggregator", 0))

    def __del__(self):
        if getattr(self, "_h", None):
            lib().orc_destroy(self._h)
            self._h = None

    def ingest(self, src, dst, ts, efeat):
        """Returns (code, D, A): D = batch endpoints, A = affected set, both ascending."""
        src = np.ascontiguousarray(src, dtype=np.uint32)
        dst = np.ascontiguousarray(dst, dtype=np.uint32)
        ts = np.ascontiguousarray(ts, dtype=np.float64)
        ef = np.ascontiguousarray(efeat, dtype=np.float32).reshape(len(src), self.d_edge)
        D = np.empty(self.N, dtype=np.uint32)
        A = np.empty(self.N, dtype=np.uint32)
        nd, na = C.c_uint32(0), C.c_uint32(0)
        rc = lib().orc_ingest(self._h, len(src), _p(src, _u32p), _p(dst, _u32p), _p(ts, _f64p), _p(ef, _f32p),
                              _p(D, _u32p), C.byref(nd), _p(A, _u32p), C.byref(na))
        if rc != 0:
            return rc, None, None
        return 0, D[:nd.value].copy(), A[:na.value].copy()

    def embed_all(self) -> np.ndarray:
        out = np.empty((self.layers, self.N, self.d_emb), dtype=np.float32)
        lib().orc_embed_all(self._h, _p(out, _f32p))
        return out

    def embed_nodes(self, nodes, layer=None) -> np.ndarray:
        nodes = np.ascontiguousarray(nodes, dtype=np.uint32)
        layer = self.layers if layer is None else layer
        out = np.empty((len(nodes), self.d_emb), dtype=np.float32)
        lib().orc_embed_nodes(self._h, layer, len(nodes), _p(nodes, _u32p), _p(out, _f32p))
        return out

    def predict(self, src, dst, ts, w, b, at_edge_time=False) -> np.ndarray:
        """Link scores of a batch that has not been ingested yet (root embeddings from the current state)."""
        src = np.ascontiguousarray(src, dtype=np.uint32)
        dst = np.ascontiguousarray(dst, dtype=np.uint32)
        ts = np.ascontiguousarray(ts, dtype=np.float64)
        w = _f32(w)
        assert w.shape == (2 * self.d_emb,)
        out = np.empty(len(src), dtype=np.float64)
        lib().orc_predict(self._h, len(src), _p(src, _u32p), _p(dst, _u32p), _p(ts, _f64p), int(at_edge_time),
                          _p(w, _f32p), float(b), _p(out, _f64p))
        return out

    # ---- delta mode and drift-aware rebuild scheduling (approximate mode of the method)
    def delta_enable(self, gamma=0.9):
        """Switches the delta mode on: every later ingest refreshes the cached rows, exactly where a row's own
        input or query time changed, by the delta update elsewhere.  Rebuilds every cache exactly first."""
        lib().orc_delta_enable(self._h, float(gamma))

    def delta_rows(self, nodes, layer=None) -> np.ndarray:
        nodes = np.ascontiguousarray(nodes, dtype=np.uint32)
        layer = self.layers if layer is None else layer
        out = np.empty((len(nodes), self.d_emb), dtype=np.float32)
        lib().orc_delta_rows(self._h, layer, len(nodes), _p(nodes, _u32p), _p(out, _f32p))
        return out

    def delta_attn(self, node, layer=None):
        """(weights in effect, scores) of a row's attention cache, each [entries x heads]."""
        layer = self.layers if layer is None else layer
        H = self.cfg.heads
        a = np.zeros(self.k * H, dtype=np.float64)
        s = np.zeros(self.k * H, dtype=np.float64)
        n = lib().orc_delta_attn(self._h, layer, int(node), _p(a, _f64p), _p(s, _f64p))
        return a[:n * H].reshape(n, H).copy(), s[:n * H].reshape(n, H).copy()

    def delta_last_fractions(self) -> np.ndarray:
        out = np.empty(self.N, dtype=np.float32)
        lib().orc_delta_last_fractions(self._h, _p(out, _f32p))
        return out

    def drift_status(self):
        """(global drift metric, size of the cumulative affected set, per-node estimates)."""
        g, c = C.c_double(0.0), C.c_uint32(0)
        per = np.empty(self.N, dtype=np.float64)
        lib().orc_drift_status(self._h, C.byref(g), C.byref(c), _p(per, _f64p))
        return g.value, c.value, per

    def maintain(self, delta_max, alpha):
        """Adaptive rebuild policy; returns (action, drifted nodes): 0 nothing, 1 partial, 2 full rebuild."""
        n = C.c_uint32(0)
        act = lib().orc_maintain(self._h, float(delta_max), float(alpha), C.byref(n))
        return act, n.value

    def delta_full_rebuild(self):
        lib().orc_delta_full_rebuild(self._h)

    def neighbors(self, node):
        nbr = np.empty(self.k, dtype=np.uint32)
        eid = np.empty(self.k, dtype=np.uint32)
        ts = np.empty(self.k, dtype=np.float64)
        n = lib().orc_neighbors(self._h, int(node), _p(nbr, _u32p), _p(eid, _u32p), _p(ts, _f64p))
        return nbr[:n].copy(), eid[:n].copy(), ts[:n].copy()

    def degree(self, node) -> int:
        return lib().orc_degree(self._h, int(node))

    def memory(self, nodes):
        nodes = np.ascontiguousarray(nodes, dtype=np.uint32)
        mem = np.empty((len(nodes), self.d_mem), dtype=np.float32)
        tl = np.empty(len(nodes), dtype=np.float64)
        lib().orc_memory(self._h, len(nodes), _p(nodes, _u32p), _p(mem, _f32p), _p(tl, _f64p))
        return mem, tl

    def set_memory(self, nodes, mem=None, t_last=None):
        nodes = np.ascontiguousarray(nodes, dtype=np.uint32)
        mem = _f32(mem)
        tl = None if t_last is None else np.ascontiguousarray(t_last, dtype=np.float64)
        lib().orc_set_memory(self._h, len(nodes), _p(nodes, _u32p), _p(mem, _f32p), _p(tl, _f64p))

    def message(self, s_self, s_other, e, dt) -> np.ndarray:
        s_self, s_other, e = _f32(s_self), _f32(s_other), _f32(e)
        out = np.empty(self.cfg.d_msg, dtype=np.float64)
        lib().orc_message(self._h, _p(s_self, _f32p), _p(s_other, _f32p), _p(e, _f32p), float(dt), _p(out, _f64p))
        return out


def time_encode(omega, phase, x) -> np.ndarray:
    omega, phase = _f32(omega), _f32(phase)
    out = np.empty(len(omega), dtype=np.float64)
    lib().orc_time_encode(len(omega), _p(omega, _f32p), _p(phase, _f32p), float(x), _p(out, _f64p))
    return out


def gru(W_z, U_z, b_z, W_r, U_r, b_r, W_h, U_h, b_h, m, s) -> np.ndarray:
    ws = [_f32(a) for a in (W_z, U_z, b_z, W_r, U_r, b_r, W_h, U_h, b_h)]
    d_msg, d_mem = ws[0].shape
    m = np.ascontiguousarray(m, dtype=np.float64)
    s = np.ascontiguousarray(s, dtype=np.float64)
    out = np.empty(d_mem, dtype=np.float64)
    lib().orc_gru(d_msg, d_mem, *[_p(a, _f32p) for a in ws], _p(m, _f64p), _p(s, _f64p), _p(out, _f64p))
    return out


def attention(q, K, V, W_O, b_O, heads) -> np.ndarray:
    q = np.ascontiguousarray(q, dtype=np.float64)
    d = len(q)
    K = np.ascontiguousarray(K, dtype=np.float64).reshape(-1, d)
    V = np.ascontiguousarray(V, dtype=np.float64).reshape(-1, d)
    W_O, b_O = _f32(W_O), _f32(b_O)
    out = np.empty(d, dtype=np.float64)
    lib().orc_attention(d, heads, K.shape[0], _p(q, _f64p), _p(K, _f64p), _p(V, _f64p),
                        _p(W_O, _f32p), _p(b_O, _f32p), _p(out, _f64p))
    return out
