"""Thin ctypes binding of libstreamtgn (argument marshalling only).

PyTorch is used for two things: the device workspace (one uint8 tensor) and the HIP stream the
library enqueues its kernels on.  Every step of the method runs inside the library's kernels;
there is no Python or CPU fallback -- if the shared library is missing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libstreamtgn.so")

STGN_MAX_LAYERS = 4
ERRORS = {0: "OK", -1: "INVALID_ARG", -2: "NODE_OUT_OF_RANGE", -3: "TIME_ORDER", -4: "SELF_LOOP",
          -5: "BATCH_TOO_LARGE", -6: "EDGE_CAPACITY", -7: "DEVICE", -8: "WORKSPACE"}

_f32p = C.POINTER(C.c_float)
_u32p = C.POINTER(C.c_uint32)
_f64p = C.POINTER(C.c_double)


class Config(C.Structure):
    _fields_ = [("num_nodes", C.c_uint32), ("max_edges", C.c_uint64), ("max_batch", C.c_uint32),
                ("d_mem", C.c_uint32), ("d_node", C.c_uint32), ("d_edge", C.c_uint32), ("d_time", C.c_uint32),
                ("d_emb", C.c_uint32), ("d_msg", C.c_uint32), ("k", C.c_uint32), ("heads", C.c_uint32),
                ("layers", C.c_uint32), ("window", C.c_double), ("aggregator", C.c_uint32), ("delta_mode", C.c_uint32),
                ("drift_gamma", C.c_double)]


class Weights(C.Structure):
    _fields_ = [(n, _f32p) for n in
                ("omega", "phase", "W_msg", "b_msg", "W_z", "U_z", "b_z", "W_r", "U_r", "b_r", "W_h", "U_h", "b_h")] + \
               [(n, C.POINTER(_f32p)) for n in ("W_Q", "W_K", "W_V", "W_O", "b_O")]


class BatchStats(C.Structure):
    _fields_ = [("n_edges", C.c_uint32), ("n_direct", C.c_uint32), ("n_affected", C.c_uint32),
                ("frontier", C.c_uint32 * (STGN_MAX_LAYERS + 1)), ("entries_scanned", C.c_uint64),
                ("pull_hops", C.c_uint32), ("reserved", C.c_uint32), ("us_stage", C.c_float * 6)]

    def as_dict(self):
        return dict(n_edges=self.n_edges, n_direct=self.n_direct, n_affected=self.n_affected,
                    frontier=list(self.frontier), entries_scanned=self.entries_scanned, pull_hops=self.pull_hops,
                    us_stage=dict(zip(("sort", "memory", "apply", "propagate", "embed", "total"), self.us_stage)))


class StgnError(RuntimeError):
    def __init__(self, code, msg=""):
        super().__init__(f"libstreamtgn: {ERRORS.get(code, code)} ({code}) {msg}")
        self.code = code


_lib = None

EXPORTS = ("stgn_query_workspace", "stgn_create", "stgn_destroy", "stgn_ingest_batch", "stgn_get_embeddings",
           "stgn_full_rebuild", "stgn_sync", "stgn_get_affected", "stgn_get_neighbors", "stgn_get_history",
           "stgn_get_memory", "stgn_get_totals", "stgn_kernel_times", "stgn_last_error", "stgn_version",
           "stgn_set_predictor", "stgn_predict_batch", "stgn_predict_batch_static", "stgn_drift_status",
           "stgn_maintain", "stgn_probe_gather")


def load_library():
    """Loads libstreamtgn.so from the package directory; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2603_21090_amd.build` "
                          "(there is no fallback path)")
    L = C.CDLL(LIB_PATH)
    vp = C.c_void_p
    L.stgn_query_workspace.argtypes = [C.POINTER(Config), C.POINTER(C.c_size_t)]
    L.stgn_create.argtypes = [C.POINTER(Config), C.POINTER(Weights), vp, vp, C.c_size_t, vp, C.POINTER(vp)]
    L.stgn_destroy.argtypes = [vp]
    L.stgn_destroy.restype = None
    L.stgn_ingest_batch.argtypes = [vp, C.c_uint32, vp, vp, vp, vp, C.c_int, C.POINTER(BatchStats)]
    L.stgn_get_embeddings.argtypes = [vp, C.c_uint32, C.c_uint32, vp, vp, C.c_int]
    L.stgn_full_rebuild.argtypes = [vp]
    L.stgn_sync.argtypes = [vp]
    L.stgn_get_affected.argtypes = [vp, vp, C.c_uint32, _u32p]
    L.stgn_get_neighbors.argtypes = [vp, C.c_uint32, vp, vp, vp, _u32p]
    L.stgn_get_history.argtypes = [vp, C.c_uint32, C.c_uint32, C.c_uint32, vp, vp, _u32p]
    L.stgn_get_memory.argtypes = [vp, C.c_uint32, vp, vp, vp]
    L.stgn_get_totals.argtypes = [vp] + [C.POINTER(C.c_uint64)] * 6
    L.stgn_kernel_times.argtypes = [vp, C.c_int, C.c_int, C.c_uint32, C.POINTER(C.c_char_p), _f64p,
                                    C.POINTER(C.c_uint64)]
    L.stgn_set_predictor.argtypes = [vp, vp, C.c_float]
    L.stgn_predict_batch.argtypes = [vp, C.c_uint32, vp, vp, vp, C.c_int, C.c_int, vp]
    L.stgn_predict_batch_static.argtypes = [vp, C.c_uint32, vp, vp, vp, C.c_int, vp]
    L.stgn_drift_status.argtypes = [vp, C.POINTER(C.c_double), _u32p, vp]
    L.stgn_maintain.argtypes = [vp, C.c_double, C.c_double, C.POINTER(C.c_int), _u32p]
    L.stgn_probe_gather.argtypes = [vp, C.c_uint64, C.c_uint32, vp, C.c_uint32, C.c_uint32, vp, vp]
    L.stgn_last_error.argtypes = [vp]
    L.stgn_last_error.restype = C.c_char_p
    L.stgn_version.restype = C.c_char_p
    _lib = L
    return L


def _host_f32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float32)


def _ptr(a):
    return None if a is None else C.c_void_p(a.ctypes.data)


def make_config(*, num_nodes, max_edges, max_batch, d_mem, d_node, d_edge, d_time, d_emb, d_msg, k, heads, layers,
                window=0.0, aggregator=0, delta_mode=0, drift_gamma=0.0):
    return Config(num_nodes, max_edges, max_batch, d_mem, d_node, d_edge, d_time, d_emb, d_msg, k, heads, layers,
                  float(window), int(aggregator), int(delta_mode), float(drift_gamma))


def query_workspace(cfg: Config) -> int:
    n = C.c_size_t(0)
    rc = load_library().stgn_query_workspace(C.byref(cfg), C.byref(n))
    if rc:
        raise StgnError(rc, load_library().stgn_last_error(None).decode())
    return n.value


def probe_gather(table, idx, per_group, out, stream=0):
    """One launch of the bare gather (stgn_probe_gather) on torch device tensors: table [rows, 64 or 256] fp32,
    idx [groups * per_group] int32, out [groups * 16] fp32.  Asynchronous."""
    row_bytes = table.shape[1] * 4
    groups = idx.numel() // per_group
    rc = load_library().stgn_probe_gather(table.data_ptr(), table.shape[0], row_bytes, idx.data_ptr(), groups, per_group,
                                          out.data_ptr(), stream)
    if rc:
        raise StgnError(rc)


def _marshal_weights(weights: dict, layers: int, has_memory: bool):
    keep = []
    w = Weights()
    names = ["omega", "phase"] + (["W_msg", "b_msg", "W_z", "U_z", "b_z", "W_r", "U_r", "b_r", "W_h", "U_h", "b_h"]
                                   if has_memory else [])
    for name in names:
        a = _host_f32(weights[name])
        keep.append(a)
        setattr(w, name, a.ctypes.data_as(_f32p))
    for name in ("W_Q", "W_K", "W_V", "W_O", "b_O"):
        arrs = [_host_f32(a) for a in weights[name]]
        if len(arrs) != layers:
            raise ValueError(f"{name}: expected {layers} layers")
        ptrs = (_f32p * layers)(*[a.ctypes.data_as(_f32p) for a in arrs])
        keep += [arrs, ptrs]
        setattr(w, name, ptrs)
    return w, keep


class StreamTGN:
    """One device-resident serving state.  Methods mirror the C entry points one to one."""

    def __init__(self, cfg: Config, weights: dict, node_feat=None, device="cuda:0", stream=None):
        import torch
        self._L = load_library()
        self.cfg = cfg
        self._torch = torch
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        nbytes = query_workspace(cfg)
        self.workspace_bytes = nbytes
        self._ws = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
        base = (self._ws.data_ptr() + 255) & ~255
        self._stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        w, keep = _marshal_weights(weights, cfg.layers, cfg.d_mem > 0)
        nf = _host_f32(node_feat)
        if nf is not None and nf.shape != (cfg.num_nodes, cfg.d_node):
            raise ValueError("node_feat shape")
        h = C.c_void_p(None)
        rc = self._L.stgn_create(C.byref(cfg), C.byref(w), _ptr(nf), C.c_void_p(base), nbytes,
                                 C.c_void_p(self._stream.cuda_stream), C.byref(h))
        if rc:
            raise StgnError(rc, self._L.stgn_last_error(None).decode())
        self._h = h

    @classmethod
    def from_workload(cls, w, weights, node_feat=None, max_edges=None, max_batch=None, delta_mode=0, drift_gamma=0.0, **kw):
        cfg = make_config(num_nodes=w.num_nodes, max_edges=max_edges or w.num_edges, max_batch=max_batch or w.batch,
                          d_mem=w.d_mem, d_node=w.d_node, d_edge=w.d_edge, d_time=w.d_time, d_emb=w.d_emb,
                          d_msg=w.d_msg, k=w.k, heads=w.heads, layers=w.layers, window=getattr(w, "window", 0.0),
                          aggregator=getattr(w, "aggregator", 0), delta_mode=delta_mode, drift_gamma=drift_gamma)
        return cls(cfg, weights, node_feat, **kw)

    def close(self):
        if getattr(self, "_h", None):
            self._L.stgn_destroy(self._h)
            self._h = None
            self._ws = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc):
        if rc:
            raise StgnError(rc, self._L.stgn_last_error(self._h).decode())

    def last_error(self) -> str:
        return self._L.stgn_last_error(self._h).decode()

    # ---- hot path
    def ingest_batch(self, src, dst, ts, efeat, stats=False, check=True):
        """Host (NumPy) or device (torch, on this device) arrays; returns the code, or stats dict."""
        torch = self._torch
        on_dev = isinstance(src, torch.Tensor)
        n = int(src.shape[0])
        if on_dev:
            assert src.dtype == torch.int32 or src.dtype == torch.uint32
            assert ts.dtype == torch.float64 and (efeat is None or efeat.dtype == torch.float32)
            assert src.is_contiguous() and dst.is_contiguous() and ts.is_contiguous()
            assert efeat is None or efeat.is_contiguous()
            ptrs = [C.c_void_p(t.data_ptr()) if t is not None and t.numel() else None for t in (src, dst, ts, efeat)]
        else:
            src = np.ascontiguousarray(src, dtype=np.uint32)
            dst = np.ascontiguousarray(dst, dtype=np.uint32)
            ts = np.ascontiguousarray(ts, dtype=np.float64)
            efeat = None if efeat is None else np.ascontiguousarray(efeat, dtype=np.float32)
            ptrs = [_ptr(a) for a in (src, dst, ts, efeat)]
        st = BatchStats() if stats else None
        rc = self._L.stgn_ingest_batch(self._h, n, *ptrs, 1 if on_dev else 0, C.byref(st) if stats else None)
        if check:
            self._check(rc)
        if stats:
            return st.as_dict() if rc == 0 else rc
        return rc

    def get_embeddings(self, nodes, layer=0):
        torch = self._torch
        if isinstance(nodes, torch.Tensor):
            out = torch.empty((nodes.shape[0], self.cfg.d_emb), dtype=torch.float32, device=nodes.device)
            self._check(self._L.stgn_get_embeddings(self._h, layer, nodes.shape[0], C.c_void_p(nodes.data_ptr()),
                                                    C.c_void_p(out.data_ptr()), 1))
            return out
        nodes = np.ascontiguousarray(nodes, dtype=np.uint32)
        out = np.empty((len(nodes), self.cfg.d_emb), dtype=np.float32)
        self._check(self._L.stgn_get_embeddings(self._h, layer, len(nodes), _ptr(nodes), _ptr(out), 0))
        return out

    def set_predictor(self, w, b):
        w = np.ascontiguousarray(w, dtype=np.float32)
        assert w.shape == (2 * self.cfg.d_emb,)
        self._check(self._L.stgn_set_predictor(self._h, _ptr(w), float(b)))

    def predict_batch(self, src, dst, ts, at_edge_time=False):
        """Link scores of edges that have not been ingested yet: numpy in, numpy out (synchronises), or
        torch device tensors in, a device tensor out (asynchronous)."""
        torch = self._torch
        if isinstance(src, torch.Tensor):
            out = torch.empty(src.shape[0], dtype=torch.float32, device=src.device)
            self._check(self._L.stgn_predict_batch(self._h, src.shape[0], C.c_void_p(src.data_ptr()),
                                                   C.c_void_p(dst.data_ptr()), C.c_void_p(ts.data_ptr()),
                                                   int(at_edge_time), 1, C.c_void_p(out.data_ptr())))
            return out
        src = np.ascontiguousarray(src, dtype=np.uint32)
        dst = np.ascontiguousarray(dst, dtype=np.uint32)
        ts = np.ascontiguousarray(ts, dtype=np.float64)
        out = np.empty(len(src), dtype=np.float32)
        self._check(self._L.stgn_predict_batch(self._h, len(src), _ptr(src), _ptr(dst), _ptr(ts), int(at_edge_time), 0,
                                               _ptr(out)))
        return out

    def predict_batch_static(self, src, dst, ts, at_edge_time=False, out=None, check=True):
        """The variant that allocates nothing inside the library: device tensors in, scores into `out`
        (a device tensor the caller provides; created here when omitted).  Returns `out`, or the
        error code when check is off and the call failed."""
        torch = self._torch
        if out is None:
            out = torch.empty(src.shape[0], dtype=torch.float32, device=src.device)
        rc = self._L.stgn_predict_batch_static(self._h, src.shape[0], C.c_void_p(src.data_ptr()),
                                               C.c_void_p(dst.data_ptr()), C.c_void_p(ts.data_ptr()),
                                               int(at_edge_time), C.c_void_p(out.data_ptr()))
        if check:
            self._check(rc)
        return out if rc == 0 else rc

    def full_rebuild(self):
        self._check(self._L.stgn_full_rebuild(self._h))

    def drift_status(self, per_node=False):
        """(global drift metric, size of the cumulative affected set[, per-node estimates]) -- delta mode."""
        g, n = C.c_double(0.0), C.c_uint32(0)
        out = np.empty(self.cfg.num_nodes, dtype=np.float32) if per_node else None
        self._check(self._L.stgn_drift_status(self._h, C.byref(g), C.byref(n), _ptr(out)))
        return (g.value, n.value, out) if per_node else (g.value, n.value)

    def maintain(self, delta_max, alpha):
        """Adaptive rebuild policy; returns (action 0 none / 1 partial / 2 full, |V_drift|) -- delta mode."""
        act, nd = C.c_int(0), C.c_uint32(0)
        self._check(self._L.stgn_maintain(self._h, C.c_double(delta_max), C.c_double(alpha), C.byref(act), C.byref(nd)))
        return act.value, nd.value

    def sync(self, check=True):
        rc = self._L.stgn_sync(self._h)
        if check:
            self._check(rc)
        return rc

    # ---- inspection hooks
    def get_affected(self):
        out = np.empty(self.cfg.num_nodes, dtype=np.uint32)
        cnt = C.c_uint32(0)
        self._check(self._L.stgn_get_affected(self._h, _ptr(out), len(out), C.byref(cnt)))
        return out[:cnt.value].copy()

    def get_neighbors(self, node):
        k = self.cfg.k
        nbr, eid, ts = np.empty(k, np.uint32), np.empty(k, np.uint32), np.empty(k, np.float64)
        cnt = C.c_uint32(0)
        self._check(self._L.stgn_get_neighbors(self._h, int(node), _ptr(nbr), _ptr(eid), _ptr(ts), C.byref(cnt)))
        return nbr[:cnt.value].copy(), eid[:cnt.value].copy(), ts[:cnt.value].copy()

    def get_degree(self, node) -> int:
        dg = C.c_uint32(0)
        self._check(self._L.stgn_get_history(self._h, int(node), 0, 0, None, None, C.byref(dg)))
        return dg.value

    def get_history(self, node, first=0, count=None):
        dg = self.get_degree(node)
        count = dg - first if count is None else count
        nbr, eid = np.empty(count, np.uint32), np.empty(count, np.uint32)
        self._check(self._L.stgn_get_history(self._h, int(node), first, count, _ptr(nbr), _ptr(eid), None))
        return nbr, eid

    def get_memory(self, nodes):
        nodes = np.ascontiguousarray(nodes, dtype=np.uint32)
        mem = np.empty((len(nodes), self.cfg.d_mem), dtype=np.float32)
        tl = np.empty(len(nodes), dtype=np.float64)
        self._check(self._L.stgn_get_memory(self._h, len(nodes), _ptr(nodes), _ptr(mem) if self.cfg.d_mem else None,
                                            _ptr(tl)))
        return mem, tl

    def totals(self):
        v = [C.c_uint64(0) for _ in range(6)]
        self._check(self._L.stgn_get_totals(self._h, *[C.byref(x) for x in v]))
        return dict(zip(("edges", "direct", "affected", "scanned", "gathered", "rows"), [x.value for x in v]))

    def kernel_times(self, enable=True, reset=False):
        cap = 16
        names = (C.c_char_p * cap)()
        us = (C.c_double * cap)()
        ln = (C.c_uint64 * cap)()
        n = self._L.stgn_kernel_times(self._h, int(enable), int(reset), cap, names, us, ln)
        if n < 0:
            self._check(n)
        return {names[i].decode(): dict(usec=us[i], launches=ln[i]) for i in range(n)}


def paper_affected_bound(batch: int, fanout: int, layers: int) -> int:
    """The paper's bound 2 B L^K on the affected-set size (Eq. affected_bound); reported beside
    the measured |A| as context -- it belongs to a looser propagation rule than the exact one."""
    return 2 * batch * fanout ** layers
