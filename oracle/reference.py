"""ctypes front end of the C oracle (atgnn_oracle.c): compiles it with gcc on first use.

TEST INFRASTRUCTURE ONLY - see the header of atgnn_oracle.c.  All floating-point arrays cross this
boundary as float64; callers convert their fp32 / bf16-representable inputs exactly.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Dict, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "atgnn_oracle.c")
_LIB = os.path.join(_HERE, "libatgnn_oracle.so")
_MODEL = {"gt": 0, "gat": 1, "agnn": 2, "gatv2": 3}


class _CLayer(ctypes.Structure):
    _fields_ = [("model", ctypes.c_int32), ("H", ctypes.c_int32), ("D", ctypes.c_int32),
                ("scale", ctypes.c_double), ("neg_slope", ctypes.c_double), ("eps", ctypes.c_double)]


@dataclass
class Layer:
    model: str
    H: int
    D: int
    scale: float = 1.0       # GT: score scale, AGNN: beta
    neg_slope: float = 0.2   # GAT, GATv2
    eps: float = 1e-12       # AGNN

    def _c(self) -> _CLayer:
        return _CLayer(_MODEL[self.model], self.H, self.D, float(self.scale), float(self.neg_slope), float(self.eps))


def build_oracle(force: bool = False) -> str:
    """Compile the oracle: -O2, no fast-math, no OpenMP (single-threaded by construction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build_oracle())
        _lib.atgnn_oracle_forward.restype = ctypes.c_int
        _lib.atgnn_oracle_backward.restype = ctypes.c_int
    return _lib


def _f64(a: Optional[np.ndarray]):
    if a is None:
        return None, ctypes.c_void_p(None)
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(ctypes.c_void_p)


def _rows(rows):
    if rows is None:
        return None, ctypes.c_int64(0), ctypes.c_void_p(None)
    r = np.ascontiguousarray(rows, dtype=np.int64)
    return r, ctypes.c_int64(r.size), r.ctypes.data_as(ctypes.c_void_p)


def _graph(indptr, indices):
    ip = np.ascontiguousarray(indptr, dtype=np.int32)
    ix = np.ascontiguousarray(indices, dtype=np.int32)
    n = ip.size - 1
    assert ip[0] == 0 and ip[-1] == ix.size and np.all(np.diff(ip) >= 0)
    assert ix.size == 0 or (ix.min() >= 0 and ix.max() < n)
    return ip, ix, n


def forward(layer: Layer, indptr, indices, *, x, k=None, v=None, a_l=None, a_r=None, edge_bias=None, rows=None,
            want_p: bool = False) -> Dict[str, np.ndarray]:
    """x: GT Q / GAT Wh / AGNN h / GATv2 destination-side features, [N,H,D]; k: GT K / GATv2 source-side
    features; a_l: GAT left vector / GATv2 attention vector; edge_bias: optional [nnz,H] term added to the
    scores (CSR edge order).  Returns out [N,H,D], row_max, row_sum [N,H] (float64)
    and optionally p [nnz,H].  With `rows`, only those rows are filled (others stay NaN)."""
    lib = _load()
    ip, ix, n = _graph(indptr, indices)
    H, D = layer.H, layer.D
    x_, xp = _f64(x); k_, kp = _f64(k); v_, vp = _f64(v); al_, alp = _f64(a_l); ar_, arp = _f64(a_r)
    assert x_.size == n * H * D
    if layer.model == "gt":
        assert k_ is not None and v_ is not None and k_.size == x_.size and v_.size == x_.size
    if layer.model == "gat":
        assert al_ is not None and ar_ is not None and al_.size == H * D and ar_.size == H * D
    if layer.model == "gatv2":
        assert k_ is not None and k_.size == x_.size and al_ is not None and al_.size == H * D
    b_, bp = _f64(edge_bias)
    assert b_ is None or b_.size == ix.size * H
    r_, nr, rp = _rows(rows)
    fill = np.nan if rows is not None else 0.0
    out = np.full((n, H, D), fill, dtype=np.float64)
    rmax = np.full((n, H), fill, dtype=np.float64)
    rsum = np.full((n, H), fill, dtype=np.float64)
    p = np.full((ix.size, H), np.nan, dtype=np.float64) if want_p else None
    cl = layer._c()
    rc = lib.atgnn_oracle_forward(ctypes.byref(cl), ctypes.c_int64(n), ip.ctypes.data_as(ctypes.c_void_p),
                                  ix.ctypes.data_as(ctypes.c_void_p), xp, kp, vp, alp, arp, bp, nr, rp,
                                  out.ctypes.data_as(ctypes.c_void_p), rmax.ctypes.data_as(ctypes.c_void_p),
                                  rsum.ctypes.data_as(ctypes.c_void_p),
                                  p.ctypes.data_as(ctypes.c_void_p) if want_p else ctypes.c_void_p(None))
    if rc != 0:
        raise MemoryError("oracle forward failed")
    res = {"out": out, "row_max": rmax, "row_sum": rsum}
    if want_p:
        res["p"] = p
    return res


def backward(layer: Layer, indptr, indices, *, x, k=None, v=None, a_l=None, a_r=None, edge_bias=None, d_out,
             rows=None, want_ds: bool = False) -> Dict[str, np.ndarray]:
    """Gradients of sum(O * d_out): d_x [N,H,D]; GT also d_k, d_v; GAT also d_a_l, d_a_r [H,D];
    AGNN also d_scale (d beta); GATv2 also d_k, d_a_l; with want_ds, ds [nnz,H] (which is also the gradient
    of edge_bias).  With `rows`, see the completeness note in atgnn_oracle.c."""
    lib = _load()
    ip, ix, n = _graph(indptr, indices)
    H, D = layer.H, layer.D
    x_, xp = _f64(x); k_, kp = _f64(k); v_, vp = _f64(v); al_, alp = _f64(a_l); ar_, arp = _f64(a_r)
    g_, gp = _f64(d_out)
    b_, bp = _f64(edge_bias)
    assert x_.size == n * H * D and g_.size == x_.size
    assert b_ is None or b_.size == ix.size * H
    r_, nr, rp = _rows(rows)
    null = ctypes.c_void_p(None)
    dx = np.empty((n, H, D), dtype=np.float64)
    res = {"d_x": dx}
    dkp = dvp = dalp = darp = null
    if layer.model == "gt":
        res["d_k"] = np.empty((n, H, D), dtype=np.float64)
        res["d_v"] = np.empty((n, H, D), dtype=np.float64)
        dkp = res["d_k"].ctypes.data_as(ctypes.c_void_p)
        dvp = res["d_v"].ctypes.data_as(ctypes.c_void_p)
    if layer.model == "gat":
        res["d_a_l"] = np.empty((H, D), dtype=np.float64)
        res["d_a_r"] = np.empty((H, D), dtype=np.float64)
        dalp = res["d_a_l"].ctypes.data_as(ctypes.c_void_p)
        darp = res["d_a_r"].ctypes.data_as(ctypes.c_void_p)
    if layer.model == "gatv2":
        res["d_k"] = np.empty((n, H, D), dtype=np.float64)
        res["d_a_l"] = np.empty((H, D), dtype=np.float64)
        dkp = res["d_k"].ctypes.data_as(ctypes.c_void_p)
        dalp = res["d_a_l"].ctypes.data_as(ctypes.c_void_p)
    dscale = ctypes.c_double(0.0)
    ds = np.full((ix.size, H), np.nan, dtype=np.float64) if want_ds else None
    cl = layer._c()
    rc = lib.atgnn_oracle_backward(ctypes.byref(cl), ctypes.c_int64(n), ip.ctypes.data_as(ctypes.c_void_p),
                                   ix.ctypes.data_as(ctypes.c_void_p), xp, kp, vp, alp, arp, bp, gp, nr, rp,
                                   dx.ctypes.data_as(ctypes.c_void_p), dkp, dvp, dalp, darp, ctypes.byref(dscale),
                                   ds.ctypes.data_as(ctypes.c_void_p) if want_ds else null)
    if rc != 0:
        raise MemoryError("oracle backward failed")
    if layer.model == "agnn":
        res["d_scale"] = float(dscale.value)
    if want_ds:
        res["ds"] = ds
    return res
