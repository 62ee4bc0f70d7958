"""ctypes front end of ``fullgraph.c`` (the fp64 full-graph oracle).  Test infrastructure."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build as _build

GCN, SAGE = 0, 1
_MODEL = {"gcn": GCN, "sage": SAGE, GCN: GCN, SAGE: SAGE}
_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path) or os.path.getmtime(path) < os.path.getmtime(_build.SRC):
            _build.build()
        _lib = C.CDLL(path)
        _lib.oracle_loss.restype = C.c_double
        _lib.oracle_num_threads.restype = C.c_int
    return _lib


def _p(a, t):
    return a.ctypes.data_as(C.POINTER(t))


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _ptr_array(arrs):
    out = (C.POINTER(C.c_double) * max(1, len(arrs)))()
    for i, a in enumerate(arrs):
        out[i] = _p(a, C.c_double) if a is not None else None
    return out


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def set_num_threads(t: int) -> None:
    lib().oracle_set_num_threads(int(t))


def aggregate(model, rowptr, colidx, X, transpose=False):
    """``S X`` (or ``S^T X``) with ``S`` the model's normalised aggregation operator."""
    X = _f64(X)
    n, d = X.shape
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int64)
    colidx = np.ascontiguousarray(colidx, dtype=np.int32)
    Z = np.empty_like(X)
    fn = lib().oracle_aggregate_transpose if transpose else lib().oracle_aggregate
    rc = fn(C.c_int(_MODEL[model]), C.c_int64(n), _p(rowptr, C.c_int64), _p(colidx, C.c_int32),
            C.c_int64(d), _p(X, C.c_double), _p(Z, C.c_double))
    if rc != 0:
        raise MemoryError("oracle_aggregate failed")
    return Z


def loss(logits, labels, mask, want_grad=True):
    logits = _f64(logits)
    n, c = logits.shape
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    g = np.empty_like(logits) if want_grad else None
    val = lib().oracle_loss(C.c_int64(n), C.c_int64(c), _p(logits, C.c_double),
                            _p(labels, C.c_int32), _p(mask, C.c_uint8),
                            _p(g, C.c_double) if want_grad else None)
    return float(val), g


def epoch(model, rowptr, colidx, dims, X, weights, labels, mask, backward=True,
          input_grad=False):
    """One full-graph epoch.

    ``weights``: list (one per layer) of dicts with ``W``, ``Ws`` (SAGE) and ``b`` (or None).
    Returns a dict: ``act`` (list of A^1..A^L), ``z`` (list of aggregated inputs Z^1..Z^L),
    ``loss``, and when ``backward``: ``gW``, ``gWs``, ``gb`` (lists) and ``gact``
    (list of dLoss/dA^1..dLoss/dA^L), plus ``gX`` = dLoss/dA^0 when ``input_grad``.
    """
    m = _MODEL[model]
    L = len(dims) - 1
    X = _f64(X)
    n = X.shape[0]
    assert X.shape[1] == dims[0]
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int64)
    colidx = np.ascontiguousarray(colidx, dtype=np.int32)
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    dims_a = np.ascontiguousarray(dims, dtype=np.int32)
    W = [_f64(w["W"]) for w in weights]
    Ws = [_f64(w["Ws"]) if (m == SAGE) else None for w in weights]
    b = [_f64(w["b"]) if w.get("b") is not None else None for w in weights]
    act = [np.empty((n, dims[l + 1]), dtype=np.float64) for l in range(L)]
    z = [np.empty((n, dims[l]), dtype=np.float64) for l in range(L)]
    gW = [np.zeros_like(w) for w in W] if backward else [None] * L
    gWs = [np.zeros_like(w) if w is not None else None for w in Ws] if backward else [None] * L
    gb = [np.zeros_like(x) if x is not None else None for x in b] if backward else [None] * L
    gact = [np.empty_like(a) for a in act] if backward else [None] * L
    gX = np.empty_like(X) if (backward and input_grad) else None
    lossv = C.c_double(0.0)
    rc = lib().oracle_epoch(
        C.c_int(m), C.c_int64(n), _p(rowptr, C.c_int64), _p(colidx, C.c_int32), C.c_int(L),
        _p(dims_a, C.c_int32), _p(X, C.c_double), _ptr_array(W), _ptr_array(Ws), _ptr_array(b),
        _p(labels, C.c_int32), _p(mask, C.c_uint8), _ptr_array(act), _ptr_array(z),
        C.byref(lossv), C.c_int(1 if backward else 0), _ptr_array(gW), _ptr_array(gWs),
        _ptr_array(gb), _ptr_array(gact), _p(gX, C.c_double) if gX is not None else None)
    if rc != 0:
        raise MemoryError("oracle_epoch failed")
    out = {"act": act, "z": z, "loss": float(lossv.value)}
    if backward:
        out.update(gW=gW, gWs=gWs, gb=gb, gact=gact, gX=gX)
    return out
