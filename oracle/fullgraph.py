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


class Forward:
    """Inputs and results of one forward pass, kept so that the backward pass can follow."""


def forward(model, rowptr, colidx, dims, X, weights):
    """Forward pass only.  Returns a ``Forward`` holding ``act`` (A^1..A^L) and ``z``."""
    f = Forward()
    f.m = _MODEL[model]
    f.dims = [int(d) for d in dims]
    f.L = len(dims) - 1
    f.X = _f64(X)
    f.n = f.X.shape[0]
    assert f.X.shape[1] == dims[0]
    f.rowptr = np.ascontiguousarray(rowptr, dtype=np.int64)
    f.colidx = np.ascontiguousarray(colidx, dtype=np.int32)
    f.dims_a = np.ascontiguousarray(f.dims, dtype=np.int32)
    f.W = [_f64(w["W"]) for w in weights]
    f.Ws = [_f64(w["Ws"]) if (f.m == SAGE) else None for w in weights]
    f.b = [_f64(w["b"]) if w.get("b") is not None else None for w in weights]
    f.act = [np.empty((f.n, dims[l + 1]), dtype=np.float64) for l in range(f.L)]
    f.z = [np.empty((f.n, dims[l]), dtype=np.float64) for l in range(f.L)]
    rc = lib().oracle_forward(
        C.c_int(f.m), C.c_int64(f.n), _p(f.rowptr, C.c_int64), _p(f.colidx, C.c_int32),
        C.c_int(f.L), _p(f.dims_a, C.c_int32), _p(f.X, C.c_double), _ptr_array(f.W),
        _ptr_array(f.Ws), _ptr_array(f.b), _ptr_array(f.act), _ptr_array(f.z))
    if rc != 0:
        raise MemoryError("oracle_forward failed")
    return f


def backward(f, labels, mask, input_grad=False, relu_on=None):
    """Loss and backward pass after :func:`forward`.

    ``relu_on`` (optional): list with one uint8 ``[n, d_l]`` array (or None) per hidden layer
    giving the activation decision to use instead of ``act > 0``; see ``oracle_backward``.
    Returns ``loss``, ``gW``, ``gWs``, ``gb``, ``gact`` and ``gX`` (when ``input_grad``).
    """
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    gW = [np.zeros_like(w) for w in f.W]
    gWs = [np.zeros_like(w) if w is not None else None for w in f.Ws]
    gb = [np.zeros_like(x) if x is not None else None for x in f.b]
    gact = [np.empty_like(a) for a in f.act]
    gX = np.empty_like(f.X) if input_grad else None
    on_arr = None
    keep = []
    if relu_on is not None:
        on_arr = (C.POINTER(C.c_uint8) * max(1, f.L))()
        for l in range(f.L):
            a = relu_on[l] if l < len(relu_on) else None
            if a is not None:
                a = np.ascontiguousarray(a, dtype=np.uint8)
                assert a.shape == f.act[l].shape
                keep.append(a)
                on_arr[l] = _p(a, C.c_uint8)
            else:
                on_arr[l] = None
    lossv = C.c_double(0.0)
    rc = lib().oracle_backward(
        C.c_int(f.m), C.c_int64(f.n), _p(f.rowptr, C.c_int64), _p(f.colidx, C.c_int32),
        C.c_int(f.L), _p(f.dims_a, C.c_int32), _p(f.X, C.c_double), _ptr_array(f.W),
        _ptr_array(f.Ws), _ptr_array(f.act), _ptr_array(f.z), _p(labels, C.c_int32),
        _p(mask, C.c_uint8), on_arr, C.byref(lossv), _ptr_array(gW), _ptr_array(gWs),
        _ptr_array(gb), _ptr_array(gact), _p(gX, C.c_double) if gX is not None else None)
    if rc != 0:
        raise MemoryError("oracle_backward failed")
    return {"loss": float(lossv.value), "gW": gW, "gWs": gWs, "gb": gb, "gact": gact, "gX": gX}


def epoch(model, rowptr, colidx, dims, X, weights, labels, mask, backward=True,
          input_grad=False):
    """One full-graph epoch.

    ``weights``: list (one per layer) of dicts with ``W``, ``Ws`` (SAGE) and ``b`` (or None).
    Returns a dict: ``act`` (list of A^1..A^L), ``z`` (list of aggregated inputs Z^1..Z^L),
    ``loss``, and when ``backward``: ``gW``, ``gWs``, ``gb`` (lists) and ``gact``
    (list of dLoss/dA^1..dLoss/dA^L), plus ``gX`` = dLoss/dA^0 when ``input_grad``.
    """
    f = forward(model, rowptr, colidx, dims, X, weights)
    out = {"act": f.act, "z": f.z}
    if backward:
        out.update(globals()["backward"](f, labels, mask, input_grad=input_grad))
    else:
        out["loss"], _ = loss(f.act[-1], labels, mask, want_grad=False)
    return out
