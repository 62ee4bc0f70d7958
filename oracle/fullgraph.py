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


def forward(model, rowptr, colidx, dims, X, weights, drop=None):
    """Forward pass only.  Returns a ``Forward`` holding ``act`` (A^1..A^L) and ``z``.
    ``drop``: optional list with one ``[n, d_l]`` array of dropout multipliers (0 or 1/(1-p))
    or None per hidden layer; see :func:`dropout_multipliers`."""
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
    f.drop = [None] * f.L
    if drop is not None:
        for l in range(min(f.L - 1, len(drop))):
            if drop[l] is not None:
                f.drop[l] = _f64(drop[l])
                assert f.drop[l].shape == f.act[l].shape
    rc = lib().oracle_forward(
        C.c_int(f.m), C.c_int64(f.n), _p(f.rowptr, C.c_int64), _p(f.colidx, C.c_int32),
        C.c_int(f.L), _p(f.dims_a, C.c_int32), _p(f.X, C.c_double), _ptr_array(f.W),
        _ptr_array(f.Ws), _ptr_array(f.b), _ptr_array(f.drop), _ptr_array(f.act), _ptr_array(f.z))
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
        _p(mask, C.c_uint8), on_arr, _ptr_array(f.drop), C.byref(lossv), _ptr_array(gW), _ptr_array(gWs),
        _ptr_array(gb), _ptr_array(gact), _p(gX, C.c_double) if gX is not None else None)
    if rc != 0:
        raise MemoryError("oracle_backward failed")
    return {"loss": float(lossv.value), "gW": gW, "gWs": gWs, "gb": gb, "gact": gact, "gX": gX}


def epoch(model, rowptr, colidx, dims, X, weights, labels, mask, backward=True,
          input_grad=False, drop=None):
    """One full-graph epoch.

    ``weights``: list (one per layer) of dicts with ``W``, ``Ws`` (SAGE) and ``b`` (or None).
    Returns a dict: ``act`` (list of A^1..A^L), ``z`` (list of aggregated inputs Z^1..Z^L),
    ``loss``, and when ``backward``: ``gW``, ``gWs``, ``gb`` (lists) and ``gact``
    (list of dLoss/dA^1..dLoss/dA^L), plus ``gX`` = dLoss/dA^0 when ``input_grad``.
    """
    f = forward(model, rowptr, colidx, dims, X, weights, drop=drop)
    out = {"act": f.act, "z": f.z}
    if backward:
        out.update(globals()["backward"](f, labels, mask, input_grad=input_grad))
    else:
        out["loss"], _ = loss(f.act[-1], labels, mask, want_grad=False)
    return out


# ----------------------------------------------------------------------------------------
# training around the epoch (datasets table: learning rate, dropout, number of epochs)
# ----------------------------------------------------------------------------------------
_M64 = (1 << 64) - 1


def _splitmix64_vec(x):
    """SplitMix64 output for states ``x`` (numpy uint64, wrapping arithmetic)."""
    with np.errstate(over="ignore"):
        z = x + np.uint64(0x9E3779B97F4A7C15)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        return z ^ (z >> np.uint64(31))


def dropout_multipliers(n, d, p, seed, epoch_index, layer):
    """Multipliers (0 or 1/(1-p)) of the dropout that follows hidden layer ``layer`` (1-based)
    in epoch ``epoch_index``.  The paper fixes only the rate; the random stream is this
    build's: element ``(v, j)`` (``v`` an original vertex id) draws the 32-bit number
    ``splitmix64(key + v d + j) >> 32`` with ``key = splitmix64(seed xor
    splitmix64(64 epoch_index + layer))`` and is dropped when the draw is below
    ``floor(p 2^32)``, ``p`` rounded to single precision.  Counter-based, so it can be
    re-drawn anywhere and does not depend on the partitioning."""
    p32 = float(np.float32(p))
    thr = int(np.floor(p32 * 4294967296.0))
    inner = int(_splitmix64_vec(np.array([(64 * epoch_index + layer) & _M64], dtype=np.uint64))[0])
    key = _splitmix64_vec(np.array([(seed & _M64) ^ inner], dtype=np.uint64))[0]
    with np.errstate(over="ignore"):
        idx = np.arange(n * d, dtype=np.uint64) + key
    draw = _splitmix64_vec(idx) >> np.uint64(32)
    keepm = draw >= np.uint64(thr)
    return np.where(keepm, 1.0 / (1.0 - p32), 0.0).reshape(n, d)


def sgd_step(params, grads, lr, weight_decay=0.0):
    """``w <- w - lr (g + weight_decay w)`` for every tensor (None entries skipped)."""
    return [None if w is None else w - lr * (g + weight_decay * w) for w, g in zip(params, grads)]


def adam_step(params, grads, m, v, t, lr, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0):
    """One step of Adam (Kingma & Ba, algorithm 1) with L2 weight decay added to the gradient;
    ``t`` is the 1-based step number.  Returns the new ``(params, m, v)`` lists."""
    out_w, out_m, out_v = [], [], []
    for w, g, mi, vi in zip(params, grads, m, v):
        if w is None:
            out_w.append(None); out_m.append(None); out_v.append(None)
            continue
        g = g + weight_decay * w
        mi = beta1 * mi + (1.0 - beta1) * g
        vi = beta2 * vi + (1.0 - beta2) * g * g
        mhat = mi / (1.0 - beta1 ** t)
        vhat = vi / (1.0 - beta2 ** t)
        out_w.append(w - lr * mhat / (np.sqrt(vhat) + eps))
        out_m.append(mi)
        out_v.append(vi)
    return out_w, out_m, out_v


def train(model, rowptr, colidx, dims, X, weights, labels, mask, epochs, optimizer="adam",
          lr=0.01, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0, dropout=0.0, seed=0,
          first_epoch=0, relu_on=None, weight_round=None):
    """``epochs`` training epochs: forward with dropout on the hidden activations, loss,
    backward, one optimizer step.  Returns the losses, the final weights (same layout as
    ``weights``) and the last epoch's results.  ``relu_on``: optional callable
    ``(epoch, Forward) -> list`` giving activation decisions for the backward pass.
    ``weight_round``: optional callable applied to the matrices ``W`` and ``Ws`` (not the
    biases) before every forward pass, for weights kept in a narrower storage type: the epoch
    sees the rounded matrices, the optimizer steps the unrounded ones (weight decay included),
    and those are what is returned.  The paper trains in one precision; this is the customary
    master-copy arrangement."""
    L = len(dims) - 1
    n = len(rowptr) - 1
    sage = model == "sage"
    cur = [{"W": _f64(w["W"]).copy(), "Ws": _f64(w["Ws"]).copy() if sage else None,
            "b": _f64(w["b"]).copy() if w.get("b") is not None else None} for w in weights]
    flat = lambda ws: [t for w in ws for t in (w["W"], w["Ws"], w["b"])]
    m = [None if t is None else np.zeros_like(t) for t in flat(cur)]
    v = [None if t is None else np.zeros_like(t) for t in flat(cur)]
    losses, last = [], None
    for e in range(epochs):
        ep = first_epoch + e
        drop = None
        if dropout > 0:
            drop = [dropout_multipliers(n, dims[l + 1], dropout, seed, ep, l + 1) for l in range(L - 1)]
        seen = cur
        if weight_round is not None:
            seen = [{"W": _f64(weight_round(w["W"])), "Ws": _f64(weight_round(w["Ws"])) if sage else None,
                     "b": w["b"]} for w in cur]
        f = forward(model, rowptr, colidx, dims, X, seen, drop=drop)
        r = backward(f, labels, mask, relu_on=relu_on(ep, f) if relu_on else None)
        last = dict(r, act=f.act)
        losses.append(r["loss"])
        grads = [t for l in range(L) for t in (r["gW"][l], r["gWs"][l], r["gb"][l])]
        if optimizer == "adam":
            new, m, v = adam_step(flat(cur), grads, m, v, ep + 1, lr, beta1, beta2, eps, weight_decay)
        else:
            new = sgd_step(flat(cur), grads, lr, weight_decay)
        cur = [{"W": new[3 * l], "Ws": new[3 * l + 1], "b": new[3 * l + 2]} for l in range(L)]
    return losses, cur, last
