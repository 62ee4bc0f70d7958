"""Full-graph graph-attention (GAT) layers: forward, loss and backward in fp64 numpy.

TEST INFRASTRUCTURE ONLY (see ``oracle/__init__.py``).

The paper evaluates GAT as a second model family and notes that attention needs the gathered
inputs themselves in the backward pass (section on grad-engine activation regathering); it
does not restate the layer and gives no head count, so the definition is the published one
(Velickovic et al., "Graph Attention Networks"), as PyG's ``GATConv`` computes it; with one head:

    H = A^{l-1} W                                   [n, f]
    e(u -> v) = LeakyReLU_0.2(a_src . H[u] + a_dst . H[v])      for u in N(v) + {v}
    alpha(u -> v) = softmax over the sources u of v
    Z[v] = sum_u alpha(u -> v) H[u];   A^l = act(Z + b),  act = ReLU on hidden layers

With several heads every head runs these formulas on its own f / heads columns of H, a_src, a_dst
and the heads' rows of Z are concatenated (the published layer's rule for hidden layers; taken for
every layer here, a model that wants a single head at the output says so per layer).

``N(v)`` is row ``v`` of the CSR (sources of v) and every vertex gets exactly one self-loop,
as in the GCN operator.  Everything is written per edge with plain numpy gathers and
``np.add.at`` scatters, in the order of the formulas.
"""
from __future__ import annotations

import numpy as np

from . import fullgraph

SLOPE = 0.2


def edges_with_self_loops(rowptr, colidx):
    """(dst, src) arrays of the attention graph: the CSR's entries plus one self-loop for every
    vertex that has none, sorted by (dst, src)."""
    n = len(rowptr) - 1
    dst = np.repeat(np.arange(n, dtype=np.int64), np.diff(rowptr))
    src = np.asarray(colidx, dtype=np.int64)
    has = np.zeros(n, dtype=bool)
    has[dst[dst == src]] = True
    extra = np.flatnonzero(~has)
    dst = np.concatenate([dst, extra])
    src = np.concatenate([src, extra])
    order = np.lexsort((src, dst))
    return dst[order], src[order]


def layer_forward(dst, src, n, A, W, a_src, a_dst, b, relu, heads=1):
    """One layer with ``heads`` attention heads: head j owns columns [j f, (j+1) f) of H, of the
    attention vectors and of the output (f = d_out / heads), takes its own softmax over the
    sources of every vertex, and the heads' results stand side by side (concatenation)."""
    H = A @ W
    f = H.shape[1] // heads
    assert f * heads == H.shape[1], "the output width must be a multiple of the head count"
    Hh = H.reshape(n, heads, f)
    s_src = np.einsum("nhf,hf->nh", Hh, a_src.reshape(heads, f))
    s_dst = np.einsum("nhf,hf->nh", Hh, a_dst.reshape(heads, f))
    x = s_src[src] + s_dst[dst]                                   # [entries, heads]
    e = np.where(x > 0, x, SLOPE * x)
    m = np.full((n, heads), -np.inf)
    np.maximum.at(m, dst, e)
    ex = np.exp(e - m[dst])
    den = np.zeros((n, heads))
    np.add.at(den, dst, ex)
    alpha = ex / den[dst]
    Z = np.zeros_like(Hh)
    np.add.at(Z, dst, alpha[:, :, None] * Hh[src])
    Z = Z.reshape(n, heads * f)
    Y = Z + (b if b is not None else 0.0)
    out = np.maximum(Y, 0.0) if relu else Y
    return out, dict(H=H, x=x, alpha=alpha, Z=Z, heads=heads)


def layer_backward(dst, src, n, A, W, a_src, a_dst, cache, dY):
    """Gradients of one layer given dLoss/d(Z + b) = ``dY``."""
    H, x, alpha, heads = cache["H"], cache["x"], cache["alpha"], cache["heads"]
    f = H.shape[1] // heads
    Hh = H.reshape(n, heads, f)
    dYh = dY.reshape(n, heads, f)
    dH = np.zeros_like(Hh)
    np.add.at(dH, src, alpha[:, :, None] * dYh[dst])             # through Z = sum alpha H[u]
    dalpha = np.einsum("ehf,ehf->eh", dYh[dst], Hh[src])
    t = np.zeros((n, heads))
    np.add.at(t, dst, alpha * dalpha)
    de = alpha * (dalpha - t[dst])                               # softmax
    dx = de * np.where(x > 0, 1.0, SLOPE)                        # LeakyReLU
    ds_src = np.zeros((n, heads))
    ds_dst = np.zeros((n, heads))
    np.add.at(ds_src, src, dx)
    np.add.at(ds_dst, dst, dx)
    da_src = np.einsum("nhf,nh->hf", Hh, ds_src).reshape(-1)
    da_dst = np.einsum("nhf,nh->hf", Hh, ds_dst).reshape(-1)
    dH += ds_src[:, :, None] * a_src.reshape(1, heads, f) + ds_dst[:, :, None] * a_dst.reshape(1, heads, f)
    dH = dH.reshape(n, heads * f)
    return dict(gW=A.T @ dH, ga_src=da_src, ga_dst=da_dst, gb=dY.sum(axis=0), gA=dH @ W.T)


def forward(rowptr, colidx, dims, X, weights, drop=None):
    """``weights``: per layer a dict with ``W`` [d_in, d_out], ``a_src``, ``a_dst`` [d_out],
    ``b`` [d_out] or None, and optionally ``heads`` (default 1; must divide d_out).  Returns the activations A^1..A^L and the per-layer caches."""
    n = len(rowptr) - 1
    dst, src = edges_with_self_loops(rowptr, colidx)
    L = len(dims) - 1
    A = np.asarray(X, dtype=np.float64)
    acts, caches = [], []
    for l in range(L):
        w = weights[l]
        A_in = A
        A, cache = layer_forward(dst, src, n, A_in, np.asarray(w["W"], dtype=np.float64),
                                 np.asarray(w["a_src"], dtype=np.float64),
                                 np.asarray(w["a_dst"], dtype=np.float64),
                                 None if w.get("b") is None else np.asarray(w["b"], dtype=np.float64),
                                 relu=l < L - 1, heads=int(w.get("heads", 1)))
        cache["A_in"] = A_in
        cache["on"] = A > 0                              # ReLU decision, before any dropout
        if drop is not None and l < L - 1 and l < len(drop) and drop[l] is not None:
            # dropout after the activation of a hidden layer: multipliers 0 or 1 / (1 - p)
            A = A * np.asarray(drop[l], dtype=np.float64)
        acts.append(A)
        caches.append(cache)
    return acts, caches, (dst, src)


def epoch(rowptr, colidx, dims, X, weights, labels, mask, relu_on=None, drop=None):
    """One full-graph epoch.  Returns ``act``, ``loss``, ``gW``, ``ga_src``, ``ga_dst``, ``gb``
    (lists per layer) and ``gact`` (dLoss/dA^1..dLoss/dA^L).  ``drop``: optional list with one
    ``[n, d_l]`` array of dropout multipliers (0 or 1 / (1 - p)) or None per hidden layer, applied
    after the activation (``act`` then holds the activations after dropout, ``gact`` the gradient
    with respect to them)."""
    n = len(rowptr) - 1
    L = len(dims) - 1
    acts, caches, (dst, src) = forward(rowptr, colidx, dims, X, weights, drop=drop)
    lossv, G = fullgraph.loss(acts[-1], labels, mask)
    out = {"act": acts, "loss": lossv, "gW": [None] * L, "ga_src": [None] * L, "ga_dst": [None] * L,
           "gb": [None] * L, "gact": [None] * L}
    for l in range(L - 1, -1, -1):
        out["gact"][l] = G
        if l < L - 1:
            on = caches[l]["on"] if relu_on is None or relu_on[l] is None else (np.asarray(relu_on[l]) != 0)
            dY = G * on
            if drop is not None and l < len(drop) and drop[l] is not None:
                dY = dY * np.asarray(drop[l], dtype=np.float64)
        else:
            dY = G
        w = weights[l]
        g = layer_backward(dst, src, n, caches[l]["A_in"], np.asarray(w["W"], dtype=np.float64),
                           np.asarray(w["a_src"], dtype=np.float64),
                           np.asarray(w["a_dst"], dtype=np.float64), caches[l], dY)
        out["gW"][l], out["ga_src"][l], out["ga_dst"][l] = g["gW"], g["ga_src"], g["ga_dst"]
        out["gb"][l] = g["gb"] if w.get("b") is not None else None
        G = g["gA"]
    out["gX"] = G
    return out


def train(rowptr, colidx, dims, X, weights, labels, mask, epochs, optimizer="adam", lr=0.01, beta1=0.9,
          beta2=0.999, eps=1e-8, weight_decay=0.0, dropout=0.0, seed=0, first_epoch=0):
    """``epochs`` training epochs of the attention model: forward with dropout on the hidden
    activations (the multipliers of ``fullgraph.dropout_multipliers``), loss, backward, one
    optimizer step (``fullgraph.adam_step`` / ``sgd_step``) on W, the two attention vectors and
    the bias of every layer.  Returns the losses, the final weights (the layout of ``weights``)
    and the last epoch's results."""
    L = len(dims) - 1
    n = len(rowptr) - 1
    keys = ("W", "a_src", "a_dst", "b")
    cur = [{k: (None if w.get(k) is None else np.asarray(w[k], dtype=np.float64).copy()) for k in keys}
           for w in weights]
    heads = [int(w.get("heads", 1)) for w in weights]
    flat = lambda ws: [w[k] for w in ws for k in keys]
    m = [None if t is None else np.zeros_like(t) for t in flat(cur)]
    v = [None if t is None else np.zeros_like(t) for t in flat(cur)]
    losses, last = [], None
    for e in range(epochs):
        ep = first_epoch + e
        drop = None
        if dropout > 0:
            drop = [fullgraph.dropout_multipliers(n, dims[l + 1], dropout, seed, ep, l + 1) for l in range(L - 1)]
        seen = [dict(w, heads=h) for w, h in zip(cur, heads)]
        last = epoch(rowptr, colidx, dims, X, seen, labels, mask, drop=drop)
        losses.append(last["loss"])
        grads = [t for l in range(L) for t in (last["gW"][l], last["ga_src"][l], last["ga_dst"][l], last["gb"][l])]
        if optimizer == "adam":
            new, m, v = fullgraph.adam_step(flat(cur), grads, m, v, ep + 1, lr, beta1, beta2, eps, weight_decay)
        else:
            new = fullgraph.sgd_step(flat(cur), grads, lr, weight_decay)
        cur = [dict(zip(keys, new[4 * l:4 * l + 4])) for l in range(L)]
    return losses, [dict(w, heads=h) for w, h in zip(cur, heads)], last
