"""Small shared test utilities (no method arithmetic of the GPU path, none of the oracle's)."""
import numpy as np

from synth import csr_from_edges, rmat_graph


def small_graph(n, m_draw, seed, symmetric=True, self_loops=False):
    return rmat_graph(n, m_draw, seed, symmetric=symmetric, self_loops=self_loops)


def ring_graph(n, r):
    """r-regular ring lattice (r even): v is joined to v +- 1 .. v +- r/2."""
    src, dst = [], []
    for v in range(n):
        for s in range(1, r // 2 + 1):
            for u in ((v + s) % n, (v - s) % n):
                src.append(u)
                dst.append(v)
    from synth import csr_from_edges
    return csr_from_edges(n, np.array(src), np.array(dst))


def complete_graph(n, self_loops):
    from synth import csr_from_edges
    s, t = np.meshgrid(np.arange(n), np.arange(n))
    s, t = s.ravel(), t.ravel()
    if not self_loops:
        keep = s != t
        s, t = s[keep], t[keep]
    return csr_from_edges(n, s, t)


def empty_graph(n):
    return np.zeros(n + 1, dtype=np.int64), np.zeros(0, dtype=np.int32)


def rel_err(got, ref):
    """max |got - ref| / max |ref| over the tensor (the gate used for parity)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if ref.size == 0:
        return 0.0
    den = np.abs(ref).max()
    num = np.abs(got - ref).max()
    return float(num / den) if den > 0 else float(num)


def random_weights(dims, seed, sage, bias=True):
    rng = np.random.default_rng(seed)
    out = []
    for l in range(len(dims) - 1):
        a = np.sqrt(6.0 / (dims[l] + dims[l + 1]))
        out.append({
            "W": rng.uniform(-a, a, (dims[l], dims[l + 1])),
            "Ws": rng.uniform(-a, a, (dims[l], dims[l + 1])) if sage else None,
            "b": 0.1 * rng.standard_normal(dims[l + 1]) if bias else None,
        })
    return out


def aligned_backward(og, fwd, got_act, weights, X, labels, mask, tol, say=None):
    """Oracle backward with the activation decisions of the other implementation on the
    elements where the two disagree, after checking that each disagreement is legitimate:
    the oracle's pre-activation and the other side's activation both lie within
    ``tol * max|A^l|`` of zero, i.e. inside the forward tolerance band, where either decision
    is a correct result.  Returns the oracle's backward dict (plus ``act``)."""
    relu_on = []
    L = fwd.L
    for l in range(L - 1):
        on_got = np.asarray(got_act[l]) > 0
        on_ref = fwd.act[l] > 0
        diff = np.argwhere(on_got != on_ref)
        band = tol * np.abs(fwd.act[l]).max()
        prev = np.asarray(X, dtype=np.float64) if l == 0 else fwd.act[l - 1]
        W = np.asarray(weights[l]["W"], dtype=np.float64)
        Ws = weights[l].get("Ws")
        b = weights[l].get("b")
        if len(diff):
            v, c = diff[:, 0], diff[:, 1]
            pre = np.einsum("ij,ji->i", fwd.z[l][v], W[:, c])
            if Ws is not None and fwd.m == 1:
                pre = pre + np.einsum("ij,ji->i", prev[v], np.asarray(Ws, dtype=np.float64)[:, c])
            if b is not None:
                pre = pre + np.asarray(b, dtype=np.float64)[c]
            assert np.abs(pre).max() <= band, (l, float(np.abs(pre).max()), band)
            assert np.abs(np.asarray(got_act[l])[v, c]).max() <= band
        if say:
            say("layer %d: %d of %d activation decisions differ, all within +-%.2g of zero"
                % (l + 1, len(diff), on_ref.size, band))
        on = on_ref.astype(np.uint8)
        if len(diff):
            on[diff[:, 0], diff[:, 1]] = on_got[diff[:, 0], diff[:, 1]]
        relu_on.append(on)
    out = og.backward(fwd, labels, mask, relu_on=relu_on)
    out["act"] = fwd.act
    return out


def ring_of_blocks(k, per, seed):
    """k groups of `per` vertices on a ring: every vertex aggregates from a few vertices of its
    own group and of the next group on the ring; group ids are scrambled."""
    rng = np.random.default_rng(seed)
    label = rng.permutation(k)                       # position on the ring -> partition id
    n = k * per
    part = np.empty(n, dtype=np.int32)
    src, dst = [], []
    for pos in range(k):
        ids = np.arange(pos * per, (pos + 1) * per)
        part[ids] = label[pos]
        nxt = np.arange(((pos + 1) % k) * per, ((pos + 1) % k + 1) * per)
        for v in ids:
            for u in list(rng.choice(ids, 3, replace=False)) + list(rng.choice(nxt, 2, replace=False)):
                src.append(int(u)); dst.append(int(v))
                src.append(int(v)); dst.append(int(u))
    pairs = np.unique(np.array(dst, dtype=np.int64) * n + np.array(src, dtype=np.int64))
    rowptr, colidx = csr_from_edges(n, pairs % n, pairs // n)
    return rowptr, colidx, part, label


def gat_sampled_errors(rowptr, colidx, dims, weights, X, act, gact, gb, V, say=None):
    """Graph-attention layers checked on the sampled vertices ``V`` of a symmetric graph whose
    CSR holds no self-loops: rows ``V`` of every layer's output, every bias gradient, and rows
    ``V`` of every hidden input gradient, each recomputed in fp64 from the layer's definition
    (one head, LeakyReLU slope 0.2, one self-loop per vertex) and from the given tensors of the
    step before (``act``: A^1..A^L, ``gact``: dLoss/dA^1..dLoss/dA^L).  Returns the relative
    errors by name.

    The softmax gradient of an edge u -> v needs sum_u' alpha(u' -> v) dY[v] . H[u'], which is
    dY[v] . Z[v]; Z = A^l - b wherever dY is not zero (dY vanishes where the ReLU is off)."""
    n = len(rowptr) - 1
    L = len(dims) - 1
    deg = np.diff(rowptr)
    dst = np.concatenate([np.repeat(np.arange(n, dtype=np.int64), deg), np.arange(n, dtype=np.int64)])
    src = np.concatenate([np.asarray(colidx, dtype=np.int64), np.arange(n, dtype=np.int64)])
    assert not np.any(dst[:rowptr[-1]] == src[:rowptr[-1]])
    assert np.array_equal(np.bincount(colidx, minlength=n), deg)        # mirrored edges
    A = [X] + list(act)

    def leaky(x):
        return np.where(x > 0, x, 0.2 * x)

    def around(v):
        """Sources of v (= targets of v: the graph is symmetric), v itself included."""
        return np.concatenate([np.asarray(colidx[rowptr[v]:rowptr[v + 1]], dtype=np.int64), [v]])

    worst = {}
    for l in range(L, 0, -1):
        W = np.asarray(weights[l - 1]["W"], dtype=np.float64)
        a_s = np.asarray(weights[l - 1]["a_src"], dtype=np.float64)
        a_d = np.asarray(weights[l - 1]["a_dst"], dtype=np.float64)
        b = np.asarray(weights[l - 1]["b"], dtype=np.float64)
        H = np.empty((n, dims[l]))
        for r0 in range(0, n, 1 << 18):
            H[r0:r0 + (1 << 18)] = np.asarray(A[l - 1][r0:r0 + (1 << 18)], dtype=np.float64) @ W
        s_src, s_dst = H @ a_s, H @ a_d

        # forward rows by the definition
        ref = []
        for v in V:
            u = around(v)
            e = leaky(s_src[u] + s_dst[v])
            ex = np.exp(e - e.max())
            z = (ex / ex.sum()) @ H[u] + b
            ref.append(np.maximum(z, 0.0) if l < L else z)
        worst["act[%d] rows" % (l - 1)] = rel_err(np.asarray(A[l])[V], np.array(ref))

        # per-vertex softmax statistics over all edges, then the input gradient of sampled rows
        e = leaky(s_src[src] + s_dst[dst])
        mx = np.full(n, -np.inf)
        np.maximum.at(mx, dst, e)
        den = np.zeros(n)
        np.add.at(den, dst, np.exp(e - mx[dst]))
        del e
        dY = np.asarray(gact[l - 1], dtype=np.float64)
        if l < L:
            dY = np.where(np.asarray(A[l]) > 0, dY, 0.0)
        c = np.einsum("ij,ij->i", dY, np.asarray(A[l], dtype=np.float64) - b)
        worst["gb[%d]" % (l - 1)] = rel_err(gb[l - 1], dY.sum(axis=0))
        if l == 1:
            break                                   # the gradient of the input features is not kept
        ref = []
        for u in V:
            t = around(u)
            # edges u -> t
            x = s_src[u] + s_dst[t]
            alpha = np.exp(leaky(x) - mx[t]) / den[t]
            dx = alpha * (dY[t] @ H[u] - c[t]) * np.where(x > 0, 1.0, 0.2)
            dH = alpha @ dY[t] + dx.sum() * a_s
            # edges t -> u
            x = s_src[t] + s_dst[u]
            alpha = np.exp(leaky(x) - mx[u]) / den[u]
            dx = alpha * (H[t] @ dY[u] - c[u]) * np.where(x > 0, 1.0, 0.2)
            dH = dH + dx.sum() * a_d
            ref.append(dH @ W.T)
        worst["gact[%d] rows" % (l - 2)] = rel_err(np.asarray(gact[l - 2])[V], np.array(ref))
        if say:
            say("layer %d checked" % l)
    return worst
