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
