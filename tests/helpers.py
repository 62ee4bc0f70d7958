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


def elem_err(got, ref):
    """Element-wise relative error max_i |got_i - ref_i| / max(|ref_i|, 1e-3 max|ref|): reported
    next to the gate (it is stricter on small elements; not itself gated)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if ref.size == 0:
        return 0.0
    floor = 1e-3 * np.abs(ref).max()
    if floor == 0:
        return float(np.abs(got - ref).max())
    worst = 0.0
    flat_g, flat_r = got.reshape(-1), ref.reshape(-1)
    for i in range(0, flat_r.size, 1 << 26):          # by chunks: the tensors can hold 6e8 elements
        r = flat_r[i:i + (1 << 26)]
        worst = max(worst, float((np.abs(flat_g[i:i + (1 << 26)] - r) / np.maximum(np.abs(r), floor)).max()))
    return worst


def both_errs(got, ref):
    """(gate, element-wise) errors of one tensor."""
    return rel_err(got, ref), elem_err(got, ref)


def fmt_errs(worst):
    """'name=gate (elem)' for a dict name -> (gate, elem) or name -> gate."""
    out = []
    for k, v in sorted(worst.items()):
        out.append("%s=%.2g (elem %.2g)" % (k, v[0], v[1]) if isinstance(v, tuple) else "%s=%.2g" % (k, v))
    return ", ".join(out)


FP32_BAND_CEILING = 1e-5      # fp32: the band may not exceed this fraction of max|A^l|
FLIP_CEILING = {False: 1e-6, True: 1e-2}   # fp32 / bf16: largest accepted fraction of differing decisions


def aligned_backward(og, fwd, got_act, weights, X, labels, mask, tol, say=None, bf16=False,
                     got_gact=None):
    """Oracle backward with the activation decisions of the other implementation on the
    elements where the two disagree, after checking that each disagreement is legitimate.

    The backward pass branches on A^l > 0, and a pre-activation within rounding distance of
    zero can fall on either side.  What "rounding distance" is comes from the oracle's side
    only:

    * fp32 storage: 8 x the forward error of that layer as measured here, max|got - oracle|
      over the whole tensor (taken before any alignment; the forward pass does not depend on
      the decisions), and never more than 1e-5 max|A^l|;
    * bfloat16 storage: per element, from the terms that were summed into it.  The aggregate
      (or the transformed row) is rounded to bfloat16 once before the sum and its inputs once
      before that; each rounding moves a term t_j = z_j W_jc by at most 2^-9 |t_j|, uniformly
      distributed, so the sum moves with a standard deviation of 2^-9 sqrt(2/3) |t|_2.  The
      band is about 13 of those: 2^-6 sqrt(2) |t|_2 with
      t = (S|A^{l-1}| * |W|, |A^{l-1}| * |W_s|, |b|)[v, c].

    Both the oracle's pre-activation and the other side's stored activation must lie inside
    the band at every disagreement, and the number of disagreements is capped (1e-6 of the
    elements + 4 in fp32, 1 % in bfloat16).  Prints the count, the band and the largest oracle
    pre-activation among them; with ``got_gact`` also how many rows of each hidden gradient
    would fail the gate had the oracle kept its own decisions.  Returns the oracle's backward
    dict (plus ``act``)."""
    relu_on = []
    L = fwd.L
    for l in range(L - 1):
        got = np.asarray(got_act[l])
        on_got = got > 0
        on_ref = fwd.act[l] > 0
        diff = np.argwhere(on_got != on_ref)
        amax = float(np.abs(fwd.act[l]).max())
        fwd_err = 0.0
        for r0 in range(0, fwd.n, 1 << 18):
            fwd_err = max(fwd_err, float(np.abs(got[r0:r0 + (1 << 18)] - fwd.act[l][r0:r0 + (1 << 18)]).max()))
        prev = np.asarray(X, dtype=np.float64) if l == 0 else fwd.act[l - 1]
        W = np.asarray(weights[l]["W"], dtype=np.float64)
        Ws = weights[l].get("Ws") if fwd.m == 1 else None
        b = weights[l].get("b")
        ceiling = FLIP_CEILING[bool(bf16)] * on_ref.size + (0 if bf16 else 4)
        assert len(diff) <= ceiling, (l, len(diff), ceiling)
        worst_pre = 0.0
        band_txt = ""
        if len(diff):
            v, c = diff[:, 0], diff[:, 1]
            pre = np.einsum("ij,ji->i", fwd.z[l][v], W[:, c])
            if Ws is not None:
                pre = pre + np.einsum("ij,ji->i", prev[v], np.asarray(Ws, dtype=np.float64)[:, c])
            if b is not None:
                pre = pre + np.asarray(b, dtype=np.float64)[c]
            if bf16:
                # magnitudes summed into each of these pre-activations (A^{l-1} >= 0 above layer 1)
                zabs = np.abs(fwd.z[l][v]) if l > 0 else \
                    og.aggregate(fwd.m, fwd.rowptr, fwd.colidx, np.abs(prev))[v]
                sq = np.einsum("ij,ji->i", zabs ** 2, W[:, c] ** 2)
                if Ws is not None:
                    sq = sq + np.einsum("ij,ji->i", prev[v] ** 2, np.asarray(Ws, dtype=np.float64)[:, c] ** 2)
                if b is not None:
                    sq = sq + np.asarray(b, dtype=np.float64)[c] ** 2
                band = 2.0 ** -6 * np.sqrt(2.0 * sq)
                band_txt = "per-element bands up to %.2g max|A|" % (float(band.max()) / amax)
            else:
                band = 8.0 * fwd_err
                assert band <= FP32_BAND_CEILING * amax, (l, band, amax)
                band_txt = "band %.2g max|A| (8 x the measured forward error)" % (band / amax)
            worst_pre = float(np.abs(pre).max())
            assert np.all(np.abs(pre) <= band), (l, worst_pre, float(np.max(band)))
            assert np.all(np.abs(got[v, c]) <= band), (l, float(np.abs(got[v, c]).max()))
        if say:
            say("layer %d: %d of %d activation decisions differ (ceiling %d), %s; largest oracle "
                "pre-activation among them %.2g max|A|; forward error %.2g max|A|"
                % (l + 1, len(diff), on_ref.size, int(ceiling), band_txt or "no band needed",
                   worst_pre / amax, fwd_err / amax))
        on = on_ref.astype(np.uint8)
        if len(diff):
            on[diff[:, 0], diff[:, 1]] = on_got[diff[:, 0], diff[:, 1]]
        relu_on.append(on)
    if got_gact is not None and say:
        own = og.backward(fwd, labels, mask)
        for l in range(L - 1):
            den = float(np.abs(own["gact"][l]).max())
            bad = 0
            for r0 in range(0, fwd.n, 1 << 18):
                d = np.abs(np.asarray(got_gact[l][r0:r0 + (1 << 18)], dtype=np.float64) - own["gact"][l][r0:r0 + (1 << 18)])
                bad += int(np.count_nonzero(d.max(axis=1) > tol * den))
            say("with the oracle's own decisions %d of %d rows of the gradient of A^%d would miss the gate"
                % (bad, fwd.n, l + 1))
        del own
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
    (``weights[l]["heads"]`` heads side by side, default one; LeakyReLU slope 0.2, one self-loop
    per vertex) and from the given tensors of the
    step before (``act``: A^1..A^L, ``gact``: dLoss/dA^1..dLoss/dA^L).  Returns the relative
    errors by name.

    The softmax gradient of an edge u -> v needs sum_u' alpha(u' -> v) dY[v] . H[u'], which is
    dY[v] . Z[v]; Z = A^l - b wherever dY is not zero (dY vanishes where the ReLU is off)."""
    n = len(rowptr) - 1
    L = len(dims) - 1
    deg = np.diff(rowptr)
    assert not np.any(np.repeat(np.arange(n, dtype=np.int64), deg) == np.asarray(colidx))     # no self-loops stored
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
        # heads: head j is a one-head layer on columns cols[j] of H, a_src, a_dst and of the output
        nh = int(weights[l - 1].get("heads", 1))
        f = dims[l] // nh
        cols = [slice(j * f, (j + 1) * f) for j in range(nh)]
        H = np.empty((n, dims[l]))
        for r0 in range(0, n, 1 << 18):
            H[r0:r0 + (1 << 18)] = np.asarray(A[l - 1][r0:r0 + (1 << 18)], dtype=np.float64) @ W
        s_src = np.stack([H[:, cj] @ a_s[cj] for cj in cols], axis=1)          # [n, heads]
        s_dst = np.stack([H[:, cj] @ a_d[cj] for cj in cols], axis=1)

        # forward rows by the definition
        ref = []
        for v in V:
            u = around(v)
            z = np.empty(dims[l])
            for j, cj in enumerate(cols):
                e = leaky(s_src[u, j] + s_dst[v, j])
                ex = np.exp(e - e.max())
                z[cj] = (ex / ex.sum()) @ H[u][:, cj]
            z = z + b
            ref.append(np.maximum(z, 0.0) if l < L else z)
        worst["act[%d] rows" % (l - 1)] = rel_err(np.asarray(A[l])[V], np.array(ref))

        # Softmax statistics (row maximum and denominator) of the vertices the gradient rows
        # below ask for: the sampled vertices and their neighbours.  Their entries are their CSR
        # rows plus one self-loop each; per-row maxima and sums are segment reductions over the
        # gathered rows plus the self-loop's term.
        need = np.unique(np.concatenate([around(v) for v in V]))
        pos = np.full(n, -1, dtype=np.int64)
        pos[need] = np.arange(len(need))
        cnt = deg[need].astype(np.int64)
        first = np.cumsum(cnt) - cnt
        rows_of = np.repeat(np.arange(len(need)), cnt)
        ent = np.repeat(np.asarray(rowptr[:-1], dtype=np.int64)[need] - first, cnt) + np.arange(int(cnt.sum()))
        src_e = np.asarray(colidx, dtype=np.int64)[ent]
        has = cnt > 0
        mx = np.full((len(need), nh), -np.inf)
        den = np.zeros((len(need), nh))
        for j in range(nh):
            e = leaky(s_src[src_e, j] + s_dst[need[rows_of], j])
            m1 = leaky(s_src[need, j] + s_dst[need, j])              # the self-loops
            own = m1.copy()
            m1[has] = np.maximum(m1[has], np.maximum.reduceat(e, first[has]))
            ex = np.exp(e - m1[rows_of])
            d1 = np.exp(own - m1)
            d1[has] += np.add.reduceat(ex, first[has])
            mx[:, j], den[:, j] = m1, d1
            del e, ex
        dY = np.asarray(gact[l - 1], dtype=np.float64)
        if l < L:
            dY = np.where(np.asarray(A[l]) > 0, dY, 0.0)
        Zb = np.asarray(A[l], dtype=np.float64) - b
        c = np.stack([np.einsum("ij,ij->i", dY[:, cj], Zb[:, cj]) for cj in cols], axis=1)
        del Zb
        worst["gb[%d]" % (l - 1)] = rel_err(gb[l - 1], dY.sum(axis=0))
        if l == 1:
            break                                   # the gradient of the input features is not kept
        ref = []
        for u in V:
            t = around(u)
            dH = np.empty(dims[l])
            for j, cj in enumerate(cols):
                # edges u -> t
                x = s_src[u, j] + s_dst[t, j]
                alpha = np.exp(leaky(x) - mx[pos[t], j]) / den[pos[t], j]
                dx = alpha * (dY[t][:, cj] @ H[u, cj] - c[t, j]) * np.where(x > 0, 1.0, 0.2)
                dHj = alpha @ dY[t][:, cj] + dx.sum() * a_s[cj]
                # edges t -> u
                x = s_src[t, j] + s_dst[u, j]
                alpha = np.exp(leaky(x) - mx[pos[u], j]) / den[pos[u], j]
                dx = alpha * (H[t][:, cj] @ dY[u, cj] - c[u, j]) * np.where(x > 0, 1.0, 0.2)
                dH[cj] = dHj + dx.sum() * a_d[cj]
            ref.append(dH @ W.T)
        worst["gact[%d] rows" % (l - 2)] = rel_err(np.asarray(gact[l - 2])[V], np.array(ref))
        if say:
            say("layer %d checked" % l)
    return worst
