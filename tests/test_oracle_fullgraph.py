"""Pins for the full-graph oracle: each checks it against something that is not itself
(dense matrices written out from the definition, finite differences, textbook special
cases, library routines, closed forms)."""
import numpy as np
import pytest
from scipy.special import log_softmax

from helpers import (complete_graph, empty_graph, random_weights, rel_err, ring_graph,
                     small_graph)
from oracle import fullgraph as og


# ---------------------------------------------------------------------------------------
# dense brute force
# ---------------------------------------------------------------------------------------
def dense_operator(model, rowptr, colidx):
    """The aggregation operator as a dense [n, n] matrix, straight from the definition."""
    n = len(rowptr) - 1
    A = np.zeros((n, n))
    for v in range(n):
        A[v, colidx[rowptr[v]:rowptr[v + 1]]] = 1.0
    if model == "gcn":
        A[np.arange(n), np.arange(n)] = 1.0            # A + I, one self-loop per vertex
        deg = A.sum(axis=1)                            # row length of A~
        dm = np.diag(deg ** -0.5)
        return dm @ A @ dm
    deg = A.sum(axis=1)
    inv = np.where(deg > 0, 1.0 / np.maximum(deg, 1), 0.0)
    return inv[:, None] * A


def dense_forward(model, S, dims, X, weights):
    acts, zs = [], []
    A = np.asarray(X, dtype=np.float64)
    L = len(dims) - 1
    for l in range(L):
        Z = S @ A
        Y = Z @ weights[l]["W"]
        if model == "sage":
            Y = Y + A @ weights[l]["Ws"]
        if weights[l]["b"] is not None:
            Y = Y + weights[l]["b"]
        A = np.maximum(Y, 0) if l < L - 1 else Y
        acts.append(A)
        zs.append(Z)
    return acts, zs


def dense_loss(logits, y, m):
    ls = log_softmax(logits, axis=1)
    idx = np.flatnonzero(m)
    return -ls[idx, y[idx]].mean()


CASES = [
    ("gcn", dict(symmetric=True, self_loops=True)),
    ("gcn", dict(symmetric=True, self_loops=False)),     # the oracle must add the self-loops
    ("gcn", dict(symmetric=False, self_loops=False)),    # directed: in-degree + 1 on both ends
    ("sage", dict(symmetric=True, self_loops=False)),
    ("sage", dict(symmetric=False, self_loops=False)),   # has empty rows
]


@pytest.mark.parametrize("model,gkw", CASES)
def test_forward_matches_dense_brute_force(model, gkw):
    n, dims = 48, (7, 9, 6, 5)
    rowptr, colidx = small_graph(n, 160, seed=5, **gkw)
    rng = np.random.default_rng(0)
    X = rng.standard_normal((n, dims[0]))
    y = rng.integers(0, dims[-1], n).astype(np.int32)
    m = (rng.random(n) < 0.5).astype(np.uint8)
    w = random_weights(dims, 1, sage=(model == "sage"))
    out = og.epoch(model, rowptr, colidx, dims, X, w, y, m, backward=False)
    S = dense_operator(model, rowptr, colidx)
    acts, zs = dense_forward(model, S, dims, X, w)
    for l in range(3):
        assert np.abs(out["z"][l] - zs[l]).max() < 1e-12
        assert np.abs(out["act"][l] - acts[l]).max() < 1e-12
    assert abs(out["loss"] - dense_loss(acts[-1], y, m)) < 1e-12


def test_mixed_self_loops_are_not_doubled():
    # some vertices already carry a self-loop, others do not: A~ has exactly one each
    n = 20
    rowptr, colidx = small_graph(n, 60, seed=2, symmetric=True, self_loops=False)
    src = np.repeat(np.arange(n), np.diff(rowptr))
    extra = np.arange(0, n, 3)
    from synth import csr_from_edges
    rp2, ci2 = csr_from_edges(n, np.concatenate([colidx, extra]), np.concatenate([src, extra]))
    X = np.random.default_rng(3).standard_normal((n, 4))
    assert np.abs(og.aggregate("gcn", rp2, ci2, X) - og.aggregate("gcn", rowptr, colidx, X)).max() == 0
    assert np.abs(og.aggregate("gcn", rp2, ci2, X) - dense_operator("gcn", rowptr, colidx) @ X).max() < 1e-13


# ---------------------------------------------------------------------------------------
# gradients: central finite differences on every weight, bias and a sample of inputs
# ---------------------------------------------------------------------------------------
def _loss_only(model, rowptr, colidx, dims, X, w, y, m):
    return og.epoch(model, rowptr, colidx, dims, X, w, y, m, backward=False)["loss"]


@pytest.mark.parametrize("model,gkw", [CASES[0], CASES[2], CASES[3], CASES[4]])
def test_gradients_match_finite_differences(model, gkw):
    n, dims = 24, (5, 6, 4, 3)
    rowptr, colidx = small_graph(n, 70, seed=7, **gkw)
    rng = np.random.default_rng(11)
    X = rng.standard_normal((n, dims[0]))
    y = rng.integers(0, dims[-1], n).astype(np.int32)
    m = (rng.random(n) < 0.6).astype(np.uint8)
    w = random_weights(dims, 4, sage=(model == "sage"))
    out = og.epoch(model, rowptr, colidx, dims, X, w, y, m, backward=True, input_grad=True)
    h = 1e-6
    worst = 0.0

    def fd(arr, idx):
        old = arr[idx]
        arr[idx] = old + h
        lp = _loss_only(model, rowptr, colidx, dims, X, w, y, m)
        arr[idx] = old - h
        lm = _loss_only(model, rowptr, colidx, dims, X, w, y, m)
        arr[idx] = old
        return (lp - lm) / (2 * h)

    for l in range(3):
        names = [("W", "gW"), ("b", "gb")] + ([("Ws", "gWs")] if model == "sage" else [])
        for pname, gname in names:
            arr, g = w[l][pname], out[gname][l]
            scale = np.abs(g).max()
            for idx in np.ndindex(arr.shape):
                worst = max(worst, abs(fd(arr, idx) - g[idx]) / scale)
    scale = np.abs(out["gX"]).max()
    for _ in range(40):
        idx = (int(rng.integers(n)), int(rng.integers(dims[0])))
        worst = max(worst, abs(fd(X, idx) - out["gX"][idx]) / scale)
    assert worst < 1e-6, worst


@pytest.mark.parametrize("model", ["gcn", "sage"])
def test_activation_gradients_match_subnetwork_input_gradients(model):
    # dLoss/dA^l of the full network is the input gradient of the network made of layers
    # l+1..L fed with A^l; the input gradient itself is pinned by finite differences above.
    n, dims = 30, (6, 5, 7, 4)
    rowptr, colidx = small_graph(n, 90, seed=9, symmetric=True, self_loops=False)
    rng = np.random.default_rng(5)
    X = rng.standard_normal((n, dims[0]))
    y = rng.integers(0, dims[-1], n).astype(np.int32)
    m = (rng.random(n) < 0.5).astype(np.uint8)
    w = random_weights(dims, 6, sage=(model == "sage"))
    full = og.epoch(model, rowptr, colidx, dims, X, w, y, m)
    for l in (1, 2):
        sub = og.epoch(model, rowptr, colidx, dims[l:], full["act"][l - 1], w[l:], y, m,
                       input_grad=True)
        assert np.abs(sub["gX"] - full["gact"][l - 1]).max() < 1e-14
    # last entry: gradient of the loss w.r.t. the logits
    _, g = og.loss(full["act"][-1], y, m)
    assert np.abs(g - full["gact"][-1]).max() == 0


@pytest.mark.parametrize("model,gkw", CASES)
def test_adjoint_identity(model, gkw):
    n, d = 60, 5
    rowptr, colidx = small_graph(n, 200, seed=3, **gkw)
    rng = np.random.default_rng(8)
    x, yv = rng.standard_normal((n, d)), rng.standard_normal((n, d))
    lhs = (og.aggregate(model, rowptr, colidx, x) * yv).sum()
    rhs = (x * og.aggregate(model, rowptr, colidx, yv, transpose=True)).sum()
    assert abs(lhs - rhs) < 1e-12 * max(1.0, abs(lhs))
    S = dense_operator(model, rowptr, colidx)
    assert np.abs(og.aggregate(model, rowptr, colidx, yv, transpose=True) - S.T @ yv).max() < 1e-13


# ---------------------------------------------------------------------------------------
# special cases that reduce to textbook routines
# ---------------------------------------------------------------------------------------
def test_edgeless_gcn_is_an_mlp():
    n, dims = 17, (4, 6, 3)
    rowptr, colidx = empty_graph(n)
    rng = np.random.default_rng(1)
    X = rng.standard_normal((n, 4))
    w = random_weights(dims, 2, sage=False)
    y = rng.integers(0, 3, n).astype(np.int32)
    m = np.ones(n, dtype=np.uint8)
    out = og.epoch("gcn", rowptr, colidx, dims, X, w, y, m, backward=False)
    H = np.maximum(X @ w[0]["W"] + w[0]["b"], 0)
    assert np.abs(out["act"][1] - (H @ w[1]["W"] + w[1]["b"])).max() < 1e-13


def test_edgeless_sage_aggregates_zero():
    n = 9
    rowptr, colidx = empty_graph(n)
    X = np.random.default_rng(1).standard_normal((n, 3))
    assert np.all(og.aggregate("sage", rowptr, colidx, X) == 0)


def test_complete_graph_gives_column_mean():
    n = 13
    X = np.random.default_rng(2).standard_normal((n, 5))
    rowptr, colidx = complete_graph(n, self_loops=False)
    Z = og.aggregate("gcn", rowptr, colidx, X)          # A + I is all ones, deg = n
    assert np.abs(Z - X.mean(axis=0)).max() < 1e-14
    Zs = og.aggregate("sage", *complete_graph(n, self_loops=True), X)
    assert np.abs(Zs - X.mean(axis=0)).max() < 1e-14


def test_regular_ring():
    n, r = 20, 4
    rowptr, colidx = ring_graph(n, r)
    X = np.random.default_rng(4).standard_normal((n, 3))
    A = np.zeros((n, n))
    for v in range(n):
        for s in (1, 2):
            A[v, (v + s) % n] = A[v, (v - s) % n] = 1
    assert np.abs(og.aggregate("gcn", rowptr, colidx, X) - (A + np.eye(n)) @ X / (r + 1)).max() < 1e-14
    assert np.abs(og.aggregate("sage", rowptr, colidx, X) - A @ X / r).max() < 1e-14


def test_single_layer_identity_weight_gives_operator_times_x():
    n, d = 25, 6
    rowptr, colidx = small_graph(n, 80, seed=6, symmetric=True, self_loops=True)
    X = np.random.default_rng(3).standard_normal((n, d))
    w = [{"W": np.eye(d), "Ws": None, "b": np.zeros(d)}]
    y = np.zeros(n, dtype=np.int32)
    m = np.ones(n, dtype=np.uint8)
    out = og.epoch("gcn", rowptr, colidx, (d, d), X, w, y, m, backward=False)
    assert np.abs(out["act"][0] - dense_operator("gcn", rowptr, colidx) @ X).max() < 1e-13


# ---------------------------------------------------------------------------------------
# loss
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("C,lnC", [(16, 2.772589), (47, 3.850148), (172, 5.147494), (64, 4.158883)])
def test_zero_weights_give_log_num_classes(C, lnC):
    n, dims = 40, (8, 8, C)
    rowptr, colidx = small_graph(n, 120, seed=1, symmetric=True, self_loops=True)
    rng = np.random.default_rng(0)
    X = rng.standard_normal((n, 8))
    w = [{"W": np.zeros((8, 8)), "Ws": None, "b": np.zeros(8)},
         {"W": np.zeros((8, C)), "Ws": None, "b": np.zeros(C)}]
    y = rng.integers(0, C, n).astype(np.int32)
    m = (rng.random(n) < 0.5).astype(np.uint8)
    out = og.epoch("gcn", rowptr, colidx, dims, X, w, y, m, backward=False)
    assert abs(out["loss"] - lnC) < 1e-6
    assert abs(out["loss"] - np.log(C)) < 1e-14


def test_loss_against_library_log_softmax_and_gradient_structure():
    n, C = 50, 11
    rng = np.random.default_rng(9)
    logits = 5 * rng.standard_normal((n, C))
    logits[3] += 800.0                                  # needs the max-subtracted form
    y = rng.integers(0, C, n).astype(np.int32)
    m = (rng.random(n) < 0.4).astype(np.uint8)
    val, g = og.loss(logits, y, m)
    assert abs(val - dense_loss(logits, y, m)) < 1e-12
    assert np.all(g[m == 0] == 0)
    assert np.abs(g.sum(axis=1)).max() < 1e-15
    onehot = np.zeros((n, C))
    onehot[np.arange(n), y] = 1
    ref = (np.exp(log_softmax(logits, axis=1)) - onehot) * m[:, None] / m.sum()
    assert np.abs(g - ref).max() < 1e-15


def test_thread_count_does_not_change_any_bit():
    n, dims = 200, (12, 10, 7)
    rowptr, colidx = small_graph(n, 1500, seed=21, symmetric=True, self_loops=False)
    rng = np.random.default_rng(2)
    X = rng.standard_normal((n, 12))
    y = rng.integers(0, 7, n).astype(np.int32)
    m = (rng.random(n) < 0.5).astype(np.uint8)
    w = random_weights(dims, 3, sage=True)
    keep = og.num_threads()
    try:
        og.set_num_threads(1)
        a = og.epoch("sage", rowptr, colidx, dims, X, w, y, m)
        og.set_num_threads(max(2, keep))
        b = og.epoch("sage", rowptr, colidx, dims, X, w, y, m)
    finally:
        og.set_num_threads(keep)
    for key in ("act", "gW", "gWs", "gb", "gact"):
        for u, v in zip(a[key], b[key]):
            assert np.array_equal(u, v)
    assert a["loss"] == b["loss"]


def test_supplied_activation_decision_is_used_as_given():
    # the optional decision array replaces act > 0; checked against reverse mode written out
    # with dense matrices and the same explicit masks
    n, dims = 20, (4, 6, 5, 3)
    rowptr, colidx = small_graph(n, 70, seed=12, symmetric=True, self_loops=False)
    rng = np.random.default_rng(4)
    X = rng.standard_normal((n, dims[0]))
    y = rng.integers(0, dims[-1], n).astype(np.int32)
    m = (rng.random(n) < 0.6).astype(np.uint8)
    w = random_weights(dims, 8, sage=True)
    f = og.forward("sage", rowptr, colidx, dims, X, w)
    same = og.backward(f, y, m, relu_on=[(a > 0).astype(np.uint8) for a in f.act[:-1]])
    plain = og.backward(f, y, m)
    for key in ("gW", "gWs", "gb", "gact"):
        for a, b in zip(same[key], plain[key]):
            assert np.array_equal(a, b)
    masks = [(rng.random(a.shape) < 0.5).astype(np.uint8) for a in f.act[:-1]]
    got = og.backward(f, y, m, relu_on=masks)
    S = dense_operator("sage", rowptr, colidx)
    _, G = og.loss(f.act[-1], y, m)
    acts = [X] + f.act
    for l in (2, 1, 0):
        dY = G * masks[l] if l < 2 else G
        assert np.abs(got["gW"][l] - (S @ acts[l]).T @ dY).max() < 1e-13
        assert np.abs(got["gWs"][l] - acts[l].T @ dY).max() < 1e-13
        assert np.abs(got["gb"][l] - dY.sum(axis=0)).max() < 1e-13
        G = S.T @ (dY @ w[l]["W"].T) + dY @ w[l]["Ws"].T
        if l >= 1:
            assert np.abs(got["gact"][l - 1] - G).max() < 1e-13


def test_rel_err_helper():
    assert rel_err([1.0, 2.0], [1.0, 2.0]) == 0.0
    assert abs(rel_err([1.0, 2.2], [1.0, 2.0]) - 0.1) < 1e-12


def test_decision_alignment_accepts_rounding_and_rejects_everything_else():
    """The helper that aligns activation decisions near zero: a copy of the oracle's
    activations rounded to single precision passes (with few or no flips); the same copy with
    one clearly positive activation switched off, or with one far-from-zero element switched
    on, is refused; so is a copy whose forward error is large enough to widen the band past
    its ceiling."""
    from helpers import aligned_backward, elem_err
    n, dims = 400, (12, 16, 16, 5)
    rowptr, colidx = small_graph(n, 3000, seed=21, symmetric=True, self_loops=False)
    rng = np.random.default_rng(9)
    X = rng.standard_normal((n, dims[0])).astype(np.float32)
    y = rng.integers(0, dims[-1], n).astype(np.int32)
    m = (rng.random(n) < 0.5).astype(np.uint8)
    w = random_weights(dims, 3, sage=True)
    f = og.forward("sage", rowptr, colidx, dims, X, w)
    lines = []
    got = [a.astype(np.float32) for a in f.act]
    plain = og.backward(f, y, m)
    out = aligned_backward(og, f, got, w, X, y, m, 1e-4, lines.append, got_gact=plain["gact"])
    assert any("0 of %d rows" % n in s for s in lines)
    for a, b in zip(out["gact"], plain["gact"]):
        assert rel_err(a, b) < 1e-12
    # a decision flipped where the pre-activation is nowhere near zero
    v, c = np.unravel_index(np.argmax(f.act[0]), f.act[0].shape)
    bad = [a.copy() for a in got]
    bad[0][v, c] = 0.0
    with pytest.raises(AssertionError):
        aligned_backward(og, f, bad, w, X, y, m, 1e-4)
    neg = np.argwhere(f.act[1] == 0)
    bad = [a.copy() for a in got]
    bad[1][neg[0, 0], neg[0, 1]] = 1e-3 * f.act[1].max()
    with pytest.raises(AssertionError):
        aligned_backward(og, f, bad, w, X, y, m, 1e-4)
    # a flip near zero that a sloppy forward pass (error 1e-3 of the maximum) would excuse
    pos = f.act[0][f.act[0] > 0]
    thr = np.sort(pos)[3]
    v, c = np.argwhere(f.act[0] == thr)[0]
    bad = [a.copy() for a in got]
    bad[0][v, c] = 0.0
    bad[0][0, 0] += 1e-3 * f.act[0].max()
    with pytest.raises(AssertionError):
        aligned_backward(og, f, bad, w, X, y, m, 1e-4)
    assert elem_err([1.0, 1e-6], [1.0, 2e-6]) < 1.1e-3 and abs(elem_err([1.0, 0.5], [1.0, 0.4]) - 0.25) < 1e-12
