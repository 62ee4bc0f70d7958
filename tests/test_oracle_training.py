"""Pins for the oracle's training pieces: the dropout stream, dropout inside the forward and
backward passes, and the optimizer steps (datasets table of the paper: learning rate,
dropout rate, number of epochs; the optimizer is not named there, Adam and plain SGD are
provided)."""
import numpy as np
import pytest
import torch

from helpers import random_weights, small_graph
from oracle import fullgraph as og
from oracle import partition as op
from test_oracle_fullgraph import dense_operator


def test_dropout_stream_is_the_documented_counter_based_draw():
    n, d, p, seed, ep, layer = 7, 5, 0.3, 1234, 3, 2
    got = og.dropout_multipliers(n, d, p, seed, ep, layer)
    p32 = float(np.float32(p))
    thr = int(np.floor(p32 * 2.0 ** 32))
    key = op.splitmix64(seed ^ op.splitmix64(64 * ep + layer))     # plain Python integers
    for v in range(n):
        for j in range(d):
            draw = op.splitmix64((key + v * d + j) & op.MASK64) >> 32
            want = 0.0 if draw < thr else 1.0 / (1.0 - p32)
            assert got[v, j] == want
    assert np.all(og.dropout_multipliers(50, 8, 0.0, 1, 0, 1) == 1.0)


def test_dropout_rate_and_independence():
    a = og.dropout_multipliers(4000, 64, 0.5, 9, 0, 1)
    b = og.dropout_multipliers(4000, 64, 0.5, 9, 0, 2)
    c = og.dropout_multipliers(4000, 64, 0.5, 9, 1, 1)
    N = a.size
    for x in (a, b, c):
        dropped = np.count_nonzero(x == 0)
        assert abs(dropped - 0.5 * N) < 5 * np.sqrt(0.25 * N)
        assert set(np.unique(x)) == {0.0, 2.0}
    for x, y in ((a, b), (a, c), (b, c)):                 # unrelated streams agree half the time
        agree = np.count_nonzero((x == 0) == (y == 0))
        assert abs(agree - 0.5 * N) < 5 * np.sqrt(0.25 * N)
    d3 = og.dropout_multipliers(20000, 16, 0.3, 5, 0, 1)
    assert abs(np.count_nonzero(d3 == 0) / d3.size - 0.3) < 0.01
    assert np.allclose(d3.mean(), 1.0, atol=0.02)         # inverted dropout keeps the mean


@pytest.mark.parametrize("model", ["gcn", "sage"])
def test_forward_with_dropout_equals_dense_definition(model):
    n, dims = 30, (6, 8, 5, 4)
    rowptr, colidx = small_graph(n, 100, seed=3, symmetric=True, self_loops=False)
    rng = np.random.default_rng(2)
    X = rng.standard_normal((n, dims[0]))
    w = random_weights(dims, 8, sage=(model == "sage"))
    drop = [og.dropout_multipliers(n, dims[l + 1], 0.4, 77, 5, l + 1) for l in range(2)]
    f = og.forward(model, rowptr, colidx, dims, X, w, drop=drop)
    S = dense_operator(model, rowptr, colidx)
    A = X
    for l in range(3):
        Y = S @ A @ w[l]["W"] + (A @ w[l]["Ws"] if model == "sage" else 0.0) + w[l]["b"]
        A = np.maximum(Y, 0.0) * drop[l] if l < 2 else Y
        assert np.abs(A - f.act[l]).max() < 1e-12


@pytest.mark.parametrize("model", ["gcn", "sage"])
def test_gradients_with_dropout_match_finite_differences(model):
    n, dims = 20, (4, 6, 5, 3)
    rowptr, colidx = small_graph(n, 60, seed=5, symmetric=True, self_loops=False)
    rng = np.random.default_rng(8)
    X = rng.standard_normal((n, dims[0]))
    y = rng.integers(0, dims[-1], n).astype(np.int32)
    m = (rng.random(n) < 0.7).astype(np.uint8)
    w = random_weights(dims, 3, sage=(model == "sage"))
    drop = [og.dropout_multipliers(n, dims[l + 1], 0.3, 11, 0, l + 1) for l in range(2)]
    out = og.epoch(model, rowptr, colidx, dims, X, w, y, m, drop=drop)
    h, worst = 1e-6, 0.0
    for l in range(3):
        names = [("W", "gW"), ("b", "gb")] + ([("Ws", "gWs")] if model == "sage" else [])
        for pname, gname in names:
            arr, g = w[l][pname], out[gname][l]
            for idx in np.ndindex(arr.shape):
                old = arr[idx]
                arr[idx] = old + h
                lp = og.epoch(model, rowptr, colidx, dims, X, w, y, m, backward=False, drop=drop)["loss"]
                arr[idx] = old - h
                lm = og.epoch(model, rowptr, colidx, dims, X, w, y, m, backward=False, drop=drop)["loss"]
                arr[idx] = old
                worst = max(worst, abs((lp - lm) / (2 * h) - g[idx]) / np.abs(g).max())
    assert worst < 1e-6, worst
    # and the masks matter: without them the gradient is a different one
    plain = og.epoch(model, rowptr, colidx, dims, X, w, y, m)
    assert np.abs(plain["gW"][0] - out["gW"][0]).max() > 1e-3 * np.abs(plain["gW"][0]).max()


@pytest.mark.parametrize("wd", [0.0, 0.05])
def test_adam_and_sgd_equal_the_library_optimizers(wd):
    rng = np.random.default_rng(4)
    shapes = [(5, 7), (7,), (3, 2)]
    params = [rng.standard_normal(s) for s in shapes]
    tp = [torch.tensor(p.copy(), dtype=torch.float64, requires_grad=True) for p in params]
    ts = [torch.tensor(p.copy(), dtype=torch.float64, requires_grad=True) for p in params]
    adam = torch.optim.Adam(tp, lr=0.003, betas=(0.9, 0.999), eps=1e-8, weight_decay=wd)
    sgd = torch.optim.SGD(ts, lr=0.1, weight_decay=wd)
    pa, ps = [p.copy() for p in params], [p.copy() for p in params]
    m = [np.zeros_like(p) for p in params]
    v = [np.zeros_like(p) for p in params]
    for t in range(1, 7):
        grads = [rng.standard_normal(s) * (10.0 ** rng.integers(-3, 2)) for s in shapes]
        for tens, g in zip(tp, grads):
            tens.grad = torch.tensor(g.copy())
        for tens, g in zip(ts, grads):
            tens.grad = torch.tensor(g.copy())
        adam.step()
        sgd.step()
        pa, m, v = og.adam_step(pa, grads, m, v, t, 0.003, 0.9, 0.999, 1e-8, wd)
        ps = og.sgd_step(ps, grads, 0.1, wd)
        for a, b in zip(pa, tp):
            assert np.abs(a - b.detach().numpy()).max() < 1e-12
        for a, b in zip(ps, ts):
            assert np.abs(a - b.detach().numpy()).max() < 1e-12


def test_first_adam_step_moves_every_weight_by_the_learning_rate():
    g = np.array([3.0, -0.002, 40.0])
    w, m, v = og.adam_step([np.zeros(3)], [g], [np.zeros(3)], [np.zeros(3)], 1, 0.01, eps=1e-12)
    assert np.allclose(w[0], -0.01 * np.sign(g), rtol=1e-8)


def test_training_loop_chains_epochs_and_lowers_the_loss():
    n, dims = 60, (8, 16, 16, 4)
    rowptr, colidx = small_graph(n, 240, seed=6, symmetric=True, self_loops=False)
    rng = np.random.default_rng(1)
    X = rng.standard_normal((n, dims[0]))
    y = rng.integers(0, dims[-1], n).astype(np.int32)
    m = (rng.random(n) < 0.8).astype(np.uint8)
    w = random_weights(dims, 2, sage=True)
    losses, final, last = og.train("sage", rowptr, colidx, dims, X, w, y, m, epochs=40, lr=0.01,
                                   dropout=0.3, seed=5)
    assert losses[-1] < 0.6 * losses[0]
    # the same by hand for two epochs
    drop = [og.dropout_multipliers(n, dims[l + 1], 0.3, 5, 0, l + 1) for l in range(2)]
    r0 = og.epoch("sage", rowptr, colidx, dims, X, w, y, m, drop=drop)
    assert r0["loss"] == losses[0]
    flat = [t for l in range(3) for t in (w[l]["W"], w[l]["Ws"], w[l]["b"])]
    grads = [t for l in range(3) for t in (r0["gW"][l], r0["gWs"][l], r0["gb"][l])]
    new, _, _ = og.adam_step(flat, grads, [np.zeros_like(t) for t in flat],
                             [np.zeros_like(t) for t in flat], 1, 0.01)
    w1 = [{"W": new[3 * l], "Ws": new[3 * l + 1], "b": new[3 * l + 2]} for l in range(3)]
    drop1 = [og.dropout_multipliers(n, dims[l + 1], 0.3, 5, 1, l + 1) for l in range(2)]
    r1 = og.epoch("sage", rowptr, colidx, dims, X, w1, y, m, drop=drop1)
    assert r1["loss"] == losses[1]


def test_training_with_rounded_weights_steps_the_unrounded_copies():
    """``weight_round``: the epoch sees the rounded matrices, the optimizer steps the unrounded
    ones (weight decay on the unrounded value too), biases are never rounded."""
    n, dims = 50, (6, 10, 4)
    rowptr, colidx = small_graph(n, 200, seed=8, symmetric=True, self_loops=False)
    rng = np.random.default_rng(3)
    X = rng.standard_normal((n, dims[0]))
    y = rng.integers(0, dims[-1], n).astype(np.int32)
    m = (rng.random(n) < 0.7).astype(np.uint8)
    w = random_weights(dims, 4, sage=True)
    coarse = lambda a: np.round(np.asarray(a, dtype=np.float64) * 8.0) / 8.0     # a visibly coarse grid
    # the identity changes nothing
    a = og.train("sage", rowptr, colidx, dims, X, w, y, m, epochs=2, lr=0.05, weight_decay=0.1)
    b = og.train("sage", rowptr, colidx, dims, X, w, y, m, epochs=2, lr=0.05, weight_decay=0.1,
                 weight_round=lambda t: t)
    assert a[0] == b[0]
    for l in range(2):
        for key in ("W", "Ws", "b"):
            assert np.array_equal(a[1][l][key], b[1][l][key])
    # two epochs by hand
    for opt in ("adam", "sgd"):
        losses, final, _ = og.train("sage", rowptr, colidx, dims, X, w, y, m, epochs=2, optimizer=opt,
                                    lr=0.05, weight_decay=0.1, weight_round=coarse)
        rounded = lambda ws: [{"W": coarse(t["W"]), "Ws": coarse(t["Ws"]), "b": t["b"]} for t in ws]
        r0 = og.epoch("sage", rowptr, colidx, dims, X, rounded(w), y, m)
        assert r0["loss"] == losses[0]
        assert r0["loss"] != og.epoch("sage", rowptr, colidx, dims, X, w, y, m)["loss"]
        flat = [np.asarray(t, dtype=np.float64) for l in range(2) for t in (w[l]["W"], w[l]["Ws"], w[l]["b"])]
        grads = [t for l in range(2) for t in (r0["gW"][l], r0["gWs"][l], r0["gb"][l])]
        if opt == "adam":
            new, m1, v1 = og.adam_step(flat, grads, [np.zeros_like(t) for t in flat],
                                       [np.zeros_like(t) for t in flat], 1, 0.05, weight_decay=0.1)
        else:
            new = og.sgd_step(flat, grads, 0.05, 0.1)
        w1 = [{"W": new[3 * l], "Ws": new[3 * l + 1], "b": new[3 * l + 2]} for l in range(2)]
        assert not np.array_equal(w1[0]["W"], coarse(w1[0]["W"]))      # the copies leave the grid
        r1 = og.epoch("sage", rowptr, colidx, dims, X, rounded(w1), y, m)
        assert r1["loss"] == losses[1]
        grads1 = [t for l in range(2) for t in (r1["gW"][l], r1["gWs"][l], r1["gb"][l])]
        if opt == "adam":
            new2, _, _ = og.adam_step(new, grads1, m1, v1, 2, 0.05, weight_decay=0.1)
        else:
            new2 = og.sgd_step(new, grads1, 0.05, 0.1)
        for l in range(2):
            for j, key in enumerate(("W", "Ws", "b")):
                assert np.array_equal(final[l][key], new2[3 * l + j]), (opt, l, key)
