"""Pins for the graph-attention oracle (oracle/gat.py): the dense definition, automatic
differentiation of that dense definition by a library (torch, fp64), finite differences, and
the special cases in which attention reduces to a plain mean."""
import numpy as np
import pytest
import torch

from helpers import small_graph
from oracle import fullgraph as og
from oracle import gat


def make(n, dims, seed, m_draw=None, symmetric=True):
    rowptr, colidx = small_graph(n, m_draw or 4 * n, seed=seed, symmetric=symmetric, self_loops=False)
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((n, dims[0]))
    y = rng.integers(0, dims[-1], n).astype(np.int32)
    m = (rng.random(n) < 0.6).astype(np.uint8)
    w = []
    for l in range(len(dims) - 1):
        w.append({"W": rng.standard_normal((dims[l], dims[l + 1])) / np.sqrt(dims[l]),
                  "a_src": rng.standard_normal(dims[l + 1]) * 0.7,
                  "a_dst": rng.standard_normal(dims[l + 1]) * 0.7,
                  "b": rng.standard_normal(dims[l + 1]) * 0.1})
    return rowptr, colidx, X, y, m, w


def dense_mask(rowptr, colidx):
    n = len(rowptr) - 1
    M = np.zeros((n, n), dtype=bool)                 # M[v, u]: u is a source of v
    for v in range(n):
        M[v, colidx[rowptr[v]:rowptr[v + 1]]] = True
    M[np.arange(n), np.arange(n)] = True             # one self-loop each
    return M


def torch_dense_epoch(rowptr, colidx, dims, X, w, y, m):
    """The layer definition on a dense [n, n] attention matrix, differentiated by autograd."""
    M = torch.tensor(dense_mask(rowptr, colidx))
    A = torch.tensor(X, dtype=torch.float64)
    params = [{k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in wl.items()}
              for wl in w]
    acts = []
    L = len(dims) - 1
    for l in range(L):
        p = params[l]
        H = A @ p["W"]
        x = (H @ p["a_dst"])[:, None] + (H @ p["a_src"])[None, :]          # [v, u]
        e = torch.nn.functional.leaky_relu(x, 0.2)
        e = torch.where(M, e, torch.tensor(-float("inf"), dtype=torch.float64))
        alpha = torch.softmax(e, dim=1)
        Y = alpha @ H + p["b"]
        A = torch.relu(Y) if l < L - 1 else Y
        A.retain_grad()
        acts.append(A)
    idx = torch.tensor(np.flatnonzero(m))
    loss = torch.nn.functional.cross_entropy(acts[-1][idx], torch.tensor(y[m != 0].astype(np.int64)))
    loss.backward()
    return loss.item(), acts, params


@pytest.mark.parametrize("symmetric", [True, False])
def test_gat_epoch_equals_dense_definition_and_autograd(symmetric):
    n, dims = 40, (6, 7, 5, 4)
    rowptr, colidx, X, y, m, w = make(n, dims, seed=3, symmetric=symmetric)
    out = gat.epoch(rowptr, colidx, dims, X, w, y, m)
    loss, acts, params = torch_dense_epoch(rowptr, colidx, dims, X, w, y, m)
    assert abs(out["loss"] - loss) < 1e-12
    for l in range(3):
        assert np.abs(out["act"][l] - acts[l].detach().numpy()).max() < 1e-12
        assert np.abs(out["gact"][l] - acts[l].grad.numpy()).max() < 1e-12
        for ours, name in (("gW", "W"), ("ga_src", "a_src"), ("ga_dst", "a_dst"), ("gb", "b")):
            ref = params[l][name].grad.numpy()
            assert np.abs(out[ours][l] - ref).max() < 1e-11 * max(1.0, np.abs(ref).max()), (l, name)


def test_gat_gradients_match_finite_differences():
    n, dims = 25, (4, 5, 3)
    rowptr, colidx, X, y, m, w = make(n, dims, seed=8)
    out = gat.epoch(rowptr, colidx, dims, X, w, y, m)
    h, worst = 1e-6, 0.0
    for l in range(2):
        for pname, gname in (("W", "gW"), ("a_src", "ga_src"), ("a_dst", "ga_dst"), ("b", "gb")):
            arr, g = w[l][pname], out[gname][l]
            for idx in np.ndindex(arr.shape):
                old = arr[idx]
                arr[idx] = old + h
                lp = gat.epoch(rowptr, colidx, dims, X, w, y, m)["loss"]
                arr[idx] = old - h
                lm = gat.epoch(rowptr, colidx, dims, X, w, y, m)["loss"]
                arr[idx] = old
                worst = max(worst, abs((lp - lm) / (2 * h) - g[idx]) / np.abs(g).max())
    assert worst < 1e-6, worst


def test_zero_attention_vectors_give_the_mean_over_the_closed_neighbourhood():
    n, dims = 30, (5, 6, 4)
    rowptr, colidx, X, y, m, w = make(n, dims, seed=5)
    for wl in w:
        wl["a_src"][:] = 0
        wl["a_dst"][:] = 0
    acts, caches, (dst, src) = gat.forward(rowptr, colidx, dims, X, w)
    M = dense_mask(rowptr, colidx).astype(np.float64)
    S = M / M.sum(axis=1, keepdims=True)                 # row-normalised A + I
    A = X
    for l in range(2):
        Y = S @ (A @ w[l]["W"]) + w[l]["b"]
        A = np.maximum(Y, 0) if l == 0 else Y
        assert np.abs(A - acts[l]).max() < 1e-12
    # attention weights of a vertex sum to one, always
    rowptr2, colidx2, X2, y2, m2, w2 = make(n, dims, seed=6)
    _, caches, (dst, src) = gat.forward(rowptr2, colidx2, dims, X2, w2)
    sums = np.zeros(n)
    np.add.at(sums, dst, caches[0]["alpha"][:, 0])
    assert np.abs(sums - 1).max() < 1e-13


def test_attention_is_invariant_to_a_shift_of_the_destination_score_sign_region():
    # softmax over sources is unchanged when the same constant is added to every score of a
    # destination, as long as no score crosses the LeakyReLU kink; checked per vertex on a star
    n = 6
    rowptr = np.array([0, 5, 5, 5, 5, 5, 5], dtype=np.int64)      # vertex 0 aggregates from 1..5
    colidx = np.array([1, 2, 3, 4, 5], dtype=np.int32)
    dst, src = gat.edges_with_self_loops(rowptr, colidx)
    assert list(dst[:6]) == [0] * 6 and list(src[:6]) == [0, 1, 2, 3, 4, 5]
    H_in = np.eye(n)
    W = np.eye(n)
    a_src = np.array([0.0, 1.0, 2.0, 3.0, 4.0, 5.0])
    a_dst = np.zeros(n)
    out, cache = gat.layer_forward(dst, src, n, H_in, W, a_src, a_dst, None, relu=False)
    want = np.exp(a_src) / np.exp(a_src).sum()                     # all scores >= 0: identity branch
    assert np.abs(cache["alpha"][:6, 0] - want).max() < 1e-14
    assert np.abs(out[0] - want).max() < 1e-14                     # Z[0] = sum alpha_u e_u
    a_dst2 = np.zeros(n)
    a_dst2[0] = 10.0                                               # shifts every score of vertex 0
    _, cache2 = gat.layer_forward(dst, src, n, H_in, W, a_src, a_dst2, None, relu=False)
    assert np.abs(cache2["alpha"][:6, 0] - want).max() < 1e-14
    # negative scores go through the 0.2 slope
    _, cache3 = gat.layer_forward(dst, src, n, H_in, W, -a_src, a_dst, None, relu=False)
    want3 = np.exp(-0.2 * a_src) / np.exp(-0.2 * a_src).sum()
    assert np.abs(cache3["alpha"][:6, 0] - want3).max() < 1e-14


@pytest.mark.parametrize("heads", [None, (3, 2, 1), (4, 5, 5)])
def test_sampled_row_check_agrees_with_the_whole_graph_epoch(heads):
    """The per-vertex recomputation that the full-size GPU test uses (helpers.gat_sampled_errors)
    reproduces the oracle's whole-graph epoch on every vertex, and reports a planted mistake in
    an input gradient or an output row."""
    from helpers import gat_sampled_errors
    dims = (9, 12, 10, 5)
    rowptr, colidx, X, y, m, w = make(70, dims, seed=8)
    for wl, h in zip(w, heads or ()):
        wl["heads"] = h
    ref = gat.epoch(rowptr, colidx, dims, X, w, y, m)
    V = np.arange(70)
    errs = gat_sampled_errors(rowptr, colidx, dims, w, X, ref["act"], ref["gact"], ref["gb"], V)
    assert set(errs) == {"act[0] rows", "act[1] rows", "act[2] rows", "gb[0]", "gb[1]", "gb[2]",
                         "gact[0] rows", "gact[1] rows"}
    assert max(errs.values()) < 1e-12, errs
    # a dropped destination-score term in one input gradient, and a shifted output row
    bad_g = [g.copy() for g in ref["gact"]]
    bad_g[0][17] *= 1.01
    assert gat_sampled_errors(rowptr, colidx, dims, w, X, ref["act"], bad_g, ref["gb"], V)["gact[0] rows"] > 1e-4
    bad_a = [a.copy() for a in ref["act"]]
    bad_a[1][3, 2] += 0.01
    assert gat_sampled_errors(rowptr, colidx, dims, w, X, bad_a, ref["gact"], ref["gb"], V)["act[1] rows"] > 1e-4


# ---- several attention heads -----------------------------------------------------------------

def torch_dense_loss(M, dims, X, params, heads, y, m, drop=None):
    """Loss of the multi-head model written head by head on dense [n, n] attention matrices (each
    head owns a column slice of H and of the attention vectors, the heads' outputs are
    concatenated), as a torch graph over ``params``; ``drop``: multipliers after the hidden
    activations.  Returns the loss tensor and the activations."""
    A = torch.tensor(X, dtype=torch.float64)
    acts = []
    L = len(dims) - 1
    for l in range(L):
        p = params[l]
        H = A @ p["W"]
        f = dims[l + 1] // heads[l]
        outs = []
        for j in range(heads[l]):
            Hj = H[:, j * f:(j + 1) * f]
            x = (Hj @ p["a_dst"][j * f:(j + 1) * f])[:, None] + (Hj @ p["a_src"][j * f:(j + 1) * f])[None, :]
            e = torch.nn.functional.leaky_relu(x, 0.2)
            e = torch.where(M, e, torch.tensor(-float("inf"), dtype=torch.float64))
            outs.append(torch.softmax(e, dim=1) @ Hj)
        Y = torch.cat(outs, dim=1) + p["b"]
        A = torch.relu(Y) if l < L - 1 else Y
        if drop is not None and l < L - 1:
            A = A * torch.tensor(drop[l], dtype=torch.float64)
        A.retain_grad()
        acts.append(A)
    idx = torch.tensor(np.flatnonzero(m))
    loss = torch.nn.functional.cross_entropy(acts[-1][idx], torch.tensor(y[m != 0].astype(np.int64)))
    return loss, acts


def torch_params(w):
    return [{k: torch.tensor(v, dtype=torch.float64, requires_grad=True)
             for k, v in wl.items() if k != "heads"} for wl in w]


def torch_dense_epoch_heads(rowptr, colidx, dims, X, w, heads, y, m, drop=None):
    M = torch.tensor(dense_mask(rowptr, colidx))
    params = torch_params(w)
    loss, acts = torch_dense_loss(M, dims, X, params, heads, y, m, drop=drop)
    loss.backward()
    return loss.item(), acts, params


@pytest.mark.parametrize("symmetric", [True, False])
def test_multi_head_epoch_equals_dense_definition_and_autograd(symmetric):
    n, dims, heads = 40, (6, 12, 10, 4), (3, 5, 2)
    rowptr, colidx, X, y, m, w = make(n, dims, seed=13, symmetric=symmetric)
    for wl, h in zip(w, heads):
        wl["heads"] = h
    out = gat.epoch(rowptr, colidx, dims, X, w, y, m)
    loss, acts, params = torch_dense_epoch_heads(rowptr, colidx, dims, X, w, heads, y, m)
    assert abs(out["loss"] - loss) < 1e-12
    for l in range(3):
        assert np.abs(out["act"][l] - acts[l].detach().numpy()).max() < 1e-12
        assert np.abs(out["gact"][l] - acts[l].grad.numpy()).max() < 1e-12
        for ours, name in (("gW", "W"), ("ga_src", "a_src"), ("ga_dst", "a_dst"), ("gb", "b")):
            ref = params[l][name].grad.numpy()
            assert np.abs(out[ours][l] - ref).max() < 1e-11 * max(1.0, np.abs(ref).max()), (l, name)


def test_heads_are_independent_one_head_layers_side_by_side():
    """A layer with h heads equals h one-head layers, each on its own column slice of W, a_src,
    a_dst and b, with the outputs concatenated; and the gradients of a sum of losses split the
    same way.  Ties the multi-head code to the one-head layer pinned above."""
    n, din, f, heads = 35, 7, 4, 3
    rowptr, colidx, X, y, m, w = make(n, (din, f * heads), seed=21)
    dst, src = gat.edges_with_self_loops(rowptr, colidx)
    wl = w[0]
    out, cache = gat.layer_forward(dst, src, n, X, wl["W"], wl["a_src"], wl["a_dst"], wl["b"], relu=True,
                                   heads=heads)
    rng = np.random.default_rng(4)
    dY = rng.standard_normal(out.shape)
    g = gat.layer_backward(dst, src, n, X, wl["W"], wl["a_src"], wl["a_dst"], cache, dY)
    gA = np.zeros_like(X)
    for j in range(heads):
        sl = slice(j * f, (j + 1) * f)
        o1, c1 = gat.layer_forward(dst, src, n, X, wl["W"][:, sl], wl["a_src"][sl], wl["a_dst"][sl],
                                   wl["b"][sl], relu=True)
        assert np.abs(o1 - out[:, sl]).max() < 1e-13
        assert np.abs(c1["alpha"][:, 0] - cache["alpha"][:, j]).max() < 1e-14
        g1 = gat.layer_backward(dst, src, n, X, wl["W"][:, sl], wl["a_src"][sl], wl["a_dst"][sl], c1, dY[:, sl])
        assert np.abs(g1["gW"] - g["gW"][:, sl]).max() < 1e-12
        assert np.abs(g1["ga_src"] - g["ga_src"][sl]).max() < 1e-12
        assert np.abs(g1["ga_dst"] - g["ga_dst"][sl]).max() < 1e-12
        gA += g1["gA"]
    assert np.abs(gA - g["gA"]).max() < 1e-12
    # every head's attention weights sum to one over the sources of every vertex
    sums = np.zeros((n, heads))
    np.add.at(sums, dst, cache["alpha"])
    assert np.abs(sums - 1).max() < 1e-13


def test_multi_head_gradients_match_finite_differences():
    n, dims, heads = 20, (4, 6, 4), (2, 2)
    rowptr, colidx, X, y, m, w = make(n, dims, seed=31)
    for wl, h in zip(w, heads):
        wl["heads"] = h
    out = gat.epoch(rowptr, colidx, dims, X, w, y, m)
    h, worst = 1e-6, 0.0
    for l in range(2):
        for pname, gname in (("W", "gW"), ("a_src", "ga_src"), ("a_dst", "ga_dst"), ("b", "gb")):
            arr, g = w[l][pname], out[gname][l]
            for idx in np.ndindex(arr.shape):
                old = arr[idx]
                arr[idx] = old + h
                lp = gat.epoch(rowptr, colidx, dims, X, w, y, m)["loss"]
                arr[idx] = old - h
                lm = gat.epoch(rowptr, colidx, dims, X, w, y, m)["loss"]
                arr[idx] = old
                worst = max(worst, abs((lp - lm) / (2 * h) - g[idx]) / np.abs(g).max())
    assert worst < 1e-6, worst


def test_dropout_after_hidden_activations_equals_autograd_of_the_dense_definition():
    n, dims, heads = 40, (6, 12, 10, 4), (3, 1, 2)
    rowptr, colidx, X, y, m, w = make(n, dims, seed=17)
    for wl, h in zip(w, heads):
        wl["heads"] = h
    drop = [og.dropout_multipliers(n, dims[l + 1], 0.4, 5, 2, l + 1) for l in range(2)]
    assert all(0.2 < (d == 0).mean() < 0.6 for d in drop)
    out = gat.epoch(rowptr, colidx, dims, X, w, y, m, drop=drop)
    loss, acts, params = torch_dense_epoch_heads(rowptr, colidx, dims, X, w, heads, y, m, drop=drop)
    assert abs(out["loss"] - loss) < 1e-12
    for l in range(3):
        assert np.abs(out["act"][l] - acts[l].detach().numpy()).max() < 1e-12
        assert np.abs(out["gact"][l] - acts[l].grad.numpy()).max() < 1e-12
        for ours, name in (("gW", "W"), ("ga_src", "a_src"), ("ga_dst", "a_dst"), ("gb", "b")):
            ref = params[l][name].grad.numpy()
            assert np.abs(out[ours][l] - ref).max() < 1e-11 * max(1.0, np.abs(ref).max()), (l, name)
    # without multipliers nothing changes
    plain = gat.epoch(rowptr, colidx, dims, X, w, y, m)
    again = gat.epoch(rowptr, colidx, dims, X, w, y, m, drop=[None, None])
    assert plain["loss"] == again["loss"]


@pytest.mark.parametrize("opt,dropout", [("adam", 0.0), ("sgd", 0.0), ("adam", 0.3)])
def test_training_epochs_follow_a_library_optimizer_on_the_dense_definition(opt, dropout):
    """gat.train against torch.optim (Adam with L2 weight decay / SGD) stepping the dense
    definition's parameters; with dropout the torch model takes the same multipliers."""
    n, dims, heads, epochs, lr, wd = 30, (5, 8, 6, 3), (2, 3, 1), 3, 0.02, 0.01
    rowptr, colidx, X, y, m, w = make(n, dims, seed=23)
    for wl, h in zip(w, heads):
        wl["heads"] = h
    losses, final, last = gat.train(rowptr, colidx, dims, X, w, y, m, epochs, optimizer=opt, lr=lr,
                                    weight_decay=wd, dropout=dropout, seed=11, first_epoch=0)
    M = torch.tensor(dense_mask(rowptr, colidx))
    params = torch_params(w)
    flat = [p[k] for p in params for k in ("W", "a_src", "a_dst", "b")]
    optim = (torch.optim.Adam(flat, lr=lr, weight_decay=wd) if opt == "adam"
             else torch.optim.SGD(flat, lr=lr, weight_decay=wd))
    for e in range(epochs):
        drop = None
        if dropout > 0:
            drop = [og.dropout_multipliers(n, dims[l + 1], dropout, 11, e, l + 1) for l in range(2)]
        optim.zero_grad()
        loss, _ = torch_dense_loss(M, dims, X, params, heads, y, m, drop=drop)
        loss.backward()
        assert abs(losses[e] - loss.item()) < 1e-10, (e, losses[e], loss.item())
        optim.step()
    assert losses[0] != losses[1]
    for l in range(3):
        for k in ("W", "a_src", "a_dst", "b"):
            ref = params[l][k].detach().numpy()
            assert np.abs(final[l][k] - ref).max() < 1e-9 * max(1.0, np.abs(ref).max()), (l, k)
        assert final[l]["heads"] == heads[l]
