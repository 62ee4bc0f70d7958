"""Parity at the bench's full sizes.

`mid` (2.4 M vertices, 131 M operator entries, 3-layer SAGE-mean, k = 16 switching-aware
partitions) in exactly the launch configuration bench.py times, against one full fp64 oracle
epoch on the host cores: about 60 GB of host memory and two minutes (most of it the oracle).

The streaming schedule on `mid` with pools far smaller than the working set must reproduce the
resident schedule bit for bit: at this size kernels run for milliseconds beside the copies, so
a missing dependency between the three streams would show.

`dense` (4 M vertices, bfloat16, GCN 512-1024-1024-64, k = 16) is too wide for a whole oracle
epoch in reasonable time; there sampled rows and columns of every tensor are recomputed from
their definitions, each from the path's own inputs to that step, which the oracle's
aggregation routine and plain numpy can do one by one.

`mid_gat` (graph attention on the `mid` graph, with one head and with eight): sampled vertices
(with one head eight hubs among them) of every layer's output and input gradient, by a helper that a CPU test pins to the oracle's
whole-graph epoch.

`large` (50 M vertices, 870 M entries, k = 64): the same kind of sampled check with the tensors
left on the device."""
import os
import sys
import time

import numpy as np
import pytest

from helpers import aligned_backward, both_errs, fmt_errs, gat_sampled_errors, rel_err

pytestmark = pytest.mark.gpu
TOL = 1e-4


def test_mid_workload_full_size(capsys):
    import psutil
    if psutil.virtual_memory().available < 90 * 2 ** 30:
        pytest.skip("needs ~60 GB of free host memory for the fp64 oracle at full size")
    from oracle import fullgraph as og
    from oracle import partition as op
    from paper_2605_11517_amd import Session
    from synth import features, glorot_weights, labels_and_mask, make_config

    def say(msg):
        with capsys.disabled():
            print("[fullsize %.0fs] %s" % (time.time() - t0, msg), flush=True)

    t0 = time.time()
    cfg, rowptr, colidx = make_config("mid")
    n, dims = cfg["n"], cfg["dims"]
    X = features(n, dims[0], cfg["seed"])
    y, m = labels_and_mask(n, dims[-1], cfg["train_frac"], cfg["seed"])
    w = glorot_weights(dims, cfg["seed"], sage=True, bias_scale=0.05)
    say("inputs ready: n=%d entries=%d" % (n, rowptr[-1]))

    # the configuration bench.py times: switching-aware partitions, layer order by rows moved
    s = Session("sage", dims, rowptr, colidx, cfg["k"], cfg["part"], cfg["seed"], X, w, y, m,
                layer_order="auto", fuse_gather=True, masked_backward=True,
                keep_forward="auto")                                          # the configuration bench.py times
    assert s.ctx.gather_is_fused() and s.keeps_forward
    assert [s.ctx.layer_is_transform_first(l) for l in (1, 2, 3)] == [False, True, True]
    loss = s.epoch()
    loss2 = s.epoch()
    assert loss == loss2
    got = s.results()
    part, k = s.ctx.get_partition()
    stats = s.ctx.get_stats()
    bnd = [s.ctx.get_boundary(p) for p in range(k)]
    del s
    say("GPU epoch done, loss %.6f" % loss)

    # partition structure: assignment bit-exact against the oracle's rule, boundary lists
    # against a vectorised restatement of the definition for every partition
    # (the switching-aware partitioner's assignment at this size is compared through the digest
    # that tests/golden/make_switching_digest.py wrote from the oracle's partitioner alone)
    if cfg["part"] == "lp":
        want = op.assign_lp(rowptr, colidx, cfg["k"], cfg["seed"])
        assert np.array_equal(part, want)
    else:
        import hashlib
        fx = {}
        for line in open(os.path.join(os.path.dirname(__file__), "golden", "mid_switching_digest.txt")):
            if not line.startswith("#"):
                key, *vals = line.split()
                fx[key] = vals
        assert cfg["part"] == "switching"
        assert [int(fx["n"][0]), int(fx["k"][0]), int(fx["seed"][0])] == [n, cfg["k"], cfg["seed"]]
        assert [int(x) for x in fx["sizes"]] == list(np.bincount(part, minlength=k))
        assert hashlib.sha256(np.ascontiguousarray(part, dtype="<i4").tobytes()).hexdigest() == fx["sha256"][0]
    dst = np.repeat(np.arange(n, dtype=np.int32), np.diff(rowptr))
    cross = part[dst] != part[colidx]
    pair = np.unique(part[dst][cross].astype(np.int64) * n + colidx[cross])
    total = 0
    for p in range(k):
        u = (pair[(pair >= p * n) & (pair < (p + 1) * n)] - p * n).astype(np.int32)
        order = np.lexsort((u, part[u]))          # by (partition id, vertex id)
        assert np.array_equal(bnd[p], u[order]), p
        total += len(u)
    assert stats["sum_boundary"] == total
    del dst, cross, pair
    say("partition assignment and %d boundary entries bit-exact" % total)

    fwd = og.forward("sage", rowptr, colidx, dims, X, w)
    say("oracle forward done")
    for l, (a, b) in enumerate(zip(got["act"], fwd.act)):
        assert rel_err(a, b) <= TOL, ("act", l)

    # The backward pass branches on A^l > 0.  Where a pre-activation lies within rounding
    # distance of zero the two sides may legitimately decide differently; the helper checks
    # that every disagreement is of that kind and lets the oracle take the same decision there.
    ref = aligned_backward(og, fwd, got["act"], w, X, y, m, TOL, say, got_gact=got["gact"])
    say("oracle epoch done, loss %.6f" % ref["loss"])
    assert abs(loss - ref["loss"]) <= TOL * abs(ref["loss"])
    worst = {}
    for key in ("gact", "gW", "gWs", "gb"):
        for l, (a, b) in enumerate(zip(got[key], ref[key])):
            worst["%s[%d]" % (key, l)] = both_errs(a, b)
    say("relative errors, gate (element-wise): " + fmt_errs(worst))
    worst = {k_: v[0] for k_, v in worst.items()}
    bad = {k_: v for k_, v in worst.items() if not v <= TOL}
    assert not bad, bad


def test_mid_streaming_matches_resident_bit_for_bit(capsys):
    import psutil
    if psutil.virtual_memory().available < 60 * 2 ** 30:
        pytest.skip("needs ~40 GB of free host memory")
    from paper_2605_11517_amd import Session
    from synth import features, glorot_weights, labels_and_mask, make_config

    def say(msg):
        with capsys.disabled():
            print("[stream %.0fs] %s" % (time.time() - t0, msg), flush=True)

    t0 = time.time()
    cfg, rowptr, colidx = make_config("mid")
    n, dims = cfg["n"], cfg["dims"]
    X = features(n, dims[0], cfg["seed"])
    y, m = labels_and_mask(n, dims[-1], cfg["train_frac"], cfg["seed"])
    w = glorot_weights(dims, cfg["seed"], sage=True, bias_scale=0.05)
    s = Session("sage", dims, rowptr, colidx, cfg["k"], cfg["part"], cfg["seed"], X, w, y, m)
    loss = s.epoch()
    ref = s.results()
    del s
    say("resident epoch done, loss %.6f" % loss)
    for gib, epochs in ((4, 2), (1.5, 1)):
        s = Session("sage", dims, rowptr, colidx, cfg["k"], cfg["part"], cfg["seed"], X, w, y, m,
                    hbm_budget_bytes=int(gib * 2 ** 30))
        for rep in range(epochs):
            assert s.epoch() == loss
            got = s.results()
            for key in ("act", "gact", "gW", "gWs", "gb"):
                for l, (a, b) in enumerate(zip(got[key], ref[key])):
                    assert np.array_equal(a, b), (gib, rep, key, l)
            st = s.ctx.get_stream_stats()
            say("pool %g GiB, epoch %d bit-identical; %d block loads, %d direct row gathers, %.1f GB in, %.1f GB out"
                % (gib, rep, st["act_loads"] + st["grad_loads"], st["direct_gathers"], st["h2d_bytes"] / 1e9,
                   st["d2h_bytes"] / 1e9))
        # pools this small cannot hold the gather source: blocks are loaded and rows are read directly
        assert st["act_loads"] > cfg["k"] and st["direct_gathers"] > 0
        del s


BF16_TOL = 2e-2


def test_dense_workload_sampled(capsys):
    import psutil
    if psutil.virtual_memory().available < 140 * 2 ** 30:
        pytest.skip("needs ~100 GB of free host memory for the result tensors at full size")
    from oracle import fullgraph as og
    from paper_2605_11517_amd import Session
    from synth import features, glorot_weights, labels_and_mask, make_config, to_bf16_grid

    def say(msg):
        with capsys.disabled():
            print("[dense %.0fs] %s" % (time.time() - t0, msg), flush=True)

    t0 = time.time()
    cfg, rowptr, colidx = make_config("dense")
    n, dims = cfg["n"], cfg["dims"]
    X = to_bf16_grid(features(n, dims[0], cfg["seed"]))
    y, m = labels_and_mask(n, dims[-1], cfg["train_frac"], cfg["seed"])
    w = glorot_weights(dims, cfg["seed"], sage=False, bias_scale=0.05)
    for layer in w:
        layer["W"] = to_bf16_grid(layer["W"])
    say("inputs ready: n=%d entries=%d" % (n, rowptr[-1]))
    s = Session("gcn", dims, rowptr, colidx, cfg["k"], cfg["part"], cfg["seed"], X, w, y, m,
                dtype="bf16", layer_order="auto", fuse_gather=True, masked_backward=True,
                keep_forward="auto")                                                        # as bench.py times it
    assert s.ctx.gather_is_fused() and s.keeps_forward
    assert [s.ctx.layer_is_transform_first(l) for l in (1, 2, 3)] == [False, True, True]
    loss = s.epoch()
    got = s.results()
    del s
    say("GPU epoch done, loss %.6f" % loss)
    A = [X] + got["act"]                     # A[l]: activations the path itself produced
    W = [np.asarray(l["W"], dtype=np.float64) for l in w]
    b = [np.asarray(l["b"], dtype=np.float64) for l in w]

    # the operator by its definition: deg(v) = row length, entry weight 1 / sqrt(deg(u) deg(v));
    # the graph is symmetric, so the transposed operator has the same rows
    deg = np.diff(rowptr).astype(np.float64)
    inv = np.where(deg > 0, 1.0 / np.sqrt(np.maximum(deg, 1.0)), 0.0)
    rng = np.random.default_rng(11)
    V = np.unique(np.concatenate([rng.choice(n, 768, replace=False), np.argsort(deg)[-8:]]))

    def agg_rows(rows_of, verts):
        out = []
        for v in verts:
            cols = colidx[rowptr[v]:rowptr[v + 1]]
            out.append((rows_of(cols) * inv[cols][:, None]).sum(axis=0) * inv[v])
        return np.array(out)

    worst = {}
    # forward, layer by layer, each from the path's own previous activations
    for l in (1, 2, 3):
        z = agg_rows(lambda c, l=l: A[l - 1][c].astype(np.float64), V)
        ref = z @ W[l - 1] + b[l - 1]
        if l < 3:
            ref = np.maximum(ref, 0.0)
        worst["act[%d] rows" % (l - 1)] = rel_err(A[l][V], ref)
    say("forward rows checked")

    # loss and its gradient from the path's logits
    lref, gref = og.loss(A[3], y, m)
    assert abs(loss - lref) <= BF16_TOL * abs(lref)
    worst["gact[2]"] = rel_err(got["gact"][2], gref)
    dY3 = np.asarray(got["gact"][2], dtype=np.float64)

    def at_times(Aleft, G):
        """Aleft^T G in fp64, by row chunks."""
        acc = np.zeros((Aleft.shape[1], G.shape[1]))
        for r0 in range(0, n, 1 << 18):
            acc += Aleft[r0:r0 + (1 << 18)].astype(np.float64).T @ G[r0:r0 + (1 << 18)]
        return acc

    # output layer (transform-first): grad H = S^T dY, grad W = A2^T grad H, grad A2 = grad H W^T
    G3 = og.aggregate("gcn", rowptr, colidx, dY3, transpose=True)
    worst["gW[2]"] = rel_err(got["gW"][2], at_times(A[2], G3))
    worst["gb[2]"] = rel_err(got["gb"][2], dY3.sum(axis=0))
    worst["gact[1] rows"] = rel_err(got["gact"][1][V], G3[V] @ W[2].T)
    del G3
    say("output layer checked")

    # hidden layers on sampled columns (weight gradients) and sampled rows (input gradients)
    J = np.sort(rng.choice(dims[2], 8, replace=False))
    dY2J = np.where(A[2][:, J] > 0, got["gact"][1][:, J], 0.0).astype(np.float64)
    G2J = og.aggregate("gcn", rowptr, colidx, dY2J, transpose=True)
    worst["gW[1] cols"] = rel_err(got["gW"][1][:, J], at_times(A[1], G2J))
    worst["gb[1] cols"] = rel_err(got["gb"][1][J], dY2J.sum(axis=0))
    del G2J, dY2J
    g2 = agg_rows(lambda c: np.where(A[2][c] > 0, got["gact"][1][c], 0.0).astype(np.float64), V)
    worst["gact[0] rows"] = rel_err(got["gact"][0][V], g2 @ W[1].T)
    J1 = np.sort(rng.choice(dims[1], 8, replace=False))
    dY1J = np.where(A[1][:, J1] > 0, got["gact"][0][:, J1], 0.0).astype(np.float64)
    # aggregate-first layer: grad W = (S X)^T dY = X^T (S^T dY)
    G1J = og.aggregate("gcn", rowptr, colidx, dY1J, transpose=True)
    worst["gW[0] cols"] = rel_err(got["gW"][0][:, J1], at_times(A[0], G1J))
    worst["gb[0] cols"] = rel_err(got["gb"][0][J1], dY1J.sum(axis=0))
    say("worst relative errors: " + ", ".join("%s=%.2g" % kv for kv in sorted(worst.items())))
    bad = {k_: v for k_, v in worst.items() if not v <= BF16_TOL}
    assert not bad, bad


def test_dense_widths_end_to_end_against_oracle(capsys):
    """The widths of the dense workload (bfloat16, GCN 512-1024-1024-64) on 80,000 vertices in 4
    partitions against ONE whole oracle epoch from the same inputs: some 20,000 rows per partition
    are 78 row tiles of the 256 x 256-tile bfloat16 kernels plus a ragged tail, and errors
    compound through the layers as they do at full size.  Both layer orders."""
    from oracle import fullgraph as og
    from paper_2605_11517_amd import Session
    from synth import features, glorot_weights, labels_and_mask, rmat_graph, to_bf16_grid

    def say(msg):
        with capsys.disabled():
            print("[dense-e2e %.0fs] %s" % (time.time() - t0, msg), flush=True)

    t0 = time.time()
    n, dims, k, seed = 80_000, (512, 1024, 1024, 64), 4, 4
    rowptr, colidx = rmat_graph(n, 1_100_000, seed, symmetric=True, self_loops=True)
    X = to_bf16_grid(features(n, dims[0], seed))
    y, m = labels_and_mask(n, dims[-1], 0.1, seed)
    w = glorot_weights(dims, seed, sage=False, bias_scale=0.05)
    for layer in w:
        layer["W"] = to_bf16_grid(layer["W"])
    say("inputs ready: n=%d entries=%d" % (n, rowptr[-1]))
    fwd = og.forward("gcn", rowptr, colidx, dims, X, w)
    say("oracle forward done")
    for order in ("auto", "aggregate"):
        s = Session("gcn", dims, rowptr, colidx, k, "lp", seed, X, w, y, m, dtype="bf16", layer_order=order)
        assert [s.ctx.layer_is_transform_first(l) for l in (1, 2, 3)] == \
            ([False, True, True] if order == "auto" else [False, False, False])
        loss = s.epoch()
        got = s.results()
        del s
        worst = {"act[%d]" % l: both_errs(a, b) for l, (a, b) in enumerate(zip(got["act"], fwd.act))}
        assert all(v[0] <= BF16_TOL for v in worst.values()), worst
        ref = aligned_backward(og, fwd, got["act"], w, X, y, m, BF16_TOL, say, bf16=True,
                               got_gact=got["gact"] if order == "auto" else None)
        assert abs(loss - ref["loss"]) <= BF16_TOL * abs(ref["loss"])
        for key in ("gact", "gW", "gb"):
            for l, (a, b) in enumerate(zip(got[key], ref[key])):
                worst["%s[%d]" % (key, l)] = both_errs(a, b)
        say("layer order %s, loss %.6f (oracle %.6f); relative errors, gate (element-wise): %s"
            % (order, loss, ref["loss"], fmt_errs(worst)))
        bad = {k_: v[0] for k_, v in worst.items() if not v[0] <= BF16_TOL}
        assert not bad, (order, bad)


def test_beyond_recipe_streams_below_its_working_set(capsys):
    """The beyond-HBM recipe (GraphSAGE-mean 128-256-256-64, k = 256 switching-aware partitions,
    average degree 20) at a fifteenth of the `beyond` workload's vertices, where a whole fp64 oracle
    epoch is affordable: the streaming schedule with a block cache of a fifth of the activations
    and gradients against that oracle epoch, and bit for bit against the resident schedule."""
    from oracle import fullgraph as og
    from paper_2605_11517_amd import Session
    from synth import features, glorot_weights, labels_and_mask, make_config

    def say(msg):
        with capsys.disabled():
            print("[beyond %.0fs] %s" % (time.time() - t0, msg), flush=True)

    t0 = time.time()
    cfg, rowptr, colidx = make_config("beyond", n=400_000, m_draw=4_270_000)
    n, dims, k = cfg["n"], cfg["dims"], cfg["k"]
    assert k == 256 and cfg["model"] == "sage"
    X = features(n, dims[0], cfg["seed"], gen=cfg["gen"])
    y, m = labels_and_mask(n, dims[-1], cfg["train_frac"], cfg["seed"])
    w = glorot_weights(dims, cfg["seed"], sage=True, bias_scale=0.05)
    say("inputs ready: n=%d entries=%d, average degree %.1f" % (n, rowptr[-1], rowptr[-1] / n))
    working_set = n * (sum(dims) + sum(dims[1:])) * 4          # activations + gradients
    budget = working_set // 5
    results = {}
    # a second budget, three quarters of the working set: room for the transform-first layers'
    # whole-graph buffer beside two whole per-layer arrays, so the layers that narrow transform
    # first as in the resident schedule, and the epoch must reproduce it bit for bit
    roomy = int(working_set * 0.75)
    for name, kw in (("resident", {}), ("streaming", {"hbm_budget_bytes": budget}),
                     ("streaming-roomy", {"hbm_budget_bytes": roomy})):
        s = Session("sage", dims, rowptr, colidx, k, cfg["part"], cfg["seed"], X, w, y, m,
                    layer_order="auto", **kw)
        loss = s.epoch()
        results[name] = (loss, s.results(), [s.ctx.layer_is_transform_first(l) for l in (1, 2, 3)])
        if kw:
            st = s.ctx.get_stream_stats()
            stats = s.ctx.get_stats()
            say("%s: budget %.2f GB of a %.2f GB working set, alpha %.2f, %d block loads, %d hits, "
                "%d direct row gathers, %.1f GB in, %.1f GB out" % (
                    name, kw["hbm_budget_bytes"] / 1e9, working_set / 1e9, stats["sum_required"] / n,
                    st["act_loads"] + st["grad_loads"], st["act_hits"] + st["grad_hits"], st["direct_gathers"],
                    st["h2d_bytes"] / 1e9, st["d2h_bytes"] / 1e9))
            assert st["act_loads"] + st["direct_gathers"] >= k and st["d2h_bytes"] > 0
            if name == "streaming":
                # the pool cannot hold a layer: blocks are loaded, evicted and written back
                assert st["act_loads"] + st["direct_gathers"] > k
            if name == "streaming-roomy":
                # every output and gradient goes out once; inputs come in a few times at most
                assert st["d2h_bytes"] <= working_set and st["h2d_bytes"] <= 4 * working_set
        del s
    (loss_r, res, order_r), (loss_s, got, order_s) = results["resident"], results["streaming"]
    loss_m, got_m, order_m = results["streaming-roomy"]
    say("layer order resident %s, streaming %s, streaming-roomy %s" % (order_r, order_s, order_m))
    assert order_m == order_r == [False, True, True] and order_s == [False, False, False]
    assert loss_m == loss_r
    for key in ("act", "gact", "gW", "gWs", "gb"):
        for l, (a, b) in enumerate(zip(got_m[key], res[key])):
            assert np.array_equal(a, b), (key, l)
    say("roomy streaming epoch bit-identical to the resident one")
    del got_m, res
    fwd = og.forward("sage", rowptr, colidx, dims, X, w)
    worst = {"act[%d]" % l: both_errs(a, b) for l, (a, b) in enumerate(zip(got["act"], fwd.act))}
    assert all(v[0] <= TOL for v in worst.values()), worst
    ref = aligned_backward(og, fwd, got["act"], w, X, y, m, TOL, say, got_gact=got["gact"])
    assert abs(loss_s - ref["loss"]) <= TOL * abs(ref["loss"])
    for key in ("gact", "gW", "gWs", "gb"):
        for l, (a, b) in enumerate(zip(got[key], ref[key])):
            worst["%s[%d]" % (key, l)] = both_errs(a, b)
    say("loss %.6f (oracle %.6f); relative errors, gate (element-wise): %s" % (loss_s, ref["loss"], fmt_errs(worst)))
    bad = {k_: v[0] for k_, v in worst.items() if not v[0] <= TOL}
    assert not bad, bad


@pytest.mark.parametrize("heads", [None, (8, 8, 1)], ids=["one_head", "eight_heads"])
def test_mid_gat_workload_sampled(capsys, heads):
    """Graph attention at the bench's `mid_gat` size, with one head per layer and with eight
    32-column heads in the hidden layers.  A whole oracle epoch would need the
    edge-by-feature products of 134 M edges in memory; instead every layer's outputs and input
    gradients are recomputed for sampled vertices (eight hubs among them) from the layer's
    definition, one vertex at a time, from the path's own inputs to that step.  The softmax
    gradient of an edge u -> v needs sum_u' alpha(u' -> v) dY[v] . H[u'], which equals
    dY[v] . Z[v]: a per-vertex dot product."""
    import psutil
    if psutil.virtual_memory().available < 60 * 2 ** 30:
        pytest.skip("needs ~40 GB of free host memory")
    from oracle import fullgraph as og
    from paper_2605_11517_amd import Session
    from synth import attention_vectors, features, glorot_weights, labels_and_mask, make_config

    def say(msg):
        with capsys.disabled():
            print("[gat %.0fs] %s" % (time.time() - t0, msg), flush=True)

    t0 = time.time()
    cfg, rowptr, colidx = make_config("mid_gat")
    n, dims = cfg["n"], cfg["dims"]
    L = len(dims) - 1
    assert cfg["symmetric"] and not cfg["self_loops"]
    X = features(n, dims[0], cfg["seed"])
    y, m = labels_and_mask(n, dims[-1], cfg["train_frac"], cfg["seed"])
    w = attention_vectors(glorot_weights(dims, cfg["seed"], sage=False, bias_scale=0.05), cfg["seed"])
    for wl, h in zip(w, heads or ()):
        wl["heads"] = h
    say("inputs ready: n=%d entries=%d heads=%s" % (n, rowptr[-1], heads))
    # (the eight-head run as the bench runs it, with the gather fused into the kernels; the
    # one-head run through the staging buffer)
    s = Session("gat", dims, rowptr, colidx, cfg["k"], cfg["part"], cfg["seed"], X, w, y, m,
                fuse_gather=heads is not None, keep_forward=heads is not None)
    loss = s.epoch()
    got = s.results()
    del s
    say("GPU epoch done, loss %.6f" % loss)
    deg = np.diff(rowptr)
    rng = np.random.default_rng(5)
    # (with heads the per-vertex recomputation runs head by head: fewer sampled vertices, and the
    # eight hubs - 10^5 neighbours each - stay with the one-head run; hub rows with several heads
    # are compared with the whole oracle epoch on the smaller cases)
    V = (np.unique(np.concatenate([rng.choice(n, 504, replace=False), np.argsort(deg)[-8:]])) if heads is None
         else np.unique(rng.choice(n, 128, replace=False)))
    lref, gref = og.loss(got["act"][L - 1], y, m)
    assert abs(loss - lref) <= TOL * abs(lref)
    worst = {"gact[%d]" % (L - 1): rel_err(got["gact"][L - 1], gref)}
    worst.update(gat_sampled_errors(rowptr, colidx, dims, w, X, got["act"], got["gact"], got["gb"], V, say))
    say("worst relative errors: " + ", ".join("%s=%.2g" % kv for kv in sorted(worst.items())))
    bad = {k_: v for k_, v in worst.items() if not v <= TOL}
    assert not bad, bad


def test_large_workload_sampled(capsys):
    """`large` (50 M vertices, 868 M operator entries, directed, 3-layer GCN, k = 64) as bench.py
    runs it.  Tensors stay on the device (about 200 GB); the test fetches only what a check needs:
    rows of sampled vertices and of their in- and out-neighbours, sampled columns, and whole
    tensors chunk by chunk for the loss and the weight-gradient reductions."""
    import psutil
    import torch
    if psutil.virtual_memory().available < 120 * 2 ** 30:
        pytest.skip("needs ~80 GB of free host memory")
    if torch.cuda.get_device_properties(0).total_memory < 250 * 2 ** 30:
        pytest.skip("needs 250 GB of device memory")
    from oracle import fullgraph as og
    from paper_2605_11517_amd import Session
    from synth import features, glorot_weights, labels_and_mask, make_config

    def say(msg):
        with capsys.disabled():
            print("[large %.0fs] %s" % (time.time() - t0, msg), flush=True)

    t0 = time.time()
    cfg, rowptr, colidx = make_config("large")
    n, dims = cfg["n"], cfg["dims"]
    assert cfg["self_loops"] and len(dims) == 4
    say("graph ready: n=%d entries=%d" % (n, rowptr[-1]))
    X = features(n, dims[0], cfg["seed"], gen=cfg["gen"])
    y, m = labels_and_mask(n, dims[-1], cfg["train_frac"], cfg["seed"])
    w = glorot_weights(dims, cfg["seed"], sage=False, bias_scale=0.05)
    say("inputs ready")
    # the configuration bench.py times: device-counted switching-aware partitions, layer order by rows moved
    s = Session("gcn", dims, rowptr, colidx, cfg["k"], cfg["part"], cfg["seed"], X, w, y, m,
                layer_order="auto", fuse_gather=True, masked_backward=True, progress=say)   # as bench.py times it,
    # except that the backward pass recomputes layer 1's aggregate here: the bench keeps it (the
    # same bits, shown on the smaller cases and on `mid` at full size) when 24 GiB more fit, and
    # this test needs that room for the rows and columns it fetches
    assert s.ctx.gather_is_fused()
    assert cfg["part"] == "switching_device"
    assert [s.ctx.layer_is_transform_first(l) for l in (1, 2, 3)] == [False, True, True]
    del X
    loss = s.epoch()
    torch.cuda.synchronize()
    say("GPU epoch done, loss %.6f" % loss)
    order = s.ctx.get_order()[0].astype(np.int64)        # library row i holds original vertex order[i]
    pos = np.empty(n, dtype=np.int64)
    pos[order] = np.arange(n, dtype=np.int64)
    W = [np.asarray(l["W"], dtype=np.float64) for l in w]
    b = [np.asarray(l["b"], dtype=np.float64) for l in w]
    feat_act = [s.feat] + s.act                          # device tensors, library order

    def rows(dev_tensor, verts):
        """Rows of original vertices `verts` as fp64."""
        idx = torch.from_numpy(pos[np.asarray(verts, dtype=np.int64)]).to(dev_tensor.device)
        return dev_tensor[idx].cpu().numpy().astype(np.float64)

    def columns(dev_tensor, cols):
        """Columns `cols` of every vertex, original order, fp64."""
        c = dev_tensor[:, torch.from_numpy(np.asarray(cols, dtype=np.int64)).to(dev_tensor.device)].cpu().numpy()
        out = np.empty(c.shape, dtype=np.float64)
        out[order] = c
        return out

    CH = 1 << 21

    pin = torch.empty((CH, max(dims)), dtype=torch.float32).pin_memory()

    def at_times(dev_tensor, G):
        """dev_tensor^T G in fp64 with G in original order: fetched through a pinned buffer and
        multiplied by row chunks (plain CPU tensor operations, all host cores)."""
        d = dev_tensor.shape[1]
        acc = torch.zeros((d, G.shape[1]), dtype=torch.float64)
        for r0 in range(0, n, CH):
            cnt = min(CH, n - r0)
            buf = pin.view(-1)[:cnt * d].view(cnt, d)
            buf.copy_(dev_tensor[r0:r0 + cnt])
            acc += buf.double().T @ torch.from_numpy(G[order[r0:r0 + cnt]])
        return acc.numpy()

    # the operator by its definition: deg(v) = row length (the CSR holds the self-loops),
    # entry weight 1 / sqrt(deg(u) deg(v))
    deg = np.diff(rowptr).astype(np.float64)
    inv = 1.0 / np.sqrt(deg)
    rng = np.random.default_rng(13)
    V = np.unique(np.concatenate([rng.choice(n, 256, replace=False), np.argsort(deg)[-4:]]))
    # out-edges of the sampled vertices: entries whose column is sampled, with their rows
    lut = np.zeros(n, dtype=bool)
    lut[V] = True
    ent = np.flatnonzero(lut[colidx])
    ent_src = colidx[ent].astype(np.int64)
    ent_dst = np.searchsorted(rowptr, ent, side="right") - 1
    del lut
    say("%d sampled vertices, %d in-entries, %d out-entries"
        % (len(V), int(deg[V].sum()), len(ent)))

    worst = {}
    # forward rows, each layer from the path's own previous activations
    for l in (1, 2, 3):
        ref = []
        for v in V:
            u = colidx[rowptr[v]:rowptr[v + 1]].astype(np.int64)
            z = (rows(feat_act[l - 1], u) * inv[u][:, None]).sum(axis=0) * inv[v]
            r = z @ W[l - 1] + b[l - 1]
            ref.append(np.maximum(r, 0.0) if l < 3 else r)
        worst["act[%d] rows" % (l - 1)] = both_errs(rows(feat_act[l], V), np.array(ref))
    say("forward rows checked")

    # loss and its gradient: the oracle's routine on the rows of the train mask (fetched from the
    # device, library order); every other row of the gradient must be exactly zero
    y_lib, m_lib = y[order], m[order]
    tr = np.flatnonzero(m_lib)
    tr_dev = torch.from_numpy(tr).to(s.dev)
    lref, gref = og.loss(s.act[2][tr_dev].cpu().numpy(), y_lib[tr], np.ones(len(tr), dtype=np.uint8))
    assert abs(loss - lref) <= TOL * abs(lref), (loss, lref)
    worst["gact[2]"] = both_errs(s.gact[2][tr_dev].cpu().numpy(), gref)
    rest = torch.ones(n, dtype=torch.bool, device=s.dev)
    rest[tr_dev] = False
    for r0 in range(0, n, CH * 4):
        assert not bool(s.gact[2][r0:r0 + CH * 4][rest[r0:r0 + CH * 4]].any())
    del rest, tr_dev, gref
    say("loss and its gradient checked (%d train rows)" % len(tr))

    def dY_rows(l, verts):
        """Rows of dLoss/d(pre-activation) of layer l."""
        g = rows(s.gact[l - 1], verts)
        return g if l == 3 else np.where(rows(s.act[l - 1], verts) > 0, g, 0.0)

    def dY_columns(l, cols):
        g = columns(s.gact[l - 1], cols)
        return g if l == 3 else np.where(columns(s.act[l - 1], cols) > 0, g, 0.0)

    # transform-first layers 3 and 2: grad H = S^T dY, grad W = A^{l-1 T} grad H,
    # grad A^{l-1} = grad H W^T; rows of S^T from the sampled vertices' out-entries
    for l in (3, 2):
        d = dY_rows(l, ent_dst) * (inv[ent_src] * inv[ent_dst])[:, None]
        GH = np.zeros((len(V), dims[l]))
        np.add.at(GH, np.searchsorted(V, ent_src), d)
        worst["gact[%d] rows" % (l - 2)] = both_errs(rows(s.gact[l - 2], V), GH @ W[l - 1].T)
        J = np.sort(rng.choice(dims[l], 8, replace=False))
        dYJ = dY_columns(l, J)
        GJ = og.aggregate("gcn", rowptr, colidx, dYJ, transpose=True)
        worst["gW[%d] cols" % (l - 1)] = both_errs(s.gw[3 * (l - 1)][:, torch.from_numpy(J).to(s.dev)].cpu().numpy(),
                                                   at_times(feat_act[l - 1], GJ))
        worst["gb[%d] cols" % (l - 1)] = both_errs(s.gw[3 * (l - 1) + 2].cpu().numpy()[J], dYJ.sum(axis=0))
        del dYJ, GJ
        say("layer %d checked" % l)
    # aggregate-first layer 1: grad W = (S X)^T dY = X^T (S^T dY)
    J = np.sort(rng.choice(dims[1], 8, replace=False))
    dYJ = dY_columns(1, J)
    GJ = og.aggregate("gcn", rowptr, colidx, dYJ, transpose=True)
    worst["gW[0] cols"] = both_errs(s.gw[0][:, torch.from_numpy(J).to(s.dev)].cpu().numpy(), at_times(s.feat, GJ))
    worst["gb[0] cols"] = both_errs(s.gw[2].cpu().numpy()[J], dYJ.sum(axis=0))
    say("relative errors, gate (element-wise): " + fmt_errs(worst))
    bad = {k_: v[0] for k_, v in worst.items() if not v[0] <= TOL}
    assert not bad, bad
