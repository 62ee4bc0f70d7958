#!/usr/bin/env python3
"""One-GPU benchmark of the partition-wise full-graph GNN epoch (forward + loss + backward).

A "step" is one gnn_epoch over the whole synthetic graph: for every layer and partition
gather -> aggregate -> transform, the loss, then for every layer and partition regather ->
recompute -> dW / dZ -> transposed aggregate -> scatter-add.  Inputs are resident in HBM
before the timed region.  Prints ONE JSON line (see the keys below).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload large|mid|dense|beyond|...]

The headline is the largest HBM-resident configuration (`large`); with no --workload the same
line carries the `mid` workload's result under "other_workloads" (the configuration whose
oracle epoch is affordable in full, timed on the same inputs).
"""
from __future__ import annotations

import argparse
import json
import os
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_F32_PEAK_TFLOPS = 157.3   # dense fp32 matrix cores
MFMA_BF16_PEAK_TFLOPS = 2500.0 # dense bf16 matrix cores


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def padded_width(d):
    """Row width (elements) of H = A W in a transform-first layer; mirrors gnn_ctx::padded()."""
    return (d + 3) // 4 * 4


def algorithmic_bytes(stats, dims, model, n_parts, es=4, fused_scatter=False, xf=None, pad=padded_width,
                      masked=None, first_touch=False, kept=False):
    """HBM bytes the method has to move per epoch, by kernel class (lower bound: every needed
    source row is read once per partition).  es = bytes per stored activation (4 fp32, 2 bf16);
    gradients of activations are always fp32.  xf[l-1]: layer l transforms first, so it
    gathers, aggregates and scatter-accumulates rows of its (padded) output width, once
    forward and once backward, with no regather and no recompute.  masked = (entries, rows,
    train vertices) of the output layer's transposed operator over train vertices, when in use:
    that pass then reads only those entries and the gradient rows of train vertices, and adds
    onto `rows` rows.  first_touch: the epoch stores the first contribution to a row of a
    gradient array instead of adding it onto a zeroed one (every row once: n rows are written
    without being read; not with the operator over train vertices).  kept: aggregate-first layers
    keep their aggregate from the forward pass, so the backward pass neither regathers nor
    aggregates again."""
    n, nnz, k = stats["n"], stats["nnz"], stats["k"]
    sum_r = n + stats["sum_boundary"]            # sum over partitions of |own_p| + |B_p|
    sum_b = stats["sum_boundary"]
    L = len(dims) - 1
    per_entry = 4 + (4 if model in ("gcn", "gat") else 0)  # column index (+ entry weight: GCN, GAT)
    out = {"gather": 0, "spmm": 0, "spmm_t": 0, "scatter": 0}
    xf = xf or [False] * L
    for l in range(1, L + 1):
        if xf[l - 1]:
            wp = pad(dims[l])
            row = wp * 4                         # aggregated sums and gradients of H: fp32
            hrow = wp * es                       # rows of H (and of dY) in the storage type
            one_gather = 2 * sum_b * hrow + 4 * sum_b
            one_spmm = per_entry * nnz + 8 * (n + k) + sum_r * hrow + n * row + (4 * n if model == "sage" else 0)
            # graph attention regathers, and reads every needed row once more for the edge-wise
            # products dY[v] . H[u] (same traffic as an aggregation, 4 bytes written per entry)
            out["gather"] += one_gather * (2 if model == "gat" else 1)
            out["spmm"] += one_spmm * (2 if model == "gat" else 1)
            if masked and l == L:
                m_e, m_r, m_v = masked
                out["spmm_t"] += 8 * m_e + 12 * (m_r + k) + m_v * hrow + 2 * m_r * row
            else:
                out["spmm_t"] += 8 * nnz + 8 * (sum_r + k) + n * hrow + 2 * sum_r * row + 4 * sum_b
                if first_touch and model != "gat":
                    out["spmm_t"] -= n * row
            continue
        d = dims[l - 1]
        row = d * es
        grow = d * 4
        # forward + backward regather
        out["gather"] += (1 if kept else 2) * (2 * sum_b * row + 4 * sum_b)
        # forward + recompute
        spmm = per_entry * nnz + 8 * (n + k) + sum_r * row + n * row + (4 * n if model == "sage" else 0)
        out["spmm"] += (1 if kept else 2) * spmm
        if l >= 2:
            if fused_scatter and masked and l == L:
                m_e, m_r, m_v = masked
                out["spmm_t"] += 8 * m_e + 12 * (m_r + k) + m_v * row + 2 * m_r * grow
            elif fused_scatter:
                # transposed aggregation adds its rows straight onto their owners: read dZ once,
                # read-modify-write every required row of grad A^{l-1}
                out["spmm_t"] += 8 * nnz + 8 * (sum_r + k) + n * row + 2 * sum_r * grow + 4 * sum_b
                if first_touch:
                    out["spmm_t"] -= n * grow
            else:
                out["spmm_t"] += 8 * nnz + 8 * (sum_r + k) + n * row + sum_r * grow
                out["scatter"] += 3 * sum_r * grow + 4 * sum_b
    return out


def fused_layers(dims, xf, dtype):
    """Layers (0-based) whose forward contraction runs inside the aggregation kernel (the
    aggregated tile stays in LDS); mirrors spmm_gemm_fused_ok() of the library."""
    if dtype != "f32" or os.environ.get("GNNMI_FUSE_AGG", "0")[:1] != "1":
        return []
    return [l for l in range(len(dims) - 1)
            if not xf[l] and dims[l] % 4 == 0 and 32 < dims[l] <= 128 and dims[l + 1] <= 256]


def gemm_flops(stats, dims, model, fused=()):
    """Flops of the contractions that run as kernels of their own, by class (the forward
    contraction of a fused layer is part of the aggregation kernel's time, so it is left out)."""
    n = stats["n"]
    L = len(dims) - 1
    mult = 2 if model == "sage" else 1
    fwd = sum(2 * n * dims[l] * dims[l + 1] * mult for l in range(L) if l not in fused)
    dw = fwd
    dz = sum(2 * n * dims[l] * dims[l + 1] * mult for l in range(1, L))
    return {"gemm_fwd": fwd, "gemm_dw": dw, "gemm_dz": dz}


def oracle_epoch_seconds(cfg, rowptr, colidx, X, w, y, m):
    """One fp64 full-graph epoch (forward + loss + backward) of the oracle, as it stands."""
    from oracle import fullgraph as og
    t0 = time.perf_counter()
    if cfg["model"] == "gat":
        from oracle import gat as ogat
        ogat.epoch(rowptr, colidx, cfg["dims"], X, w, y, m)
    else:
        og.epoch(cfg["model"], rowptr, colidx, cfg["dims"], X, w, y, m)
    return time.perf_counter() - t0


GAT_HEADS = None     # --gat-heads: attention heads per layer of the graph-attention workloads


def make_inputs(name, cfg_over):
    from synth import attention_vectors, features, glorot_weights, labels_and_mask, make_config
    cfg, rowptr, colidx = make_config(name, **cfg_over)
    n, dims, model = cfg["n"], cfg["dims"], cfg["model"]
    X = features(n, dims[0], cfg["seed"], gen=cfg.get("gen", "numpy"))
    y, m = labels_and_mask(n, dims[-1], cfg["train_frac"], cfg["seed"])
    w = glorot_weights(dims, cfg["seed"], sage=(model == "sage"))
    if model == "gat":
        attention_vectors(w, cfg["seed"])
        if GAT_HEADS:
            if len(GAT_HEADS) != len(w):
                raise SystemExit("--gat-heads needs one head count per layer (%d)" % len(w))
            for wl, h in zip(w, GAT_HEADS):
                wl["heads"] = h
    return cfg, rowptr, colidx, X, y, m, w


def cpu_baseline(name, cfg, inputs, mode, sample_n, log_fn):
    """The oracle timed on the host cores.  mode "same": on the very inputs the GPU epoch ran on
    (affordable for `mid`, `tiny`, `mini_*`: about a minute on a GPU box).  mode "scaled": on a
    down-scaled instance of the same workload (same generator and seed, same average degree and
    layer widths, n and the number of draws multiplied by one factor), sized by a short probe to
    roughly 15 s of CPU work unless sample_n is given; the factor is stated."""
    from oracle import fullgraph as og
    if mode == "same":
        c, rowptr, colidx, X, y, m, w = inputs
        dt = oracle_epoch_seconds(c, rowptr, colidx, X, w, y, m)
        nnz = int(rowptr[-1]) + (c["n"] if c["model"] in ("gcn", "gat") and not c["self_loops"] else 0)
        log_fn("cpu oracle on the same inputs: epoch %.2f s on %d threads" % (dt, og.num_threads()))
        return {"value": nnz / dt, "unit": "edges/s", "cores": og.num_threads(), "kind": "oracle",
                "sample": "the same inputs in full (n=%d, %d operator entries): one fp64 full-graph epoch "
                          "(fwd+loss+bwd) in %.2f s" % (c["n"], nnz, dt), "epoch_s": dt}

    def run(nn):
        f = nn / cfg["n"]
        c, rowptr, colidx, X, y, m, w = make_inputs(name, {"n": nn, "m_draw": int(cfg["m_draw"] * f)})
        dt = oracle_epoch_seconds(c, rowptr, colidx, X, w, y, m)
        nnz = int(rowptr[-1]) + (nn if c["model"] in ("gcn", "gat") and not c["self_loops"] else 0)
        return dt, nnz

    if sample_n <= 0:
        probe_n = max(2000, min(cfg["n"], 2000 if cfg["model"] == "gat" else 20000))
        dt, _ = run(probe_n)
        sample_n = int(max(probe_n, min(cfg["n"], 1_000_000, probe_n * 15.0 / max(dt, 1e-3))))
        log_fn("cpu oracle probe: n=%d took %.2f s -> sample n=%d" % (probe_n, dt, sample_n))
    dt, nnz = run(sample_n)
    log_fn("cpu oracle: n=%d nnz=%d epoch %.2f s on %d threads" % (sample_n, nnz, dt, og.num_threads()))
    return {"value": nnz / dt, "unit": "edges/s", "cores": og.num_threads(), "kind": "oracle",
            "sample": "the same workload scaled by %.4g (same generator, seed, average degree and layer widths; "
                      "n=%d, %d operator entries): one fp64 full-graph epoch (fwd+loss+bwd) in %.2f s"
                      % (sample_n / cfg["n"], sample_n, nnz, dt),
            "epoch_s": dt}


def git_head():
    try:
        return subprocess.run(["git", "-C", ROOT, "rev-parse", "--short", "HEAD"], capture_output=True,
                              text=True, timeout=10).stdout.strip() or None
    except Exception:
        return None


def run_workload(name, args, steps, warmup, want_cpu):
    """Builds the inputs of one named workload, times `steps` epochs after `warmup` and returns
    the result dict (the JSON line's fields for this workload)."""
    import torch
    from paper_2605_11517_amd import Session
    from synth import CONFIGS

    t0 = time.perf_counter()
    over = {}
    if args.graph_scale != 1.0:
        base = CONFIGS[name]
        over = {"n": int(base["n"] * args.graph_scale), "m_draw": int(base["m_draw"] * args.graph_scale)}
    inputs = make_inputs(name, over)
    cfg, rowptr, colidx, X, y, m, w = inputs
    n, dims, model = cfg["n"], cfg["dims"], cfg["model"]
    log("[%s] inputs: n=%d entries=%d (%.1f s)" % (name, n, rowptr[-1], time.perf_counter() - t0))
    t1 = time.perf_counter()
    if args.partitioner:
        cfg["part"] = args.partitioner
    budget = int(args.hbm_budget_gb * 2 ** 30)
    if name == "beyond" and not budget:
        # the beyond-HBM recipe always streams, with HBM in the proportion the full recipe would
        # find on this device: 288 GB for 512 GB of activations and gradients
        budget = int(n * (sum(dims) + sum(dims[1:])) * 4 * 0.56)
    s = Session(model, dims, rowptr, colidx, cfg["k"], cfg["part"], cfg["seed"], X, w, y, m,
                dtype=cfg["dtype"], hbm_budget_bytes=budget,
                layer_order=args.layer_order, fuse_gather=not args.staged_gather,
                keep_forward=(False if args.recompute or budget else "auto"),
                masked_backward=not args.full_backward, storage_dir=args.storage_dir,
                host_budget_bytes=int(args.host_budget_gb * 2 ** 30), progress=lambda msg: log("  " + msg))
    if args.storage_dir and args.storage_drop_results:
        s.ctx.storage_keep_results(False)
    gather_fused = s.ctx.gather_is_fused()
    keeps_forward = s.keeps_forward        # (as the timed epochs run; the paper-order run below recomputes)
    m_entries, m_rows = s.ctx.masked_backward_size()
    masked = (m_entries, m_rows, int((m != 0).sum())) if m_rows or m_entries else None
    xf = [s.ctx.layer_is_transform_first(l) for l in range(1, len(dims))]
    # gnn_epoch runs a transform-first layer's contractions beside the aggregate-first layer below it
    overlapped = (cfg["dtype"] != "bf16" and model != "gat" and not budget and
                  any((not a) and b for a, b in zip(xf, xf[1:])) and
                  os.environ.get("GNNMI_OVERLAP", "1")[:1] != "0")
    es = 2 if cfg["dtype"] == "bf16" else 4
    mfma_peak = MFMA_BF16_PEAK_TFLOPS if cfg["dtype"] == "bf16" else MFMA_F32_PEAK_TFLOPS
    stats = s.ctx.get_stats()
    setup_s = time.perf_counter() - t1        # partitioner, metadata, upload, binding
    log("[%s] partitions built and bound: k=%d alpha=%.3f sum_boundary=%d (%.1f s)" % (
        name, stats["k"], stats["sum_required"] / n, stats["sum_boundary"], time.perf_counter() - t1))
    if not (want_cpu and name in SAME_INPUT_ORACLE):
        del X, rowptr, colidx
        inputs = None

    if args.copy_calibration:
        a = torch.empty(1 << 28, dtype=torch.float32, device="cuda:0").normal_()
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        b.copy_(a)                             # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del a, b

    def step(i):
        if args.train:
            return s.train(1, optimizer="adam", lr=0.01, dropout=0.5, seed=cfg["seed"], first_epoch=i)[0]
        return s.epoch()                       # synchronises the stream before returning

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    # Timed region: HIP events bracket only the dominant kernel (every aggregation launch), which
    # costs about 1 % of the epoch.  Bracketing every kernel class puts ~10 us of idle time between
    # most of an epoch's ~800 launches (4-6 %), so that breakdown comes from one more epoch after
    # the timed region.
    prof = {}
    s.ctx.set_profiling(0 if args.no_profile else 2)
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    loss = 0.0
    for i in range(steps):
        loss = step(warmup + i)
        if not args.no_profile:
            for cname, (ms, launches) in s.ctx.get_profile().items():
                a = prof.setdefault(cname, [0.0, 0])
                a[0] += ms
                a[1] += launches
    torch.cuda.synchronize()
    dt = time.perf_counter() - t2
    breakdown = {}
    if not args.no_profile:
        # one-stream schedule for the breakdown (GNNMI_OVERLAP is read per epoch): in the timed
        # region some contractions run on a side stream beside the aggregation kernels, which is
        # faster in wall time but stretches each of the kernels that share the chip
        previous = os.environ.get("GNNMI_OVERLAP")
        os.environ["GNNMI_OVERLAP"] = "0"
        s.ctx.set_profiling(1)
        step(warmup + steps)
        torch.cuda.synchronize()
        breakdown = {cname: (ms, launches) for cname, (ms, launches) in s.ctx.get_profile().items()}
        if previous is None:
            del os.environ["GNNMI_OVERLAP"]
        else:
            os.environ["GNNMI_OVERLAP"] = previous
    s.ctx.set_profiling(0)
    ms_per_step = dt / steps * 1e3
    nnz = stats["nnz"]
    log("[%s] epoch %.2f ms, loss %.5f" % (name, ms_per_step, loss))

    stream_stats = s.ctx.get_stream_stats() if budget else None
    storage_stats = s.ctx.get_storage_stats() if args.storage_dir else None

    # the same epoch with every layer in the paper's order (aggregate, then transform; regather
    # and recompute in the backward pass of every layer): context, not the headline
    # and with the gather as a step of its own, through the staging buffer
    paper_ms, paper_gather = None, None
    # the timed schedule with the paper's backward rule: forward results recomputed (regather +
    # recompute of aggregate-first layers; H, scores and attention weights of attention layers)
    recompute_ms = None
    if keeps_forward and not args.no_paper_order and not args.train and not budget:
        s.set_keep_forward(False)
        for i in range(min(warmup, 1)):
            s.epoch()
        torch.cuda.synchronize()
        t3 = time.perf_counter()
        reps = max(1, min(steps, 3))
        for i in range(reps):
            s.epoch()
        torch.cuda.synchronize()
        recompute_ms = (time.perf_counter() - t3) / reps * 1e3
        log("[%s] forward results recomputed in the backward pass: epoch %.2f ms" % (name, recompute_ms))
    if ((args.layer_order == "auto" and any(xf)) or gather_fused) and not args.no_paper_order and \
            model != "gat" and not args.train and not budget:
        s.set_keep_forward(False)               # the paper's backward pass regathers and recomputes
        if any(xf):
            s.set_layer_order("aggregate")
        s.set_gather_fusion(False)
        s.set_masked_backward(False)
        for i in range(min(warmup, 1)):
            s.epoch()
        torch.cuda.synchronize()
        t3 = time.perf_counter()
        reps = max(1, min(steps, 3))
        for i in range(reps):
            s.epoch()
        torch.cuda.synchronize()
        paper_ms = (time.perf_counter() - t3) / reps * 1e3
        log("[%s] every layer aggregate-first, gather through staging: epoch %.2f ms" % (name, paper_ms))
        if not args.no_profile:
            s.ctx.set_profiling(1)
            s.epoch()
            torch.cuda.synchronize()
            g_ms, g_launches = s.ctx.get_profile()["gather"]
            s.ctx.set_profiling(0)
            g_bytes = algorithmic_bytes(stats, dims, model, stats["k"], es, fused_scatter=True)["gather"]
            if g_ms > 0:
                paper_gather = {"ms_per_epoch": g_ms, "launches_per_epoch": g_launches,
                                "algorithmic_GBps": g_bytes / (g_ms * 1e-3) / 1e9,
                                "frac_hbm_peak": g_bytes / (g_ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
    elif args.layer_order == "auto" and any(xf) and not args.no_paper_order and model != "gat" and not args.train:
        s.set_keep_forward(False)
        s.set_layer_order("aggregate")
        for i in range(min(warmup, 1)):
            s.epoch()
        torch.cuda.synchronize()
        t3 = time.perf_counter()
        reps = max(1, min(steps, 3))
        for i in range(reps):
            s.epoch()
        torch.cuda.synchronize()
        paper_ms = (time.perf_counter() - t3) / reps * 1e3
        log("[%s] every layer aggregate-first: epoch %.2f ms" % (name, paper_ms))
    del s
    torch.cuda.empty_cache()

    out = {
        "metric": ("full-graph training-step throughput (fwd with dropout+loss+bwd+Adam step), operator "
                   "entries per second" if args.train else
                   "full-graph epoch throughput (fwd+loss+bwd), operator entries per second"),
        "value": nnz / (dt / steps),
        "unit": "edges/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg["dtype"], "data": "synthetic",
        "config": {"workload": name + ("" if args.graph_scale == 1.0 else " x%g" % args.graph_scale) +
                               (" heads=%s" % args.gat_heads if args.gat_heads and model == "gat" else "") +
                   ("" if not budget else " (streaming, %.3g GiB block cache)" % (budget / 2 ** 30)),
                   "n": n, "operator_entries": nnz, "model": model,
                   "dims": list(dims), "k": stats["k"], "partitioner": cfg["part"],
                   "alpha": stats["sum_required"] / n, "sum_boundary": stats["sum_boundary"],
                   "layer_order": ["transform-first" if t else "aggregate-first" for t in xf],
                   "forward_results": ("kept for the backward pass (aggregate of aggregate-first layers; H, scores "
                                       "and attention weights of attention layers)" if keeps_forward
                                       else "recomputed in the backward pass (regather + recompute)"),
                   "gather": ("fused into the aggregation (rows read from the whole-graph array through B_p)"
                              if gather_fused else "a step of its own, through the staging buffer"),
                   "output_layer_backward": ("%d operator entries of train vertices of %d (the loss gradient is "
                                             "zero elsewhere)" % (masked[0], nnz) if masked
                                             else "every operator entry"),
                   "side_stream_overlap": overlapped,
                   "setup_s": setup_s},
        "loss": loss,
    }
    if recompute_ms is not None:
        # the same schedule with the paper's backward rule (nothing kept from the forward pass)
        out["ms_per_step_recompute"] = recompute_ms
    if paper_ms is not None:
        out["ms_per_step_paper_order"] = paper_ms
        if paper_gather is not None:
            out["paper_order_gather"] = paper_gather
    if prof:
        # resident epochs store the first contribution to a gradient row (GNNMI_FIRST_TOUCH=0: off)
        first_touch = not budget and model != "gat" and os.environ.get("GNNMI_FIRST_TOUCH", "1")[:1] != "0"
        out["config"]["gradient_rows_first_touch_store"] = first_touch
        ab = algorithmic_bytes(stats, dims, model, stats["k"], es,
                               fused_scatter=prof.get("scatter", (0, 0))[1] == 0, xf=xf, masked=masked,
                               first_touch=first_touch, kept=keeps_forward)
        if gather_fused:
            ab["gather"] = 0                    # no staging copy is made
        fused = fused_layers(dims, xf, cfg["dtype"]) if model != "gat" else []
        fl = gemm_flops(stats, dims, model, fused)
        out["config"]["forward_fused_with_aggregation"] = [l + 1 for l in fused]
        # per kernel class, from the one epoch run after the timed region with every class bracketed,
        # on one stream
        classes = {}
        for cname, (ms, launches) in breakdown.items():
            e = {"ms_per_epoch": ms, "launches_per_epoch": launches}
            if cname in ab and ms > 0:
                e["algorithmic_GBps"] = ab[cname] / (ms * 1e-3) / 1e9
                e["frac_hbm_peak"] = e["algorithmic_GBps"] / HBM_PEAK_GBS
            if cname in fl and ms > 0:
                e["TFLOPps"] = fl[cname] / (ms * 1e-3) / 1e12
                e["frac_mfma_peak"] = e["TFLOPps"] / mfma_peak
            classes[cname] = e
        g_ms = breakdown.get("gather", (0, 0))[0] + breakdown.get("spmm", (0, 0))[0] + \
            breakdown.get("spmm_t", (0, 0))[0] + breakdown.get("scatter", (0, 0))[0] + \
            breakdown.get("spmm_reduce", (0, 0))[0]
        if g_ms > 0:
            classes["gather+spmm"] = {"ms_per_epoch": g_ms,
                                      "algorithmic_GBps": sum(ab.values()) / (g_ms * 1e-3) / 1e9,
                                      "frac_hbm_peak": sum(ab.values()) / (g_ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
        out["kernel_classes"] = classes
        sp_ms, sp_launches = prof["spmm"]
        passes = sum(1 if t else 2 for t in xf)       # forward (+ recompute) aggregations
        if model == "gat":
            passes = 2 * len(xf)                        # aggregation + edge-wise products
        tp_ms = prof["spmm_t"][0]
        transposed = (len(dims) - 2) + (1 if xf[0] else 0)   # a transform-first layer 1 still pushes grad H
        if sp_ms + tp_ms > 0:
            out["aggregated_edges_per_s"] = nnz * (passes + transposed) * steps / ((sp_ms + tp_ms) * 1e-3)
        # dominant kernel: the aggregation, every launch of it (forward, recompute and transposed)
        k_ms = sp_ms + tp_ms
        k_launches = sp_launches + prof["spmm_t"][1]
        k_bytes = (ab["spmm"] + ab["spmm_t"]) * steps
        if k_ms > 0 and k_launches > 0:
            achieved = k_bytes / (k_ms * 1e-3) / 1e9
            # measured HBM-side traffic of the same kernels from the committed counter summary
            # (rocprofv3 FETCH_SIZE + WRITE_SIZE, scaled by a plain copy), per launch
            traffic, source = None, None
            from paper_2605_11517_amd.profiling import read_traffic, read_taken_at
            path = os.path.join(ROOT, "profiles", "pmc_%s_epoch.md" % name)
            table = read_traffic(path)
            if table and args.graph_scale == 1.0:
                rows = [v for kk, v in table.items() if kk.startswith(("k_spmm_items", "k_spmm_slots", "k_spmm_short"))]
                if rows:
                    tot_l = sum(r["launches"] for r in rows)
                    traffic = sum(r["bytes_per_launch"] * r["launches"] for r in rows) / tot_l
                    source = {"file": "profiles/pmc_%s_epoch.md" % name, "taken_at_commit": read_taken_at(path),
                              "this_run_commit": git_head()}
            L = len(dims) - 1
            upper = 0
            for l in range(L):
                # the output layer's transposed pass over train vertices only reads that many rows
                last_t = (masked[0], masked[1]) if masked and l == L - 1 else (stats["nnz"], n)
                if xf[l]:
                    roww = padded_width(dims[l + 1]) * 4
                    upper += (2 if model == "gat" else 1) * (stats["nnz"] * (4 + roww) + n * roww)
                    upper += last_t[0] * (4 + roww) + last_t[1] * roww
                else:
                    upper += 2 * (stats["nnz"] * (4 + dims[l] * es) + n * dims[l] * es)
                    if l > 0:
                        upper += last_t[0] * (4 + dims[l] * es) + last_t[1] * dims[l] * es
            out["roofline"] = {
                "kernel": "k_spmm_slots / k_spmm_short / k_spmm_items (aggregation over T_p and T_p^T: forward, recompute, "
                          "transposed; column-sliced variant where rows are whole 128-byte lines)",
                "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": source,
                "bytes_per_launch": k_bytes / k_launches,
                "avg_launch_ms": k_ms / k_launches, "launches_per_epoch": k_launches / steps,
                "no_reuse_bytes_per_launch": upper * steps / k_launches,
                "traffic_GBps": None if traffic is None else traffic / (k_ms / k_launches * 1e-3) / 1e9,
                "traffic_over_algorithmic": None if traffic is None else traffic / (k_bytes / k_launches),
                "note": "achieved = bytes the method must move if every needed source row is read "
                        "once per partition, over the HIP-event time of the kernel in the timed region" +
                        (" (where contractions of the next layer run beside part of its launches on a side "
                         "stream and stretch them; kernel_classes come from a one-stream epoch)"
                         if overlapped else "") + "; traffic = measured "
                        "fetch+write bytes per launch (rocprofv3 counters, from the named summary); no_reuse = "
                        "one source row read per operator entry",
            }
        out["profiled_ms_per_step"] = sum(v[0] for v in breakdown.values())
    if storage_stats is not None:
        # file traffic of the whole run (placement of the features, warm-up and timed epochs)
        storage_stats["epochs_run"] = warmup + steps + (1 if not args.no_profile else 0)
        out["storage"] = storage_stats
        out["config"]["workload"] += " (storage tier: %.3g GiB host pool over %.3g GiB of arrays)" % (
            storage_stats["host_pool_bytes"] / 2 ** 30, storage_stats["array_bytes"] / 2 ** 30)
    if stream_stats is not None:
        stream_stats["pcie_GBps"] = (stream_stats["h2d_bytes"] + stream_stats["d2h_bytes"]) / (ms_per_step * 1e-3) / 1e9
        out["streaming"] = stream_stats
    if want_cpu:
        mode = "same" if (name in SAME_INPUT_ORACLE and args.graph_scale == 1.0 and inputs is not None) else "scaled"
        out["cpu_baseline"] = cpu_baseline(name, cfg, inputs, mode, args.cpu_sample_n, log)
    return out


# workloads whose whole oracle epoch on the same inputs takes about a minute or less on a GPU machine
SAME_INPUT_ORACLE = ("tiny", "mid", "mini_sage", "mini_gcn_directed")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default=None,
                    help="one workload only (default: large as the headline, with mid nested under "
                         "other_workloads)")
    ap.add_argument("--also", default=None, help="comma-separated workloads to nest under other_workloads")
    ap.add_argument("--cpu-sample-n", type=int, default=0, help="vertices of the scaled oracle sample (0 = auto)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--partitioner", choices=["random", "lp", "switching", "switching_device"], default=None,
                    help="override the workload's partitioner")
    ap.add_argument("--graph-scale", type=float, default=1.0,
                    help="shrink the workload's graph (vertices and drawn edges) by this factor; "
                         "for runs that would not fit the host otherwise")
    ap.add_argument("--recompute", action="store_true",
                    help="recompute in the backward pass what the forward pass computed (the paper's rule: the "
                         "aggregate of aggregate-first layers; H, scores and attention weights of attention "
                         "layers) instead of keeping it in device memory when it fits")
    ap.add_argument("--gat-heads", default=None,
                    help="graph-attention workloads: attention heads per layer, comma-separated (e.g. 8,8,1)")
    ap.add_argument("--train", action="store_true",
                    help="time training steps instead of bare epochs: epoch with dropout 0.5 after "
                         "the hidden layers, then one Adam step (lr 0.01), as in the paper's runs")
    ap.add_argument("--layer-order", choices=["auto", "aggregate"], default="auto",
                    help="auto: layers that narrow transform first (same results up to rounding, "
                         "fewer bytes); aggregate: every layer aggregates first, as in the paper")
    ap.add_argument("--staged-gather", action="store_true",
                    help="keep the gather a step of its own (staging buffer) instead of fusing it into the "
                         "aggregation kernels")
    ap.add_argument("--full-backward", action="store_true",
                    help="output layer's transposed aggregation over every operator entry instead of those of "
                         "train vertices only")
    ap.add_argument("--no-paper-order", action="store_true",
                    help="skip the extra epochs that time the paper's layer order (ms_per_step_paper_order)")
    ap.add_argument("--hbm-budget-gb", type=float, default=0.0,
                    help="> 0: run the streaming schedule (activations and gradients in pinned host "
                         "memory) with this much HBM for the partition-block caches")
    ap.add_argument("--storage-dir", default=None,
                    help="streaming schedule with the storage tier: per-layer arrays in files of this directory")
    ap.add_argument("--storage-drop-results", action="store_true",
                    help="storage tier: arrays the epoch is done with are dropped instead of written back "
                         "(a training loop reads only the weight gradients)")
    ap.add_argument("--host-budget-gb", type=float, default=0.0,
                    help="size of the storage tier's pinned host pool in GiB")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy (a dispatch of known "
                         "size, used to scale hardware byte counters)")
    ap.add_argument("--no-profile", action="store_true",
                    help="leave the per-kernel HIP events out of the timed region")
    args = ap.parse_args()
    if args.gat_heads:
        global GAT_HEADS
        GAT_HEADS = [int(h) for h in args.gat_heads.split(",")]
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no sharding or collectives are "
                 "built); run with --gpus 1")

    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")

    primary = args.workload or "large"
    others = [x for x in (args.also.split(",") if args.also else ([] if args.workload else ["mid", "dense"])) if x]
    if primary == "large" and torch.cuda.get_device_properties(0).total_memory < 250 * 2 ** 30:
        sys.exit("bench.py: the large workload needs 250 GB of device memory")
    out = run_workload(primary, args, args.steps, args.warmup, not args.no_cpu_baseline)
    nested = {}
    for name in others:
        nested[name] = run_workload(name, args, args.steps, args.warmup, not args.no_cpu_baseline)
    if nested:
        out["other_workloads"] = nested
    out["paper_context"] = ("paper reports whole-system epochs only (SSD+PCIe bound): 7.2 s for a "
                            "3-layer GCN on ogbn-products (2.45M nodes / 61.9M edges) and 9.07 min on "
                            "ogbn-papers100M (111M nodes / 1.6B edges), one RTX A5000 workstation")
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
