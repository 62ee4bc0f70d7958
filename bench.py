#!/usr/bin/env python3
"""One-GPU benchmark of the partition-wise full-graph GNN epoch (forward + loss + backward).

A "step" is one gnn_epoch over the whole synthetic graph: for every layer and partition
gather -> aggregate -> transform, the loss, then for every layer and partition regather ->
recompute -> dW / dZ -> transposed aggregate -> scatter-add.  Inputs are resident in HBM
before the timed region.  Prints ONE JSON line (see the keys below).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload mid|tiny|...]
"""
from __future__ import annotations

import argparse
import json
import os
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


def algorithmic_bytes(stats, dims, model, n_parts, es=4, fused_scatter=False, xf=None):
    """HBM bytes the method has to move per epoch, by kernel class (lower bound: every needed
    source row is read once per partition).  es = bytes per stored activation (4 fp32, 2 bf16);
    gradients of activations are always fp32.  xf[l-1]: layer l transforms first, so it
    gathers, aggregates and scatter-accumulates rows of its (padded) output width, once
    forward and once backward, with no regather and no recompute."""
    n, nnz, k = stats["n"], stats["nnz"], stats["k"]
    sum_r = n + stats["sum_boundary"]            # sum over partitions of |own_p| + |B_p|
    sum_b = stats["sum_boundary"]
    L = len(dims) - 1
    per_entry = 4 + (4 if model in ("gcn", "gat") else 0)  # column index (+ entry weight: GCN, GAT)
    out = {"gather": 0, "spmm": 0, "spmm_t": 0, "scatter": 0}
    xf = xf or [False] * L
    for l in range(1, L + 1):
        if xf[l - 1]:
            wp = (dims[l] + 3) // 4 * 4
            row = wp * 4                         # aggregated sums and gradients of H: fp32
            hrow = wp * es                       # rows of H (and of dY) in the storage type
            one_gather = 2 * sum_b * hrow + 4 * sum_b
            one_spmm = per_entry * nnz + 8 * (n + k) + sum_r * hrow + n * row + (4 * n if model == "sage" else 0)
            # graph attention regathers, and reads every needed row once more for the edge-wise
            # products dY[v] . H[u] (same traffic as an aggregation, 4 bytes written per entry)
            out["gather"] += one_gather * (2 if model == "gat" else 1)
            out["spmm"] += one_spmm * (2 if model == "gat" else 1)
            out["spmm_t"] += 8 * nnz + 8 * (sum_r + k) + n * hrow + 2 * sum_r * row + 4 * sum_b
            continue
        d = dims[l - 1]
        row = d * es
        grow = d * 4
        # forward + backward regather
        out["gather"] += 2 * (2 * sum_b * row + 4 * sum_b)
        # forward + recompute
        spmm = per_entry * nnz + 8 * (n + k) + sum_r * row + n * row + (4 * n if model == "sage" else 0)
        out["spmm"] += 2 * spmm
        if l >= 2:
            if fused_scatter:
                # transposed aggregation adds its rows straight onto their owners: read dZ once,
                # read-modify-write every required row of grad A^{l-1}
                out["spmm_t"] += 8 * nnz + 8 * (sum_r + k) + n * row + 2 * sum_r * grow + 4 * sum_b
            else:
                out["spmm_t"] += 8 * nnz + 8 * (sum_r + k) + n * row + sum_r * grow
                out["scatter"] += 3 * sum_r * grow + 4 * sum_b
    return out


def gemm_flops(stats, dims, model):
    n = stats["n"]
    L = len(dims) - 1
    mult = 2 if model == "sage" else 1
    fwd = sum(2 * n * dims[l] * dims[l + 1] * mult for l in range(L))
    dw = fwd
    dz = sum(2 * n * dims[l] * dims[l + 1] * mult for l in range(1, L))
    return {"gemm_fwd": fwd, "gemm_dw": dw, "gemm_dz": dz}


def _oracle_epoch_seconds(cfg, n):
    from oracle import fullgraph as og
    from synth import features, glorot_weights, labels_and_mask, rmat_graph
    m_draw = int(cfg["m_draw"] * (n / cfg["n"]))
    rowptr, colidx = rmat_graph(n, m_draw, cfg["seed"] + 1000, symmetric=cfg["symmetric"],
                                self_loops=cfg["self_loops"])
    dims = cfg["dims"]
    X = features(n, dims[0], cfg["seed"])
    y, m = labels_and_mask(n, dims[-1], cfg["train_frac"], cfg["seed"])
    w = glorot_weights(dims, cfg["seed"], sage=(cfg["model"] == "sage"))
    t0 = time.perf_counter()
    if cfg["model"] == "gat":
        from oracle import gat as ogat
        from synth import attention_vectors
        ogat.epoch(rowptr, colidx, dims, X, attention_vectors(w, cfg["seed"]), y, m)
    else:
        og.epoch(cfg["model"], rowptr, colidx, dims, X, w, y, m)
    dt = time.perf_counter() - t0
    nnz = int(rowptr[-1]) + (n if cfg["model"] in ("gcn", "gat") and not cfg["self_loops"] else 0)
    return dt, nnz


def cpu_baseline(cfg, scale_n, log_fn):
    """The oracle, as it stands, timed on the host cores on a down-scaled instance of the same
    workload (same generator, degree and widths; fewer vertices).  With scale_n == 0 a short
    probe run picks the sample size that gives roughly 15 s of CPU work on this machine."""
    from oracle import fullgraph as og
    if scale_n <= 0:
        probe_n = max(2000, min(cfg["n"], 2000 if cfg["model"] == "gat" else 20000))
        dt, _ = _oracle_epoch_seconds(cfg, probe_n)
        scale_n = int(max(probe_n, min(cfg["n"], 1_000_000, probe_n * 15.0 / max(dt, 1e-3))))
        log_fn("cpu oracle probe: n=%d took %.2f s -> sample n=%d" % (probe_n, dt, scale_n))
    dt, nnz = _oracle_epoch_seconds(cfg, scale_n)
    log_fn("cpu oracle: n=%d nnz=%d epoch %.2f s on %d threads" % (scale_n, nnz, dt, og.num_threads()))
    return {"value": nnz / dt, "unit": "edges/s", "cores": og.num_threads(), "kind": "oracle",
            "sample": "same R-MAT recipe and layer widths at n=%d (%d operator entries), one fp64 "
                      "full-graph epoch (fwd+loss+bwd) in %.2f s" % (scale_n, nnz, dt),
            "epoch_s": dt}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="mid")
    ap.add_argument("--cpu-sample-n", type=int, default=0, help="vertices of the oracle sample (0 = auto)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--partitioner", choices=["random", "lp", "switching", "switching_device"], default=None,
                    help="override the workload's partitioner")
    ap.add_argument("--graph-scale", type=float, default=1.0,
                    help="shrink the workload's graph (vertices and drawn edges) by this factor; "
                         "for runs that would not fit the host otherwise")
    ap.add_argument("--train", action="store_true",
                    help="time training steps instead of bare epochs: epoch with dropout 0.5 after "
                         "the hidden layers, then one Adam step (lr 0.01), as in the paper's runs")
    ap.add_argument("--layer-order", choices=["auto", "aggregate"], default="auto",
                    help="auto: layers that narrow transform first (same results up to rounding, "
                         "fewer bytes); aggregate: every layer aggregates first, as in the paper")
    ap.add_argument("--hbm-budget-gb", type=float, default=0.0,
                    help="> 0: run the streaming schedule (activations and gradients in pinned host "
                         "memory) with this much HBM for the partition-block caches")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy (a dispatch of known "
                         "size, used to scale hardware byte counters)")
    ap.add_argument("--no-profile", action="store_true",
                    help="leave the per-kernel HIP events out of the timed region")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no sharding or collectives are "
                 "built); run with --gpus 1")

    import numpy as np
    import torch
    from paper_2605_11517_amd import Session
    from synth import CONFIGS, attention_vectors, features, glorot_weights, labels_and_mask, make_config

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")

    t0 = time.perf_counter()
    over = {}
    if args.graph_scale != 1.0:
        base = CONFIGS[args.workload]
        over = {"n": int(base["n"] * args.graph_scale), "m_draw": int(base["m_draw"] * args.graph_scale)}
    cfg, rowptr, colidx = make_config(args.workload, **over)
    n, dims, model = cfg["n"], cfg["dims"], cfg["model"]
    log("graph %s: n=%d entries=%d (%.1f s)" % (args.workload, n, rowptr[-1], time.perf_counter() - t0))
    X = features(n, dims[0], cfg["seed"])
    y, m = labels_and_mask(n, dims[-1], cfg["train_frac"], cfg["seed"])
    w = glorot_weights(dims, cfg["seed"], sage=(model == "sage"))
    if model == "gat":
        attention_vectors(w, cfg["seed"])
    t1 = time.perf_counter()
    if args.partitioner:
        cfg["part"] = args.partitioner
    s = Session(model, dims, rowptr, colidx, cfg["k"], cfg["part"], cfg["seed"], X, w, y, m,
                dtype=cfg["dtype"], hbm_budget_bytes=int(args.hbm_budget_gb * 2 ** 30),
                layer_order=args.layer_order, progress=lambda msg: log("  " + msg))
    xf = [s.ctx.layer_is_transform_first(l) for l in range(1, len(dims))]
    # gnn_epoch runs a transform-first layer's contractions beside the aggregate-first layer below it
    overlapped = (cfg["dtype"] != "bf16" and model != "gat" and not args.hbm_budget_gb and
                  any((not a) and b for a, b in zip(xf, xf[1:])) and
                  os.environ.get("GNNMI_OVERLAP", "1")[:1] != "0")
    es = 2 if cfg["dtype"] == "bf16" else 4
    mfma_peak = MFMA_BF16_PEAK_TFLOPS if cfg["dtype"] == "bf16" else MFMA_F32_PEAK_TFLOPS
    stats = s.ctx.get_stats()
    setup_s = time.perf_counter() - t1        # partitioner, metadata, upload, binding
    log("partitions built and bound: k=%d alpha=%.3f sum_boundary=%d (%.1f s)" % (
        stats["k"], stats["sum_required"] / n, stats["sum_boundary"], time.perf_counter() - t1))
    del X, rowptr, colidx

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

    for i in range(args.warmup):
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
    for i in range(args.steps):
        loss = step(args.warmup + i)
        if not args.no_profile:
            for name, (ms, launches) in s.ctx.get_profile().items():
                a = prof.setdefault(name, [0.0, 0])
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
        step(args.warmup + args.steps)
        torch.cuda.synchronize()
        breakdown = {name: (ms, launches) for name, (ms, launches) in s.ctx.get_profile().items()}
        if previous is None:
            del os.environ["GNNMI_OVERLAP"]
        else:
            os.environ["GNNMI_OVERLAP"] = previous
    s.ctx.set_profiling(0)
    ms_per_step = dt / args.steps * 1e3
    nnz = stats["nnz"]
    log("epoch %.2f ms, loss %.5f" % (ms_per_step, loss))

    out = {
        "metric": ("full-graph training-step throughput (fwd with dropout+loss+bwd+Adam step), operator "
                   "entries per second" if args.train else
                   "full-graph epoch throughput (fwd+loss+bwd), operator entries per second"),
        "value": nnz / (dt / args.steps),
        "unit": "edges/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg["dtype"], "data": "synthetic",
        "config": {"workload": args.workload + ("" if args.graph_scale == 1.0 else " x%g" % args.graph_scale) +
                   ("" if not args.hbm_budget_gb else
                                                 " (streaming, %.3g GiB block cache)" % args.hbm_budget_gb),
                   "n": n, "operator_entries": nnz, "model": model,
                   "dims": list(dims), "k": stats["k"], "partitioner": cfg["part"],
                   "alpha": stats["sum_required"] / n, "sum_boundary": stats["sum_boundary"],
                   "layer_order": ["transform-first" if t else "aggregate-first" for t in xf],
                   "side_stream_overlap": overlapped,
                   "setup_s": setup_s},
        "loss": loss,
    }
    if prof:
        ab = algorithmic_bytes(stats, dims, model, stats["k"], es,
                               fused_scatter=prof.get("scatter", (0, 0))[1] == 0, xf=xf)
        fl = gemm_flops(stats, dims, model)
        # per kernel class, from the one epoch run after the timed region with every class bracketed,
        # on one stream
        classes = {}
        for name, (ms, launches) in breakdown.items():
            e = {"ms_per_epoch": ms, "launches_per_epoch": launches}
            if name in ab and ms > 0:
                e["algorithmic_GBps"] = ab[name] / (ms * 1e-3) / 1e9
                e["frac_hbm_peak"] = e["algorithmic_GBps"] / HBM_PEAK_GBS
            if name in fl and ms > 0:
                e["TFLOPps"] = fl[name] / (ms * 1e-3) / 1e12
                e["frac_mfma_peak"] = e["TFLOPps"] / mfma_peak
            classes[name] = e
        out["kernel_classes"] = classes
        sp_ms, sp_launches = prof["spmm"]
        passes = sum(1 if t else 2 for t in xf)       # forward (+ recompute) aggregations
        if model == "gat":
            passes = 2 * len(xf)                        # aggregation + edge-wise products
        tp_ms = prof["spmm_t"][0]
        transposed = (len(dims) - 2) + (1 if xf[0] else 0)   # a transform-first layer 1 still pushes grad H
        out["aggregated_edges_per_s"] = nnz * (passes + transposed) * args.steps / ((sp_ms + tp_ms) * 1e-3)
        # dominant kernel: k_spmm_items, every launch of it (forward, recompute and transposed)
        k_ms = sp_ms + tp_ms
        k_launches = sp_launches + prof["spmm_t"][1]
        k_bytes = (ab["spmm"] + ab["spmm_t"]) * args.steps
        achieved = k_bytes / (k_ms * 1e-3) / 1e9
        # measured HBM-side traffic of the same kernel from the committed counter summary
        # (rocprofv3 FETCH_SIZE + WRITE_SIZE, scaled by a plain copy), per launch
        traffic = None
        from paper_2605_11517_amd.profiling import read_traffic
        table = read_traffic(os.path.join(ROOT, "profiles", "pmc_%s_epoch.md" % args.workload))
        if table:
            rows = [v for k, v in table.items() if k.startswith(("k_spmm_items", "k_spmm_slots"))]
            if rows:
                tot_l = sum(r["launches"] for r in rows)
                traffic = sum(r["bytes_per_launch"] * r["launches"] for r in rows) / tot_l
        L = len(dims) - 1
        upper = 0
        for l in range(L):
            if xf[l]:
                roww = (dims[l + 1] + 3) // 4 * 4 * 4
                upper += (3 if model == "gat" else 2) * (stats["nnz"] * (4 + roww) + n * roww)
            else:
                upper += (2 if l == 0 else 3) * (stats["nnz"] * (4 + dims[l] * es) + n * dims[l] * es)
        out["roofline"] = {
            "kernel": "k_spmm_slots / k_spmm_items (aggregation over T_p and T_p^T: forward, recompute, "
                      "transposed; column-sliced variant where rows are whole 128-byte lines)",
            "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
            "bytes_per_launch": k_bytes / k_launches,
            "avg_launch_ms": k_ms / k_launches, "launches_per_epoch": k_launches / args.steps,
            "no_reuse_bytes_per_launch": upper * args.steps / k_launches,
            "traffic_GBps": None if traffic is None else traffic / (k_ms / k_launches * 1e-3) / 1e9,
            "note": "achieved = bytes the method must move if every needed source row is read "
                    "once per partition, over the HIP-event time of the kernel in the timed region" +
                    (" (where contractions of the next layer run beside part of its launches on a side "
                     "stream and stretch them; kernel_classes come from a one-stream epoch)"
                     if overlapped else "") + "; traffic = measured "
                    "fetch+write bytes per launch (rocprofv3 counters); no_reuse = one source row "
                    "read per operator entry",
        }
        out["profiled_ms_per_step"] = sum(v[0] for v in breakdown.values())
    if args.hbm_budget_gb:
        st = s.ctx.get_stream_stats()              # of the last epoch
        st["pcie_GBps"] = (st["h2d_bytes"] + st["d2h_bytes"]) / (ms_per_step * 1e-3) / 1e9
        out["streaming"] = st
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, args.cpu_sample_n, log)
    out["paper_context"] = ("paper reports whole-system epochs only (SSD+PCIe bound): 7.2 s for a "
                            "3-layer GCN on ogbn-products (2.45M nodes / 61.9M edges) on one RTX A5000")
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
