"""Host logic of bench.py's byte model (no GPU): the algorithmic bytes per kernel class that the
roofline fraction is priced against must follow the schedule that was timed."""
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))

import bench  # noqa: E402

STATS = dict(n=1000, nnz=20000, k=4, sum_boundary=1500)


def test_kept_forward_results_drop_one_gather_and_one_aggregation_pass_per_aggregate_first_layer():
    dims = (64, 32, 32, 16)
    for model in ("gcn", "sage"):
        for xf in ([False, False, False], [False, True, True], [True, True, True]):
            a = bench.algorithmic_bytes(STATS, dims, model, 4, xf=xf)
            b = bench.algorithmic_bytes(STATS, dims, model, 4, xf=xf, kept=True)
            # what one aggregate-first layer moves per pass, by the same formulas
            n, nnz, k, sum_b = STATS["n"], STATS["nnz"], STATS["k"], STATS["sum_boundary"]
            per_entry = 4 + (4 if model == "gcn" else 0)
            gather = spmm = 0
            for l in range(1, 4):
                if not xf[l - 1]:
                    row = dims[l - 1] * 4
                    gather += 2 * sum_b * row + 4 * sum_b
                    spmm += per_entry * nnz + 8 * (n + k) + (n + sum_b) * row + n * row + (4 * n if model == "sage" else 0)
            assert a["gather"] - b["gather"] == gather, (model, xf)
            assert a["spmm"] - b["spmm"] == spmm, (model, xf)
            assert a["spmm_t"] == b["spmm_t"] and a["scatter"] == b["scatter"]
            if all(xf):
                assert a == b


def test_transform_first_layers_move_rows_of_the_output_width_once_each_way():
    wide_in = bench.algorithmic_bytes(STATS, (512, 16), "gcn", 4, xf=[False])
    narrow = bench.algorithmic_bytes(STATS, (512, 16), "gcn", 4, xf=[True])
    assert narrow["spmm"] < wide_in["spmm"] / 8 and narrow["gather"] < wide_in["gather"] / 8
    # the operator over train vertices and first-touch stores only ever lower the transposed pass
    full = bench.algorithmic_bytes(STATS, (64, 32, 16), "gcn", 4, xf=[False, True], fused_scatter=True)
    masked = bench.algorithmic_bytes(STATS, (64, 32, 16), "gcn", 4, xf=[False, True], fused_scatter=True,
                                     masked=(2000, 300, 100))
    first = bench.algorithmic_bytes(STATS, (64, 32, 16), "gcn", 4, xf=[False, True], fused_scatter=True,
                                    first_touch=True)
    assert masked["spmm_t"] < full["spmm_t"] and first["spmm_t"] < full["spmm_t"]
    assert masked["spmm"] == full["spmm"] == first["spmm"]


def test_more_than_one_gpu_is_refused():
    import subprocess
    r = subprocess.run([sys.executable, os.path.join(os.path.dirname(bench.__file__), "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in (r.stderr + r.stdout)
