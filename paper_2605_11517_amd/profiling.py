"""Turn rocprofv3 CSV output into the short text summaries kept under ``profiles/``.

    python -m paper_2605_11517_amd.profiling stats  <dir-with-*_kernel_stats.csv>  <out.md> "<command>"
    python -m paper_2605_11517_amd.profiling pmc    <fetch-dir> <write-dir> <out.md> "<command>"

    python -m paper_2605_11517_amd.profiling mfma   <pmc-dir> <out.md> "<command>"
    python -m paper_2605_11517_amd.profiling counters <pmc-dir> <out.md> "<command>"

``counters`` takes any ``--pmc ... --kernel-trace`` run and lists, per kernel, the number of
dispatches and the sum of every collected counter over them.

``mfma`` expects one counter run with ``--pmc SQ_BUSY_CU_CYCLES SQ_VALU_MFMA_BUSY_CYCLES
--kernel-trace`` and reports, per contraction kernel, the clock the compute units ran at
(busy cycles of the 256 CUs over the kernel's duration) and the share of those cycles in which
a SIMD's matrix pipe was busy (four SIMDs per CU).

An optional last argument of every mode is the commit the run was taken at; it is written into
the summary ("Taken at commit ...").

``pmc`` expects two counter runs of the same command (``--pmc FETCH_SIZE`` and
``--pmc WRITE_SIZE``, each with ``--kernel-trace``) that include one plain 1 GiB device copy
(``bench.py --copy-calibration``).  The counters are reported in KiB per dispatch; each is
scaled by (1 GiB / what the same counter shows for that copy) before use.
"""
from __future__ import annotations

import collections
import csv
import glob
import json
import os
import re
import sys

GIB = float(1 << 30)


def short_name(name: str) -> str:
    name = re.sub(r"\(anonymous namespace\)::", "", name)
    name = re.sub(r"gnnmi::", "", name)
    name = re.sub(r"^void ", "", name)
    return name.split("(")[0]


def _one(pattern):
    """The first file matching `pattern`, also in sub-directories of its directory (rocprofv3
    may put its files under a directory named after the host)."""
    hits = sorted(glob.glob(pattern))
    if not hits:
        d, base = os.path.split(pattern)
        hits = sorted(glob.glob(os.path.join(d, "**", base), recursive=True))
    if not hits:
        raise FileNotFoundError(pattern)
    return hits[0]


def summarize_stats(src_dir: str, out_path: str, command: str, commit: str = "") -> None:
    rows = list(csv.DictReader(open(_one(os.path.join(src_dir, "*kernel_stats.csv")))))
    total = sum(float(r["TotalDurationNs"]) for r in rows)
    lines = ["# rocprofv3 --kernel-trace --stats", "", "Command:", "", "    " + command, ""]
    if commit:
        lines += ["Taken at commit %s." % commit, ""]
    lines += ["| kernel | calls | total ms | avg us | % |", "|---|---:|---:|---:|---:|"]
    for r in rows:
        t = float(r["TotalDurationNs"])
        if t / total < 0.001:
            continue
        lines.append("| %s | %s | %.3f | %.1f | %.2f |" % (
            short_name(r["Name"]), r["Calls"], t / 1e6, float(r["AverageNs"]) / 1e3, 100 * t / total))
    lines.append("")
    lines.append("Total kernel time %.3f ms." % (total / 1e6))
    open(out_path, "w").write("\n".join(lines) + "\n")


def _per_kernel(path, counter):
    out = collections.OrderedDict()
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] != counter:
            continue
        e = out.setdefault(short_name(r["Kernel_Name"]), {"kib": 0.0, "launches": 0, "ns": 0, "max_kib": 0.0})
        e["kib"] += float(r["Counter_Value"])
        e["max_kib"] = max(e["max_kib"], float(r["Counter_Value"]))
        e["launches"] += 1
        e["ns"] += int(r["End_Timestamp"]) - int(r["Start_Timestamp"])
    return out


def summarize_pmc(fetch_dir: str, write_dir: str, out_path: str, command: str, commit: str = "") -> None:
    fetch = _per_kernel(_one(os.path.join(fetch_dir, "*counter_collection.csv")), "FETCH_SIZE")
    write = _per_kernel(_one(os.path.join(write_dir, "*counter_collection.csv")), "WRITE_SIZE")

    def copy_scale(table):
        # the calibration copy is the largest dispatch of the runtime's copy kernel
        best = 0.0
        for name, e in table.items():
            if "copyBuffer" in name or "copy" in name.lower():
                best = max(best, e["max_kib"])
        return (GIB / 1024.0) / best if best > 0 else 1.0

    fs, ws = copy_scale(fetch), copy_scale(write)
    lines = ["# rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (two runs)", "", "Command (run once per counter):",
             "", "    " + command, ""] + (["Taken at commit %s." % commit, ""] if commit else []) + [
             "Scale factors from the 1 GiB calibration copy: FETCH_SIZE x %.3f, WRITE_SIZE x %.3f "
             "(counter KiB -> real KiB)." % (fs, ws), "",
             "| kernel | launches | read GB | written GB | GB per launch | ms per launch | GB/s |",
             "|---|---:|---:|---:|---:|---:|---:|"]
    table = {}
    for name, e in fetch.items():
        rd = e["kib"] * fs * 1024 / 1e9
        w = write.get(name, {"kib": 0.0})
        wr = w["kib"] * ws * 1024 / 1e9
        ms = e["ns"] / 1e6
        if rd + wr < 0.05:
            continue
        table[name] = {"launches": e["launches"], "read_GB": rd, "written_GB": wr,
                       "bytes_per_launch": (rd + wr) * 1e9 / e["launches"],
                       "ms_per_launch": ms / e["launches"]}
        lines.append("| %s | %d | %.2f | %.2f | %.4f | %.4f | %.0f |" % (
            name, e["launches"], rd, wr, (rd + wr) / e["launches"], ms / e["launches"],
            (rd + wr) / (ms / 1e3) if ms > 0 else 0.0))
    lines += ["", "TRAFFIC_JSON: " + json.dumps(table)]
    open(out_path, "w").write("\n".join(lines) + "\n")


def summarize_mfma(src_dir: str, out_path: str, command: str, commit: str = "") -> None:
    path = _one(os.path.join(src_dir, "*counter_collection.csv"))
    per = collections.OrderedDict()
    seen = set()
    for r in csv.DictReader(open(path)):
        name = short_name(r["Kernel_Name"])
        e = per.setdefault(name, {"busy": 0.0, "mfma": 0.0, "launches": 0, "ns": 0})
        if r["Counter_Name"] == "SQ_BUSY_CU_CYCLES":
            e["busy"] += float(r["Counter_Value"])
        elif r["Counter_Name"] == "SQ_VALU_MFMA_BUSY_CYCLES":
            e["mfma"] += float(r["Counter_Value"])
        key = (r["Dispatch_Id"], name)
        if key not in seen:
            seen.add(key)
            e["launches"] += 1
            e["ns"] += int(r["End_Timestamp"]) - int(r["Start_Timestamp"])
    lines = ["# rocprofv3 --pmc SQ_BUSY_CU_CYCLES SQ_VALU_MFMA_BUSY_CYCLES (matrix-pipe utilisation)", "",
             "Command:", "", "    " + command, ""]
    if commit:
        lines += ["Taken at commit %s." % commit, ""]
    lines += ["clock = SQ_BUSY_CU_CYCLES / (256 CUs x duration); pipe busy = SQ_VALU_MFMA_BUSY_CYCLES / "
              "(4 SIMDs x SQ_BUSY_CU_CYCLES); vs 2.4 GHz = SQ_VALU_MFMA_BUSY_CYCLES / (1024 SIMDs x duration x 2.4 GHz), "
              "the share of the published peak's issue slots that held a matrix instruction.", "",
             "| kernel | launches | avg us | clock GHz | MFMA pipe busy | vs 2.4 GHz |", "|---|---:|---:|---:|---:|---:|"]
    for name, e in per.items():
        if e["mfma"] <= 0 or e["ns"] <= 0 or e["busy"] <= 0:
            continue
        dur = e["ns"] * 1e-9
        lines.append("| %s | %d | %.1f | %.2f | %.3f | %.3f |" % (
            name, e["launches"], e["ns"] / e["launches"] / 1e3, e["busy"] / 256.0 / dur / 1e9,
            e["mfma"] / (4.0 * e["busy"]), e["mfma"] / (1024.0 * dur * 2.4e9)))
    open(out_path, "w").write("\n".join(lines) + "\n")


def summarize_counters(src_dir: str, out_path: str, command: str, commit: str = "") -> None:
    path = _one(os.path.join(src_dir, "*counter_collection.csv"))
    per = collections.OrderedDict()
    names = []
    for r in csv.DictReader(open(path)):
        e = per.setdefault(short_name(r["Kernel_Name"]), collections.OrderedDict())
        cn = r["Counter_Name"]
        if cn not in names:
            names.append(cn)
        tot, cnt = e.get(cn, (0.0, 0))
        e[cn] = (tot + float(r["Counter_Value"]), cnt + 1)
    lines = ["# rocprofv3 --pmc " + " ".join(names), "", "Command:", "", "    " + command, ""]
    if commit:
        lines += ["Taken at commit %s." % commit, ""]
    lines += ["Sums over all dispatches of a kernel.", "",
              "| kernel | dispatches | " + " | ".join(names) + " |", "|---|---:|" + "---:|" * len(names)]
    for k, e in per.items():
        n = max(c for _, c in e.values())
        lines.append("| %s | %d | " % (k, n) + " | ".join("%.4g" % e.get(cn, (0.0, 0))[0] for cn in names) + " |")
    open(out_path, "w").write("\n".join(lines) + "\n")


def read_taken_at(path: str):
    """The commit a summary says it was taken at (a line 'Taken at commit <hash>'), or None."""
    try:
        for line in open(path):
            m = re.match(r"Taken at commit (\w+)", line.strip())
            if m:
                return m.group(1)
    except OSError:
        pass
    return None


def read_traffic(path: str):
    """The per-kernel table written by ``summarize_pmc`` (or None)."""
    try:
        for line in open(path):
            if line.startswith("TRAFFIC_JSON: "):
                return json.loads(line[len("TRAFFIC_JSON: "):])
    except OSError:
        pass
    return None


if __name__ == "__main__":
    if len(sys.argv) >= 5 and sys.argv[1] == "stats":
        summarize_stats(sys.argv[2], sys.argv[3], sys.argv[4], *sys.argv[5:6])
    elif len(sys.argv) >= 5 and sys.argv[1] == "mfma":
        summarize_mfma(sys.argv[2], sys.argv[3], sys.argv[4], *sys.argv[5:6])
    elif len(sys.argv) >= 5 and sys.argv[1] == "counters":
        summarize_counters(sys.argv[2], sys.argv[3], sys.argv[4], *sys.argv[5:6])
    elif len(sys.argv) >= 6 and sys.argv[1] == "pmc":
        summarize_pmc(sys.argv[2], sys.argv[3], sys.argv[4], sys.argv[5], *sys.argv[6:7])
    else:
        sys.exit(__doc__)
