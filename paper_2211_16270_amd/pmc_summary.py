"""Turns rocprofv3 output into the short text summaries kept under profiles/.

  python -m paper_2211_16270_amd.pmc_summary stats  <dir with *_kernel_stats.csv>  "<command>"
  python -m paper_2211_16270_amd.pmc_summary traffic <FETCH_SIZE dir> <WRITE_SIZE dir> <copy_bytes> "<commands>"

`traffic` expects two counter runs of `bench.py --calibrate-copy`: the plain copy kernel of known
size in them gives the factor between what FETCH_SIZE / WRITE_SIZE report (KiB) and real bytes.
"""
from __future__ import annotations

import collections
import csv
import glob
import os
import sys

KERNEL_ALIASES = [
    ("k_joint_bwd_fused", "joint_bwd_fused"), ("k_joint_scores<0", "joint_scores_fwd"),
    ("k_joint_scores<1", "joint_scores_bwd"), ("k_gemm_dw256", "gemm_dw_db"), ("k_dw_reduce", "dw_reduce"), ("k_gemm_dz256", "gemm_dz"),
    ("k_joint_scores<2", "joint_scores_fwd_keep"), ("k_kept_to_dh", "kept_scores_to_dh"),
    ("k_lattice", "lattice"), ("k_copy_f32", "copy_f32"), ("k_prepare", "prepare"),
    ("k_fwd_f32", "fwd_f32"), ("k_bwd_f32", "bwd_f32"),
    ("k_rows_z_f32", "rows_z_f32"),
    ("k_rows_stats_f32", "rows_stats_f32"), ("k_rows_dh_f32", "rows_dh_f32"), ("k_rows_dz_f32", "rows_dz_f32"),
    ("k_col_sum", "col_sum"),
]


def alias(name: str):
    if "k_gemm_f32<" in name:
        # operand classes OperandF32<k-slow?> / OperandF32Edge<k-slow?> of A and B
        slow = [name[i + 1:].startswith("true") for i in range(len(name)) if name[i] == "<" and name[:i].endswith(("OperandF32", "OperandF32Edge"))]
        kind = {(False, True): "scores = Z W", (True, True): "dW = Z^T dh", (False, False): "dZ = dh W^T"}.get(tuple(slow[:2]), "")
        return "gemm_f32 " + ("(edges) " if "OperandF32Edge" in name else "") + kind
    for key, short in KERNEL_ALIASES:
        if key in name:
            return short
    return None


def _one(pattern: str) -> str:
    hits = glob.glob(pattern, recursive=True)
    if not hits:
        raise SystemExit(f"no file matches {pattern}")
    return hits[0]


def stats(directory: str, command: str) -> str:
    path = _one(os.path.join(directory, "**", "*kernel_stats.csv"))
    rows = list(csv.DictReader(open(path)))
    out = [f"# rocprofv3 --kernel-trace --stats summary", f"# command: {command}",
           "# kernel, calls, total_ms, average_us, percent"]
    for r in rows:
        short = alias(r["Name"]) or r["Name"][:60]
        if float(r["Percentage"]) < 0.01:
            continue
        out.append(f"{short}, {r['Calls']}, {float(r['TotalDurationNs']) / 1e6:.3f}, "
                   f"{float(r['AverageNs']) / 1e3:.2f}, {float(r['Percentage']):.2f}")
    return "\n".join(out) + "\n"


def _counter(directory: str, counter: str):
    path = _one(os.path.join(directory, "**", "*counter_collection.csv"))
    agg = collections.defaultdict(lambda: [0, 0.0])
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] != counter:
            continue
        short = alias(r["Kernel_Name"])
        if short is None:
            continue
        agg[short][0] += 1
        agg[short][1] += float(r["Counter_Value"])
    return agg


def traffic(fetch_dir: str, write_dir: str, copy_bytes: int, command: str) -> str:
    f, w = _counter(fetch_dir, "FETCH_SIZE"), _counter(write_dir, "WRITE_SIZE")
    if "copy_f32" not in f or "copy_f32" not in w:
        raise SystemExit("the runs hold no copy_f32 launches: use bench.py --calibrate-copy")
    fr = copy_bytes / (f["copy_f32"][1] / f["copy_f32"][0] * 1024.0)
    fw = copy_bytes / (w["copy_f32"][1] / w["copy_f32"][0] * 1024.0)
    out = ["# HBM traffic per launch from rocprofv3 --pmc FETCH_SIZE and --pmc WRITE_SIZE (two runs)",
           f"# commands: {command}",
           f"# calibration: copy_f32 moves {copy_bytes} B each way per launch; FETCH_SIZE reports "
           f"{f['copy_f32'][1] / f['copy_f32'][0]:.1f} KiB (factor {fr:.4f}), WRITE_SIZE reports "
           f"{w['copy_f32'][1] / w['copy_f32'][0]:.1f} KiB (factor {fw:.4f})",
           "# kernel launches fetch_KiB_per_launch write_KiB_per_launch fetch_bytes write_bytes hbm_bytes_per_launch"]
    for k in sorted(set(f) | set(w)):
        if k == "copy_f32":
            continue
        n = max(f.get(k, [0, 0])[0], w.get(k, [0, 0])[0])
        fk = f[k][1] / f[k][0] if k in f and f[k][0] else 0.0
        wk = w[k][1] / w[k][0] if k in w and w[k][0] else 0.0
        fb, wb = fk * 1024.0 * fr, wk * 1024.0 * fw
        out.append(f"{k} {n} {fk:.1f} {wk:.1f} {fb:.0f} {wb:.0f} {fb + wb:.0f}")
    return "\n".join(out) + "\n"


def read_traffic(path: str) -> dict:
    """{kernel: hbm bytes per launch} from a file written by `traffic`."""
    res = {}
    if not os.path.exists(path):
        return res
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        parts = line.split()
        res[parts[0]] = float(parts[-1])
    return res


if __name__ == "__main__":
    if len(sys.argv) >= 4 and sys.argv[1] == "stats":
        sys.stdout.write(stats(sys.argv[2], sys.argv[3]))
    elif len(sys.argv) >= 6 and sys.argv[1] == "traffic":
        sys.stdout.write(traffic(sys.argv[2], sys.argv[3], int(sys.argv[4]), sys.argv[5]))
    else:
        raise SystemExit(__doc__)
