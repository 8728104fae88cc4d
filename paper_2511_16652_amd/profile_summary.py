"""Turns rocprofv3 CSV output into the short text summaries kept under profiles/.

    python -m paper_2511_16652_amd.profile_summary --stats DIR --fetch DIR --write DIR \
        --workload cfg2 --command "..." --out profiles/

DIR are the -d directories of three rocprofv3 runs of the same bench.py command:
  --kernel-trace --stats            (per-kernel durations)
  --pmc FETCH_SIZE, --pmc WRITE_SIZE (HBM traffic per dispatch, KiB), both run with --calibrate-copy so
                                     that a plain copy of known size (64 MiB read, 64 MiB written) is
                                     in the same profile; its reading gives the scale of each counter.
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import os

COPY_BYTES = 64 << 20


def _one(pattern):
    files = glob.glob(pattern, recursive=True)
    if not files:
        raise FileNotFoundError(pattern)
    return files[0]


def short(name: str) -> str:
    name = name.replace("void ", "").replace("egg::", "")
    return name.split("(")[0][:96]


def kernel_stats(d):
    rows = list(csv.DictReader(open(_one(os.path.join(d, "**", "*kernel_stats.csv")))))
    return [(short(r["Name"]), int(r["Calls"]), float(r["AverageNs"]) / 1e3, float(r["MinNs"]) / 1e3,
             float(r["MaxNs"]) / 1e3, float(r["Percentage"])) for r in rows]


def counter_per_kernel(d):
    rows = list(csv.DictReader(open(_one(os.path.join(d, "**", "*counter_collection.csv")))))
    acc = collections.defaultdict(list)
    for r in rows:
        acc[short(r["Kernel_Name"])].append(float(r["Counter_Value"]))
    return acc


def copy_scale(acc):
    """bytes per counter KiB-unit, from the 64 MiB calibration copies (the largest readings of the
    runtime's copy kernel)."""
    vals = sorted(acc.get("__amd_rocclr_copyBuffer", []), reverse=True)[:3]
    if not vals:
        return None
    return COPY_BYTES / (sum(vals) / len(vals) * 1024.0)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--stats", required=True)
    ap.add_argument("--fetch")
    ap.add_argument("--write")
    ap.add_argument("--workload", required=True)
    ap.add_argument("--command", required=True)
    ap.add_argument("--out", default="profiles")
    a = ap.parse_args()
    os.makedirs(a.out, exist_ok=True)
    stats = kernel_stats(a.stats)
    fetch = counter_per_kernel(a.fetch) if a.fetch else {}
    write = counter_per_kernel(a.write) if a.write else {}
    fs, ws = (copy_scale(fetch) if fetch else None), (copy_scale(write) if write else None)
    lines = ["# rocprofv3 summary: %s" % a.workload, "",
             "command (per run, from the repo root, `cd /tmp && export TMPDIR=/tmp` first):", "",
             "    rocprofv3 --kernel-trace --stats -d <dir> -o %s --output-format csv -- %s" % (a.workload, a.command)]
    if fetch:
        lines += ["    rocprofv3 --pmc FETCH_SIZE -d <dir> -o %s --output-format csv -- %s --calibrate-copy" % (a.workload, a.command),
                  "    rocprofv3 --pmc WRITE_SIZE -d <dir> -o %s --output-format csv -- %s --calibrate-copy" % (a.workload, a.command)]
    lines += ["", "## kernel durations (--kernel-trace --stats)", "",
              "| kernel | calls | avg us | min us | max us | % of GPU time |", "|---|---|---|---|---|---|"]
    for n, c, av, mn, mx, pc in stats:
        lines.append("| %s | %d | %.1f | %.1f | %.1f | %.1f |" % (n, c, av, mn, mx, pc))
    if fetch and fs and ws:
        lines += ["", "## HBM traffic per dispatch (--pmc FETCH_SIZE / WRITE_SIZE)", "",
                  "counter scale from the 64 MiB calibration copy in the same profile: FETCH_SIZE x %.3f, WRITE_SIZE x %.3f "
                  "(bytes per reported KiB / 1024)" % (fs, ws), "",
                  "| kernel | dispatches | fetched MiB | written MiB | traffic_bytes_per_launch |", "|---|---|---|---|---|"]
        for n in fetch:
            if n not in write:
                continue
            f = sum(fetch[n]) / len(fetch[n]) * 1024 * fs
            w = sum(write[n]) / len(write[n]) * 1024 * ws
            lines.append("| %s | %d | %.1f | %.1f | %d |" % (n, len(fetch[n]), f / 2**20, w / 2**20, int(f + w)))
    path = os.path.join(a.out, "%s_kernels.md" % a.workload)
    open(path, "w").write("\n".join(lines) + "\n")
    print(path)


if __name__ == "__main__":
    main()
