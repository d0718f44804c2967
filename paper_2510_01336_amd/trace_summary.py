"""Summarise a `rocprofv3 --kernel-trace --output-format csv` run (…_kernel_trace.csv).

Dispatches are grouped by kernel name and launch shape (workgroups x workgroup size), so the launches of
the timed verify steps can be told from the context build's, which uses the same kernels at other shapes.
Prints calls, mean / min / max duration and the share of the total GPU time, largest first.

    python -m paper_2510_01336_amd.trace_summary <dir>/<name>_kernel_trace.csv [rows]
"""
from __future__ import annotations

import collections
import csv
import re
import sys


def summarise(path: str):
    groups = collections.OrderedDict()
    total = 0.0
    for r in csv.DictReader(open(path)):
        name = re.sub(r"\(.*", "", r["Kernel_Name"]).replace("void ", "")
        wg = int(r["Workgroup_Size_X"]) * int(r["Workgroup_Size_Y"]) * int(r["Workgroup_Size_Z"])
        grid = int(r["Grid_Size_X"]) * int(r["Grid_Size_Y"]) * int(r["Grid_Size_Z"]) // max(wg, 1)
        dur = (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3
        groups.setdefault((name, grid, wg), []).append(dur)
        total += dur
    out = [(n, g, w, len(v), sum(v) / len(v), min(v), max(v), sum(v)) for (n, g, w), v in groups.items()]
    out.sort(key=lambda t: -t[7])
    return total, out


def main():
    path = sys.argv[1]
    rows = int(sys.argv[2]) if len(sys.argv) > 2 else 30
    total, out = summarise(path)
    print(f"total GPU time in kernels: {total / 1e3:.3f} ms")
    print(f"{'kernel':44s} {'wgs':>7s} {'thr':>4s} {'calls':>6s} {'mean us':>9s} {'min us':>8s} {'max us':>8s} {'share':>6s}")
    for n, g, w, c, mean, lo, hi, tot in out[:rows]:
        print(f"{n[:44]:44s} {g:7d} {w:4d} {c:6d} {mean:9.2f} {lo:8.2f} {hi:8.2f} {100 * tot / total:5.1f}%")


if __name__ == "__main__":
    main()
