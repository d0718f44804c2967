"""Summarise a `rocprofv3 --pmc FETCH_SIZE` or `--pmc WRITE_SIZE` run of bench.py (csv output).

Prints, per kernel name and grid size, the number of dispatches and the mean counter value, and the
same scaled to bytes with the factor the calibration copy (stream_copy_kernel, a kernel that reads
and writes exactly CALIBRATION_COPY_BYTES) gives:  factor = copy bytes / counter value of the copy.

    python -m paper_2510_01336_amd.pmc_summary <dir>/b8_counter_collection.csv [copy_bytes]

With `--counters` in place of copy_bytes the file may hold several counters per dispatch (one run of SQ
counters, say): the mean of each per kernel name and grid size is printed, no scaling.
"""
from __future__ import annotations

import collections
import csv
import re
import sys


def summarise(path: str, copy_bytes: int = 1 << 30):
    rows = list(csv.DictReader(open(path)))
    counter = rows[0]["Counter_Name"]
    groups = collections.OrderedDict()
    for r in rows:
        name = re.sub(r"\(.*", "", r["Kernel_Name"])
        key = (name, int(r["Grid_Size"]), int(r["Workgroup_Size"]))
        groups.setdefault(key, []).append(float(r["Counter_Value"]))
    copy = [v for (n, g, w), vs in groups.items() if "stream_copy_kernel" in n for v in vs]
    factor = copy_bytes / (sum(copy) / len(copy)) if copy else float("nan")
    out = []
    for (name, grid, wg), vs in groups.items():
        mean = sum(vs) / len(vs)
        out.append((name, grid, wg, len(vs), mean, mean * factor))
    return counter, factor, out


def summarise_counters(path: str):
    """{(kernel, grid, workgroup): (dispatches, {counter: mean value})}, kernels in order of first dispatch."""
    sums = collections.OrderedDict()
    for r in csv.DictReader(open(path)):
        name = re.sub(r"\(.*", "", r["Kernel_Name"])
        key = (name, int(r["Grid_Size"]), int(r["Workgroup_Size"]))
        per = sums.setdefault(key, collections.OrderedDict())
        tot = per.setdefault(r["Counter_Name"], [0.0, 0])
        tot[0] += float(r["Counter_Value"])
        tot[1] += 1
    return collections.OrderedDict((k, (max(n for _, n in per.values()), {c: t / n for c, (t, n) in per.items()}))
                                   for k, per in sums.items())


def main():
    path = sys.argv[1]
    if len(sys.argv) > 2 and sys.argv[2] == "--counters":
        out = summarise_counters(path)
        names = sorted({c for _, per in out.values() for c in per})
        print(f"{'kernel':50s} {'grid':>9s} {'wg':>4s} {'calls':>6s} " + " ".join(f"{c[-22:]:>22s}" for c in names))
        for (name, grid, wg), (n, per) in out.items():
            print(f"{name[:50]:50s} {grid:9d} {wg:4d} {n:6d} " + " ".join(f"{per.get(c, float('nan')):22.1f}" for c in names))
        return
    copy_bytes = int(sys.argv[2]) if len(sys.argv) > 2 else 1 << 30
    counter, factor, out = summarise(path, copy_bytes)
    print(f"counter {counter}; calibration: {copy_bytes} bytes / copy-kernel reading -> {factor:.1f} bytes per count")
    print(f"{'kernel':58s} {'grid':>9s} {'wg':>4s} {'calls':>6s} {'mean count':>14s} {'mean MB':>10s}")
    for name, grid, wg, n, mean, b in sorted(out, key=lambda t: -t[5] * t[3])[:24]:
        print(f"{name[:58]:58s} {grid:9d} {wg:4d} {n:6d} {mean:14.1f} {b / 1e6:10.3f}")


if __name__ == "__main__":
    main()
