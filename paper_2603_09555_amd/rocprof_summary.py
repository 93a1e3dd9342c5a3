"""Condense rocprofv3 CSV output into the per-kernel tables kept under ``profiles/``.

    python3 -m paper_2603_09555_amd.rocprof_summary trace    <..._kernel_trace.csv>
    python3 -m paper_2603_09555_amd.rocprof_summary counters <..._counter_collection.csv>

``trace``: one row per (kernel, grid): calls, mean / min / max of End_Timestamp - Start_Timestamp in
microseconds.  ``counters``: one row per (kernel, grid, counter): launches, median / min / max of the
counter value (medians, because the first launches of a kernel often find the caches in another state).
One bench run covers several workloads; the grid tells them apart.  Only this library's kernels are
listed, plus the runtime's buffer copy (the calibration launch of the counter runs).
"""
from __future__ import annotations

import collections
import csv
import re
import statistics
import sys


def short_name(full: str) -> str | None:
    m = re.search(r"ssd::(?:\(anonymous namespace\)::)?(\w+(?:<[^>(]*>)?)", full)
    if m:
        return m.group(1).replace("ssd::", "")
    if "copyBuffer" in full:
        return full.split("(")[0]
    return None


def grid_of(row: dict) -> str:
    if row.get("Grid_Size"):
        return row["Grid_Size"]
    return "x".join(row.get(k, "1") for k in ("Grid_Size_X", "Grid_Size_Y", "Grid_Size_Z"))


def trace(path: str) -> None:
    acc = collections.defaultdict(list)
    with open(path) as f:
        for row in csv.DictReader(f):
            name = short_name(row["Kernel_Name"])
            if name is None:
                continue
            wg = row.get("Workgroup_Size") or row.get("Workgroup_Size_X", "")
            acc[(name, grid_of(row), wg)].append(int(row["End_Timestamp"]) - int(row["Start_Timestamp"]))
    print("%-44s %-14s %-5s %6s %10s %10s %10s" % ("kernel", "grid(threads)", "wg", "calls", "avg_us", "min_us", "max_us"))
    for (name, grid, wg), v in sorted(acc.items()):
        print("%-44s %-14s %-5s %6d %10.2f %10.2f %10.2f" % (name[:44], grid, wg, len(v), sum(v) / len(v) / 1e3,
                                                              min(v) / 1e3, max(v) / 1e3))


def counters(path: str) -> None:
    acc = collections.defaultdict(list)
    with open(path) as f:
        for row in csv.DictReader(f):
            name = short_name(row["Kernel_Name"])
            if name is None:
                continue
            acc[(name, grid_of(row), row["Counter_Name"])].append(float(row["Counter_Value"]))
    print("%-44s %-10s %-28s %5s %14s %14s %14s" % ("kernel", "grid", "counter", "n", "median", "min", "max"))
    for (name, grid, counter), v in sorted(acc.items()):
        print("%-44s %-10s %-28s %5d %14.1f %14.1f %14.1f" % (name[:44], grid, counter, len(v), statistics.median(v),
                                                             min(v), max(v)))


def main(argv: list[str]) -> int:
    if len(argv) != 3 or argv[1] not in ("trace", "counters"):
        print(__doc__)
        return 2
    (trace if argv[1] == "trace" else counters)(argv[2])
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv))
