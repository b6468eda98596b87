"""Turns rocprofv3 CSV output into the short tables kept under profiles/.

    python -m paper_2508_12407_amd.profile_summary kernels  <dir with *_kernel_trace.csv> [top]
    python -m paper_2508_12407_amd.profile_summary counters <dir with *_counter_collection.csv> [kernel substring[|substring...]]

`kernels`: dispatches grouped by (kernel, grid, workgroup): calls, average / minimum / maximum duration
in microseconds, share of the GPU time of the run.  `counters`: per (kernel, grid, counter): dispatches,
average / minimum / maximum of the values rocprofv3 reports per dispatch.  The rocprofv3 commands that
produce the directories are quoted in each file under profiles/ (run with --output-format csv)."""
from __future__ import annotations

import collections
import csv
import glob
import os
import re
import sys


def short(name: str) -> str:
    name = re.sub(r"\(anonymous namespace\)::", "", name)
    name = re.sub(r"^void ", "", name)
    return name if len(name) <= 86 else name[:83] + "..."


def find(directory: str, suffix: str):
    hits = sorted(glob.glob(os.path.join(directory, "**", "*" + suffix), recursive=True))
    if not hits:
        raise SystemExit("no *%s under %s" % (suffix, directory))
    return hits


def kernels(directory: str, top: int = 12) -> str:
    groups = collections.defaultdict(list)
    for path in find(directory, "kernel_trace.csv"):
        for r in csv.DictReader(open(path)):
            dur = (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3
            key = (r["Kernel_Name"], (int(r["Grid_Size_X"]), int(r["Grid_Size_Y"]), int(r["Grid_Size_Z"])), int(r["Workgroup_Size_X"]),
                   int(r.get("LDS_Block_Size", 0) or 0))
            groups[key].append(dur)
    total = sum(sum(v) for v in groups.values())
    rows = sorted(groups.items(), key=lambda kv: -sum(kv[1]))
    out = ["%-88s %22s %4s %6s %10s %10s %10s %6s %6s" % ("kernel", "grid (threads)", "wg", "calls", "avg_us", "min_us", "max_us", "%time", "lds_B")]
    for (name, grid, wg, lds), v in rows[:top]:
        out.append("%-88s %22s %4d %6d %10.2f %10.2f %10.2f %6.2f %6d" % (short(name), str(grid), wg, len(v), sum(v) / len(v), min(v), max(v),
                                                                   100 * sum(v) / total, lds))
    out.append("GPU time of all dispatches: %.3f ms" % (total / 1e3))
    return "\n".join(out)


def counters(directory: str, only: str = "") -> str:
    groups = collections.defaultdict(list)
    for path in find(directory, "counter_collection.csv"):
        for r in csv.DictReader(open(path)):
            if only and not any(o in r["Kernel_Name"] for o in only.split("|")):
                continue
            key = (r["Kernel_Name"], int(r["Grid_Size"]) if "Grid_Size" in r and r["Grid_Size"] else 0, r["Counter_Name"])
            groups[key].append(float(r["Counter_Value"]))
    out = ["%-88s %12s %28s %6s %16s %16s %16s" % ("kernel", "grid threads", "counter", "calls", "avg", "min", "max")]
    for (name, grid, ctr), v in sorted(groups.items(), key=lambda kv: (kv[0][0], kv[0][1], kv[0][2])):
        out.append("%-88s %12d %28s %6d %16.1f %16.1f %16.1f" % (short(name), grid, ctr, len(v), sum(v) / len(v), min(v), max(v)))
    return "\n".join(out)


if __name__ == "__main__":
    if len(sys.argv) < 3 or sys.argv[1] not in ("kernels", "counters"):
        raise SystemExit(__doc__)
    if sys.argv[1] == "kernels":
        print(kernels(sys.argv[2], int(sys.argv[3]) if len(sys.argv) > 3 else 12))
    else:
        print(counters(sys.argv[2], sys.argv[3] if len(sys.argv) > 3 else ""))
