"""Condenses rocprofv3 CSV output into the short text summaries kept under profiles/.

  python -m paper_2605_16154_amd.profile_summary stats   <dir>   # --kernel-trace --stats runs
  python -m paper_2605_16154_amd.profile_summary counter <dir>   # --pmc runs (per-kernel means)
"""
from __future__ import annotations

import collections
import csv
import glob
import os
import sys


def _short(name: str, width: int = 96) -> str:
    name = name.replace("void ", "").replace("pcm::(anonymous namespace)::", "pcm::")
    return name if len(name) <= width else name[:width - 3] + "..."


def stats(path: str) -> str:
    rows = []
    for f in glob.glob(os.path.join(path, "**", "*kernel_stats.csv"), recursive=True):
        rows += list(csv.DictReader(open(f)))
    if not rows:
        return "no kernel_stats.csv found\n"
    rows.sort(key=lambda r: -float(r["TotalDurationNs"]))
    total = sum(float(r["TotalDurationNs"]) for r in rows)
    out = [f"{'kernel':96s} {'calls':>6s} {'avg_us':>10s} {'total_ms':>10s} {'share':>7s}"]
    for r in rows[:40]:
        out.append(f"{_short(r['Name']):96s} {int(r['Calls']):6d} {float(r['AverageNs']) / 1e3:10.2f} "
                   f"{float(r['TotalDurationNs']) / 1e6:10.3f} {100 * float(r['TotalDurationNs']) / total:6.2f}%")
    out.append(f"total kernel time: {total / 1e6:.3f} ms over {len(rows)} kernels")
    return "\n".join(out) + "\n"


def counter(path: str) -> str:
    agg = collections.defaultdict(list)
    for f in glob.glob(os.path.join(path, "**", "*counter_collection.csv"), recursive=True):
        for row in csv.DictReader(open(f)):
            agg[(_short(row["Kernel_Name"], 80), row["Counter_Name"])].append(float(row["Counter_Value"]))
    if not agg:
        return "no counter_collection.csv found\n"
    out = [f"{'kernel':80s} {'counter':28s} {'n':>5s} {'mean':>14s}"]
    for (k, c), v in sorted(agg.items()):
        out.append(f"{k:80s} {c:28s} {len(v):5d} {sum(v) / len(v):14.6g}")
    return "\n".join(out) + "\n"


if __name__ == "__main__":
    if len(sys.argv) != 3 or sys.argv[1] not in ("stats", "counter"):
        sys.exit(__doc__)
    sys.stdout.write(stats(sys.argv[2]) if sys.argv[1] == "stats" else counter(sys.argv[2]))
