"""Condenses rocprofv3 CSV output into the short text summaries kept under profiles/.

  python -m paper_2605_16154_amd.profile_summary stats   <dir>   # --kernel-trace --stats runs
  python -m paper_2605_16154_amd.profile_summary counter <dir>   # --pmc runs (per-kernel means)
  python -m paper_2605_16154_amd.profile_summary traffic <fetch_dir> <write_dir> <kernel substring>
                                                                  # HBM-side bytes per launch of one kernel
  python -m paper_2605_16154_amd.profile_summary tail <dir> <kernel substring> <n>
                                                                  # mean duration of a kernel's last n launches
  python -m paper_2605_16154_amd.profile_summary table <fetch_dir> <write_dir> <kernel substring> [...]
                                                                  # HBM-side bytes per launch of several kernels, one row each
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


def tail(path: str, kernel_substr: str, n: int) -> str:
    """Mean duration of the last n dispatches of a kernel in a --kernel-trace run (e.g. the timed steps of a
    benchmark whose set-up launches the same kernel)."""
    rows = []
    for f in glob.glob(os.path.join(path, "**", "*kernel_trace.csv"), recursive=True):
        for row in csv.DictReader(open(f)):
            if kernel_substr in row["Kernel_Name"]:
                rows.append((int(row["Start_Timestamp"]), int(row["End_Timestamp"])))
    rows.sort()
    if not rows:
        return "no matching dispatch found\n"
    last = rows[-n:]
    mean_all = sum(e - b for b, e in rows) / len(rows)
    mean_last = sum(e - b for b, e in last) / len(last)
    return (f"kernel={kernel_substr}\nlaunches={len(rows)}\navg_us_all={mean_all / 1e3:.2f}\n"
            f"last_n={len(last)}\navg_us_last_n={mean_last / 1e3:.2f}\n")


KERNEL_SOURCES = ("gemm_bf16.h", "actor_bf16.hip")


def kernel_source_hash() -> str:
    """Hash of the code of the bf16 GEMM (comments and white space left out); byte counters are only valid for
    the code they were taken on."""
    import hashlib
    import re
    h = hashlib.sha256()
    here = os.path.join(os.path.dirname(os.path.abspath(__file__)), "csrc")
    for name in KERNEL_SOURCES:
        text = open(os.path.join(here, name), encoding="utf-8").read()
        text = re.sub(r"//[^\n]*", "", text)            # line comments (the sources use no block comments or // in strings)
        h.update("".join(text.split()).encode())
    return h.hexdigest()[:16]


def _mean_counter(path: str, counter_name: str, kernel_substr: str, large_only: bool = False):
    """Mean of a counter over the launches of the kernels whose name contains kernel_substr.  large_only keeps the
    launches within a factor two of the largest: the calibration kernel is a library elementwise kernel that the
    program may also launch on a handful of elements."""
    vals = []
    for f in glob.glob(os.path.join(path, "**", "*counter_collection.csv"), recursive=True):
        for row in csv.DictReader(open(f)):
            if row["Counter_Name"] == counter_name and kernel_substr in row["Kernel_Name"]:
                vals.append(float(row["Counter_Value"]))
    if large_only and vals:
        vals = [v for v in vals if 2 * v >= max(vals)]
    return (sum(vals) / len(vals), len(vals)) if vals else (float("nan"), 0)


def traffic(fetch_dir: str, write_dir: str, kernel_substr: str) -> str:
    fetch, nf = _mean_counter(fetch_dir, "FETCH_SIZE", kernel_substr)
    write, nw = _mean_counter(write_dir, "WRITE_SIZE", kernel_substr)
    cal_f, _ = _mean_counter(fetch_dir, "FETCH_SIZE", "CUDAFunctorOnSelf_add<double>", large_only=True)
    cal_w, _ = _mean_counter(write_dir, "WRITE_SIZE", "CUDAFunctorOnSelf_add<double>", large_only=True)
    gib = float(1 << 20)   # KiB in 1 GiB
    return (f"kernel={kernel_substr}\nlaunches_fetch={nf}\nlaunches_write={nw}\n"
            f"fetch_kib_per_launch={fetch:.1f}\nwrite_kib_per_launch={write:.1f}\n"
            f"calibration_fetch_kib_for_1GiB_read={cal_f:.1f}\ncalibration_write_kib_for_1GiB_write={cal_w:.1f}\n"
            f"scale_fetch={gib / cal_f:.4f}\nscale_write={gib / cal_w:.4f}\n"
            f"source_hash={kernel_source_hash()}\n")


def table(fetch_dir: str, write_dir: str, kernels) -> str:
    """One row per kernel: launches, FETCH_SIZE and WRITE_SIZE per launch scaled to bytes with the factors that the
    1 GiB elementwise calibration kernel of the same runs gives."""
    cal_f, _ = _mean_counter(fetch_dir, "FETCH_SIZE", "CUDAFunctorOnSelf_add<double>", large_only=True)
    cal_w, _ = _mean_counter(write_dir, "WRITE_SIZE", "CUDAFunctorOnSelf_add<double>", large_only=True)
    gib = float(1 << 20)
    sf, sw = gib / cal_f, gib / cal_w
    out = [f"# scale_fetch={sf:.4f} scale_write={sw:.4f} (FETCH_SIZE / WRITE_SIZE of a kernel that reads and writes exactly 1 GiB)",
           f"{'kernel':34s} {'launches':>8s} {'read_MB':>12s} {'written_MB':>12s}"]
    for k in kernels:
        f, nf = _mean_counter(fetch_dir, "FETCH_SIZE", k)
        w, _ = _mean_counter(write_dir, "WRITE_SIZE", k)
        out.append(f"{k:34s} {nf:8d} {f * sf * 1024 / 1e6:12.3f} {w * sw * 1024 / 1e6:12.3f}")
    return "\n".join(out) + "\n"


if __name__ == "__main__":
    if len(sys.argv) >= 5 and sys.argv[1] == "table":
        sys.stdout.write(table(sys.argv[2], sys.argv[3], sys.argv[4:]))
        sys.exit(0)
    if len(sys.argv) == 5 and sys.argv[1] == "traffic":
        sys.stdout.write(traffic(sys.argv[2], sys.argv[3], sys.argv[4]))
        sys.exit(0)
    if len(sys.argv) == 5 and sys.argv[1] == "tail":
        sys.stdout.write(tail(sys.argv[2], sys.argv[3], int(sys.argv[4])))
        sys.exit(0)
    if len(sys.argv) != 3 or sys.argv[1] not in ("stats", "counter"):
        sys.exit(__doc__)
    sys.stdout.write(stats(sys.argv[2]) if sys.argv[1] == "stats" else counter(sys.argv[2]))
