"""Condense rocprofv3 output into the short text summaries kept under profiles/.

    python profile_summary.py stats  <dir with *_kernel_stats.csv>
    python profile_summary.py pmc    <dir with *_counter_collection.csv> [--copy-bytes N]

`stats` prints per-kernel calls / total / average duration.  `pmc` prints, per kernel, the average of every
collected counter per dispatch; with --copy-bytes it also derives the scale factor of FETCH_SIZE / WRITE_SIZE
from the plain elementwise kernel bench.py --copy-probe runs (torch's bitwise_not: reads and writes exactly N bytes).
"""
from __future__ import annotations

import collections
import csv
import glob
import os
import sys


def _short(name: str) -> str:
    name = name.replace("void evomoe::(anonymous namespace)::", "").replace("evomoe::", "")
    if "bitwise_not" in name:
        return "torch bitwise_not elementwise kernel (copy probe)"
    return name if len(name) <= 96 else name[:93] + "..."


def stats(d: str) -> None:
    files = glob.glob(os.path.join(d, "**", "*kernel_stats.csv"), recursive=True)
    if not files:
        sys.exit(f"no *kernel_stats.csv under {d}")
    rows = list(csv.DictReader(open(files[0])))
    print(f"{'kernel':98s} {'calls':>6s} {'total_us':>12s} {'avg_us':>10s} {'pct':>6s}")
    for r in rows:
        print(f"{_short(r['Name']):98s} {int(r['Calls']):6d} {float(r['TotalDurationNs']) / 1e3:12.1f} "
              f"{float(r['AverageNs']) / 1e3:10.2f} {float(r['Percentage']):6.2f}")


def pmc(d: str, copy_bytes: int | None) -> None:
    files = glob.glob(os.path.join(d, "**", "*counter_collection.csv"), recursive=True)
    if not files:
        sys.exit(f"no *counter_collection.csv under {d}")
    per = collections.defaultdict(lambda: collections.defaultdict(float))   # dispatch -> counter -> value
    name = {}
    for r in csv.DictReader(open(files[0])):
        per[r["Dispatch_Id"]][r["Counter_Name"]] += float(r["Counter_Value"])
        name[r["Dispatch_Id"]] = r["Kernel_Name"]
    agg = collections.defaultdict(lambda: collections.defaultdict(list))
    for did, c in per.items():
        for k, v in c.items():
            agg[name[did]][k].append(v)
    counters = sorted({k for c in per.values() for k in c})
    print(f"{'kernel':98s} {'disp':>5s} " + " ".join(f"{c:>16s}" for c in counters))
    scale = {}
    for kn, c in agg.items():
        n = len(next(iter(c.values())))
        print(f"{_short(kn):98s} {n:5d} " + " ".join(f"{sum(c[k]) / len(c[k]):16.1f}" for k in counters))
        if copy_bytes and "bitwise_not" in kn:
            for k in counters:
                if k in ("FETCH_SIZE", "WRITE_SIZE"):
                    scale[k] = (copy_bytes / 1024.0) / (sum(c[k]) / len(c[k]))
    for k, v in scale.items():
        print(f"# {k}: copy kernel moved {copy_bytes} bytes each way -> true KiB = counter x {v:.4f}")


if __name__ == "__main__":
    if len(sys.argv) < 3 or sys.argv[1] not in ("stats", "pmc"):
        sys.exit(__doc__)
    if sys.argv[1] == "stats":
        stats(sys.argv[2])
    else:
        cb = int(sys.argv[sys.argv.index("--copy-bytes") + 1]) if "--copy-bytes" in sys.argv else None
        pmc(sys.argv[2], cb)
