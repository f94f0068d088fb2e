"""Condense rocprofv3 CSV output into the short text summaries kept under profiles/.

    python3 rocprof_summary.py <rocprofv3 output dir> [--all-kernels]

Reads every *kernel_trace.csv (per-kernel call count and duration statistics) and every
*counter_collection.csv (per-kernel mean of each counter) found below the directory.  Only this
library's kernels are listed unless --all-kernels is given (a plain copy kernel used to
calibrate FETCH_SIZE / WRITE_SIZE is not one of ours).
"""
from __future__ import annotations

import collections
import csv
import glob
import sys


def _short(name: str) -> str:
    name = name.replace("fb::(anonymous namespace)::", "fb::").replace("void ", "")
    cut = name.find("(")
    if cut > 0 and "fb::" in name:
        name = name[:cut]
    return name[:90]


def summarize(root: str, all_kernels: bool = False) -> str:
    lines = []
    for f in sorted(glob.glob(root + "/**/*kernel_trace.csv", recursive=True)):
        acc = collections.defaultdict(list)
        for r in csv.DictReader(open(f)):
            k = r["Kernel_Name"]
            if "fb::" not in k and not all_kernels:
                continue
            acc[_short(k)].append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
        lines.append(f"# kernel trace: {f.split('/')[-1]}")
        lines.append(f"{'kernel':60s} {'calls':>6s} {'avg_us':>9s} {'med_us':>9s} {'min_us':>9s} {'max_us':>9s}")
        for k, v in sorted(acc.items(), key=lambda kv: -sum(kv[1])):
            s = sorted(v)
            lines.append(f"{k:60s} {len(v):6d} {sum(v) / len(v):9.2f} {s[len(s) // 2]:9.2f} {s[0]:9.2f} {s[-1]:9.2f}")
    for f in sorted(glob.glob(root + "/**/*counter_collection.csv", recursive=True)):
        acc = collections.defaultdict(lambda: collections.defaultdict(list))
        for r in csv.DictReader(open(f)):
            k = r["Kernel_Name"]
            if "fb::" not in k and not all_kernels:
                continue
            acc[_short(k)][r["Counter_Name"]].append(float(r["Counter_Value"]))
        lines.append(f"# counters: {f.split('/')[-1]}")
        for k, cs in acc.items():
            for c, v in sorted(cs.items()):
                lines.append(f"{k:60s} {c:28s} dispatches={len(v):4d} mean={sum(v) / len(v):16.1f}")
    return "\n".join(lines)


if __name__ == "__main__":
    if len(sys.argv) < 2:
        print(__doc__)
        sys.exit(1)
    print(summarize(sys.argv[1], "--all-kernels" in sys.argv))
