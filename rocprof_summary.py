"""Condense rocprofv3 CSV output into the short text summaries kept under profiles/.

    python3 rocprof_summary.py <rocprofv3 output dir> [--all-kernels] [--last N]

Reads every *kernel_trace.csv (per-kernel call count and duration statistics) and every
*counter_collection.csv (per-kernel mean of each counter) found below the directory.  Only this
library's kernels are listed unless --all-kernels is given (a plain copy kernel used to
calibrate FETCH_SIZE / WRITE_SIZE is not one of ours).  --last N keeps, per kernel, only its last N
dispatches (by start time): the launches before them are the warm-up during which the clock governor settles.
"""
from __future__ import annotations

import collections
import csv
import glob
import sys


def _ours(name: str) -> bool:
    """Kernels of libflashblock.so (namespace fb) and of the calibration library (anonymous namespace of fb_calib.hip)."""
    if "fb::" in name:
        return True
    return "(anonymous namespace)::" in name and any(t in name for t in ("read_vgpr_kernel", "read_lds_kernel", "copy_kernel", "mfma_kernel")) \
        and "at::" not in name


def _short(name: str) -> str:
    name = name.replace("fb::(anonymous namespace)::", "fb::").replace("(anonymous namespace)::", "fbc::").replace("void ", "")
    cut = name.find("(")
    if cut > 0 and ("fb::" in name or "fbc::" in name):
        name = name[:cut]
    return name[:90]


def summarize(root: str, all_kernels: bool = False, last: int = 0) -> str:
    lines = []
    for f in sorted(glob.glob(root + "/**/*kernel_trace.csv", recursive=True)):
        acc = collections.defaultdict(list)
        rows = sorted(csv.DictReader(open(f)), key=lambda r: int(r["Start_Timestamp"]))
        for r in rows:
            k = r["Kernel_Name"]
            if not all_kernels and not _ours(k):
                continue
            acc[_short(k)].append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
        if last > 0:
            acc = {k: v[-last:] for k, v in acc.items()}
        lines.append(f"# kernel trace: {f.split('/')[-1]}" + (f" (last {last} dispatches of every kernel)" if last > 0 else ""))
        lines.append(f"{'kernel':60s} {'calls':>6s} {'avg_us':>9s} {'med_us':>9s} {'min_us':>9s} {'max_us':>9s}")
        for k, v in sorted(acc.items(), key=lambda kv: -sum(kv[1])):
            s = sorted(v)
            lines.append(f"{k:60s} {len(v):6d} {sum(v) / len(v):9.2f} {s[len(s) // 2]:9.2f} {s[0]:9.2f} {s[-1]:9.2f}")
    for f in sorted(glob.glob(root + "/**/*counter_collection.csv", recursive=True)):
        acc = collections.defaultdict(lambda: collections.defaultdict(list))
        for r in csv.DictReader(open(f)):
            k = r["Kernel_Name"]
            if not all_kernels and not _ours(k):
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
    n_last = int(sys.argv[sys.argv.index("--last") + 1]) if "--last" in sys.argv else 0
    print(summarize(sys.argv[1], "--all-kernels" in sys.argv, n_last))
