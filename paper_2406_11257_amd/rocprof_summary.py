"""Turn a rocprofv3 CSV output directory into the short text summaries kept under profiles/.

    python3 -m paper_2406_11257_amd.rocprof_summary stats   <dir>   # from --kernel-trace --stats
    python3 -m paper_2406_11257_amd.rocprof_summary counter <dir>   # from --pmc FETCH_SIZE / WRITE_SIZE ...

Only the library's own kernels (k_*) are listed; names are shortened to the kernel identifier.
"""
from __future__ import annotations

import collections
import csv
import glob
import re
import sys


def short(name: str):
    m = re.search(r"(k_[a-z0-9_]+(<[^>]*>)?)", name)
    return m.group(1).replace(" ", "") if m else None        # no blanks: the tables are split on them


def stats(directory: str) -> None:
    paths = glob.glob(directory + "/**/*kernel_trace.csv", recursive=True)
    if not paths:
        raise SystemExit("no *kernel_trace.csv under " + directory)
    dur = collections.defaultdict(list)
    for r in csv.DictReader(open(paths[0])):
        k = short(r["Kernel_Name"])
        if k:
            dur[k].append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) * 1e-6)
    total = sum(sum(v) for v in dur.values())
    print(f"{'kernel':28s} {'calls':>7s} {'total ms':>10s} {'avg ms':>9s} {'min ms':>9s} {'max ms':>9s} {'%':>6s}")
    for k, v in sorted(dur.items(), key=lambda kv: -sum(kv[1])):
        print(f"{k:28s} {len(v):7d} {sum(v):10.3f} {sum(v) / len(v):9.4f} {min(v):9.4f} {max(v):9.4f} "
              f"{100 * sum(v) / total:6.2f}")
    print(f"{'all library kernels':28s} {sum(len(v) for v in dur.values()):7d} {total:10.3f}")


def counter(directory: str) -> None:
    paths = glob.glob(directory + "/**/*counter_collection.csv", recursive=True)
    if not paths:
        raise SystemExit("no *counter_collection.csv under " + directory)
    agg = collections.defaultdict(lambda: collections.defaultdict(float))
    disp = collections.defaultdict(set)
    for r in csv.DictReader(open(paths[0])):
        k = short(r["Kernel_Name"])
        if k:
            agg[k][r["Counter_Name"]] += float(r["Counter_Value"])
            disp[k].add(r["Dispatch_Id"])
    names = sorted({c for v in agg.values() for c in v})
    print(f"{'kernel':28s} {'dispatches':>10s} " + " ".join(f"{n + ' per dispatch':>26s}" for n in names))
    for k, v in sorted(agg.items(), key=lambda kv: -sum(kv[1].values())):
        nd = len(disp[k])
        print(f"{k:28s} {nd:10d} " + " ".join(f"{v.get(n, 0.0) / nd:26.1f}" for n in names))


if __name__ == "__main__":
    if len(sys.argv) != 3 or sys.argv[1] not in ("stats", "counter"):
        raise SystemExit(__doc__)
    (stats if sys.argv[1] == "stats" else counter)(sys.argv[2])
