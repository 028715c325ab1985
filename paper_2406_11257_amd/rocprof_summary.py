"""Turn a rocprofv3 CSV output directory into the short text summaries kept under profiles/.

    python3 -m paper_2406_11257_amd.rocprof_summary stats   <dir>   # from --kernel-trace --stats
    python3 -m paper_2406_11257_amd.rocprof_summary counter <dir>   # from --pmc FETCH_SIZE / WRITE_SIZE ...
    python3 -m paper_2406_11257_amd.rocprof_summary traffic <workload> <fetch dir> <write dir>
                                                            # the table bench.py reads (profiles/hbm_traffic.txt)

Only the library's own kernels (k_*) are listed; names are shortened to the kernel identifier.
The traffic table is stamped with a hash of the kernel sources it was measured on, so that a reader
can tell a table that no longer describes the code.
"""
from __future__ import annotations

import collections
import csv
import glob
import hashlib
import os
import re
import sys

CSRC = os.path.join(os.path.dirname(os.path.abspath(__file__)), "csrc")


def sources_hash() -> str:
    """First 16 hex digits of the SHA-256 over the kernel and host sources (names and contents)."""
    h = hashlib.sha256()
    for name in sorted(os.listdir(CSRC)):
        if name.endswith((".hip", ".h")):
            h.update(name.encode())
            with open(os.path.join(CSRC, name), "rb") as f:
                h.update(f.read())
    return h.hexdigest()[:16]


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


def read_counters(directory: str):
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
    return agg, disp


def counter(directory: str) -> None:
    agg, disp = read_counters(directory)
    names = sorted({c for v in agg.values() for c in v})
    print(f"{'kernel':28s} {'dispatches':>10s} " + " ".join(f"{n + ' per dispatch':>26s}" for n in names))
    for k, v in sorted(agg.items(), key=lambda kv: -sum(kv[1].values())):
        nd = len(disp[k])
        print(f"{k:28s} {nd:10d} " + " ".join(f"{v.get(n, 0.0) / nd:26.1f}" for n in names))


def traffic(workload: str, fetch_dir: str, write_dir: str) -> None:
    """HBM bytes per launch of every kernel: FETCH_SIZE and WRITE_SIZE (KiB per dispatch), each scaled by
    what the same counter reads for k_copy_probe, whose traffic is known (1 GiB read, 1 GiB written)."""
    per = {}
    for which, directory, cname in (("fetch", fetch_dir, "FETCH_SIZE"), ("write", write_dir, "WRITE_SIZE")):
        agg, disp = read_counters(directory)
        if "k_copy_probe" not in agg:
            raise SystemExit("the run holds no k_copy_probe launch to calibrate " + cname)
        scale = (1 << 20) / (agg["k_copy_probe"][cname] / len(disp["k_copy_probe"]))      # KiB per counted KiB
        print(f"# {cname}: k_copy_probe reads {agg['k_copy_probe'][cname] / len(disp['k_copy_probe']):.1f} for 1048576 KiB: scaled by {scale:.4f}")
        for k, v in agg.items():
            per.setdefault(k, {})[which] = v[cname] / len(disp[k]) * scale * 1024.0
    print("# Measured HBM bytes per launch.  traffic <workload> <kernel> <bytes fetched> <bytes written>")
    print("sources", sources_hash())
    for k, v in sorted(per.items(), key=lambda kv: -(kv[1].get("fetch", 0) + kv[1].get("write", 0))):
        print(f"traffic {workload} {k} {v.get('fetch', 0.0):.0f} {v.get('write', 0.0):.0f}")


if __name__ == "__main__":
    if len(sys.argv) == 5 and sys.argv[1] == "traffic":
        traffic(*sys.argv[2:])
    elif len(sys.argv) == 3 and sys.argv[1] in ("stats", "counter"):
        (stats if sys.argv[1] == "stats" else counter)(sys.argv[2])
    else:
        raise SystemExit(__doc__)
