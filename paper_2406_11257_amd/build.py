"""Compile the HIP sources of this package into libexcp.so (gfx950 only).

The build also reads the code-object metadata the compiler writes for every kernel (workgroup size,
registers, private-segment size) and refuses a library in which a kernel launched with more than 256
threads per workgroup uses private (spill) memory: those kernels are written to fit their register
budget, and a later edit or compiler that silently makes them spill must fail here, not on the GPU.
"""
from __future__ import annotations

import glob
import os
import re
import shutil
import subprocess
import tempfile

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libexcp.so")
LIB_SAN = os.path.join(HERE, "libexcp_hostsan.so")
SOURCES = ["excp_host.hip", "k_stats.hip", "k_mask.hip", "k_kmeans.hip", "k_decode.hip"]
FLAGS = [
    "-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",                       # every fp operation rounds once, as the method is defined
    "-fhip-fp32-correctly-rounded-divide-sqrt",  # sqrtf and '/' are IEEE correctly rounded (thresholds are bit-exact)
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]
# host code only (the device code is compiled as always): address and undefined-behaviour checks
SAN_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
             "-Xarch_host", "-fno-omit-frame-pointer", "-g"]
WIDE_WORKGROUP = 256                           # kernels with more threads than this must not spill


def kernel_resources(asm_dir: str) -> list[dict]:
    """Per-kernel records from the metadata of the device assembly files in `asm_dir`."""
    out = []
    for path in sorted(glob.glob(os.path.join(asm_dir, "*gfx950*.s"))):
        rec = None
        with open(path) as f:
            for line in f:
                m = re.match(r"\s*(?:- )?\.(\w+):\s*(\S+)\s*$", line)
                if not m:
                    continue
                key, val = m.group(1), m.group(2)
                if key == "max_flat_workgroup_size":       # first of the fields read here in every kernel's record
                    rec = {"file": os.path.basename(path).split("-hip-")[0], "threads": int(val)}
                    out.append(rec)
                elif rec is not None and key == "name" and "name" not in rec:
                    rec["name"] = val
                elif rec is not None and key in ("private_segment_fixed_size", "vgpr_count", "vgpr_spill_count",
                                                 "sgpr_spill_count", "group_segment_fixed_size"):
                    rec[key] = int(val)
    return [r for r in out if "name" in r and "private_segment_fixed_size" in r]


def demangled(name: str) -> str:
    try:
        return subprocess.run(["c++filt", name], capture_output=True, text=True, check=True).stdout.strip()
    except Exception:
        return name


def short_name(name: str) -> str:
    m = re.search(r"k_\w+(<[^>]*>)?", demangled(name))
    return m.group(0) if m else name


def check_resources(recs: list[dict]) -> None:
    bad = [r for r in recs if r["threads"] > WIDE_WORKGROUP and r["private_segment_fixed_size"] > 0]
    if bad:
        lines = [f"  {demangled(r['name'])}: {r['threads']} threads, {r['private_segment_fixed_size']} B/lane of private memory"
                 for r in bad]
        raise RuntimeError("kernels with wide workgroups must not use private (spill) memory:\n" + "\n".join(lines))


def build_library(verbose: bool = True, host_sanitizers: bool = False) -> str:
    """Builds libexcp.so; with host_sanitizers the same sources into libexcp_hostsan.so, the host code
    under AddressSanitizer and UBSan (for the CPU-side checks of the C ABI)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    target = LIB_SAN if host_sanitizers else LIB
    with tempfile.TemporaryDirectory(prefix="excp_build_") as tmp:
        out = os.path.join(tmp, os.path.basename(target))
        cmd = [hipcc, *FLAGS, *(SAN_FLAGS if host_sanitizers else []), "-save-temps=obj",
               *[os.path.join(CSRC, s) for s in SOURCES], "-o", out]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True, cwd=tmp)
        recs = kernel_resources(tmp)
        if not recs:
            raise RuntimeError("no kernel metadata found in the compiler's device assembly")
        check_resources(recs)
        if verbose:
            wide = [r for r in recs if r["threads"] > WIDE_WORKGROUP]
            spilling = [r for r in recs if r["private_segment_fixed_size"] > 0]
            print(f"[build] {len(recs)} kernels; {len(wide)} with more than {WIDE_WORKGROUP} threads, none of them "
                  f"uses private memory; {len(spilling)} narrower kernels spill: "
                  + ", ".join(f"{short_name(r['name'])} {r['private_segment_fixed_size']} B" for r in spilling), flush=True)
        shutil.move(out, target)
    return target


if __name__ == "__main__":
    import sys
    build_library(host_sanitizers="--host-sanitizers" in sys.argv[1:])
