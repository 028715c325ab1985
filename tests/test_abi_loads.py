"""CPU-side checks of the C ABI: the library loads and exports every symbol the header declares;
the size functions agree with the oracle's closed form (no GPU work is issued)."""
import os
import re

import pytest

import oracle as O
import paper_2406_11257_amd as X
from paper_2406_11257_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "excp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(excp_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound():
    names = declared_symbols()
    assert "excp_compress_step" in names and "excp_decompress_step" in names and len(names) >= 14
    L = X.lib()
    for name in names:
        assert hasattr(L, name), name
        assert name in binding.SYMBOLS, name


def test_size_functions_match_the_closed_form():
    for n, nw, no, nb in [(0, 0, 0, 4), (1, 1, 1, 2), (1000, 345, 76, 4), (4097, 4097, 0, 8),
                          (131072000, 45000000, 9900000, 4), (65, 64, 63, 3)]:
        assert X.excp_blob_size(n, nw, no, nb) == O.blob_size(n, nw, no, nb)
        assert X.excp_blob_bound(n, nb) == O.blob_size(n, n, n, nb)
    assert X.excp_blob_size(10, 11, 0, 4) == 0 and X.excp_blob_bound(10, 9) == 0
    assert X.excp_strerror(0) == "ok" and "finite" in X.excp_strerror(X.EXCP_E_NONFINITE)


def test_stage_names_are_listed():
    L = X.lib()
    names = [L.excp_stage_name(i).decode() for i in range(L.excp_stage_count())]
    assert {"stats_stream", "mask_slots", "km_iter", "assign_pack", "decode_main"} <= set(names)
    assert len(set(names)) == len(names)


def test_argument_errors_need_no_gpu():
    L = X.lib()
    assert L.excp_collect(None, None) == X.EXCP_E_ARG
    assert L.excp_compress_tensors(None, 0, None, 5e-5, 2.0, 4, 10, 0) == X.EXCP_E_ARG
    assert L.excp_create(None, 0, None, 1, 1) == X.EXCP_E_ARG
    assert L.excp_reconstruct_chain(None, 0, None) == X.EXCP_E_ARG


def test_host_code_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    """The library is built once more with its HOST code under AddressSanitizer and UBSan (the device
    code as always), and a small C program walks every host path that needs no GPU work -- size
    functions, names, argument and call-order checks of every entry point -- against it.  Any
    sanitizer report, or a failed check, fails the test."""
    import subprocess
    from paper_2406_11257_amd import build
    srcs = [os.path.join(build.CSRC, f) for f in os.listdir(build.CSRC)] + [os.path.join(ROOT, "include", "excp.h")]
    if not os.path.exists(build.LIB_SAN) or os.path.getmtime(build.LIB_SAN) < max(os.path.getmtime(s) for s in srcs):
        build.build_library(verbose=False, host_sanitizers=True)
    clang = os.path.join(os.path.dirname(os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")), "..", "llvm", "bin", "clang")
    exe = str(tmp_path / "abi_host_check")
    pkg = os.path.dirname(build.LIB_SAN)
    subprocess.run([clang, "-fsanitize=address,undefined", "-fno-omit-frame-pointer", "-g",
                    os.path.join(ROOT, "tests", "abi_host_check.c"), "-L" + pkg, "-lexcp_hostsan",
                    "-Wl,-rpath," + pkg, "-o", exe], check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1",
               HIP_VISIBLE_DEVICES="", ROCR_VISIBLE_DEVICES="")     # host paths only: no device is touched
    r = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=120)
    assert r.returncode == 0 and r.stdout.strip().endswith("ok"), r.stdout + r.stderr
    assert "Sanitizer" not in r.stderr and "runtime error" not in r.stderr, r.stderr
