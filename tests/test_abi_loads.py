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
