"""The C-ABI library loads and exports every symbol include/sptir.h declares
(no compute calls, so no GPU needed)."""
import ctypes
import os
import re

import paper_2207_04606_amd as sptir
from paper_2207_04606_amd import build as sptir_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "sptir.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sptir_[a-z0-9_]+)\s*\(", text)) - {"sptir_alloc_fn", "sptir_free_fn"})


def test_library_exports_every_declared_symbol():
    if sptir_build.is_stale():
        sptir_build.build()
    lib = sptir.load_library()
    names = declared_functions()
    assert len(names) >= 10
    for name in names:
        assert hasattr(lib, name), f"{name} is declared in sptir.h but not exported"
        assert name in sptir.EXPORTED_SYMBOLS


def test_host_only_entry_points():
    assert sptir.sptir_status_string(0) == "ok"
    assert "ascending" in sptir.sptir_status_string(2)
    # k = ceil(log2(nnz / n)) (section 4.2.1)
    assert sptir.sptir_default_bucket_log2(10556, 2708) == 2
    assert sptir.sptir_default_bucket_log2(114615892, 232965) == 9
    assert sptir.sptir_default_bucket_log2(8, 8) == 0
    assert sptir.sptir_default_bucket_log2(9, 8) == 1
    assert sptir.sptir_default_bucket_log2(0, 8) == 0
    # 32-bit gather offsets: column x (feat x 4) with a 24-bit multiply, so both factors stay below 2^24 and the
    # product below 2^32
    fit = sptir.sptir_gather_offsets_fit_32
    assert fit(232965, 128) and fit(232965, 512) and fit(1, 1) and fit(0, 64)
    assert fit((1 << 24) - 1, 64) and not fit(1 << 24, 64)              # columns at the 24-bit limit
    assert fit(16, (1 << 22) - 1) and not fit(16, 1 << 22)              # bytes per row at the 24-bit limit
    assert fit(1 << 23, 127) and not fit(1 << 23, 128)                  # product at the 32-bit limit
    assert not fit(-1, 64) and not fit(64, 0)


def test_null_arguments_are_rejected_without_a_gpu():
    lib = sptir.load_library()
    assert lib.sptir_hyb_build(None, 1, 1, None, None) == 1
    assert lib.sptir_hyb_info(None, None) == 1
    assert lib.sptir_hyb_destroy(None) == 0
    assert lib.sptir_spmm(None, None, None, 4, None) == 1


def test_header_is_plain_c():
    """include/sptir.h is the boundary of a C ABI: a C99 compiler must accept it on its own."""
    import subprocess
    header = os.path.join(ROOT, "include", "sptir.h")
    done = subprocess.run(["gcc", "-fsyntax-only", "-x", "c", "-std=c99", "-Wall", "-Werror", header],
                          capture_output=True, text=True)
    assert done.returncode == 0, done.stderr
