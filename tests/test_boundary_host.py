"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every declared
symbol, and its structural validation returns the documented codes."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    import paper_2007_13055_amd as b
    if not os.path.exists(b.library_path()):
        from paper_2007_13055_amd import build
        build.build()
    return b


def test_library_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "bsr_spmm.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(bsr_[a-z_]+)\s*\(", header))
    assert {"bsr_validate", "bsr_workspace_size", "bsr_create", "bsr_destroy", "bsr_spmm", "bsr_spmm_ex",
            "bsr_query_path", "bsr_status_string", "bsr_tune", "bsr_scratch_size", "bsr_set_scratch"} <= names
    so = ctypes.CDLL(lib.library_path())
    for nme in names:
        assert hasattr(so, nme), nme


def test_validate_codes(lib):
    ok = lib.bsr_validate(64, 64, 16, 16, [0, 1, 1, 2, 2], [0, 3])
    assert ok == 0
    assert lib.bsr_validate(64, 64, 16, 16, [0, 1, 1, 2, 2], [0, 4]) == 4      # column out of range
    assert lib.bsr_validate(64, 64, 16, 16, [0, 1, 1, 2, 2], [-1, 3]) == 4
    assert lib.bsr_validate(64, 64, 16, 16, [1, 1, 1, 2, 2], [0, 3]) == 3      # does not start at 0
    assert lib.bsr_validate(64, 64, 16, 16, [0, 2, 1, 2, 2], [0, 3]) == 3      # decreases
    assert lib.bsr_validate(64, 64, 16, 16, [0, 1, 1, 1, 1], [0, 3]) == 3      # end != nnzb
    assert lib.bsr_validate(60, 64, 16, 16, [0, 1, 1, 2, 2], [0, 3]) == 2      # bs_r does not divide n
    assert lib.bsr_validate(64, 60, 16, 16, [0, 1, 1, 2, 2], [0, 3]) == 2      # bs_c does not divide k
    assert lib.bsr_validate(64, 64, 0, 16, [0, 1, 1, 2, 2], [0, 3]) == 2
    assert lib.bsr_validate(64, 64, 16, 16, [0, 0, 0, 0, 0], []) == 0          # no stored block is valid
    so = lib.load_library()
    assert so.bsr_validate(64, 64, 16, 16, 0, None, None) == 1                 # NULL index_pointer


def test_workspace_size(lib):
    b = lib.bsr_workspace_size(3072, 3072, 32, 32, 922)
    assert b > 0 and b % 256 == 0 and b >= 4 * 96
    with pytest.raises(lib.BsrError):
        lib.bsr_workspace_size(3072, 3071, 32, 32, 922)


def test_status_strings(lib):
    seen = {lib.bsr_status_string(s) for s in range(10)}
    assert len(seen) == 10 and lib.bsr_status_string(0) == "ok"


def test_spmm_rejects_null_handle(lib):
    so = lib.load_library()
    assert so.bsr_spmm(None, 4, None, None, 0, None) == 1
    assert so.bsr_tune(None, 4, None, None, 0, 5, None, None, None) == 1
    out = ctypes.c_int(0)
    assert so.bsr_query_path(None, 4, ctypes.byref(out)) == 1
