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
    seen = {lib.bsr_status_string(s) for s in range(11)}
    assert len(seen) == 11 and lib.bsr_status_string(0) == "ok"


def test_spmm_rejects_null_handle(lib):
    so = lib.load_library()
    assert so.bsr_spmm(None, 4, None, None, 0, None) == 1
    assert so.bsr_tune(None, 4, None, None, 0, 5, None, None, None) == 1
    out = ctypes.c_int(0)
    assert so.bsr_query_path(None, 4, ctypes.byref(out)) == 1


def test_transpose_pattern_against_scipy(lib):
    """bsr_transpose_pattern: the pattern of W^T equals what SciPy's CSR transpose gives for the same
    block pattern; perm maps every block of W^T to its source; blocks of a block-row of W^T come by
    ascending block-row of W; duplicates survive."""
    import numpy as np
    import scipy.sparse as sp
    rng = np.random.default_rng(4)
    R, C = 9, 7
    mask = rng.random((R, C)) < 0.4
    mask[3, :] = False
    mask[:, 2] = False
    ptr = np.concatenate([[0], np.cumsum(mask.sum(1))]).astype(np.int32)
    idx = np.concatenate([np.nonzero(row)[0] for row in mask]).astype(np.int32)
    t_ptr, t_idx, perm = lib.bsr_transpose_pattern(R * 4, C * 8, 4, 8, ptr, idx)
    ref = sp.csr_matrix((np.arange(1, idx.shape[0] + 1), idx, ptr), shape=(R, C)).T.tocsr()
    ref.sort_indices()
    assert np.array_equal(t_ptr, ref.indptr) and np.array_equal(t_idx, ref.indices)
    assert np.array_equal(perm, ref.data - 1)
    # duplicates and unsorted columns: every block appears exactly once, order inside a row of W^T stable
    ptr2, idx2 = np.array([0, 3, 4], np.int32), np.array([1, 0, 1, 1], np.int32)
    t_ptr2, t_idx2, perm2 = lib.bsr_transpose_pattern(2, 2, 1, 1, ptr2, idx2)
    assert t_ptr2.tolist() == [0, 1, 4] and t_idx2.tolist() == [0, 0, 0, 1] and perm2.tolist() == [1, 0, 2, 3]
    with pytest.raises(lib.BsrError):
        lib.bsr_transpose_pattern(8, 8, 4, 4, [0, 1, 1], [5])          # column out of range


@pytest.mark.parametrize("bs_r,bs_c,dtype", [(16, 16, "bf16"), (16, 16, "f32"), (8, 8, "f32"), (8, 16, "f16"), (32, 32, "f16"),
                                              (64, 64, "f16"), (16, 64, "bf16"), (16, 1, "f32"), (3, 5, "f32")])
@pytest.mark.parametrize("pattern", ["one_per_row", "duplicates", "full", "one_long_row"])
def test_plan_fits_the_promised_workspace(lib, bs_r, bs_c, dtype, pattern):
    """bsr_create builds its whole plan (row descriptors, pair / tile / run tables) on the host before the
    upload and refuses a workspace that is too small: with exactly bsr_workspace_size() bytes it must never
    answer WORKSPACE, whatever the pattern.  No GPU: the upload then fails with HIP, which is fine here."""
    R, C = 37, 41
    if pattern == "one_per_row":
        counts = [1] * R
        idx = [(7 * r) % C for r in range(R)]
    elif pattern == "duplicates":
        counts = [6] * R
        idx = [c for r in range(R) for c in (r % C, r % C, r % C, (r + 5) % C, (r + 5) % C, (r + 9) % C)]
    elif pattern == "full":
        counts = [C] * R
        idx = list(range(C)) * R
    else:
        counts = [0] * R
        counts[5] = C
        idx = list(range(C))
    ptr = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    idx = np.asarray(idx, dtype=np.int32)
    nnzb = int(idx.shape[0])
    n, k = R * bs_r, C * bs_c
    so = lib.load_library()
    need = lib.bsr_workspace_size(n, k, bs_r, bs_c, nnzb)
    es = 4 if dtype == "f32" else 2
    data = np.zeros(nnzb * bs_r * bs_c * es + 64, dtype=np.uint8)       # stand-ins for device buffers: never read here
    ws = np.zeros(need + 64, dtype=np.uint8)
    align = lambda a: (a.ctypes.data + 15) & ~15
    handle = ctypes.c_void_p()
    code = {"f32": 0, "f16": 1, "bf16": 2}[dtype]
    st = so.bsr_create(ctypes.byref(handle), n, k, bs_r, bs_c, nnzb, code, align(data), idx.ctypes.data, ptr.ctypes.data,
                       idx.ctypes.data, ptr.ctypes.data, align(ws), need, None)
    assert st in (0, 8), lib.bsr_status_string(st)                      # OK (a GPU is present) or HIP (none): never WORKSPACE
    if st == 0:
        so.bsr_destroy(handle)
    # one byte less is refused before anything is built
    st = so.bsr_create(ctypes.byref(handle), n, k, bs_r, bs_c, nnzb, code, align(data), idx.ctypes.data, ptr.ctypes.data,
                       idx.ctypes.data, ptr.ctypes.data, align(ws), need - 256, None)
    assert st == 7
