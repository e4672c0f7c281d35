"""bsr_spmm_static: the thin-block product on the library's built-in scratch array (no allocation, nothing
lent), through the C ABI, against bsr_spmm_ex on lent scratch (same kernels: bitwise) and against the
oracle; two calls in a row, the second with a smaller input; the documented refusals."""
import ctypes

import numpy as np
import pytest

import workloads as wl
from gpu_util import check, to_device

pytestmark = pytest.mark.gpu

MFMA = 2


def _static_product(so, W, X, m, n):
    import torch
    Y = torch.full((m, n), float("nan"), dtype=torch.float32, device="cuda")
    st = so.bsr_spmm_static(W.handle, m, X.data_ptr(), Y.data_ptr(), 0, torch.cuda.current_stream().cuda_stream)
    assert st == 0, st
    return Y


def test_static_scratch_product_matches_lent_scratch_product(oracle_mod, monkeypatch):
    import torch
    import paper_2007_13055_amd as lib
    so = lib.load_library()
    # bsr_spmm_ex on the matrix-core path would by itself take the one-launch kernel that needs no scratch;
    # variant 1 is the product with the transposed copy of X in lent scratch, whose kernels bsr_spmm_static runs
    monkeypatch.setenv("BSR_SPMM_TUNE", "variant=1")
    # the thin workload at full size (4 MiB + 256 bytes of the 8 MiB array), then a smaller, ragged one
    big = wl.config(4)
    rng = np.random.default_rng(44)
    counts = rng.integers(0, 60, size=23)
    counts[0], counts[5] = 0, 130
    small = wl.make_problem("thin", 70, 130, 23 * 16, 16, 1, "f32", "f32", ("counts", counts), ("uniform", 1.0),
                            ("uniform", 1.0), 45)
    for p in (big, small):
        W = lib.bsr_create(p.n, p.k, p.block_data, p.block_indices, p.index_pointer, dtype="f32")
        X = to_device(p.X, "f32")
        Ys = _static_product(so, W, X, p.m, p.n)
        torch.cuda.synchronize()
        Yl = torch.full((p.m, p.n), float("nan"), dtype=torch.float32, device="cuda")
        lib.bsr_spmm_ex(W, X, Yl, path=MFMA)           # lends scratch through the binding
        torch.cuda.synchronize()
        assert torch.equal(Ys, Yl), f"{p.name} m={p.m}: static and lent scratch differ"
        Yo, So = oracle_mod.bsr_spmm(p.X, p.block_data, p.block_indices, p.index_pointer, p.n)
        check(Ys.double().cpu().numpy(), Yo, So, p.tau, f"static scratch {p.name} m={p.m}")


def test_static_scratch_refusals():
    import torch
    import paper_2007_13055_amd as lib
    so = lib.load_library()
    stream = torch.cuda.current_stream().cuda_stream
    # k = 4096 and m = 1024: 16 MiB of scratch, beyond the built-in 8 MiB -> refused, nothing launched
    counts = np.full(4, 3)
    p = wl.make_problem("thin", 8, 4096, 64, 16, 1, "f32", "f32", ("counts", counts), ("uniform", 1.0), ("uniform", 1.0), 46)
    W = lib.bsr_create(p.n, p.k, p.block_data, p.block_indices, p.index_pointer, dtype="f32")
    assert lib.bsr_scratch_size(W, 1024) > lib.STATIC_SCRATCH_BYTES
    X = torch.zeros((1024, 4096), device="cuda")
    Y = torch.full((1024, 64), 7.0, device="cuda")
    assert so.bsr_spmm_static(W.handle, 1024, X.data_ptr(), Y.data_ptr(), 0, stream) == 10     # BSR_ERR_SCRATCH_LIMIT
    torch.cuda.synchronize()
    assert torch.all(Y == 7.0)
    assert "scratch" in lib.bsr_status_string(10)
    # a block shape whose kernels need no scratch -> unsupported; wrong output type -> unsupported
    q = wl.make_problem("sq", 8, 64, 64, 16, 16, "f16", "f16", ("bernoulli", 0.5), ("normal", 1.0), ("normal", 1.0), 47)
    Wq = lib.bsr_create(q.n, q.k, q.block_data, q.block_indices, q.index_pointer, dtype="f16")
    Xq = to_device(q.X, "f16")
    Yq = torch.zeros((8, 64), dtype=torch.float16, device="cuda")
    assert so.bsr_spmm_static(Wq.handle, 8, Xq.data_ptr(), Yq.data_ptr(), 1, stream) == 9
    assert so.bsr_spmm_static(None, 8, Xq.data_ptr(), Yq.data_ptr(), 1, stream) == 1
