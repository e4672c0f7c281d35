"""The products under HIP-graph replay, as bench.py times them: a graph of several launches is captured once
and replayed several times with the program's own eager work and synchronisations in between; every replay
must reproduce the eager result bit for bit (same kernels, fixed summation order, no atomics)."""
import numpy as np
import pytest

import workloads as wl
from gpu_util import to_device, torch_dtype

pytestmark = pytest.mark.gpu


def _capture(fn, launches=3):
    import torch
    stream = torch.cuda.current_stream()
    fn()                                              # plans, work lists and scratch are set up before the capture
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(stream)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        fn()
        torch.cuda.synchronize()
        with torch.cuda.graph(g, stream=side):
            for _ in range(launches):
                fn()
    torch.cuda.synchronize()
    return g


@pytest.mark.parametrize("cid", [1, 2, 3, 4, 5])
def test_graph_replays_equal_eager(cid):
    import torch
    import paper_2007_13055_amd as lib
    p = wl.config(cid)                                # full size: the kernels and launch shapes bench.py times
    W = lib.bsr_create(p.n, p.k, p.block_data, p.block_indices, p.index_pointer, dtype=p.in_dtype)
    WT = lib.bsr_create_transposed(p.n, p.k, p.block_data, p.block_indices, p.index_pointer, dtype=p.in_dtype)
    X = to_device(p.X, p.in_dtype)
    G = to_device(wl.round_to_storage(np.random.default_rng(cid).normal(size=(p.m, p.n)).astype(np.float32), p.in_dtype), p.in_dtype)
    Y = torch.empty((p.m, p.n), dtype=torch_dtype(p.out_dtype), device="cuda")
    Z = torch.empty((p.m, p.k), dtype=torch_dtype(p.out_dtype), device="cuda")
    D = torch.empty((p.nnzb, p.bs_r, p.bs_c), dtype=torch_dtype(p.out_dtype), device="cuda")

    def step():
        lib.bsr_spmm(W, X, Y, y_dtype=p.out_dtype)
        lib.bsr_spmm(WT, G, Z, y_dtype=p.out_dtype)
        lib.bsr_sddmm(W, G, X, D, d_dtype=p.out_dtype)

    step()
    torch.cuda.synchronize()
    want = [t.clone() for t in (Y, Z, D)]
    g = _capture(step)
    for replay in range(4):
        for t in (Y, Z, D):
            t.fill_(float("nan"))                     # eager work between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for name, t, w in zip("YZD", (Y, Z, D), want):
            assert torch.equal(t, w), f"config {cid}: {name} differs from the eager result on replay {replay}"
        # and an eager product between two replays still gives the same
        Y.fill_(float("nan"))
        lib.bsr_spmm(W, X, Y, y_dtype=p.out_dtype)
        torch.cuda.synchronize()
        assert torch.equal(Y, want[0])
