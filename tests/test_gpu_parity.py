"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Bar: |Y_gpu - Y_oracle| <= tau * sum|x*w| with tau = 1e-5 (fp32 inputs) or 2e-3 (fp16 / bf16 inputs,
fp32 accumulation); exact zeros where the exact result is zero; bitwise equality for integer-valued
inputs.  The oracle's double result is never re-rounded to the output type.
"""
import numpy as np
import pytest

import workloads as wl
from gpu_util import check, gpu_product, to_device

pytestmark = pytest.mark.gpu

WAVE, MFMA = 1, 2


def oracle_of(oracle_mod, p, rows=None):
    return oracle_mod.bsr_spmm(p.X, p.block_data, p.block_indices, p.index_pointer, p.n, rows=rows)


# ------------------------------------------------------------------ both paths, many shapes
SHAPES = [(16, 16), (16, 32), (16, 64), (32, 16), (32, 32), (32, 64), (64, 16), (64, 32), (64, 64)]


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("bs", SHAPES)
def test_mfma_path_block_shapes(oracle_mod, dtype, bs):
    bs_r, bs_c = bs
    for m in (1, 17, 100, 300):                       # single partial tile ... several tiles + ragged tail
        p = wl.make_problem("s", m, 6 * bs_c, 5 * bs_r, bs_r, bs_c, dtype, dtype, ("bernoulli", 0.5),
                            ("normal", 1.0), ("normal", 1.0), 100 + m + bs_r + bs_c)
        Yo, So = oracle_of(oracle_mod, p)
        Yg, W = gpu_product(p, path=MFMA)
        check(Yg, Yo, So, p.tau, f"mfma {dtype} {bs} m={m}", out_dtype=dtype)
        if dtype != "f32":
            # fp32 output: the stated bar alone; and the 16-bit output must be exactly the
            # nearest-even rounding of that fp32 result (same kernel, same summation order)
            Yg32, _ = gpu_product(p, path=MFMA, y_dtype="f32", W=W)
            check(Yg32, Yo, So, p.tau, f"mfma {dtype}->f32 {bs} m={m}")
            assert np.array_equal(wl.round_to_storage(Yg32.astype(np.float32), dtype).astype(np.float64), Yg)


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("bs", [(16, 16), (8, 8), (16, 1), (1, 16), (3, 5), (32, 32), (64, 64), (1, 1), (4, 8)])
def test_wave_path_block_shapes(oracle_mod, dtype, bs):
    bs_r, bs_c = bs
    for m in (1, 3, 8, 21):
        p = wl.make_problem("s", m, 12 * bs_c, 7 * bs_r, bs_r, bs_c, dtype, dtype, ("bernoulli", 0.5),
                            ("normal", 1.0), ("normal", 1.0), 200 + m + bs_r + bs_c)
        Yo, So = oracle_of(oracle_mod, p)
        Yg, W = gpu_product(p, path=WAVE)
        check(Yg, Yo, So, p.tau, f"wave {dtype} {bs} m={m}", out_dtype=dtype)
        if dtype != "f32":
            Yg32, _ = gpu_product(p, path=WAVE, y_dtype="f32", W=W)
            check(Yg32, Yo, So, p.tau, f"wave {dtype}->f32 {bs} m={m}")
            assert np.array_equal(wl.round_to_storage(Yg32.astype(np.float32), dtype).astype(np.float64), Yg)


@pytest.mark.parametrize("rows", [0, 1, 2, 4, 8])
@pytest.mark.parametrize("dtype,bs", [("f32", (8, 8)), ("f32", (16, 2)), ("f16", (4, 8)), ("bf16", (32, 32))])
def test_wave_path_rows_per_wavefront_and_long_rows(oracle_mod, monkeypatch, rows, dtype, bs):
    """The wave path at every rows-per-wavefront setting (mt), with 16-byte and single-element loads, a
    block-row longer than a row descriptor's inline block-columns (40 > 28), and empty block-rows."""
    if rows:
        monkeypatch.setenv("BSR_SPMM_TUNE", f"mt={rows}")
    bs_r, bs_c = bs
    counts = np.array([0, 40, 1, 29, 0, 28, 7])
    for m in (1, 5, 8, 13):
        p = wl.make_problem("wl", m, 40 * bs_c, counts.shape[0] * bs_r, bs_r, bs_c, dtype, dtype, ("counts", counts),
                            ("normal", 1.0), ("normal", 1.0), 700 + m + bs_r)
        Yo, So = oracle_of(oracle_mod, p)
        Yg, _ = gpu_product(p, path=WAVE)
        check(Yg, Yo, So, p.tau, f"wave rows={rows} {dtype} {bs} m={m}", out_dtype=dtype)


# ------------------------------------------------------------------ the five configurations, full size
@pytest.mark.parametrize("cid", [1, 2, 3, 4])
def test_config_full_size_auto_path(oracle_mod, cid):
    p = wl.config(cid)
    Yo, So = oracle_of(oracle_mod, p)
    Yg, W = gpu_product(p)
    check(Yg, Yo, So, p.tau, f"config {cid} auto", out_dtype=p.out_dtype)
    if p.out_dtype != "f32":
        # the stated bar alone on the fp32 accumulator; the 16-bit Y is its nearest-even rounding
        Yg32, _ = gpu_product(p, y_dtype="f32", W=W)
        check(Yg32, Yo, So, p.tau, f"config {cid} auto, fp32 output")
        assert np.array_equal(wl.round_to_storage(Yg32.astype(np.float32), p.out_dtype).astype(np.float64), Yg)


@pytest.mark.parametrize("cid", [1, 2, 4])
def test_config_full_size_wave_path(oracle_mod, cid):
    p = wl.config(cid)
    Yo, So = oracle_of(oracle_mod, p)
    Yg, _ = gpu_product(p, path=WAVE)
    check(Yg, Yo, So, p.tau, f"config {cid} wave")


def _config5_rows(m, seed):
    """Rows of X the oracle computes for configuration 5: one seeded row out of every 32 consecutive rows (so
    every wavefront's slice of every m-tile of every kernel that may take the product is compared, 256 rows),
    plus tile edges and the first and last rows."""
    rng = np.random.default_rng(seed)
    per_slice = (np.arange(0, m, 32) + rng.integers(0, 32, size=(m + 31) // 32)).clip(max=m - 1)
    edges = [0, 1, 31, 32, 63, 64, 127, 128, 255, 256, 4095, 4096, m - 2, m - 1]
    return sorted(set(per_slice.tolist() + edges))


def test_config5_full_size_sampled_rows(oracle_mod):
    """8192 x 8192 x 8192 fp16: the GPU computes everything, the oracle the sampled rows (one in every
    32-row slice, tile edges, first / last rows)."""
    p = wl.config(5)
    rows = _config5_rows(p.m, 5)
    assert all(any(32 * s <= r < 32 * s + 32 for r in rows) for s in range(p.m // 32))
    Yo, So = oracle_of(oracle_mod, p, rows=rows)
    Yg, W = gpu_product(p, rows=rows)
    check(Yg, Yo, So, p.tau, "config 5 sampled rows", out_dtype=p.out_dtype)
    Yg32, _ = gpu_product(p, rows=rows, y_dtype="f32", W=W)
    check(Yg32, Yo, So, p.tau, "config 5 sampled rows, fp32 output")
    assert np.array_equal(wl.round_to_storage(Yg32.astype(np.float32), "f16").astype(np.float64), Yg)


# ------------------------------------------------------------------ the sibling products at full size
def _gradient_like(p, seed):
    """A seeded G (m, n) of the workload's input type: what a layer's backward pass hands to the siblings."""
    g = np.random.default_rng(seed).normal(size=(p.m, p.n)).astype(np.float32)
    return wl.round_to_storage(g, p.in_dtype)


@pytest.mark.parametrize("cid", [1, 2, 3, 4, 5])
def test_config_full_size_sampled_product(oracle_mod, cid):
    """D = (G^T X) at the stored blocks on the five configurations at full size, launched as bench.py
    launches it.  The GPU computes every block; the oracle every block (1-4) or, for configuration 5, a
    sample of blocks: first, last, some of the longest block-row, one of every block-row, a seeded random set."""
    import torch
    import paper_2007_13055_amd as lib
    p = wl.config(cid)
    G = _gradient_like(p, 900 + cid)
    W = lib.bsr_create(p.n, p.k, p.block_data, p.block_indices, p.index_pointer, dtype=p.in_dtype)
    Gd, Xd = to_device(G, p.in_dtype), to_device(p.X, p.in_dtype)
    D = lib.bsr_sddmm(W, Gd, Xd, d_dtype=p.out_dtype)
    D32 = lib.bsr_sddmm(W, Gd, Xd, d_dtype="f32")
    torch.cuda.synchronize()
    if cid < 5:
        pick = np.arange(p.nnzb)
        idx, ptr = p.block_indices, p.index_pointer
    else:
        counts = np.diff(p.index_pointer)
        longest = int(np.argmax(counts))
        a = int(p.index_pointer[longest])
        rng = np.random.default_rng(5)
        starts = p.index_pointer[:-1][counts > 0]
        per_row = starts + (rng.random(starts.shape[0]) * counts[counts > 0]).astype(np.int64)   # one block of every block-row
        pick = np.unique(np.concatenate([[0, p.nnzb - 1], a + np.array([0, 1, 2, 63, 64, int(counts[longest]) - 1]),
                                         per_row, rng.integers(0, p.nnzb, size=40)]))
        rows = np.repeat(np.arange(p.n // p.bs_r), counts)[pick]
        idx = p.block_indices[pick]
        ptr = np.concatenate([[0], np.cumsum(np.bincount(rows, minlength=p.n // p.bs_r))]).astype(np.int32)
    Do, So = oracle_mod.bsr_sddmm(G, p.X, idx, ptr, p.bs_r, p.bs_c)
    sel = torch.as_tensor(pick, device="cuda")
    flat = lambda t: t[sel].double().cpu().numpy().reshape(len(pick), -1)
    check(flat(D32), Do.reshape(len(pick), -1), So.reshape(len(pick), -1), p.tau, f"config {cid} sampled product, fp32 output")
    check(flat(D), Do.reshape(len(pick), -1), So.reshape(len(pick), -1), p.tau, f"config {cid} sampled product",
          out_dtype=p.out_dtype)


@pytest.mark.parametrize("cid", [1, 2, 3, 4, 5])
def test_config_full_size_transposed_sibling(oracle_mod, cid):
    """Z = G * W through the handle of W^T on the five configurations at full size; configuration 5 against
    the oracle on sampled rows of G, one in every 32-row slice (a row of Z depends on that row of G only)."""
    import torch
    import paper_2007_13055_amd as lib
    p = wl.config(cid)
    G = _gradient_like(p, 950 + cid)
    WT = lib.bsr_create_transposed(p.n, p.k, p.block_data, p.block_indices, p.index_pointer, dtype=p.in_dtype)
    Z = lib.bsr_spmm(WT, to_device(G, p.in_dtype), y_dtype=p.out_dtype)
    torch.cuda.synchronize()
    rows = np.arange(p.m) if cid < 5 else np.array(_config5_rows(p.m, 6))
    Zo, So = oracle_mod.bsr_spmm_w(G[rows], p.block_data, p.block_indices, p.index_pointer, p.k)
    Zg = Z[torch.as_tensor(rows, device="cuda")].double().cpu().numpy()
    check(Zg, Zo, So, p.tau, f"config {cid} transposed sibling", out_dtype=p.out_dtype)


# ------------------------------------------------------------------ exact cases
@pytest.mark.parametrize("path", [WAVE, MFMA])
@pytest.mark.parametrize("dtype,out", [("f32", "f32"), ("f16", "f32"), ("bf16", "f32"), ("f16", "f16")])
def test_small_integers_are_bitwise_exact(oracle_mod, path, dtype, out):
    """|values| <= 4 and short sums: every partial sum is an exactly representable integer, so any
    summation order must give the oracle's value bit for bit (also after fp16 rounding: |y| < 2048)."""
    p = wl.small_integer_problem(70, 8 * 16, 6 * 16, 16, 16, 0.5, seed=11, in_dtype=dtype, out_dtype=out,
                                 lo=-3, hi=3)
    Yo, So = oracle_of(oracle_mod, p)
    assert np.abs(Yo).max() < 2048
    Yg, _ = gpu_product(p, path=path)
    assert np.array_equal(Yg, Yo)


@pytest.mark.parametrize("path", [WAVE, MFMA])
def test_all_ones_closed_form(path):
    """X = 1, stored blocks = 1  =>  Y[i, r*bs_r + a] = bs_c * (stored blocks of block-row r)."""
    bs_r, bs_c, R, C, m = 32, 32, 9, 10, 40
    rng = np.random.default_rng(1)
    counts = rng.integers(0, C + 1, size=R)
    counts[3] = 0
    ptr, idx = wl.pattern_from_counts(rng, counts, C)
    p = wl.Problem("ones", m, C * bs_c, R * bs_r, bs_r, bs_c, "f32", "f32", np.ones((m, C * bs_c), np.float32),
                   np.ones((idx.shape[0], bs_r, bs_c), np.float32), idx, ptr)
    Yg, _ = gpu_product(p, path=path)
    assert np.array_equal(Yg, np.tile(np.repeat(counts * bs_c, bs_r).astype(np.float64), (m, 1)))


@pytest.mark.parametrize("path", [WAVE, MFMA])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_block_diagonal_identity_returns_x(path, dtype):
    bs, R, m = 16, 6, 37
    X = wl.round_to_storage(np.random.default_rng(3).normal(size=(m, R * bs)).astype(np.float32), dtype)
    p = wl.Problem("eye", m, R * bs, R * bs, bs, bs, dtype, dtype, X,
                   np.tile(np.eye(bs, dtype=np.float32), (R, 1, 1)), np.arange(R, dtype=np.int32),
                   np.arange(R + 1, dtype=np.int32))
    Yg, _ = gpu_product(p, path=path)
    assert np.array_equal(Yg, X.astype(np.float64))


@pytest.mark.parametrize("path", [WAVE, MFMA])
def test_single_one_selects_a_column(path):
    bs_r, bs_c, R, C, m = 16, 32, 4, 5, 19
    X = np.random.default_rng(2).normal(size=(m, C * bs_c)).astype(np.float32)
    for (r, cb, a, c) in [(0, 0, 0, 0), (2, 4, bs_r - 1, bs_c - 1), (3, 1, 7, 13)]:
        blk = np.zeros((1, bs_r, bs_c), np.float32)
        blk[0, a, c] = 1.0
        ptr = np.zeros(R + 1, np.int32)
        ptr[r + 1:] = 1
        p = wl.Problem("sel", m, C * bs_c, R * bs_r, bs_r, bs_c, "f32", "f32", X, blk,
                       np.array([cb], np.int32), ptr)
        Yg, _ = gpu_product(p, path=path)
        expect = np.zeros((m, R * bs_r))
        expect[:, r * bs_r + a] = X[:, cb * bs_c + c]
        assert np.array_equal(Yg, expect)


@pytest.mark.parametrize("path", [WAVE, MFMA])
def test_empty_rows_overwrite_with_exact_zero(oracle_mod, path):
    """Y is pre-filled with NaN: every element must be overwritten, empty block-rows with +0."""
    m, bs = 45, 16
    for counts in ([0, 3, 0, 0, 2, 0], [0] * 6, [4, 0, 0, 0, 0, 1]):
        p = wl.make_problem("e", m, 8 * bs, 6 * bs, bs, bs, "f32", "f32", ("counts", np.array(counts)),
                            ("normal", 1.0), ("normal", 1.0), 5)
        Yo, So = oracle_of(oracle_mod, p)
        Yg, _ = gpu_product(p, path=path)
        check(Yg, Yo, So, p.tau, f"empty rows {counts}")
        for r, cnt in enumerate(counts):
            if cnt == 0:
                assert np.all(Yg[:, r * bs:(r + 1) * bs] == 0)


@pytest.mark.parametrize("path", [WAVE, MFMA])
def test_unsorted_and_duplicate_blocks(oracle_mod, path):
    p = wl.small_integer_problem(33, 8 * 16, 5 * 16, 16, 16, 0.6, seed=3)
    rng = np.random.default_rng(9)
    data, idx = p.block_data.copy(), p.block_indices.copy()
    for r in range(p.n // p.bs_r):
        a, b = p.index_pointer[r], p.index_pointer[r + 1]
        perm = rng.permutation(b - a) + a
        data[a:b], idx[a:b] = p.block_data[perm], p.block_indices[perm]
    q = wl.Problem("perm", p.m, p.k, p.n, 16, 16, "f32", "f32", p.X, data, idx, p.index_pointer)
    Y0, _ = gpu_product(p, path=path)
    Y1, _ = gpu_product(q, path=path)
    assert np.array_equal(Y0, Y1)                     # integer-valued: exact under permutation
    # duplicates: the same block stored twice counts twice
    d2 = np.concatenate([p.block_data[:1], p.block_data])
    i2 = np.concatenate([p.block_indices[:1], p.block_indices])
    ptr2 = p.index_pointer.copy()
    ptr2[1:] += 1
    dup = wl.Problem("dup", p.m, p.k, p.n, 16, 16, "f32", "f32", p.X, d2, i2, ptr2)
    Yo, So = oracle_of(oracle_mod, dup)
    Yg, _ = gpu_product(dup, path=path)
    assert np.array_equal(Yg, Yo)


# ------------------------------------------------------------------ paper grid (m = 1, 8)
@pytest.mark.parametrize("cell", [(1, 128, 768, 8, 0.8), (8, 128, 768, 16, 0.95), (8, 128, 768, 32, 0.85),
                                  (1, 1024, 1024, 16, 0.85), (8, 1024, 1024, 8, 0.95),
                                  (8, 1024, 1024, 32, 0.8)])
def test_paper_grid_cells(oracle_mod, cell):
    p = wl.paper_grid_problem(*cell)
    Yo, So = oracle_of(oracle_mod, p)
    Yg, _ = gpu_product(p)
    check(Yg, Yo, So, p.tau, f"paper grid {cell}")


# ------------------------------------------------------------------ boundary behaviour
def test_degenerate_sizes_and_errors():
    import torch
    import paper_2007_13055_amd as lib
    W = lib.bsr_create(32, 32, np.zeros((0, 16, 16), np.float32), [], [0, 0, 0])
    X = torch.ones((5, 32), device="cuda")
    Y = lib.bsr_spmm(W, X)
    torch.cuda.synchronize()
    assert torch.all(Y == 0)
    Y0 = lib.bsr_spmm(W, torch.ones((0, 32), device="cuda"))         # m = 0: no device work
    assert tuple(Y0.shape) == (0, 32)
    p = wl.make_problem("t", 4, 15, 20, 5, 3, "f32", "f32", ("bernoulli", 0.5), ("normal", 1), ("normal", 1), 1)
    Wodd = lib.bsr_create(p.n, p.k, p.block_data, p.block_indices, p.index_pointer)
    assert lib.bsr_query_path(Wodd, 64) == WAVE
    with pytest.raises(lib.BsrError) as e:
        lib.bsr_spmm_ex(Wodd, to_device(p.X, "f32"), path=MFMA)
    assert e.value.status == 9
    with pytest.raises(lib.BsrError) as e:                           # misaligned X
        buf = torch.zeros(4 * 15 + 1, device="cuda")
        lib.bsr_spmm(Wodd, buf[1:].view(4, 15))
    assert e.value.status == 6



def test_products_on_other_streams_than_create(oracle_mod):
    """The handle is created on one stream and used at once on two others with two different m (two work-item
    tables of the k-split kernel in flight): the products wait on the device for the plan upload and for each
    other's table upload."""
    import torch
    import paper_2007_13055_amd as lib
    rng = np.random.default_rng(78)
    R, C, bs = 40, 24, 32
    counts = rng.integers(0, 21, size=R)
    ps = [wl.make_problem("st", m, C * bs, R * bs, bs, bs, "f32", "f32", ("counts", counts), ("normal", 1.0),
                          ("normal", 1.0), 601) for m in (330, 1000)]
    sa, sb, sc = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    Xs = [to_device(p.X, "f32") for p in ps]
    torch.cuda.synchronize()
    with torch.cuda.stream(sa):
        W = lib.bsr_create(ps[0].n, ps[0].k, ps[0].block_data, ps[0].block_indices, ps[0].index_pointer, dtype="f32")
    Ys = []
    for rep in range(2):                                  # second round: the tables are cached
        for p, X, s in zip(ps, Xs, (sb, sc)):
            with torch.cuda.stream(s):
                Ys.append(lib.bsr_spmm(W, X))
    torch.cuda.synchronize()
    for i, Y in enumerate(Ys):
        p = ps[i % 2]
        Yo, So = oracle_of(oracle_mod, p)
        check(Y.double().cpu().numpy(), Yo, So, p.tau, f"streams, m={p.m}, round {i // 2}")


def test_no_reduction_dimension():
    """k = 0 (hence nothing stored), n > 0, many rows, 16x16 bf16 blocks: every kernel family stores zeros."""
    import torch
    import paper_2007_13055_amd as lib
    W = lib.bsr_create(64, 0, np.zeros((0, 16, 16), np.float32), [], [0, 0, 0, 0, 0], dtype="bf16")
    for m in (300, 5):
        X = torch.zeros((m, 0), dtype=torch.bfloat16, device="cuda")
        for path in (0, WAVE, MFMA):
            Y = torch.full((m, 64), float("nan"), dtype=torch.bfloat16, device="cuda")
            lib.bsr_spmm_ex(W, X, Y, path=path)
            torch.cuda.synchronize()
            assert torch.all(Y == 0), (m, path)


def test_sampled_product_degenerate_sizes_and_errors():
    """bsr_sddmm's documented codes: nothing stored, m = 0 (an empty sum: zeros), NULL, negative m, an output
    type that is neither the input type nor fp32, a misaligned pointer."""
    import torch
    import paper_2007_13055_amd as lib
    so = lib.load_library()
    stream = torch.cuda.current_stream().cuda_stream
    W0 = lib.bsr_create(32, 32, np.zeros((0, 16, 16), np.float32), [], [0, 0, 0])
    G, X = torch.ones((5, 32), device="cuda"), torch.ones((5, 32), device="cuda")
    assert tuple(lib.bsr_sddmm(W0, G, X).shape) == (0, 16, 16)
    for bs in ((16, 16), (16, 1), (3, 5)):                            # matrix-core, lane-per-column, plain loop
        p = wl.make_problem("t", 4, 6 * bs[1], 5 * bs[0], bs[0], bs[1], "f32", "f32", ("bernoulli", 0.6), ("normal", 1),
                            ("normal", 1), 2)
        W = lib.bsr_create(p.n, p.k, p.block_data, p.block_indices, p.index_pointer)
        D = torch.full((p.nnzb, bs[0], bs[1]), float("nan"), device="cuda")
        lib.bsr_sddmm(W, torch.ones((0, p.n), device="cuda"), torch.ones((0, p.k), device="cuda"), D)
        torch.cuda.synchronize()
        assert torch.all(D == 0), bs                                  # m = 0: every element written, an empty sum
    G, X = to_device(np.ones((4, p.n), np.float32), "f32"), to_device(p.X, "f32")
    D = torch.empty((p.nnzb, 3, 5), device="cuda")
    args = lambda **kw: [kw.get("W", W.handle), kw.get("m", 4), kw.get("G", G.data_ptr()), kw.get("X", X.data_ptr()),
                         kw.get("D", D.data_ptr()), kw.get("t", 0), stream]
    assert so.bsr_sddmm(*args()) == 0
    assert so.bsr_sddmm(*args(W=None)) == 1                           # NULL handle
    assert so.bsr_sddmm(*args(D=None)) == 1
    assert so.bsr_sddmm(*args(G=None)) == 1
    assert so.bsr_sddmm(*args(m=-1)) == 2
    assert so.bsr_sddmm(*args(t=1)) == 5                              # fp16 output of an fp32 W
    assert so.bsr_sddmm(*args(X=X.data_ptr() + 4)) == 6
    torch.cuda.synchronize()


def test_repeat_calls_are_bitwise_identical(oracle_mod):
    """No atomics in the default plan: two runs must agree bit for bit (catches races)."""
    p = wl.config(2)
    Y1, W = gpu_product(p)
    Y2, _ = gpu_product(p, W=W)
    assert np.array_equal(Y1, Y2)


# ------------------------------------------------------------------ every matrix-core kernel variant
# BSR_SPMM_TUNE is the library's development knob; "variant" pins the matrix-core kernel:
# 1 direct (operands from global memory), 2 k-split (few rows of X; mt=1 / mt=2: 16- / 32-row tiles,
# nw wavefronts, a blocks per wavefront), 3 LDS-staged tiles (many rows).
@pytest.mark.parametrize("variant,extra", [(1, ""), (1, ",mt=2,nw=4"), (2, ""), (2, ",nw=3,a=1"), (2, ",mt=1"),
                                           (2, ",mt=2,nw=8"), (2, ",mt=1,nw=2,a=1"), (2, ",mt=2,a=3"),
                                           (3, ",mt=1,a=1"), (3, ",mt=1,a=3"), (3, ",mt=2,a=2"), (3, ",mt=1,a=2,b=3")])
@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
def test_mfma_kernel_variants(oracle_mod, monkeypatch, variant, extra, dtype):
    monkeypatch.setenv("BSR_SPMM_TUNE", f"variant={variant}{extra}")
    shapes = [(32, 32), (64, 64), (32, 64), (64, 16)] if variant == 3 else [(16, 16), (32, 32), (64, 64), (16, 64)]
    for (bs_r, bs_c) in shapes:
        for m in (5, 130, 700):                       # partial tile, two tiles, several tiles + ragged tail
            counts = np.array([0, 1, 2, 3, 40, 5, 0, 17, 9])      # empty rows, short rows, one long row
            counts = np.minimum(counts, 40)
            p = wl.make_problem("v", m, 40 * bs_c, counts.shape[0] * bs_r, bs_r, bs_c, dtype, dtype,
                                ("counts", counts), ("normal", 1.0), ("normal", 1.0), 300 + m + bs_r + bs_c)
            Yo, So = oracle_of(oracle_mod, p)
            Yg, W = gpu_product(p, path=MFMA)
            check(Yg, Yo, So, p.tau, f"variant {variant}{extra} {dtype} {bs_r}x{bs_c} m={m}", out_dtype=dtype)
            Yg2, _ = gpu_product(p, path=MFMA, W=W)
            assert np.array_equal(Yg, Yg2), "two runs differ: race"


@pytest.mark.parametrize("tile_rows", [1, 2])
@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("bs", SHAPES)
def test_ksplit_kernel_every_shape_both_tile_heights(oracle_mod, monkeypatch, tile_rows, dtype, bs):
    """variant 2 for every supported block shape and type at 16-row (mt=1) and 32-row (mt=2) tiles: one
    block-row longer than a descriptor's inline block-columns, one empty, a ragged last m-tile."""
    monkeypatch.setenv("BSR_SPMM_TUNE", f"variant=2,mt={tile_rows}")
    bs_r, bs_c = bs
    counts = np.array([3, 0, 31, 8, 1])
    p = wl.make_problem("ks", 45, 32 * bs_c, counts.shape[0] * bs_r, bs_r, bs_c, dtype, dtype, ("counts", counts),
                        ("normal", 1.0), ("normal", 1.0), 800 + bs_r + bs_c)
    Yo, So = oracle_of(oracle_mod, p)
    Yg, W = gpu_product(p, path=MFMA)
    check(Yg, Yo, So, p.tau, f"k-split mt={tile_rows} {dtype} {bs}", out_dtype=dtype)
    Yg2, _ = gpu_product(p, path=MFMA, W=W)
    assert np.array_equal(Yg, Yg2), "two runs differ: race"


def test_tile_kernel_small_integers_bitwise(oracle_mod, monkeypatch):
    monkeypatch.setenv("BSR_SPMM_TUNE", "variant=3,mt=1,a=2")
    p = wl.small_integer_problem(600, 16 * 64, 6 * 64, 64, 64, 0.5, seed=21, in_dtype="f16", out_dtype="f32", lo=-2, hi=2)
    Yo, So = oracle_of(oracle_mod, p)
    Yg, _ = gpu_product(p, path=MFMA)
    assert np.array_equal(Yg, Yo)


@pytest.mark.parametrize("extra", ["", ",mt=1", ",mt=2,a=3", ",mt=4,a=1", ",mt=4,a=7"])
@pytest.mark.parametrize("dtype,out", [("bf16", "bf16"), ("f16", "f16"), ("bf16", "f32")])
def test_stripe_kernel_variant(oracle_mod, monkeypatch, extra, dtype, out):
    """variant 4: 16x16 blocks of a 16-bit type, the X stripe staged in LDS (the 'batched' regime)."""
    monkeypatch.setenv("BSR_SPMM_TUNE", "variant=4" + extra)
    for m, R, C in ((5, 3, 4), (70, 9, 12), (300, 50, 48), (129, 13, 7)):
        rng = np.random.default_rng(m + R)
        counts = rng.integers(0, min(C, 21) + 1, size=R)
        counts[0] = 0
        counts[R // 2] = min(C, 19)                    # an odd count, longer than one chunk of 8 pairs
        counts[-1] = 1
        p = wl.make_problem("st", m, C * 16, R * 16, 16, 16, dtype, out, ("counts", counts), ("normal", 1.0),
                            ("normal", 1.0), 400 + m)
        Yo, So = oracle_of(oracle_mod, p)
        Yg, W = gpu_product(p, path=MFMA)
        check(Yg, Yo, So, p.tau, f"stripe{extra} {dtype}->{out} m={m} R={R} C={C}", out_dtype=out)
        Yg2, _ = gpu_product(p, path=MFMA, W=W)
        assert np.array_equal(Yg, Yg2), "two runs differ: race"


# ------------------------------------------------------------------ the row-group kernel (variant 5)
@pytest.mark.parametrize("extra", ["", ",b=1", ",b=3", ",b=1,nw=1"])
@pytest.mark.parametrize("dtype,out", [("f16", "f16"), ("bf16", "bf16"), ("f16", "f32"), ("bf16", "f32")])
def test_group_kernel_variant(oracle_mod, monkeypatch, extra, dtype, out):
    """variant 5: 64x64 blocks of a 16-bit type; the longest block-rows in groups of up to 8 wavefronts (a row on
    one, or cut into shares for several whose results are added) that walk the union of their block-columns,
    the other block-rows through the tile kernel.  Long, short, single-block and empty
    block-rows, more long rows than the groups hold, block-columns with 1 to 8 blocks, ragged m; b = fewest
    blocks of a grouped row (default 8), nw = groups at most."""
    monkeypatch.setenv("BSR_SPMM_TUNE", "variant=5" + extra)
    cases = [(5, np.array([3, 0, 9, 1])),
             (64, np.array([12, 12, 11, 12, 10, 12, 12, 9, 1, 0, 2])),            # a heavy group with full steps
             (130, np.array([0, 1, 2, 3, 20, 5, 0, 17, 9, 1, 1, 1, 1, 1, 1, 1, 1, 1, 4])),
             (700, np.array([20, 18, 1, 0, 0, 7, 3, 3, 2, 1, 1, 15, 6])),
             (200, np.array([19, 16, 1, 0]))]                                     # two long rows cut into shares for 8 wavefronts
    for m, counts in cases:
        C = 20
        p = wl.make_problem("grp", m, C * 64, counts.shape[0] * 64, 64, 64, dtype, out, ("counts", counts),
                            ("normal", 1.0), ("normal", 1.0), 1300 + m)
        Yo, So = oracle_of(oracle_mod, p)
        Yg, W = gpu_product(p, path=MFMA)
        check(Yg, Yo, So, p.tau, f"group{extra} {dtype}->{out} m={m}", out_dtype=out)
        Yg2, _ = gpu_product(p, path=MFMA, W=W)
        assert np.array_equal(Yg, Yg2), "two runs differ: race"


def test_group_kernel_small_integers_bitwise_duplicates_and_order(oracle_mod, monkeypatch):
    """Exact data (any summation order gives the oracle's value bit for bit), with unsorted block-columns and a
    block-column stored twice in one block-row (two steps of the same column)."""
    monkeypatch.setenv("BSR_SPMM_TUNE", "variant=5,b=1")
    p = wl.small_integer_problem(333, 12 * 64, 11 * 64, 64, 64, 0.5, seed=23, in_dtype="f16", out_dtype="f32", lo=-2, hi=2)
    Yo, So = oracle_of(oracle_mod, p)
    Yg, _ = gpu_product(p, path=MFMA)
    assert np.array_equal(Yg, Yo)
    rng = np.random.default_rng(24)
    ptr = np.array([0, 4, 4, 7, 8], dtype=np.int32)
    idx = np.array([2, 0, 2, 1, 3, 3, 0, 1], dtype=np.int32)                  # row 0: column 2 twice, unsorted; row 2: column 3 twice
    data = rng.integers(-2, 3, size=(8, 64, 64)).astype(np.float32)
    X = rng.integers(-2, 3, size=(70, 4 * 64)).astype(np.float32)
    q = wl.Problem("dup", 70, 4 * 64, 4 * 64, 64, 64, "bf16", "f32", X, data, idx, ptr)
    Yo, So = oracle_of(oracle_mod, q)
    Yg, _ = gpu_product(q, path=MFMA)
    assert np.array_equal(Yg, Yo)


def test_group_kernel_config5_sampled_rows(oracle_mod, monkeypatch):
    """The row-group kernel on the 8192^3 workload at full size, whatever the default choice is."""
    monkeypatch.setenv("BSR_SPMM_TUNE", "variant=5")
    p = wl.config(5)
    rows = _config5_rows(p.m, 7)
    Yo, So = oracle_of(oracle_mod, p, rows=rows)
    Yg, W = gpu_product(p, rows=rows)
    check(Yg, Yo, So, p.tau, "config 5, row-group kernel", out_dtype=p.out_dtype)
    Yg32, _ = gpu_product(p, rows=rows, y_dtype="f32", W=W)
    check(Yg32, Yo, So, p.tau, "config 5, row-group kernel, fp32 output")
    assert np.array_equal(wl.round_to_storage(Yg32.astype(np.float32), "f16").astype(np.float64), Yg)


@pytest.mark.parametrize("u", ["", "a=1", "a=16", "a=24", "auto"])
def test_thin_rows_staged_in_lds(oracle_mod, monkeypatch, u):
    """16x1 fp32 blocks on the matrix-core path in one launch: rows of X staged in LDS 1024 columns at a time,
    the gather of columns done there (a = MFMAs of a phase whose operands sit in registers: 8, 16 or 24).  One to
    five phases, a last phase that is not full, block-rows with none, one, and more blocks in a phase than the
    registers hold (extra passes), ragged m, fewer block-rows than a workgroup takes; no scratch is lent."""
    import torch
    import paper_2007_13055_amd as lib
    path = MFMA
    if u == "auto":
        path = 0                                                   # no knob, nothing lent: the library's own choice
    else:
        monkeypatch.setenv("BSR_SPMM_TUNE", "variant=2" + ("," + u if u else ""))
    for m, R, C in ((16, 3, 40), (70, 9, 132), (257, 20, 300), (64, 5, 8), (600, 11, 64), (48, 10, 2500), (33, 70, 4096),
                    (17, 4, 5000)):
        rng = np.random.default_rng(m + R)
        counts = rng.integers(0, min(C, 400) + 1, size=R)
        counts[0] = 0
        counts[-1] = min(C, 377)
        counts[R // 2] = 1
        p = wl.make_problem("thin", m, C, R * 16, 16, 1, "f32", "f32", ("counts", counts), ("uniform", 1.0),
                            ("uniform", 1.0), 700 + m)
        Yo, So = oracle_of(oracle_mod, p)
        W = lib.bsr_create(p.n, p.k, p.block_data, p.block_indices, p.index_pointer, dtype="f32")
        assert lib.bsr_query_path(W, m) == MFMA                    # without any scratch
        assert lib.bsr_query_path(W, 8) == WAVE
        X = to_device(p.X, "f32")
        Y = torch.full((m, p.n), float("nan"), device="cuda")
        st = lib.load_library().bsr_spmm_ex(W.handle, m, X.data_ptr(), Y.data_ptr(), 0, path,
                                            torch.cuda.current_stream().cuda_stream)
        assert st == 0
        torch.cuda.synchronize()
        Yg = Y.double().cpu().numpy()
        check(Yg, Yo, So, p.tau, f"thin rows-in-LDS {u} m={m} R={R} C={C}")
        Y.fill_(float("nan"))
        st = lib.load_library().bsr_spmm_ex(W.handle, m, X.data_ptr(), Y.data_ptr(), 0, path,
                                            torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        assert st == 0 and np.array_equal(Y.double().cpu().numpy(), Yg), "two runs differ: race"


def test_thin_rows_staged_in_lds_bitwise_and_fallback(oracle_mod):
    """Exact data: the one-launch thin kernel gives the oracle's value bit for bit (duplicates of a block-column
    included: they keep non-decreasing order).  A block-row stored out of order makes the plan leave the
    kernel out: the product then needs the scratch again and still matches."""
    import paper_2007_13055_amd as lib
    p = wl.small_integer_problem(100, 2048 + 64, 9 * 16, 16, 1, 0.3, seed=31)
    Yo, So = oracle_of(oracle_mod, p)
    Yg, W = gpu_product(p, path=MFMA)
    assert np.array_equal(Yg, Yo)
    rng = np.random.default_rng(32)
    ptr = np.array([0, 5, 5, 9], dtype=np.int32)
    idx = np.array([1, 1, 3, 3, 7, 0, 2, 2, 6], dtype=np.int32)
    data = rng.integers(-3, 4, size=(9, 16, 1)).astype(np.float32)
    X = rng.integers(-3, 4, size=(40, 8)).astype(np.float32)
    q = wl.Problem("dup", 40, 8, 48, 16, 1, "f32", "f32", X, data, idx, ptr)
    Yo, So = oracle_of(oracle_mod, q)
    Yg, Wq = gpu_product(q, path=MFMA)
    assert np.array_equal(Yg, Yo)
    idx2 = idx.copy(); idx2[[0, 4]] = idx2[[4, 0]]; data2 = data.copy(); data2[[0, 4]] = data2[[4, 0]]   # same matrix, row 0 out of order
    q2 = wl.Problem("unsorted", 40, 8, 48, 16, 1, "f32", "f32", X, data2, idx2, ptr)
    W2 = lib.bsr_create(q2.n, q2.k, q2.block_data, q2.block_indices, q2.index_pointer, dtype="f32")
    assert lib.bsr_query_path(W2, 40) == WAVE                      # no scratch lent, kernel not available
    Yg2, _ = gpu_product(q2, path=MFMA, W=W2)                      # the binding lends the scratch
    assert np.array_equal(Yg2, Yo)


def test_wide_blocks_by_block_column(oracle_mod):
    """1x16 fp32 blocks (a thin W transposed) on the matrix-core path: products by block-column, partial sums in
    LDS.  Ragged m, n not a multiple of 4 or of the 256-column range, empty block-rows and block-columns, runs of
    more than 16 blocks in a range, fewer block-columns than wavefronts, more than 512 of them (several batches of
    runs), run-to-run bitwise equality, exact data, and a block stored twice (left to the other kernels)."""
    import torch
    import paper_2007_13055_amd as lib
    for m, R, C in ((16, 40, 3), (70, 1000, 9), (257, 515, 40), (33, 4096, 64), (48, 300, 530), (600, 77, 12)):
        rng = np.random.default_rng(3 * m + R)
        counts = rng.integers(0, min(C, 30) + 1, size=R)
        counts[0] = 0
        counts[R // 2] = C
        p = wl.make_problem("wide", m, C * 16, R, 1, 16, "f32", "f32", ("counts", counts), ("uniform", 1.0),
                            ("uniform", 1.0), 900 + m)
        Yo, So = oracle_of(oracle_mod, p)
        W = lib.bsr_create(p.n, p.k, p.block_data, p.block_indices, p.index_pointer, dtype="f32")
        assert lib.bsr_query_path(W, m) == MFMA and lib.bsr_query_path(W, 8) == WAVE
        Yg, _ = gpu_product(p, path=MFMA, W=W)
        check(Yg, Yo, So, p.tau, f"wide blocks m={m} R={R} C={C}")
        Yg2, _ = gpu_product(p, path=MFMA, W=W)
        assert np.array_equal(Yg, Yg2), "two runs differ: race"
        Ya, _ = gpu_product(p, path=0, W=W)
        assert np.array_equal(Ya, Yg)                              # the library's own choice is this kernel
    q = wl.small_integer_problem(100, 40 * 16, 700, 1, 16, 0.3, seed=33)
    Yo, So = oracle_of(oracle_mod, q)
    Yg, _ = gpu_product(q, path=MFMA)
    assert np.array_equal(Yg, Yo)
    # block-row 1 stores block-column 2 twice: the matrix-core path is not available, AUTO takes the wavefront kernels
    rng = np.random.default_rng(34)
    ptr = np.array([0, 2, 5, 5, 6], dtype=np.int32)
    idx = np.array([0, 3, 2, 1, 2, 3], dtype=np.int32)
    data = rng.integers(-3, 4, size=(6, 1, 16)).astype(np.float32)
    X = rng.integers(-3, 4, size=(20, 64)).astype(np.float32)
    d = wl.Problem("dup", 20, 64, 4, 1, 16, "f32", "f32", X, data, idx, ptr)
    Yo, So = oracle_of(oracle_mod, d)
    Wd = lib.bsr_create(d.n, d.k, d.block_data, d.block_indices, d.index_pointer, dtype="f32")
    assert lib.bsr_query_path(Wd, 20) == WAVE
    Yg, _ = gpu_product(d, path=0, W=Wd)
    assert np.array_equal(Yg, Yo)
    Xd = to_device(d.X, "f32")
    Y = torch.zeros((20, 4), device="cuda")
    assert lib.load_library().bsr_spmm_ex(Wd.handle, 20, Xd.data_ptr(), Y.data_ptr(), 0, MFMA,
                                          torch.cuda.current_stream().cuda_stream) == 9   # BSR_ERR_UNSUPPORTED


@pytest.mark.parametrize("u", ["", "a=4", "a=8", "a=16", "a=6,b=1", "a=10,b=2", "b=4", "a=14,b=8"])
def test_thin_mfma_path(oracle_mod, monkeypatch, u):
    """16x1 fp32 blocks on the matrix-core path with a transposed copy of X in lent scratch (variant 1), then
    gather + MFMA (a = groups of 4 blocks per chunk, b = m-tile groups over the XCDs)."""
    import paper_2007_13055_amd as lib
    monkeypatch.setenv("BSR_SPMM_TUNE", "variant=1" + ("," + u if u else ""))
    for m, R, C in ((32, 3, 40), (70, 9, 130), (257, 20, 300), (64, 5, 7), (600, 11, 64)):
        rng = np.random.default_rng(m + R)
        counts = rng.integers(0, min(C, 90) + 1, size=R)
        counts[0] = 0
        counts[-1] = min(C, 77)
        counts[R // 2] = 1
        p = wl.make_problem("thin", m, C, R * 16, 16, 1, "f32", "f32", ("counts", counts), ("uniform", 1.0),
                            ("uniform", 1.0), 500 + m)
        Yo, So = oracle_of(oracle_mod, p)
        Yg, W = gpu_product(p, path=MFMA)
        assert lib.bsr_scratch_size(W, m) >= m * C * 4
        assert lib.bsr_query_path(W, m) == MFMA
        check(Yg, Yo, So, p.tau, f"thin mfma m={m} R={R} C={C}")
        Yw, _ = gpu_product(p, path=WAVE, W=W)
        check(Yw, Yo, So, p.tau, f"thin wave m={m} R={R} C={C}")


def test_thin_mfma_needs_scratch():
    import torch
    import paper_2007_13055_amd as lib
    p = wl.make_problem("thin", 64, 64, 64, 16, 1, "f32", "f32", ("bernoulli", 0.3), ("uniform", 1.0), ("uniform", 1.0), 9)
    # every block-row stored in descending block-column order: the one-launch kernel (which needs no scratch)
    # is not available, the matrix-core path is the one with the transposed copy
    order = np.concatenate([np.arange(p.index_pointer[r], p.index_pointer[r + 1])[::-1] for r in range(4)])
    W = lib.bsr_create(p.n, p.k, p.block_data[order], p.block_indices[order], p.index_pointer, dtype="f32")
    assert lib.bsr_query_path(W, 64) == WAVE                      # nothing lent yet: wave path
    so = lib.load_library()
    X = to_device(p.X, "f32")
    Y = torch.empty((64, 64), device="cuda")
    st = so.bsr_spmm_ex(W.handle, 64, X.data_ptr(), Y.data_ptr(), 0, MFMA, torch.cuda.current_stream().cuda_stream)
    assert st == 7                                                # BSR_ERR_WORKSPACE
    W.ensure_scratch(64)
    assert lib.bsr_query_path(W, 64) == MFMA


def test_ksplit_work_item_table_and_m_changes(oracle_mod, monkeypatch):
    """More (block-row, m-tile) items than CUs: the k-split kernel runs from its CU-balanced work-item
    table; the table is rebuilt when m changes on the same handle."""
    monkeypatch.setenv("BSR_SPMM_TUNE", "variant=2")
    rng = np.random.default_rng(77)
    R, C, bs = 40, 24, 32
    counts = rng.integers(0, 21, size=R)
    counts[3] = 0
    W = None
    for m in (330, 1000, 330, 97):                    # 440, 1280, 440 and 160 items (the last without a table)
        p = wl.make_problem("it", m, C * bs, R * bs, bs, bs, "f32", "f32", ("counts", counts), ("normal", 1.0),
                            ("normal", 1.0), 600)     # same seed: same pattern and W, X differs in size only
        Yo, So = oracle_of(oracle_mod, p)
        Yg, W = gpu_product(p, path=MFMA, W=W)
        check(Yg, Yo, So, p.tau, f"k-split items m={m}")


@pytest.mark.parametrize("case", [("f32", 32, 32, 128, 12, 12), ("bf16", 16, 16, 300, 20, 12), ("f16", 64, 64, 600, 6, 8),
                                  ("f32", 16, 1, 100, 6, 90), ("f32", 8, 8, 8, 10, 16), ("f16", 16, 32, 40, 7, 9)])
def test_tuned_product_matches_oracle(oracle_mod, case):
    """bsr_tune runs every candidate kernel for the shape and remembers the fastest; the products after
    it (whatever was chosen) meet the same bar, and Y right after tuning is already the product."""
    import torch
    import paper_2007_13055_amd as lib
    dtype, bs_r, bs_c, m, R, C = case
    rng = np.random.default_rng(m + R)
    counts = rng.integers(0, C + 1, size=R)
    counts[1] = 0
    p = wl.make_problem("tune", m, C * bs_c, R * bs_r, bs_r, bs_c, dtype, dtype, ("counts", counts), ("normal", 1.0),
                        ("normal", 1.0), 900 + m)
    Yo, So = oracle_of(oracle_mod, p)
    W = lib.bsr_create(p.n, p.k, p.block_data, p.block_indices, p.index_pointer, dtype=dtype)
    X = to_device(p.X, dtype)
    Y = torch.full((m, p.n), float("nan"), dtype=X.dtype, device="cuda")
    tried, best_us = lib.bsr_tune(W, X, Y, trials=3)
    assert tried >= 1 and best_us > 0
    check(Y.double().cpu().numpy(), Yo, So, p.tau, f"tune {case}: Y after tuning", out_dtype=dtype)
    Y2 = torch.full_like(Y, float("nan"))
    lib.bsr_spmm(W, X, Y2)
    torch.cuda.synchronize()
    check(Y2.double().cpu().numpy(), Yo, So, p.tau, f"tune {case}: tuned product", out_dtype=dtype)
    # another m on the same handle is untouched by what was remembered
    Xs = X[: max(1, m // 2)].contiguous()
    Ys = lib.bsr_spmm(W, Xs)
    torch.cuda.synchronize()
    check(Ys.double().cpu().numpy(), Yo[: Xs.shape[0]], So[: Xs.shape[0]], p.tau, f"tune {case}: other m", out_dtype=dtype)


@pytest.mark.parametrize("case", [("f32", 32, 32, 128, 10, 12), ("bf16", 16, 16, 300, 20, 12), ("f16", 64, 32, 70, 5, 9),
                                  ("f32", 16, 1, 40, 6, 50), ("f32", 8, 4, 8, 10, 16), ("f16", 16, 64, 1, 7, 3),
                                  ("f32", 3, 5, 9, 7, 11), ("bf16", 8, 16, 33, 9, 13)])
def test_sibling_product_through_transposed_handle(oracle_mod, case):
    """Z = G * W as bsr_spmm on the handle of W^T (bsr_transpose_pattern + bsr_transpose_values), against
    the oracle's own sibling product; and the transposed values are exactly W's, block by block."""
    import torch
    import paper_2007_13055_amd as lib
    dtype, bs_r, bs_c, m, R, C = case
    rng = np.random.default_rng(m + R + C)
    counts = rng.integers(0, C + 1, size=R)
    counts[0] = 0
    p = wl.make_problem("sib", m, C * bs_c, R * bs_r, bs_r, bs_c, dtype, dtype, ("counts", counts), ("normal", 1.0),
                        ("normal", 1.0), 950 + m)
    G = wl.round_to_storage(rng.normal(size=(m, p.n)).astype(np.float32), dtype)
    Zo, So = oracle_mod.bsr_spmm_w(G, p.block_data, p.block_indices, p.index_pointer, p.k)
    WT = lib.bsr_create_transposed(p.n, p.k, p.block_data, p.block_indices, p.index_pointer, dtype=dtype)
    assert (WT.n, WT.k, WT.bs_r, WT.bs_c) == (p.k, p.n, bs_c, bs_r)
    t_ptr, t_idx, perm = lib.bsr_transpose_pattern(p.n, p.k, bs_r, bs_c, p.index_pointer, p.block_indices)
    got = WT.block_data.float().cpu().numpy()
    assert np.array_equal(got, np.transpose(p.block_data[perm], (0, 2, 1)))
    Gd = to_device(G, dtype)
    Z = torch.full((m, p.k), float("nan"), dtype=Gd.dtype, device="cuda")
    lib.bsr_spmm(WT, Gd, Z)
    torch.cuda.synchronize()
    check(Z.double().cpu().numpy(), Zo, So, p.tau, f"sibling {case}", out_dtype=dtype)


@pytest.mark.parametrize("extra", ["", "nw=1,a=1", "nw=8,a=4", "nw=3,a=2"])
@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("bs", [(8, 8), (8, 16), (16, 8)])
def test_small_blocks_on_matrix_cores(oracle_mod, monkeypatch, extra, dtype, bs):
    """Blocks below the MFMA tile grouped into 16x16 tiles of W: every shape and type, empty and long
    tile-rows (more entries than a descriptor's inline columns), duplicates (a second block at a taken
    position opens a second entry), a ragged last m-tile, and the wave path on the same handle."""
    import paper_2007_13055_amd as lib
    if extra:
        monkeypatch.setenv("BSR_SPMM_TUNE", extra)
    bs_r, bs_c = bs
    R, C = 12 * (16 // bs_r), 40 * (16 // bs_c)
    rng = np.random.default_rng(bs_r * 3 + bs_c)
    counts = rng.integers(0, 12, size=R)
    counts[0] = counts[1] = 0                      # an empty tile-row (its block-rows are empty)
    counts[2] = counts[3] = C                      # a full one: 40 entries > 28 inline columns
    counts[-1] = 1
    for m in (16, 45, 300):
        p = wl.make_problem("sm", m, C * bs_c, R * bs_r, bs_r, bs_c, dtype, dtype, ("counts", counts), ("normal", 1.0),
                            ("normal", 1.0), 1000 + m + bs_r)
        Yo, So = oracle_of(oracle_mod, p)
        Yg, W = gpu_product(p, path=MFMA)
        assert lib.bsr_query_path(W, m) == MFMA
        check(Yg, Yo, So, p.tau, f"small {bs} {dtype} m={m} {extra}", out_dtype=dtype)
        Yw, _ = gpu_product(p, path=WAVE, W=W)
        check(Yw, Yo, So, p.tau, f"small {bs} {dtype} m={m} wave", out_dtype=dtype)
    # duplicates and unsorted block-columns
    ptr = np.array([0, 3, 3, 5, 6], dtype=np.int32)
    idx = np.array([2, 2, 0, 1, 1, 3], dtype=np.int32)
    data = wl.round_to_storage(rng.normal(size=(6, bs_r, bs_c)).astype(np.float32), dtype)
    X = wl.round_to_storage(rng.normal(size=(33, 4 * bs_c)).astype(np.float32), dtype)
    n4 = 4 * bs_r
    if n4 % 16 == 0 and (4 * bs_c) % 16 == 0:
        q = wl.Problem("dup", 33, 4 * bs_c, n4, bs_r, bs_c, dtype, dtype, X, data, idx, ptr)
        Yo, So = oracle_of(oracle_mod, q)
        Yg, _ = gpu_product(q, path=MFMA)
        check(Yg, Yo, So, q.tau, f"small {bs} {dtype} duplicates", out_dtype=dtype)


def test_small_blocks_need_whole_tiles():
    """n or k not a multiple of 16: no tiles, the matrix-core path is refused and AUTO is the wave path."""
    import torch
    import paper_2007_13055_amd as lib
    p = wl.make_problem("odd", 32, 24, 40, 8, 8, "f32", "f32", ("bernoulli", 0.5), ("normal", 1.0), ("normal", 1.0), 5)
    W = lib.bsr_create(p.n, p.k, p.block_data, p.block_indices, p.index_pointer, dtype="f32")
    assert lib.bsr_query_path(W, 32) == WAVE
    X = to_device(p.X, "f32")
    Y = torch.empty((32, 40), device="cuda")
    st = lib.load_library().bsr_spmm_ex(W.handle, 32, X.data_ptr(), Y.data_ptr(), 0, MFMA, torch.cuda.current_stream().cuda_stream)
    assert st == 9                                                # BSR_ERR_UNSUPPORTED


@pytest.mark.parametrize("dtype,out", [("f32", "f32"), ("f16", "f16"), ("bf16", "bf16"), ("bf16", "f32")])
@pytest.mark.parametrize("bs", SHAPES + [(8, 8), (16, 1), (1, 16), (4, 8), (2, 3), (8, 16), (3, 5)])
def test_sampled_product_block_gradients(oracle_mod, dtype, out, bs):
    """D[p] = G[:, block-row]^T X[:, block-column] for every stored block, against the oracle: every matrix-core
    shape and three shapes of the plain loop; m below one chunk, one chunk per wavefront, a ragged tail, many."""
    import torch
    import paper_2007_13055_amd as lib
    bs_r, bs_c = bs
    R, C = 5, 6
    for m in (1, 37, 128, 300):
        p = wl.make_problem("sd", m, C * bs_c, R * bs_r, bs_r, bs_c, dtype, dtype, ("bernoulli", 0.5), ("normal", 1.0),
                            ("normal", 1.0), 1100 + m + bs_r + bs_c)
        G = wl.round_to_storage(np.random.default_rng(m).normal(size=(m, p.n)).astype(np.float32), dtype)
        Do, So = oracle_mod.bsr_sddmm(G, p.X, p.block_indices, p.index_pointer, bs_r, bs_c)
        W = lib.bsr_create(p.n, p.k, p.block_data, p.block_indices, p.index_pointer, dtype=dtype)
        D = torch.full((p.nnzb, bs_r, bs_c), float("nan"), dtype=getattr(torch, {"f32": "float32", "f16": "float16", "bf16": "bfloat16"}[out]),
                       device="cuda")
        lib.bsr_sddmm(W, to_device(G, dtype), to_device(p.X, dtype), D, d_dtype=out)
        torch.cuda.synchronize()
        check(D.double().cpu().numpy().reshape(p.nnzb, -1), Do.reshape(p.nnzb, -1), So.reshape(p.nnzb, -1), p.tau,
              f"sampled {bs} {dtype}->{out} m={m}", out_dtype=out)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("bs", [(16, 16), (32, 32), (64, 64), (16, 64), (8, 8), (16, 1), (1, 16), (16, 8)])
def test_sampled_product_long_and_empty_rows(oracle_mod, dtype, bs):
    """Block-rows longer than one run of blocks (and than 64 lane slots), next to empty ones."""
    import torch
    import paper_2007_13055_amd as lib
    bs_r, bs_c = bs
    counts = [37, 0, 5, 1, 0, 40, 9]
    C, m = 40, 133
    p = wl.make_problem("sdl", m, C * bs_c, len(counts) * bs_r, bs_r, bs_c, dtype, dtype, ("counts", counts), ("normal", 1.0),
                        ("normal", 1.0), 1300 + bs_r + bs_c)
    G = wl.round_to_storage(np.random.default_rng(5).normal(size=(m, p.n)).astype(np.float32), dtype)
    Do, So = oracle_mod.bsr_sddmm(G, p.X, p.block_indices, p.index_pointer, bs_r, bs_c)
    W = lib.bsr_create(p.n, p.k, p.block_data, p.block_indices, p.index_pointer, dtype=dtype)
    D = lib.bsr_sddmm(W, to_device(G, dtype), to_device(p.X, dtype), d_dtype="f32")
    torch.cuda.synchronize()
    check(D.double().cpu().numpy().reshape(p.nnzb, -1), Do.reshape(p.nnzb, -1), So.reshape(p.nnzb, -1), p.tau,
          f"sampled long rows {bs} {dtype}", out_dtype="f32")


@pytest.mark.parametrize("bs,dtype", [((16, 16), "bf16"), ((16, 16), "f32"), ((32, 32), "f16"), ((32, 16), "f32"), ((64, 64), "f16")])
def test_sampled_product_shared_runs(oracle_mod, bs, dtype):
    """Many rows and many blocks: the stored blocks of a block-row are taken in runs that share the piece of G
    (full runs, shorter ones, single blocks, empty block-rows), ragged last chunk of rows."""
    import torch
    import paper_2007_13055_amd as lib
    bs_r, bs_c = bs
    R, C, m = 90, 24, 531
    counts = np.random.default_rng(9).integers(0, C + 1, size=R)
    counts[:4] = [0, 1, C, 5]
    assert sum((int(c) + 3) // 4 for c in counts) >= 256          # enough runs of 4 for the shared-run launch
    p = wl.make_problem("sdr", m, C * bs_c, R * bs_r, bs_r, bs_c, dtype, dtype, ("counts", counts), ("normal", 1.0),
                        ("normal", 1.0), 1400 + bs_r + bs_c)
    G = wl.round_to_storage(np.random.default_rng(6).normal(size=(m, p.n)).astype(np.float32), dtype)
    Do, So = oracle_mod.bsr_sddmm(G, p.X, p.block_indices, p.index_pointer, bs_r, bs_c)
    W = lib.bsr_create(p.n, p.k, p.block_data, p.block_indices, p.index_pointer, dtype=dtype)
    D = lib.bsr_sddmm(W, to_device(G, dtype), to_device(p.X, dtype), d_dtype="f32")
    torch.cuda.synchronize()
    check(D.double().cpu().numpy().reshape(p.nnzb, -1), Do.reshape(p.nnzb, -1), So.reshape(p.nnzb, -1), p.tau,
          f"sampled runs {bs} {dtype}", out_dtype="f32")


@pytest.mark.parametrize("bs,dtype,R,C", [((16, 16), "bf16", 70, 62), ((16, 16), "f32", 37, 35), ((32, 32), "f16", 45, 35),
                                          ((16, 64), "f16", 70, 24), ((64, 16), "bf16", 20, 66), ((32, 16), "f32", 20, 35),
                                          ((16, 32), "bf16", 70, 33)])
def test_sampled_product_line_wide_tiles(oracle_mod, bs, dtype, R, C):
    """Blocks whose pieces are narrower than a 128-byte line, many rows: workgroups take tiles of adjacent
    block-rows x block-columns.  R and C leave a partial last tile in both directions; block-columns unsorted
    inside the block-rows and one block stored twice (a second tile at the same place)."""
    import torch
    import paper_2007_13055_amd as lib
    bs_r, bs_c = bs
    m = 555
    s = 4 if dtype == "f32" else 2
    SR, LC = max(1, 128 // (bs_r * s)), max(1, 128 // (bs_c * s))
    p = wl.make_problem("sdt", m, C * bs_c, R * bs_r, bs_r, bs_c, dtype, dtype, ("bernoulli", 0.5), ("normal", 1.0),
                        ("normal", 1.0), 1500 + bs_r + bs_c)
    rng = np.random.default_rng(12)
    idx = p.block_indices.copy()
    for r in range(R):
        a, b = p.index_pointer[r], p.index_pointer[r + 1]
        idx[a:b] = p.block_indices[rng.permutation(b - a) + a]
    idx = np.concatenate([idx[:1], idx])                          # the first stored block twice
    ptr = p.index_pointer.copy()
    ptr[1:] += 1
    rows = np.repeat(np.arange(R), np.diff(ptr))
    assert len(set(zip((rows // SR).tolist(), (idx // LC).tolist()))) >= 256    # enough tiles for the tile launch
    G = wl.round_to_storage(np.random.default_rng(8).normal(size=(m, p.n)).astype(np.float32), dtype)
    Do, So = oracle_mod.bsr_sddmm(G, p.X, idx, ptr, bs_r, bs_c)
    data = np.zeros((len(idx), bs_r, bs_c), dtype=p.block_data.dtype)
    W = lib.bsr_create(p.n, p.k, data, idx, ptr, dtype=dtype)
    D = lib.bsr_sddmm(W, to_device(G, dtype), to_device(p.X, dtype), d_dtype="f32")
    torch.cuda.synchronize()
    check(D.double().cpu().numpy().reshape(len(idx), -1), Do.reshape(len(idx), -1), So.reshape(len(idx), -1), p.tau,
          f"sampled tiles {bs} {dtype}", out_dtype="f32")


@pytest.mark.parametrize("lend", [True, False])
@pytest.mark.parametrize("m", [32, 45, 256, 300, 777])
def test_sampled_product_thin_blocks(oracle_mod, m, lend):
    """16x1 fp32 blocks: with scratch lent, a transposed copy of X and the matrix-core kernel (rows of X in
    pieces of 256, partial last piece and step; block-rows of more than 64 blocks, of 16 k + 1, and empty);
    without, the lane-per-column kernel.  Same results to tolerance."""
    import torch
    import paper_2007_13055_amd as lib
    counts = [70, 0, 17, 1, 16, 64, 65, 33]
    C = 80
    p = wl.make_problem("sdthin", m, C, len(counts) * 16, 16, 1, "f32", "f32", ("counts", counts), ("uniform", 1.0),
                        ("uniform", 1.0), 1600 + m)
    G = np.random.default_rng(m).normal(size=(m, p.n)).astype(np.float32)
    Do, So = oracle_mod.bsr_sddmm(G, p.X, p.block_indices, p.index_pointer, 16, 1)
    W = lib.bsr_create(p.n, p.k, p.block_data, p.block_indices, p.index_pointer, dtype="f32")
    D = torch.full((p.nnzb, 16, 1), float("nan"), device="cuda")
    lib.bsr_sddmm(W, to_device(G, "f32"), to_device(p.X, "f32"), D, d_dtype="f32", lend_scratch=lend)
    torch.cuda.synchronize()
    check(D.double().cpu().numpy().reshape(p.nnzb, -1), Do.reshape(p.nnzb, -1), So.reshape(p.nnzb, -1), p.tau,
          f"sampled thin m={m} scratch={lend}", out_dtype="f32")


def test_sampled_product_small_integers_bitwise(oracle_mod):
    """Integer-valued G and X: every partial sum is exact in fp32, so the block gradients match bit for bit."""
    import torch
    import paper_2007_13055_amd as lib
    p = wl.small_integer_problem(200, 4 * 64, 3 * 32, 32, 64, 0.6, seed=31, in_dtype="f16", out_dtype="f32", lo=-2, hi=2)
    G = np.random.default_rng(3).integers(-2, 3, size=(p.m, p.n)).astype(np.float32)
    Do, _ = oracle_mod.bsr_sddmm(G, p.X, p.block_indices, p.index_pointer, p.bs_r, p.bs_c)
    W = lib.bsr_create(p.n, p.k, p.block_data, p.block_indices, p.index_pointer, dtype="f16")
    D = lib.bsr_sddmm(W, to_device(G, "f16"), to_device(p.X, "f16"), d_dtype="f32")
    torch.cuda.synchronize()
    assert np.array_equal(D.double().cpu().numpy(), Do)


def test_debug_mode_checks_device_arrays_before_every_product(oracle_mod, monkeypatch):
    """BSR_SPMM_DEBUG=1: a block-column, an index_pointer entry or a plan word damaged in device memory after
    bsr_create is reported by the next product (INDEX, INDPTR, WORKSPACE) and nothing is launched on the damaged
    arrays; once repaired the product is the oracle's again."""
    import torch
    import paper_2007_13055_amd as lib
    monkeypatch.setenv("BSR_SPMM_DEBUG", "1")
    p = wl.make_problem("dbg", 70, 256, 192, 32, 32, "f16", "f16", ("bernoulli", 0.5), ("normal", 1.0), ("normal", 1.0), 77)
    Yo, So = oracle_of(oracle_mod, p)
    W = lib.bsr_create(p.n, p.k, p.block_data, p.block_indices, p.index_pointer, dtype="f16")
    so = lib.load_library()
    X = to_device(p.X, "f16")
    Y = torch.full((p.m, p.n), 7.0, dtype=torch.float16, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream

    def product():
        st = so.bsr_spmm_ex(W.handle, p.m, X.data_ptr(), Y.data_ptr(), 1, 0, stream)
        torch.cuda.synchronize()
        return st

    assert product() == 0
    check(Y.double().cpu().numpy(), Yo, So, p.tau, "debug mode, intact arrays", out_dtype="f16")
    idx, ptr, ws = W._tensors[1], W._tensors[2], W._tensors[3]
    for tensor, pos, bad, code in ((idx, 3, p.k // 32, 4), (idx, 0, -1, 4), (ptr, 2, 10 ** 6, 3), (ptr, 0, 1, 3)):
        Y.fill_(7.0)
        keep = int(tensor[pos])
        tensor[pos] = bad
        assert product() == code
        assert torch.all(Y == 7.0), "a product ran on damaged arrays"
        tensor[pos] = keep
    words = ws.view(torch.int32)
    keep = int(words[5])
    words[5] = keep ^ 1                                            # a word of the plan (the slot order)
    Y.fill_(7.0)
    assert product() == 7 and torch.all(Y == 7.0)
    words[5] = keep
    assert product() == 0
    check(Y.double().cpu().numpy(), Yo, So, p.tau, "debug mode, repaired arrays", out_dtype="f16")
    G = to_device(np.zeros((p.m, p.n), dtype=np.float32), "f16")
    idx[1] = -5
    D = torch.zeros((p.nnzb, 32, 32), dtype=torch.float16, device="cuda")
    assert so.bsr_sddmm(W.handle, p.m, G.data_ptr(), X.data_ptr(), D.data_ptr(), 1, stream) == 4
    idx[1] = int(p.block_indices[1])
