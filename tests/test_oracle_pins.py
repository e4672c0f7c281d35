"""Pins for the CPU oracle: it is checked against things other than itself.

The paper prints no numerical example, so the pins are: a hand-worked fixture,
a dense GEMM of the expanded W (numpy), SciPy's BSR type built from the same
three arrays, a pure-Python brute force over the dense W, closed forms, and
the invariants of the definition.  Each pin names the mistake it would catch.
"""
import json
import os

import numpy as np
import pytest
import scipy.sparse as sp

import workloads as wl
from helpers import brute_force, dense_expand

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def run(oracle_mod, p, rows=None):
    return oracle_mod.bsr_spmm(p.X, p.block_data, p.block_indices, p.index_pointer, p.n, rows=rows)


def rand_problem(seed, m, k, n, bs_r, bs_c, density, dtype="f32"):
    return wl.make_problem("t", m, k, n, bs_r, bs_c, dtype, dtype, ("bernoulli", density),
                           ("normal", 1.0), ("normal", 1.0), seed)


# ---------------------------------------------------------------- hand-worked fixture
def test_hand_worked_fixture(oracle_mod):
    """Golden values computed by hand from the definition (Background / Approaches equation).
    Catches: a/c transposed inside a block, wrong block-column offset, lost second block."""
    with open(os.path.join(GOLDEN, "hand_worked_2x2.json")) as f:
        g = json.load(f)
    Y, S = oracle_mod.bsr_spmm(np.array(g["X"], dtype=np.float32),
                               np.array(g["block_data"], dtype=np.float32),
                               g["block_indices"], g["index_pointer"], g["n"])
    assert np.array_equal(Y, np.array(g["Y"], dtype=np.float64))
    assert np.array_equal(S, np.array(g["S"], dtype=np.float64))


# ---------------------------------------------------------------- P1 dense GEMM of expanded W
@pytest.mark.parametrize("shape", [
    (5, 64, 48, 16, 16, 0.3), (3, 40, 36, 4, 8, 0.5), (7, 36, 40, 8, 4, 0.4),
    (4, 64, 64, 16, 1, 0.2), (4, 64, 64, 1, 16, 0.2), (2, 96, 96, 32, 32, 0.5),
    (9, 128, 128, 64, 64, 0.7), (6, 30, 21, 3, 5, 0.6), (1, 16, 16, 1, 1, 0.3),
])
def test_matches_dense_gemm(oracle_mod, shape):
    m, k, n, bs_r, bs_c, d = shape
    p = rand_problem(11 + m + bs_r, m, k, n, bs_r, bs_c, d)
    Y, S = run(oracle_mod, p)
    W = dense_expand(p.block_data, p.block_indices, p.index_pointer, n, k)
    Yd = p.X.astype(np.float64) @ W.T
    Sd = np.abs(p.X.astype(np.float64)) @ np.abs(W).T
    assert np.all(np.abs(Y - Yd) <= 1e-12 * Sd + 1e-300)
    assert np.all(np.abs(S - Sd) <= 1e-12 * Sd + 1e-300)


# ---------------------------------------------------------------- P2 SciPy BSR, same three arrays
@pytest.mark.parametrize("shape", [(6, 64, 48, 16, 16, 0.3), (5, 40, 36, 4, 8, 0.5),
                                   (3, 64, 64, 16, 1, 0.2), (2, 96, 64, 32, 32, 0.6)])
def test_matches_scipy_bsr(oracle_mod, shape):
    """SciPy's own reading of (data, indices, indptr): pins field semantics."""
    m, k, n, bs_r, bs_c, d = shape
    p = rand_problem(23 + bs_c, m, k, n, bs_r, bs_c, d)
    Wb = sp.bsr_matrix((p.block_data.astype(np.float64), p.block_indices, p.index_pointer),
                       shape=(n, k))
    Ys = np.asarray((Wb @ p.X.astype(np.float64).T).T)
    Y, S = run(oracle_mod, p)
    assert np.all(np.abs(Y - Ys) <= 1e-12 * S + 1e-300)


# ---------------------------------------------------------------- P3 brute force, tiny, non-square
@pytest.mark.parametrize("bs", [(1, 1), (2, 3), (3, 2), (16, 1), (1, 16)])
@pytest.mark.parametrize("m", [1, 3])
def test_brute_force_tiny(oracle_mod, bs, m):
    bs_r, bs_c = bs
    R, C = 3, 4
    p = rand_problem(5 + bs_r * 7 + bs_c, m, C * bs_c, R * bs_r, bs_r, bs_c, 0.5)
    W = dense_expand(p.block_data, p.block_indices, p.index_pointer, p.n, p.k)
    Yb, Sb = brute_force(p.X, W)
    Y, S = run(oracle_mod, p)
    assert np.all(np.abs(Y - Yb) <= 1e-13 * Sb + 1e-300)
    assert np.all(np.abs(S - Sb) <= 1e-13 * Sb + 1e-300)


# ---------------------------------------------------------------- P4 all blocks present
def test_full_pattern_is_dense_gemm(oracle_mod):
    """All blocks stored: W is block_data re-tiled to (n, k); catches traversal mistakes."""
    m, k, n, bs_r, bs_c = 5, 48, 32, 8, 16
    p = wl.make_problem("full", m, k, n, bs_r, bs_c, "f32", "f32", ("full",), ("normal", 1.0),
                        ("normal", 1.0), 77)
    R, C = n // bs_r, k // bs_c
    W = p.block_data.reshape(R, C, bs_r, bs_c).transpose(0, 2, 1, 3).reshape(n, k).astype(np.float64)
    Y, S = run(oracle_mod, p)
    Yd = p.X.astype(np.float64) @ W.T
    assert np.all(np.abs(Y - Yd) <= 1e-12 * S)


# ---------------------------------------------------------------- P5 empty block-rows
@pytest.mark.parametrize("empty", [[0], [3], [1, 2], [0, 1, 2, 3]])
def test_empty_block_rows_give_exact_zero(oracle_mod, empty):
    m, k, n, bs_r, bs_c = 4, 32, 32, 8, 8
    counts = np.array([2, 3, 1, 4])
    counts[empty] = 0
    p = wl.make_problem("e", m, k, n, bs_r, bs_c, "f32", "f32", ("counts", counts),
                        ("normal", 1.0), ("normal", 1.0), 5)
    Y, S = run(oracle_mod, p)
    W = dense_expand(p.block_data, p.block_indices, p.index_pointer, n, k)
    Yd = p.X.astype(np.float64) @ W.T
    for r in range(4):
        cols = slice(r * bs_r, (r + 1) * bs_r)
        if r in empty:
            assert np.all(Y[:, cols] == 0.0) and np.all(S[:, cols] == 0.0)
        else:
            assert np.all(np.abs(Y[:, cols] - Yd[:, cols]) <= 1e-12 * S[:, cols])
            assert np.all(S[:, cols] > 0)


# ---------------------------------------------------------------- P6 block permutation in a row
def test_block_permutation_within_rows(oracle_mod):
    p = wl.small_integer_problem(6, 64, 48, 8, 8, 0.6, seed=3)
    Y0, S0 = run(oracle_mod, p)
    rng = np.random.default_rng(9)
    data, idx = p.block_data.copy(), p.block_indices.copy()
    for r in range(p.n // p.bs_r):
        a, b = p.index_pointer[r], p.index_pointer[r + 1]
        perm = rng.permutation(b - a) + a
        data[a:b], idx[a:b] = p.block_data[perm], p.block_indices[perm]
    Y1, S1 = oracle_mod.bsr_spmm(p.X, data, idx, p.index_pointer, p.n)
    assert np.array_equal(Y0, Y1) and np.array_equal(S0, S1)      # integers: exact
    q = rand_problem(4, 5, 64, 48, 8, 8, 0.6)
    Yq, Sq = run(oracle_mod, q)
    data, idx = q.block_data.copy(), q.block_indices.copy()
    for r in range(q.n // q.bs_r):
        a, b = q.index_pointer[r], q.index_pointer[r + 1]
        data[a:b], idx[a:b] = q.block_data[a:b][::-1], q.block_indices[a:b][::-1]
    Yr, _ = oracle_mod.bsr_spmm(q.X, data, idx, q.index_pointer, q.n)
    assert np.all(np.abs(Yq - Yr) <= 1e-12 * Sq)


def test_duplicate_blocks_are_summed(oracle_mod):
    """Two stored blocks at one position both count (the sum runs over stored blocks)."""
    X = np.arange(8, dtype=np.float32).reshape(2, 4)
    blk = np.array([[[1, 2], [3, 4]]], dtype=np.float32)
    Y1, _ = oracle_mod.bsr_spmm(X, blk, [1], [0, 1, 1], 4)
    Y2, _ = oracle_mod.bsr_spmm(X, np.concatenate([blk, blk]), [1, 1], [0, 2, 2], 4)
    assert np.array_equal(2 * Y1, Y2)


# ---------------------------------------------------------------- P7 closed form
@pytest.mark.parametrize("bs", [(16, 16), (16, 1), (4, 8), (32, 32)])
def test_all_ones_closed_form(oracle_mod, bs):
    """X = 1, stored blocks = 1  =>  Y[i, r*bs_r + a] = bs_c * (blocks in block-row r)."""
    bs_r, bs_c = bs
    R, C, m = 6, 8, 3
    rng = np.random.default_rng(1)
    counts = rng.integers(0, C + 1, size=R)
    ptr, idx = wl.pattern_from_counts(rng, counts, C)
    Y, S = oracle_mod.bsr_spmm(np.ones((m, C * bs_c), np.float32),
                               np.ones((idx.shape[0], bs_r, bs_c), np.float32), idx, ptr, R * bs_r)
    expect = np.repeat(counts * bs_c, bs_r).astype(np.float64)
    assert np.array_equal(Y, np.tile(expect, (m, 1)))
    assert np.array_equal(S, Y)


# ---------------------------------------------------------------- P8 selector
@pytest.mark.parametrize("bs", [(16, 16), (8, 4), (16, 1)])
def test_single_one_selects_a_column(oracle_mod, bs):
    bs_r, bs_c = bs
    R, C, m = 4, 5, 6
    rng = np.random.default_rng(2)
    X = rng.normal(size=(m, C * bs_c)).astype(np.float32)
    for (r, cb, a, c) in [(0, 0, 0, 0), (2, 4, bs_r - 1, bs_c - 1), (3, 1, bs_r // 2, 0)]:
        blk = np.zeros((1, bs_r, bs_c), np.float32)
        blk[0, a, c] = 1.0
        ptr = np.zeros(R + 1, np.int32)
        ptr[r + 1:] = 1
        Y, _ = oracle_mod.bsr_spmm(X, blk, [cb], ptr, R * bs_r)
        expect = np.zeros((m, R * bs_r))
        expect[:, r * bs_r + a] = X[:, cb * bs_c + c]
        assert np.array_equal(Y, expect)


# ---------------------------------------------------------------- P9 block-diagonal identity
def test_block_diagonal_identity(oracle_mod):
    bs, R, m = 8, 5, 4
    X = np.random.default_rng(3).normal(size=(m, R * bs)).astype(np.float32)
    data = np.tile(np.eye(bs, dtype=np.float32), (R, 1, 1))
    Y, _ = oracle_mod.bsr_spmm(X, data, np.arange(R), np.arange(R + 1), R * bs)
    assert np.array_equal(Y, X.astype(np.float64))


# ---------------------------------------------------------------- P10 linearity, row permutation
def test_linearity_over_disjoint_patterns_and_row_permutation(oracle_mod):
    m, k, n, bs_r, bs_c = 5, 64, 64, 8, 8
    R, C = n // bs_r, k // bs_c
    rng = np.random.default_rng(8)
    mask = rng.random((R, C)) < 0.6
    pick = rng.random((R, C)) < 0.5
    vals = rng.normal(size=(R, C, bs_r, bs_c)).astype(np.float32)
    X = rng.normal(size=(m, k)).astype(np.float32)

    def prod(msk, Xin):
        ptr, idx = wl.pattern_from_mask(msk)
        return oracle_mod.bsr_spmm(Xin, vals[msk], idx, ptr, n)

    Yall, Sall = prod(mask, X)
    Y1, _ = prod(mask & pick, X)
    Y2, _ = prod(mask & ~pick, X)
    assert np.all(np.abs(Yall - (Y1 + Y2)) <= 1e-12 * Sall + 1e-300)
    perm = rng.permutation(m)
    Yp, _ = prod(mask, X[perm])
    assert np.array_equal(Yp, Yall[perm])


# ---------------------------------------------------------------- P11 paper-grid shapes
@pytest.mark.parametrize("cell", [(1, 128, 768, 8, 0.8), (8, 128, 768, 32, 0.95),
                                  (1, 1024, 1024, 16, 0.85), (8, 1024, 1024, 32, 0.8)])
def test_paper_grid_shapes(oracle_mod, cell):
    p = wl.paper_grid_problem(*cell)
    Y, S = run(oracle_mod, p)
    W = dense_expand(p.block_data, p.block_indices, p.index_pointer, p.n, p.k)
    assert np.all(np.abs(Y - p.X.astype(np.float64) @ W.T) <= 1e-12 * S + 1e-300)


# ---------------------------------------------------------------- the five configurations
@pytest.mark.parametrize("cid,m", [(1, None), (2, 16), (3, 8), (4, 8), (5, 2)])
def test_benchmark_configs_match_dense(oracle_mod, cid, m):
    p = wl.config(cid, m=m)
    Y, S = run(oracle_mod, p)
    W = dense_expand(p.block_data, p.block_indices, p.index_pointer, p.n, p.k)
    assert np.all(np.abs(Y - p.X.astype(np.float64) @ W.T) <= 1e-12 * S + 1e-300)


def test_row_sampling_equals_full(oracle_mod):
    p = wl.config(1)
    Y, S = run(oracle_mod, p)
    rows = [127, 0, 5, 5, 64]
    Yr, Sr = run(oracle_mod, p, rows=rows)
    assert np.array_equal(Yr, Y[rows]) and np.array_equal(Sr, S[rows])


# ---------------------------------------------------------------- sensitivity of the pins
def test_pins_would_catch_a_transposed_block(oracle_mod):
    """Plant a mistake on the CPU: blocks transposed.  The dense-GEMM pin must notice."""
    p = rand_problem(31, 4, 32, 32, 8, 8, 0.5)
    W = dense_expand(p.block_data, p.block_indices, p.index_pointer, p.n, p.k)
    Ybad, S = oracle_mod.bsr_spmm(p.X, np.ascontiguousarray(p.block_data.transpose(0, 2, 1)),
                                  p.block_indices, p.index_pointer, p.n)
    assert np.any(np.abs(Ybad - p.X.astype(np.float64) @ W.T) > 1e-6 * S)


# ---------------------------------------------------------------- structural errors
def test_oracle_rejects_bad_structure(oracle_mod):
    X = np.zeros((2, 8), np.float32)
    blk = np.zeros((1, 4, 4), np.float32)
    with pytest.raises(ValueError):
        oracle_mod.bsr_spmm(X, blk, [2], [0, 1, 1], 8)        # column out of range
    with pytest.raises(ValueError):
        oracle_mod.bsr_spmm(X, blk, [0], [0, 2, 1], 8)        # pointer decreases
    with pytest.raises(ValueError):
        oracle_mod.bsr_spmm(X, blk, [0], [1, 1, 1], 8)        # does not start at 0
    with pytest.raises(ValueError):
        oracle_mod.bsr_spmm(X, blk, [0], [0, 1, 1], 8, rows=[2])


def test_empty_inputs(oracle_mod):
    Y, S = oracle_mod.bsr_spmm(np.zeros((0, 8), np.float32), np.zeros((0, 4, 4), np.float32),
                               [], [0, 0, 0], 8)
    assert Y.shape == (0, 8)
    Y, S = oracle_mod.bsr_spmm(np.ones((3, 8), np.float32), np.zeros((0, 4, 4), np.float32),
                               [], [0, 0, 0], 8)
    assert Y.shape == (3, 8) and np.all(Y == 0) and np.all(S == 0)


# ---------------------------------------------------------------- the sibling product Z = G W
def run_w(oracle_mod, p, G):
    return oracle_mod.bsr_spmm_w(G, p.block_data, p.block_indices, p.index_pointer, p.k)


def test_sibling_hand_worked_fixture(oracle_mod):
    """Z = G W on the hand-worked 4x4 example.  Catches: a/c swapped, scatter to the wrong block-column."""
    with open(os.path.join(GOLDEN, "hand_worked_2x2.json")) as f:
        g = json.load(f)
    Z, S = oracle_mod.bsr_spmm_w(np.array(g["G"], dtype=np.float32), np.array(g["block_data"], dtype=np.float32),
                                 g["block_indices"], g["index_pointer"], g["k"])
    assert np.array_equal(Z, np.array(g["Z"], dtype=np.float64))
    assert np.array_equal(S, np.array(g["S_Z"], dtype=np.float64))


@pytest.mark.parametrize("shape", [(5, 24, 18, 3, 4, 0.4), (3, 32, 48, 16, 16, 0.3), (7, 40, 64, 16, 1, 0.2), (1, 8, 8, 1, 1, 0.5)])
def test_sibling_matches_dense_gemm_and_scipy(oracle_mod, shape):
    """Z against numpy's G @ Wd with W expanded to dense, and against SciPy's BSR type built from the
    same three arrays.  Catches every indexing mistake of the scatter."""
    m, k, n, bs_r, bs_c, d = shape
    p = rand_problem(31 + m, m, k, n, bs_r, bs_c, d)
    G = np.random.default_rng(m).normal(size=(m, n)).astype(np.float32)
    Z, S = run_w(oracle_mod, p, G)
    Wd = dense_expand(p.block_data, p.block_indices, p.index_pointer, n, k)
    assert np.all(np.abs(Z - G.astype(np.float64) @ Wd) <= 1e-12 * (S + 1e-300))
    assert np.all(np.abs(S - np.abs(G.astype(np.float64)) @ np.abs(Wd)) <= 1e-12 * (S + 1e-300))
    Wsp = sp.bsr_matrix((p.block_data.astype(np.float64), p.block_indices, p.index_pointer), shape=(n, k))
    assert np.all(np.abs(Z - (Wsp.T @ G.astype(np.float64).T).T) <= 1e-12 * (S + 1e-300))


def test_sibling_is_the_adjoint_of_the_forward_product(oracle_mod):
    """<X W^T, G> = <X, G W> for any X, G: ties the two oracle functions to each other through the
    mathematics (not through shared code paths: one gathers, the other scatters)."""
    p = rand_problem(77, 6, 48, 40, 8, 16, 0.35)
    G = np.random.default_rng(5).normal(size=(p.m, p.n)).astype(np.float32)
    Y, _ = run(oracle_mod, p)
    Z, _ = run_w(oracle_mod, p, G)
    lhs, rhs = float(np.sum(Y * G)), float(np.sum(p.X.astype(np.float64) * Z))
    assert abs(lhs - rhs) <= 1e-10 * (abs(lhs) + 1.0)


def test_sibling_empty_block_columns_are_exact_zero(oracle_mod):
    """A block-column without a stored block gives exact zeros in Z (and S)."""
    rng = np.random.default_rng(9)
    ptr, idx = wl.pattern_from_mask(np.array([[1, 0, 1, 0], [0, 0, 1, 0], [1, 0, 0, 0]], dtype=bool))
    data = rng.normal(size=(idx.shape[0], 4, 2)).astype(np.float32)
    G = rng.normal(size=(5, 12)).astype(np.float32)
    Z, S = oracle_mod.bsr_spmm_w(G, data, idx, ptr, 8)
    assert np.all(Z[:, 2:4] == 0) and np.all(Z[:, 6:8] == 0) and np.all(S[:, 2:4] == 0)
    assert np.all(S[:, 0:2] > 0)


# ---------------------------------------------------------------- the sampled sibling D = (G^T X) at the stored blocks
def test_sampled_hand_worked_fixture(oracle_mod):
    """Catches: block-row / block-column swapped, a/c swapped inside a block, a lost row of the sum."""
    with open(os.path.join(GOLDEN, "hand_worked_2x2.json")) as f:
        g = json.load(f)
    D, S = oracle_mod.bsr_sddmm(np.array(g["G"], dtype=np.float32), np.array(g["X"], dtype=np.float32),
                                g["block_indices"], g["index_pointer"], g["bs_r"], g["bs_c"])
    assert np.array_equal(D, np.array(g["D"], dtype=np.float64))
    assert np.array_equal(S, np.array(g["S_D"], dtype=np.float64))


@pytest.mark.parametrize("shape", [(5, 24, 18, 3, 4, 0.4), (40, 32, 48, 16, 16, 0.3), (7, 40, 64, 16, 1, 0.2), (1, 8, 8, 1, 1, 0.5)])
def test_sampled_matches_dense_gemm(oracle_mod, shape):
    """Every stored block against the same slice of numpy's G^T @ X in double."""
    m, k, n, bs_r, bs_c, d = shape
    p = rand_problem(41 + m, m, k, n, bs_r, bs_c, d)
    G = np.random.default_rng(m).normal(size=(m, n)).astype(np.float32)
    D, S = oracle_mod.bsr_sddmm(G, p.X, p.block_indices, p.index_pointer, bs_r, bs_c)
    full = G.astype(np.float64).T @ p.X.astype(np.float64)
    full_s = np.abs(G.astype(np.float64)).T @ np.abs(p.X.astype(np.float64))
    for r in range(n // bs_r):
        for q in range(int(p.index_pointer[r]), int(p.index_pointer[r + 1])):
            c = int(p.block_indices[q])
            ref = full[r * bs_r:(r + 1) * bs_r, c * bs_c:(c + 1) * bs_c]
            assert np.all(np.abs(D[q] - ref) <= 1e-12 * (S[q] + 1e-300))
            assert np.all(np.abs(S[q] - full_s[r * bs_r:(r + 1) * bs_r, c * bs_c:(c + 1) * bs_c]) <= 1e-12 * (S[q] + 1e-300))


def test_sampled_is_the_gradient_of_the_forward_product(oracle_mod):
    """<X V^T, G> = <V, D> for any block values V on W's pattern: Y is linear in the stored blocks and D is
    the coefficient.  Ties the third oracle function to the first through the mathematics."""
    p = rand_problem(88, 9, 48, 40, 8, 16, 0.35)
    G = np.random.default_rng(6).normal(size=(p.m, p.n)).astype(np.float32)
    Y, _ = run(oracle_mod, p)
    D, _ = oracle_mod.bsr_sddmm(G, p.X, p.block_indices, p.index_pointer, p.bs_r, p.bs_c)
    lhs, rhs = float(np.sum(Y * G)), float(np.sum(p.block_data.astype(np.float64) * D))
    assert abs(lhs - rhs) <= 1e-10 * (abs(lhs) + 1.0)


def test_sampled_all_ones_and_duplicates(oracle_mod):
    """G = 1, X = 1: every entry of every stored block is m; duplicate blocks get the same values."""
    ptr, idx = np.array([0, 2, 2, 3], np.int32), np.array([1, 1, 0], np.int32)
    D, S = oracle_mod.bsr_sddmm(np.ones((7, 9), np.float32), np.ones((7, 4), np.float32), idx, ptr, 3, 2)
    assert np.all(D == 7) and np.all(S == 7) and D.shape == (3, 3, 2)
