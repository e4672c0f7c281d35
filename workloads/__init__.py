"""Seeded synthetic inputs for the BSR product: patterns, values, the five benchmark
configurations and the paper's own shape grid.

This module only DRAWS inputs (random patterns and values, and the rounding of
values to the storage type).  It holds none of the product's arithmetic and is
the one module that both the GPU side (tests, benchmark) and the CPU oracle's
tests use.

Every value is returned in a float32 numpy array that already holds the value
as stored in the problem's input type (fp32, fp16 or bf16): 16-bit problems are
drawn in float32 and rounded to nearest-even to the 16-bit type, and the rounded
value is the input for everybody.

Generator: numpy.random.default_rng(seed); draw order pattern, W values, X.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

BASE_SEED = 200713055

# tolerance factor tau in |Y_gpu - Y_oracle| <= tau * sum|x*w|, by input type
TOLERANCE = {"f32": 1e-5, "f16": 2e-3, "bf16": 2e-3}


# --------------------------------------------------------------------------- storage rounding
def round_to_storage(a: np.ndarray, dtype: str) -> np.ndarray:
    """Round float32 values to the storage type (nearest-even), returned as float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "f32":
        return a
    if dtype == "f16":
        return a.astype(np.float16).astype(np.float32)
    if dtype == "bf16":
        u = a.view(np.uint32).astype(np.uint64)
        u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
        return u.astype(np.uint32).view(np.float32).reshape(a.shape)
    raise ValueError(f"unknown storage type {dtype!r}")


# --------------------------------------------------------------------------- patterns
def pattern_from_counts(rng, counts, C):
    """Per-block-row block counts -> (index_pointer, block_indices); columns of a
    block-row are drawn uniformly without replacement and sorted ascending."""
    counts = np.asarray(counts, dtype=np.int64)
    ptr = np.zeros(counts.shape[0] + 1, dtype=np.int32)
    np.cumsum(counts, out=ptr[1:])
    idx = np.empty(int(ptr[-1]), dtype=np.int32)
    for r, cnt in enumerate(counts):
        if cnt:
            idx[ptr[r]:ptr[r + 1]] = np.sort(rng.choice(C, size=int(cnt), replace=False))
    return ptr, idx


def pattern_bernoulli(rng, R, C, prob):
    """Each of the R*C blocks present independently with probability prob."""
    mask = rng.random((R, C)) < prob
    return pattern_from_mask(mask)


def pattern_exact(rng, R, C, density):
    """Exactly round(density*R*C) blocks, drawn uniformly without replacement from the grid."""
    nnzb = int(round(density * R * C))
    flat = rng.choice(R * C, size=nnzb, replace=False)
    mask = np.zeros(R * C, dtype=bool)
    mask[flat] = True
    return pattern_from_mask(mask.reshape(R, C))


def pattern_from_mask(mask):
    mask = np.asarray(mask, dtype=bool)
    counts = mask.sum(axis=1)
    ptr = np.zeros(mask.shape[0] + 1, dtype=np.int32)
    np.cumsum(counts, out=ptr[1:])
    idx = np.nonzero(mask)[1].astype(np.int32)      # row-major order: sorted within a row
    return ptr, idx


def power_law_counts(rng, R, C, total, s):
    """Blocks per block-row following a rank power law.

    Weights rank^(-s) for rank 1..R, ranks given to block-rows by a seeded
    permutation; counts are the largest-remainder rounding of total*w/sum(w),
    capped at the row length C with the excess handed on to the uncapped rows in
    proportion to their weights (repeated until nothing exceeds the cap).
    """
    w = np.arange(1, R + 1, dtype=np.float64) ** (-float(s))
    share = np.zeros(R, dtype=np.float64)
    capped = np.zeros(R, dtype=bool)
    while True:
        rest = total - C * int(capped.sum())
        share[:] = 0.0
        share[capped] = C
        share[~capped] = rest * w[~capped] / w[~capped].sum()
        over = (~capped) & (share > C)
        if not over.any():
            break
        capped |= over
    counts = np.floor(share).astype(np.int64)
    remainder = share - counts
    short = int(total - counts.sum())
    if short > 0:
        order = np.argsort(-remainder, kind="stable")
        counts[order[:short]] += 1
    perm = rng.permutation(R)                        # rank q goes to block-row perm[q]
    out = np.zeros(R, dtype=np.int64)
    out[perm] = counts
    return out


# --------------------------------------------------------------------------- problems
@dataclass
class Problem:
    """One instance of Y = X * W^T.  Arrays hold the values as stored (see module doc)."""
    name: str
    m: int
    k: int
    n: int
    bs_r: int
    bs_c: int
    in_dtype: str                 # "f32" | "f16" | "bf16"  (X and W)
    out_dtype: str                # "f32" | "f16" | "bf16"  (Y)
    X: np.ndarray                 # (m, k) float32
    block_data: np.ndarray        # (nnzb, bs_r, bs_c) float32
    block_indices: np.ndarray     # (nnzb,) int32
    index_pointer: np.ndarray     # (n/bs_r + 1,) int32
    seed: int = 0
    note: str = ""
    extra: dict = field(default_factory=dict)

    @property
    def nnzb(self) -> int:
        return int(self.block_indices.shape[0])

    @property
    def tau(self) -> float:
        return TOLERANCE[self.in_dtype]

    @property
    def flops(self) -> int:
        """Effective flops of one product: 2 * m * nnzb * bs_r * bs_c."""
        return 2 * self.m * self.nnzb * self.bs_r * self.bs_c

    def algorithmic_bytes(self) -> int:
        """Bytes one product must move when every operand is touched once:
        the referenced columns of X, the stored blocks, the index arrays, Y."""
        s_in = 4 if self.in_dtype == "f32" else 2
        s_out = 4 if self.out_dtype == "f32" else 2
        used_cols = int(np.unique(self.block_indices).shape[0]) * self.bs_c
        R = self.n // self.bs_r
        return (self.m * used_cols * s_in + self.nnzb * self.bs_r * self.bs_c * s_in
                + 4 * (self.nnzb + R + 1) + self.m * self.n * s_out)


def _values(rng, shape, dist, dtype):
    kind, par = dist
    if kind == "uniform":
        v = rng.uniform(-par, par, size=shape)
    elif kind == "normal":
        v = rng.normal(0.0, par, size=shape)
    else:
        raise ValueError(kind)
    return round_to_storage(v.astype(np.float32), dtype)


def make_problem(name, m, k, n, bs_r, bs_c, in_dtype, out_dtype, pattern, x_dist, w_dist, seed,
                 note=""):
    """pattern: ("bernoulli", p) | ("exact", density) | ("power_law", density, s)
              | ("full",) | ("counts", array)"""
    if n % bs_r or k % bs_c:
        raise ValueError("block size must divide n and k")
    rng = np.random.default_rng(seed)
    R, C = n // bs_r, k // bs_c
    extra = {}
    if pattern[0] == "bernoulli":
        ptr, idx = pattern_bernoulli(rng, R, C, pattern[1])
    elif pattern[0] == "exact":
        ptr, idx = pattern_exact(rng, R, C, pattern[1])
    elif pattern[0] == "power_law":
        total = int(round(pattern[1] * R * C))
        counts = power_law_counts(rng, R, C, total, pattern[2])
        extra["row_counts_sorted"] = np.sort(counts)[::-1].tolist()
        ptr, idx = pattern_from_counts(rng, counts, C)
    elif pattern[0] == "full":
        ptr, idx = pattern_from_mask(np.ones((R, C), dtype=bool))
    elif pattern[0] == "counts":
        ptr, idx = pattern_from_counts(rng, pattern[1], C)
    else:
        raise ValueError(pattern[0])
    data = _values(rng, (idx.shape[0], bs_r, bs_c), w_dist, in_dtype)
    X = _values(rng, (m, k), x_dist, in_dtype)
    return Problem(name, m, k, n, bs_r, bs_c, in_dtype, out_dtype, X, data, idx, ptr,
                   seed=seed, note=note, extra=extra)


# The five benchmark configurations (ids 1..5).
CONFIG_NAMES = {1: "tiny", 2: "ffn", 3: "batched", 4: "thin", 5: "skewed"}


def config(cid: int, m: int | None = None) -> Problem:
    """Benchmark configuration cid (1..5), seed BASE_SEED + cid.  m overrides the
    number of rows of X only (to cut the problem down for a CPU-sized check; the
    pattern and W stay those of the full configuration)."""
    seed = BASE_SEED + cid
    if cid == 1:   # Tiny: fp32, 16x16 blocks, Bernoulli(0.25)
        return make_problem("tiny", m or 128, 256, 256, 16, 16, "f32", "f32",
                            ("bernoulli", 0.25), ("uniform", 1.0), ("uniform", 1.0), seed)
    if cid == 2:   # Transformer FFN weight: fp32, 32x32 blocks, density 0.10
        return make_problem("ffn", m or 128, 3072, 3072, 32, 32, "f32", "f32",
                            ("exact", 0.10), ("normal", 1.0), ("normal", 0.02), seed)
    if cid == 3:   # Batched activations: bf16 in and out, 16x16 blocks, density 0.20
        return make_problem("batched", m or 4096, 768, 3072, 16, 16, "bf16", "bf16",
                            ("exact", 0.20), ("normal", 1.0), ("normal", 0.02), seed)
    if cid == 4:   # Thin blocks: fp32, 16x1 blocks, density 0.05
        return make_problem("thin", m or 256, 4096, 4096, 16, 1, "f32", "f32",
                            ("exact", 0.05), ("uniform", 1.0), ("uniform", 1.0), seed)
    if cid == 5:   # Large skewed: fp16 in and out, 64x64 blocks, density 0.05, power law s=1.2
        return make_problem("skewed", m or 8192, 8192, 8192, 64, 64, "f16", "f16",
                            ("power_law", 0.05, 1.2), ("normal", 1.0), ("normal", 0.02), seed)
    raise ValueError("config id must be 1..5")


def paper_grid():
    """The shape grid of the paper's Tables 1 and 2: (m, k, n) x block size x sparsity."""
    out = []
    for (m, k, n) in [(1, 128, 768), (8, 128, 768), (1, 1024, 1024), (8, 1024, 1024)]:
        for bs in (8, 16, 32):
            for sparsity in (0.8, 0.85, 0.95):
                out.append((m, k, n, bs, sparsity))
    return out


def paper_grid_problem(m, k, n, bs, sparsity, dtype="f32", seed=None) -> Problem:
    """One cell of the paper's grid: square blocks, exact density 1 - sparsity, N(0,1) values."""
    if seed is None:
        seed = BASE_SEED + 1000 + (m * 131 + k * 17 + n * 7 + bs * 3 + int(round(sparsity * 100)))
    return make_problem(f"grid_m{m}_k{k}_n{n}_bs{bs}_sp{sparsity}", m, k, n, bs, bs, dtype, dtype,
                        ("exact", 1.0 - sparsity), ("normal", 1.0), ("normal", 1.0), seed)


def small_integer_problem(m, k, n, bs_r, bs_c, density, seed, in_dtype="f32", out_dtype=None,
                          lo=-4, hi=4) -> Problem:
    """Integer-valued X and W in [lo, hi]: every partial sum is an integer far below 2^24,
    so any summation order gives the same float32 result and comparisons are bitwise."""
    rng = np.random.default_rng(seed)
    R, C = n // bs_r, k // bs_c
    ptr, idx = pattern_bernoulli(rng, R, C, density)
    data = rng.integers(lo, hi + 1, size=(idx.shape[0], bs_r, bs_c)).astype(np.float32)
    X = rng.integers(lo, hi + 1, size=(m, k)).astype(np.float32)
    return Problem(f"int_m{m}_k{k}_n{n}_{bs_r}x{bs_c}", m, k, n, bs_r, bs_c, in_dtype,
                   out_dtype or in_dtype, X, data, idx, ptr, seed=seed)
