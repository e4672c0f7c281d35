"""CPU oracle for Y = X * W^T with W in BSR -- TEST INFRASTRUCTURE, not product code.

Only the tests, the smoke check and the benchmark's cpu_baseline leg may import
this package.  It shares nothing with the GPU library: its own C file
(``bsr_oracle.c``, the definition of the product from the paper's Background
and Approaches sections written as loops in double), its own structural check,
its own loader.  Nothing here imports the GPU package.

Python side: build the C file with gcc, load it with ctypes, marshal numpy
arrays.  No arithmetic of the method happens in Python.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "bsr_oracle.c")
_LIB = os.path.join(_HERE, "libbsr_oracle.so")

_STATUS = {
    1: "bad argument (null pointer, size, or block size does not divide n / k)",
    2: "bad index_pointer (must start at 0, never decrease, end at the block count)",
    3: "block_indices entry outside [0, k / b_c)",
    4: "requested row outside [0, m)",
}


def build(force: bool = False) -> str:
    """Compile bsr_oracle.c into libbsr_oracle.so next to it; returns the path.

    -ffp-contract=off keeps every product and every sum a separately rounded
    double operation, as the header of the C file states.
    """
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i64, i32, vp = ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p
        lib.oracle_bsr_spmm_rows.argtypes = [i64, i64, i64, i32, i32, i64, vp, vp, vp, vp,
                                             i64, vp, vp, vp]
        lib.oracle_bsr_spmm_rows.restype = ctypes.c_int
        lib.oracle_bsr_spmm_w.argtypes = [i64, i64, i64, i32, i32, i64, vp, vp, vp, vp, vp, vp]
        lib.oracle_bsr_spmm_w.restype = ctypes.c_int
        lib.oracle_bsr_sddmm.argtypes = [i64, i64, i64, i32, i32, i64, vp, vp, vp, vp, vp, vp]
        lib.oracle_bsr_sddmm.restype = ctypes.c_int
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_set_num_threads.argtypes = [ctypes.c_int]
        _lib = lib
    return _lib


def num_threads() -> int:
    """Threads the oracle's row loop uses (OpenMP's current maximum)."""
    return int(_load().oracle_num_threads())


def set_num_threads(t: int) -> None:
    _load().oracle_set_num_threads(int(t))


def _as_f32(a, name):
    a = np.asarray(a)
    if a.dtype == np.float64:
        b = a.astype(np.float32)
        if not np.array_equal(b.astype(np.float64), a, equal_nan=True):
            raise ValueError(f"{name}: float64 values that are not exact in float32")
        a = b
    elif a.dtype != np.float32:
        a = a.astype(np.float32)          # float16 and small integers widen exactly
    return np.ascontiguousarray(a)


def bsr_spmm(X, block_data, block_indices, index_pointer, n, rows=None):
    """Return (Y, S) as float64 arrays for the stored inputs.

    X            (m, k) array, any float type that is exact in float32
    block_data   (nnzb, b_r, b_c) array of stored blocks
    block_indices(nnzb,) block-column of each stored block
    index_pointer(n // b_r + 1,) CSR pointer over block-rows
    n            rows of W (= columns of Y)
    rows         optional 1-D list of rows of X to compute; Y, S are then
                 (len(rows), n) -- used to sample full-size problems

    Y is the product in double; S the same sum over |x * w| (tolerance scale).
    """
    X = _as_f32(X, "X")
    if X.ndim != 2:
        raise ValueError("X must be 2-D")
    m, k = X.shape
    block_data = _as_f32(block_data, "block_data")
    if block_data.ndim != 3:
        raise ValueError("block_data must be (nnzb, b_r, b_c)")
    nnzb, b_r, b_c = block_data.shape
    idx = np.ascontiguousarray(np.asarray(block_indices, dtype=np.int32).reshape(-1))
    ptr = np.ascontiguousarray(np.asarray(index_pointer, dtype=np.int32).reshape(-1))
    if idx.shape[0] != nnzb:
        raise ValueError("block_indices length differs from the number of stored blocks")
    if b_r <= 0 or b_c <= 0 or n % b_r != 0 or ptr.shape[0] != n // b_r + 1:
        raise ValueError("index_pointer must have n / b_r + 1 entries with b_r | n")
    if rows is None:
        n_rows, rows_p = m, None
    else:
        rows_arr = np.ascontiguousarray(np.asarray(rows, dtype=np.int64).reshape(-1))
        n_rows, rows_p = rows_arr.shape[0], rows_arr.ctypes.data
    Y = np.empty((n_rows, n), dtype=np.float64)
    S = np.empty((n_rows, n), dtype=np.float64)
    st = _load().oracle_bsr_spmm_rows(
        m, k, n, b_r, b_c, nnzb, X.ctypes.data, block_data.ctypes.data,
        idx.ctypes.data, ptr.ctypes.data, n_rows, rows_p, Y.ctypes.data, S.ctypes.data)
    if st != 0:
        raise ValueError("oracle: " + _STATUS.get(st, f"status {st}"))
    return Y, S


def bsr_spmm_w(G, block_data, block_indices, index_pointer, k):
    """Return (Z, S) as float64 arrays for the sibling product Z = G * W (G (m, n), W (n, k) in BSR):
    the gradient of the layer's input.  Arguments as for bsr_spmm; k = columns of W (= columns of Z)."""
    G = _as_f32(G, "G")
    if G.ndim != 2:
        raise ValueError("G must be 2-D")
    m, n = G.shape
    block_data = _as_f32(block_data, "block_data")
    if block_data.ndim != 3:
        raise ValueError("block_data must be (nnzb, b_r, b_c)")
    nnzb, b_r, b_c = block_data.shape
    idx = np.ascontiguousarray(np.asarray(block_indices, dtype=np.int32).reshape(-1))
    ptr = np.ascontiguousarray(np.asarray(index_pointer, dtype=np.int32).reshape(-1))
    if idx.shape[0] != nnzb:
        raise ValueError("block_indices length differs from the number of stored blocks")
    if b_r <= 0 or b_c <= 0 or n % b_r != 0 or ptr.shape[0] != n // b_r + 1:
        raise ValueError("index_pointer must have n / b_r + 1 entries with b_r | n")
    Z = np.empty((m, k), dtype=np.float64)
    S = np.empty((m, k), dtype=np.float64)
    st = _load().oracle_bsr_spmm_w(m, k, n, b_r, b_c, nnzb, G.ctypes.data, block_data.ctypes.data,
                                   idx.ctypes.data, ptr.ctypes.data, Z.ctypes.data, S.ctypes.data)
    if st != 0:
        raise ValueError("oracle: " + _STATUS.get(st, f"status {st}"))
    return Z, S


def bsr_sddmm(G, X, block_indices, index_pointer, b_r, b_c):
    """Return (D, S), float64 arrays of shape (nnzb, b_r, b_c): the gradient of the stored blocks,
    D[p] = G[:, block-row of p]^T @ X[:, block-column of p] (G (m, n), X (m, k)), and the same sum over
    absolute values."""
    G = _as_f32(G, "G")
    X = _as_f32(X, "X")
    if G.ndim != 2 or X.ndim != 2 or G.shape[0] != X.shape[0]:
        raise ValueError("G must be (m, n) and X (m, k)")
    m, n = G.shape
    k = X.shape[1]
    idx = np.ascontiguousarray(np.asarray(block_indices, dtype=np.int32).reshape(-1))
    ptr = np.ascontiguousarray(np.asarray(index_pointer, dtype=np.int32).reshape(-1))
    nnzb = idx.shape[0]
    if b_r <= 0 or b_c <= 0 or n % b_r != 0 or ptr.shape[0] != n // b_r + 1:
        raise ValueError("index_pointer must have n / b_r + 1 entries with b_r | n")
    D = np.zeros((nnzb, b_r, b_c), dtype=np.float64)
    S = np.zeros((nnzb, b_r, b_c), dtype=np.float64)
    st = _load().oracle_bsr_sddmm(m, k, n, b_r, b_c, nnzb, G.ctypes.data, X.ctypes.data,
                                  idx.ctypes.data, ptr.ctypes.data, D.ctypes.data, S.ctypes.data)
    if st != 0:
        raise ValueError("oracle: " + _STATUS.get(st, f"status {st}"))
    return D, S
