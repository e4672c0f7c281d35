"""ctypes binding for libbsr_spmm.so: same names as the C entry points, marshalling only."""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libbsr_spmm.so")

BSR_F32, BSR_F16, BSR_BF16 = 0, 1, 2
PATH_AUTO, PATH_WAVE, PATH_MFMA = 0, 1, 2
_DTYPE_CODE = {"f32": BSR_F32, "f16": BSR_F16, "bf16": BSR_BF16}

_lib = None


class BsrError(RuntimeError):
    """A C entry point returned a status other than BSR_OK."""

    def __init__(self, status: int, where: str):
        self.status = int(status)
        super().__init__(f"{where}: {bsr_status_string(status)} (status {int(status)})")


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load the built library; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(f"{_LIB_PATH} is missing: build it with `python -m paper_2007_13055_amd.build` "
                           "(or __graft_entry__.build()); there is no CPU fallback")
    lib = ctypes.CDLL(_LIB_PATH)
    i64, i32, vp, sz = ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p, ctypes.c_size_t
    lib.bsr_validate.argtypes = [i64, i64, i32, i32, i64, vp, vp]
    lib.bsr_workspace_size.argtypes = [i64, i64, i32, i32, i64, ctypes.POINTER(sz)]
    lib.bsr_create.argtypes = [ctypes.POINTER(vp), i64, i64, i32, i32, i64, ctypes.c_int, vp, vp, vp, vp, vp,
                               vp, sz, vp]
    lib.bsr_destroy.argtypes = [vp]
    lib.bsr_destroy.restype = None
    lib.bsr_spmm.argtypes = [vp, i64, vp, vp, ctypes.c_int, vp]
    lib.bsr_spmm_ex.argtypes = [vp, i64, vp, vp, ctypes.c_int, ctypes.c_int, vp]
    lib.bsr_spmm_static.argtypes = [vp, i64, vp, vp, ctypes.c_int, vp]
    lib.bsr_query_path.argtypes = [vp, i64, ctypes.POINTER(ctypes.c_int)]
    lib.bsr_tune.argtypes = [vp, i64, vp, vp, ctypes.c_int, ctypes.c_int, vp, ctypes.POINTER(ctypes.c_int),
                             ctypes.POINTER(ctypes.c_float)]
    lib.bsr_tune_result.argtypes = [vp, i64, ctypes.c_int, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_float)]
    lib.bsr_scratch_size.argtypes = [vp, i64, ctypes.POINTER(sz)]
    lib.bsr_set_scratch.argtypes = [vp, vp, sz]
    lib.bsr_transpose_pattern.argtypes = [i64, i64, i32, i32, i64, vp, vp, vp, vp, vp]
    lib.bsr_transpose_values.argtypes = [ctypes.c_int, i32, i32, i64, vp, vp, vp, vp]
    lib.bsr_sddmm.argtypes = [vp, i64, vp, vp, vp, ctypes.c_int, vp]
    lib.bsr_probe_mfma.argtypes = [ctypes.c_int, i32, vp, vp, ctypes.POINTER(ctypes.c_double)]
    lib.bsr_probe_mfma.restype = ctypes.c_int
    lib.bsr_status_string.argtypes = [ctypes.c_int]
    lib.bsr_status_string.restype = ctypes.c_char_p
    for f in ("bsr_validate", "bsr_workspace_size", "bsr_create", "bsr_spmm", "bsr_spmm_ex", "bsr_spmm_static",
              "bsr_query_path", "bsr_scratch_size", "bsr_set_scratch", "bsr_tune", "bsr_tune_result",
              "bsr_transpose_pattern", "bsr_transpose_values", "bsr_sddmm"):
        getattr(lib, f).restype = ctypes.c_int
    _lib = lib
    return lib


def bsr_status_string(status: int) -> str:
    return load_library().bsr_status_string(int(status)).decode()


def _i32(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32).reshape(-1))


def bsr_validate(n, k, bs_r, bs_c, index_pointer, block_indices) -> int:
    """Structural check on host arrays; returns the status code (0 = ok)."""
    ptr, idx = _i32(index_pointer), _i32(block_indices)
    return int(load_library().bsr_validate(n, k, bs_r, bs_c, idx.shape[0], ptr.ctypes.data,
                                           idx.ctypes.data if idx.size else None))


def bsr_workspace_size(n, k, bs_r, bs_c, nnzb) -> int:
    out = ctypes.c_size_t(0)
    st = load_library().bsr_workspace_size(n, k, bs_r, bs_c, nnzb, ctypes.byref(out))
    if st != 0:
        raise BsrError(st, "bsr_workspace_size")
    return int(out.value)


def _torch_dtype(name):
    import torch
    return {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}[name]


def _dtype_name(t):
    import torch
    return {torch.float32: "f32", torch.float16: "f16", torch.bfloat16: "bf16"}[t.dtype]


class BsrMatrix:
    """Owns the device tensors of one W (they must outlive the C handle) and the handle itself."""

    def __init__(self, handle, n, k, bs_r, bs_c, dtype, tensors):
        self.handle, self.n, self.k, self.bs_r, self.bs_c, self.dtype = handle, n, k, bs_r, bs_c, dtype
        self._tensors = tensors            # block_data, block_indices, index_pointer, workspace (device)
        self._scratch = None               # device scratch lent to the handle (see ensure_scratch)

    @property
    def block_data(self):
        return self._tensors[0]

    def ensure_scratch(self, m: int):
        """Lend the handle enough scratch for a product with m rows (torch allocates it; grows only)."""
        import torch
        need = bsr_scratch_size(self, m)
        have = self._scratch.numel() if self._scratch is not None else 0
        if need > have:
            self._scratch = torch.empty(need, dtype=torch.uint8, device=self._tensors[0].device)
            st = load_library().bsr_set_scratch(self.handle, self._scratch.data_ptr(), self._scratch.numel())
            if st != 0:
                raise BsrError(st, "bsr_set_scratch")

    def close(self):
        if self.handle:
            load_library().bsr_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def bsr_create(n, k, block_data, block_indices, index_pointer, dtype=None, device="cuda") -> BsrMatrix:
    """Upload the three BSR arrays (numpy or torch) and build the handle.

    block_data (nnzb, bs_r, bs_c); dtype "f32" | "f16" | "bf16" selects the storage type the values
    are converted to on upload (they must already be exact in it); torch tensors keep their dtype.
    """
    import torch
    lib = load_library()
    if isinstance(block_data, torch.Tensor):
        dtype = dtype or _dtype_name(block_data)
        data_dev = block_data.to(device=device, dtype=_torch_dtype(dtype)).contiguous()
    else:
        dtype = dtype or "f32"
        data_dev = torch.from_numpy(np.ascontiguousarray(block_data, dtype=np.float32)).to(
            device=device, dtype=_torch_dtype(dtype)).contiguous()
    if data_dev.dim() != 3:
        raise ValueError("block_data must be (nnzb, bs_r, bs_c)")
    nnzb, bs_r, bs_c = (int(v) for v in data_dev.shape)
    idx_h = _i32(block_indices.cpu().numpy() if isinstance(block_indices, torch.Tensor) else block_indices)
    ptr_h = _i32(index_pointer.cpu().numpy() if isinstance(index_pointer, torch.Tensor) else index_pointer)
    if idx_h.shape[0] != nnzb:
        raise ValueError("block_indices length differs from the number of stored blocks")
    if bs_r <= 0 or n % bs_r or ptr_h.shape[0] != n // bs_r + 1:
        raise BsrError(2 if (bs_r <= 0 or n % bs_r) else 3, "bsr_create")
    idx_dev = torch.from_numpy(idx_h).to(device) if nnzb else torch.zeros(4, dtype=torch.int32, device=device)
    ptr_dev = torch.from_numpy(ptr_h).to(device)
    if nnzb == 0:
        data_dev = torch.zeros(4, dtype=_torch_dtype(dtype), device=device)
    ws = torch.empty(bsr_workspace_size(n, k, bs_r, bs_c, nnzb), dtype=torch.uint8, device=device)
    handle = ctypes.c_void_p()
    stream = torch.cuda.current_stream().cuda_stream
    st = lib.bsr_create(ctypes.byref(handle), n, k, bs_r, bs_c, nnzb, _DTYPE_CODE[dtype],
                        data_dev.data_ptr(), idx_dev.data_ptr(), ptr_dev.data_ptr(),
                        idx_h.ctypes.data if nnzb else None, ptr_h.ctypes.data,
                        ws.data_ptr(), ws.numel(), stream)
    if st != 0:
        raise BsrError(st, "bsr_create")
    return BsrMatrix(handle, n, k, bs_r, bs_c, dtype, (data_dev, idx_dev, ptr_dev, ws))


def bsr_transpose_pattern(n, k, bs_r, bs_c, index_pointer, block_indices):
    """Pattern of W^T: (t_index_pointer, t_block_indices, perm) as int32 numpy arrays."""
    ptr, idx = _i32(index_pointer), _i32(block_indices)
    nnzb = int(idx.shape[0])
    if bs_c <= 0 or k % bs_c:
        raise BsrError(2, "bsr_transpose_pattern")
    t_ptr = np.zeros(k // bs_c + 1, dtype=np.int32)
    t_idx = np.zeros(max(nnzb, 1), dtype=np.int32)
    perm = np.zeros(max(nnzb, 1), dtype=np.int32)
    st = load_library().bsr_transpose_pattern(n, k, bs_r, bs_c, nnzb, ptr.ctypes.data, idx.ctypes.data if nnzb else None,
                                              t_ptr.ctypes.data, t_idx.ctypes.data, perm.ctypes.data)
    if st != 0:
        raise BsrError(st, "bsr_transpose_pattern")
    return t_ptr, t_idx[:nnzb], perm[:nnzb]


def bsr_create_transposed(n, k, block_data, block_indices, index_pointer, dtype=None, device="cuda") -> BsrMatrix:
    """Handle of W^T (k x n, blocks bs_c x bs_r) for the sibling product Z = G * W = bsr_spmm(W^T, G).
    Arguments as bsr_create (they describe W); the transposed values are computed on the device."""
    import torch
    if isinstance(block_data, torch.Tensor):
        dtype = dtype or _dtype_name(block_data)
        data_dev = block_data.to(device=device, dtype=_torch_dtype(dtype)).contiguous()
    else:
        dtype = dtype or "f32"
        data_dev = torch.from_numpy(np.ascontiguousarray(block_data, dtype=np.float32)).to(
            device=device, dtype=_torch_dtype(dtype)).contiguous()
    nnzb, bs_r, bs_c = (int(v) for v in data_dev.shape)
    t_ptr, t_idx, perm = bsr_transpose_pattern(n, k, bs_r, bs_c, index_pointer, block_indices)
    t_data = torch.empty((nnzb, bs_c, bs_r), dtype=data_dev.dtype, device=device)
    if nnzb:
        perm_dev = torch.from_numpy(perm).to(device)
        st = load_library().bsr_transpose_values(_DTYPE_CODE[dtype], bs_r, bs_c, nnzb, perm_dev.data_ptr(),
                                                 data_dev.data_ptr(), t_data.data_ptr(),
                                                 torch.cuda.current_stream().cuda_stream)
        if st != 0:
            raise BsrError(st, "bsr_transpose_values")
        torch.cuda.current_stream().synchronize()     # perm_dev and data_dev may be freed on return
    return bsr_create(k, n, t_data, t_idx, t_ptr, dtype=dtype, device=device)


def bsr_spmm_ex(W: BsrMatrix, X, Y=None, y_dtype=None, path=PATH_AUTO):
    """Y = X * W^T on torch's current stream; X (m, k) device tensor of W's dtype.  Returns Y."""
    import torch
    if X.dim() != 2 or X.shape[1] != W.k:
        raise ValueError("X must be (m, k)")
    if _dtype_name(X) != W.dtype or not X.is_contiguous():
        raise ValueError("X must be contiguous and of W's dtype")
    y_dtype = y_dtype or W.dtype
    m = int(X.shape[0])
    W.ensure_scratch(m)
    if Y is None:
        Y = torch.empty((m, W.n), dtype=_torch_dtype(y_dtype), device=X.device)
    elif tuple(Y.shape) != (m, W.n) or _dtype_name(Y) != y_dtype or not Y.is_contiguous():
        raise ValueError("Y must be a contiguous (m, n) tensor of y_dtype")
    st = load_library().bsr_spmm_ex(W.handle, m, X.data_ptr(), Y.data_ptr(), _DTYPE_CODE[y_dtype], int(path),
                                    torch.cuda.current_stream().cuda_stream)
    if st != 0:
        raise BsrError(st, "bsr_spmm")
    return Y


def bsr_spmm(W: BsrMatrix, X, Y=None, y_dtype=None):
    return bsr_spmm_ex(W, X, Y, y_dtype, PATH_AUTO)


STATIC_SCRATCH_BYTES = 8 << 20


def bsr_spmm_static(W: BsrMatrix, X, Y):
    """bsr_spmm for thin-block W on the library's built-in scratch array: nothing is allocated or lent, so Y
    must be given.  X (m, k) fp32, Y (m, n) fp32, both contiguous device tensors.  Returns Y."""
    import torch
    if X.dim() != 2 or X.shape[1] != W.k or _dtype_name(X) != W.dtype or not X.is_contiguous():
        raise ValueError("X must be a contiguous (m, k) tensor of W's dtype")
    m = int(X.shape[0])
    if tuple(Y.shape) != (m, W.n) or _dtype_name(Y) != "f32" or not Y.is_contiguous():
        raise ValueError("Y must be a contiguous (m, n) fp32 tensor")
    st = load_library().bsr_spmm_static(W.handle, m, X.data_ptr(), Y.data_ptr(), BSR_F32,
                                        torch.cuda.current_stream().cuda_stream)
    if st != 0:
        raise BsrError(st, "bsr_spmm_static")
    return Y


def bsr_tune(W: BsrMatrix, X, Y=None, y_dtype=None, trials: int = 20):
    """Times the library's candidate kernels for this W, X.shape[0] and output type on torch's current
    stream and makes later bsr_spmm calls of that size use the fastest.  Returns (candidates tried,
    microseconds per product of the fastest).  Waits for the stream."""
    import torch
    if X.dim() != 2 or X.shape[1] != W.k or _dtype_name(X) != W.dtype or not X.is_contiguous():
        raise ValueError("X must be a contiguous (m, k) tensor of W's dtype")
    y_dtype = y_dtype or W.dtype
    m = int(X.shape[0])
    W.ensure_scratch(m)
    if Y is None:
        Y = torch.empty((m, W.n), dtype=_torch_dtype(y_dtype), device=X.device)
    elif tuple(Y.shape) != (m, W.n) or _dtype_name(Y) != y_dtype or not Y.is_contiguous():
        raise ValueError("Y must be a contiguous (m, n) tensor of y_dtype")
    tried, best = ctypes.c_int(0), ctypes.c_float(0.0)
    st = load_library().bsr_tune(W.handle, m, X.data_ptr(), Y.data_ptr(), _DTYPE_CODE[y_dtype], int(trials),
                                 torch.cuda.current_stream().cuda_stream, ctypes.byref(tried), ctypes.byref(best))
    if st != 0:
        raise BsrError(st, "bsr_tune")
    return int(tried.value), float(best.value)


def bsr_tune_result(W: BsrMatrix, m: int, y_dtype=None):
    """What bsr_tune remembered for (m, y_dtype): dict of settings and microseconds, or None."""
    out, us = (ctypes.c_int32 * 6)(), ctypes.c_float(0.0)
    st = load_library().bsr_tune_result(W.handle, m, _DTYPE_CODE[y_dtype or W.dtype], out, ctypes.byref(us))
    if st == 9:
        return None
    if st != 0:
        raise BsrError(st, "bsr_tune_result")
    keys = ("path", "variant", "nw", "mt", "a", "b")
    return {**{k: int(v) for k, v in zip(keys, out)}, "us": float(us.value)}


def bsr_sddmm(W: BsrMatrix, G, X, D=None, d_dtype=None, lend_scratch=True):
    """D[p] = G[:, block-row of p]^T @ X[:, block-column of p] for every stored block of W (the gradient
    of the block values); G (m, n), X (m, k) device tensors of W's dtype.  Returns D (nnzb, bs_r, bs_c).
    lend_scratch: lend the handle the scratch its thin-block kernel wants (as bsr_spmm does)."""
    import torch
    if G.dim() != 2 or X.dim() != 2 or G.shape[0] != X.shape[0] or G.shape[1] != W.n or X.shape[1] != W.k:
        raise ValueError("G must be (m, n) and X (m, k)")
    if _dtype_name(G) != W.dtype or _dtype_name(X) != W.dtype or not G.is_contiguous() or not X.is_contiguous():
        raise ValueError("G and X must be contiguous and of W's dtype")
    d_dtype = d_dtype or W.dtype
    if lend_scratch:
        W.ensure_scratch(int(G.shape[0]))
    nnzb = int(W.block_data.shape[0]) if W.block_data.dim() == 3 else 0
    if D is None:
        D = torch.empty((nnzb, W.bs_r, W.bs_c), dtype=_torch_dtype(d_dtype), device=G.device)
    elif tuple(D.shape) != (nnzb, W.bs_r, W.bs_c) or _dtype_name(D) != d_dtype or not D.is_contiguous():
        raise ValueError("D must be a contiguous (nnzb, bs_r, bs_c) tensor of d_dtype")
    st = load_library().bsr_sddmm(W.handle, int(G.shape[0]), G.data_ptr(), X.data_ptr(), D.data_ptr(),
                                  _DTYPE_CODE[d_dtype], torch.cuda.current_stream().cuda_stream)
    if st != 0:
        raise BsrError(st, "bsr_sddmm")
    return D


def bsr_scratch_size(W: BsrMatrix, m: int) -> int:
    out = ctypes.c_size_t(0)
    st = load_library().bsr_scratch_size(W.handle, m, ctypes.byref(out))
    if st != 0:
        raise BsrError(st, "bsr_scratch_size")
    return int(out.value)


def bsr_query_path(W: BsrMatrix, m: int) -> int:
    out = ctypes.c_int(0)
    st = load_library().bsr_query_path(W.handle, m, ctypes.byref(out))
    if st != 0:
        raise BsrError(st, "bsr_query_path")
    return int(out.value)
