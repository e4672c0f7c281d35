"""Shared code of the GPU parity tests: run the HIP path through the binding, compare with the oracle."""
import numpy as np

import workloads as wl

_TORCH = {"f32": "float32", "f16": "float16", "bf16": "bfloat16"}


def torch_dtype(name):
    import torch
    return getattr(torch, _TORCH[name])


def to_device(arr, dtype):
    import torch
    return torch.from_numpy(np.ascontiguousarray(arr, dtype=np.float32)).to("cuda", dtype=torch_dtype(dtype))


def gpu_product(p: wl.Problem, path=0, y_dtype=None, prefill=float("nan"), X=None, W=None, rows=None):
    """Run bsr_spmm_ex on problem p; returns (Y as float64 numpy, the BsrMatrix)."""
    import torch
    import paper_2007_13055_amd as lib
    if W is None:
        W = lib.bsr_create(p.n, p.k, p.block_data, p.block_indices, p.index_pointer, dtype=p.in_dtype)
    Xd = to_device(p.X, p.in_dtype) if X is None else X
    y_dtype = y_dtype or p.out_dtype
    Y = torch.full((p.m, p.n), prefill, dtype=torch_dtype(y_dtype), device="cuda")
    lib.bsr_spmm_ex(W, Xd, Y, y_dtype=y_dtype, path=path)
    torch.cuda.synchronize()
    if rows is not None:
        Y = Y[torch.as_tensor(rows, device="cuda")]
    return Y.to(torch.float64).cpu().numpy(), W


# Unit roundoff of the OUTPUT type: storing the fp32 accumulator in a 16-bit Y rounds it to nearest,
# which moves it by up to u*|y| (bf16 keeps 8 significant bits: u = 2^-8; fp16 11 bits: u = 2^-11, and
# 2^-25 absolute in its subnormal range).  That rounding is not an error of the product: a correctly
# rounded exact result would show it too, and it can exceed tau*S when little cancels (|y| near S).
OUT_ROUNDOFF = {"f32": (0.0, 0.0), "f16": (2.0 ** -11, 2.0 ** -25), "bf16": (2.0 ** -8, 0.0)}


def check(Yg, Yo, So, tau, what="", out_dtype="f32"):
    """|Y_gpu - Y_oracle| <= tau * S (+ the output type's rounding when Y is 16-bit) elementwise;
    exact zero where S == 0; no NaN anywhere."""
    assert Yg.shape == Yo.shape, what
    assert np.all(np.isfinite(Yg)), f"{what}: non-finite output (Y not fully written?)"
    err = np.abs(Yg - Yo)
    u_rel, u_abs = OUT_ROUNDOFF[out_dtype]
    bound = tau * So + u_rel * np.abs(Yo) + np.where(So > 0, u_abs, 0.0)
    bad = err > bound
    if bad.any():
        i = np.unravel_index(np.argmax(err - bound), err.shape)
        raise AssertionError(f"{what}: {int(bad.sum())} elements beyond tau*S; worst at {i}: gpu {Yg[i]!r} "
                             f"oracle {Yo[i]!r} S {So[i]!r} err/S {err[i] / max(So[i], 1e-300):.3e} tau {tau}")
    assert np.all(Yg[So == 0] == 0), f"{what}: non-zero where the exact result is zero"
