"""Products through every kernel that places the waits of its loads by hand (k-split, tile and small-block
kernels), as a list of seeded cases.  tests/test_gpu_plain_loads.py runs the list twice -- here in the test
process with the library proper, and in one child process with the checking build (the same sources with
ordinary loads and compiler-placed waits) -- and compares the results bit for bit.

Run as a script: python tests/plain_loads_cases.py <library.so> <out.npz>"""
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
for d in (ROOT, HERE):
    if d not in sys.path:
        sys.path.insert(0, d)


def cases():
    import workloads as wl
    out = []
    # k-split kernel: fp32 32x32 (the ffn shape), fp32 16x16, bf16 16x16 with few rows of X
    out.append(("ffn", "variant=2", wl.config(2)))
    out.append(("tiny", "variant=2", wl.config(1)))
    rng = np.random.default_rng(5)
    out.append(("ksplit bf16", "variant=2", wl.make_problem("kb", 40, 24 * 16, 30 * 16, 16, 16, "bf16", "f32",
                                                             ("counts", rng.integers(0, 20, size=30)), ("normal", 1.0),
                                                             ("normal", 1.0), 77)))
    # tile kernel: fp32 32x32 with 128- and 256-row tiles, fp16 64x64 with one, two and three blocks in flight
    counts32 = rng.integers(0, 9, size=12)
    counts32[3] = 16
    for tune in ("variant=3,mt=1", "variant=3,mt=2,a=1"):
        out.append(("tile f32 " + tune, tune, wl.make_problem("tf", 600, 16 * 32, 12 * 32, 32, 32, "f32", "f32",
                                                               ("counts", counts32), ("normal", 1.0), ("normal", 1.0), 78)))
    counts64 = rng.integers(0, 7, size=9)
    counts64[0] = 14
    for tune in ("variant=3,mt=1,a=1", "variant=3,mt=1,a=2", "variant=3,mt=1,a=3"):
        out.append(("tile f16 " + tune, tune, wl.make_problem("th", 700, 14 * 64, 9 * 64, 64, 64, "f16", "f16",
                                                               ("counts", counts64), ("normal", 1.0), ("normal", 1.0), 79)))
    # small-block kernel: 8x8, 8x16, 16x8
    for bs_r, bs_c in ((8, 8), (8, 16), (16, 8)):
        R, C = 12 * (16 // bs_r), 40 * (16 // bs_c)
        counts = rng.integers(0, 12, size=R)
        counts[2] = C
        out.append((f"small {bs_r}x{bs_c}", "", wl.make_problem("sm", 300, C * bs_c, R * bs_r, bs_r, bs_c, "f32", "f32",
                                                                ("counts", counts), ("normal", 1.0), ("normal", 1.0), 80 + bs_r)))
    return out


def run_cases():
    """{case name: Y} through the MFMA path of whichever library the binding has loaded."""
    import paper_2007_13055_amd as lib
    from gpu_util import gpu_product
    results = {}
    for name, tune, p in cases():
        if tune:
            os.environ["BSR_SPMM_TUNE"] = tune
        else:
            os.environ.pop("BSR_SPMM_TUNE", None)
        try:
            Y, W = gpu_product(p, path=lib.PATH_MFMA)
            Y2, _ = gpu_product(p, path=lib.PATH_MFMA, W=W)
        finally:
            os.environ.pop("BSR_SPMM_TUNE", None)
        assert np.array_equal(Y, Y2), f"{name}: two runs differ"
        results[name] = Y
    return results


if __name__ == "__main__":
    import paper_2007_13055_amd.binding as binding
    binding._LIB_PATH = os.path.abspath(sys.argv[1])
    print("library", binding.library_path(), flush=True)
    np.savez(sys.argv[2], **run_cases())
    print("done", flush=True)
