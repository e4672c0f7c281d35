#!/usr/bin/env python3
"""Benchmark of bsr_spmm on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-all-configs] [--no-cpu] [--paper-grid] [--cold] [--sibling] [--peaks]

A step is one whole product Y = X * W^T (one bsr_spmm call) on the headline workload, the
"Transformer FFN weight" configuration (fp32, m=128, k=n=3072, 32x32 blocks, density 0.10), with
X, W and Y already resident in HBM.  Prints ONE JSON line: effective TFLOP/s
(2*m*nnzb*bs_r*bs_c per call), the roofline object of the product kernel, the CPU oracle timed on
this machine's host cores, and a per-configuration table for the other four workloads.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# Published MI355X peaks used as roofline ceilings.
PEAK_HBM_GBS = 8000.0
PEAK_MFMA_TFLOPS = {"f32": 157.3, "f16": 2500.0, "bf16": 2500.0}
WORKLOAD_TEXT = {
    "tiny": "tiny: X fp32 (128,256) U(-1,1); W (256,256) BSR 16x16, Bernoulli(0.25) blocks, U(-1,1); Y fp32",
    "ffn": "ffn: X fp32 (128,3072) N(0,1); W (3072,3072) BSR 32x32, 922 blocks (density 0.10) uniform without "
           "replacement, N(0,0.02); Y fp32",
    "batched": "batched: X bf16 (4096,768) N(0,1); W (3072,768) BSR 16x16, 1843 blocks (density 0.20), N(0,0.02); Y bf16",
    "thin": "thin: X fp32 (256,4096) U(-1,1); W (4096,4096) BSR 16x1, 52429 blocks (density 0.05), U(-1,1); Y fp32",
    "skewed": "skewed: X fp16 (8192,8192) N(0,1); W (8192,8192) BSR 64x64, 819 blocks (density 0.05), blocks per "
              "block-row by rank power law s=1.2; N(0,0.02); Y fp16",
}


def _upload(p):
    import torch
    import paper_2007_13055_amd as lib
    tdt = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}
    W = lib.bsr_create(p.n, p.k, p.block_data, p.block_indices, p.index_pointer, dtype=p.in_dtype)
    X = torch.from_numpy(p.X).to("cuda", dtype=tdt[p.in_dtype])
    Y = torch.empty((p.m, p.n), dtype=tdt[p.out_dtype], device="cuda")
    return W, X, Y


def _time_steps(fn, steps, warmup, graph_chunk):
    """Time exactly `steps` calls of fn() on torch's current stream.

    Returns (wall seconds over the region, HIP-event seconds over the same region, mode).  With
    graph_chunk > 0 the calls are captured once into a HIP graph of graph_chunk launches and the
    region replays it steps/graph_chunk times (same kernels, same work, host launch cost amortised).
    """
    import torch
    stream = torch.cuda.current_stream()
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    run, mode = None, "eager"
    if graph_chunk > 0 and steps % graph_chunk == 0:
        try:
            side = torch.cuda.Stream()
            side.wait_stream(stream)
            g = torch.cuda.CUDAGraph()
            with torch.cuda.stream(side):
                fn()
                torch.cuda.synchronize()
                with torch.cuda.graph(g, stream=side):
                    for _ in range(graph_chunk):
                        fn()
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            reps = steps // graph_chunk

            def run():
                for _ in range(reps):
                    g.replay()
            mode = f"hipgraph x{graph_chunk}"
        except Exception as e:                       # capture refused: fall back to plain launches
            sys.stderr.write(f"[bench] graph capture unavailable ({e}); timing eager launches\n")
            run = None
    if run is None:
        def run():
            for _ in range(steps):
                fn()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record(stream)
    run()
    e1.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    return wall, e0.elapsed_time(e1) * 1e-3, mode


def _measured_traffic(name):
    """HBM bytes per product from the committed rocprofv3 FETCH_SIZE / WRITE_SIZE summary (None if absent).
    A stored measurement of an earlier profiling run of this same command, not something timed here."""
    try:
        with open(os.path.join(ROOT, "profiles", "hbm_traffic.json")) as f:
            return json.load(f).get(name)
    except (OSError, ValueError):
        return None


def _roofline(p, sec_per_launch):
    """Both ceilings for one launch; the binding one is the slower of the two at peak."""
    t_hbm = p.algorithmic_bytes() / (PEAK_HBM_GBS * 1e9)
    t_mfma = p.flops / (PEAK_MFMA_TFLOPS[p.in_dtype] * 1e12)
    traffic = _measured_traffic(p.name)
    if t_mfma >= t_hbm:
        ach = p.flops / sec_per_launch / 1e12
        return {"bound": "mfma", "achieved": ach, "peak": PEAK_MFMA_TFLOPS[p.in_dtype], "unit": "TFLOP/s",
                "frac": ach / PEAK_MFMA_TFLOPS[p.in_dtype], "traffic": traffic}
    ach = p.algorithmic_bytes() / sec_per_launch / 1e9
    return {"bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": ach / PEAK_HBM_GBS,
            "traffic": traffic}


def _bench_config(cid, steps, warmup, graph_chunk):
    import workloads as wl
    import paper_2007_13055_amd as lib
    p = wl.config(cid)
    W, X, Y = _upload(p)
    fn = lambda: lib.bsr_spmm(W, X, Y)
    wall, ev, mode = _time_steps(fn, steps, warmup, graph_chunk)
    eager_wall, _, _ = _time_steps(fn, steps, 0, 0)
    return p, W, {"wall_s": wall, "event_s": ev, "mode": mode, "eager_wall_s": eager_wall,
                  "path": {1: "wave", 2: "mfma"}[lib.bsr_query_path(W, p.m)], "X": X, "Y": Y}


def _spread(p, W, X, Y, steps, graph_chunk, repeats=10):
    """Run-to-run spread of the time per product: `repeats` further timed regions of `steps` launches each
    (after the headline region, not part of it): median, 10th and 90th percentile in microseconds."""
    import paper_2007_13055_amd as lib
    fn = lambda: lib.bsr_spmm(W, X, Y)
    us = sorted(_time_steps(fn, steps, 0, graph_chunk)[1] / steps * 1e6 for _ in range(repeats))
    pick = lambda q: us[min(len(us) - 1, int(round(q * (len(us) - 1))))]
    return {"repeats": repeats, "steps_each": steps, "median_us": pick(0.5), "p10_us": pick(0.1), "p90_us": pick(0.9)}


def _launch_floor(steps, graph_chunk):
    """Average time of a do-nothing kernel (a 1-element fill) under the same launch protocol."""
    import torch
    t = torch.zeros(1, device="cuda")
    _, ev, _ = _time_steps(lambda: t.zero_(), steps, 10, graph_chunk)
    return ev / steps


# The paper's Table 2, column "PRWB+AT" (its tuned kernel on an NVIDIA T4), in microseconds, keyed by
# (m, k, n, block size) with the three sparsities 0.8 / 0.85 / 0.95 -- context beside our numbers for
# the same shapes, another machine's and not a target.
PAPER_TABLE2_T4_US = {
    (1, 128, 768, 8): (5.1, 3.6, 3.6), (1, 128, 768, 16): (4.0, 3.7, 3.7), (1, 128, 768, 32): (3.6, 3.6, 3.7),
    (8, 128, 768, 8): (10.0, 8.5, 5.1), (8, 128, 768, 16): (7.0, 8.3, 4.7), (8, 128, 768, 32): (10.0, 4.3, 4.8),
    (1, 1024, 1024, 8): (13.0, 11.0, 5.9), (1, 1024, 1024, 16): (13.0, 11.0, 5.8), (1, 1024, 1024, 32): (12.0, 4.7, 4.2),
    (8, 1024, 1024, 8): (78.0, 61.0, 26.0), (8, 1024, 1024, 16): (74.0, 58.0, 25.0), (8, 1024, 1024, 32): (18.0, 17.0, 14.0),
}


def _paper_grid(steps, chunk):
    """The shape grid of the paper's Tables 1 and 2 (m = 1 and 8, fp32, square blocks 8/16/32, block
    sparsity 0.8/0.85/0.95) on synthetic patterns of the same density: microseconds per product."""
    import workloads as wl
    import paper_2007_13055_amd as lib
    rows = []
    for (m, k, n, bs, sp) in wl.paper_grid():
        p = wl.paper_grid_problem(m, k, n, bs, sp)
        W, X, Y = _upload(p)
        _, ev, _ = _time_steps(lambda: lib.bsr_spmm(W, X, Y), steps, 20, chunk)
        s = ev / steps
        t4 = PAPER_TABLE2_T4_US[(m, k, n, bs)][(0.8, 0.85, 0.95).index(sp)]
        rows.append({"m": m, "k": k, "n": n, "bs": bs, "sparsity": sp, "us_per_call": s * 1e6,
                     "gflops": p.flops / s / 1e9, "path": {1: "wave", 2: "mfma"}[lib.bsr_query_path(W, m)],
                     "paper_t4_us": t4})
        del W
    return rows


def _sibling(p, steps, chunk):
    """The sibling products on workload p: Z = G * W (gradient of the layer's input; the same kernels on
    the handle of W^T, plus the time of re-transposing the block values on the device, needed once per
    update of W) and the sampled product D = (G^T X) at the stored blocks (gradient of the blocks)."""
    import torch
    import numpy as np
    import paper_2007_13055_amd as lib
    tdt = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}
    WT = lib.bsr_create_transposed(p.n, p.k, p.block_data, p.block_indices, p.index_pointer, dtype=p.in_dtype)
    G = torch.randn((p.m, p.n), device="cuda").to(tdt[p.in_dtype])
    Z = torch.empty((p.m, p.k), dtype=tdt[p.out_dtype], device="cuda")
    _, ev, mode = _time_steps(lambda: lib.bsr_spmm(WT, G, Z), steps, 20, chunk)
    _, _, perm = lib.bsr_transpose_pattern(p.n, p.k, p.bs_r, p.bs_c, p.index_pointer, p.block_indices)
    perm_dev = torch.from_numpy(perm).to("cuda")
    src = torch.from_numpy(np.ascontiguousarray(p.block_data, dtype=np.float32)).to("cuda", dtype=tdt[p.in_dtype])
    dst = torch.empty((p.nnzb, p.bs_c, p.bs_r), dtype=src.dtype, device="cuda")
    so, code = lib.load_library(), {"f32": 0, "f16": 1, "bf16": 2}[p.in_dtype]
    stream = lambda: torch.cuda.current_stream().cuda_stream
    tr = lambda: so.bsr_transpose_values(code, p.bs_r, p.bs_c, p.nnzb, perm_dev.data_ptr(), src.data_ptr(),
                                         dst.data_ptr(), stream())
    _, ev_t, _ = _time_steps(tr, steps, 20, chunk)
    # the sampled sibling D[p] = G[:, block-row]^T X[:, block-column] (gradient of the stored blocks)
    W, X, _ = _upload(p)
    D = torch.empty((p.nnzb, p.bs_r, p.bs_c), dtype=tdt[p.out_dtype], device="cuda")
    _, ev_d, _ = _time_steps(lambda: lib.bsr_sddmm(W, G, X, D, d_dtype=p.out_dtype), steps, 20, chunk)
    s, sd = ev / steps, ev_d / steps
    return {"us_per_product": s * 1e6, "tflops": p.flops / s / 1e12, "launch": mode,
            "transpose_values_us": ev_t / steps * 1e6,
            "sampled_us_per_product": sd * 1e6, "sampled_tflops": p.flops / sd / 1e12}


def _cold(p, steps):
    """The headline product with operands that are NOT resident in the 256 MB last-level cache: the calls
    rotate through enough distinct (X, Y) pairs (and copies of W's values) that 1 GiB of other data
    passes between two uses of the same buffer.  Plain launches (a graph would pin one buffer set)."""
    import torch
    import paper_2007_13055_amd as lib
    tdt = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}
    per_set = p.algorithmic_bytes()
    sets = max(2, min(512, int((1 << 30) // max(per_set, 1)) + 1))
    Ws, Xs, Ys = [], [], []
    for _ in range(sets):
        W, X, Y = _upload(p)
        Ws.append(W); Xs.append(X); Ys.append(Y)
    state = {"i": 0}

    def fn():
        i = state["i"] = (state["i"] + 1) % sets
        lib.bsr_spmm(Ws[i], Xs[i], Ys[i])
    _, ev, _ = _time_steps(fn, steps, sets, 0)
    s = ev / steps
    return {"us_per_product": s * 1e6, "tflops": p.flops / s / 1e12, "buffer_sets": sets,
            "hbm_GBs_algorithmic": per_set / s / 1e9, "launch": "eager"}


def _measured_peaks():
    """What this machine delivers on plain library work, for context beside the published peaks the roofline
    uses: a 1 GiB device-to-device copy (read + written bytes per second) and large dense GEMMs through
    torch (rocBLAS / hipBLASLt).  Library figures, not limits."""
    import torch
    out = {}
    src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
    dst = torch.empty_like(src)
    _, ev, _ = _time_steps(lambda: dst.copy_(src), 20, 3, 0)
    out["copy_1GiB_GBs"] = 2 * src.numel() * 4 / (ev / 20) / 1e9
    del src, dst
    for name, dt, nn in (("gemm_f32_8192_TFLOPs", torch.float32, 8192), ("gemm_bf16_8192_TFLOPs", torch.bfloat16, 8192)):
        a = torch.randn(nn, nn, device="cuda", dtype=dt)
        b = torch.randn(nn, nn, device="cuda", dtype=dt)
        c = torch.empty(nn, nn, device="cuda", dtype=dt)
        _, ev, _ = _time_steps(lambda: torch.mm(a, b, out=c), 10, 3, 0)
        out[name] = 2 * nn ** 3 / (ev / 10) / 1e12
        del a, b, c
    return out


def _cpu_baseline(p, repeats=5):
    import oracle
    best = float("inf")
    for _ in range(repeats):
        t0 = time.perf_counter()
        oracle.bsr_spmm(p.X, p.block_data, p.block_indices, p.index_pointer, p.n)
        best = min(best, time.perf_counter() - t0)
    return {"value": p.flops / best / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"the whole '{p.name}' workload, best of {repeats} runs ({best * 1e3:.1f} ms each); "
                      "plain double-precision loops, a correctness reference and not a tuned CPU SpMM"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--graph-chunk", type=int, default=100,
                    help="launches per captured HIP graph (0 = plain launches only)")
    ap.add_argument("--no-all-configs", action="store_true", help="skip the per-configuration table")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--cold", action="store_true",
                    help="also time the headline product on operands rotated out of the last-level cache")
    ap.add_argument("--sibling", action="store_true",
                    help="also time the sibling product Z = G * W (through the handle of W^T) on the headline workload")
    ap.add_argument("--peaks", action="store_true",
                    help="also time a 1 GiB copy and two large torch GEMMs on this box and add them as 'measured_peaks'")
    ap.add_argument("--paper-grid", action="store_true",
                    help="also time the 36 cells of the paper's own shape grid (m = 1, 8) and add them as 'paper_grid'")
    ap.add_argument("--workload", default="ffn", choices=["tiny", "ffn", "batched", "thin", "skewed"],
                    help="workload of the headline line (default: the FFN configuration); the others are for "
                         "profiling one kernel at a time")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MiB",
                    help="only run 20 device-to-device copies of this many MiB and exit: the reference a "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE reading is scaled by")
    a = ap.parse_args()
    if a.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (the product needs no exchange between GPUs: "
                 "block-rows of W and rows of X both split without one). Use --gpus 1.")
    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP path has no CPU fallback")
    import paper_2007_13055_amd as lib
    lib.load_library()
    torch.cuda.set_device(0)
    chunk = a.graph_chunk if (a.graph_chunk > 0 and a.steps % a.graph_chunk == 0) else 0
    if a.copy_calibration > 0:
        src = torch.ones(a.copy_calibration * (1 << 20) // 4, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(20):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_MiB": a.copy_calibration, "copies": 20}))
        return
    headline = {"tiny": 1, "ffn": 2, "batched": 3, "thin": 4, "skewed": 5}[a.workload]
    if headline == 5:
        a.steps = min(a.steps, 200)
        chunk = chunk if a.steps % max(chunk, 1) == 0 else 0

    p, W, r = _bench_config(headline, a.steps, a.warmup, chunk)
    sec = r["wall_s"] / a.steps
    out = {
        "metric": "effective TFLOP/s of bsr_spmm (2*m*nnzb*bs_r*bs_c per call)",
        "value": p.flops / sec / 1e12, "unit": "TFLOP/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": sec * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if p.in_dtype == "f32" else p.in_dtype, "data": "synthetic",
        "config": {"workload": WORKLOAD_TEXT[p.name],
                   "m": p.m, "k": p.k, "n": p.n, "bs_r": p.bs_r, "bs_c": p.bs_c, "nnzb": p.nnzb,
                   "path": r["path"], "launch": r["mode"], "seed": p.seed},
        "roofline": _roofline(p, r["event_s"] / a.steps),
        "eager_ms_per_step": r["eager_wall_s"] / a.steps * 1e3,
        "launch_floor_us": _launch_floor(a.steps, chunk) * 1e6,
        "spread": _spread(p, W, r["X"], r["Y"], min(a.steps, 200), chunk if min(a.steps, 200) % max(chunk, 1) == 0 else 0),
    }
    out["cpu_baseline"] = None if a.no_cpu else _cpu_baseline(p)

    if not a.no_all_configs:
        table = {}
        for cid in (c for c in (1, 2, 3, 4, 5) if c != headline):
            steps = 200 if cid == 5 else a.steps
            ch = chunk if steps % max(chunk, 1) == 0 else 0
            q, Wq, rq = _bench_config(cid, steps, 20, ch)
            s = rq["event_s"] / steps
            t_hbm = q.algorithmic_bytes() / (PEAK_HBM_GBS * 1e9)
            t_mfma = q.flops / (PEAK_MFMA_TFLOPS[q.in_dtype] * 1e12)
            table[q.name] = {"us_per_call": s * 1e6, "tflops": q.flops / s / 1e12, "hbm_frac": t_hbm / s,
                             "mfma_frac": t_mfma / s, "bound": "mfma" if t_mfma >= t_hbm else "hbm",
                             "path": rq["path"], "launch": rq["mode"],
                             "eager_us_per_call": rq["eager_wall_s"] / steps * 1e6}
            del Wq
        out["per_config"] = table
    if a.paper_grid:
        out["paper_grid"] = _paper_grid(a.steps, chunk)
    if a.cold:
        out["cold"] = _cold(p, min(a.steps, 1000))
    if a.sibling:
        out["sibling"] = _sibling(p, a.steps, chunk)
    if a.peaks:
        out["measured_peaks"] = _measured_peaks()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
