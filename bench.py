#!/usr/bin/env python3
"""Benchmark of bsr_spmm on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-all-configs] [--no-cpu]
                    [--no-cold] [--no-peaks] [--paper-grid] [--sibling]

A step is one whole product Y = X * W^T (one bsr_spmm call) on the headline workload -- by default the
"large skewed" configuration (fp16, m = k = n = 8192, 64x64 blocks, density 0.05, power-law block-rows), the
largest of the five -- with X, W and Y already resident in HBM.  The K steps are timed as replays of a HIP
graph of the launches (the graph holds the largest divisor of K that is at most --graph-chunk launches), with
HIP events on the launch stream; plain launches are timed beside it.  Prints ONE JSON line: effective TFLOP/s
(2*m*nnzb*bs_r*bs_c per call), the roofline object of the product kernel, the CPU oracle timed on this machine's
host cores, what this chip delivers on a copy and on bare MFMA loops, and the same measurements for the
other four workloads under "per_config".
"""
from __future__ import annotations

import argparse
import ctypes
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
CONFIG_ID = {"tiny": 1, "ffn": 2, "batched": 3, "thin": 4, "skewed": 5}
RAMP_S = 0.03                                        # untimed replays of the timed launches before every timed region


def _graph_chunk(steps, limit):
    """Launches per captured graph: the largest divisor of `steps` that is at most `limit` (0 = no graph)."""
    if limit <= 0 or steps <= 0:
        return 0
    return max(d for d in range(1, min(steps, limit) + 1) if steps % d == 0)


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
    if graph_chunk > 0 and steps % graph_chunk == 0 and steps > 0:
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
    # untimed ramp: a short region after an idle spell runs at lower clocks (20 launches of the largest
    # workload: 157 instead of 137 us per launch), so the same launches are replayed for RAMP_S seconds first
    t_ramp = time.perf_counter()
    while time.perf_counter() - t_ramp < RAMP_S:
        run()
        torch.cuda.synchronize()
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
    """HBM-side bytes per product from the committed rocprofv3 FETCH_SIZE / WRITE_SIZE summary (None if absent):
    a stored reading of separate profiler runs of this command (profiles/hbm_traffic_all_workloads.md says
    which), since counters cannot be read from inside the timed run."""
    try:
        with open(os.path.join(ROOT, "profiles", "hbm_traffic.json")) as f:
            return json.load(f).get(name)
    except (OSError, ValueError):
        return None


def _roofline(p, sec_per_launch):
    """Both ceilings for one launch; the binding one is the slower of the two at peak."""
    t_hbm = p.algorithmic_bytes() / (PEAK_HBM_GBS * 1e9)
    t_mfma = p.flops / (PEAK_MFMA_TFLOPS[p.in_dtype] * 1e12)
    both = {"hbm_frac": t_hbm / sec_per_launch, "mfma_frac": t_mfma / sec_per_launch,
            "algorithmic_bytes": p.algorithmic_bytes(), "flops": p.flops, "traffic": _measured_traffic(p.name),
            "traffic_source": "profiles/hbm_traffic.json (rocprofv3 --pmc FETCH_SIZE, WRITE_SIZE of this command)"}
    if t_mfma >= t_hbm:
        ach = p.flops / sec_per_launch / 1e12
        return {"bound": "mfma", "achieved": ach, "peak": PEAK_MFMA_TFLOPS[p.in_dtype], "unit": "TFLOP/s",
                "frac": ach / PEAK_MFMA_TFLOPS[p.in_dtype], **both}
    ach = p.algorithmic_bytes() / sec_per_launch / 1e9
    return {"bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": ach / PEAK_HBM_GBS, **both}


ROW_SUBSET = None                                    # --row-subset: ("longest" | "rest", N), analysis only


def _row_subset(p, which, count):
    """The workload with only its `count` longest block-rows ("longest") or all but those ("rest") keeping
    their stored blocks; the others become empty block-rows (their columns of Y are still written).  An analysis
    aid: which block-rows a kernel's time and traffic come from."""
    import numpy as np
    ptr = p.index_pointer.astype(np.int64)
    counts = np.diff(ptr)
    longest = np.argsort(-counts, kind="stable")[:count]
    keep = np.zeros(counts.shape[0], dtype=bool)
    keep[longest] = True
    if which == "rest":
        keep = ~keep
    sel = np.concatenate([np.arange(ptr[r], ptr[r + 1]) for r in range(counts.shape[0]) if keep[r]]
                         + [np.zeros(0, dtype=np.int64)]).astype(np.int64)
    new_ptr = np.zeros(counts.shape[0] + 1, dtype=np.int32)
    np.cumsum(np.where(keep, counts, 0), out=new_ptr[1:])
    p.block_indices, p.block_data, p.index_pointer = p.block_indices[sel].copy(), p.block_data[sel].copy(), new_ptr
    p.note = f"{which} {count} block-rows only"
    return p


def _bench_config(cid, steps, warmup, graph_chunk):
    import workloads as wl
    import paper_2007_13055_amd as lib
    p = wl.config(cid)
    if ROW_SUBSET:
        p = _row_subset(p, *ROW_SUBSET)
    W, X, Y = _upload(p)
    fn = lambda: lib.bsr_spmm(W, X, Y)
    wall, ev, mode = _time_steps(fn, steps, warmup, graph_chunk)
    eager_wall, eager_ev, _ = _time_steps(fn, steps, 0, 0)
    return p, W, {"wall_s": wall, "event_s": ev, "mode": mode, "eager_wall_s": eager_wall, "eager_event_s": eager_ev,
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
    """The product with operands that are NOT resident in the 256 MB last-level cache: the calls rotate
    through enough distinct (W, X, Y) sets that 1 GiB of other data passes between two uses of the same
    buffer.  Plain launches (a graph would pin one buffer set), so for the microsecond-scale workloads the
    host's launch rate is part of the figure; "hbm_GBs_algorithmic" is the algorithmic bytes over that time."""
    import torch
    import paper_2007_13055_amd as lib
    per_set = p.algorithmic_bytes()
    sets = max(2, min(256, int((1 << 30) // max(per_set, 1)) + 1))
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
    """What this chip delivers, for context beside the published peaks the roofline uses: a 1 GiB
    device-to-device copy (bytes read + written per second) and a loop of independent MFMAs without memory
    traffic per input type (bsr_probe_mfma)."""
    import torch
    import paper_2007_13055_amd as lib
    so = lib.load_library()
    out = {}
    src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
    dst = torch.empty_like(src)
    _, ev, _ = _time_steps(lambda: dst.copy_(src), 20, 3, 0)
    out["copy_1GiB_GBs"] = 2 * src.numel() * 4 / (ev / 20) / 1e9
    del src, dst
    sink = torch.zeros(1, device="cuda")
    for name, code in (("f32", 0), ("f16", 1), ("bf16", 2)):
        flops = ctypes.c_double(0.0)

        def fn():
            st = so.bsr_probe_mfma(code, 2000, sink.data_ptr(), torch.cuda.current_stream().cuda_stream, ctypes.byref(flops))
            if st != 0:
                raise RuntimeError(f"bsr_probe_mfma: status {st}")
        _, ev, _ = _time_steps(fn, 5, 2, 0)
        out[f"mfma_{name}_TFLOPs"] = flops.value / (ev / 5) / 1e12
    return out


def _cpu_baseline(p):
    """The oracle as it stands, timed on this machine's host cores.  Small workloads: the whole product, best of 5.
    The skewed workload: the whole product once (about 15 core-seconds on 16 threads)."""
    import numpy as np
    import oracle
    if p.name == "skewed":
        t0 = time.perf_counter()
        oracle.bsr_spmm(p.X, p.block_data, p.block_indices, p.index_pointer, p.n)
        best = time.perf_counter() - t0
        flops = p.flops
        sample = f"the whole 'skewed' workload (all {p.m} rows of X against the whole W), one run ({best:.2f} s)"
    else:
        best = float("inf")
        for _ in range(5):
            t0 = time.perf_counter()
            oracle.bsr_spmm(p.X, p.block_data, p.block_indices, p.index_pointer, p.n)
            best = min(best, time.perf_counter() - t0)
        flops = p.flops
        sample = f"the whole '{p.name}' workload, best of 5 runs ({best * 1e3:.1f} ms each)"
    return {"value": flops / best / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": sample + "; plain double-precision loops, a correctness reference and not a tuned CPU SpMM"}


def _entry(p, W, r, steps, chunk, floor_us, cold):
    """Everything measured for one workload: graph-replay and plain-launch time, roofline, spread, cold operands."""
    s = r["event_s"] / steps
    sp_steps = min(steps, 200)
    e = {"us_per_call": s * 1e6, "tflops": p.flops / s / 1e12, "path": r["path"], "launch": r["mode"],
         "eager_us_per_call": r["eager_wall_s"] / steps * 1e6, "launch_floor_us": floor_us,
         "roofline": _roofline(p, s),
         "spread": _spread(p, W, r["X"], r["Y"], sp_steps, _graph_chunk(sp_steps, chunk))}
    if cold:
        e["cold"] = _cold(p, min(steps, 200))
    return e


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--graph-chunk", type=int, default=100,
                    help="most launches per captured HIP graph (0 = plain launches only)")
    ap.add_argument("--no-all-configs", action="store_true", help="skip the other four workloads")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--no-cold", action="store_true", help="skip the runs on operands rotated out of the last-level cache")
    ap.add_argument("--no-peaks", action="store_true", help="skip the copy and MFMA-loop measurements of this chip")
    ap.add_argument("--sibling", action="store_true",
                    help="also time the sibling products (Z = G * W through the handle of W^T, and the sampled product)")
    ap.add_argument("--paper-grid", action="store_true",
                    help="also time the 36 cells of the paper's own shape grid (m = 1, 8) and add them as 'paper_grid'")
    ap.add_argument("--workload", default="skewed", choices=list(CONFIG_ID),
                    help="workload of the headline line (default: the largest, 'skewed')")
    ap.add_argument("--row-subset", default="", metavar="longest:N|rest:N",
                    help="analysis: keep only the N longest block-rows of the headline workload, or all but those")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MiB",
                    help="only run 20 device-to-device copies of this many MiB and exit: the reference a "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE reading is scaled by")
    a = ap.parse_args()
    if a.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (the product needs no exchange between GPUs: "
                 "block-rows of W and rows of X both split without one). Use --gpus 1.")
    if a.steps < 1 or a.warmup < 0:
        sys.exit("bench.py: --steps must be at least 1 and --warmup non-negative")
    if a.row_subset:
        global ROW_SUBSET
        which, _, count = a.row_subset.partition(":")
        if which not in ("longest", "rest") or not count.isdigit():
            sys.exit("bench.py: --row-subset takes longest:N or rest:N")
        ROW_SUBSET = (which, int(count))
        a.no_all_configs = True                      # the subset applies to the headline workload only
    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP path has no CPU fallback")
    import paper_2007_13055_amd as lib
    lib.load_library()
    torch.cuda.set_device(0)
    if a.copy_calibration > 0:
        src = torch.ones(a.copy_calibration * (1 << 20) // 4, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(20):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_MiB": a.copy_calibration, "copies": 20}))
        return
    headline = CONFIG_ID[a.workload]
    chunk = _graph_chunk(a.steps, a.graph_chunk)
    floor_us = _launch_floor(a.steps, chunk) * 1e6
    cold = not a.no_cold

    p, W, r = _bench_config(headline, a.steps, a.warmup, chunk)
    e = _entry(p, W, r, a.steps, a.graph_chunk, floor_us, cold)
    sec = r["event_s"] / a.steps                      # HIP events on the launch stream: the clock of every figure below
    out = {
        "metric": "effective TFLOP/s of bsr_spmm (2*m*nnzb*bs_r*bs_c per call)",
        "value": p.flops / sec / 1e12, "unit": "TFLOP/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ramp_ms": RAMP_S * 1e3,
        "ms_per_step": sec * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": p.in_dtype, "data": "synthetic",
        "config": {"workload": WORKLOAD_TEXT[p.name],
                   "m": p.m, "k": p.k, "n": p.n, "bs_r": p.bs_r, "bs_c": p.bs_c, "nnzb": p.nnzb,
                   "path": r["path"], "launch": r["mode"], "seed": p.seed},
        "roofline": e["roofline"],
        "wall_ms_per_step": r["wall_s"] / a.steps * 1e3,
        "eager_ms_per_step": r["eager_wall_s"] / a.steps * 1e3,
        "launch_floor_us": floor_us,
        "spread": e["spread"],
    }
    if cold:
        out["cold"] = e["cold"]
    out["cpu_baseline"] = None if a.no_cpu else _cpu_baseline(p)
    if not a.no_peaks:
        out["measured_peaks"] = mp = _measured_peaks()
        rf = out["roofline"]
        rf["frac_of_measured_peak"] = (rf["achieved"] / mp["copy_1GiB_GBs"] if rf["bound"] == "hbm"
                                       else rf["achieved"] / mp[f"mfma_{p.in_dtype}_TFLOPs"])
    del W

    if not a.no_all_configs:
        table = {}
        for cid in (c for c in (1, 2, 3, 4, 5) if c != headline):
            steps = 200 if cid == 5 else 1000
            ch = _graph_chunk(steps, a.graph_chunk)
            q, Wq, rq = _bench_config(cid, steps, 20, ch)
            table[q.name] = _entry(q, Wq, rq, steps, a.graph_chunk, floor_us, cold)
            if not a.no_peaks:
                rf = table[q.name]["roofline"]
                rf["frac_of_measured_peak"] = (rf["achieved"] / mp["copy_1GiB_GBs"] if rf["bound"] == "hbm"
                                               else rf["achieved"] / mp[f"mfma_{q.in_dtype}_TFLOPs"])
            del Wq
        out["per_config"] = table
    if a.paper_grid:
        out["paper_grid"] = _paper_grid(1000, 100)
    if a.sibling:
        import workloads as wl
        out["sibling"] = _sibling(wl.config(headline), a.steps, chunk)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
