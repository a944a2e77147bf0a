#!/usr/bin/env python3
"""Benchmark of the matrix-free dense MTTKRP on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-configs]
    python bench.py --schedules --dims 16384,2048,64 --rank 128 [--dtype f64] [--mode 2]

One "step" is one pass of the whole hot path over the workload: one MTTKRP
call per mode (k = 0..d-1) on the same resident tensor, i.e. d streaming
passes over X.  The default workload is benchmark configuration 2
(1024 x 1024 x 512 fp64, R = 32, 4 GiB), the one the target (>= 70 % of HBM
bandwidth for R <= 32) is quoted on.  Inputs are seeded synthetic data already
resident in HBM when the timed region starts.

Prints ONE JSON line.  ``value`` is GB/s of X streamed over the whole step
(d * N * s_f / t_step, wall clock between device synchronisations).
``roofline`` is for the main kernel of the calls (the streaming kernel, or the
row-contraction kernel where the planner takes the second schedule):
algorithmic bytes per launch, s_f (N + R sum_n I_n) (the paper's
infinite-cache model m_inf, Sec. IV-B), or executed flops 2 N R where the
rank makes the path compute-bound, divided by the mean launch duration
measured with HIP events recorded by the library on the launch stream around
each launch of the timed region.  ``configs`` repeats the measurement (its own
warm-up and timed steps, same HIP-event timing) for every other benchmark
configuration and for the paper's two tensor shapes, each with its own
``roofline`` object and per-mode figures.  ``cpu_baseline`` times the CPU oracle
(long-double accumulation, as used for parity) on a bounded slab of the same
tensor on the host cores; ``cpu_baseline_native`` the same loop with the
accumulator in the data type.

``--schedules`` instead times one shape and mode (k != first) three ways, as the
planner chooses, with the streaming kernel forced and with the second schedule
(MFMA contraction over mode 0) forced, and prints a markdown table.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0            # MI355X HBM3E, published
FP_PEAK_TFLOPS = {"f64": 78.6, "f32": 157.3}   # dense MFMA = vector peak for these types
DEFAULT_WORKLOAD = "c2_1024x1024x512_f64_R32"
# measured next to the default workload when it is the one that is run
OTHER_CONFIGS = (
    "c1_64x64x64_f64_R16",
    "c3_192x192x192x192_f64_R16",
    "c4_48x48x48x48x48_f32_R64",
    "c5_16384x2048x64_f64_R4",
    "c5_16384x2048x64_f64_R8",
    "c5_16384x2048x64_f64_R128",
    "paperA_401x201x12x501_f64_R32",
    "paperA_401x201x12x501_f64_R10",
    "paperB_129x129x129x12x39_f64_R32",
    "paperB_cp10_129x129x129x12x39_f64_R10",
)


def measured_traffic(workload: str):
    """HBM bytes per main-kernel launch from the rocprofv3 counter runs summarised under
    profiles/ (fetched + written, each scaled by what the same counter reads for a plain copy of
    known size), or None when none was recorded for the workload."""
    try:
        with open(os.path.join(ROOT, "profiles", "pmc_traffic.json")) as f:
            return json.load(f).get(workload)
    except (OSError, ValueError):
        return None


def roofline_of(w, kernel_ms, launches, perf_model):
    """The roofline object of one workload from the mean duration of its main kernel."""
    alg_bytes = perf_model.m_inf(w.dims, w.R, w.itemsize)   # per launch
    exec_flops = 2.0 * w.numel * w.R
    mem_bound = exec_flops / (FP_PEAK_TFLOPS[w.dtype] * 1e12) <= alg_bytes / (HBM_PEAK_GBPS * 1e9)
    if mem_bound:
        achieved = alg_bytes / (kernel_ms * 1e-3) / 1e9
        r = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
             "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4)}
    else:
        achieved = exec_flops / (kernel_ms * 1e-3) / 1e12
        r = {"bound": "mfma", "achieved": round(achieved, 2),
             "peak": FP_PEAK_TFLOPS[w.dtype], "unit": "TFLOP/s",
             "frac": round(achieved / FP_PEAK_TFLOPS[w.dtype], 4)}
    r["kernel"] = "mttkrp_stream_kernel (mttkrp_rowsum_kernel for modes on the second schedule)"
    r["kernel_ms_mean"] = round(kernel_ms, 4)
    r["launches_timed"] = launches
    r["algorithmic_bytes_per_launch"] = alg_bytes
    r["executed_flops_per_launch"] = exec_flops
    detail = measured_traffic(w.name)
    r["traffic"] = detail["total_bytes"] if detail else None
    r["traffic_detail"] = detail
    return r


def run_workload(mt, perf_model, w, X, A, steps, warmup):
    """W warm-up steps, then exactly K timed steps between two synchronisations, with the
    library's HIP events around every kernel.  Returns (ms_per_step, per_mode, roofline)."""
    import torch
    M = [torch.empty((I, w.R), dtype=w.torch_dtype, device=X.device) for I in w.dims]

    def step():
        for k in range(w.ndim):
            mt.mttkrp_dense(X, w.dims, A, k, M=M[k])

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    mt.mttkrp_timing_enable(True)
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    t_wall = time.perf_counter() - t0
    mt.mttkrp_timing_enable(False)
    ms_per_step = 1e3 * t_wall / steps

    n_calls = mt.mttkrp_timing_count()
    first = max(0, n_calls - 512)           # the library keeps the last 512 timed calls
    first += (-first) % w.ndim              # start on a mode-1 call
    s_ms = [[] for _ in range(w.ndim)]
    c_ms = [[] for _ in range(w.ndim)]
    for i in range(first, n_calls):
        a, b = mt.mttkrp_timing_get(i)
        s_ms[i % w.ndim].append(a)
        c_ms[i % w.ndim].append(b)
    per_mode = []
    main_all = []
    xb = w.numel * w.itemsize
    mem_floor = perf_model.m_inf(w.dims, w.R, w.itemsize) / (HBM_PEAK_GBPS * 1e9) * 1e3
    fp_floor = 2.0 * w.numel * w.R / (FP_PEAK_TFLOPS[w.dtype] * 1e12) * 1e3
    for k in range(w.ndim):
        main_all += s_ms[k]
        sm = sum(s_ms[k]) / len(s_ms[k])
        cm = sum(c_ms[k]) / len(c_ms[k])
        plan = mt.mttkrp_plan_describe(w.dims, w.R, k, w.itemsize)
        per_mode.append({
            "mode": k + 1,
            "main_kernel_ms": round(sm, 4),
            "main_kernel_ms_min": round(min(s_ms[k]), 4),
            "combine_kernel_ms": round(cm, 4),
            "GBps_X": round(xb / (sm + cm) / 1e6, 1),
            "pct_hbm": round(100 * xb / (sm + cm) / 1e6 / HBM_PEAK_GBPS, 1),
            "gflops_exec_2NR": round(2 * w.numel * w.R / (sm + cm) / 1e6, 1),
            "pct_fp_peak": round(100 * 2 * w.numel * w.R / (sm + cm) / 1e9 / FP_PEAK_TFLOPS[w.dtype], 1),
            "gflops_paper_NRd": round(w.numel * w.R * w.ndim / (sm + cm) / 1e6, 1),
            "roofline_frac": round(max(mem_floor, fp_floor) / sm, 4),
            "schedule": "rows" if "shape=rows" in plan else "streaming",
            "plan": plan,
        })
    kernel_ms = sum(main_all) / len(main_all)
    return ms_per_step, per_mode, roofline_of(w, kernel_ms, len(main_all), perf_model)


def shared_sweep_entry(mt, w, X, A, budget_s=0.12):
    """The all-modes sweep that shares partial contractions (two passes over X) beside the
    same d results from d separate calls: wall time per sweep of each, after a warm-up, for
    about ``budget_s`` seconds each.  Not part of ``value``."""
    import torch
    nbytes = mt.mttkrp_dense_all_modes_shared_bytes(w.dims, w.R, w.itemsize)
    if nbytes == 0:
        return {"supported": False}
    M = [torch.empty((I, w.R), dtype=w.torch_dtype, device=X.device) for I in w.dims]
    out = {"supported": True, "workspace_bytes": nbytes,
           "workspace_over_x": round(nbytes / (w.numel * w.itemsize), 4)}
    for label, fn in (("separate", mt.mttkrp_dense_all_modes), ("shared", mt.mttkrp_dense_all_modes_shared)):
        fn(X, w.dims, A, M_out=M)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        fn(X, w.dims, A, M_out=M)
        torch.cuda.synchronize()
        t1 = max(time.perf_counter() - t0, 1e-5)
        n = int(min(300, max(3, math.ceil(budget_s / t1))))
        for _ in range(n):
            fn(X, w.dims, A, M_out=M)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            fn(X, w.dims, A, M_out=M)
        torch.cuda.synchronize()
        out["ms_" + label] = round(1e3 * (time.perf_counter() - t0) / n, 4)
    out["speedup"] = round(out["ms_separate"] / out["ms_shared"], 3)
    return out


def config_entry(mt, perf_model, inputs, w, X, A, sweep=True):
    """One element of ``configs``: warm up for about 0.15 s of load (the shader clock settles over
    the first ~0.1 s), then time about 0.25 s worth of steps."""
    import torch
    for k in range(w.ndim):
        mt.mttkrp_dense(X, w.dims, A, k)
    torch.cuda.synchronize()                 # first calls also grow the workspace
    t0 = time.perf_counter()
    for k in range(w.ndim):
        mt.mttkrp_dense(X, w.dims, A, k)
    torch.cuda.synchronize()
    t_step = max(time.perf_counter() - t0, 1e-5)
    warmup = int(min(200, max(3, math.ceil(0.15 / t_step))))
    steps = int(min(512 // w.ndim, max(5, math.ceil(0.25 / t_step))))
    ms_per_step, per_mode, roofline = run_workload(mt, perf_model, w, X, A, steps, warmup)
    xb = w.numel * w.itemsize
    return {
        "workload": w.name, "dims": list(w.dims), "R": w.R, "dtype": w.dtype, "x_bytes": xb,
        "steps": steps, "warmup": warmup, "ms_per_step": round(ms_per_step, 4),
        "value": round(w.ndim * xb / (ms_per_step * 1e-3) / 1e9, 1), "unit": "GB/s",
        "per_mode": per_mode, "roofline": roofline,
        "shared_sweep": shared_sweep_entry(mt, w, X, A) if sweep else None,
    }


def cpu_baseline(w, X, A, budget_s, native):
    """Time the oracle on the slab X[..., :s] of the workload (all modes).

    The slab is the first s entries of the slowest mode, which is a contiguous
    prefix of X, so it is the same tensor with a shorter last mode; oracle work
    is linear in s.  s is chosen from a short calibration run so that the timed
    part takes about ``budget_s`` seconds.
    """
    from oracle import mttkrp_oracle as orc
    from paper_2510_14891_amd import inputs
    orc.build()
    cores = orc.max_threads()
    lead = w.numel // w.dims[-1]

    def run(s):
        dims = tuple(w.dims[:-1]) + (s,)
        Xs = inputs.as_ndarray_view(X[: lead * s].cpu(), dims)
        As = [a.cpu().numpy() for a in A]
        As[-1] = As[-1][:s]
        t0 = time.perf_counter()
        for k in range(w.ndim):
            orc.mttkrp(Xs, As, k, native_acc=native)
        return time.perf_counter() - t0

    s0 = max(1, min(w.dims[-1], (1 << 22) // max(lead, 1)))
    t_cal = run(s0)
    s = int(max(s0, min(w.dims[-1], s0 * budget_s / max(t_cal, 1e-3))))
    t = run(s) if s > s0 else t_cal
    x_bytes = w.ndim * lead * s * w.itemsize
    return {
        "value": round(x_bytes / t / 1e9, 3),
        "unit": "GB/s of X streamed",
        "cores": cores,
        "kind": "oracle",
        "accumulator": ("the data type (%s)" % w.dtype) if native else "long double",
        "seconds": round(t, 3),
        "gflops_paper": round(w.ndim * (lead * s) * w.R * w.ndim / t / 1e9, 2),
        "sample": "slab X[..., :%d] of the last mode (%d of %d entries, %.1f %% of the tensor), "
                  "all %d modes, one run" % (s, lead * s, w.numel, 100.0 * s / w.dims[-1], w.ndim),
    }


def compare_schedules(args) -> int:
    """The library's two schedules side by side on one shape and mode (k != first)."""
    import torch
    from paper_2510_14891_amd import binding as mt
    mt.lib()
    dims = tuple(int(t) for t in args.dims.split(","))
    k = args.mode - 1
    if not 1 <= k < len(dims):
        print("bench.py --schedules: --mode must be between 2 and the number of modes", file=sys.stderr)
        return 2
    R = args.rank
    dt = torch.float64 if args.dtype == "f64" else torch.float32
    sb = 8 if args.dtype == "f64" else 4
    n = math.prod(dims)
    g = torch.Generator(device="cuda")
    g.manual_seed(1)
    X = torch.rand(n, dtype=dt, device="cuda", generator=g)
    A = [torch.rand((I, R), dtype=dt, device="cuda", generator=g) for I in dims]
    M = torch.empty((dims[k], R), dtype=dt, device="cuda")
    settings = (("planner", 0), ("streaming kernel", 2), ("second schedule", 1))
    reps, ref, rows = 11, None, {}
    try:
        for _ in range(2):                   # the second pass is reported: none sits in the clock ramp
            for name, val in settings:
                mt.mttkrp_tune_set("contract_rows", val)
                desc = mt.mttkrp_plan_describe(dims, R, k, sb)
                for _ in range(3):
                    mt.mttkrp_dense(X, dims, A, k, M=M)
                torch.cuda.synchronize()
                mt.mttkrp_timing_enable(True)
                for _ in range(reps):
                    mt.mttkrp_dense(X, dims, A, k, M=M)
                torch.cuda.synchronize()
                c = mt.mttkrp_timing_count()
                ts = sorted(sum(mt.mttkrp_timing_get(i)) for i in range(c - reps, c))
                mt.mttkrp_timing_enable(False)
                if ref is None:
                    ref = M.clone()
                diff = float(torch.linalg.vector_norm(M - ref) / torch.linalg.vector_norm(ref))
                rows[name] = (ts[reps // 2], desc, diff)
    finally:
        mt.mttkrp_tune_set("contract_rows", 0)
    print("| shape | R | type | mode | setting | ms | GB/s of X | TFLOP/s | schedule | rel. difference |")
    print("|---|---|---|---|---|---|---|---|---|---|")
    for name, _ in settings:
        ms, desc, diff = rows[name]
        sched = "second (rows)" if "shape=rows" in desc else "streaming"
        print("| %s | %d | %s | %d | %s | %.3f | %.0f | %.1f | %s | %.1e |" % (
            "x".join(str(d) for d in dims), R, args.dtype, args.mode, name, ms, n * sb / ms / 1e6,
            2.0 * n * R / ms / 1e9, sched, diff))
    return 0


def time_shape(args) -> int:
    """Every mode of one arbitrary shape (--dims, --rank, --dtype) on random data, as a
    Markdown row per mode: median kernel time of 15 calls after a warm-up, the plan, and the
    fraction of the shape's roofline bound."""
    import torch
    from paper_2510_14891_amd import binding as mt, perf_model
    if not torch.cuda.is_available():
        print("bench.py --shape: no GPU visible", file=sys.stderr)
        return 3
    mt.lib()
    dims = tuple(int(t) for t in args.dims.split(","))
    R = args.rank
    dt = torch.float64 if args.dtype == "f64" else torch.float32
    sb = 8 if args.dtype == "f64" else 4
    n = math.prod(dims)
    g = torch.Generator(device="cuda")
    g.manual_seed(1)
    X = torch.rand(n, dtype=dt, device="cuda", generator=g)
    A = [torch.rand((I, R), dtype=dt, device="cuda", generator=g) for I in dims]
    M = [torch.empty((I, R), dtype=dt, device="cuda") for I in dims]
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < 0.3:
        for k in range(len(dims)):
            mt.mttkrp_dense(X, dims, A, k, M=M[k])
        torch.cuda.synchronize()
    floor = max(perf_model.m_inf(dims, R, sb) / (HBM_PEAK_GBPS * 1e9),
                2.0 * n * R / (FP_PEAK_TFLOPS[args.dtype] * 1e12)) * 1e3
    reps = 15
    print("| shape | R | type | mode | main + combine ms | GB/s of X | TFLOP/s | roofline fraction (main kernel) | rows per wavefront x row blocks | items x steps |")
    print("|---|---|---|---|---|---|---|---|---|---|")
    for k in range(len(dims)):
        for _ in range(3):
            mt.mttkrp_dense(X, dims, A, k, M=M[k])
        torch.cuda.synchronize()
        mt.mttkrp_timing_enable(True)
        for _ in range(reps):
            mt.mttkrp_dense(X, dims, A, k, M=M[k])
        torch.cuda.synchronize()
        c = mt.mttkrp_timing_count()
        tm = sorted(mt.mttkrp_timing_get(i)[0] for i in range(c - reps, c))[reps // 2]
        tc = sorted(mt.mttkrp_timing_get(i)[1] for i in range(c - reps, c))[reps // 2]
        mt.mttkrp_timing_enable(False)
        desc = dict(t.split("=") for t in mt.mttkrp_plan_describe(dims, R, k, sb).split())
        rows = ("%s x %s" % (desc.get("rows_per_wave"), desc.get("row_blocks"))
                if "rows_per_wave" in desc else
                ("last mode over all others" if desc.get("shape") == "leading" else "second schedule"))
        print("| %s | %d | %s | %d | %.3f + %.3f | %.0f | %.1f | %.3f | %s | %s x %s |" % (
            "x".join(str(d) for d in dims), R, args.dtype, k + 1, tm, tc, n * sb / (tm + tc) / 1e6,
            2.0 * n * R / (tm + tc) / 1e9, floor / tm, rows, desc.get("items"), desc.get("steps_per_item")))
    return 0


def time_leading(args) -> int:
    """The partial contraction over the leading index (mttkrp_contract_leading_*) on a P x Q
    matrix of random data (--dims P,Q, --rank, --dtype): one Markdown row, wall clock of 20 calls
    between two synchronisations after 20 warm-up calls."""
    import torch
    from paper_2510_14891_amd import binding as mt
    if not torch.cuda.is_available():
        print("bench.py --leading: no GPU visible", file=sys.stderr)
        return 3
    mt.lib()
    P, Q = (int(t) for t in args.dims.split(","))
    R = args.rank
    dt = torch.float64 if args.dtype == "f64" else torch.float32
    sb = 8 if args.dtype == "f64" else 4
    g = torch.Generator(device="cuda")
    g.manual_seed(1)
    X = torch.rand(P * Q, dtype=dt, device="cuda", generator=g)
    K = torch.rand((P, R), dtype=dt, device="cuda", generator=g)
    T = torch.empty((Q, R), dtype=dt, device="cuda")
    for _ in range(20):
        mt.mttkrp_contract_leading(X, P, Q, K, T_out=T)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(20):
        mt.mttkrp_contract_leading(X, P, Q, K, T_out=T)
    torch.cuda.synchronize()
    ms = 1e3 * (time.perf_counter() - t0) / 20
    print("| P x Q | R | type | ms | GB/s of X | TFLOP/s |")
    print("|---|---|---|---|---|---|")
    print("| %d x %d | %d | %s | %.3f | %.0f | %.1f |" % (P, Q, R, args.dtype, ms, P * Q * sb / ms / 1e6,
                                                         2.0 * P * Q * R / ms / 1e9))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # defaults: the shader clock settles over the first ~0.1 s of sustained load, so warm up that long
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD)
    ap.add_argument("--no-configs", action="store_true",
                    help="skip the `configs` array (the other configurations, measured after the main one)")
    ap.add_argument("--no-sweep", action="store_true",
                    help="skip the `shared_sweep` objects (the all-modes sweeps timed beside the headline)")
    ap.add_argument("--cpu-budget", type=float, default=10.0,
                    help="seconds of oracle time for each of the two CPU baselines (0 = skip)")
    ap.add_argument("--copy-only", action="store_true",
                    help="run only K plain device copies of the X buffer (the known-size "
                         "kernel the rocprofv3 FETCH_SIZE/WRITE_SIZE counters are scaled by)")
    ap.add_argument("--schedules", action="store_true", help="compare the two schedules on --dims/--rank/--mode")
    ap.add_argument("--shape", action="store_true", help="time every mode of the shape --dims/--rank/--dtype")
    ap.add_argument("--leading", action="store_true",
                    help="time the partial contraction over the leading index on --dims P,Q / --rank / --dtype")
    ap.add_argument("--dims", default="16384,2048,64")
    ap.add_argument("--rank", type=int, default=128)
    ap.add_argument("--dtype", default="f64", choices=["f64", "f32"])
    ap.add_argument("--mode", type=int, default=2, help="1-based mode k for --schedules")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (the path is one GPU's share at its "
              "real shape; sharding over several GPUs is described in the design notes, not built). Use --gpus 1.", file=sys.stderr)
        return 2

    import torch
    from paper_2510_14891_amd import binding as mt, inputs, perf_model

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    mt.lib()   # fails loudly when the HIP library is missing
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.schedules:
        return compare_schedules(args)
    if args.shape:
        return time_shape(args)
    if args.leading:
        return time_leading(args)
    w = inputs.WORKLOADS[args.workload]
    X = inputs.make_tensor(w, device=dev)
    A = inputs.make_factors(w, device=dev)
    torch.cuda.synchronize()
    if args.copy_only:
        Y = torch.empty_like(X)
        for _ in range(args.steps):
            Y.copy_(X)
        torch.cuda.synchronize()
        print(json.dumps({"copy_only": True, "bytes_read_per_copy": w.numel * w.itemsize,
                          "bytes_written_per_copy": w.numel * w.itemsize, "copies": args.steps}))
        return 0

    # timed region: exactly K steps, wall clock between synchronisations.  The
    # library records HIP events on the launch stream around every kernel of
    # these K steps; they are read back after the region has ended.
    ms_per_step, per_mode, roofline = run_workload(mt, perf_model, w, X, A, args.steps, args.warmup)
    kernel_ms = roofline["kernel_ms_mean"]
    alg_bytes = roofline["algorithmic_bytes_per_launch"]
    exec_flops = roofline["executed_flops_per_launch"]

    x_gbps = w.ndim * w.numel * w.itemsize / (ms_per_step * 1e-3) / 1e9
    out = {
        "metric": "dense MTTKRP GB/s of X streamed (all modes), with GFLOP/s and % of "
                  "HBM/FP roofline per mode",
        "value": round(x_gbps, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic",
        "config": {"workload": w.name, "dims": list(w.dims), "R": w.R,
                   "modes_per_step": w.ndim, "x_bytes": w.numel * w.itemsize},
        "pct_hbm_peak": round(100 * x_gbps / HBM_PEAK_GBPS, 1),
        "gflops_exec_2NR": round(w.ndim * exec_flops / (ms_per_step * 1e-3) / 1e9, 1),
        "gflops_paper_NRd": round(w.ndim * w.numel * w.R * w.ndim / (ms_per_step * 1e-3) / 1e9, 1),
        "per_mode": per_mode,
        "roofline": roofline,
    }
    # What the box sustains on its own (outside the timed region): a read-only pass over the same X
    # buffer and back-to-back MFMAs of the data type for as many flops as one launch executes.
    stream_gbps = mt.mttkrp_calibrate_stream(X, launches=10)
    mfma_tflops = mt.mttkrp_calibrate_mfma(w.itemsize, exec_flops / 1e9, launches=10)
    floor_ms = max(alg_bytes / (stream_gbps * 1e9), exec_flops / (mfma_tflops * 1e12)) * 1e3
    out["ceilings_measured"] = {
        "stream_read_GBps": round(stream_gbps, 1),
        "mfma_TFLOPs": round(mfma_tflops, 2),
        "floor_ms_from_probes": round(floor_ms, 4),
        "floor_over_kernel_ms": round(floor_ms / kernel_ms, 4),
        "how": "mttkrp_calibrate_stream over X (non-temporal 16-byte loads only) and mttkrp_calibrate_mfma "
               "(independent 16x16x4 MFMAs on register operands, 2 N R flops per launch); floor = the larger "
               "of bytes / stream rate and flops / MFMA rate; the MFMA probe runs 32 wavefronts per CU and "
               "its clock drops further than the kernel's, so a ratio above 1 can occur",
    }
    # beside the headline (d separate MTTKRPs per step): the same d results from the sweep that
    # shares partial contractions between the modes
    if not args.no_sweep:
        out["shared_sweep"] = shared_sweep_entry(mt, w, X, A, budget_s=0.3)
    if args.cpu_budget > 0:
        out["cpu_baseline"] = cpu_baseline(w, X, A, args.cpu_budget, native=False)
        out["cpu_baseline_native"] = cpu_baseline(w, X, A, args.cpu_budget, native=True)

    # Every other configuration, each with its own warm-up, timed steps and roofline object
    # (same HIP-event timing).  Tensors that share a recipe (configuration 5's three ranks)
    # are generated once.
    if not args.no_configs and args.workload == DEFAULT_WORKLOAD:
        del X, A
        torch.cuda.empty_cache()
        configs = []
        cache_key, Xc = None, None
        for name in OTHER_CONFIGS:
            wc = inputs.WORKLOADS[name]
            key = (wc.dims, wc.dtype, wc.x_dist, wc.seed_id)
            if key != cache_key:
                Xc = None
                torch.cuda.empty_cache()
                Xc = inputs.make_tensor(wc, device=dev)
                cache_key = key
            Ac = inputs.make_factors(wc, device=dev)
            configs.append(config_entry(mt, perf_model, inputs, wc, Xc, Ac, sweep=not args.no_sweep))
        out["configs"] = configs
        if not args.no_sweep:
            out["shared_sweep_speedup_by_workload"] = dict(
                [(w.name, out["shared_sweep"].get("speedup"))] +
                [(c["workload"], c["shared_sweep"].get("speedup")) for c in configs])
        out["roofline_frac_by_workload"] = dict(
            [(w.name, roofline["frac"])] + [(c["workload"], c["roofline"]["frac"]) for c in configs])
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
