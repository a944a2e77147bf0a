#!/usr/bin/env python3
"""The two schedules of the library side by side on one shape and mode (k != 0), one MI355X.

    python -m paper_2510_14891_amd.schedule_bench --dims 16384,2048,64 --rank 128 [--dtype f64] [--mode 2]

Times `mttkrp_dense` three ways through the `contract_rows` tuning key: as the planner
chooses, with the streaming kernel forced (`contract_rows` = 2) and with the second schedule
(MFMA contraction over mode 0) forced (`contract_rows` = 1), and prints one markdown table row
per setting: milliseconds (main kernel + combine kernel, median of the timed calls, HIP events
recorded by the library on the launch stream), GB/s of X, executed TFLOP/s (2 N R), the plan,
and the normwise difference from the planner's result (both schedules compute the same sums in
another order).  Random data made on the GPU; `--mode` is 1-based like the paper's mode k.
The settings are run twice and the second pass is reported, so that none of them sits in the
clock ramp of a cold GPU.
"""
from __future__ import annotations

import argparse
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--dims", required=True, help="comma-separated extents, first index fastest")
    ap.add_argument("--rank", type=int, required=True)
    ap.add_argument("--dtype", default="f64", choices=["f64", "f32"])
    ap.add_argument("--mode", type=int, default=2, help="1-based mode k (not 1: the schedules differ for k != first)")
    ap.add_argument("--reps", type=int, default=11)
    args = ap.parse_args()

    import torch
    from paper_2510_14891_amd import binding as mt

    if not torch.cuda.is_available():
        print("schedule_bench: no GPU visible", file=sys.stderr)
        return 3
    mt.lib()
    dims = tuple(int(t) for t in args.dims.split(","))
    k = args.mode - 1
    if not 1 <= k < len(dims):
        print("schedule_bench: --mode must be between 2 and the number of modes", file=sys.stderr)
        return 2
    R = args.rank
    dt = torch.float64 if args.dtype == "f64" else torch.float32
    sb = 8 if args.dtype == "f64" else 4
    n = 1
    for d in dims:
        n *= d
    g = torch.Generator(device="cuda")
    g.manual_seed(1)
    X = torch.rand(n, dtype=dt, device="cuda", generator=g)
    A = [torch.rand((I, R), dtype=dt, device="cuda", generator=g) for I in dims]
    M = torch.empty((dims[k], R), dtype=dt, device="cuda")

    settings = (("planner", 0), ("streaming kernel", 2), ("second schedule", 1))
    ref = None
    rows = {}
    try:
        for rep in range(2):
            for name, val in settings:
                mt.mttkrp_tune_set("contract_rows", val)
                desc = mt.mttkrp_plan_describe(dims, R, k, sb)
                for _ in range(3):
                    mt.mttkrp_dense(X, dims, A, k, M=M)
                torch.cuda.synchronize()
                mt.mttkrp_timing_enable(True)
                for _ in range(args.reps):
                    mt.mttkrp_dense(X, dims, A, k, M=M)
                torch.cuda.synchronize()
                c = mt.mttkrp_timing_count()
                ts = sorted(sum(mt.mttkrp_timing_get(i)) for i in range(c - args.reps, c))
                ms = ts[args.reps // 2]
                if ref is None:
                    ref = M.clone()
                diff = float(torch.linalg.vector_norm(M - ref) / torch.linalg.vector_norm(ref))
                rows[name] = (ms, desc, diff)
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


if __name__ == "__main__":
    sys.exit(main())
