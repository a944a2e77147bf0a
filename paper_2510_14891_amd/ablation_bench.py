#!/usr/bin/env python3
"""Side-by-side of the paper's own schedules and the streaming kernel on one MI355X.

    python -m paper_2510_14891_amd.ablation_bench [--workload NAME] [--reps N] [--widths 2,4,6,8,10,12]

For every mode of the workload (default: the paper's 4-way tensor shape
401 x 201 x 12 x 501, R = 32, random values as in the paper's Sec. IV) it times

  * the streaming kernel of this library (mttkrp_dense),
  * MTTKRP-ELEM (Sec. III-B),
  * MTTKRP-TILE (Sec. III-D) at the heuristic tile width of Eq. (heuristic) for this GPU and at
    every width of the paper's sweep (Table "width"),
  * MTTKRP-SUB (Sec. III-C) where its serial walk is expected to finish within a few seconds,

and prints a markdown table: milliseconds, GFLOP/s in the paper's convention (N R d / t / 1024^3,
comparable with its tables), and the analytical times T_inf, T_0,LM, T_0 of Sec. IV-B for this
machine's nominal rates.  Timing: HIP events on the stream the kernels run on.
"""
from __future__ import annotations

import argparse
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_BPS = 8.0e12
FP_PEAK = {"f64": 78.6e12, "f32": 157.3e12}
L1_BYTES = 32 * 1024          # vector L1 per compute unit
TILES_PER_CU = 64             # 32 resident wavefronts x two 32-lane team threads at R = 32
SUB_NS_PER_ENTRY = 60.0       # rough serial cost used only to decide whether SUB is run


def time_ms(fn, reps, warm=1):
    import torch
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
    ev[0].record()
    for i in range(reps):
        fn()
        ev[i + 1].record()
    torch.cuda.synchronize()
    ts = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(reps))
    return ts[len(ts) // 2]


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="paperA_401x201x12x501_f64_R32")
    ap.add_argument("--reps", type=int, default=5)
    ap.add_argument("--widths", default="2,4,6,8,10,12")
    ap.add_argument("--sub-budget", type=float, default=4.0, help="seconds one SUB launch may be expected to take")
    args = ap.parse_args()

    import torch
    from paper_2510_14891_amd import binding as mt, inputs, perf_model

    if not torch.cuda.is_available():
        print("ablation_bench: no GPU visible", file=sys.stderr)
        return 3
    mt.lib()
    w = inputs.WORKLOADS[args.workload]
    X = inputs.make_tensor(w, device="cuda")
    A = inputs.make_factors(w, device="cuda")
    widths = [int(t) for t in args.widths.split(",") if t]
    hw, hvol = mt.mttkrp_tile_volume(w.dims, L1_BYTES, w.itemsize, TILES_PER_CU)
    f_paper = perf_model.flops_paper(w.dims, w.R)

    def gf(ms):
        return perf_model.gflops_paper_units(f_paper, ms * 1e-3)

    print("# Paper schedules vs streaming kernel: %s (%s, R = %d), one MI355X" % (w.name, w.dtype, w.R))
    print()
    print("Tile-volume heuristic for this GPU (s_LM = %d B of L1 per CU, c = %d tiles per CU): width %d, "
          "N_T = %d." % (L1_BYTES, TILES_PER_CU, hw, hvol))
    print("GFLOP/s in the paper's convention: N R d / t / 1024^3.  ms = median of %d launches (stream: of %d, "
          "after 20 warm-up launches; it includes the combine kernel)." % (args.reps, max(args.reps, 15)))
    print()
    cols = ["stream"] + ["ELEM"] + ["TILE w=%d%s" % (x, " (heur.)" if x == hw else "") for x in sorted(set(widths + [hw]))] + ["SUB"]
    print("| mode | " + " | ".join(cols) + " | T_inf / T_0,LM(l=16) / T_0 model ms |")
    print("|---" * (len(cols) + 2) + "|")
    sums = {c: 0.0 for c in cols}
    done = {c: 0 for c in cols}
    for k in range(w.ndim):
        M = torch.empty((w.dims[k], w.R), dtype=w.torch_dtype, device="cuda")
        cells = []
        ms = time_ms(lambda: mt.mttkrp_dense(X, w.dims, A, k, M=M), max(args.reps, 15), warm=20)
        ref = M.clone()
        cells.append((cols[0], ms))
        ms = time_ms(lambda: mt.mttkrp_ablation(mt.MTTKRP_SCHEDULE_ELEM, X, w.dims, A, k, M=M), args.reps)
        err = float(torch.linalg.vector_norm(M - ref) / torch.linalg.vector_norm(ref))
        assert err < 1e-4, ("ELEM", k, err)
        cells.append((cols[1], ms))
        ci = 2
        for x in sorted(set(widths + [hw])):
            ms = time_ms(lambda: mt.mttkrp_ablation(mt.MTTKRP_SCHEDULE_TILE, X, w.dims, A, k, tile_width=x, M=M),
                         args.reps)
            err = float(torch.linalg.vector_norm(M - ref) / torch.linalg.vector_norm(ref))
            assert err < 1e-4, ("TILE", x, k, err)
            cells.append((cols[ci], ms))
            ci += 1
        n_s = w.numel // w.dims[k]
        if n_s * SUB_NS_PER_ENTRY * 1e-9 * max(1, w.R // 64) <= args.sub_budget:
            ms = time_ms(lambda: mt.mttkrp_ablation(mt.MTTKRP_SCHEDULE_SUB, X, w.dims, A, k, M=M), 1)
            cells.append((cols[ci], ms))
        else:
            cells.append((cols[ci], None))
        n_t = hvol
        t_inf = perf_model.predicted_time(f_paper, perf_model.m_inf(w.dims, w.R, w.itemsize), FP_PEAK[w.dtype], HBM_BPS)
        t_lm = perf_model.predicted_time(f_paper, perf_model.m_0_lm(w.dims, w.R, w.itemsize, k, n_t, 16.0),
                                         FP_PEAK[w.dtype], HBM_BPS)
        t_0 = perf_model.predicted_time(f_paper, perf_model.m_0(w.dims, w.R, w.itemsize, k, n_t), FP_PEAK[w.dtype], HBM_BPS)
        row = []
        for name, ms in cells:
            if ms is None:
                row.append("not run (serial walk of %d entries per team thread)" % n_s)
            else:
                row.append("%.3f ms, %.0f" % (ms, gf(ms)))
                sums[name] += ms
                done[name] += 1
        print("| %d | %s | %.2f / %.2f / %.2f |" % (k + 1, " | ".join(row), t_inf * 1e3, t_lm * 1e3, t_0 * 1e3), flush=True)
    row = []
    for c in cols:
        if done[c] == w.ndim:
            row.append("%.3f ms, %.0f" % (sums[c] / w.ndim, gf(sums[c] / w.ndim)))
        else:
            row.append("—")
    print("| mean | " + " | ".join(row) + " | |")
    return 0


if __name__ == "__main__":
    sys.exit(main())
