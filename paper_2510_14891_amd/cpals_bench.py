#!/usr/bin/env python3
"""CP-ALS on one MI355X: time per sweep and the share of it spent in the MTTKRP.

    python -m paper_2510_14891_amd.cpals_bench [--workload NAME] [--rank R] [--max-iters N] [--tol T] [--shared]

Default: the shape of the paper's 5-way tensor (129 x 129 x 129 x 12 x 39) filled with a seeded
rank-10 Kruskal tensor plus 1 % noise, R = 10, tolerance 1e-4 (the setting of the paper's CP-ALS
experiment, Sec. IV-C, at its smallest rank).  The MTTKRP share comes from the HIP events the
library records around its own kernels; the rest is "other CP-ALS operations" (Gram matrices,
Cholesky solve, normalisation, fit) plus one stream synchronisation per sweep.  With --shared
the sweeps share partial contractions between the modes (mttkrp_cpals_shared_f64: two passes
over X per sweep); the run is then followed by the plain driver on the same start, for the
time per sweep side by side and the largest difference of the fits.
"""
from __future__ import annotations

import argparse
import os
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="paperB_cp10_129x129x129x12x39_f64_R10")
    ap.add_argument("--rank", type=int, default=0, help="0 = the workload's rank")
    ap.add_argument("--max-iters", type=int, default=50)
    ap.add_argument("--tol", type=float, default=1e-4)
    ap.add_argument("--shared", action="store_true", help="sweeps that share partial contractions")
    args = ap.parse_args()

    import torch
    from paper_2510_14891_amd import binding as mt, inputs

    if not torch.cuda.is_available():
        print("cpals_bench: no GPU visible", file=sys.stderr)
        return 3
    mt.lib()
    w = inputs.WORKLOADS[args.workload]
    R = args.rank or w.R
    X = inputs.make_tensor(w, device="cuda")
    A0 = inputs.make_factors(w, device="cuda", R=R)
    torch.cuda.synchronize()

    # untimed warm-up of two sweeps (workspace growth, clocks)
    mt.mttkrp_cpals(X, w.dims, [a.clone() for a in A0], 2, 0.0)
    torch.cuda.synchronize()

    A = [a.clone() for a in A0]
    mt.mttkrp_timing_enable(True)
    t0 = time.perf_counter()
    lam, fits = mt.mttkrp_cpals(X, w.dims, A, args.max_iters, args.tol)
    torch.cuda.synchronize()
    t = time.perf_counter() - t0
    n_calls = mt.mttkrp_timing_count()
    mt.mttkrp_timing_enable(False)
    first = max(0, n_calls - 512)
    mttkrp_ms = 0.0
    for i in range(first, n_calls):
        a, b = mt.mttkrp_timing_get(i)
        mttkrp_ms += a + b
    if first > 0:       # only the last 512 calls are kept: scale to all of them
        mttkrp_ms *= n_calls / float(n_calls - first)
    sweeps = len(fits)
    print("# CP-ALS: %s, R = %d, tolerance %g, one MI355X" % (w.name, R, args.tol))
    print()
    print("| sweeps | final fit | total s | ms per sweep | MTTKRP ms per sweep (%d calls) | MTTKRP share | other ms per sweep |" % w.ndim)
    print("|---|---|---|---|---|---|---|")
    per = 1e3 * t / sweeps
    mper = mttkrp_ms / sweeps
    print("| %d | %.6f | %.3f | %.3f | %.3f | %.1f %% | %.3f |" % (sweeps, fits[-1], t, per, mper, 100 * mper / per, per - mper))
    print()
    print("fit per sweep: " + " ".join("%.5f" % f for f in fits))
    if args.shared:
        mt.mttkrp_cpals(X, w.dims, [a.clone() for a in A0], 2, 0.0, shared=True)
        torch.cuda.synchronize()
        A = [a.clone() for a in A0]
        t0 = time.perf_counter()
        lam_s, fits_s = mt.mttkrp_cpals(X, w.dims, A, args.max_iters, args.tol, shared=True)
        torch.cuda.synchronize()
        ts = time.perf_counter() - t0
        print()
        print("Sweeps that share partial contractions (two passes over X): %d sweeps, final fit %.6f, "
              "%.3f ms per sweep (%.2f x), largest |fit difference| over the common sweeps %.2e, workspace %.1f MiB"
              % (len(fits_s), fits_s[-1], 1e3 * ts / len(fits_s), per / (1e3 * ts / len(fits_s)),
                 max(abs(a - b) for a, b in zip(fits, fits_s)),
                 mt.mttkrp_dense_all_modes_shared_bytes(w.dims, R, 8) / 2**20))
    return 0


if __name__ == "__main__":
    sys.exit(main())
