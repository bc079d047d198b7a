"""Writes tests/golden/<workload>[_f<f>]_trajectory.json: the exact double-precision ALS trajectory of the oracle
on one of the named workloads (Section 2: per sweep update X with Theta fixed, then Theta with the new X;
weighted-lambda regulariser of equation (1); training RMSE as in Section 5.2 but on the training entries).

Calls only `oracle/` and the seeded input generator.  The Mid file (tests/golden/mid_trajectory.json) was
written by make_mid_trajectory.py, which this script generalises: any workload, any factor width.

    python tests/golden/make_trajectory.py --workload large_square            # 5 sweeps, f = 100
    python tests/golden/make_trajectory.py --workload mid --f 64              # factor-width sweep, 10 sweeps

Cost on 8 cores: large_square about 4 minutes per sweep and 25 GB; mid at f = 32 / 64 / 128 / 256 about
10 s / 35 s / 2 min / 9 min per sweep.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
import workload as W  # noqa: E402


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", required=True, choices=sorted(W.CONFIGS))
    ap.add_argument("--f", type=int, default=0, help="factor width (0 = the workload's own)")
    ap.add_argument("--sweeps", type=int, default=0, help="0 = the workload's own number of sweeps")
    ap.add_argument("--out", default="")
    args = ap.parse_args()
    w = W.CONFIGS[args.workload]
    if args.f and args.f != w.f:
        w = w.with_f(args.f)
    sweeps = args.sweeps or w.sweeps
    out_path = args.out or os.path.join(ROOT, "tests", "golden", f"{w.name}_trajectory.json")
    a = W.generate(w)
    cptr, cidx, cval = oracle.csr_to_csc(w.m, w.n, a.ptr, a.idx, a.val)
    X0, T0 = W.init_factors(w)
    X = X0.astype(np.float64)
    T = T0.astype(np.float64)
    # rows and columns whose final values are stored: seeded picks plus the heaviest and lightest of each side
    rng = np.random.default_rng(w.seed + 99)
    deg_r, deg_c = np.diff(a.ptr), np.diff(cptr)
    rows = np.unique(np.concatenate([rng.choice(w.m, 24, replace=False), np.argsort(deg_r, kind="stable")[[0, 1, -2, -1]]]))
    cols = np.unique(np.concatenate([rng.choice(w.n, 24, replace=False), np.argsort(deg_c, kind="stable")[[0, 1, -2, -1]]]))
    hist = []
    for s in range(sweeps):
        t0 = time.perf_counter()
        X = oracle.update_rows(a.ptr, a.idx, a.val, T, w.lam)
        T = oracle.update_rows(cptr, cidx, cval, X, w.lam)
        rec = {"sweep": s + 1, "rmse": oracle.rmse(a.ptr, a.idx, a.val, X, T),
               "objective": oracle.objective(a.ptr, a.idx, a.val, X, T, w.lam)}
        hist.append(rec)
        print(f"{w.name} sweep {s + 1}: rmse {rec['rmse']:.9f} J {rec['objective']:.6e} ({time.perf_counter() - t0:.1f} s)",
              flush=True)
    out = {
        "what": f"exact fp64 oracle ALS trajectory on the {w.name} workload; written by tests/golden/make_trajectory.py",
        "workload": {"name": w.name, "m": w.m, "n": w.n, "nnz": int(a.nnz), "f": w.f, "lambda": w.lam, "seed": w.seed},
        "history": hist,
        "rows": [int(r) for r in rows], "X_rows": [[float(v) for v in X[r]] for r in rows],
        "cols": [int(c) for c in cols], "Theta_cols": [[float(v) for v in T[c]] for c in cols],
    }
    with open(out_path, "w") as fh:
        json.dump(out, fh)
    print("wrote", out_path, flush=True)


if __name__ == "__main__":
    main()
