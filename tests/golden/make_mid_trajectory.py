"""Writes tests/golden/mid_trajectory.json: the exact double-precision ALS trajectory of the oracle on the
Mid workload (Section 2: per sweep update X with Theta fixed, then Theta with the new X; weighted-lambda
regulariser of equation (1); training RMSE as in Section 5.2 but on the training entries).

Calls only `oracle/` and the seeded input generator.  About ten minutes on 8 cores, ~10 GB of memory.

    python tests/golden/make_mid_trajectory.py [--sweeps 10]
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
    ap.add_argument("--sweeps", type=int, default=10)
    ap.add_argument("--out", default=os.path.join(ROOT, "tests", "golden", "mid_trajectory.json"))
    args = ap.parse_args()
    w = W.MID
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
    for s in range(args.sweeps):
        t0 = time.perf_counter()
        X = oracle.update_rows(a.ptr, a.idx, a.val, T, w.lam)
        T = oracle.update_rows(cptr, cidx, cval, X, w.lam)
        rec = {"sweep": s + 1, "rmse": oracle.rmse(a.ptr, a.idx, a.val, X, T),
               "objective": oracle.objective(a.ptr, a.idx, a.val, X, T, w.lam)}
        hist.append(rec)
        print(f"sweep {s + 1}: rmse {rec['rmse']:.9f} J {rec['objective']:.6e} ({time.perf_counter() - t0:.1f} s)", flush=True)
    out = {
        "what": "exact fp64 oracle ALS trajectory on the Mid workload; written by tests/golden/make_mid_trajectory.py",
        "workload": {"name": w.name, "m": w.m, "n": w.n, "nnz": int(a.nnz), "f": w.f, "lambda": w.lam, "seed": w.seed},
        "history": hist,
        "rows": [int(r) for r in rows], "X_rows": [[float(v) for v in X[r]] for r in rows],
        "cols": [int(c) for c in cols], "Theta_cols": [[float(v) for v in T[c]] for c in cols],
    }
    with open(args.out, "w") as fh:
        json.dump(out, fh)
    print("wrote", args.out, flush=True)


if __name__ == "__main__":
    main()
