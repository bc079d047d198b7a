"""ctypes front end of the CPU oracle (oracle/als_oracle.c).

TEST INFRASTRUCTURE ONLY: double-precision reference for alternating least
squares (Section 2, eq. (1)-(3); Algorithm 1).  Nothing in the product package
imports this module; only tests, the smoke check and the benchmark's
cpu_baseline leg do.  It takes plain numpy arrays (CSR pieces, factors) and
shares no code with the GPU path.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "als_oracle.c")


def _cpu_tag() -> str:
    """-march=native output only runs on a CPU with the same features: key the file name on them."""
    import hashlib
    try:
        with open("/proc/cpuinfo") as fh:
            flags = next((ln for ln in fh if ln.startswith("flags")), "")
    except OSError:
        flags = ""
    return hashlib.sha1(flags.encode()).hexdigest()[:10]


_LIB = os.path.join(_HERE, f"libals_oracle_{_cpu_tag()}.so")


def build(force: bool = True) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O3", "-march=native", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None
_i64, _i32, _f32, _f64 = np.int64, np.int32, np.float32, np.float64


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        lib = ctypes.CDLL(_LIB)
        vp, i64, ci, d = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_double
        lib.oracle_normal_eq.argtypes = [ci, i64, vp, vp, vp, d, vp, vp]
        lib.oracle_cholesky_solve.argtypes = [ci, vp, vp]
        lib.oracle_cholesky_solve.restype = ci
        lib.oracle_cg.argtypes = [ci, vp, vp, vp, ci, d]
        lib.oracle_cg.restype = ci
        lib.oracle_update_rows.argtypes = [i64, vp, vp, vp, vp, ci, d, vp]
        lib.oracle_update_rows.restype = i64
        lib.oracle_update_selected.argtypes = [i64, vp, vp, vp, vp, vp, ci, d, vp]
        lib.oracle_update_selected.restype = i64
        lib.oracle_update_rows_cg.argtypes = [i64, vp, vp, vp, vp, ci, d, ci, d, vp]
        lib.oracle_sse.argtypes = [i64, vp, vp, vp, vp, vp, ci]
        lib.oracle_sse.restype = d
        lib.oracle_sse_parallel.argtypes = [i64, vp, vp, vp, vp, vp, ci]
        lib.oracle_sse_parallel.restype = d
        lib.oracle_sse_parallel_f32.argtypes = [i64, vp, vp, vp, vp, vp, ci]
        lib.oracle_sse_parallel_f32.restype = d
        lib.oracle_regulariser.argtypes = [i64, i64, vp, vp, vp, vp, ci, d]
        lib.oracle_regulariser.restype = d
        lib.oracle_csr_to_csc.argtypes = [i64, i64, vp, vp, vp, vp, vp, vp]
        lib.oracle_bin_rows.argtypes = [i64, vp, ci, vp, vp]
        lib.oracle_implicit_normal_eq.argtypes = [ci, i64, i64, vp, vp, vp, d, d, vp, vp, vp]
        lib.oracle_implicit_update_selected.argtypes = [i64, vp, vp, vp, vp, vp, i64, ci, d, d, vp]
        lib.oracle_implicit_update_selected.restype = i64
        lib.oracle_implicit_objective.argtypes = [i64, i64, vp, vp, vp, vp, vp, ci, d, d]
        lib.oracle_implicit_objective.restype = d
        lib.oracle_num_threads.restype = ci
        _lib = lib
    return _lib


def _c(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


def _p(a):
    return a.ctypes.data


def normal_eq(idx, r, Theta, lam):
    """A_u (f x f, full) and b_u of one row with column ids idx and ratings r  (Section 2, step (i), eq. (2))."""
    idx, r, Theta = _c(idx, _i32), _c(r, _f32), _c(Theta, _f64)
    f = Theta.shape[1]
    A = np.empty((f, f), _f64)
    b = np.empty(f, _f64)
    _load().oracle_normal_eq(f, len(idx), _p(idx), _p(r), _p(Theta), float(lam), _p(A), _p(b))
    return A, b


def cholesky_solve(A, b):
    """x = A^-1 b by Cholesky (Section 2, step (ii), exact)."""
    A, b = _c(A, _f64).copy(), _c(b, _f64).copy()
    rc = _load().oracle_cholesky_solve(A.shape[0], _p(A), _p(b))
    if rc != 0:
        raise np.linalg.LinAlgError("non-positive pivot")
    return b


def cg(A, x0, b, fs, eps=0.0):
    """Algorithm 1 (CGSolve): returns (x, iterations)."""
    A, x, b = _c(A, _f64), _c(x0, _f64).copy(), _c(b, _f64)
    it = _load().oracle_cg(A.shape[0], _p(A), _p(x), _p(b), int(fs), float(eps))
    return x, it


def update_rows(ptr, idx, val, Theta, lam):
    """Exact "Update X" (eq. (2)) for all rows of a CSR; pass the CSC of R and X for "Update Theta" (eq. (3))."""
    ptr, idx, val, Theta = _c(ptr, _i64), _c(idx, _i32), _c(val, _f32), _c(Theta, _f64)
    m, f = len(ptr) - 1, Theta.shape[1]
    X = np.empty((m, f), _f64)
    bad = _load().oracle_update_rows(m, _p(ptr), _p(idx), _p(val), _p(Theta), f, float(lam), _p(X))
    if bad:
        raise np.linalg.LinAlgError(f"{bad} rows with a non-positive pivot")
    return X


def update_selected(rows, ptr, idx, val, Theta, lam):
    """Exact update of the listed rows only: returns len(rows) x f."""
    rows = _c(rows, _i64)
    ptr, idx, val, Theta = _c(ptr, _i64), _c(idx, _i32), _c(val, _f32), _c(Theta, _f64)
    f = Theta.shape[1]
    X = np.empty((len(rows), f), _f64)
    bad = _load().oracle_update_selected(len(rows), _p(rows), _p(ptr), _p(idx), _p(val), _p(Theta), f,
                                         float(lam), _p(X))
    if bad:
        raise np.linalg.LinAlgError(f"{bad} rows with a non-positive pivot")
    return X


def update_rows_cg(ptr, idx, val, Theta, lam, X_warm, fs, eps=0.0):
    """"Update X" with Algorithm 1 warm-started from X_warm (Section 4.1)."""
    ptr, idx, val, Theta = _c(ptr, _i64), _c(idx, _i32), _c(val, _f32), _c(Theta, _f64)
    X = _c(X_warm, _f64).copy()
    m, f = len(ptr) - 1, Theta.shape[1]
    assert X.shape == (m, f)
    _load().oracle_update_rows_cg(m, _p(ptr), _p(idx), _p(val), _p(Theta), f, float(lam), int(fs), float(eps), _p(X))
    return X


def sse(ptr, idx, val, X, Theta, parallel=True):
    """Sum of squared errors over stored entries (data term of eq. (1))."""
    ptr, idx, val = _c(ptr, _i64), _c(idx, _i32), _c(val, _f32)
    X, Theta = _c(X, _f64), _c(Theta, _f64)
    fn = _load().oracle_sse_parallel if parallel else _load().oracle_sse
    return fn(len(ptr) - 1, _p(ptr), _p(idx), _p(val), _p(X), _p(Theta), X.shape[1])


def rmse_f32(ptr, idx, val, X, Theta):
    """Training RMSE for float32 factors without a double-precision copy of them (arithmetic in double)."""
    ptr, idx, val = _c(ptr, _i64), _c(idx, _i32), _c(val, _f32)
    X, Theta = _c(X, _f32), _c(Theta, _f32)
    s = _load().oracle_sse_parallel_f32(len(ptr) - 1, _p(ptr), _p(idx), _p(val), _p(X), _p(Theta), X.shape[1])
    return float(np.sqrt(s / max(int(ptr[-1]), 1)))


def rmse(ptr, idx, val, X, Theta):
    """Training RMSE over the stored entries (Section 5.2 metric applied to the training set)."""
    nnz = int(ptr[-1])
    return float(np.sqrt(sse(ptr, idx, val, X, Theta) / max(nnz, 1)))


def objective(ptr, idx, val, X, Theta, lam):
    """J of eq. (1): squared error over stored entries + weighted-lambda regulariser."""
    ptr_c, idx_c = _c(ptr, _i64), _c(idx, _i32)
    Xc, Tc = _c(X, _f64), _c(Theta, _f64)
    reg = _load().oracle_regulariser(len(ptr_c) - 1, Tc.shape[0], _p(ptr_c), _p(idx_c), _p(Xc), _p(Tc),
                                     Xc.shape[1], float(lam))
    return sse(ptr, idx, val, X, Theta) + reg


def csr_to_csc(m, n, ptr, idx, val):
    """CSC of R (as ptr/idx/val over columns) from its CSR."""
    ptr, idx, val = _c(ptr, _i64), _c(idx, _i32), _c(val, _f32)
    cptr = np.empty(n + 1, _i64)
    cidx = np.empty(len(idx), _i32)
    cval = np.empty(len(idx), _f32)
    _load().oracle_csr_to_csc(m, n, _p(ptr), _p(idx), _p(val), _p(cptr), _p(cidx), _p(cval))
    return cptr, cidx, cval


def bin_rows(ptr, nclass):
    """Rows grouped by degree class, heaviest first, stable inside a class: (perm, class_start)."""
    ptr = _c(ptr, _i64)
    m = len(ptr) - 1
    perm = np.empty(m, _i32)
    start = np.empty(nclass + 1, _i64)
    _load().oracle_bin_rows(m, _p(ptr), int(nclass), _p(perm), _p(start))
    return perm, start


def als(csr, csc, X0, Theta0, lam, sweeps, solver="cholesky", fs=6, eps=0.0):
    """ALS of Section 2: per sweep "Update X" with Theta fixed, then "Update Theta" with the new X.

    csr / csc are (ptr, idx, val) triples of R and of R^T.  Returns X, Theta and
    the per-sweep training RMSE and objective J.
    """
    X = np.array(X0, dtype=_f64)
    T = np.array(Theta0, dtype=_f64)
    hist = []
    for _ in range(sweeps):
        if solver == "cholesky":
            X = update_rows(*csr, T, lam)
            T = update_rows(*csc, X, lam)
        else:
            X = update_rows_cg(*csr, T, lam, X, fs, eps)
            T = update_rows_cg(*csc, X, lam, T, fs, eps)
        hist.append({"rmse": rmse(*csr, X, T), "objective": objective(*csr, X, T, lam)})
    return X, T, hist


def implicit_update_selected(rows, ptr, idx, val, Theta, lam, alpha):
    """Implicit-feedback update (Section 5.6) of the listed rows (None: all), exact: len(rows) x f."""
    ptr, idx, val, Theta = _c(ptr, _i64), _c(idx, _i32), _c(val, _f32), _c(Theta, _f64)
    n, f = Theta.shape
    if rows is None:
        nsel, rp = len(ptr) - 1, None
    else:
        rows = _c(rows, _i64)
        nsel, rp = len(rows), _p(rows)
    X = np.empty((nsel, f), _f64)
    bad = _load().oracle_implicit_update_selected(nsel, rp, _p(ptr), _p(idx), _p(val), _p(Theta), n, f,
                                                  float(lam), float(alpha), _p(X))
    if bad:
        raise np.linalg.LinAlgError(f"{bad} rows with a non-positive pivot")
    return X


def implicit_update_rows(ptr, idx, val, Theta, lam, alpha):
    return implicit_update_selected(None, ptr, idx, val, Theta, lam, alpha)


def implicit_normal_eq(idx, r, Theta, lam, alpha):
    """A_u, b_u of one row under the implicit cost, summed over all columns (the definition)."""
    idx, r, Theta = _c(idx, _i32), _c(r, _f32), _c(Theta, _f64)
    n, f = Theta.shape
    A, b = np.empty((f, f), _f64), np.empty(f, _f64)
    scratch = np.zeros(n, _f64)
    _load().oracle_implicit_normal_eq(f, n, len(idx), _p(idx), _p(r), _p(Theta), float(lam), float(alpha),
                                      _p(A), _p(b), _p(scratch))
    return A, b


def implicit_objective(ptr, idx, val, X, Theta, lam, alpha):
    """Implicit cost over all m*n pairs plus lambda*(|X|^2 + |Theta|^2) (Section 5.6); O(m n f)."""
    ptr, idx, val = _c(ptr, _i64), _c(idx, _i32), _c(val, _f32)
    X, Theta = _c(X, _f64), _c(Theta, _f64)
    return _load().oracle_implicit_objective(X.shape[0], Theta.shape[0], _p(ptr), _p(idx), _p(val), _p(X),
                                             _p(Theta), X.shape[1], float(lam), float(alpha))


def num_threads() -> int:
    return int(_load().oracle_num_threads())
