"""Seeded synthetic workloads shared by the oracle tests and the GPU tests.

Holds input generation only (sparse rating matrices, initial factors, the
named workload shapes); none of the factorisation arithmetic lives here.
The shapes follow the paper's Table 2 (Netflix, YahooMusic, Hugewiki sizes);
the real datasets are not used, seeded synthetic matrices stand in for them.
"""
from __future__ import annotations

import ctypes
import dataclasses
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "synth.c")
_LIB = os.path.join(_HERE, "libsynth.so")


def build(force: bool = True) -> str:
    """Compile the generator with gcc (portable flags: output must not depend on the host CPU)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _Cfg(ctypes.Structure):
    _fields_ = [
        ("m", ctypes.c_int64), ("n", ctypes.c_int64), ("nnz", ctypes.c_int64),
        ("row_s", ctypes.c_double), ("dmin", ctypes.c_int64), ("dmax", ctypes.c_int64),
        ("col_s", ctypes.c_double), ("hidden_rank", ctypes.c_int32),
        ("factor_std", ctypes.c_double), ("noise_std", ctypes.c_double),
        ("rating_kind", ctypes.c_int32), ("seed", ctypes.c_uint64),
    ]


_lib = None


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        lib = ctypes.CDLL(_LIB)
        lib.synth_create.restype = ctypes.c_void_p
        lib.synth_create.argtypes = [ctypes.POINTER(_Cfg)]
        lib.synth_destroy.argtypes = [ctypes.c_void_p]
        lib.synth_degrees.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        lib.synth_fill_rows.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64,
                                        ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        lib.synth_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


@dataclasses.dataclass(frozen=True)
class Workload:
    """A named workload: matrix shape + generator knobs + the ALS parameters it is run with."""
    name: str
    m: int
    n: int
    nnz: int
    f: int
    lam: float
    row_s: float
    dmin: int
    dmax: int
    col_s: float
    hidden_rank: int
    rating_kind: int = 0          # 0: ratings 1..5, 1: ratings 0..100 in steps of 10
    factor_std: float = 0.6
    noise_std: float = 0.5
    seed: int = 0
    sweeps: int = 5

    def with_f(self, f: int) -> "Workload":
        return dataclasses.replace(self, f=f, name=f"{self.name}_f{f}")


# The five configurations (shapes of the paper's Table 2 datasets) and two
# reduced shapes that the CPU oracle finishes in seconds.
TINY = Workload("tiny", 2_000, 1_000, 60_000, 16, 0.05, 1.1, 1, 300, 0.8, 8, seed=0, sweeps=5)
MID = Workload("mid", 480_189, 17_770, 99_072_112, 100, 0.05, 1.0, 1, 17_000, 1.0, 20, seed=1, sweeps=10)
LARGE_SQUARE = Workload("large_square", 1_000_990, 624_961, 252_800_275, 100, 1.0, 1.0, 1, 60_000, 1.1, 20,
                        rating_kind=1, seed=2, sweeps=5)
VERY_TALL = Workload("very_tall", 50_082_603, 39_780, 3_101_144_313, 100, 0.05, 1.0, 1, 20_000, 1.0, 20,
                     seed=3, sweeps=3)
# reduced shapes: same generator, same f / lambda, sizes the oracle handles quickly
MID_SMALL = Workload("mid_small", 12_000, 2_400, 1_500_000, 100, 0.05, 1.0, 1, 2_300, 1.0, 20, seed=11, sweeps=10)
SQUARE_SMALL = Workload("square_small", 9_000, 7_000, 600_000, 100, 1.0, 1.0, 0, 1_500, 1.1, 20,
                        rating_kind=1, seed=12, sweeps=5)

CONFIGS = {w.name: w for w in (TINY, MID, LARGE_SQUARE, VERY_TALL, MID_SMALL, SQUARE_SMALL)}


@dataclasses.dataclass
class CSR:
    """Compressed sparse rows (or, for a CSC of R, compressed sparse columns of R)."""
    nrows: int
    ncols: int
    ptr: np.ndarray     # int64 [nrows+1]
    idx: np.ndarray     # int32 [nnz], ascending inside each row
    val: np.ndarray     # float32 [nnz]

    @property
    def nnz(self) -> int:
        return int(self.ptr[-1])


class Generator:
    """Row-addressable generator for one workload (rows are pure functions of (seed, row))."""

    def __init__(self, w: Workload):
        self.w = w
        lib = _load()
        self._cfg = _Cfg(w.m, w.n, w.nnz, w.row_s, w.dmin, w.dmax, w.col_s, w.hidden_rank,
                         w.factor_std, w.noise_std, w.rating_kind, w.seed)
        self._h = lib.synth_create(ctypes.byref(self._cfg))
        if not self._h:
            raise RuntimeError("synth_create failed")
        self._deg: Optional[np.ndarray] = None

    def __del__(self):
        if getattr(self, "_h", None):
            _load().synth_destroy(self._h)
            self._h = None

    def degrees(self) -> np.ndarray:
        if self._deg is None:
            deg = np.empty(self.w.m, dtype=np.int64)
            rc = _load().synth_degrees(self._h, deg.ctypes.data)
            if rc != 0:
                raise RuntimeError("synth_degrees: nnz not reachable with these degree bounds")
            self._deg = deg
        return self._deg

    def rows(self, u0: int, u1: int) -> CSR:
        """CSR slice holding rows [u0, u1) (ptr is relative to the slice)."""
        deg = self.degrees()[u0:u1]
        ptr = np.zeros(u1 - u0 + 1, dtype=np.int64)
        np.cumsum(deg, out=ptr[1:])
        nnz = int(ptr[-1])
        idx = np.empty(nnz, dtype=np.int32)
        val = np.empty(nnz, dtype=np.float32)
        rc = _load().synth_fill_rows(self._h, u0, u1, ptr.ctypes.data, idx.ctypes.data, val.ctypes.data)
        if rc != 0:
            raise RuntimeError("synth_fill_rows failed")
        return CSR(u1 - u0, self.w.n, ptr, idx, val)

    def csr(self) -> CSR:
        return self.rows(0, self.w.m)


def generate(w: Workload) -> CSR:
    return Generator(w).csr()


def transpose(a: CSR) -> CSR:
    """CSC of R from its CSR (as the CSR of R^T), through scipy: plumbing for test inputs.

    The oracle and the GPU library each have a transposer of their own; this
    third one only feeds inputs and serves as a cross-check for both.
    """
    import scipy.sparse as sp
    mat = sp.csr_matrix((a.val, a.idx, a.ptr), shape=(a.nrows, a.ncols))
    t = mat.tocsc()
    t.sort_indices()
    return CSR(a.ncols, a.nrows, t.indptr.astype(np.int64), t.indices.astype(np.int32),
               t.data.astype(np.float32))


def split(a: CSR, test_frac: float, seed: int = 0):
    """Seeded train / held-out split of the stored entries (the protocol of Section 5.2: fit on the training
    entries, report the RMSE on entries that were held out).  Entry (u, v) goes to the test set iff a 64-bit
    mix of (seed, u, v) falls below test_frac: a pure function of the entry, independent of the order of work.
    Returns (train, test), both canonical CSR of the full shape."""
    rows = np.repeat(np.arange(a.nrows, dtype=np.uint64), np.diff(a.ptr).astype(np.int64))
    with np.errstate(over="ignore"):
        h = (rows * np.uint64(0x9E3779B97F4A7C15) + a.idx.astype(np.uint64) * np.uint64(0xC2B2AE3D27D4EB4F)
             + np.uint64(seed) * np.uint64(0x165667B19E3779F9))
        h ^= h >> np.uint64(30); h *= np.uint64(0xBF58476D1CE4E5B9)
        h ^= h >> np.uint64(27); h *= np.uint64(0x94D049BB133111EB)
        h ^= h >> np.uint64(31)
    is_test = (h >> np.uint64(11)).astype(np.float64) * (1.0 / (1 << 53)) < test_frac
    out = []
    for keep in (~is_test, is_test):
        cnt = np.bincount(rows[keep].astype(np.int64), minlength=a.nrows)
        ptr = np.concatenate([[0], np.cumsum(cnt)]).astype(np.int64)
        out.append(CSR(a.nrows, a.ncols, ptr, a.idx[keep].copy(), a.val[keep].copy()))
    return out[0], out[1]


def init_factors(w: Workload, seed: Optional[int] = None):
    """X0 = 0 (m x f) and Theta0 ~ U(0, 1/sqrt(f)) (n x f), float32."""
    rng = np.random.default_rng(w.seed + 1000 if seed is None else seed)
    theta0 = (rng.random((w.n, w.f), dtype=np.float32) / np.float32(np.sqrt(w.f))).astype(np.float32)
    x0 = np.zeros((w.m, w.f), dtype=np.float32)
    return x0, theta0


def random_factors(rows: int, f: int, seed: int, scale: float = 1.0) -> np.ndarray:
    """A seeded dense factor matrix ~ N(0, scale), float32 (synthetic input for one-sided tests)."""
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((rows, f), dtype=np.float32) * np.float32(scale)).astype(np.float32)


def num_threads() -> int:
    return int(_load().synth_num_threads())
