"""Rows with fewer than 64 stored entries (128 with fp32 factors at f = 100 and 128) under the CG solver: Algorithm 1
(Section 4.1) runs on the gathered theta_v themselves, A_u p = G^T (G p) + lambda n_u p, and A_u is never formed.  Same iteration as the dense route, so every row
is held to the double-precision Algorithm 1 of the oracle (same warm start, same f_s) at the bar of the dense route,
and the two routes must agree to fp32 rounding."""
import numpy as np
import pytest

import oracle
import workload as W

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def P():
    import paper_1808_03843_amd as pkg
    return pkg


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def _rel(x, ref):
    return np.linalg.norm(x.astype(np.float64) - ref, axis=1) / np.maximum(np.linalg.norm(ref, axis=1), 1e-30)


def _matrix(seed, ncols):
    """Every degree from 0 to 70 (both sides of the 64-entry boundary, every fill of the last 4-entry step), a few
    longer rows, and empty rows between them; ratings 0 .. 5 with stored zeros."""
    rng = np.random.default_rng(seed)
    degrees = np.concatenate([np.arange(0, 71), [0, 63, 64, 1, 127, 200, 0, 33, 62, 63]])
    rng.shuffle(degrees)
    ptr = np.concatenate([[0], np.cumsum(degrees)]).astype(np.int64)
    idx = np.concatenate([np.sort(rng.choice(ncols, d, replace=False)) for d in degrees]).astype(np.int32)
    val = rng.integers(0, 6, size=int(ptr[-1])).astype(np.float32)
    return degrees, ptr, idx, val


@pytest.mark.parametrize("f,dtype", [(f, d) for f in (16, 32, 64, 100, 128, 256) for d in ("f32", "bf16", "f16", "f32x3", "f32x2")
                                     if f <= 128 or d in ("f32", "bf16", "f16")])   # (the routes through 16-bit parts: f <= 128)
def test_short_rows_follow_double_precision_algorithm_1(P, f, dtype):
    ncols, lam = 900, 0.2
    degrees, ptr, idx, val = _matrix(100 + f, ncols)
    Theta = W.random_factors(ncols, f, seed=7 + f, scale=0.4)
    warm = W.random_factors(len(degrees), f, seed=9 + f, scale=0.05)
    code = {"f32": P.F32, "bf16": P.BF16, "f16": P.F16, "f32x3": P.F32X3, "f32x2": P.F32X2}[dtype]
    tdt = {"bf16": torch.bfloat16, "f16": torch.float16}.get(dtype)
    Td = _dev(Theta) if tdt is None else _dev(Theta).to(tdt)
    Tref = Theta if tdt is None else Td.to(torch.float32).cpu().numpy()   # the oracle gets the rounded factor
    for fs, p64 in ((6, False), (3, True), (0, False)):
        sp = P.SparseMatrix.from_host(len(degrees), ncols, ptr, idx, val, ptr64=p64)
        ref = oracle.update_rows_cg(ptr, idx, val, Tref, lam, warm, fs=fs)
        out = {}
        for dense in (False, True):
            als = P.Als(f, solver=P.SOLVER_CG, cg_iters=fs, factor_dtype=code, dense_short_rows=dense, profile=True)
            X = _dev(warm.copy())
            als.update_rows(sp, Td, lam, X)
            als.synchronize()
            short_launches = als.kernel_time(P.K_SHORT)[1]
            assert (short_launches == 0) == dense
            assert als.short_row_limit() == (0 if dense else 128 if (dtype == "f32" and f in (100, 128)) else 64)
            out[dense] = X.cpu().numpy()
            als.close()
        live = degrees > 0
        assert not out[False][~live].any() and not out[True][~live].any()           # rows without entries: 0
        err = _rel(out[False][live], ref[live])
        # a row with fewer entries than iterations has converged before the last one: the later steps divide rounding
        # noise by rounding noise (on both routes); the bar applies where f_s stays below the rank of the row's system
        settled = degrees[live] > fs
        assert err[settled].max() <= 2e-3, (dtype, f, fs, float(err[settled].max()))
        both = _rel(out[False][live], out[True][live].astype(np.float64))
        assert both[settled].max() <= 2e-3, (dtype, f, fs, float(both[settled].max()))
        if fs == 0:
            assert np.array_equal(out[False][live], warm[live])                     # no iteration: the warm start stays


def test_short_rows_in_a_whole_cg_run_match_the_dense_route(P):
    """Ten CG(6) sweeps of the reduced Mid shape on both routes end at the same training RMSE (and within 2e-3 of the
    exact oracle's, the bar of the approximate mode)."""
    w = W.MID_SMALL
    a = W.generate(w)
    c = W.transpose(a)
    X0, T0 = W.init_factors(w)
    _, _, hist = oracle.als((a.ptr, a.idx, a.val), (c.ptr, c.idx, c.val), X0, T0, w.lam, w.sweeps)
    csr = P.SparseMatrix.from_host(a.nrows, a.ncols, a.ptr, a.idx, a.val)
    csc = P.SparseMatrix.from_host(c.nrows, c.ncols, c.ptr, c.idx, c.val)
    rm = {}
    for dense in (False, True):
        als = P.Als(w.f, solver=P.SOLVER_CG, cg_iters=6, dense_short_rows=dense)
        X, T = _dev(X0), _dev(T0)
        for _ in range(w.sweeps):
            als.update_rows(csr, T, w.lam, X)
            als.update_cols(csc, X, w.lam, T)
        rm[dense] = als.rmse(csr, X, T)
        als.synchronize()
        als.close()
    print(f"mid_small CG(6): rmse {rm[False]:.6f} (short rows on their gathered rows), {rm[True]:.6f} (every row builds A_u), "
          f"exact oracle {hist[-1]['rmse']:.6f}")
    assert abs(rm[False] - rm[True]) <= 1e-4 and abs(rm[False] - hist[-1]["rmse"]) <= 2e-3


@pytest.mark.parametrize("solver", ["cg", "cholesky"])
def test_a_non_finite_factor_entry_is_reported_by_every_route(P, solver):
    """A NaN in one factor row reaches rows of every length (short rows on their gathered rows, fused rows, split rows):
    the next als_synchronize reports ALS_ENUMERIC, the rows that do not gather it are unharmed."""
    f, ncols, lam = 100, 600, 0.2
    degrees, ptr, idx, val = _matrix(3, ncols)
    degrees = np.concatenate([degrees, [500]])                       # one row that is split at chunk = 256
    rng = np.random.default_rng(8)
    idx = np.concatenate([idx, np.sort(rng.choice(ncols, 500, replace=False)).astype(np.int32)])
    val = np.concatenate([val, rng.integers(1, 6, 500).astype(np.float32)])
    ptr = np.concatenate([[0], np.cumsum(degrees)]).astype(np.int64)
    Theta = W.random_factors(ncols, f, seed=2, scale=0.4)
    bad_col = 17
    Theta[bad_col, 5] = np.nan
    warm = W.random_factors(len(degrees), f, seed=4, scale=0.05)
    hit = np.array([bad_col in idx[ptr[u]:ptr[u + 1]] for u in range(len(degrees))])
    assert hit[degrees < 64].any() and hit[(degrees >= 64) & (degrees < 256)].any() and hit[-1]
    als = P.Als(f, solver=P.SOLVER_CG if solver == "cg" else P.SOLVER_CHOLESKY, cg_iters=6, chunk=256)
    sp = P.SparseMatrix.from_host(len(degrees), ncols, ptr, idx, val)
    X = _dev(warm.copy())
    als.update_rows(sp, _dev(Theta), lam, X)
    with pytest.raises(P.AlsError) as info:
        als.synchronize()
    assert info.value.code == P.ALS_ENUMERIC
    got = X.cpu().numpy()
    clean = (~hit) & (degrees > 0)
    assert np.isfinite(got[clean]).all() and not np.isfinite(got[hit]).all(axis=1).any()
    als.synchronize()          # the report clears the status word
    als.close()
