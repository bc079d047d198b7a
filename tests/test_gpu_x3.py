"""factor_dtype = F32X3 / F32X2: fp32 factors multiplied on the 16-bit matrix cores as three bf16 parts (six products)
or, scaled by a power of two, as two fp16 parts (three products).
Both modes claim the accuracy of the fp32 path, so they are held to its bars: A_u and b_u element by element, the exact
solver at 1e-4 per row, Algorithm 1 against its double-precision run, the stored Mid trajectory."""
import numpy as np
import pytest

import oracle
import workload as W

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def _rel(g, o, floor=1e-30):
    return np.linalg.norm(g.astype(np.float64) - o, axis=1) / np.maximum(np.linalg.norm(o, axis=1), floor)


@pytest.fixture(scope="module")
def P():
    import paper_1808_03843_amd as pkg
    return pkg


MODES = ["f32x3", "f32x2"]


def _code(P, mode):
    return {"f32x3": P.F32X3, "f32x2": P.F32X2}[mode]


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("f", [16, 32, 64, 100, 128])
def test_hermitian_and_bias_from_16_bit_parts(P, f, mode):
    """A_u and b_u against the oracle: degrees around the step size (32) and the chunk size, ratings and factors that
    use all 24 significant bits, values of very different magnitude in one row."""
    n = 5000
    degrees = [0, 1, 2, 7, 8, 9, 15, 16, 17, 31, 32, 33, 63, 64, 65, 95, 96, 97, 255, 256, 257, 300, 1000, 1024, 1025, 2500]
    rng = np.random.default_rng(13)
    ptr = np.concatenate([[0], np.cumsum(degrees)]).astype(np.int64)
    idx = np.concatenate([np.sort(rng.choice(n, d, replace=False)) for d in degrees] + [np.zeros(0, int)]).astype(np.int32)
    val = (rng.standard_normal(int(ptr[-1])) * 37.123).astype(np.float32)
    Theta = W.random_factors(n, f, seed=5, scale=0.5)
    Theta[::7] *= np.float32(1e-3)        # rows of small magnitude next to ordinary ones
    Theta[3::11] *= np.float32(250.0)
    als = P.Als(f, chunk=256, factor_dtype=_code(P, mode))
    sp = P.SparseMatrix.from_host(len(degrees), n, ptr, idx, val)
    A, b = als.hermitian(sp, _dev(Theta), 0.05, 0, len(degrees))
    A, b = A.cpu().numpy(), b.cpu().numpy()
    worst = 0.0
    for u, d in enumerate(degrees):
        s, e = ptr[u], ptr[u + 1]
        Ao, bo = oracle.normal_eq(idx[s:e], val[s:e], Theta, 0.05)
        # the bar of the fp32 path: fp32 summation of d products
        assert np.abs(A[u] - Ao).max() <= 2e-6 * max(np.abs(Ao).max(), 1e-30) * max(1, np.sqrt(d)), (u, d)
        assert np.abs(b[u] - bo).max() <= 2e-6 * max(np.abs(bo).max(), 1e-30) * max(1, np.sqrt(d)) + 1e-30, (u, d)
        assert np.array_equal(A[u], A[u].T)
        if d:
            worst = max(worst, np.abs(A[u] - Ao).max() / np.abs(Ao).max())
    print(f"{mode} f={f}: worst |dA| / max|A| = {worst:.2e}")
    als.close()


def _matrix(seed, ncols):
    rng = np.random.default_rng(seed)
    fixed = [0, 1, 2, 3, 4, 5, 15, 16, 17, 31, 32, 33, 63, 64, 65, 127, 129, 255, 256, 257, 511, 1000, 1025, 2049, 3100, 4000]
    rnd = [int(np.exp(rng.uniform(0, np.log(3500)))) for _ in range(40)]
    degrees = fixed + rnd
    ptr = np.concatenate([[0], np.cumsum(degrees)]).astype(np.int64)
    idx = np.concatenate([np.sort(rng.choice(ncols, d, replace=False)) for d in degrees] + [np.zeros(0, int)]).astype(np.int32)
    val = rng.integers(0, 6, size=int(ptr[-1])).astype(np.float32)   # stored zeros included
    return degrees, ptr, idx, val


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("f,solver,chunk,p64", [(f, s, c, p) for f in (16, 32, 64, 100, 128) for s in ("cholesky", "cg")
                                                for c, p in ((0, False), (256, True), (64, False))])
def test_half_sweep_with_inputs_in_16_bit_parts(P, f, solver, chunk, p64, mode):
    """Every kernel the mode dispatches to (fused rows, slot rows, both solvers, both offset widths), rows from empty
    to split over several work items, against the oracle at the bars of the fp32 path."""
    ncols, lam = 4000, 0.3
    degrees, ptr, idx, val = _matrix(124, ncols)
    Theta = W.random_factors(ncols, f, seed=47 + f, scale=0.3)
    warm = W.random_factors(len(degrees), f, seed=48 + f, scale=0.05)
    sp = P.SparseMatrix.from_host(len(degrees), ncols, ptr, idx, val, ptr64=p64)
    code = P.SOLVER_CHOLESKY if solver == "cholesky" else P.SOLVER_CG
    als = P.Als(f, solver=code, cg_iters=5, chunk=chunk, factor_dtype=_code(P, mode))
    X = _dev(warm.copy())
    als.update_rows(sp, _dev(Theta), lam, X)
    als.synchronize()
    got = X.cpu().numpy()
    als.close()
    if solver == "cholesky":
        ref, tol = oracle.update_rows(ptr, idx, val, Theta, lam), 1e-4
    else:
        ref, tol = oracle.update_rows_cg(ptr, idx, val, Theta, lam, warm, fs=5), 2e-3
    # (a row whose only rating is 0 has the solution 0: Algorithm 1 then ends in rounding noise, 1e-17 in double and
    # 1e-7 in float, so the norm in the denominator gets a floor far below any real solution, whose norm is about 1)
    err = _rel(got, ref, floor=1e-2)
    assert np.all(got[0] == 0.0)           # the empty row
    assert err[1:].max() <= tol, (int(err[1:].argmax()) + 1, float(err.max()))


@pytest.mark.parametrize("mode", MODES)
def test_one_exact_sweep_on_mid_small_with_inputs_in_16_bit_parts(P, mode):
    """A whole exact sweep (rows, then columns from the oracle's X) of the reduced Mid shape at 1e-4 per row."""
    w = W.MID_SMALL
    a = W.generate(w)
    c = W.transpose(a)
    X0, T0 = W.init_factors(w)
    als = P.Als(w.f, solver=P.SOLVER_CHOLESKY, factor_dtype=_code(P, mode))
    csr = P.SparseMatrix.from_host(a.nrows, a.ncols, a.ptr, a.idx, a.val)
    csc = P.SparseMatrix.from_host(c.nrows, c.ncols, c.ptr, c.idx, c.val)
    X = torch.zeros((w.m, w.f), device="cuda:0")
    als.update_rows(csr, _dev(T0), w.lam, X)
    Xo = oracle.update_rows(a.ptr, a.idx, a.val, T0, w.lam)
    T = torch.zeros((w.n, w.f), device="cuda:0")
    als.update_cols(csc, _dev(Xo.astype(np.float32)), w.lam, T)
    als.synchronize()
    To = oracle.update_rows(c.ptr, c.idx, c.val, Xo.astype(np.float32), w.lam)
    ex, et = _rel(X.cpu().numpy(), Xo), _rel(T.cpu().numpy(), To)
    print(f"mid_small, {mode} inputs: X max {ex.max():.2e}, Theta max {et.max():.2e}")
    assert ex.max() <= 1e-4 and et.max() <= 1e-4
    als.close()


@pytest.mark.parametrize("mode", MODES)
def test_mid_ten_sweeps_with_inputs_in_16_bit_parts_follow_the_stored_oracle_trajectory(P, mode):
    """Mid at full size: the exact solver with inputs in 16-bit parts follows the stored fp64 trajectory like the fp32 path
    (2e-5 relative per sweep, stored rows at 5e-4), and CG(6) ends within 2e-3 of the exact oracle's RMSE."""
    from test_gpu_full_size import _follow_trajectory, _golden
    gold = _golden("mid")
    w = W.MID
    a = W.generate(w)
    csr = P.SparseMatrix.from_host(a.nrows, a.ncols, a.ptr, a.idx, a.val)
    del a
    _follow_trajectory(P, w, gold, csr, [
        (f"exact, {mode} inputs", dict(solver=P.SOLVER_CHOLESKY, factor_dtype=_code(P, mode)), None),
        (f"CG(6), {mode} inputs", dict(solver=P.SOLVER_CG, cg_iters=6, factor_dtype=_code(P, mode)), None),
    ])


@pytest.mark.parametrize("scale", [2.0 ** -40, 1e-6, 1.0, 3e4, 2.0 ** 50])
def test_two_part_route_follows_the_magnitude_of_the_factor(P, scale):
    """The two fp16 parts are cut after a power-of-two scaling found from max |Theta| on the device, so a factor matrix
    of any magnitude gives the A_u of the fp32 path to the same relative accuracy (fp16 alone spans 6e-8 .. 65504)."""
    f, n = 100, 3000
    degrees = [1, 5, 40, 300, 1500]
    rng = np.random.default_rng(3)
    ptr = np.concatenate([[0], np.cumsum(degrees)]).astype(np.int64)
    idx = np.concatenate([np.sort(rng.choice(n, d, replace=False)) for d in degrees]).astype(np.int32)
    val = rng.integers(1, 6, size=int(ptr[-1])).astype(np.float32)
    Theta = (W.random_factors(n, f, seed=9, scale=0.5).astype(np.float64) * scale).astype(np.float32)
    als = P.Als(f, chunk=256, factor_dtype=P.F32X2)
    sp = P.SparseMatrix.from_host(len(degrees), n, ptr, idx, val)
    A, b = als.hermitian(sp, _dev(Theta), 0.0, 0, len(degrees))
    A, b = A.cpu().numpy().astype(np.float64), b.cpu().numpy().astype(np.float64)
    for u, d in enumerate(degrees):
        s, e = ptr[u], ptr[u + 1]
        Ao, bo = oracle.normal_eq(idx[s:e], val[s:e], Theta, 0.0)
        assert np.abs(A[u] - Ao).max() <= 2e-6 * np.abs(Ao).max() * np.sqrt(d), (scale, d)
        assert np.abs(b[u] - bo).max() <= 2e-6 * np.abs(bo).max() * np.sqrt(d), (scale, d)
    als.close()
