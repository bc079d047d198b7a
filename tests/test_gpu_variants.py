"""Every kernel variant the library can dispatch to, on one small matrix whose rows run from empty to
split over several work items: factor width x solver x explicit / implicit x chunk size (fused rows vs
slots) x pointer width x element type of the gathered factor.  One half-sweep each, against the oracle
fed the same (rounded, where 16-bit) inputs.  Seeded and synthetic.

The point of the grid is the code that differs between template instantiations (register allocation,
tile counts, load widths): a mistake there shows up in one width or one path only.
"""
import itertools

import numpy as np
import pytest

import oracle
import workload as W

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

N_COLS = 4000
LAM, ALPHA = 0.3, 1.5


def _matrix(seed):
    rng = np.random.default_rng(seed)
    fixed = [0, 1, 2, 3, 4, 5, 15, 16, 17, 31, 33, 63, 64, 65, 127, 129, 255, 256, 257, 511, 1000, 1025, 2049, 3100, 4000]
    rnd = [int(np.exp(rng.uniform(0, np.log(3500)))) for _ in range(40)]
    degrees = fixed + rnd
    ptr = np.concatenate([[0], np.cumsum(degrees)]).astype(np.int64)
    idx = np.concatenate([np.sort(rng.choice(N_COLS, d, replace=False)) for d in degrees]
                         + [np.zeros(0, int)]).astype(np.int32)
    val = rng.integers(0, 6, size=int(ptr[-1])).astype(np.float32)   # stored zeros included
    return degrees, ptr, idx, val


def _rel(g, o):
    return np.linalg.norm(g.astype(np.float64) - o, axis=1) / np.maximum(np.linalg.norm(o, axis=1), 1e-30)


@pytest.fixture(scope="module")
def P():
    import paper_1808_03843_amd as pkg
    return pkg


@pytest.fixture(scope="module")
def mat():
    return _matrix(123)


GRID = [(f, solver, chunk, p64)
        for f in (16, 32, 64, 100, 128, 256)
        for solver in ("cholesky", "cg")
        for chunk, p64 in ((0, False), (256, True), (64, False))]


@pytest.mark.parametrize("f,solver,chunk,p64", GRID)
def test_explicit_half_sweep(P, mat, f, solver, chunk, p64):
    degrees, ptr, idx, val = mat
    Theta = W.random_factors(N_COLS, f, seed=7 + f, scale=0.3)
    warm = W.random_factors(len(degrees), f, seed=8 + f, scale=0.05)
    sp = P.SparseMatrix.from_host(len(degrees), N_COLS, ptr, idx, val, ptr64=p64)
    code = P.SOLVER_CHOLESKY if solver == "cholesky" else P.SOLVER_CG
    als = P.Als(f, solver=code, cg_iters=5, chunk=chunk)
    X = torch.from_numpy(warm.copy()).cuda()
    als.update_rows(sp, torch.from_numpy(Theta).cuda(), LAM, X)
    als.synchronize()
    got = X.cpu().numpy()
    als.close()
    if solver == "cholesky":
        ref, tol = oracle.update_rows(ptr, idx, val, Theta, LAM), 1e-4
    else:
        ref, tol = oracle.update_rows_cg(ptr, idx, val, Theta, LAM, warm, fs=5), 2e-3
    err = _rel(got, ref)
    assert np.all(got[0] == 0.0)           # the empty row
    assert err[1:].max() <= tol, (int(err[1:].argmax()) + 1, float(err.max()))


@pytest.mark.parametrize("f,solver,chunk", [(f, s, c) for f in (16, 32, 64, 100, 128, 256) for s in ("cholesky", "cg")
                                           for c in (0, 128)])
def test_implicit_half_sweep(P, mat, f, solver, chunk):
    degrees, ptr, idx, val = mat
    Theta = W.random_factors(N_COLS, f, seed=17 + f, scale=0.3)
    warm = W.random_factors(len(degrees), f, seed=18 + f, scale=0.05)
    sp = P.SparseMatrix.from_host(len(degrees), N_COLS, ptr, idx, val)
    code = P.SOLVER_CHOLESKY if solver == "cholesky" else P.SOLVER_CG
    als = P.Als(f, solver=code, cg_iters=f, chunk=chunk)   # f iterations: Algorithm 1 is then exact
    X = torch.from_numpy(warm.copy()).cuda()
    als.update_rows_implicit(sp, torch.from_numpy(Theta).cuda(), LAM, ALPHA, X)
    als.synchronize()
    got = X.cpu().numpy()
    als.close()
    ref = oracle.implicit_update_rows(ptr, idx, val, Theta, LAM, ALPHA)
    err = _rel(got[1:], ref[1:])
    assert np.all(got[0] == 0.0)
    assert err.max() <= (1e-4 if solver == "cholesky" else 1e-3), (int(err.argmax()) + 1, float(err.max()))


@pytest.mark.parametrize("f,name,chunk", [(f, n, c) for f in (16, 32, 64, 100, 128, 256) for n in ("bf16", "f16")
                                         for c in (0, 256)])
def test_sixteen_bit_factor_inputs(P, mat, f, name, chunk):
    degrees, ptr, idx, val = mat
    tdt, code = (torch.bfloat16, P.BF16) if name == "bf16" else (torch.float16, P.F16)
    T16 = torch.from_numpy(W.random_factors(N_COLS, f, seed=27 + f, scale=0.3)).cuda().to(tdt)
    T_rounded = T16.to(torch.float32).cpu().numpy()
    warm = W.random_factors(len(degrees), f, seed=28 + f, scale=0.05)
    sp = P.SparseMatrix.from_host(len(degrees), N_COLS, ptr, idx, val)
    for solver, fs, tol in ((P.SOLVER_CHOLESKY, 0, 1e-4), (P.SOLVER_CG, 5, 2e-3)):
        als = P.Als(f, solver=solver, cg_iters=fs, chunk=chunk, factor_dtype=code)
        X = torch.from_numpy(warm.copy()).cuda()
        als.update_rows(sp, T16, LAM, X)
        als.synchronize()
        got = X.cpu().numpy()
        als.close()
        ref = (oracle.update_rows(ptr, idx, val, T_rounded, LAM) if solver == P.SOLVER_CHOLESKY
               else oracle.update_rows_cg(ptr, idx, val, T_rounded, LAM, warm, fs=fs))
        err = _rel(got[1:], ref[1:])
        assert err.max() <= tol, (name, int(err.argmax()) + 1, float(err.max()))


@pytest.mark.parametrize("f", [16, 32, 64, 100, 128, 256])
def test_bf16_slots_and_rmse_kernels(P, mat, f):
    degrees, ptr, idx, val = mat
    Theta = W.random_factors(N_COLS, f, seed=37 + f, scale=0.3)
    warm = W.random_factors(len(degrees), f, seed=38 + f, scale=0.05)
    sp = P.SparseMatrix.from_host(len(degrees), N_COLS, ptr, idx, val)
    T = torch.from_numpy(Theta).cuda()
    # bf16 storage of split rows: close to the fp32-slot result (the rounding of A_u is the only difference)
    outs = []
    for hd in (P.F32, P.BF16):
        als = P.Als(f, solver=P.SOLVER_CG, cg_iters=5, chunk=64, herm_dtype=hd)
        X = torch.from_numpy(warm.copy()).cuda()
        als.update_rows(sp, T, LAM, X)
        als.synchronize()
        outs.append(X.cpu().numpy())
        r = als.rmse(sp, torch.from_numpy(warm).cuda(), T)   # seeded factors: the oracle sees nothing the GPU computed
        ro = oracle.rmse(ptr, idx, val, warm, Theta)
        assert abs(r - ro) <= 1e-5 * ro
        als.close()
    dev = _rel(outs[1][1:], outs[0][1:].astype(np.float64))
    assert dev.max() <= 5e-2
