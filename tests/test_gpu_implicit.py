"""GPU parity of the implicit-feedback path (Section 5.6) against the CPU oracle, through the C ABI.

The oracle sums over all columns (the definition); the library uses Theta^T Theta plus a weighted sum
over the stored entries.  Inputs are seeded and synthetic: the rating generator's values 1..5 stand in
for interaction counts.
"""
import numpy as np
import pytest

import oracle
import workload as W

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

LAM, ALPHA = 0.5, 2.0
# Per-row tolerance of the exact fp32 mode.  The Gram matrix carries a relative rounding error of about
# 1e-6 (256-row fp32 partial sums, combined in fp64) that the solve amplifies by cond(A_u); for the
# factor matrices used here cond(A_u) stays below ~1e2.
TOL_EXACT = 1e-4


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def _rel(g, o):
    return np.linalg.norm(g.astype(np.float64) - o, axis=1) / np.maximum(np.linalg.norm(o, axis=1), 1e-30)


@pytest.fixture(scope="module")
def P():
    import paper_1808_03843_amd as pkg
    return pkg


@pytest.mark.parametrize("f,n", [(16, 1), (16, 777), (32, 5001), (64, 300), (100, 4099), (128, 2500), (256, 1), (256, 3001)])
def test_gram_matches_double_precision(P, f, n):
    G = W.random_factors(n, f, seed=100 + f, scale=0.4) + 0.1
    als = P.Als(f)
    got = als.gram(_dev(G)).cpu().numpy().astype(np.float64)
    als.close()
    ref = G.astype(np.float64).T @ G.astype(np.float64)
    assert np.abs(got - ref).max() <= 2e-6 * np.abs(ref).max()
    assert np.array_equal(got, got.T)


@pytest.mark.parametrize("chunk", [0, 64])
def test_one_exact_implicit_sweep_on_tiny(P, chunk):
    w = W.TINY
    a = W.generate(w)
    c = W.transpose(a)
    _, T0 = W.init_factors(w)
    als = P.Als(w.f, solver=P.SOLVER_CHOLESKY, chunk=chunk)
    csr = P.SparseMatrix.from_host(a.nrows, a.ncols, a.ptr, a.idx, a.val)
    csc = P.SparseMatrix.from_host(c.nrows, c.ncols, c.ptr, c.idx, c.val)
    X = torch.zeros((w.m, w.f), device="cuda:0")
    T = _dev(T0.copy())
    als.update_rows_implicit(csr, T, LAM, ALPHA, X)
    Xo = oracle.implicit_update_rows(a.ptr, a.idx, a.val, T0, LAM, ALPHA)
    ex = _rel(X.cpu().numpy(), Xo)
    # column side from the oracle's X (no oracle input comes from the GPU)
    Xin = Xo.astype(np.float32)
    als.update_cols_implicit(csc, _dev(Xin), LAM, ALPHA, T)
    als.synchronize()
    To = oracle.implicit_update_rows(c.ptr, c.idx, c.val, Xin, LAM, ALPHA)
    et = _rel(T.cpu().numpy(), To)
    als.close()
    print(f"tiny implicit chunk={chunk}: max row err X {ex.max():.2e}, Theta {et.max():.2e}", flush=True)
    assert ex.max() <= TOL_EXACT and et.max() <= TOL_EXACT


def test_implicit_f100_rows_of_every_kind(P):
    """f = 100 (strip tile row), rows from empty to split over several work items, stored zeros."""
    f, n = 100, 3000
    rng = np.random.default_rng(5)
    degrees = [0, 1, 2, 3, 4, 5, 63, 64, 65, 100, 255, 256, 257, 1023, 1024, 1025, 2047, 2500, 3000] + [int(d) for d in rng.integers(1, 400, 40)]
    ptr = np.concatenate([[0], np.cumsum(degrees)]).astype(np.int64)
    idx = np.concatenate([np.sort(rng.choice(n, d, replace=False)) for d in degrees] + [np.zeros(0, int)]).astype(np.int32)
    val = rng.integers(0, 6, size=int(ptr[-1])).astype(np.float32)   # zeros are stored but carry no weight
    Theta = W.random_factors(n, f, seed=9, scale=0.3)
    ref = oracle.implicit_update_rows(ptr, idx, val, Theta, LAM, ALPHA)
    for solver, chunk in [(P.SOLVER_CHOLESKY, 0), (P.SOLVER_CHOLESKY, 256)]:
        als = P.Als(f, solver=solver, chunk=chunk)
        sp = P.SparseMatrix.from_host(len(degrees), n, ptr, idx, val)
        X = torch.full((len(degrees), f), 7.0, device="cuda:0")
        als.update_rows_implicit(sp, _dev(Theta), LAM, ALPHA, X)
        als.synchronize()
        got = X.cpu().numpy()
        als.close()
        err = _rel(got, ref)
        print(f"implicit f=100 chunk={chunk}: max row err {err.max():.2e}", flush=True)
        assert np.all(got[0] == 0.0)            # n_u = 0
        assert err[1:].max() <= TOL_EXACT


def test_implicit_cg_sweeps_reach_the_exact_cost(P):
    """Approximate mode: after 10 sweeps the cost is within 2e-3 (relative) of the exact oracle's."""
    w = W.TINY
    a = W.generate(w)
    c = W.transpose(a)
    X0, T0 = W.init_factors(w)
    Xo, To = X0.astype(np.float64), T0.astype(np.float64)
    for _ in range(10):
        Xo = oracle.implicit_update_rows(a.ptr, a.idx, a.val, To, LAM, ALPHA)
        To = oracle.implicit_update_rows(c.ptr, c.idx, c.val, Xo, LAM, ALPHA)
    J_exact = oracle.implicit_objective(a.ptr, a.idx, a.val, Xo, To, LAM, ALPHA)
    als = P.Als(w.f, solver=P.SOLVER_CG, cg_iters=6)
    csr = P.SparseMatrix.from_host(a.nrows, a.ncols, a.ptr, a.idx, a.val)
    csc = P.SparseMatrix.from_host(c.nrows, c.ncols, c.ptr, c.idx, c.val)
    X, T = _dev(X0.copy()), _dev(T0.copy())
    for _ in range(10):
        als.update_rows_implicit(csr, T, LAM, ALPHA, X)
        als.update_cols_implicit(csc, X, LAM, ALPHA, T)
    als.synchronize()
    # the cost of the GPU's factors by the library's own cost kernel, which
    # test_implicit_loss_matches_the_sum_over_all_pairs checks against the oracle on seeded factors
    J_gpu = als.implicit_loss(csr, X, T, LAM, ALPHA)
    als.close()
    print(f"implicit CG(6) x10: J exact {J_exact:.6f}, J of the GPU factors {J_gpu:.6f}", flush=True)
    assert abs(J_gpu - J_exact) <= 2e-3 * J_exact


@pytest.mark.parametrize("name", ["tiny", "mid_small"])
def test_implicit_loss_matches_the_sum_over_all_pairs(P, name):
    w = W.CONFIGS[name]
    a = W.generate(w)
    X = W.random_factors(w.m, w.f, seed=31, scale=0.1)
    T = W.random_factors(w.n, w.f, seed=32, scale=0.1)
    als = P.Als(w.f)
    csr = P.SparseMatrix.from_host(a.nrows, a.ncols, a.ptr, a.idx, a.val)
    got = als.implicit_loss(csr, _dev(X), _dev(T), LAM, ALPHA)
    als.close()
    ref = oracle.implicit_objective(a.ptr, a.idx, a.val, X, T, LAM, ALPHA)
    print(f"{name}: implicit cost gpu {got:.6f} oracle {ref:.6f}", flush=True)
    assert abs(got - ref) <= 1e-5 * abs(ref)


def test_implicit_exact_sweeps_on_mid_small_never_raise_the_cost(P):
    """Sampled rows and columns against the oracle from seeded factors; then exact block-coordinate
    minimisation: the cost of the GPU's factors cannot go up."""
    w = W.MID_SMALL
    a = W.generate(w)
    c = W.transpose(a)
    X0, T0 = W.init_factors(w)
    als = P.Als(w.f, solver=P.SOLVER_CHOLESKY)
    csr = P.SparseMatrix.from_host(a.nrows, a.ncols, a.ptr, a.idx, a.val)
    csc = P.SparseMatrix.from_host(c.nrows, c.ncols, c.ptr, c.idx, c.val)
    rng = np.random.default_rng(3)
    rows = np.unique(np.concatenate([rng.choice(w.m, 150, replace=False), np.argsort(np.diff(a.ptr))[-4:]]))
    cols = np.unique(np.concatenate([rng.choice(w.n, 60, replace=False), np.argsort(np.diff(c.ptr))[-4:]]))
    # parity on seeded inputs only: rows from T0, columns from a seeded X
    Xs = W.random_factors(w.m, w.f, seed=41, scale=0.2)
    out_x = torch.zeros((w.m, w.f), device="cuda:0")
    out_t = torch.zeros((w.n, w.f), device="cuda:0")
    als.update_rows_implicit(csr, _dev(T0), LAM, ALPHA, out_x)
    als.update_cols_implicit(csc, _dev(Xs), LAM, ALPHA, out_t)
    als.synchronize()
    ex = _rel(out_x.cpu().numpy()[rows], oracle.implicit_update_selected(rows, a.ptr, a.idx, a.val, T0, LAM, ALPHA))
    et = _rel(out_t.cpu().numpy()[cols], oracle.implicit_update_selected(cols, c.ptr, c.idx, c.val, Xs, LAM, ALPHA))
    print(f"mid_small implicit: sampled rows {ex.max():.2e}, columns {et.max():.2e}", flush=True)
    assert ex.max() <= TOL_EXACT and et.max() <= TOL_EXACT
    X, T = _dev(X0.copy()), _dev(T0.copy())
    prev = oracle.implicit_objective(a.ptr, a.idx, a.val, X0, T0, LAM, ALPHA)
    for sweep in range(2):
        als.update_rows_implicit(csr, T, LAM, ALPHA, X)
        als.update_cols_implicit(csc, X, LAM, ALPHA, T)
        als.synchronize()
        cur = als.implicit_loss(csr, X, T, LAM, ALPHA)   # checked against the oracle on seeded factors elsewhere
        print(f"mid_small implicit sweep {sweep + 1}: cost {cur:.4f} (before {prev:.4f})", flush=True)
        assert cur <= prev * (1 + 1e-6)
        prev = cur
    als.close()


def test_implicit_argument_errors(P):
    w = W.TINY
    a = W.generate(w)
    csr = P.SparseMatrix.from_host(a.nrows, a.ncols, a.ptr, a.idx, a.val)
    X = torch.zeros((w.m, w.f), device="cuda:0")
    T = torch.zeros((w.n, w.f), device="cuda:0")
    als = P.Als(w.f)
    with pytest.raises(P.AlsError):
        als.update_rows_implicit(csr, T, LAM, -1.0, X)
    als.close()
    als = P.Als(w.f, solver=P.SOLVER_CG, factor_dtype=P.F32X3)      # the three-part route is explicit feedback only
    with pytest.raises(P.AlsError):
        als.update_rows_implicit(csr, T, LAM, ALPHA, X)
    als.close()
    als = P.Als(256, solver=P.SOLVER_CG, factor_dtype=P.BF16)        # 16-bit implicit updates exist for f <= 128
    with pytest.raises(P.AlsError):
        als.update_rows_implicit(csr, torch.zeros((w.n, 256), device="cuda:0", dtype=torch.bfloat16), LAM, ALPHA,
                                 torch.zeros((w.m, 256), device="cuda:0"))
    als.close()
    als = P.Als(w.f, solver=P.SOLVER_CG, herm_dtype=P.BF16)   # reduced-precision storage of A_u: explicit mode only
    with pytest.raises(P.AlsError):
        als.update_rows_implicit(csr, T, LAM, ALPHA, X)
    als.close()


@pytest.mark.parametrize("f,name,chunk", [(f, n, c) for f in (16, 32, 64, 100, 128) for n in ("bf16", "f16") for c in (0, 128)])
def test_implicit_with_sixteen_bit_factor_inputs(P, f, name, chunk):
    """The gathered factor in 16 bits (f <= 128): the weighted sum runs on the 16-bit matrix cores with w * theta cut
    into three 16-bit parts, Theta^T Theta from the same rounded factor.  Against the all-columns oracle on the
    rounded factor: exact solver at 1e-4 per row, and Algorithm 1 with f iterations (exact then) at 1e-3."""
    ncols = 3000
    rng = np.random.default_rng(77)
    degrees = [0, 1, 2, 3, 5, 15, 16, 17, 31, 32, 33, 63, 64, 65, 127, 129, 255, 257, 511, 1000, 1025, 2049, 2900]
    degrees += [int(np.exp(rng.uniform(0, np.log(2500)))) for _ in range(25)]
    ptr = np.concatenate([[0], np.cumsum(degrees)]).astype(np.int64)
    idx = np.concatenate([np.sort(rng.choice(ncols, d, replace=False)) for d in degrees] + [np.zeros(0, int)]).astype(np.int32)
    val = (rng.integers(0, 6, size=int(ptr[-1])) * 1.37).astype(np.float32)     # stored zeros, non-integer counts
    tdt, code = (torch.bfloat16, P.BF16) if name == "bf16" else (torch.float16, P.F16)
    T16 = torch.from_numpy(W.random_factors(ncols, f, seed=67 + f, scale=0.3)).cuda().to(tdt)
    T_rounded = T16.to(torch.float32).cpu().numpy()
    warm = W.random_factors(len(degrees), f, seed=68 + f, scale=0.05)
    sp = P.SparseMatrix.from_host(len(degrees), ncols, ptr, idx, val)
    ref = oracle.implicit_update_rows(ptr, idx, val, T_rounded, LAM, ALPHA)
    for solver, fs, tol in ((P.SOLVER_CHOLESKY, 0, TOL_EXACT), (P.SOLVER_CG, f, 1e-3)):
        als = P.Als(f, solver=solver, cg_iters=fs, chunk=chunk, factor_dtype=code)
        X = _dev(warm.copy())
        als.update_rows_implicit(sp, T16, LAM, ALPHA, X)
        als.synchronize()
        got = X.cpu().numpy()
        als.close()
        assert np.all(got[0] == 0.0)
        err = _rel(got[1:], ref[1:])
        assert err.max() <= tol, (name, int(err.argmax()) + 1, float(err.max()))


def test_implicit_cg_sweeps_with_bf16_inputs_reach_the_exact_cost(P):
    """Ten implicit sweeps of the tiny workload with CG(6) and bf16 factor inputs end within 2e-3 (relative) of the
    cost the exact double-precision oracle sweeps reach (the all-columns oracle is O(m n f^2) per half-sweep)."""
    w = W.TINY
    a = W.generate(w)
    c = W.transpose(a)
    X0, T0 = W.init_factors(w)
    Xo, To = X0.astype(np.float64), T0.astype(np.float64)
    for _ in range(10):
        Xo = oracle.implicit_update_rows(a.ptr, a.idx, a.val, To, LAM, ALPHA)
        To = oracle.implicit_update_rows(c.ptr, c.idx, c.val, Xo, LAM, ALPHA)
    cost_o = oracle.implicit_objective(a.ptr, a.idx, a.val, Xo, To, LAM, ALPHA)
    als = P.Als(w.f, solver=P.SOLVER_CG, cg_iters=6, factor_dtype=P.BF16)
    ev = P.Als(w.f)
    csr = P.SparseMatrix.from_host(a.nrows, a.ncols, a.ptr, a.idx, a.val)
    csc = P.SparseMatrix.from_host(c.nrows, c.ncols, c.ptr, c.idx, c.val)
    X, T = _dev(X0), _dev(T0)
    for _ in range(10):
        als.update_rows_implicit(csr, T.to(torch.bfloat16), LAM, ALPHA, X)
        als.update_cols_implicit(csc, X.to(torch.bfloat16), LAM, ALPHA, T)
    als.synchronize()
    cost = ev.implicit_loss(csr, X, T, LAM, ALPHA)
    print(f"tiny implicit, bf16 inputs, CG(6): cost {cost:.4f}, exact oracle {cost_o:.4f}")
    assert abs(cost - cost_o) <= 2e-3 * cost_o
    als.close()
    ev.close()
