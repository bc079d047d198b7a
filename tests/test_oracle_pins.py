"""Pins of the CPU oracle against facts the paper and the mathematics fix.

The paper prints no worked numeric example, so the pins are closed forms,
brute force by an independent route (QR least squares, no normal equations),
invariants of exact block-coordinate minimisation and CG theory.
"""
import numpy as np
import pytest

import oracle
import workload as W


def _rand_row(rng, n, f, d):
    idx = np.sort(rng.choice(n, size=d, replace=False)).astype(np.int32)
    r = rng.integers(1, 6, size=d).astype(np.float32)
    Theta = rng.standard_normal((n, f)) * 0.7
    return idx, r, Theta


# ---- P1: brute force, eq. (2) is the minimiser of the row's part of eq. (1) -------------
@pytest.mark.parametrize("f,d", [(1, 1), (3, 2), (4, 9), (7, 7), (16, 40), (10, 3)])
def test_row_update_equals_qr_least_squares(f, d):
    rng = np.random.default_rng(100 + 10 * f + d)
    n, lam = 60, 0.05
    idx, r, Theta = _rand_row(rng, n, f, d)
    # min_x sum_v (r_v - x.theta_v)^2 + lam*n_u*|x|^2  ==  min || [G; sqrt(lam n_u) I] x - [r; 0] ||
    G = Theta[idx]
    aug = np.vstack([G, np.sqrt(lam * d) * np.eye(f)])
    rhs = np.concatenate([r.astype(np.float64), np.zeros(f)])
    x_ref = np.linalg.lstsq(aug, rhs, rcond=None)[0]
    ptr = np.array([0, d], np.int64)
    x = oracle.update_rows(ptr, idx, r, Theta, lam)[0]
    assert np.allclose(x, x_ref, rtol=1e-9, atol=1e-11)


def test_regulariser_is_weighted_by_row_degree():
    # plain lambda*I (no n_u) must NOT reproduce the oracle: guards the reading of eq. (2)
    rng = np.random.default_rng(5)
    idx, r, Theta = _rand_row(rng, 30, 4, 6)
    x = oracle.update_rows(np.array([0, 6], np.int64), idx, r, Theta, 0.3)[0]
    G = Theta[idx]
    x_unweighted = np.linalg.solve(G.T @ G + 0.3 * np.eye(4), G.T @ r)
    x_weighted = np.linalg.solve(G.T @ G + 0.3 * 6 * np.eye(4), G.T @ r)
    assert np.allclose(x, x_weighted, rtol=1e-10)
    assert not np.allclose(x, x_unweighted, rtol=1e-3)


# ---- P2: f = 1 closed form ------------------------------------------------------------------
def test_f1_closed_form():
    rng = np.random.default_rng(1)
    idx, r, Theta = _rand_row(rng, 40, 1, 11)
    lam = 0.2
    t = Theta[idx, 0]
    expect = np.sum(r * t) / (np.sum(t * t) + lam * 11)
    x = oracle.update_rows(np.array([0, 11], np.int64), idx, r, Theta, lam)[0, 0]
    assert x == pytest.approx(expect, rel=1e-13)


# ---- P3: all theta equal (Sherman-Morrison), includes n_u = 1 ------------------------------
@pytest.mark.parametrize("d", [1, 2, 17])
def test_identical_theta_closed_form(d):
    rng = np.random.default_rng(7 + d)
    f, n, lam = 6, 50, 0.05
    theta = rng.standard_normal(f)
    Theta = np.tile(theta, (n, 1))
    idx = np.sort(rng.choice(n, d, replace=False)).astype(np.int32)
    r = rng.integers(1, 6, d).astype(np.float32)
    expect = (r.astype(np.float64).sum() / d) * theta / (theta @ theta + lam)
    x = oracle.update_rows(np.array([0, d], np.int64), idx, r, Theta, lam)[0]
    assert np.allclose(x, expect, rtol=1e-11, atol=1e-13)


# ---- P4: orthonormal thetas -----------------------------------------------------------------
def test_orthonormal_closed_form():
    f, lam = 9, 0.4
    Theta = np.eye(f)
    idx = np.arange(f, dtype=np.int32)
    r = np.arange(1, f + 1).astype(np.float32)
    x = oracle.update_rows(np.array([0, f], np.int64), idx, r, Theta, lam)[0]
    assert np.allclose(x, r.astype(np.float64) / (1 + lam * f), rtol=1e-13)


# ---- stored zeros are observations; empty rows give zero -----------------------------------
def test_stored_zero_counts_as_observation_and_empty_row_is_zero():
    rng = np.random.default_rng(3)
    f, n, lam = 5, 20, 0.1
    Theta = rng.standard_normal((n, f))
    idx = np.array([2, 5, 9], np.int32)
    r = np.array([4.0, 0.0, 2.0], np.float32)
    ptr = np.array([0, 3, 3], np.int64)          # second row is empty
    X = oracle.update_rows(ptr, idx, r, Theta, lam)
    G = Theta[idx]
    expect = np.linalg.solve(G.T @ G + lam * 3 * np.eye(f), G.T @ r)
    assert np.allclose(X[0], expect, rtol=1e-11)
    assert np.all(X[1] == 0.0)
    A, b = oracle.normal_eq(idx, r, Theta, lam)
    assert np.allclose(A, G.T @ G + lam * 3 * np.eye(f), rtol=1e-13)
    assert np.allclose(b, G.T @ r, rtol=1e-13)


# ---- P5: residual of the normal equations, on the tiny workload -----------------------------
def test_normal_equation_residual_on_tiny():
    w = W.TINY
    a = W.generate(w)
    _, T0 = W.init_factors(w)
    X = oracle.update_rows(a.ptr, a.idx, a.val, T0, w.lam)
    worst = 0.0
    for u in range(0, w.m, 37):
        s, e = a.ptr[u], a.ptr[u + 1]
        A, b = oracle.normal_eq(a.idx[s:e], a.val[s:e], T0, w.lam)
        # A must be symmetric and the gradient of the row objective must vanish
        assert np.array_equal(A, A.T)
        worst = max(worst, np.linalg.norm(A @ X[u] - b) / np.linalg.norm(b))
    assert worst < 1e-12


def test_cholesky_matches_library_solver():
    rng = np.random.default_rng(9)
    for f in (1, 2, 5, 33):
        M = rng.standard_normal((f + 3, f))
        A = M.T @ M + 0.1 * np.eye(f)
        b = rng.standard_normal(f)
        assert np.allclose(oracle.cholesky_solve(A, b), np.linalg.solve(A, b), rtol=1e-9, atol=1e-12)
    with pytest.raises(np.linalg.LinAlgError):
        oracle.cholesky_solve(np.array([[1.0, 2.0], [2.0, 1.0]]), np.ones(2))


# ---- P6: exact half-sweeps never increase the objective of eq. (1) --------------------------
def test_objective_non_increasing_and_rmse_trend_on_tiny():
    w = W.TINY
    a = W.generate(w)
    c = W.transpose(a)
    X0, T0 = W.init_factors(w)
    csr, csc = (a.ptr, a.idx, a.val), (c.ptr, c.idx, c.val)
    X, T = X0.astype(np.float64), T0.astype(np.float64)
    J = [oracle.objective(*csr, X, T, w.lam)]
    rm = []
    for _ in range(w.sweeps):
        X = oracle.update_rows(*csr, T, w.lam)
        J.append(oracle.objective(*csr, X, T, w.lam))
        T = oracle.update_rows(*csc, X, w.lam)
        J.append(oracle.objective(*csr, X, T, w.lam))
        rm.append(oracle.rmse(*csr, X, T))
    assert all(J[i + 1] <= J[i] * (1 + 1e-12) for i in range(len(J) - 1)), J
    assert all(rm[i + 1] <= rm[i] + 1e-12 for i in range(len(rm) - 1)), rm
    assert rm[-1] < 0.5 * rm[0] or rm[-1] < 0.6


def test_objective_and_rmse_against_dense_numpy():
    rng = np.random.default_rng(21)
    m, n, f, lam = 13, 11, 3, 0.07
    mask = rng.random((m, n)) < 0.35
    R = np.where(mask, rng.integers(0, 6, (m, n)), 0).astype(np.float32)   # stored zeros possible
    ptr = np.concatenate([[0], np.cumsum(mask.sum(1))]).astype(np.int64)
    idx = np.concatenate([np.nonzero(mask[u])[0] for u in range(m)]).astype(np.int32)
    val = np.concatenate([R[u, mask[u]] for u in range(m)]).astype(np.float32)
    X, T = rng.standard_normal((m, f)), rng.standard_normal((n, f))
    E = (R - X @ T.T) * mask
    sse = float((E ** 2).sum())
    reg = lam * ((mask.sum(1) * (X ** 2).sum(1)).sum() + (mask.sum(0) * (T ** 2).sum(1)).sum())
    assert oracle.sse(ptr, idx, val, X, T, parallel=False) == pytest.approx(sse, rel=1e-12)
    assert oracle.sse(ptr, idx, val, X, T, parallel=True) == oracle.sse(ptr, idx, val, X, T, parallel=False)
    assert oracle.objective(ptr, idx, val, X, T, lam) == pytest.approx(sse + reg, rel=1e-12)
    assert oracle.rmse(ptr, idx, val, X, T) == pytest.approx(np.sqrt(sse / mask.sum()), rel=1e-12)


# ---- P7 / P8: Algorithm 1 ---------------------------------------------------------------------
def test_cg_with_f_iterations_is_exact():
    rng = np.random.default_rng(31)
    for f in (4, 16, 40):
        idx, r, Theta = _rand_row(rng, 200, f, 3 * f)
        A, b = oracle.normal_eq(idx, r, Theta, 0.05)
        x, it = oracle.cg(A, np.zeros(f), b, fs=f, eps=0.0)
        assert it <= f
        assert np.allclose(x, oracle.cholesky_solve(A, b), rtol=1e-7, atol=1e-9)


def test_cg_finite_termination_two_eigenvalues():
    # A = n (theta theta^T + lam I) has two distinct eigenvalues: exact after 2 iterations from x = 0
    rng = np.random.default_rng(33)
    f = 12
    theta = rng.standard_normal(f)
    A = 5 * (np.outer(theta, theta) + 0.3 * np.eye(f))
    b = rng.standard_normal(f)
    x2, _ = oracle.cg(A, np.zeros(f), b, fs=2)
    x1, _ = oracle.cg(A, np.zeros(f), b, fs=1)
    exact = np.linalg.solve(A, b)
    assert np.allclose(x2, exact, rtol=1e-10, atol=1e-12)
    assert not np.allclose(x1, exact, rtol=1e-4)


def test_cg_residual_decreases_in_energy_norm_and_guards():
    rng = np.random.default_rng(35)
    f = 20
    idx, r, Theta = _rand_row(rng, 100, f, 50)
    A, b = oracle.normal_eq(idx, r, Theta, 0.05)
    exact = np.linalg.solve(A, b)
    x0 = rng.standard_normal(f)
    prev = None
    for fs in range(0, 8):
        x, it = oracle.cg(A, x0, b, fs=fs)
        err = (x - exact) @ A @ (x - exact)
        assert it == fs
        if prev is not None:
            assert err < prev      # CG minimises the A-norm error over growing Krylov spaces
        prev = err
    # warm start at the solution / zero right-hand side: nothing to do, no 0/0
    x, it = oracle.cg(A, np.zeros(f), np.zeros(f), fs=6)
    assert it == 0 and np.all(x == 0)
    # tolerance stops early
    _, it = oracle.cg(A, x0, b, fs=f, eps=1e-3 * np.linalg.norm(b))
    assert it < f


def test_cg_first_step_is_steepest_descent():
    # independent closed form of iteration 1: x1 = x0 + (r.r / r.A r) r
    rng = np.random.default_rng(36)
    f = 7
    M = rng.standard_normal((f + 2, f))
    A = M.T @ M + 0.2 * np.eye(f)
    b, x0 = rng.standard_normal(f), rng.standard_normal(f)
    r0 = b - A @ x0
    expect = x0 + (r0 @ r0) / (r0 @ A @ r0) * r0
    x1, _ = oracle.cg(A, x0, b, fs=1)
    assert np.allclose(x1, expect, rtol=1e-12)


def test_cg_sweep_approaches_exact_sweep():
    w = W.TINY
    a = W.generate(w)
    X0, T0 = W.init_factors(w)
    exact = oracle.update_rows(a.ptr, a.idx, a.val, T0, w.lam)
    approx = oracle.update_rows_cg(a.ptr, a.idx, a.val, T0, w.lam, X0, fs=w.f)
    assert np.allclose(approx, exact, rtol=1e-6, atol=1e-8)
    rough = oracle.update_rows_cg(a.ptr, a.idx, a.val, T0, w.lam, X0, fs=3)
    assert np.linalg.norm(rough - exact) / np.linalg.norm(exact) < 0.2


def _krylov_minimiser(A, x0, b, k):
    """Iterate k of CG by its defining property, with no recurrence: the point of x0 + span{r0, A r0, ..., A^(k-1) r0}
    that minimises the A-norm of the error (equivalently solves the projected system)."""
    r0 = b - A @ x0
    if k == 0:
        return x0.copy()
    K = np.empty((len(b), k))
    v = r0.copy()
    for j in range(k):
        K[:, j] = v / np.linalg.norm(v)
        v = A @ K[:, j]
    Q, _ = np.linalg.qr(K)          # orthonormal basis: the projected system stays well conditioned
    y = np.linalg.solve(Q.T @ A @ Q, Q.T @ r0)
    return x0 + Q @ y


@pytest.mark.parametrize("fs", [0, 1, 3])
def test_cg_sweep_uses_each_rows_warm_start(fs):
    # Algorithm 1 takes x as an input: the sweep must start row u from row u of the matrix handed in
    # (not from 0, not from another row), must leave it alone for f_s = 0 and must zero rows without entries.
    rng = np.random.default_rng(70 + fs)
    m, n, f, lam = 9, 40, 6, 0.05
    deg = [12, 0, 7, 25, 1, 0, 9, 30, 14]
    ptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int64)
    idx = np.concatenate([np.sort(rng.choice(n, size=d, replace=False)) for d in deg]).astype(np.int32)
    val = rng.integers(1, 6, size=int(ptr[-1])).astype(np.float32)
    Theta = rng.standard_normal((n, f)) * 0.7
    warm = rng.standard_normal((m, f))
    got = oracle.update_rows_cg(ptr, idx, val, Theta, lam, warm, fs=fs)
    for u in range(m):
        s, e = ptr[u], ptr[u + 1]
        if e == s:
            assert np.all(got[u] == 0.0)          # no entries: x_u = 0 whatever the warm start
            continue
        A, b = oracle.normal_eq(idx[s:e], val[s:e], Theta, lam)
        via_cg, _ = oracle.cg(A, warm[u], b, fs=fs)
        assert np.array_equal(got[u], via_cg)      # the same routine on the same row: bit for bit
        # and by an independent route: the Krylov-space minimiser started from THIS row's warm start
        assert np.allclose(got[u], _krylov_minimiser(A, warm[u], b, fs), rtol=1e-8, atol=1e-10)
        if fs == 0:
            assert np.array_equal(got[u], warm[u])
        elif e - s >= f:   # (a row with few entries has few distinct eigenvalues: CG is exact from any start)
            other = _krylov_minimiser(A, warm[(u + 2) % m], b, fs)
            cold = _krylov_minimiser(A, np.zeros(f), b, fs)
            assert not np.allclose(got[u], other, rtol=1e-3) and not np.allclose(got[u], cold, rtol=1e-3)


def test_cg_sweep_stays_at_the_exact_solution():
    # a warm start that already solves every row's system is a fixed point (r0 = 0 guard), to rounding
    w = W.TINY
    a = W.generate(w)
    _, T0 = W.init_factors(w)
    exact = oracle.update_rows(a.ptr, a.idx, a.val, T0, w.lam)
    again = oracle.update_rows_cg(a.ptr, a.idx, a.val, T0, w.lam, exact, fs=4)
    assert np.allclose(again, exact, rtol=1e-9, atol=1e-12)


# ---- P9 / P10: index work -------------------------------------------------------------------
def test_csr_to_csc_invariants_and_scipy_crosscheck():
    for w in (W.TINY, W.SQUARE_SMALL):
        a = W.generate(w)
        cptr, cidx, cval = oracle.csr_to_csc(w.m, w.n, a.ptr, a.idx, a.val)
        assert cptr[0] == 0 and cptr[-1] == a.nnz
        assert np.array_equal(np.diff(cptr), np.bincount(a.idx, minlength=w.n))
        for v in range(0, w.n, 41):
            seg = cidx[cptr[v]:cptr[v + 1]]
            assert np.all(np.diff(seg) > 0)
        t = W.transpose(a)
        assert np.array_equal(t.ptr, cptr) and np.array_equal(t.idx, cidx) and np.array_equal(t.val, cval)
        # transposing twice is the identity
        p2, i2, v2 = oracle.csr_to_csc(w.n, w.m, cptr, cidx, cval)
        assert np.array_equal(p2, a.ptr) and np.array_equal(i2, a.idx) and np.array_equal(v2, a.val)


def test_column_update_is_row_update_of_transpose():
    w = W.TINY
    a = W.generate(w)
    c = W.transpose(a)
    rng = np.random.default_rng(2)
    X = rng.standard_normal((w.m, w.f))
    T = oracle.update_rows(c.ptr, c.idx, c.val, X, w.lam)
    # theta_v by brute force from the column's entries (eq. (3))
    for v in (0, 17, 999):
        rows = c.idx[c.ptr[v]:c.ptr[v + 1]]
        r = c.val[c.ptr[v]:c.ptr[v + 1]].astype(np.float64)
        G = X[rows]
        expect = np.linalg.solve(G.T @ G + w.lam * len(rows) * np.eye(w.f), G.T @ r)
        assert np.allclose(T[v], expect, rtol=1e-9, atol=1e-12)


def test_update_selected_equals_full_update():
    w = W.TINY
    a = W.generate(w)
    _, T0 = W.init_factors(w)
    full = oracle.update_rows(a.ptr, a.idx, a.val, T0, w.lam)
    rows = np.array([0, 5, 77, 1999], np.int64)
    sel = oracle.update_selected(rows, a.ptr, a.idx, a.val, T0, w.lam)
    assert np.array_equal(sel, full[rows])


def test_bin_rows_is_stable_partition_by_class():
    ptr = np.concatenate([[0], np.cumsum([0, 1, 5, 2, 300, 0, 3, 64, 63, 1, 100000])]).astype(np.int64)
    nclass = 12
    perm, start = oracle.bin_rows(ptr, nclass)
    deg = np.diff(ptr)
    cls = np.where(deg > 0, 1 + np.floor(np.log2(np.maximum(deg, 1))).astype(int), 0)
    cls = np.minimum(cls, nclass - 1)
    expect = np.argsort(-cls, kind="stable").astype(np.int32)
    assert np.array_equal(perm, expect)
    assert start[0] == 0 and start[-1] == len(deg)
    for c in range(nclass):
        seg = perm[start[nclass - 1 - c]:start[nclass - c]]
        assert np.all(cls[seg] == c)


def test_rmse_f32_variant_equals_the_double_one_on_float_inputs():
    w = W.TINY
    a = W.generate(w)
    X = W.random_factors(w.m, w.f, seed=1, scale=0.3)
    T = W.random_factors(w.n, w.f, seed=2, scale=0.3)
    assert oracle.rmse_f32(a.ptr, a.idx, a.val, X, T) == oracle.rmse(a.ptr, a.idx, a.val, X, T)


@pytest.mark.parametrize("f,d", [(8, 1), (8, 5), (16, 15), (40, 31), (100, 63)])
def test_row_update_equals_the_dual_form(f, d):
    """For a row with fewer entries than features the minimiser of eq. (2) is also x = G^T y with
    (G G^T + lambda n I_n) y = r (push-through identity), the form the library solves for such rows.  The oracle
    forms the f x f system; the dual one is solved here with a library routine."""
    rng = np.random.default_rng(40 + f + d)
    n = 200
    Theta = W.random_factors(n, f, seed=3 * f + d, scale=0.4)
    cols = np.sort(rng.choice(n, d, replace=False)).astype(np.int32)
    r = rng.standard_normal(d).astype(np.float32) * 3
    lam = 0.07
    ptr = np.array([0, d], np.int64)
    x = oracle.update_rows(ptr, cols, r, Theta, lam)[0]
    G = Theta[cols].astype(np.float64)
    y = np.linalg.solve(G @ G.T + lam * d * np.eye(d), r.astype(np.float64))
    assert np.abs(x - G.T @ y).max() <= 1e-10 * max(np.abs(x).max(), 1e-30)
