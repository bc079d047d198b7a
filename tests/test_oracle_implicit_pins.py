"""Pins of the implicit-feedback oracle (Section 5.6) against facts independent of it.

The paper gives the cost function only: sum over all pairs of c_uv (p_uv - x_u.theta_v)^2 with
p_uv = [r_uv > 0], c_uv = 1 + alpha r_uv.  The pins are the weighted least-squares problem solved by QR
over all columns, closed forms, the reduction to the (already pinned) explicit update, and the
monotone cost of exact block-coordinate minimisation.
"""
import numpy as np
import pytest

import oracle


def _row(rng, n, f, d, zeros=0):
    idx = np.sort(rng.choice(n, size=d, replace=False)).astype(np.int32)
    r = rng.integers(1, 6, size=d).astype(np.float32)
    if zeros:
        r[rng.choice(d, size=zeros, replace=False)] = 0.0   # stored, but not a positive observation
    Theta = rng.standard_normal((n, f)) * 0.5
    return idx, r, Theta


def _dense(n, idx, r):
    full = np.zeros(n)
    full[idx] = np.maximum(r.astype(np.float64), 0.0)
    return full


@pytest.mark.parametrize("f,d,n,alpha", [(1, 1, 7, 2.0), (3, 4, 25, 0.5), (6, 10, 40, 40.0), (16, 30, 90, 1.0),
                                         (5, 0, 12, 3.0)])
def test_row_update_equals_weighted_qr_over_all_columns(f, d, n, alpha):
    rng = np.random.default_rng(7 * f + d)
    lam = 0.3
    idx, r, Theta = _row(rng, n, f, d, zeros=min(d // 3, 2))
    full = _dense(n, idx, r)
    c, p = 1.0 + alpha * full, (full > 0).astype(np.float64)
    # min_x sum_v c_v (p_v - x.theta_v)^2 + lam |x|^2 as one least-squares problem (no normal equations)
    aug = np.vstack([np.sqrt(c)[:, None] * Theta, np.sqrt(lam) * np.eye(f)])
    rhs = np.concatenate([np.sqrt(c) * p, np.zeros(f)])
    x_ref = np.linalg.lstsq(aug, rhs, rcond=None)[0]
    x = oracle.implicit_update_rows(np.array([0, d], np.int64), idx, r, Theta, lam, alpha)[0]
    assert np.allclose(x, x_ref, rtol=1e-9, atol=1e-11)


def test_f1_closed_form():
    rng = np.random.default_rng(3)
    n, d, lam, alpha = 30, 8, 0.7, 4.0
    idx, r, Theta = _row(rng, n, 1, d)
    t = Theta[:, 0]
    full = _dense(n, idx, r)
    expect = np.sum((1 + alpha * full) * (full > 0) * t) / (np.sum((1 + alpha * full) * t * t) + lam)
    x = oracle.implicit_update_rows(np.array([0, d], np.int64), idx, r, Theta, lam, alpha)[0, 0]
    assert x == pytest.approx(expect, rel=1e-12)


def test_alpha_zero_is_ridge_regression_on_the_indicator():
    rng = np.random.default_rng(4)
    n, f, d, lam = 50, 6, 12, 0.2
    idx, r, Theta = _row(rng, n, f, d)
    x = oracle.implicit_update_rows(np.array([0, d], np.int64), idx, r, Theta, lam, 0.0)[0]
    expect = np.linalg.solve(Theta.T @ Theta + lam * np.eye(f), Theta[idx].sum(axis=0))
    assert np.allclose(x, expect, rtol=1e-10)


def test_regulariser_is_not_weighted_by_degree_and_every_column_counts():
    rng = np.random.default_rng(8)
    n, f, d, lam, alpha = 40, 4, 6, 0.5, 2.0
    idx, r, Theta = _row(rng, n, f, d)
    A, b = oracle.implicit_normal_eq(idx, r, Theta, lam, alpha)
    G = Theta[idx]
    w = alpha * r.astype(np.float64)
    expect_A = Theta.T @ Theta + (G * w[:, None]).T @ G + lam * np.eye(f)   # the shortcut of the method's source
    assert np.allclose(A, expect_A, rtol=1e-11)
    assert np.allclose(b, ((1 + w)[:, None] * G).sum(axis=0), rtol=1e-11)
    # leaving out the unobserved columns, or weighting lambda by n_u, must fail
    assert not np.allclose(A, (G * (1 + w)[:, None]).T @ G + lam * np.eye(f), rtol=1e-3)
    assert not np.allclose(A, expect_A + lam * (d - 1) * np.eye(f), rtol=1e-3)


def test_fully_observed_row_reduces_to_the_explicit_update():
    # every column observed with r > 0: the implicit row problem is an ordinary weighted least squares,
    # i.e. the explicit update (eq. (2)) on theta' = sqrt(c) theta, r' = sqrt(c), lambda' = lambda / n
    rng = np.random.default_rng(9)
    n, f, lam, alpha = 14, 5, 0.35, 1.5
    idx = np.arange(n, dtype=np.int32)
    r = rng.integers(1, 6, size=n).astype(np.float32)
    Theta = rng.standard_normal((n, f))
    c = 1 + alpha * r.astype(np.float64)
    ptr = np.array([0, n], np.int64)
    x_imp = oracle.implicit_update_rows(ptr, idx, r, Theta, lam, alpha)[0]
    x_exp = oracle.update_rows(ptr, idx, np.sqrt(c).astype(np.float32), np.sqrt(c)[:, None] * Theta, lam / n)[0]
    assert np.allclose(x_imp, x_exp, rtol=1e-6)   # sqrt(c) passes through float32 on the explicit side


def test_stored_nonpositive_rating_counts_as_missing():
    rng = np.random.default_rng(10)
    n, f, lam, alpha = 20, 3, 0.1, 2.0
    idx, r, Theta = _row(rng, n, f, 6)
    r2 = r.copy()
    r2[[1, 4]] = [0.0, -3.0]
    keep = r2 > 0
    ptr = lambda k: np.array([0, k], np.int64)
    a = oracle.implicit_update_rows(ptr(6), idx, r2, Theta, lam, alpha)[0]
    b = oracle.implicit_update_rows(ptr(int(keep.sum())), idx[keep], r2[keep], Theta, lam, alpha)[0]
    assert np.allclose(a, b, rtol=1e-12)


def test_objective_is_the_dense_sum_and_decreases_under_exact_half_sweeps():
    rng = np.random.default_rng(11)
    m, n, f, lam, alpha = 30, 22, 4, 0.4, 3.0
    dense = (rng.random((m, n)) < 0.2) * rng.integers(1, 6, size=(m, n))
    ptr = np.concatenate([[0], np.cumsum((dense > 0).sum(axis=1))]).astype(np.int64)
    idx = np.concatenate([np.nonzero(row)[0] for row in dense]).astype(np.int32)
    val = dense[dense > 0].astype(np.float32)   # row-major order == CSR order
    cptr, cidx, cval = oracle.csr_to_csc(m, n, ptr, idx, val)
    X = rng.standard_normal((m, f)) * 0.1
    T = rng.standard_normal((n, f)) * 0.1
    C, P = 1 + alpha * dense, (dense > 0).astype(np.float64)
    J = lambda X, T: float((C * (P - X @ T.T) ** 2).sum() + lam * ((X ** 2).sum() + (T ** 2).sum()))
    assert oracle.implicit_objective(ptr, idx, val, X, T, lam, alpha) == pytest.approx(J(X, T), rel=1e-12)
    prev = J(X, T)
    for _ in range(3):
        X = oracle.implicit_update_rows(ptr, idx, val, T, lam, alpha)
        mid = J(X, T)
        T = oracle.implicit_update_rows(cptr, cidx, cval, X, lam, alpha)
        cur = J(X, T)
        assert mid <= prev * (1 + 1e-12) and cur <= mid * (1 + 1e-12)
        prev = cur
    # gradient of the cost in x_u vanishes at the update
    u = 3
    g = -2 * ((C[u] * (P[u] - T @ X[u]))[:, None] * T).sum(axis=0) + 2 * lam * X[u]
    X = oracle.implicit_update_rows(ptr, idx, val, T, lam, alpha)
    g = -2 * ((C[u] * (P[u] - T @ X[u]))[:, None] * T).sum(axis=0) + 2 * lam * X[u]
    assert np.abs(g).max() < 1e-9
