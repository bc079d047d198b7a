"""Seeded random sweep over the configuration space: factor width, solver, input type, chunk, batch size, offset
width, explicit / implicit, bf16 slot storage, and degree patterns drawn around every boundary the kernels have
(steps of 4, 16 and 32 entries, the dual-form sizes, the chunk size and its multiples, full rows, empty rows).
Every case is one half-sweep through the C ABI against the oracle on the same seeded inputs; the side entry points
(A_u and b_u, RMSE, binning, CSR -> CSC) get a sweep of their own."""
import numpy as np
import pytest

import oracle
import workload as W

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _rel(g, o):
    # rows whose exact solution is 0 (all ratings 0 in implicit mode) are compared absolutely
    return np.linalg.norm(g.astype(np.float64) - o, axis=1) / np.maximum(np.linalg.norm(o, axis=1), 1e-3)


def _matrix(rng, n, m, chunk, implicit):
    special = [0, 1, 2, 3, 4, 5, 15, 16, 17, 31, 32, 33, 47, 48, 63, 64, 65, 95, 96, 127, 128, 129, chunk - 1, chunk,
               chunk + 1, 2 * chunk, 2 * chunk + 3, n]
    deg = np.where(rng.random(m) < 0.5, rng.choice(special, m), rng.integers(0, min(n, 3 * chunk) + 1, m))
    deg = np.minimum(deg, n).astype(np.int64)
    ptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int64)
    idx = np.concatenate([np.sort(rng.choice(n, d, replace=False)) for d in deg] + [np.zeros(0, np.int64)]).astype(np.int32)
    val = (rng.integers(0, 6, int(ptr[-1])) if implicit else rng.standard_normal(int(ptr[-1])) * 2 + 3).astype(np.float32)
    return deg, ptr, idx, val


@pytest.mark.parametrize("seed", [1, 2, 3, 4])
def test_random_half_sweeps(seed):
    import paper_1808_03843_amd as P
    rng = np.random.default_rng(seed)
    # seeds from 3 on also draw the routes of fp32 factors through 16-bit parts and the switch that sends rows with
    # fewer than 64 entries through get_hermitian (the earlier seeds keep their cases)
    wide_choice = seed >= 3
    for case in range(60):
        f = int(rng.choice([16, 32, 64, 100, 128, 256]))
        solver = int(rng.choice([P.SOLVER_CG, P.SOLVER_CHOLESKY]))
        dt = str(rng.choice(["f32", "f32x3", "f32x2", "bf16", "f16"] if wide_choice else ["f32", "f32", "bf16", "f16"]))
        if dt in ("f32x3", "f32x2") and f == 256:
            dt = "f32"   # those routes exist for f <= 128
        dense_short = bool(wide_choice and rng.random() < 0.3)
        chunk = int(rng.choice([64, 128, 256, 1024, 4096]))
        implicit = dt == "f32" and rng.random() < 0.3
        herm16 = (not implicit) and solver == P.SOLVER_CG and rng.random() < 0.2 and (f != 256 or dt == "f32")
        p64 = bool(rng.random() < 0.3)
        n, m = int(rng.integers(300, 6000)), int(rng.integers(20, 300))
        lam = float(rng.choice([0.05, 0.3, 1.0]))
        # Algorithm 1 is compared row by row while it is still converging, against the same iteration in double
        # precision (with few columns Theta^T Theta is ill-conditioned and no fixed iteration count reaches the exact
        # solution, so the exact oracle cannot be the reference of the implicit CG cases either)
        fs = 6 if implicit else int(rng.choice([3, 6]))
        batch = int(rng.choice([0, 8, 64]))
        deg, ptr, idx, val = _matrix(rng, n, m, chunk, implicit)
        tag = (f"seed {seed} case {case}: f={f} solver={solver} {dt} chunk={chunk} implicit={implicit} bf16 slots={herm16} "
               f"dense_short_rows={dense_short} "
               f"ptr64={p64} n={n} m={m} lambda={lam} f_s={fs} batch_slots={batch} max degree {deg.max()}")
        print(tag, flush=True)
        Theta = W.random_factors(n, f, seed=1000 * seed + case, scale=0.3)
        warm = W.random_factors(m, f, seed=1000 * seed + case + 500, scale=0.05)
        tdt, code = {"f32": (torch.float32, P.F32), "bf16": (torch.bfloat16, P.BF16), "f16": (torch.float16, P.F16),
                     "f32x3": (torch.float32, P.F32X3), "f32x2": (torch.float32, P.F32X2)}[dt]
        Td = torch.from_numpy(Theta).cuda().to(tdt)
        Th = Td.to(torch.float32).cpu().numpy()
        als = P.Als(f, solver=solver, cg_iters=fs, chunk=chunk, batch_slots=batch, factor_dtype=code,
                    herm_dtype=P.BF16 if herm16 else P.F32, dense_short_rows=dense_short)
        sp = P.SparseMatrix.from_host(m, n, ptr, idx, val, ptr64=p64)
        als.check_matrix(sp)
        X = torch.from_numpy(warm.copy()).cuda()
        rows = np.flatnonzero(deg > 0)
        if implicit and solver == P.SOLVER_CHOLESKY:
            als.update_rows_implicit(sp, Td, lam, 2.0, X)
            ref, tol = oracle.implicit_update_rows(ptr, idx, val, Th, lam, 2.0), 1e-4
        elif implicit:
            als.update_rows_implicit(sp, Td, lam, 2.0, X)
            # the definition sums over every column: a sample of rows (shortest, longest, evenly spaced between)
            rows = rows[np.argsort(deg[rows], kind="stable")]
            rows = np.unique(rows[np.linspace(0, len(rows) - 1, min(len(rows), 8)).astype(np.int64)])
            ref, tol = np.zeros((m, f)), 2e-3
            for u in rows:
                A, b = oracle.implicit_normal_eq(idx[ptr[u]:ptr[u + 1]], val[ptr[u]:ptr[u + 1]], Th, lam, 2.0)
                ref[u], _ = oracle.cg(A, warm[u], b, fs)
        else:
            als.update_rows(sp, Td, lam, X)
            if solver == P.SOLVER_CHOLESKY:
                ref, tol = oracle.update_rows(ptr, idx, val, Th, lam), 1e-4
            else:   # bf16 storage of the split rows' A_u: its rounding is the difference
                ref, tol = oracle.update_rows_cg(ptr, idx, val, Th, lam, warm, fs=fs), (5e-2 if herm16 else 2e-3)
        als.synchronize()
        got = X.cpu().numpy()
        als.close()
        assert not got[deg == 0].any(), tag
        err = _rel(got[rows], ref[rows])
        assert err.max() <= tol, (tag, float(err.max()), int(deg[rows][err.argmax()]))


def _tailed_matrix(rng, n, m, mean, chunk):
    """Heavy-tailed degrees (Pareto, as in the rating data sets of Section 5.1: most rows short, a few long), 5 % empty
    rows, and rows planted at the boundaries of the kernels; no duplicate column in a row."""
    deg = np.minimum(np.floor(rng.pareto(1.3, m) * mean * 0.4).astype(np.int64), n)
    deg[rng.random(m) < 0.05] = 0
    planted = [1, 15, 16, 31, 32, 63, 64, 65, 127, 128, 129, 255, 256, chunk - 1, chunk, chunk + 1, 3 * chunk + 2]
    deg[rng.integers(0, m, 40)] = np.minimum(rng.choice(planted, 40), n)
    ptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int64)
    idx = np.empty(int(ptr[-1]), np.int32)
    perm = rng.permutation(n).astype(np.int32)
    for u in np.flatnonzero(deg):   # a window of a fixed permutation of the columns, from a random start
        idx[ptr[u]:ptr[u + 1]] = np.sort(perm[(int(rng.integers(0, n)) + np.arange(deg[u])) % n])
    val = rng.integers(1, 6, int(ptr[-1])).astype(np.float32)
    return deg, ptr, idx, val


@pytest.mark.parametrize("block", [0, 1, 2, 3])
def test_random_half_sweeps_over_thousands_of_rows(block):
    """Thousands of rows with heavy-tailed degrees: many launches' worth of short rows (the packed and the two-wavefront
    routes of Algorithm 1 on gathered rows), several batches of split rows, both entry points of the half-sweep."""
    import paper_1808_03843_amd as P
    for seed in range(10 * block, 10 * block + 10):
        rng = np.random.default_rng(7000 + seed)
        f = int(rng.choice([16, 32, 64, 100, 128, 256]))
        solver = int(rng.choice([P.SOLVER_CG, P.SOLVER_CG, P.SOLVER_CHOLESKY]))
        dt = str(rng.choice(["f32", "f32x3", "f32x2", "bf16", "f16"]))
        if dt in ("f32x3", "f32x2") and f == 256:
            dt = "f32"
        dense_short = bool(rng.random() < 0.2)
        chunk = int(rng.choice([64, 256, 1024, 4096]))
        p64 = bool(rng.random() < 0.3)
        n = int(rng.integers(200, 20000))
        mean = float(rng.choice([3, 10, 30, 80, 200]))
        m = int(min(30000, max(50, (150_000 if f == 256 else 600_000) / mean)))
        deg, ptr, idx, val = _tailed_matrix(rng, n, m, mean, chunk)
        lam, fs = float(rng.choice([0.05, 0.3])), int(rng.choice([3, 6]))
        batch = int(rng.choice([0, 8, 64]))
        cols = bool(rng.random() < 0.5)
        tag = (f"seed {seed}: f={f} solver={solver} {dt} chunk={chunk} dense_short_rows={dense_short} ptr64={p64} n={n} m={m} "
               f"entries={ptr[-1]} lambda={lam} f_s={fs} batch_slots={batch} {'update_cols' if cols else 'update_rows'} "
               f"max degree {deg.max()}")
        print(tag, flush=True)
        Theta = W.random_factors(n, f, seed=seed, scale=0.3)
        warm = W.random_factors(m, f, seed=seed + 500, scale=0.05)
        tdt, code = {"f32": (torch.float32, P.F32), "bf16": (torch.bfloat16, P.BF16), "f16": (torch.float16, P.F16),
                     "f32x3": (torch.float32, P.F32X3), "f32x2": (torch.float32, P.F32X2)}[dt]
        Td = torch.from_numpy(Theta).cuda().to(tdt)
        Th = Td.to(torch.float32).cpu().numpy()
        als = P.Als(f, solver=solver, cg_iters=fs, chunk=chunk, batch_slots=batch, factor_dtype=code, dense_short_rows=dense_short)
        sp = P.SparseMatrix.from_host(m, n, ptr, idx, val, ptr64=p64)
        als.check_matrix(sp)
        X = torch.from_numpy(warm.copy()).cuda()
        (als.update_cols if cols else als.update_rows)(sp, Td, lam, X)   # the same operation under its two names
        als.synchronize()
        got = X.cpu().numpy()
        als.close()
        if solver == P.SOLVER_CHOLESKY:
            ref, tol = oracle.update_rows(ptr, idx, val, Th, lam), 1e-4
        else:
            ref, tol = oracle.update_rows_cg(ptr, idx, val, Th, lam, warm, fs=fs), 2e-3
        live = deg > 0
        assert not got[~live].any(), tag
        err = _rel(got[live], ref[live])
        assert err.max() <= tol, (tag, float(err.max()), int(deg[live][err.argmax()]))


def test_random_side_entry_points():
    import paper_1808_03843_amd as P
    rng = np.random.default_rng(5)
    for case in range(60):
        f = int(rng.choice([16, 32, 64, 100, 128, 256]))
        dt = str(rng.choice(["f32", "bf16", "f16"]))
        chunk = int(rng.choice([64, 128, 1024, 4096]))
        p64 = bool(rng.random() < 0.3)
        n, m = int(rng.integers(50, 3000)), int(rng.integers(1, 200))
        deg, ptr, idx, val = _matrix(rng, n, m, chunk, False)
        val = (val * 10).astype(np.float32)
        tag = f"case {case}: f={f} {dt} chunk={chunk} ptr64={p64} n={n} m={m} max degree {deg.max()}"
        print(tag, flush=True)
        Theta = W.random_factors(n, f, seed=case + 1, scale=0.3)
        Xf = W.random_factors(m, f, seed=case + 77, scale=0.3)
        tdt, code = {"f32": (torch.float32, P.F32), "bf16": (torch.bfloat16, P.BF16), "f16": (torch.float16, P.F16),
                     "f32x3": (torch.float32, P.F32X3), "f32x2": (torch.float32, P.F32X2)}[dt]
        Td = torch.from_numpy(Theta).cuda().to(tdt)
        Th = Td.to(torch.float32).cpu().numpy()
        als = P.Als(f, chunk=chunk, factor_dtype=code)
        sp = P.SparseMatrix.from_host(m, n, ptr, idx, val, ptr64=p64)
        r0 = int(rng.integers(0, m))
        nr = int(rng.integers(1, min(m - r0, 40) + 1))
        A, b = als.hermitian(sp, Td, 0.07, r0, nr)
        A, b = A.cpu().numpy(), b.cpu().numpy()
        for k in range(nr):
            s, e = ptr[r0 + k], ptr[r0 + k + 1]
            Ao, bo = oracle.normal_eq(idx[s:e], val[s:e], Th, 0.07)
            d = np.sqrt(max(1, e - s))
            assert np.abs(A[k] - Ao).max() <= 2e-6 * max(np.abs(Ao).max(), 1e-30) * d, (tag, r0 + k)
            # (fp16 factors: the parts of a rating stop at the spacing 2^-24 of the smallest fp16 numbers)
            floor = 2.0 ** -24 * np.abs(Th[idx[s:e]]).sum(0).max() if dt == "f16" and e > s else 0.0
            assert np.abs(b[k] - bo).max() <= 2e-6 * max(np.abs(bo).max(), 1e-30) * d + floor + 1e-30, (tag, r0 + k)
            assert np.array_equal(A[k], A[k].T), (tag, r0 + k)
        perm, start = als.bin_rows(sp, 12)
        po, so = oracle.bin_rows(ptr, 12)
        assert np.array_equal(perm.cpu().numpy(), po) and list(start) == list(so), tag
        if ptr[-1] > 0:
            ev = P.Als(f, chunk=chunk)
            rg = ev.rmse(sp, torch.from_numpy(Xf).cuda(), torch.from_numpy(Theta).cuda())
            ev.close()
            ro = oracle.rmse(ptr, idx, val, Xf, Theta)
            assert abs(rg - ro) <= 1e-5 * ro, tag
            csc = als.csr_to_csc(sp)
            cptr, cidx, cval = oracle.csr_to_csc(m, n, ptr, idx, val)
            assert np.array_equal(csc.ptr.cpu().numpy(), cptr) and np.array_equal(csc.idx.cpu().numpy(), cidx), tag
            assert np.array_equal(csc.val.cpu().numpy(), cval), tag
        als.synchronize()
        als.close()
