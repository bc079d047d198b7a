"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs."""
import numpy as np
import pytest

import oracle
import workload as W

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def _row_rel_err(x_gpu, x_ref):
    num = np.linalg.norm(x_gpu.astype(np.float64) - x_ref, axis=1)
    den = np.maximum(np.linalg.norm(x_ref, axis=1), 1e-30)
    return num / den


def _edge_matrix(n, f, seed, degrees):
    """Rows with chosen degrees (0 allowed), distinct sorted columns, ratings 0..5 (stored zeros included)."""
    rng = np.random.default_rng(seed)
    ptr = np.concatenate([[0], np.cumsum(degrees)]).astype(np.int64)
    idx = np.concatenate([np.sort(rng.choice(n, d, replace=False)) for d in degrees] + [np.zeros(0, int)])
    val = rng.integers(0, 6, size=int(ptr[-1])).astype(np.float32)
    return W.CSR(len(degrees), n, ptr, idx.astype(np.int32), val)


@pytest.fixture(scope="module")
def P():
    import paper_1808_03843_amd as pkg
    return pkg


# tolerance of the exact fp32 mode (per row, 2-norm relative): 1e-4
TOL_EXACT = 1e-4


@pytest.mark.parametrize("f", [16, 32, 64, 100, 128, 256])
def test_hermitian_and_bias_match_oracle_on_edge_degrees(P, f):
    n = 5000
    degrees = [0, 1, 2, 3, 4, 5, 7, 8, 63, 64, 65, 127, 255, 256, 257, 300, 1023, 1024, 1025, 2048, 2500, 4095, 4096, 4097, 0, 1]
    a = _edge_matrix(n, f, 7, degrees)
    Theta = W.random_factors(n, f, seed=3, scale=0.5)
    lam = 0.05
    als = P.Als(f, chunk=256)          # several work items per long row
    sp = P.SparseMatrix.from_host(a.nrows, a.ncols, a.ptr, a.idx, a.val)
    A, b = als.hermitian(sp, _dev(Theta), lam, 0, a.nrows)
    A, b = A.cpu().numpy(), b.cpu().numpy()
    for u, d in enumerate(degrees):
        s, e = a.ptr[u], a.ptr[u + 1]
        Ao, bo = oracle.normal_eq(a.idx[s:e], a.val[s:e], Theta, lam)
        scale = max(np.abs(Ao).max(), 1e-30)
        assert np.abs(A[u] - Ao).max() <= 2e-6 * scale * max(1, np.sqrt(d)), (u, d)
        assert np.abs(b[u] - bo).max() <= 2e-6 * max(np.abs(bo).max(), 1e-30) * max(1, np.sqrt(d)) + 1e-30, (u, d)
        assert np.array_equal(A[u], A[u].T)
    als.close()


@pytest.mark.parametrize("f", [16, 32, 64, 100, 128])
@pytest.mark.parametrize("name", ["bf16", "f16"])
def test_hermitian_and_bias_on_the_16_bit_matrix_cores(P, f, name):
    """16-bit factor inputs at f <= 128 run on the 16-bit MFMAs, 32 entries per step, with b_u carried as a
    three-part split of the rating: A_u and b_u against the oracle on the same rounded factors, with ratings
    that no 16-bit format holds, and degrees around the step size and the chunk size."""
    n = 5000
    degrees = [0, 1, 2, 7, 8, 9, 15, 16, 17, 31, 32, 33, 63, 64, 65, 95, 96, 97, 255, 256, 257, 300, 1000, 1024, 1025, 2500]
    rng = np.random.default_rng(11)
    ptr = np.concatenate([[0], np.cumsum(degrees)]).astype(np.int64)
    idx = np.concatenate([np.sort(rng.choice(n, d, replace=False)) for d in degrees] + [np.zeros(0, int)]).astype(np.int32)
    val = (rng.standard_normal(int(ptr[-1])) * 37.123).astype(np.float32)
    tdt, code = (torch.bfloat16, P.BF16) if name == "bf16" else (torch.float16, P.F16)
    T16 = torch.from_numpy(W.random_factors(n, f, seed=4, scale=0.5)).cuda().to(tdt)
    T_rounded = T16.to(torch.float32).cpu().numpy()
    als = P.Als(f, chunk=256, factor_dtype=code)
    sp = P.SparseMatrix.from_host(len(degrees), n, ptr, idx, val)
    A, b = als.hermitian(sp, T16, 0.05, 0, len(degrees))
    A, b = A.cpu().numpy(), b.cpu().numpy()
    for u, d in enumerate(degrees):
        s, e = ptr[u], ptr[u + 1]
        Ao, bo = oracle.normal_eq(idx[s:e], val[s:e], T_rounded, 0.05)
        assert np.abs(A[u] - Ao).max() <= 2e-6 * max(np.abs(Ao).max(), 1e-30) * max(1, np.sqrt(d)), (u, d)
        assert np.abs(b[u] - bo).max() <= 2e-6 * max(np.abs(bo).max(), 1e-30) * max(1, np.sqrt(d)) + 1e-30, (u, d)
        assert np.array_equal(A[u], A[u].T)
    als.close()


@pytest.mark.parametrize("f", [100, 128, 256])
@pytest.mark.parametrize("p64,name", [(False, "f32"), (True, "f32"), (False, "bf16"), (True, "f16")])
def test_exact_rows_with_fewer_entries_than_features(P, f, p64, name):
    """The exact solver handles rows with fewer than 32 / 64 / 128 entries in the dual form (an n_u x n_u system).
    Every degree from 0 to 140, so that both sides of every switch and the padding of every size are hit,
    non-integer ratings, against the oracle's f x f solve (on the rounded factors when the input is 16-bit)."""
    n = 3000
    degrees = list(range(0, 141)) + [200, 500]
    rng = np.random.default_rng(21)
    ptr = np.concatenate([[0], np.cumsum(degrees)]).astype(np.int64)
    idx = np.concatenate([np.sort(rng.choice(n, d, replace=False)) for d in degrees] + [np.zeros(0, int)]).astype(np.int32)
    val = (rng.standard_normal(int(ptr[-1])) * 2.5 + 3.0).astype(np.float32)
    Theta = W.random_factors(n, f, seed=31 + f, scale=0.4)
    tdt, code = {"f32": (torch.float32, P.F32), "bf16": (torch.bfloat16, P.BF16), "f16": (torch.float16, P.F16)}[name]
    Td = _dev(Theta).to(tdt)
    Theta = Td.to(torch.float32).cpu().numpy()
    sp = P.SparseMatrix.from_host(len(degrees), n, ptr, idx, val, ptr64=p64)
    als = P.Als(f, solver=P.SOLVER_CHOLESKY, factor_dtype=code)
    X = torch.full((len(degrees), f), 7.0, device="cuda:0")
    als.update_rows(sp, Td, 0.3, X)
    als.synchronize()
    got = X.cpu().numpy()
    ref = oracle.update_rows(ptr, idx, val, Theta, 0.3)
    assert np.all(got[0] == 0.0)
    err = _row_rel_err(got[1:], ref[1:])
    assert err.max() <= TOL_EXACT, (int(err.argmax()) + 1, float(err.max()))
    als.close()


@pytest.mark.parametrize("chunk", [64, 1024])
def test_one_exact_sweep_on_tiny(P, chunk):
    w = W.TINY
    a = W.generate(w)
    c = W.transpose(a)
    X0, T0 = W.init_factors(w)
    als = P.Als(w.f, solver=P.SOLVER_CHOLESKY, chunk=chunk)
    csr = P.SparseMatrix.from_host(a.nrows, a.ncols, a.ptr, a.idx, a.val)
    csc = P.SparseMatrix.from_host(c.nrows, c.ncols, c.ptr, c.idx, c.val)
    X, T = _dev(X0), _dev(T0)
    als.update_rows(csr, T, w.lam, X)
    als.update_cols(csc, X, w.lam, T)
    als.synchronize()
    Xo = oracle.update_rows(a.ptr, a.idx, a.val, T0, w.lam)
    To = oracle.update_rows(c.ptr, c.idx, c.val, Xo, w.lam)
    ex, et = _row_rel_err(X.cpu().numpy(), Xo), _row_rel_err(T.cpu().numpy(), To)
    print(f"tiny one sweep: max row rel err X {ex.max():.2e} Theta {et.max():.2e}")
    assert ex.max() <= TOL_EXACT and et.max() <= TOL_EXACT
    # RMSE through the library against the oracle's on the same (GPU-independent) factors
    r_gpu = als.rmse(csr, _dev(Xo.astype(np.float32)), _dev(To.astype(np.float32)))
    r_orc = oracle.rmse(a.ptr, a.idx, a.val, Xo.astype(np.float32), To.astype(np.float32))
    assert abs(r_gpu - r_orc) <= 1e-5 * max(r_orc, 1e-30)
    als.close()


def test_exact_sweeps_follow_oracle_trajectory_on_tiny(P):
    w = W.TINY
    a = W.generate(w)
    c = W.transpose(a)
    X0, T0 = W.init_factors(w)
    _, _, hist = oracle.als((a.ptr, a.idx, a.val), (c.ptr, c.idx, c.val), X0, T0, w.lam, w.sweeps)
    als = P.Als(w.f)
    csr = P.SparseMatrix.from_host(a.nrows, a.ncols, a.ptr, a.idx, a.val)
    csc = P.SparseMatrix.from_host(c.nrows, c.ncols, c.ptr, c.idx, c.val)
    X, T = _dev(X0), _dev(T0)
    for s in range(w.sweeps):
        als.update_rows(csr, T, w.lam, X)
        als.update_cols(csc, X, w.lam, T)
        assert abs(als.rmse(csr, X, T) - hist[s]["rmse"]) <= 2e-4
    als.synchronize()
    als.close()


def test_one_exact_sweep_f100_several_tiles_ragged_tails(P):
    w = W.MID_SMALL
    a = W.generate(w)
    c = W.transpose(a)
    X0, T0 = W.init_factors(w)
    als = P.Als(w.f, solver=P.SOLVER_CHOLESKY, chunk=512, batch_slots=4096)   # several batches, split rows
    csr = P.SparseMatrix.from_host(a.nrows, a.ncols, a.ptr, a.idx, a.val)
    csc = P.SparseMatrix.from_host(c.nrows, c.ncols, c.ptr, c.idx, c.val)
    X, T = _dev(X0), _dev(T0)
    als.update_rows(csr, T, w.lam, X)
    als.update_cols(csc, X, w.lam, T)
    als.synchronize()
    Xo = oracle.update_rows(a.ptr, a.idx, a.val, T0, w.lam)
    To = oracle.update_rows(c.ptr, c.idx, c.val, Xo, w.lam)
    ex, et = _row_rel_err(X.cpu().numpy(), Xo), _row_rel_err(T.cpu().numpy(), To)
    print(f"mid_small one sweep: X max {ex.max():.2e} p99.9 {np.quantile(ex, 0.999):.2e}; "
          f"Theta max {et.max():.2e} p99.9 {np.quantile(et, 0.999):.2e}")
    assert ex.max() <= TOL_EXACT and et.max() <= TOL_EXACT
    fro = np.linalg.norm(X.cpu().numpy() - Xo) / np.linalg.norm(Xo)
    assert fro <= TOL_EXACT
    als.close()


def test_cg_update_matches_double_precision_algorithm_1(P):
    # same Algorithm 1, same warm start, same f_s: only fp32 rounding separates the two
    w = W.MID_SMALL
    a = W.generate(w)
    _, T0 = W.init_factors(w)
    Xw = W.random_factors(w.m, w.f, seed=5, scale=0.1)
    als = P.Als(w.f, solver=P.SOLVER_CG, cg_iters=6, chunk=512)
    csr = P.SparseMatrix.from_host(a.nrows, a.ncols, a.ptr, a.idx, a.val)
    X = _dev(Xw.copy())
    als.update_rows(csr, _dev(T0), w.lam, X)
    als.synchronize()
    Xo = oracle.update_rows_cg(a.ptr, a.idx, a.val, T0, w.lam, Xw, fs=6)
    err = _row_rel_err(X.cpu().numpy(), Xo)
    print(f"cg(6) vs double Algorithm 1: max {err.max():.2e}")
    assert err.max() <= 2e-3
    als.close()


def test_cg_ten_sweeps_rmse_within_tolerance_of_exact_oracle(P):
    w = W.MID_SMALL
    a = W.generate(w)
    c = W.transpose(a)
    X0, T0 = W.init_factors(w)
    _, _, hist = oracle.als((a.ptr, a.idx, a.val), (c.ptr, c.idx, c.val), X0, T0, w.lam, w.sweeps)
    als = P.Als(w.f, solver=P.SOLVER_CG, cg_iters=6)
    csr = P.SparseMatrix.from_host(a.nrows, a.ncols, a.ptr, a.idx, a.val)
    csc = P.SparseMatrix.from_host(c.nrows, c.ncols, c.ptr, c.idx, c.val)
    X, T = _dev(X0), _dev(T0)
    for _ in range(w.sweeps):
        als.update_rows(csr, T, w.lam, X)
        als.update_cols(csc, X, w.lam, T)
    r = als.rmse(csr, X, T)
    als.synchronize()
    print(f"cg(6) 10 sweeps rmse {r:.5f} vs exact oracle {hist[-1]['rmse']:.5f}")
    assert abs(r - hist[-1]["rmse"]) <= 2e-3
    als.close()


def test_empty_rows_stored_zeros_and_int64_pointers(P):
    f, n = 32, 300
    degrees = [0, 0, 5, 1, 0, 40, 300, 0]
    a = _edge_matrix(n, f, 11, degrees)
    Theta = W.random_factors(n, f, seed=4, scale=0.4)
    Xo = oracle.update_rows(a.ptr, a.idx, a.val, Theta, 0.1)
    for ptr64 in (False, True):
        als = P.Als(f)
        sp = P.SparseMatrix.from_host(a.nrows, a.ncols, a.ptr, a.idx, a.val, ptr64=ptr64)
        X = torch.full((a.nrows, f), 7.0, device="cuda:0")
        als.update_rows(sp, _dev(Theta), 0.1, X)
        als.synchronize()
        Xg = X.cpu().numpy()
        assert not Xg[[0, 1, 4, 7]].any()
        live = [2, 3, 5, 6]
        assert _row_rel_err(Xg[live], Xo[live]).max() <= TOL_EXACT
        als.close()


def test_index_work_is_bit_exact(P):
    for w in (W.TINY, W.SQUARE_SMALL):
        a = W.generate(w)
        als = P.Als(w.f)
        for ptr64 in (False, True):
            sp = P.SparseMatrix.from_host(a.nrows, a.ncols, a.ptr, a.idx, a.val, ptr64=ptr64)
            perm, start = als.bin_rows(sp, 12)
            perm_o, start_o = oracle.bin_rows(a.ptr, 12)
            assert np.array_equal(perm.cpu().numpy(), perm_o) and list(start_o) == start
            t = als.csr_to_csc(sp)
            cptr, cidx, cval = oracle.csr_to_csc(w.m, w.n, a.ptr, a.idx, a.val)
            assert np.array_equal(t.ptr.cpu().numpy(), cptr)
            assert np.array_equal(t.idx.cpu().numpy(), cidx)
            assert np.array_equal(t.val.cpu().numpy(), cval)
        als.close()


@pytest.mark.parametrize("ncols", [1, 2, 2048, 2049, 70_000, 5_000_000, 40_000_000])
def test_csr_to_csc_over_the_digit_widths_of_the_column_ids(P, ncols):
    """The transpose is a radix sort of the column ids in one to three passes of up to 11 bits: column counts on both
    sides of the 11-bit and 22-bit boundaries, heavy columns (every row hits column 0), empty rows, ties that must
    keep their row order, against the oracle's transpose bit for bit."""
    rng = np.random.default_rng(ncols % 1000 + 5)
    m = 3000
    deg = rng.integers(0, min(ncols, 40) + 1, m)
    deg[rng.random(m) < 0.1] = 0
    rows = []
    for d in deg:
        c = rng.choice(ncols, d, replace=False) if ncols <= 100_000 else np.unique(rng.integers(0, ncols, d))
        if d > 0 and rng.random() < 0.7:
            c = np.unique(np.concatenate([[0, ncols - 1], c]))   # two columns that most rows share
        rows.append(np.sort(c))
    ptr = np.concatenate([[0], np.cumsum([len(r) for r in rows])]).astype(np.int64)
    idx = np.concatenate(rows + [np.zeros(0, np.int64)]).astype(np.int32)
    val = rng.standard_normal(len(idx)).astype(np.float32)
    als = P.Als(16)
    for ptr64 in (False, True):
        sp = P.SparseMatrix.from_host(m, ncols, ptr, idx, val, ptr64=ptr64)
        t = als.csr_to_csc(sp)
        cptr, cidx, cval = oracle.csr_to_csc(m, ncols, ptr, idx, val)
        assert np.array_equal(t.ptr.cpu().numpy(), cptr)
        assert np.array_equal(t.idx.cpu().numpy(), cidx)
        assert np.array_equal(t.val.cpu().numpy(), cval)
    als.close()


def test_bad_arguments_are_errors_not_crashes(P):
    with pytest.raises(P.AlsError):
        P.Als(17)
    als = P.Als(16)
    a = W.generate(W.TINY)
    sp = P.SparseMatrix.from_host(a.nrows, a.ncols, a.ptr, a.idx, a.val)
    T = torch.zeros((a.ncols, 16), device="cuda:0")
    X = torch.zeros((a.nrows, 16), device="cuda:0")
    with pytest.raises(P.AlsError):
        als.update_rows(sp, T, -1.0, X)
    with pytest.raises(P.AlsError, match="aligned"):   # a view that starts 4 bytes into an allocation
        buf = torch.zeros(a.ncols * 16 + 1, device="cuda:0")
        als._check(als._lib.als_update_rows(als._ctx, __import__("ctypes").byref(sp.desc), buf.data_ptr() + 4, 0.1, 16,
                                            X.data_ptr()))
    # lambda = 0 and a rank-deficient row: the exact solver must flag it, not hang or crash
    als.update_rows(sp, T, 0.0, X)
    with pytest.raises(P.AlsError) as ei:
        als.synchronize()
    assert ei.value.code == -3
    als.close()


@pytest.mark.parametrize("f,n", [(16, 67_200_000), (32, 33_600_000), (64, 16_800_000), (100, 10_800_000),
                                 (128, 8_400_000), (256, 4_200_000)])
def test_factor_matrix_beyond_4_gib_uses_64_bit_offsets(P, f, n):
    """A gathered factor matrix of 4 GiB or more switches the gathers to 64-bit row addresses (another
    template instantiation of every get_hermitian kernel, and of the Gram kernel in implicit mode).  The
    matrix is zero except for the rows the test touches; the oracle sees a compact copy."""
    assert n * f * 4 >= 2 ** 32
    rng = np.random.default_rng(5)
    degrees = [1, 3, 40, 700, 2000]
    ptr = np.concatenate([[0], np.cumsum(degrees)]).astype(np.int64)
    # ids spread over the whole matrix, the last row included
    idx = np.concatenate([np.sort(np.unique(np.concatenate([rng.choice(n, d, replace=False)[: d - 1], [n - 1]]))[:d])
                          for d in degrees]).astype(np.int32)
    assert len(idx) == ptr[-1]
    val = rng.integers(1, 6, size=int(ptr[-1])).astype(np.float32)
    used = np.unique(idx)
    rows_val = W.random_factors(len(used), f, seed=8, scale=0.5)
    Theta = torch.zeros((n, f), device="cuda:0")
    Theta[torch.from_numpy(used.astype(np.int64)).cuda()] = torch.from_numpy(rows_val).cuda()
    # the oracle sees a compact copy: column ids renumbered to the used rows
    remap = np.searchsorted(used, idx).astype(np.int32)
    sp = P.SparseMatrix.from_host(len(degrees), n, ptr, idx, val)
    for solver in (P.SOLVER_CHOLESKY, P.SOLVER_CG):
        als = P.Als(f, solver=solver, cg_iters=f, chunk=256)
        X = torch.zeros((len(degrees), f), device="cuda:0")
        # lambda = 0.5: the row with one entry has cond(A_u) = (|theta|^2 + lambda) / lambda, and fp32 cannot
        # hold 1e-4 at f = 256 with a smaller lambda
        als.update_rows(sp, Theta, 0.5, X)
        als.synchronize()
        ref = oracle.update_rows(ptr, remap, val, rows_val, 0.5)
        assert _row_rel_err(X.cpu().numpy(), ref).max() <= TOL_EXACT
        als.close()
    # implicit mode: the zero rows add nothing to Theta^T Theta, so the compact problem is the same problem
    als = P.Als(f, solver=P.SOLVER_CHOLESKY, chunk=256)
    X = torch.zeros((len(degrees), f), device="cuda:0")
    als.update_rows_implicit(sp, Theta, 0.4, 2.0, X)
    als.synchronize()
    ref = oracle.implicit_update_rows(ptr, remap, val, rows_val, 0.4, 2.0)
    assert _row_rel_err(X.cpu().numpy(), ref).max() <= TOL_EXACT
    als.close()
    del Theta
    torch.cuda.empty_cache()


@pytest.mark.parametrize("f,n", [(100, 17_000_000), (128, 16_800_000), (256, 8_400_000)])
def test_16_bit_factor_with_64_bit_row_addresses(P, f, n):
    """16-bit factor inputs whose rows need 64-bit addresses.  f = 100: the row pitch (200 bytes) is not a power
    of two and the 32-bit row offsets are formed with a 24-bit multiply, so a matrix of 2^24 rows or more (still
    below 4 GiB) must take the 64-bit path; f = 128, 256: 4 GiB or more.  Zero matrix except for the touched rows;
    the oracle sees a compact copy."""
    assert n >= 2 ** 24 or n * f * 2 >= 2 ** 32
    rng = np.random.default_rng(6)
    degrees = [2, 50, 900]
    ptr = np.concatenate([[0], np.cumsum(degrees)]).astype(np.int64)
    lo = n - 300_000   # every touched row lies beyond the 32-bit / 24-bit limit
    idx = np.concatenate([np.sort(np.unique(np.concatenate([rng.choice(n - lo - 1, d - 1, replace=False) + lo,
                                                            [n - 1]]))[:d]) for d in degrees]).astype(np.int32)
    assert len(idx) == ptr[-1] and idx.max() == n - 1
    val = rng.integers(1, 6, size=int(ptr[-1])).astype(np.float32)
    used = np.unique(idx)
    rows16 = torch.from_numpy(W.random_factors(len(used), f, seed=9, scale=0.5)).to(torch.bfloat16)
    Theta = torch.zeros((n, f), device="cuda:0", dtype=torch.bfloat16)
    Theta[torch.from_numpy(used.astype(np.int64)).cuda()] = rows16.cuda()
    remap = np.searchsorted(used, idx).astype(np.int32)
    sp = P.SparseMatrix.from_host(len(degrees), n, ptr, idx, val)
    ref = oracle.update_rows(ptr, remap, val, rows16.to(torch.float32).numpy(), 0.5)
    # (f iterations of Algorithm 1: exact up to fp32 rounding)
    for solver, tol in ((P.SOLVER_CG, 1e-3), (P.SOLVER_CHOLESKY, TOL_EXACT)):
        als = P.Als(f, solver=solver, cg_iters=f, chunk=256, factor_dtype=P.BF16)
        X = torch.zeros((len(degrees), f), device="cuda:0")
        als.update_rows(sp, Theta, 0.5, X)
        als.synchronize()
        assert _row_rel_err(X.cpu().numpy(), ref).max() <= tol, solver
        als.close()
    del Theta
    torch.cuda.empty_cache()


@pytest.mark.parametrize("name", ["bf16", "f16"])
def test_reduced_precision_factor_inputs(P, name):
    """16-bit factor inputs, fp32 accumulate: same arithmetic as fp32 on the rounded values, and the
    10-sweep training RMSE stays within the approximate-mode tolerance of the exact oracle."""
    tdt, code = (torch.bfloat16, P.BF16) if name == "bf16" else (torch.float16, P.F16)
    w = W.MID_SMALL
    a = W.generate(w)
    c = W.transpose(a)
    X0, T0 = W.init_factors(w)
    csr = P.SparseMatrix.from_host(a.nrows, a.ncols, a.ptr, a.idx, a.val)
    csc = P.SparseMatrix.from_host(c.nrows, c.ncols, c.ptr, c.idx, c.val)
    # (1) get_hermitian on rounded inputs against the oracle fed the same rounded values
    T16 = _dev(T0).to(tdt)
    T_rounded = T16.to(torch.float32).cpu().numpy()
    als = P.Als(w.f, solver=P.SOLVER_CHOLESKY, chunk=256, factor_dtype=code)
    rows = [0, 1, 17, 500, 11999]
    for u in rows:
        A, b = als.hermitian(csr, T16, w.lam, u, 1)
        s, e = a.ptr[u], a.ptr[u + 1]
        Ao, bo = oracle.normal_eq(a.idx[s:e], a.val[s:e], T_rounded, w.lam)
        d = e - s
        assert np.abs(A[0].cpu().numpy() - Ao).max() <= 2e-6 * np.abs(Ao).max() * max(1, np.sqrt(d))
        assert np.abs(b[0].cpu().numpy() - bo).max() <= 2e-6 * np.abs(bo).max() * max(1, np.sqrt(d))
    # exact solve from the rounded Theta: per-row 1e-4 against the oracle on the same rounded values
    X = _dev(X0)
    als.update_rows(csr, T16, w.lam, X)
    als.synchronize()
    Xo = oracle.update_rows(a.ptr, a.idx, a.val, T_rounded, w.lam)
    assert _row_rel_err(X.cpu().numpy(), Xo).max() <= TOL_EXACT
    als.close()
    # (2) approximate mode end to end: CG(6), 16-bit gathers, 10 sweeps
    _, _, hist = oracle.als((a.ptr, a.idx, a.val), (c.ptr, c.idx, c.val), X0, T0, w.lam, w.sweeps)
    als = P.Als(w.f, solver=P.SOLVER_CG, cg_iters=6, factor_dtype=code)
    X, T = _dev(X0), _dev(T0)
    for _ in range(w.sweeps):
        als.update_rows(csr, T.to(tdt), w.lam, X)
        als.update_cols(csc, X.to(tdt), w.lam, T)
    als.synchronize()
    r = P.Als(w.f).rmse(csr, X, T)
    print(f"{name} inputs, CG(6), 10 sweeps: rmse {r:.5f} vs exact oracle {hist[-1]['rmse']:.5f}")
    assert abs(r - hist[-1]["rmse"]) <= 2e-3
    als.close()


def test_reduced_precision_storage_of_split_rows(P):
    """Section 4.2: A_u stored in 16 bits where it is materialised (here: the partial Gram matrices of
    split rows, bf16).  Approximate mode only; judged by the 10-sweep RMSE against the exact oracle."""
    w = W.MID_SMALL
    a = W.generate(w)
    c = W.transpose(a)
    X0, T0 = W.init_factors(w)
    csr = P.SparseMatrix.from_host(a.nrows, a.ncols, a.ptr, a.idx, a.val)
    csc = P.SparseMatrix.from_host(c.nrows, c.ncols, c.ptr, c.idx, c.val)
    with pytest.raises(P.AlsError):
        P.Als(w.f, solver=P.SOLVER_CHOLESKY, herm_dtype=P.BF16)     # exact mode keeps fp32
    _, _, hist = oracle.als((a.ptr, a.idx, a.val), (c.ptr, c.idx, c.val), X0, T0, w.lam, w.sweeps)
    # chunk 64: every row of this workload is split, so every A_u goes through bf16 slots
    als = P.Als(w.f, solver=P.SOLVER_CG, cg_iters=6, chunk=64, herm_dtype=P.BF16)
    ref = P.Als(w.f, solver=P.SOLVER_CG, cg_iters=6, chunk=64)
    X, T = _dev(X0), _dev(T0)
    X32 = _dev(X0)
    als.update_rows(csr, T, w.lam, X)
    ref.update_rows(csr, T, w.lam, X32)
    dev = _row_rel_err(X.cpu().numpy(), X32.cpu().numpy().astype(np.float64))
    print(f"bf16 slot storage: first half-sweep deviates from fp32 storage by max {dev.max():.2e} per row")
    assert 0 < dev.max() <= 5e-2
    als.update_cols(csc, X, w.lam, T)
    for _ in range(w.sweeps - 1):
        als.update_rows(csr, T, w.lam, X)
        als.update_cols(csc, X, w.lam, T)
    als.synchronize()
    r = ref.rmse(csr, X, T)
    print(f"bf16 slot storage, CG(6), 10 sweeps: rmse {r:.5f} vs exact oracle {hist[-1]['rmse']:.5f}")
    assert abs(r - hist[-1]["rmse"]) <= 2e-3
    als.close()
    ref.close()


@pytest.mark.parametrize("f", [32, 64, 128, 256])
def test_factor_width_sweep_exact_and_cg(P, f):
    """The factor-width sweep on a reduced shape: one exact sweep per row 1e-4, CG(4/6/8) against the same
    Algorithm 1 in double, and the 10-sweep CG(6) training RMSE against the exact oracle."""
    w = W.Workload(f"width_{f}", 3_000, 1_200, 240_000, f, 0.05, 1.0, 1, 1_100, 1.0, 20, seed=40 + f, sweeps=10)
    a = W.generate(w)
    c = W.transpose(a)
    X0, T0 = W.init_factors(w)
    csr = P.SparseMatrix.from_host(a.nrows, a.ncols, a.ptr, a.idx, a.val)
    csc = P.SparseMatrix.from_host(c.nrows, c.ncols, c.ptr, c.idx, c.val)
    als = P.Als(f, solver=P.SOLVER_CHOLESKY, chunk=256)
    X, T = _dev(X0), _dev(T0)
    als.update_rows(csr, T, w.lam, X)
    als.update_cols(csc, X, w.lam, T)
    als.synchronize()
    Xo = oracle.update_rows(a.ptr, a.idx, a.val, T0, w.lam)
    To = oracle.update_rows(c.ptr, c.idx, c.val, Xo, w.lam)
    ex, et = _row_rel_err(X.cpu().numpy(), Xo), _row_rel_err(T.cpu().numpy(), To)
    print(f"f={f} exact sweep: X max {ex.max():.2e} Theta max {et.max():.2e}")
    assert ex.max() <= TOL_EXACT and et.max() <= TOL_EXACT
    als.close()
    warm = W.random_factors(w.m, f, seed=6, scale=0.1)
    for fs in (4, 6, 8):
        als = P.Als(f, solver=P.SOLVER_CG, cg_iters=fs, chunk=256)
        Xc = _dev(warm.copy())
        als.update_rows(csr, _dev(T0), w.lam, Xc)
        als.synchronize()
        ref = oracle.update_rows_cg(a.ptr, a.idx, a.val, T0, w.lam, warm, fs=fs)
        assert _row_rel_err(Xc.cpu().numpy(), ref).max() <= 2e-3
        als.close()
    _, _, hist = oracle.als((a.ptr, a.idx, a.val), (c.ptr, c.idx, c.val), X0, T0, w.lam, w.sweeps)
    als = P.Als(f, solver=P.SOLVER_CG, cg_iters=6)
    X, T = _dev(X0), _dev(T0)
    for _ in range(w.sweeps):
        als.update_rows(csr, T, w.lam, X)
        als.update_cols(csc, X, w.lam, T)
    r = als.rmse(csr, X, T)
    als.synchronize()
    print(f"f={f} CG(6) 10 sweeps: rmse {r:.5f} vs exact oracle {hist[-1]['rmse']:.5f}")
    assert abs(r - hist[-1]["rmse"]) <= 2e-3
    als.close()


def test_held_out_rmse_follows_the_oracle(P):
    """Protocol of Section 5.2: fit on the training entries, RMSE on held-out entries (a second CSR into
    als_rmse).  Exact mode must follow the oracle's held-out RMSE sweep by sweep."""
    w = W.TINY
    a = W.generate(w)
    train, test = W.split(a, 0.1, seed=5)
    ct = W.transpose(train)
    X0, T0 = W.init_factors(w)
    Xo, To = X0.astype(np.float64), T0.astype(np.float64)
    als = P.Als(w.f, solver=P.SOLVER_CHOLESKY)
    tr = P.SparseMatrix.from_host(train.nrows, train.ncols, train.ptr, train.idx, train.val)
    trc = P.SparseMatrix.from_host(ct.nrows, ct.ncols, ct.ptr, ct.idx, ct.val)
    te = P.SparseMatrix.from_host(test.nrows, test.ncols, test.ptr, test.idx, test.val)
    X, T = _dev(X0.copy()), _dev(T0.copy())
    for sweep in range(4):
        Xo = oracle.update_rows(train.ptr, train.idx, train.val, To, w.lam)
        To = oracle.update_rows(ct.ptr, ct.idx, ct.val, Xo, w.lam)
        als.update_rows(tr, T, w.lam, X)
        als.update_cols(trc, X, w.lam, T)
        r_gpu = als.rmse(te, X, T)
        r_orc = oracle.rmse(test.ptr, test.idx, test.val, Xo, To)
        print(f"held-out rmse sweep {sweep + 1}: gpu {r_gpu:.6f} oracle {r_orc:.6f}", flush=True)
        assert abs(r_gpu - r_orc) <= 1e-4 * r_orc
    als.close()


@pytest.mark.parametrize("f,m", [(16, (1 << 25) + 777), (256, (1 << 22) + 300)])
def test_more_rows_than_one_launch_holds(P, f, m):
    """A launch holds fewer than 2^32 threads, so more than 2^31 / 64 rows (2^31 / 512 at f = 256) go out in
    several launches: one entry per row, sampled rows from both ends and the middle against the oracle, and the
    RMSE over all work items against the closed form of the same factors."""
    n = 1000
    rng = np.random.default_rng(77)
    ptr = np.arange(m + 1, dtype=np.int32)
    idx = rng.integers(0, n, size=m, dtype=np.int32)
    val = rng.integers(1, 6, size=m).astype(np.float32)
    Theta = W.random_factors(n, f, seed=5, scale=0.5)
    sp = P.SparseMatrix.from_host(m, n, ptr, idx, val)
    als = P.Als(f, solver=P.SOLVER_CHOLESKY)
    X = torch.full((m, f), 7.0, device="cuda:0")
    Td = _dev(Theta)
    als.update_rows(sp, Td, 0.1, X)
    als.synchronize()
    rows = np.unique(np.concatenate([np.arange(0, 300), np.arange(m - 300, m), rng.integers(0, m, 2000)]))
    got = X[torch.from_numpy(rows).cuda()].cpu().numpy()
    sub_ptr = np.arange(len(rows) + 1, dtype=np.int64)
    ref = oracle.update_rows(sub_ptr, idx[rows], val[rows], Theta, 0.1)
    err = _row_rel_err(got, ref)
    assert err.max() <= TOL_EXACT, (int(rows[err.argmax()]), float(err.max()))
    assert bool((X != 7.0).any(dim=1).all())          # every row was written
    # with one entry per row the residual is r * lam / (|theta|^2 + lam): the RMSE in closed form, in double
    t2 = (Theta.astype(np.float64) ** 2).sum(axis=1)[idx]
    want = np.sqrt(np.mean((val.astype(np.float64) * 0.1 / (t2 + 0.1)) ** 2))
    r = als.rmse(sp, X, Td)
    als.close()
    print(f"f={f} m={m}: max row err {err.max():.2e}; rmse {r:.8f} closed form {want:.8f}", flush=True)
    assert abs(r - want) <= 1e-4 * want


def test_plans_are_dropped_when_a_matrix_changes_in_place(P):
    """The plan of a matrix is keyed on its address and sizes: after its arrays are overwritten by another matrix
    of the same nrows and nnz (other degrees: short rows become long and the other way round), als_drop_plans
    makes the next call build a new plan, and the result is that of the new matrix.  Without it the call is flagged."""
    f, n, m = 100, 3000, 600
    rng = np.random.default_rng(8)
    Theta = W.random_factors(n, f, seed=3, scale=0.4)

    def matrix(degrees, seed):
        r = np.random.default_rng(seed)
        ptr = np.concatenate([[0], np.cumsum(degrees)]).astype(np.int32)
        idx = np.concatenate([np.sort(r.choice(n, d, replace=False)) for d in degrees]).astype(np.int32)
        val = r.integers(1, 6, size=int(ptr[-1])).astype(np.float32)
        return ptr, idx, val

    deg_a = rng.integers(1, 200, size=m)
    deg_a[:5] = 2500                                  # rows that go through slots with chunk 256
    deg_b = deg_a[::-1].copy()                        # same sum, other rows are the long ones
    pa, ia, va = matrix(deg_a, 1)
    pb, ib, vb = matrix(deg_b, 2)
    assert pa[-1] == pb[-1]
    for solver, tol in ((P.SOLVER_CG, 2e-3), (P.SOLVER_CHOLESKY, TOL_EXACT)):
        als = P.Als(f, solver=solver, cg_iters=f, chunk=256)   # f iterations from zero: the exact solution up to fp32 rounding
        sp = P.SparseMatrix.from_host(m, n, pa, ia, va)
        X = torch.zeros((m, f), device="cuda:0")
        Td = _dev(Theta)
        als.update_rows(sp, Td, 0.2, X)
        als.synchronize()
        assert _row_rel_err(X.cpu().numpy(), oracle.update_rows(pa.astype(np.int64), ia, va, Theta, 0.2)).max() <= tol
        sp.ptr.copy_(torch.from_numpy(pb))            # the same device arrays now hold matrix b
        sp.idx.copy_(torch.from_numpy(ib))
        sp.val.copy_(torch.from_numpy(vb))
        als.update_rows(sp, Td, 0.2, X)               # stale plan: the fingerprint of ptr no longer matches
        with pytest.raises(P.AlsError, match="als_drop_plans"):
            als.synchronize()
        als.drop_plans()
        X.zero_()
        als.update_rows(sp, Td, 0.2, X)
        als.synchronize()
        err = _row_rel_err(X.cpu().numpy(), oracle.update_rows(pb.astype(np.int64), ib, vb, Theta, 0.2))
        als.close()
        assert err.max() <= tol, float(err.max())


def test_binding_tells_apart_matrices_at_a_reused_address(P):
    """torch's allocator hands the memory of a freed matrix to the next one of the same size; the binding notices
    (every SparseMatrix has a serial number) and drops the plans, so the second matrix gets its own."""
    f, n, m = 32, 500, 400
    Theta = W.random_factors(n, f, seed=3, scale=0.4)
    als = P.Als(f, solver=P.SOLVER_CHOLESKY, chunk=64)
    Td = _dev(Theta)
    X = torch.zeros((m, f), device="cuda:0")
    addresses = set()
    for seed in (1, 2, 3):
        r = np.random.default_rng(seed)
        deg = r.permutation(np.concatenate([np.full(10, 300), np.full(m - 10, 5)]))   # same sizes, other long rows
        ptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int32)
        idx = np.concatenate([np.sort(r.choice(n, d, replace=False)) for d in deg]).astype(np.int32)
        val = r.integers(1, 6, size=int(ptr[-1])).astype(np.float32)
        sp = P.SparseMatrix.from_host(m, n, ptr, idx, val)
        addresses.add(sp.ptr.data_ptr())
        als.update_rows(sp, Td, 0.2, X)
        als.synchronize()
        err = _row_rel_err(X.cpu().numpy(), oracle.update_rows(ptr.astype(np.int64), idx, val, Theta, 0.2))
        assert err.max() <= TOL_EXACT, (seed, float(err.max()))
        del sp
    als.close()
    print(f"distinct ptr addresses over three matrices: {len(addresses)}", flush=True)


@pytest.mark.parametrize("f", [16, 100, 256])
def test_matrix_without_entries_and_without_rows(P, f):
    """Degenerate inputs: no stored entry at all (every x_u = 0, RMSE 0 by convention), and no rows."""
    n, m = 50, 7
    Theta = W.random_factors(n, f, seed=4, scale=0.4)
    Td = _dev(Theta)
    for solver in (P.SOLVER_CG, P.SOLVER_CHOLESKY):
        als = P.Als(f, solver=solver)
        sp = P.SparseMatrix.from_host(m, n, np.zeros(m + 1, np.int32), np.zeros(0, np.int32), np.zeros(0, np.float32))
        X = torch.full((m, f), 7.0, device="cuda:0")
        als.update_rows(sp, Td, 0.1, X)
        als.synchronize()
        assert not X.cpu().numpy().any()
        X.fill_(7.0)
        als.update_rows_implicit(sp, Td, 0.1, 2.0, X)     # b_u = 0: x_u = 0 as well
        als.synchronize()
        assert not X.cpu().numpy().any()
        assert als.rmse(sp, X, Td) == 0.0
        csc = als.csr_to_csc(sp)                          # its transpose: n empty rows
        assert csc.nrows == n and csc.nnz == 0 and not csc.ptr.cpu().numpy().any()
        als.check_matrix(sp)
        none = P.SparseMatrix.from_host(0, n, np.zeros(1, np.int32), np.zeros(0, np.int32), np.zeros(0, np.float32))
        als.update_rows(none, Td, 0.1, torch.zeros((0, f), device="cuda:0"))
        als.synchronize()
        als.close()


def test_check_matrix_finds_what_the_updates_assume(P):
    """als_check_matrix: a generated matrix passes (int32 and int64 offsets, empty rows); an id out of range, ids out
    of order or repeated inside a row, and broken offsets are named."""
    w = W.TINY
    a = W.generate(w)
    als = P.Als(w.f)
    for p64 in (False, True):
        als.check_matrix(P.SparseMatrix.from_host(a.nrows, a.ncols, a.ptr, a.idx, a.val, ptr64=p64))
    ptr = np.array([0, 0, 3, 3, 5, 5], np.int32)             # empty rows at both ends and in the middle
    idx = np.array([1, 4, 9, 0, 9], np.int32)                # a descent only across the row boundary
    val = np.ones(5, np.float32)
    als.check_matrix(P.SparseMatrix.from_host(5, 10, ptr, idx, val))
    cases = [
        (ptr, np.array([1, 4, 10, 0, 9], np.int32), "outside"),
        (ptr, np.array([1, 4, -1, 0, 9], np.int32), "outside"),
        (ptr, np.array([4, 1, 9, 0, 9], np.int32), "ascending"),
        (ptr, np.array([1, 4, 4, 0, 9], np.int32), "ascending"),
        (np.array([0, 0, 3, 2, 5, 5], np.int32), idx, "offsets"),
        (np.array([0, 0, 3, 3, 4, 4], np.int32), idx, "offsets"),
        (np.array([1, 1, 3, 3, 5, 5], np.int32), idx, "offsets"),
    ]
    for bad_ptr, bad_idx, word in cases:
        sp = P.SparseMatrix(5, 10, _dev(bad_ptr), _dev(bad_idx), _dev(val))
        with pytest.raises(P.AlsError, match=word):
            als.check_matrix(sp)
    als.close()


def test_measured_peaks_are_plausible(P):
    """als_measure_peak: what the box sustains lies below the published peaks and within a factor of them."""
    als = P.Als(16)
    f32, bf16, f16, cp = (als.measure_peak(k) for k in (P.PEAK_MFMA_F32, P.PEAK_MFMA_BF16, P.PEAK_MFMA_F16, P.PEAK_COPY))
    als.close()
    print(f"sustained: fp32 MFMA {f32 / 1e12:.1f}, bf16 {bf16 / 1e12:.0f}, fp16 {f16 / 1e12:.0f} TFLOP/s; copy {cp / 1e9:.0f} GB/s",
          flush=True)
    assert 0.3 * 157.3e12 < f32 <= 1.02 * 157.3e12
    assert 0.2 * 2.5e15 < bf16 <= 1.02 * 2.5e15 and 0.2 * 2.5e15 < f16 <= 1.02 * 2.5e15
    assert 0.2 * 8e12 < cp <= 1.02 * 8e12
    with pytest.raises(P.AlsError):
        als2 = P.Als(16)
        try:
            als2.measure_peak(7)
        finally:
            als2.close()


def test_more_matrices_than_cached_plans(P):
    """One context keeps four plans: seven matrices taken in turn force plans to be dropped and rebuilt, between
    updates and RMSE calls, and every result is still that of its own matrix."""
    rng = np.random.default_rng(3)
    f, n = 100, 2000
    Theta = W.random_factors(n, f, seed=1, scale=0.3)
    Td = _dev(Theta)
    als = P.Als(f, solver=P.SOLVER_CHOLESKY, chunk=128, batch_slots=16)
    mats = []
    for k in range(7):
        m = int(rng.integers(50, 300))
        deg = np.minimum(rng.choice([0, 1, 5, 40, 63, 64, 127, 128, 129, 300, 700, 2000], m), n)
        ptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int64)
        idx = np.concatenate([np.sort(rng.choice(n, d, replace=False)) for d in deg] + [np.zeros(0, np.int64)]).astype(np.int32)
        val = (rng.standard_normal(int(ptr[-1])) * 2 + 3).astype(np.float32)
        Xs = W.random_factors(m, f, seed=k + 10, scale=0.3)
        mats.append((P.SparseMatrix.from_host(m, n, ptr, idx, val), oracle.update_rows(ptr, idx, val, Theta, 0.1), deg, Xs,
                     oracle.rmse(ptr, idx, val, Xs, Theta)))
    for rnd in range(3):
        for k in rng.permutation(7):
            sp, ref, deg, Xs, ro = mats[k]
            X = torch.zeros((sp.nrows, f), device="cuda:0")
            als.update_rows(sp, Td, 0.1, X)
            if rnd == 1:
                assert abs(als.rmse(sp, _dev(Xs), Td) - ro) <= 1e-5 * ro
            als.synchronize()
            got, live = X.cpu().numpy(), deg > 0
            assert not got[~live].any()
            assert _row_rel_err(got[live], ref[live]).max() <= TOL_EXACT, (rnd, int(k))
    als.close()


@pytest.mark.parametrize("f,chunk", [(32, 64), (100, 256), (256, 128)])
def test_epsilon_stopping_rule_of_algorithm_1(P, f, chunk):
    """Algorithm 1 stops when sqrt(r^T r) < epsilon.  With f_s = 30 and an epsilon large enough to leave a visible
    distance to the converged solution, rows of different degree stop after different numbers of iterations (the
    oracle's counts are checked to spread).  The result follows the double-precision Algorithm 1 with the same
    epsilon, and where stopping early changes a row by more than 3e-4 it is the early-stopped row that the GPU has.
    A row whose residual passes within rounding of epsilon may stop one iteration apart in fp32 and fp64: two such
    rows are allowed."""
    n, fs, lam, eps = 1500, 30, 0.1, 0.1
    rng = np.random.default_rng(17)
    degrees = np.concatenate([[0, 1, 2, 3, 5, 8, 16, 33, 64, 100, 257, 600, 1500], rng.integers(1, 3 * chunk, 80)])
    ptr = np.concatenate([[0], np.cumsum(degrees)]).astype(np.int64)
    idx = np.concatenate([np.sort(rng.choice(n, d, replace=False)) for d in degrees] + [np.zeros(0, np.int64)]).astype(np.int32)
    val = (rng.standard_normal(int(ptr[-1])) + 3).astype(np.float32)
    Theta = W.random_factors(n, f, seed=f, scale=0.3)
    warm = W.random_factors(len(degrees), f, seed=f + 1, scale=0.05)
    counts = []
    for u in (1, 4, 8, 10, 12):   # iterations the oracle takes on a few rows: the rule must bite, and not at once
        s, e = ptr[u], ptr[u + 1]
        A, b = oracle.normal_eq(idx[s:e], val[s:e], Theta, lam)
        counts.append(oracle.cg(A, warm[u], b, fs=fs, eps=eps)[1])
    assert max(counts) < fs and len(set(counts)) >= 3, counts
    ref = oracle.update_rows_cg(ptr, idx, val, Theta, lam, warm, fs=fs, eps=eps)[1:]
    full = oracle.update_rows_cg(ptr, idx, val, Theta, lam, warm, fs=fs, eps=0.0)[1:]
    als = P.Als(f, solver=P.SOLVER_CG, cg_iters=fs, cg_eps=eps, chunk=chunk)
    sp = P.SparseMatrix.from_host(len(degrees), n, ptr, idx, val)
    X = _dev(warm.copy())
    als.update_rows(sp, _dev(Theta), lam, X)
    als.synchronize()
    got = X.cpu().numpy()
    als.close()
    assert not got[0].any()
    err = _row_rel_err(got[1:], ref)
    to_full = _row_rel_err(got[1:], full)
    moved = _row_rel_err(ref, full) > 3e-4          # rows on which the rule makes a visible difference
    print(f"f={f}: oracle iteration counts {counts}; rows moved by the rule {int(moved.sum())}; "
          f"rows off the epsilon oracle by more than 2e-3: {int((err > 2e-3).sum())}, median {np.median(err):.2e}", flush=True)
    assert moved.sum() >= 10
    assert (err > 2e-3).sum() <= 2
    assert (err[moved] < to_full[moved]).mean() >= 0.9


@pytest.mark.parametrize("f", [100, 256])
def test_zero_iterations_leave_the_warm_start(P, f):
    """f_s = 0: Algorithm 1 computes the residual and returns x unchanged (rows without entries still become 0)."""
    n = 400
    rng = np.random.default_rng(2)
    degrees = np.array([0, 1, 7, 64, 300, 400, 130, 0, 33])
    ptr = np.concatenate([[0], np.cumsum(degrees)]).astype(np.int64)
    idx = np.concatenate([np.sort(rng.choice(n, d, replace=False)) for d in degrees] + [np.zeros(0, np.int64)]).astype(np.int32)
    val = rng.integers(1, 6, int(ptr[-1])).astype(np.float32)
    warm = W.random_factors(len(degrees), f, seed=3, scale=0.2)
    als = P.Als(f, solver=P.SOLVER_CG, cg_iters=0, chunk=128)
    sp = P.SparseMatrix.from_host(len(degrees), n, ptr, idx, val)
    X = _dev(warm.copy())
    als.update_rows(sp, _dev(W.random_factors(n, f, seed=4, scale=0.3)), 0.1, X)
    als.synchronize()
    got = X.cpu().numpy()
    als.close()
    live = degrees > 0
    assert np.array_equal(got[live], warm[live]) and not got[~live].any()


def test_kernel_times_are_recorded_when_profiling_is_on(P):
    w = W.TINY
    a = W.generate(w)
    _, T0 = W.init_factors(w)
    als = P.Als(w.f, solver=P.SOLVER_CG, chunk=64, profile=True)
    sp = P.SparseMatrix.from_host(a.nrows, a.ncols, a.ptr, a.idx, a.val)
    X = torch.zeros((w.m, w.f), device="cuda:0")
    als.update_rows(sp, _dev(T0), w.lam, X)
    als.rmse(sp, X, _dev(T0))
    # (chunk = 64: rows of 64 entries or more go through slots, every other row runs Algorithm 1 on its gathered rows)
    for kid in (P.K_HERMITIAN, P.K_SOLVE, P.K_SHORT, P.K_RMSE, P.K_PLAN):
        ms, launches = als.kernel_time(kid)
        assert launches >= 1 and ms > 0.0, kid
    assert als.kernel_time(P.K_GRAM) == (0.0, 0) and als.kernel_time(P.K_FUSED) == (0.0, 0)
    dense = P.Als(w.f, solver=P.SOLVER_CG, chunk=64, profile=True, dense_short_rows=True)   # every row builds A_u
    dense.update_rows(sp, _dev(T0), w.lam, X)
    assert dense.kernel_time(P.K_FUSED)[1] >= 1 and dense.kernel_time(P.K_SHORT) == (0.0, 0)
    dense.close()
    als.profile_reset()
    assert als.kernel_time(P.K_HERMITIAN) == (0.0, 0)
    with pytest.raises(P.AlsError):
        als.kernel_time(99)
    als.close()
    quiet = P.Als(w.f, solver=P.SOLVER_CG, chunk=64)        # profiling off: nothing is recorded
    quiet.update_rows(sp, _dev(T0), w.lam, X)
    assert quiet.kernel_time(P.K_HERMITIAN) == (0.0, 0)
    quiet.close()


def test_row_ranges_and_empty_gram(P):
    """als_hermitian takes any row range inside the matrix, also the last rows and an empty one, and rejects a range
    outside it; the Gram matrix of a factor without rows is zero."""
    f, n = 32, 200
    a = _edge_matrix(n, f, 5, [3, 0, 40, 17, 1])
    Theta = W.random_factors(n, f, seed=6, scale=0.4)
    als = P.Als(f)
    sp = P.SparseMatrix.from_host(a.nrows, a.ncols, a.ptr, a.idx, a.val)
    A, b = als.hermitian(sp, _dev(Theta), 0.2, 3, 2)          # the last two rows
    for k, u in enumerate((3, 4)):
        s, e = a.ptr[u], a.ptr[u + 1]
        Ao, bo = oracle.normal_eq(a.idx[s:e], a.val[s:e], Theta, 0.2)
        assert np.abs(A[k].cpu().numpy() - Ao).max() <= 1e-5 * np.abs(Ao).max()
        assert np.abs(b[k].cpu().numpy() - bo).max() <= 1e-5 * max(np.abs(bo).max(), 1e-30)
    import ctypes
    dummy = torch.zeros(f * f, device="cuda:0")
    desc = ctypes.byref(sp.desc)
    assert als._lib.als_hermitian(als._ctx, desc, _dev(Theta).data_ptr(), 0.2, f, 5, 0, dummy.data_ptr(), dummy.data_ptr()) == 0
    for row0, nrows in ((4, 2), (-1, 1), (0, 6)):
        assert als._lib.als_hermitian(als._ctx, desc, _dev(Theta).data_ptr(), 0.2, f, row0, nrows, dummy.data_ptr(),
                                      dummy.data_ptr()) == -1
    G = als.gram(torch.zeros((0, f), device="cuda:0"))
    assert tuple(G.shape) == (f, f) and not G.cpu().numpy().any()
    als.close()
