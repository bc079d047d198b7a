"""A caller-owned workspace (als_workspace_bytes + als_config.workspace): with it the update, RMSE, implicit and
check calls take no device memory of their own, and compute exactly what the library-allocated path computes."""
import ctypes

import numpy as np
import pytest

import workload as W

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def _pair(P, w):
    a = W.generate(w)
    c = W.transpose(a)
    return (P.SparseMatrix.from_host(a.nrows, a.ncols, a.ptr, a.idx, a.val),
            P.SparseMatrix.from_host(c.nrows, c.ncols, c.ptr, c.idx, c.val))


def _sweeps(als, csr, csc, w, n, implicit=None):
    X0, T0 = W.init_factors(w)
    X, T = _dev(X0), _dev(T0)
    for _ in range(n):
        if implicit is None:
            als.update_rows(csr, T, w.lam, X)
            als.update_cols(csc, X, w.lam, T)
        else:
            als.update_rows_implicit(csr, T, w.lam, implicit, X)
            als.update_cols_implicit(csc, X, w.lam, implicit, T)
    return X, T, als.rmse(csr, X, T)


@pytest.mark.parametrize("mode", ["cg", "exact", "cg_bf16_storage", "implicit"])
def test_workspace_path_allocates_nothing_and_equals_the_library_owned_path(mode):
    import paper_1808_03843_amd as P
    w1, w2 = W.MID_SMALL, W.SQUARE_SMALL
    kw = {"cg": dict(solver=P.SOLVER_CG, cg_iters=6), "exact": dict(solver=P.SOLVER_CHOLESKY),
          "cg_bf16_storage": dict(solver=P.SOLVER_CG, cg_iters=6, herm_dtype=P.BF16),
          "implicit": dict(solver=P.SOLVER_CG, cg_iters=6)}[mode]
    kw["chunk"] = 256          # long rows of these small shapes go through slots and several batches
    kw["batch_slots"] = 512
    implicit = 2.0 if mode == "implicit" else None
    m1, m2 = _pair(P, w1), _pair(P, w2)
    # library-owned memory first: the reference results, and every kernel has run once (code objects are loaded)
    ref = P.Als(w1.f, **kw)
    want = [_sweeps(ref, *m1, w1, 3, implicit), _sweeps(ref, *m2, w2, 3, implicit)]
    ref.check_matrix(m1[0])
    ref.synchronize()
    ref.close()
    rows = max(w1.m, w1.n, w2.m, w2.n)
    nnz = max(w1.nnz, w2.nnz)
    als = P.Als(w1.f, workspace_rows=rows, workspace_nnz=nnz, **kw)      # torch allocates the workspace here
    assert als.workspace is not None and als.workspace.numel() == P.load_library().als_workspace_bytes(
        ctypes.byref(als.cfg), rows, nnz)
    als.workspace.fill_(0x5A)                                              # the library must not rely on zeroed memory ...
    als.close()
    als = P.Als(w1.f, workspace_rows=rows, workspace_nnz=nnz, **kw)       # ... beyond what als_create clears itself
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info(0)[0]
    held = torch.cuda.memory_allocated(0)
    # plain library calls only between the two readings (inputs and outputs are allocated by torch: counted separately)
    X0, T0 = W.init_factors(w1)
    got = []
    for (csr, csc), w in ((m1, w1), (m2, w2), (m1, w1)):                  # the third pair finds or rebuilds its plans
        got.append(_sweeps(als, csr, csc, w, 3, implicit))
    als.check_matrix(m2[1])
    als.synchronize()
    torch.cuda.synchronize()
    # the library took nothing: what torch did not hand out for the new X / Theta tensors is still free
    new_tensors = torch.cuda.memory_allocated(0) - held
    reserved_growth = free_before - torch.cuda.mem_get_info(0)[0]
    assert reserved_growth <= max(new_tensors, 0) + (64 << 20), (reserved_growth, new_tensors)
    for (X, T, r), (Xw, Tw, rw) in zip(got, want + [want[0]]):
        assert torch.equal(X, Xw) and torch.equal(T, Tw) and r == rw      # bit for bit
    als.close()


def test_no_device_allocation_between_two_readings_with_preallocated_factors():
    """The strict form: inputs and outputs exist before the first reading, so the free device memory must not move
    at all across plan builds, three sweeps over two matrices, RMSE and synchronize."""
    import paper_1808_03843_amd as P
    w = W.MID_SMALL
    csr, csc = _pair(P, w)
    warm = P.Als(w.f, solver=P.SOLVER_CG, cg_iters=6)
    _sweeps(warm, csr, csc, w, 1)
    warm.synchronize()
    warm.close()
    als = P.Als(w.f, solver=P.SOLVER_CG, cg_iters=6, workspace_rows=max(w.m, w.n), workspace_nnz=w.nnz)
    X0, T0 = W.init_factors(w)
    X, T = _dev(X0), _dev(T0)
    als.synchronize()
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info(0)[0]
    for _ in range(3):
        als.update_rows(csr, T, w.lam, X)
        als.update_cols(csc, X, w.lam, T)
    r = als.rmse(csr, X, T)
    als.synchronize()
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info(0)[0] == free_before
    assert np.isfinite(r)
    als.close()


def test_matrix_beyond_the_workspace_is_refused_with_the_needed_size():
    import paper_1808_03843_amd as P
    w = W.TINY
    csr, csc = _pair(P, w)
    als = P.Als(w.f, workspace_rows=w.m // 2, workspace_nnz=w.nnz)
    X0, T0 = W.init_factors(w)
    with pytest.raises(P.AlsError) as err:
        als.update_rows(csr, _dev(T0), w.lam, _dev(X0))
    assert err.value.code == P.ALS_EINVAL and "workspace too small" in str(err.value) and "needs" in str(err.value)
    als.update_cols(csc, _dev(X0), w.lam, _dev(T0))     # the transpose has n = 1000 rows: fits
    als.synchronize()
    als.close()
