"""A sweep captured in a HIP graph replays to the same factors as the eager calls.

After the first call on a matrix (which builds the plan and sizes the work buffers) an update call only
enqueues kernels on the context's stream: no allocation, no host synchronisation, no memset.  Such a call
can be captured.  The kernels sum in a fixed order, so a replay must reproduce the eager result bit for bit;
every replay is checked, with eager work and a synchronisation in between.
"""
import numpy as np
import pytest

import workload as W

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.mark.parametrize("mode", ["cg", "exact", "implicit_cg"])
def test_captured_sweep_replays_match_eager(mode):
    import paper_1808_03843_amd as P
    w = W.MID_SMALL
    a = W.generate(w)
    c = W.transpose(a)
    X0, T0 = W.init_factors(w)
    side = torch.cuda.Stream()
    implicit = mode.startswith("implicit")
    with torch.cuda.stream(side):
        als = P.Als(w.f, solver=P.SOLVER_CHOLESKY if mode == "exact" else P.SOLVER_CG, chunk=256,
                    stream=side.cuda_stream)
        csr = P.SparseMatrix.from_host(a.nrows, a.ncols, a.ptr, a.idx, a.val)
        csc = P.SparseMatrix.from_host(c.nrows, c.ncols, c.ptr, c.idx, c.val)
        X = torch.from_numpy(X0.copy()).cuda()
        T = torch.from_numpy(T0.copy()).cuda()
        start = (X.clone(), T.clone())

        def sweep():
            if implicit:
                als.update_rows_implicit(csr, T, 0.5, 2.0, X)
                als.update_cols_implicit(csc, X, 0.5, 2.0, T)
            else:
                als.update_rows(csr, T, w.lam, X)
                als.update_cols(csc, X, w.lam, T)

        eager = []
        for _ in range(4):   # the first of these also builds the plans and buffers
            sweep()
            als.synchronize()
            eager.append((X.clone(), T.clone()))
        X.copy_(start[0])
        T.copy_(start[1])
        side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        sweep()
    for k in range(4):
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(X, eager[k][0]) and torch.equal(T, eager[k][1]), (mode, k)
        with torch.cuda.stream(side):   # eager work between the replays: reads only
            if implicit:
                als.implicit_loss(csr, X, T, 0.5, 2.0)
            else:
                als.rmse(csr, X, T)
    with torch.cuda.stream(side):
        als.synchronize()
        als.close()
