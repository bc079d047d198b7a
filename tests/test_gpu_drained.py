"""The production library against the canary build in which every hand-written MFMA waits for its operands and for
its result (ALS_DRAINED_MFMA in csrc/tiles.h).  The fp32 MFMAs are inline asm, invisible to the compiler's hazard
handling; the production code keeps the required distances by hand, and twice a missing wait produced wrong numbers
that only a parity test caught.  The sums are deterministic, so the two builds must agree bit for bit on every
variant; any difference is a hazard the hand-placed waits do not cover."""
import os

import numpy as np
import pytest

import workload as W

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

N_COLS = 3000
LAM, ALPHA = 0.3, 1.5


@pytest.fixture(scope="module")
def libs():
    import paper_1808_03843_amd as P
    from paper_1808_03843_amd import build as B
    assert os.path.exists(B.LIB_DRAINED), "the canary library is built by paper_1808_03843_amd.build.build()"
    return P, P.load_library(), P.load_library(B.LIB_DRAINED)


@pytest.fixture(scope="module")
def mat():
    rng = np.random.default_rng(321)
    degrees = [0, 1, 2, 3, 4, 5, 15, 16, 17, 31, 33, 63, 64, 65, 127, 129, 255, 256, 257, 511, 1000, 1025, 2049, 2900]
    degrees += [int(np.exp(rng.uniform(0, np.log(2500)))) for _ in range(30)]
    ptr = np.concatenate([[0], np.cumsum(degrees)]).astype(np.int64)
    idx = np.concatenate([np.sort(rng.choice(N_COLS, d, replace=False)) for d in degrees] + [np.zeros(0, int)]).astype(np.int32)
    val = (rng.integers(0, 11, size=int(ptr[-1])) * 0.5).astype(np.float32)
    return degrees, ptr, idx, val


def _run(P, lib, mat, f, solver, chunk, mode, dtype):
    degrees, ptr, idx, val = mat
    Theta = torch.from_numpy(W.random_factors(N_COLS, f, seed=57 + f, scale=0.3)).cuda()
    warm = torch.from_numpy(W.random_factors(len(degrees), f, seed=58 + f, scale=0.05)).cuda()
    sp = P.SparseMatrix.from_host(len(degrees), N_COLS, ptr, idx, val)
    code, tdt = {"f32": (P.F32, torch.float32), "bf16": (P.BF16, torch.bfloat16), "f32x3": (P.F32X3, torch.float32), "f32x2": (P.F32X2, torch.float32)}[dtype]
    als = P.Als(f, solver=P.SOLVER_CHOLESKY if solver == "cholesky" else P.SOLVER_CG, cg_iters=5, chunk=chunk,
                factor_dtype=code, library=lib)
    X = warm.clone()
    if mode == "implicit":
        als.update_rows_implicit(sp, Theta, LAM, ALPHA, X)
    else:
        als.update_rows(sp, Theta.to(tdt), LAM, X)
    A, b = als.hermitian(sp, Theta.to(tdt), LAM, 0, len(degrees)) if mode == "explicit" else (None, None)
    als.synchronize()
    als.close()
    return X, A, b


GRID = [(f, solver, chunk, mode, dtype)
        for f in (16, 32, 64, 100, 128, 256) for solver in ("cholesky", "cg") for chunk in (0, 64)
        for mode, dtype in (("explicit", "f32"), ("implicit", "f32"), ("explicit", "bf16"), ("explicit", "f32x3"), ("explicit", "f32x2"))
        if not (dtype in ("f32x3", "f32x2") and f == 256)]     # the three-part route exists for f <= 128


@pytest.mark.parametrize("f,solver,chunk,mode,dtype", GRID)
def test_production_build_equals_the_drained_build_bit_for_bit(libs, mat, f, solver, chunk, mode, dtype):
    P, prod, drained = libs
    X1, A1, b1 = _run(P, prod, mat, f, solver, chunk, mode, dtype)
    X2, A2, b2 = _run(P, drained, mat, f, solver, chunk, mode, dtype)
    assert torch.isfinite(X1).all()
    assert torch.equal(X1, X2), float((X1 - X2).abs().max())
    if A1 is not None:
        assert torch.equal(A1, A2) and torch.equal(b1, b2)
