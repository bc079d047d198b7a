"""als_gram_static: the entry point that allocates nothing (partial Gram matrices in a file-scope device array)
against als_gram, which allocates its slots, through the C ABI.  Two calls in a row on the shared array, the
second with a smaller input; then a matrix tall enough for the two calls to split the rows differently.
Collected last (the name sorts after every other test file): a failure here must not hide other tests."""
import ctypes

import numpy as np
import pytest

import workload as W

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


@pytest.mark.parametrize("f", [100, 256, 16])
def test_gram_static_equals_gram(f):
    import paper_1808_03843_amd as P
    als = P.Als(f)
    lib = P.load_library()
    out = torch.empty((f, f), dtype=torch.float32, device="cuda:0")
    # first 5,000 rows, then 700 in the same array, then 1 and 0: the array keeps the last call's contents
    for n in (5000, 700, 1, 0):
        G = _dev(W.random_factors(n, f, seed=300 + f + n, scale=0.4) + 0.1) if n else torch.empty((0, f), device="cuda:0")
        want = als.gram(G)
        out.fill_(float("nan"))
        als.synchronize()           # (the first use of a kernel or of a copy path may make the runtime allocate:
        torch.cuda.synchronize()    # torch's fill, the library's kernels and its status copy have all run by now)
        free_before = torch.cuda.mem_get_info(0)[0]
        rc = lib.als_gram_static(als._ctx, G.data_ptr(), n, f, out.data_ptr())   # through the C ABI
        assert rc == P.ALS_OK, lib.als_last_error(als._ctx)
        als.synchronize()
        assert torch.cuda.mem_get_info(0)[0] == free_before          # no device memory was taken or returned
        # up to 256 * (slots the array holds) rows both calls split the rows the same way: bit for bit
        assert torch.equal(out, want), (f, n, float((out - want).abs().max()))
        ref = G.double().T @ G.double()
        assert float((out.double() - ref).abs().max()) <= 2e-6 * max(float(ref.abs().max()), 1e-30)
    # taller than 256 rows per slot of the array at f = 256 (118 slots): fewer, longer work items than als_gram's
    n = 70_000 if f == 256 else 200_000
    G = _dev(W.random_factors(n, f, seed=400 + f, scale=0.4) + 0.1)
    want = als.gram(G)
    als.gram_static(G, out)
    als.synchronize()
    ref = G.double().T @ G.double()
    tol = 2e-6 * float(ref.abs().max())
    assert float((out.double() - ref).abs().max()) <= tol
    assert float((out - want).abs().max()) <= tol
    assert torch.equal(out, out.T)
    # and a smaller input again after the large one
    G = _dev(W.random_factors(333, f, seed=500 + f, scale=0.4) + 0.1)
    als.gram_static(G, out)
    assert torch.equal(out, als.gram(G))
    als.close()


def test_gram_static_rejects_sizes_beyond_its_maximum():
    import paper_1808_03843_amd as P
    als = P.Als(16)
    lib = P.load_library()
    out = torch.empty((16, 16), dtype=torch.float32, device="cuda:0")
    G = torch.zeros((4, 16), device="cuda:0")
    rc = lib.als_gram_static(als._ctx, G.data_ptr(), ctypes.c_int64((1 << 30) + 1), 16, out.data_ptr())
    assert rc == P.ALS_EINVAL and b"ALS_GRAM_STATIC_MAX_ROWS" in lib.als_last_error(als._ctx)
    assert lib.als_gram_static(als._ctx, G.data_ptr(), 4, 32, out.data_ptr()) == P.ALS_EINVAL   # f of another context
    als.close()
