"""The seeded input generator: exact sizes, canonical CSR, row addressability, determinism."""
import numpy as np

import workload as W


def test_tiny_shape_and_canonical_form():
    w = W.TINY
    a = W.generate(w)
    assert a.nnz == w.nnz and len(a.ptr) == w.m + 1
    deg = np.diff(a.ptr)
    assert deg.min() >= w.dmin and deg.max() <= w.dmax
    assert a.idx.min() >= 0 and a.idx.max() < w.n
    for u in range(w.m):
        assert np.all(np.diff(a.idx[a.ptr[u]:a.ptr[u + 1]]) > 0)
    assert set(np.unique(a.val)) <= {1.0, 2.0, 3.0, 4.0, 5.0}


def test_rows_are_pure_functions_of_seed_and_row():
    g = W.Generator(W.MID_SMALL)
    full = g.csr()
    part = g.rows(1000, 1100)
    s, e = full.ptr[1000], full.ptr[1100]
    assert np.array_equal(part.idx, full.idx[s:e]) and np.array_equal(part.val, full.val[s:e])
    again = W.Generator(W.MID_SMALL).rows(1000, 1100)
    assert np.array_equal(part.idx, again.idx) and np.array_equal(part.val, again.val)


def test_large_square_rating_range_and_skew():
    w = W.SQUARE_SMALL
    a = W.generate(w)
    assert a.nnz == w.nnz
    assert set(np.unique(a.val)) <= set(float(10 * i) for i in range(11))
    assert (a.val == 0).any()          # stored zeros exist and must count as observations
    col_deg = np.bincount(a.idx, minlength=w.n)
    assert col_deg.max() > 20 * np.median(col_deg)     # popularity skew


def test_mid_degrees_match_the_stated_moments():
    deg = W.Generator(W.MID).degrees()
    assert deg.sum() == W.MID.nnz
    assert deg.max() == 17_000 and abs(deg.mean() - 206.3) < 0.1


def test_init_factors():
    x0, t0 = W.init_factors(W.TINY)
    assert x0.shape == (2000, 16) and not x0.any()
    assert t0.dtype == np.float32 and t0.min() >= 0 and t0.max() <= 0.25


def test_split_is_a_seeded_partition_of_the_entries():
    a = W.generate(W.TINY)
    tr, te = W.split(a, 0.1, seed=3)
    tr2, te2 = W.split(a, 0.1, seed=3)
    assert tr.nnz + te.nnz == a.nnz and 0.08 * a.nnz < te.nnz < 0.12 * a.nnz
    assert np.array_equal(te.idx, te2.idx) and np.array_equal(tr.ptr, tr2.ptr)
    # every entry lands in exactly one part, rows keep ascending columns
    key = lambda m: set(zip(np.repeat(np.arange(m.nrows), np.diff(m.ptr)).tolist(), m.idx.tolist()))
    assert key(tr) | key(te) == key(a) and not (key(tr) & key(te))
    for m in (tr, te):
        for u in range(0, m.nrows, 97):
            seg = m.idx[m.ptr[u]:m.ptr[u + 1]]
            assert np.all(np.diff(seg) > 0)
    _, te3 = W.split(a, 0.1, seed=4)
    assert not np.array_equal(te.idx, te3.idx)
