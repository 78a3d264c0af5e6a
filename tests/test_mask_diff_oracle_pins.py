"""Pins of oracle/mask_diff.py (CPU only): the dense definition (boolean masks subtracted
entry by entry), the paper's own sizes (k_success = 6, k_fail = 3 at T = 1000, b = 32), and
the algebra of set difference."""
import numpy as np

from oracle import bruteforce as bf
from oracle import stream_oracle as so
from oracle.mask_diff import mask_diff


def _lists(rng, rows, k, N, sorted_=True):
    idx = np.full((rows, k), -1, dtype=np.int32)
    cnt = rng.integers(0, k + 1, size=rows).astype(np.int32)
    for r in range(rows):
        c = min(int(cnt[r]), N)
        cnt[r] = c
        idx[r, :c] = np.sort(rng.choice(N, size=c, replace=False))
    return idx, cnt


def test_equals_dense_boolean_subtraction():
    rng = np.random.default_rng(3)
    rows, N = 200, 40
    ia, ca = _lists(rng, rows, 9, N)
    ib, cb = _lists(rng, rows, 5, N)
    sa = rng.standard_normal((rows, 9))
    out, cnt, wt = mask_diff(ia, ca, sa, ib, cb)
    A = np.zeros((rows, N), bool); B = np.zeros((rows, N), bool); W = np.full((rows, N), np.nan)
    for r in range(rows):
        A[r, ia[r, :ca[r]]] = True
        B[r, ib[r, :cb[r]]] = True
        W[r, ia[r, :ca[r]]] = sa[r, :ca[r]]
    D = A & ~B
    for r in range(rows):
        cols = np.nonzero(D[r])[0]
        assert cnt[r] == len(cols)
        np.testing.assert_array_equal(out[r, :cnt[r]], cols)
        np.testing.assert_array_equal(wt[r, :cnt[r]], W[r, cols])
        assert (out[r, cnt[r]:] == -1).all() and np.isneginf(wt[r, cnt[r]:]).all()


def test_paper_sizes_on_the_pruning_oracle():
    """T = 1000, b = 32, k_success = 6, k_fail = 3 (Section 4.2.2): the difference of the two
    estimated masks, checked against dense masks built from the two index lists."""
    rng = np.random.default_rng(11)
    T, d, b = 1000, 16, 32
    Q = rng.standard_normal((T, d)).astype(np.float32)
    K = rng.standard_normal((T, d)).astype(np.float32)
    a = so.prune_head(Q, K, b, 6)
    f = so.prune_head(Q, K, b, 3)
    out, cnt, wt = mask_diff(a["idx"], a["cnt"], a["score"], f["idx"], f["cnt"])
    N = -(-T // b)
    Ma = bf.mask_from_blocks([list(a["idx"][q, :a["cnt"][q]]) for q in range(N)], T, b)
    Mf = bf.mask_from_blocks([list(f["idx"][q, :f["cnt"][q]]) for q in range(N)], T, b)
    Md = bf.mask_from_blocks([list(out[q, :cnt[q]]) for q in range(N)], T, b)
    np.testing.assert_array_equal(Md, Ma & ~Mf)
    # Stream's masks are not nested in k, so the difference is neither empty nor everything
    assert 0 < cnt.sum() < a["cnt"].sum()


def test_algebra():
    rng = np.random.default_rng(5)
    ia, ca = _lists(rng, 100, 8, 30)
    ib, cb = _lists(rng, 100, 8, 30)
    sa = rng.standard_normal((100, 8))
    d1, c1, _ = mask_diff(ia, ca, sa, ib, cb)
    # a \\ a = empty; a \\ empty = a; (a \\ b) \\ b = a \\ b; |a \\ b| + |a & b| = |a|
    _, c0, _ = mask_diff(ia, ca, sa, ia, ca)
    assert (c0 == 0).all()
    d2, c2, w2 = mask_diff(ia, ca, sa, ib, np.zeros_like(cb))
    np.testing.assert_array_equal(c2, ca)
    for r in range(100):
        np.testing.assert_array_equal(d2[r, :c2[r]], ia[r, :ca[r]])
        np.testing.assert_array_equal(w2[r, :c2[r]], sa[r, :ca[r]])
        inter = len(set(ia[r, :ca[r]]) & set(ib[r, :cb[r]]))
        assert c1[r] + inter == ca[r]
    d3, c3, _ = mask_diff(d1, c1, None, ib, cb)
    np.testing.assert_array_equal(c3, c1)
    np.testing.assert_array_equal(d3, d1)
