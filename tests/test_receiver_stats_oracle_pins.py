"""Pins of oracle/receiver_stats.py (CPU only): closed forms for uniform attention, the
row-stochastic invariant, brute force with Python loops on tiny inputs, library and textbook
values of the kurtosis, invariances of the softmax, and a planted receiver block."""
import math
from fractions import Fraction

import numpy as np
import pytest
import scipy.stats

from oracle import receiver_stats as rs


def _qk(rng, H, Hkv, T, d):
    return rng.standard_normal((H, T, d)), rng.standard_normal((Hkv, T, d))


def test_uniform_attention_closed_form():
    # Q = 0: every query t spreads 1/(t+1) over its t+1 visible keys.  Below the diagonal
    # M[i,j] = (H_{(i+1)b} - H_{ib}) / b with H_n the harmonic numbers; on the diagonal the
    # query at offset m sees m+1 keys of the block.
    b, N, d = 4, 5, 8
    L = b * N
    P = rs.dense_probabilities(np.zeros((L, d)), np.ones((L, d)), 0.3)
    M, C = rs.block_means(P, b)
    for i in range(N):
        below = sum(Fraction(1, i * b + m + 1) for m in range(b)) / b
        diag = sum(Fraction(m + 1, i * b + m + 1) for m in range(b)) / (b * b)
        for j in range(N):
            want = float(below) if j < i else float(diag) if j == i else 0.0
            assert M[i, j] == pytest.approx(want, rel=1e-14, abs=0)
            assert C[i, j] == (j <= i)


def test_full_mask_uniform_is_flat():
    b, L = 4, 14                                        # ragged: last block has 2 tokens
    P = rs.dense_probabilities(np.zeros((L, 3)), np.ones((L, 3)), 1.0, mask="full")
    M, C = rs.block_means(P, b, mask="full")
    assert C.all()
    np.testing.assert_allclose(M, 1.0 / L, rtol=1e-14)   # mean over real pairs only
    mean, kurt, n = rs.column_stats(M, C)
    assert (n == 4).all() and np.allclose(mean, 1.0 / L)
    assert np.abs(kurt).max() < 1e-6 or (kurt == 0).all()


@pytest.mark.parametrize("mask,window", [("causal", 0), ("full", 0), ("sliding", 5), ("sliding", 1)])
def test_equals_python_loops(mask, window):
    rng = np.random.default_rng(11)
    L, d, b, scale = 11, 3, 4, 0.7
    Q = rng.standard_normal((L, d))
    K = rng.standard_normal((L, d))
    N = -(-L // b)
    want = [[0.0] * N for _ in range(N)]
    valid = [[False] * N for _ in range(N)]
    for t in range(L):
        vis = [u for u in range(L)
               if mask == "full" or (u <= t and (mask == "causal" or t - u < window))]
        s = {u: scale * sum(Q[t, c] * K[u, c] for c in range(d)) for u in vis}
        z = sum(math.exp(v) for v in s.values())
        for u in vis:
            want[t // b][u // b] += math.exp(s[u]) / z
            valid[t // b][u // b] = True
    ntok = [min(b, L - i * b) for i in range(N)]
    P = rs.dense_probabilities(Q, K, scale, mask, window)
    M, C = rs.block_means(P, b, mask, window)
    for i in range(N):
        for j in range(N):
            assert bool(C[i, j]) == valid[i][j]
            assert M[i, j] == pytest.approx(want[i][j] / (ntok[i] * ntok[j]), rel=1e-12, abs=1e-300)


def test_rows_of_block_means_sum_to_one():
    # every query's probabilities sum to 1, so sum_j M[i,j] * n_k(j) = 1 for every query block
    rng = np.random.default_rng(5)
    L, b = 150, 16
    Q, K = rng.standard_normal((L, 8)), rng.standard_normal((L, 8))
    for mask, w in (("causal", 0), ("sliding", 40), ("full", 0)):
        M, _ = rs.block_means(rs.dense_probabilities(Q, K, 0.5, mask, w), b, mask, w)
        ntok = np.minimum(b, L - np.arange(M.shape[0]) * b)
        np.testing.assert_allclose(M @ ntok, 1.0, rtol=1e-12)


def test_softmax_invariances():
    rng = np.random.default_rng(6)
    L, d = 70, 8
    Q, K = rng.standard_normal((L, d)), rng.standard_normal((L, d))
    P = rs.dense_probabilities(Q, K, 0.4)
    # a vector added to every key shifts each row of the scores by a constant
    np.testing.assert_allclose(rs.dense_probabilities(Q, K + rng.standard_normal(d), 0.4), P, atol=1e-13)
    # scale and Q trade off
    np.testing.assert_allclose(rs.dense_probabilities(2 * Q, K, 0.2), P, atol=1e-13)
    # a window that covers the sequence is the causal mask
    np.testing.assert_array_equal(rs.dense_probabilities(Q, K, 0.4, "sliding", L), P)
    assert (np.triu(P, 1) == 0).all() and (P >= 0).all()
    # window 1: every query sees only itself
    np.testing.assert_array_equal(rs.dense_probabilities(Q, K, 0.4, "sliding", 1), np.eye(L))


def test_valid_columns_counts():
    L, b = 64, 8
    N = L // b
    P = np.full((L, L), 1.0)
    _, C = rs.block_means(P, b, "causal")
    assert [int(C[:, j].sum()) for j in range(N)] == [N - j for j in range(N)]
    _, C = rs.block_means(P, b, "sliding", 9)
    # query block i sees key blocks i-1 and i (window 9 reaches 8 keys back), i-2 never
    for i in range(N):
        assert [j for j in range(N) if C[i, j]] == [j for j in (i - 1, i) if j >= 0]
    _, C = rs.block_means(P, b, "sliding", 10)
    for i in range(N):
        assert [j for j in range(N) if C[i, j]] == [j for j in (i - 2, i - 1, i) if j >= 0]


def test_kurtosis_against_library_and_closed_forms():
    rng = np.random.default_rng(7)
    for n in (4, 5, 17, 300):
        x = rng.standard_normal(n) ** 3
        assert rs.excess_kurtosis(x) == pytest.approx(scipy.stats.kurtosis(x, fisher=True, bias=True), rel=1e-12)
    # one spike among n values is a Bernoulli(1/n) sample: excess kurtosis (1 - 6pq) / (pq)
    for n in (4, 10, 1000):
        p, q = 1.0 / n, 1.0 - 1.0 / n
        x = np.zeros(n); x[n // 3] = 2.5
        assert rs.excess_kurtosis(x) == pytest.approx((1 - 6 * p * q) / (p * q), rel=1e-12)
    # equally spaced values: -6 (n^2 + 1) / (5 (n^2 - 1))
    n = 12
    assert rs.excess_kurtosis(3.0 + 0.5 * np.arange(n)) == pytest.approx(-6 * (n * n + 1) / (5 * (n * n - 1)), rel=1e-12)
    # degenerate inputs
    assert rs.excess_kurtosis([1.0, 2.0, 9.0]) == 0.0
    assert rs.excess_kurtosis([2.0] * 8) == 0.0
    # shift and scale invariance
    x = rng.standard_normal(50)
    assert rs.excess_kurtosis(7 - 3 * x) == pytest.approx(rs.excess_kurtosis(x), rel=1e-10)


def test_column_and_head_stats_follow_their_definitions():
    rng = np.random.default_rng(8)
    N = 9
    M = np.tril(rng.random((N, N)))
    C = np.tril(np.ones((N, N), bool))
    mean, kurt, n = rs.column_stats(M, C)
    for j in range(N):
        col = M[j:, j]
        assert n[j] == N - j and mean[j] == pytest.approx(col.mean())
        want = scipy.stats.kurtosis(col, fisher=True, bias=True) if N - j >= 4 else 0.0
        assert kurt[j] == pytest.approx(want, rel=1e-11, abs=1e-12)
    mx, vk = rs.head_stats(mean, kurt, n)
    assert mx == pytest.approx(max(kurt[j] for j in range(N) if N - j >= 4))
    assert vk == pytest.approx(scipy.stats.kurtosis(mean, fisher=True, bias=True))
    # a short sequence has no column with 4 values
    assert rs.head_stats(mean[:3], kurt[:3], np.array([3, 2, 1])) == (0.0, 0.0)


def test_planted_receiver_block_stands_out():
    # one key block that every later query attends to strongly: its vertical score is the
    # largest and the head's vertical kurtosis exceeds that of an unplanted head
    rng = np.random.default_rng(9)
    H, T, d, b = 2, 512, 16, 16
    Q, K = _qk(rng, H, H, T, d)
    u = rng.standard_normal(d); u /= np.linalg.norm(u)
    Q[1] += 2.0 * u
    K[1, 5 * b:6 * b] = 6.0 * u
    out = rs.receiver_stats(Q, K, H, H, b, 1.0 / math.sqrt(d))
    cm = out["col_mean"]
    assert int(np.argmax(cm[1][1:])) + 1 == 5          # block 0 aside (it is all a first query sees)
    assert out["head"][1, 0, 1] > out["head"][0, 0, 1] + 1.0
    assert out["head"][1, 0, 0] >= out["col_kurt"][1][:T // b - 3].max() - 1e-12


def test_packed_batch_gqa_and_entry_helper():
    rng = np.random.default_rng(10)
    H, Hkv, d, b = 4, 2, 8, 8
    cu = [0, 37, 37 + 64, 37 + 64 + 21]
    T = cu[-1]
    Q, K = _qk(rng, H, Hkv, T, d)
    out = rs.receiver_stats(Q, K, H, Hkv, b, 0.3, cu_seqlens=cu, mask="sliding", window=20)
    nblk = [5, 8, 3]
    blk0 = [0, 5, 13]
    assert out["block_mean"].shape == (H, 16, 16) and out["head"].shape == (H, 3, 2)
    for h in (0, 3):
        for s in range(3):
            a, e = cu[s], cu[s + 1]
            alone = rs.receiver_stats(Q[h:h + 1, a:e], K[h // 2:h // 2 + 1, a:e], 1, 1, b, 0.3,
                                      mask="sliding", window=20)
            lo, hi = blk0[s], blk0[s] + nblk[s]
            np.testing.assert_array_equal(out["block_mean"][h, lo:hi, lo:hi], alone["block_mean"][0])
            np.testing.assert_array_equal(out["col_kurt"][h, lo:hi], alone["col_kurt"][0])
            np.testing.assert_array_equal(out["head"][h, s], alone["head"][0, 0])
            # nothing across sequences
            assert out["block_mean"][h, lo:hi, :lo].sum() == 0 and out["block_mean"][h, lo:hi, hi:].sum() == 0
            for (i, j) in ((nblk[s] - 1, nblk[s] - 1), (nblk[s] - 1, nblk[s] - 2), (2, 1)):
                got = rs.block_mean_entry(Q[h, a:e], K[h // 2, a:e], b, 0.3, i, j, "sliding", 20)
                assert got == pytest.approx(alone["block_mean"][0][i, j], rel=1e-12, abs=1e-300)


def test_rectangular_spans_are_weighted_means_of_square_ones():
    # a span of 2b queries is the union of two spans of b queries (likewise for keys): its mean is
    # the mean of the two, weighted by their real tokens; and every real query's row still sums to 1
    rng = np.random.default_rng(12)
    L, b = 45, 4
    Q, K = rng.standard_normal((L, 5)), rng.standard_normal((L, 5))
    for mask, w in (("causal", 0), ("sliding", 11), ("full", 0)):
        P = rs.dense_probabilities(Q, K, 0.6, mask, w)
        Ms, Cs = rs.block_means(P, b, mask, w)                       # square, 12 x 12 (T_p = 48)
        n = np.clip(L - np.arange(12) * b, 0, b)
        Mq, Cq = rs.block_means(P, 2 * b, mask, w, block_k=b)        # 6 x 12
        Mk, Ck = rs.block_means(P, b, mask, w, block_k=2 * b)        # 12 x 6
        assert Mq.shape == (6, 12) and Mk.shape == (12, 6)
        for i in range(6):
            for j in range(12):
                num = Ms[2 * i, j] * n[2 * i] + Ms[2 * i + 1, j] * n[2 * i + 1]
                assert Mq[i, j] == pytest.approx(num / max(n[2 * i] + n[2 * i + 1], 1), rel=1e-12, abs=1e-300)
                assert Cq[i, j] == (Cs[2 * i, j] or Cs[2 * i + 1, j])
        for i in range(12):
            for j in range(6):
                num = Ms[i, 2 * j] * n[2 * j] + Ms[i, 2 * j + 1] * n[2 * j + 1]
                assert Mk[i, j] == pytest.approx(num / max(n[2 * j] + n[2 * j + 1], 1), rel=1e-12, abs=1e-300)
                assert Ck[i, j] == (Cs[i, 2 * j] or Cs[i, 2 * j + 1])
        np.testing.assert_allclose(Mq @ n, np.where(np.arange(6) * 2 * b < L, 1.0, 0.0), rtol=1e-12)
    # lcm padding: b_q = 2, b_k = 8, L = 5 -> T_p = 8: four query blocks (the last is padding), one key block
    M, C = rs.block_means(rs.dense_probabilities(Q[:5], K[:5], 1.0), 2, block_k=8)
    assert M.shape == (4, 1) and C[:, 0].tolist() == [True, True, True, False] and M[3, 0] == 0
    out = rs.receiver_stats(Q[None], K[None], 1, 1, 2, 1.0, block_k=8)
    assert out["block_mean"].shape == (1, 23 * 4 // 4 + 1, 6)        # T_p = 48: 24 x 6
    got = rs.block_mean_entry(Q, K, 2, 1.0, 9, 2, block_k=8)
    assert got == pytest.approx(out["block_mean"][0, 9, 2], rel=1e-12)


def test_explicit_array_equals_python_loops_and_the_rules():
    """The mask as an explicit array: Python loops over the visible pairs (with a query that sees
    nothing and a key block nobody sees), rectangular spans included; an array that spells out a
    rule gives what the rule gives."""
    rng = np.random.default_rng(12)
    L, d, scale = 13, 3, 0.6
    Q = rng.standard_normal((L, d))
    K = rng.standard_normal((L, d))
    C = rng.random((L, L)) < 0.45
    C[5, :] = False                      # a query without a key
    C[:, 8:12] = False                   # keys nobody sees (a whole key block for b_k = 4)
    for bq, bk in ((4, 4), (2, 4), (4, 2)):
        ell = bq * bk // math.gcd(bq, bk)
        Tp = -(-L // ell) * ell
        Nq, Nk = Tp // bq, Tp // bk
        want = [[0.0] * Nk for _ in range(Nq)]
        valid = [[False] * Nk for _ in range(Nq)]
        for t in range(L):
            vis = [u for u in range(L) if C[t, u]]
            s = {u: scale * sum(Q[t, c] * K[u, c] for c in range(d)) for u in vis}
            z = sum(math.exp(v) for v in s.values())
            for u in vis:
                want[t // bq][u // bk] += math.exp(s[u]) / z
                valid[t // bq][u // bk] = True
        nq = [max(0, min(bq, L - i * bq)) for i in range(Nq)]
        nk = [max(0, min(bk, L - j * bk)) for j in range(Nk)]
        P = rs.dense_probabilities(Q, K, scale, C=C)
        assert (P[5] == 0).all() and np.allclose(np.delete(P, 5, axis=0).sum(axis=1), 1.0)
        M, Cb = rs.block_means(P, bq, block_k=bk, C=C)
        for i in range(Nq):
            for j in range(Nk):
                assert bool(Cb[i, j]) == valid[i][j]
                if valid[i][j]:
                    assert M[i, j] == pytest.approx(want[i][j] / (nq[i] * nk[j]), rel=1e-12, abs=1e-300)
                else:
                    assert M[i, j] == 0.0
    t = np.arange(L)
    for mask, window in (("causal", 0), ("sliding", 5), ("full", 0)):
        arr = rs.visible(mask, window, t[:, None], t[None, :])
        a = rs.receiver_stats(Q[None], K[None], 1, 1, 4, scale, C=arr)
        r = rs.receiver_stats(Q[None], K[None], 1, 1, 4, scale, mask=mask, window=window)
        for key in ("block_mean", "col_mean", "col_kurt", "head"):
            np.testing.assert_array_equal(a[key], r[key])


def test_kurtosis_gradient_of_the_parity_checker_matches_finite_differences():
    """tests/parity.py derives the tolerance of a column kurtosis from the error of the block
    means through the gradient of the moment formula; the gradient is checked here against central
    differences of the oracle's excess_kurtosis, and the tolerance against actual perturbations."""
    from tests import parity

    rng = np.random.default_rng(8)
    for n, spread in ((4, 1.0), (9, 0.01), (40, 1.0), (200, 1e-3)):
        x = 1.0 + spread * rng.standard_normal(n)
        x[rng.integers(n)] += 6 * spread                      # a heavy tail, as a receiver block gives
        g = parity.kurtosis_gradient(x)
        for i in range(n):
            h = 1e-6 * spread
            xp, xm = x.copy(), x.copy()
            xp[i] += h
            xm[i] -= h
            fd = (rs.excess_kurtosis(xp) - rs.excess_kurtosis(xm)) / (2 * h)
            assert abs(fd - g[i]) <= 1e-5 * (1 + abs(g).max()), (n, i, fd, g[i])
        k0 = rs.excess_kurtosis(x)
        for rel in (1e-6, 1e-5, 2e-4):
            y = x * (1 + rel * rng.uniform(-1, 1, n))
            assert abs(rs.excess_kurtosis(y) - k0) <= parity.kurtosis_tolerance(x, y, k0)
