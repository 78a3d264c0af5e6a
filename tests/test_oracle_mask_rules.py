"""Pins of the oracle's rule-based masks C (causal / sliding window / no mask), CPU only:
each rule against the explicit T x T mask it stands for (the explicit path is pinned by brute
force in test_oracle_pins.py), attention against dense masked softmax, and closed forms."""
import numpy as np
import pytest

from oracle import bruteforce as bf
from oracle import stream_oracle as so


def gauss(rng, T, d):
    return rng.standard_normal((T, d)).astype(np.float32)


def rule_mask(T, mask, window):
    t = np.arange(T)[:, None]
    u = np.arange(T)[None, :]
    if mask == "full":
        return np.ones((T, T), np.uint8)
    C = u <= t
    if mask == "sliding":
        C = C & (t - u < window)
    return C.astype(np.uint8)


def lists(idx, cnt):
    return [list(map(int, idx[q, :cnt[q]])) for q in range(len(cnt))]


@pytest.mark.parametrize("mask,window", [("sliding", 1), ("sliding", 5), ("sliding", 8), ("sliding", 13),
                                          ("sliding", 1000), ("full", 0), ("causal", 0)])
def test_rule_equals_explicit_mask(mask, window):
    rng = np.random.default_rng(window + len(mask))
    b, d = 4, 6
    for N, k in [(9, 2), (16, 3), (21, 5)]:
        T = N * b - 1
        Q, K = gauss(rng, T, d), gauss(rng, T, d)
        C = rule_mask(T, mask, window)
        a = so.prune_head(Q, K, b, k, mask=mask, window=window, want_trace=True)
        e = so.prune_head(Q, K, b, k, C=C, want_trace=True)
        for x in ("idx", "cnt", "score", "trace", "evals"):
            np.testing.assert_array_equal(a[x], e[x], err_msg=x)
        # and both equal the brute-force recursion over the dense masked score table
        A, Cblk = bf.block_score_table(Q, K, b, C)
        assert lists(a["idx"], a["cnt"]) == bf.stream_from_table(A, Cblk, k)


@pytest.mark.parametrize("mask,window", [("sliding", 6), ("sliding", 9), ("full", 0)])
def test_attention_under_a_rule_equals_dense_masked_softmax(mask, window):
    rng = np.random.default_rng(5 + window)
    b, d, N, k = 4, 8, 11, 3
    T = N * b - 3
    Q, K, V = gauss(rng, T, d), gauss(rng, T, d), gauss(rng, T, d)
    C = rule_mask(T, mask, window).astype(bool)
    p = so.prune_head(Q, K, b, k, mask=mask, window=window)
    o = so.sparse_attn(Q[None], K[None], V[None], 1, 1, b, p["idx"][None], p["cnt"][None], 0.25,
                       mask=mask, window=window)
    # block pattern M from the lists (all tokens of a retained block), times C
    M = np.zeros((T, T), bool)
    for q, lst in enumerate(lists(p["idx"], p["cnt"])):
        for r in lst:
            M[q * b:(q + 1) * b, r * b:(r + 1) * b] = True
    O, lse, mass = bf.dense_attention(Q, K, V, M & C, 0.25)
    np.testing.assert_allclose(o["O"][0], O, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(o["lse"][0], lse, rtol=1e-12)
    np.testing.assert_allclose(o["mass"][0], mass, rtol=1e-10, atol=1e-14)


def test_closed_forms_of_the_sliding_window_and_the_full_mask():
    rng = np.random.default_rng(8)
    b, d, N, k = 4, 6, 24, 4
    T = N * b
    Q, K = gauss(rng, T, d), gauss(rng, T, d)
    # a window that covers everything is the causal mask
    c = so.prune_head(Q, K, b, k)
    w = so.prune_head(Q, K, b, k, mask="sliding", window=T)
    np.testing.assert_array_equal(c["idx"], w["idx"])
    # window 1: a token sees only itself -> only the diagonal block is valid
    w1 = so.prune_head(Q, K, b, k, mask="sliding", window=1)
    for q in range(N):
        assert lists(w1["idx"], w1["cnt"])[q] == [q]
    # count law: min(k, number of valid blocks); valid blocks of row q are r_min(q) .. q
    for W in (3, 4, 9, 16, 30):
        o = so.prune_head(Q, K, b, k, mask="sliding", window=W)
        for q in range(N):
            rmin = max(0, -((-(q * b - W - b + 2)) // b))      # ceil((q b - W - b + 2) / b)
            lst = lists(o["idx"], o["cnt"])[q]
            assert len(lst) == min(k, q - rmin + 1), (W, q)
            assert all(rmin <= r <= q for r in lst)
            # a window of at most k blocks keeps every valid block (no pruning possible)
            if q - rmin + 1 <= k:
                assert lst == list(range(rmin, q + 1))
    # no mask: every row keeps min(k, N) blocks, and keys after the query are allowed
    f = so.prune_head(Q, K, b, k, mask="full")
    assert (f["cnt"] == min(k, N)).all()
    assert any(max(l) > q for q, l in enumerate(lists(f["idx"], f["cnt"])))
    # no mask + k >= N: attention is plain (bidirectional) softmax attention
    V = gauss(rng, T, d)
    fa = so.prune_head(Q, K, b, N, mask="full")
    o = so.sparse_attn(Q[None], K[None], V[None], 1, 1, b, fa["idx"][None], fa["cnt"][None], 1.0, mask="full")
    S = Q.astype(np.float64) @ K.astype(np.float64).T
    P = np.exp(S - S.max(1, keepdims=True)); P /= P.sum(1, keepdims=True)
    np.testing.assert_allclose(o["O"][0], P @ V.astype(np.float64), rtol=1e-10, atol=1e-12)
