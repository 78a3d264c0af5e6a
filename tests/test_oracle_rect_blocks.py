"""Pins of the oracle for b_q != b_k (preamble of Alg. 2: pad to a multiple of lcm(b_q, b_k),
Q viewed in blocks of b_q tokens, K in blocks of b_k; the nodes range over the T_p / b_k key
blocks).  CPU only: dense brute force written separately, coarsening laws that tie rectangular
blocks to square ones, exact top-k when every block is scored, dense softmax for the attention."""
import math

import numpy as np
import pytest

from oracle import bruteforce as bf
from oracle import stream_oracle as so


def _qk(rng, T, d, ints=False):
    if ints:
        return (rng.integers(-3, 4, size=(T, d)).astype(np.float64), rng.integers(-3, 4, size=(T, d)).astype(np.float64))
    f = lambda: rng.standard_normal((T, d)).astype(np.float32).astype(np.float64)   # the oracle's input type
    return f(), f()


def _lists(out):
    return [sorted(int(x) for x in row[:c]) for row, c in zip(out["idx"], out["cnt"])]


SHAPES = [(2, 4), (4, 2), (1, 4), (4, 1), (2, 8), (8, 2), (3, 5), (5, 3), (6, 4), (4, 4)]


@pytest.mark.parametrize("bq,bk", SHAPES)
def test_matches_dense_brute_force(bq, bk):
    rng = np.random.default_rng(100 * bq + bk)
    n = 0
    for T in (1, 5, 16, 23, 40, 61):
        for k in (1, 2, 3, 5, 8):
            for ints in (False, True):
                Q, K = _qk(rng, T, 4, ints)
                A, Cblk = bf.block_score_table(Q, K, bq, block_k=bk)
                want = bf.stream_from_table(A, Cblk, k)
                got = so.prune_head(Q, K, bq, k, block_k=bk)
                assert got["idx"].shape[0] == A.shape[0] == so.padded_len(T, bq, bk) // bq
                assert _lists(got) == want, (T, k, ints)
                for q, lst in enumerate(want):
                    for j, r in enumerate(lst):
                        assert got["score"][q, j] == pytest.approx(A[q, r], rel=1e-12, abs=1e-12)
                n += 1
    assert n == 60


@pytest.mark.parametrize("mask,window", [("full", 0), ("sliding", 7), ("sliding", 1), ("sliding", 30)])
def test_mask_rules_and_explicit_masks_with_rectangular_blocks(mask, window):
    rng = np.random.default_rng(5)
    for (bq, bk) in ((2, 8), (8, 2), (4, 2), (3, 5)):
        for T in (19, 48):
            Q, K = _qk(rng, T, 3)
            t = np.arange(T)
            C = np.ones((T, T), np.uint8) if mask == "full" else \
                ((t[None, :] <= t[:, None]) & (t[:, None] - t[None, :] < window)).astype(np.uint8)
            A, Cblk = bf.block_score_table(Q, K, bq, C, block_k=bk)
            for k in (1, 3, 4):
                want = bf.stream_from_table(A, Cblk, k)
                assert _lists(so.prune_head(Q, K, bq, k, mask=mask, window=window, block_k=bk)) == want
                assert _lists(so.prune_head(Q, K, bq, k, C=C, block_k=bk)) == want
    # an arbitrary mask
    C = (rng.random((48, 48)) < 0.2).astype(np.uint8)
    Q, K = _qk(rng, 48, 3)
    A, Cblk = bf.block_score_table(Q, K, 8, C, block_k=2)
    assert _lists(so.prune_head(Q, K, 8, 3, C=C, block_k=2)) == bf.stream_from_table(A, Cblk, 3)


def test_square_blocks_are_unchanged_by_the_generalisation():
    rng = np.random.default_rng(6)
    Q, K = _qk(rng, 77, 5)
    a = so.prune_head(Q, K, 8, 3, want_trace=True)
    b = so.prune_head(Q, K, 8, 3, want_trace=True, block_k=8)
    for key in ("idx", "cnt", "score", "trace", "evals"):
        np.testing.assert_array_equal(a[key], b[key])
    assert so.padded_len(77, 8) == 80 and so.padded_len(77, 8, 12) == 96 and so.n_it(77, 8, 12) == 3


def test_coarsening_laws_of_the_block_score():
    # a query block of 2b tokens is the union of two query blocks of b tokens, and likewise for
    # keys: the masked maximum over the union is the maximum of the two maxima
    rng = np.random.default_rng(7)
    T, b = 50, 4
    Q, K = _qk(rng, T, 6)
    for mask, w in (("causal", 0), ("sliding", 9), ("full", 0)):
        for q in range(0, 6):
            for r in range(0, 6):
                wide_q = so.block_score(Q, K, 2 * b, q, r, mask=mask, window=w, block_k=b)
                parts = [so.block_score(Q, K, b, 2 * q + i, r, mask=mask, window=w) for i in (0, 1)]
                assert wide_q == max(parts)
                wide_k = so.block_score(Q, K, b, q, r, mask=mask, window=w, block_k=2 * b)
                parts = [so.block_score(Q, K, b, q, 2 * r + i, mask=mask, window=w) for i in (0, 1)]
                assert wide_k == max(parts)


def test_exact_top_k_when_every_key_block_is_scored_at_the_first_level():
    rng = np.random.default_rng(8)
    for (bq, bk, T, k) in ((2, 8, 64, 4), (8, 2, 32, 8), (4, 2, 24, 6)):
        Q, K = _qk(rng, T, 4)
        A, Cblk = bf.block_score_table(Q, K, bq, block_k=bk)
        assert A.shape[1] <= 2 * k
        assert _lists(so.prune_head(Q, K, bq, k, block_k=bk)) == bf.exact_block_topk(A, Cblk, k)


def test_padding_to_the_lcm():
    rng = np.random.default_rng(9)
    # b_q = 2, b_k = 8, T = 5: T_p = 8, four query blocks, the last one is padding only
    Q, K = _qk(rng, 5, 3)
    out = so.prune_head(Q, K, 2, 2, block_k=8)
    assert out["idx"].shape == (4, 2)
    assert out["cnt"].tolist() == [1, 1, 1, 0] and out["idx"][3].tolist() == [-1, -1]
    # b_q = 8, b_k = 2, T = 11: T_p = 16, two query blocks, eight key blocks of which 0..5 hold keys
    Q, K = _qk(rng, 11, 3)
    out = so.prune_head(Q, K, 8, 8, block_k=2)
    assert out["cnt"].tolist() == [4, 6]
    assert out["idx"][0, :4].tolist() == [0, 1, 2, 3] and out["idx"][1, :6].tolist() == [0, 1, 2, 3, 4, 5]


def test_count_law():
    # cnt = min(k, valid key blocks); causal: key block r is valid iff r * b_k <= last real query
    rng = np.random.default_rng(10)
    for (bq, bk, T) in ((2, 8, 45), (8, 2, 45), (3, 5, 31)):
        Q, K = _qk(rng, T, 3)
        Tp = so.padded_len(T, bq, bk)
        for k in (1, 2, 5):
            out = so.prune_head(Q, K, bq, k, block_k=bk)
            for q in range(Tp // bq):
                last = min((q + 1) * bq, T) - 1
                valid = 0 if q * bq >= T else last // bk + 1
                assert out["cnt"][q] == min(k, valid)


def test_attention_with_rectangular_blocks_equals_dense_masked_softmax():
    rng = np.random.default_rng(11)
    H, T, d = 2, 45, 4
    Q, K, V = (rng.standard_normal((H, T, d)).astype(np.float32).astype(np.float64) for _ in range(3))
    for (bq, bk) in ((2, 8), (8, 2), (3, 5)):
        pr = so.prune(Q, K, H, H, bq, 3, block_k=bk)
        at = so.sparse_attn(Q, K, V, H, H, bq, pr["idx"], pr["cnt"], 0.5, block_k=bk)
        for h in range(H):
            lists = [[int(x) for x in row[:c]] for row, c in zip(pr["idx"][h], pr["cnt"][h])]
            M = bf.mask_from_blocks(lists, T, bq, bk)
            O, lse, mass = bf.dense_attention(Q[h].astype(np.float32), K[h].astype(np.float32),
                                              V[h].astype(np.float32), M, 0.5)
            np.testing.assert_allclose(at["O"][h], O, atol=1e-12)
            np.testing.assert_allclose(at["lse"][h], lse, atol=1e-12)
            np.testing.assert_allclose(at["mass"][h], mass, atol=1e-12)


def test_attention_with_an_explicit_mask_equals_dense_masked_softmax():
    # Eq. (2) with M from Alg. 2 and an arbitrary C inside the retained blocks; a query that sees
    # none of its retained keys gets lse = -inf and a zero output
    rng = np.random.default_rng(12)
    H, T, d = 2, 45, 4
    Q, K, V = (rng.standard_normal((H, T, d)).astype(np.float32).astype(np.float64) for _ in range(3))
    C = (rng.random((T, T)) < 0.1).astype(np.uint8)
    C[np.arange(0, T, 2), np.arange(0, T, 2)] = 1
    unseen = 0
    for (bq, bk) in ((4, 4), (2, 8), (8, 2)):
        pr = so.prune(Q, K, H, H, bq, 3, block_k=bk, C=C)
        at = so.sparse_attn(Q, K, V, H, H, bq, pr["idx"], pr["cnt"], 0.5, block_k=bk, C=C)
        for h in range(H):
            A, Cb = bf.block_score_table(Q[h], K[h], bq, C, block_k=bk)
            assert [sorted(int(x) for x in r[:c]) for r, c in zip(pr["idx"][h], pr["cnt"][h])] == \
                bf.stream_from_table(A, Cb, 3)
            M = np.zeros((T, T), np.uint8)
            for q, (row, c) in enumerate(zip(pr["idx"][h], pr["cnt"][h])):
                for r in row[:c]:
                    M[q * bq:(q + 1) * bq, r * bk:(r + 1) * bk] = 1
            seen = (M * C).any(axis=1)
            unseen += int((~seen).sum())
            with np.errstate(invalid="ignore"):
                O, lse, _ = bf.dense_attention(Q[h], K[h], V[h], M * C, 0.5)
            np.testing.assert_allclose(at["O"][h][seen], O[seen], atol=1e-12)
            np.testing.assert_allclose(at["lse"][h][seen], lse[seen], atol=1e-12)
            assert np.isneginf(at["lse"][h][~seen]).all() and (at["O"][h][~seen] == 0).all()
            P = np.where((M * C)[seen] != 0, np.exp(0.5 * (Q[h][seen] @ K[h].T) - lse[seen][:, None]), 0.0)
            np.testing.assert_allclose(at["mass"][h], P.sum(axis=0), atol=1e-12)
    assert unseen > 0
