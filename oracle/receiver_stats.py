"""Receiver-head statistics of dense attention (TEST INFRASTRUCTURE ONLY).

Only tests, the smoke check and the bench's CPU-baseline leg may import this.

Section 4.1 ("Thought Anchors") looks for heads whose attention concentrates on a few parts of
the context: it averages a head's attention probabilities over b_q x b_k spans (the "block mean"
pattern of the attention-patterns figure) and ranks heads by the maximum vertical kurtosis of
these block means.  Written out here from the definitions, in fp64, with the whole T x T
probability matrix of one (head, sequence) in memory:

  P        = softmax over visible keys of scale * Q K^T              (the dense pattern, mask C:
             a rule, or an explicit T x T array; a query that sees no key has a zero row)
  M[i, j]  = sum of P over (queries of block i) x (keys of block j) / (n_q(i) * n_k(j)),
             n_q, n_k the real tokens of the two blocks (a hidden pair counts as probability 0);
             defined where block j is valid for block i (C^blk[i, j] = 1 in the notation of
             Alg. 2), 0 elsewhere
  (b_q and b_k may differ: the sequence is then padded to a multiple of lcm(b_q, b_k) as in the
   preamble of Alg. 2, M is T_p / b_q by T_p / b_k, and a block of padding only is never valid)
  column j : the values M[i, j] over the valid i ("vertical" = along the query axis);
             col_mean[j] their mean (the vertical score of block j), col_kurt[j] their excess
             kurtosis m4 / m2^2 - 3 with biased central moments, 0 when there are fewer than
             4 values or no spread
  head     : max_kurt = max of col_kurt over the columns with at least 4 values (0 if none);
             vert_kurt = excess kurtosis of col_mean over the columns of the sequence that
             hold a real key (0 for fewer than 4 columns): the per-head statistic of the thought-anchors work the
             section follows, with blocks in place of sentences.

The arithmetic is pinned (tests/test_receiver_stats_oracle_pins.py: closed forms, brute force,
library kurtosis).  Which of the two head numbers the section means by "maximum vertical
kurtosis" is a reading of one sentence; the paper prints no value that would decide it: parity
unpinned for that choice, both numbers are returned.
"""
from __future__ import annotations

import math

import numpy as np


def visible(mask: str, window: int, tq: np.ndarray, tk: np.ndarray) -> np.ndarray:
    """The mask C at token level: causal (u <= t), full, sliding (u <= t and t - u < window)."""
    if mask == "full":
        return np.ones(np.broadcast(tq, tk).shape, dtype=bool)
    ok = tk <= tq
    if mask == "sliding":
        ok = ok & (tq - tk < window)
    elif mask != "causal":
        raise ValueError(mask)
    return ok


def token_mask(L: int, mask: str = "causal", window: int = 0, C=None) -> np.ndarray:
    """The mask C [L, L] of one sequence: a rule, or the explicit array given (mask = "array")."""
    if C is not None:
        C = np.asarray(C) != 0
        assert C.shape == (L, L)
        return C
    t = np.arange(L)
    return visible(mask, window, t[:, None], t[None, :])


def dense_probabilities(Qh: np.ndarray, Kh: np.ndarray, scale: float, mask: str = "causal",
                        window: int = 0, C=None) -> np.ndarray:
    """P [L, L] of one head and one sequence, fp64.  A query that sees no key at all (possible
    only with an explicit array) attends to nothing: its row of P is zero."""
    Qh = np.asarray(Qh, dtype=np.float64)
    Kh = np.asarray(Kh, dtype=np.float64)
    L = Qh.shape[0]
    S = scale * (Qh @ Kh.T)
    Cm = token_mask(L, mask, window, C)
    S = np.where(Cm, S, -np.inf)
    top = S.max(axis=1, keepdims=True)
    E = np.exp(S - np.where(np.isfinite(top), top, 0.0))
    den = E.sum(axis=1, keepdims=True)
    return np.where(den > 0, E / np.where(den > 0, den, 1.0), 0.0)


def block_means(P: np.ndarray, block: int, mask: str = "causal", window: int = 0, block_k=None, C=None):
    """(M [T_p / b_q, T_p / b_k], Cblk of the same shape) of one L x L probability matrix:
    spans of b_q = block queries by b_k = block_k keys (default b_k = b_q); T_p is L rounded up
    to a multiple of lcm(b_q, b_k) as in the preamble of Alg. 2."""
    L = P.shape[0]
    bq, bk = block, (block_k or block)
    ell = bq * bk // math.gcd(bq, bk)
    Tp = -(-L // ell) * ell
    Pp = np.pad(P, ((0, Tp - L), (0, Tp - L)))
    sums = Pp.reshape(Tp // bq, bq, Tp // bk, bk).sum(axis=(1, 3))
    nq = np.clip(L - np.arange(Tp // bq) * bq, 0, bq).astype(np.float64)   # real tokens per block
    nk = np.clip(L - np.arange(Tp // bk) * bk, 0, bk).astype(np.float64)
    t = np.arange(Tp)
    real = t < L
    if C is not None:
        Cp = np.pad(np.asarray(C) != 0, ((0, Tp - L), (0, Tp - L)))
    else:
        Cp = visible(mask, window, t[:, None], t[None, :]) & real[:, None] & real[None, :]
    Cblk = Cp.reshape(Tp // bq, bq, Tp // bk, bk).any(axis=(1, 3))
    M = np.where(Cblk, sums / np.maximum(np.outer(nq, nk), 1.0), 0.0)
    return M, Cblk


def excess_kurtosis(x) -> float:
    """m4 / m2^2 - 3 with the biased central moments; 0 for fewer than 4 values or no spread."""
    x = np.asarray(x, dtype=np.float64)
    n = x.size
    if n < 4:
        return 0.0
    c = x - x.mean()
    m2 = float(np.mean(c * c))
    if not m2 > 0.0:
        return 0.0
    m4 = float(np.mean(c ** 4))
    return m4 / (m2 * m2) - 3.0


def column_stats(M: np.ndarray, Cblk: np.ndarray):
    """col_mean [N], col_kurt [N], col_n [N] of one sequence's block means."""
    N = M.shape[1]
    mean = np.zeros(N)
    kurt = np.zeros(N)
    n = np.zeros(N, dtype=np.int64)
    for j in range(N):
        vals = M[Cblk[:, j], j]
        n[j] = vals.size
        mean[j] = vals.mean() if vals.size else 0.0
        kurt[j] = excess_kurtosis(vals)
    return mean, kurt, n


def head_stats(col_mean: np.ndarray, col_kurt: np.ndarray, col_n: np.ndarray):
    """(max_kurt, vert_kurt) of one (head, sequence)."""
    enough = col_n >= 4
    max_kurt = float(col_kurt[enough].max()) if enough.any() else 0.0
    # (a key block of padding only - possible when b_k < b_q - is no column of the pattern)
    return max_kurt, excess_kurtosis(np.asarray(col_mean)[np.asarray(col_n) > 0])


def receiver_stats(Q, K, heads: int, kv_heads: int, block: int, scale: float, cu_seqlens=None,
                   mask: str = "causal", window: int = 0, want_block_mean: bool = True, block_k=None, C=None):
    """Q [heads, T, d], K [kv_heads, T, d].  Returns a dict with
    block_mean [heads, NBq, NBk] (global block ids, zero across sequences; None if not wanted),
    col_mean, col_kurt [heads, NBk], head [heads, batch, 2] = (max_kurt, vert_kurt); NBq / NBk
    count the query / key blocks of all sequences (equal when b_q = b_k)."""
    Q = np.asarray(Q)
    K = np.asarray(K)
    T = Q.shape[1]
    bq, bk = block, (block_k or block)
    ell = bq * bk // math.gcd(bq, bk)
    cu = [0, T] if cu_seqlens is None else [int(c) for c in cu_seqlens]
    tp = [-(-(cu[s + 1] - cu[s]) // ell) * ell for s in range(len(cu) - 1)]
    q0 = np.concatenate([[0], np.cumsum([t // bq for t in tp])]).astype(int)
    k0 = np.concatenate([[0], np.cumsum([t // bk for t in tp])]).astype(int)
    g = heads // kv_heads
    bm = np.zeros((heads, q0[-1], k0[-1])) if want_block_mean else None
    cm = np.zeros((heads, k0[-1]))
    ck = np.zeros((heads, k0[-1]))
    hs = np.zeros((heads, len(tp), 2))
    for h in range(heads):
        for s in range(len(tp)):
            a, e = cu[s], cu[s + 1]
            assert C is None or len(tp) == 1                 # an explicit array covers one sequence
            P = dense_probabilities(Q[h, a:e], K[h // g, a:e], scale, mask, window, C)
            M, Cblk = block_means(P, bq, mask, window, bk, C)
            mean, kurt, n = column_stats(M, Cblk)
            if bm is not None:
                bm[h, q0[s]:q0[s + 1], k0[s]:k0[s + 1]] = M
            cm[h, k0[s]:k0[s + 1]] = mean
            ck[h, k0[s]:k0[s + 1]] = kurt
            hs[h, s] = head_stats(mean, kurt, n)
    return {"block_mean": bm, "col_mean": cm, "col_kurt": ck, "head": hs}


def block_mean_entry(Qh, Kh, block: int, scale: float, i: int, j: int, mask: str = "causal",
                     window: int = 0, block_k=None) -> float:
    """M[i, j] of one head and one sequence from the rows of block i alone (no L x L matrix):
    for checks at sizes where the dense pattern does not fit in memory."""
    Qh = np.asarray(Qh)
    Kh = np.asarray(Kh, dtype=np.float64)
    L = Qh.shape[0]
    bk = block_k or block
    q0, q1 = i * block, min(L, (i + 1) * block)
    k0, k1 = j * bk, min(L, (j + 1) * bk)
    S = scale * (np.asarray(Qh[q0:q1], dtype=np.float64) @ Kh.T)
    C = visible(mask, window, np.arange(q0, q1)[:, None], np.arange(L)[None, :])
    S = np.where(C, S, -np.inf)
    S = S - S.max(axis=1, keepdims=True)
    E = np.exp(S)
    P = E / E.sum(axis=1, keepdims=True)
    return float(P[:, k0:k1].sum() / ((q1 - q0) * (k1 - k0)))
