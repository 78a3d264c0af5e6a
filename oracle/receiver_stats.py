"""Receiver-head statistics of dense attention (TEST INFRASTRUCTURE ONLY).

Only tests, the smoke check and the bench's CPU-baseline leg may import this.

Section 4.1 ("Thought Anchors") looks for heads whose attention concentrates on a few parts of
the context: it averages a head's attention probabilities over b_q x b_k spans (the "block mean"
pattern of the attention-patterns figure) and ranks heads by the maximum vertical kurtosis of
these block means.  Written out here from the definitions, in fp64, with the whole T x T
probability matrix of one (head, sequence) in memory:

  P        = softmax over visible keys of scale * Q K^T              (the dense pattern, mask C)
  M[i, j]  = sum of P over (queries of block i) x (keys of block j) / (n_q(i) * n_k(j)),
             n_q, n_k the real tokens of the two blocks (a hidden pair counts as probability 0);
             defined where block j is valid for block i (C^blk[i, j] = 1 in the notation of
             Alg. 2), 0 elsewhere
  column j : the values M[i, j] over the valid i ("vertical" = along the query axis);
             col_mean[j] their mean (the vertical score of block j), col_kurt[j] their excess
             kurtosis m4 / m2^2 - 3 with biased central moments, 0 when there are fewer than
             4 values or no spread
  head     : max_kurt = max of col_kurt over the columns with at least 4 values (0 if none);
             vert_kurt = excess kurtosis of col_mean over all columns of the sequence (0 for
             fewer than 4 columns): the per-head statistic of the thought-anchors work the
             section follows, with blocks in place of sentences.
"""
from __future__ import annotations

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


def dense_probabilities(Qh: np.ndarray, Kh: np.ndarray, scale: float, mask: str = "causal",
                        window: int = 0) -> np.ndarray:
    """P [L, L] of one head and one sequence, fp64."""
    Qh = np.asarray(Qh, dtype=np.float64)
    Kh = np.asarray(Kh, dtype=np.float64)
    L = Qh.shape[0]
    S = scale * (Qh @ Kh.T)
    t = np.arange(L)
    C = visible(mask, window, t[:, None], t[None, :])
    S = np.where(C, S, -np.inf)
    S = S - S.max(axis=1, keepdims=True)
    E = np.exp(S)
    return E / E.sum(axis=1, keepdims=True)


def block_means(P: np.ndarray, block: int, mask: str = "causal", window: int = 0):
    """(M [N, N], Cblk [N, N] bool) of one L x L probability matrix."""
    L = P.shape[0]
    N = -(-L // block)
    pad = N * block - L
    Pp = np.pad(P, ((0, pad), (0, pad)))
    sums = Pp.reshape(N, block, N, block).sum(axis=(1, 3))
    n_tok = np.minimum(block, L - np.arange(N) * block).astype(np.float64)
    t = np.arange(N * block)
    real = t < L
    C = visible(mask, window, t[:, None], t[None, :]) & real[:, None] & real[None, :]
    Cblk = C.reshape(N, block, N, block).any(axis=(1, 3))
    M = np.where(Cblk, sums / np.outer(n_tok, n_tok), 0.0)
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
    return max_kurt, excess_kurtosis(col_mean)


def receiver_stats(Q, K, heads: int, kv_heads: int, block: int, scale: float, cu_seqlens=None,
                   mask: str = "causal", window: int = 0, want_block_mean: bool = True):
    """Q [heads, T, d], K [kv_heads, T, d].  Returns a dict with
    block_mean [heads, NB, NB] (global block ids, zero across sequences; None if not wanted),
    col_mean, col_kurt [heads, NB], head [heads, batch, 2] = (max_kurt, vert_kurt)."""
    Q = np.asarray(Q)
    K = np.asarray(K)
    T = Q.shape[1]
    cu = [0, T] if cu_seqlens is None else [int(c) for c in cu_seqlens]
    nblk = [-(-(cu[s + 1] - cu[s]) // block) for s in range(len(cu) - 1)]
    blk0 = np.concatenate([[0], np.cumsum(nblk)]).astype(int)
    NB = int(blk0[-1])
    g = heads // kv_heads
    bm = np.zeros((heads, NB, NB)) if want_block_mean else None
    cm = np.zeros((heads, NB))
    ck = np.zeros((heads, NB))
    hs = np.zeros((heads, len(nblk), 2))
    for h in range(heads):
        for s in range(len(nblk)):
            a, e = cu[s], cu[s + 1]
            P = dense_probabilities(Q[h, a:e], K[h // g, a:e], scale, mask, window)
            M, Cblk = block_means(P, block, mask, window)
            mean, kurt, n = column_stats(M, Cblk)
            lo, hi = blk0[s], blk0[s + 1]
            if bm is not None:
                bm[h, lo:hi, lo:hi] = M
            cm[h, lo:hi] = mean
            ck[h, lo:hi] = kurt
            hs[h, s] = head_stats(mean, kurt, n)
    return {"block_mean": bm, "col_mean": cm, "col_kurt": ck, "head": hs}


def block_mean_entry(Qh, Kh, block: int, scale: float, i: int, j: int, mask: str = "causal",
                     window: int = 0) -> float:
    """M[i, j] of one head and one sequence from the rows of block i alone (no L x L matrix):
    for checks at sizes where the dense pattern does not fit in memory."""
    Qh = np.asarray(Qh)
    Kh = np.asarray(Kh, dtype=np.float64)
    L = Qh.shape[0]
    q0, q1 = i * block, min(L, (i + 1) * block)
    k0, k1 = j * block, min(L, (j + 1) * block)
    S = scale * (np.asarray(Qh[q0:q1], dtype=np.float64) @ Kh.T)
    C = visible(mask, window, np.arange(q0, q1)[:, None], np.arange(L)[None, :])
    S = np.where(C, S, -np.inf)
    S = S - S.max(axis=1, keepdims=True)
    E = np.exp(S)
    P = E / E.sum(axis=1, keepdims=True)
    return float(P[:, k0:k1].sum() / ((q1 - q0) * (k1 - k0)))
