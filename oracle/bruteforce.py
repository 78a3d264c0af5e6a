"""Brute-force cross-checks for the oracle (TEST INFRASTRUCTURE ONLY, tiny inputs).

Everything here materialises the dense T x T score matrix, which the method
exists to avoid; it is the independent yardstick the C oracle is pinned to.

  * block_score_table: S = Q K^T in fp64 (numpy matmul), masked by C, padded with
    zero rows/columns as in the preamble of Alg. 2, then max-pooled over
    b x b tiles -> A[q, r] and C^blk[q, r].
  * stream_from_table: the level recursion of Alg. 2 on that table (pure Python
    lists; written separately from the C code).
  * exact_block_topk: the k best causal blocks by A[q, :] - what Stream equals
    whenever every block is scored at the first level (N <= 2k).
  * dense_attention: textbook masked softmax attention (Eq. (2) with an explicit
    token mask).
"""
from __future__ import annotations

import math

import numpy as np


def causal_mask(T: int) -> np.ndarray:
    return np.tril(np.ones((T, T), dtype=np.uint8))


def block_score_table(Qh: np.ndarray, Kh: np.ndarray, block: int, C: np.ndarray | None = None,
                      block_k: int | None = None):
    """A [T_p / b_q, T_p / b_k] and C^blk of the same shape (block = b_q, block_k = b_k,
    default the same; T_p = T rounded up to a multiple of lcm(b_q, b_k))."""
    Qh = np.asarray(Qh, dtype=np.float64)
    Kh = np.asarray(Kh, dtype=np.float64)
    T = Qh.shape[0]
    bk = block if block_k is None else block_k
    C = causal_mask(T) if C is None else np.asarray(C)
    ell = math.lcm(block, bk)
    Tp = -(-T // ell) * ell
    S = np.full((Tp, Tp), -np.inf)
    S[:T, :T] = np.where(C != 0, Qh @ Kh.T, -np.inf)
    Cp = np.zeros((Tp, Tp), dtype=np.uint8)
    Cp[:T, :T] = C != 0
    A = S.reshape(Tp // block, block, Tp // bk, bk).max(axis=(1, 3))
    Cblk = Cp.reshape(Tp // block, block, Tp // bk, bk).max(axis=(1, 3))
    return A, Cblk


def stream_from_table(A: np.ndarray, Cblk: np.ndarray, k: int, n_levels: int | None = None):
    """Alg. 2 with every block score read from the dense table.  Returns list of index lists."""
    N = A.shape[1]                       # the nodes range over the key blocks
    n_it = (0 if N <= 1 else math.ceil(math.log2(N))) if n_levels is None else n_levels
    out = []
    for q in range(A.shape[0]):
        nodes = [((j * N) // k, ((j + 1) * N) // k - 1) for j in range(k)]
        for _ in range(n_it):
            branches = []
            for (f, l) in nodes:
                m = (f + l + 1) // 2
                branches.append((f, m - 1))
                branches.append((m, l))
            scored = []
            for pos, (f, l) in enumerate(branches):
                valid = [r for r in range(f, l + 1) if Cblk[q, r]]
                s = A[q, valid[0]] if valid else -np.inf
                scored.append((-s, pos))
            keep = sorted(pos for _, pos in sorted(scored)[:k])
            nodes = [branches[pos] for pos in keep]
        I = []
        for (f, l) in nodes:
            valid = [r for r in range(f, l + 1) if Cblk[q, r]]
            if valid:
                I.append(valid[0])
        out.append(sorted(I))
    return out


def exact_block_topk(A: np.ndarray, Cblk: np.ndarray, k: int):
    out = []
    for q in range(A.shape[0]):
        valid = [r for r in range(A.shape[1]) if Cblk[q, r]]
        best = sorted(valid, key=lambda r: (-A[q, r], r))[:k]
        out.append(sorted(best))
    return out


def dense_attention(Qh, Kh, Vh, token_mask: np.ndarray, scale: float):
    """softmax(mask(scale * Q K^T)) V with an explicit [T, T] 0/1 token mask; also lse and column sums."""
    Qh, Kh, Vh = (np.asarray(x, dtype=np.float64) for x in (Qh, Kh, Vh))
    S = scale * (Qh @ Kh.T)
    S = np.where(token_mask != 0, S, -np.inf)
    mx = S.max(axis=1, keepdims=True)
    E = np.exp(S - mx)
    Z = E.sum(axis=1, keepdims=True)
    P = E / Z
    return P @ Vh, (mx + np.log(Z))[:, 0], P.sum(axis=0)


def mask_from_blocks(idx_lists, T: int, block: int, block_k: int | None = None) -> np.ndarray:
    """Token-level mask M * C from per-query-block key-block lists (causal inside blocks)."""
    bk = block if block_k is None else block_k
    M = np.zeros((T, T), dtype=np.uint8)
    for q, lst in enumerate(idx_lists):
        t0, t1 = min(q * block, T), min((q + 1) * block, T)
        for r in lst:
            if r < 0:
                continue
            M[t0:t1, r * bk:min((r + 1) * bk, T)] = 1
    return M * causal_mask(T)
