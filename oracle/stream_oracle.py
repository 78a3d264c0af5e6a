"""Python face of the CPU oracle (TEST INFRASTRUCTURE ONLY).

Only tests, the smoke check and the bench's CPU-baseline leg may import this.
It wraps oracle/stream_oracle.c (Algorithm 2 of the paper and Eq. (2) on the
retained blocks, fp64) and adds what the listing leaves to the caller:

  * one call per query head: the mask is estimated "for each attention head"
    (Section 3); with grouped-query attention query head h reads key/value head
    h // (heads // kv_heads) (Section 2, background on GQA);
  * a packed ragged batch is a set of independent sequences: each is sliced out
    and handled on its own, block ids are local to the sequence.

Inputs are numpy float32 arrays that hold exactly the workload dtype's values.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "stream_oracle.c")
_LIB = os.path.join(_HERE, "libstream_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, OpenMP over independent rows only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        fp = ctypes.POINTER(ctypes.c_float)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int)
        up = ctypes.POINTER(ctypes.c_ubyte)
        lib.stream_oracle_block_score.restype = ctypes.c_double
        lib.stream_oracle_block_score.argtypes = [fp, fp, up, ctypes.c_long, ctypes.c_int,
                                                  ctypes.c_int, ctypes.c_long, ctypes.c_long]
        lib.stream_oracle_block_score_rule.restype = ctypes.c_double
        lib.stream_oracle_block_score_rule.argtypes = [fp, fp, ctypes.c_int, ctypes.c_long, ctypes.c_long,
                                                       ctypes.c_int, ctypes.c_int, ctypes.c_long, ctypes.c_long]
        lib.stream_oracle_n_it.restype = ctypes.c_long
        lib.stream_oracle_n_it.argtypes = [ctypes.c_long, ctypes.c_int]
        lib.stream_oracle_prune_head.restype = ctypes.c_int
        lib.stream_oracle_prune_head.argtypes = [fp, fp, up, ctypes.c_long, ctypes.c_int,
                                                 ctypes.c_int, ctypes.c_int, ctypes.c_int, ip,
                                                 ctypes.c_int, ip, ip, dp, ip,
                                                 ctypes.POINTER(ctypes.c_longlong)]
        lib.stream_oracle_prune_head_rule.restype = ctypes.c_int
        lib.stream_oracle_prune_head_rule.argtypes = [fp, fp, up, ctypes.c_int, ctypes.c_long,
                                                      ctypes.c_long, ctypes.c_int,
                                                      ctypes.c_int, ctypes.c_int, ctypes.c_int, ip,
                                                      ctypes.c_int, ip, ip, dp, ip,
                                                      ctypes.POINTER(ctypes.c_longlong)]
        lib.stream_oracle_attn_head_rule.restype = ctypes.c_int
        lib.stream_oracle_attn_head_rule.argtypes = [fp, fp, fp, ctypes.c_int, ctypes.c_long,
                                                     ctypes.c_long, ctypes.c_int,
                                                     ctypes.c_int, ctypes.c_int, ctypes.c_double, ip,
                                                     ctypes.c_int, ip, ip, dp, dp, dp]
        lib.stream_oracle_prune_head_rect.restype = ctypes.c_int
        lib.stream_oracle_prune_head_rect.argtypes = [fp, fp, up, ctypes.c_int, ctypes.c_long,
                                                      ctypes.c_long, ctypes.c_int, ctypes.c_int,
                                                      ctypes.c_int, ctypes.c_int, ctypes.c_int, ip,
                                                      ctypes.c_int, ip, ip, dp, ip,
                                                      ctypes.POINTER(ctypes.c_longlong)]
        lib.stream_oracle_attn_head_rect.restype = ctypes.c_int
        lib.stream_oracle_attn_head_rect.argtypes = [fp, fp, fp, ctypes.c_int, ctypes.c_long,
                                                     ctypes.c_long, ctypes.c_int, ctypes.c_int,
                                                     ctypes.c_int, ctypes.c_int, ctypes.c_double, ip,
                                                     ctypes.c_int, ip, ip, dp, dp, dp]
        lib.stream_oracle_attn_head_mask.restype = ctypes.c_int
        lib.stream_oracle_attn_head_mask.argtypes = [fp, fp, fp, up, ctypes.c_int, ctypes.c_long,
                                                     ctypes.c_long, ctypes.c_int, ctypes.c_int,
                                                     ctypes.c_int, ctypes.c_int, ctypes.c_double, ip,
                                                     ctypes.c_int, ip, ip, dp, dp, dp]
        lib.stream_oracle_block_score_rect.restype = ctypes.c_double
        lib.stream_oracle_block_score_rect.argtypes = [fp, fp, up, ctypes.c_int, ctypes.c_long,
                                                       ctypes.c_long, ctypes.c_int, ctypes.c_int,
                                                       ctypes.c_int, ctypes.c_long, ctypes.c_long]
        lib.stream_oracle_padded_len.restype = ctypes.c_long
        lib.stream_oracle_padded_len.argtypes = [ctypes.c_long, ctypes.c_int, ctypes.c_int]
        lib.stream_oracle_attn_head.restype = ctypes.c_int
        lib.stream_oracle_attn_head.argtypes = [fp, fp, fp, ctypes.c_long, ctypes.c_int,
                                                ctypes.c_int, ctypes.c_int, ctypes.c_double, ip,
                                                ctypes.c_int, ip, ip, dp, dp, dp]
        _lib = lib
    return _lib


MASKS = {"causal": 0, "full": 1, "sliding": 2}


def _mask_code(mask: str, window: int):
    """Rule-based masks C: "causal" (u <= t), "full" (no mask: Alg. 1), "sliding" (u <= t and
    t - u < window: sliding-window layers)."""
    if mask not in MASKS:
        raise ValueError(f"unknown mask {mask!r}")
    return MASKS[mask], int(window)


def _f32(a) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def _ptr(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct)) if a is not None else None


def threads() -> int:
    """Host threads the oracle's row loops use."""
    lib = _load()
    lib.stream_oracle_threads.restype = ctypes.c_int
    return int(lib.stream_oracle_threads())


def padded_len(T: int, block: int, block_k: Optional[int] = None) -> int:
    """T_p of the preamble of Alg. 2: T rounded up to a multiple of lcm(b_q, b_k)."""
    return int(_load().stream_oracle_padded_len(int(T), int(block), int(block_k or block)))


def n_it(T: int, block: int, block_k: Optional[int] = None) -> int:
    """n_it = ceil(log2(T_p / b_k)) (iteration count line of Alg. 2)."""
    if block_k is None or block_k == block:
        return int(_load().stream_oracle_n_it(int(T), int(block)))
    return int(_load().stream_oracle_n_it(padded_len(T, block, block_k), int(block_k)))


def block_score(Qh: np.ndarray, Kh: np.ndarray, block: int, q: int, r: int, C=None,
                mask: str = "causal", window: int = 0, block_k: Optional[int] = None) -> float:
    """Score of key block r for query block q of one head: masked max of the b_q x b_k dot
    products (block = b_q; block_k = b_k, default the same)."""
    Qh, Kh = _f32(Qh), _f32(Kh)
    if block_k is not None and block_k != block:
        kind, win = _mask_code(mask, window)
        Cc = None if C is None else np.ascontiguousarray(C, dtype=np.uint8)
        return float(_load().stream_oracle_block_score_rect(
            _ptr(Qh, ctypes.c_float), _ptr(Kh, ctypes.c_float), _ptr(Cc, ctypes.c_ubyte), kind, win,
            Qh.shape[0], Qh.shape[1], int(block), int(block_k), int(q), int(r)))
    if C is None and mask != "causal":
        kind, win = _mask_code(mask, window)
        return float(_load().stream_oracle_block_score_rule(
            _ptr(Qh, ctypes.c_float), _ptr(Kh, ctypes.c_float), kind, win, Qh.shape[0], Qh.shape[1],
            int(block), int(q), int(r)))
    Cc = None if C is None else np.ascontiguousarray(C, dtype=np.uint8)
    return float(_load().stream_oracle_block_score(_ptr(Qh, ctypes.c_float), _ptr(Kh, ctypes.c_float),
                                                   _ptr(Cc, ctypes.c_ubyte), Qh.shape[0],
                                                   Qh.shape[1], int(block), int(q), int(r)))


def prune_head(Qh, Kh, block: int, topk: int, qblocks: Optional[Sequence[int]] = None,
               n_levels: int = -1, C=None, want_trace: bool = False, mask: str = "causal",
               window: int = 0, block_k: Optional[int] = None):
    """Algorithm 2 for one head / one sequence.  Returns dict(idx, cnt, score, trace, evals).
    The mask C is the explicit [T, T] array if given, else the rule `mask` / `window`.
    block = b_q, block_k = b_k (default the same); there are T_p / b_q query blocks."""
    Qh, Kh = _f32(Qh), _f32(Kh)
    T, d = Qh.shape
    bk = int(block_k or block)
    N = padded_len(T, block, bk) // block
    ql = np.arange(N, dtype=np.int32) if qblocks is None else np.ascontiguousarray(qblocks, dtype=np.int32)
    nq = len(ql)
    idx = np.full((nq, topk), -1, dtype=np.int32)
    cnt = np.zeros((nq,), dtype=np.int32)
    score = np.full((nq, topk), -np.inf, dtype=np.float64)
    levels = n_it(T, block, bk) if n_levels < 0 else n_levels
    trace = np.full((nq, levels, topk, 2), -1, dtype=np.int32) if want_trace else None
    evals = np.zeros(2, dtype=np.int64)
    Cc = None if C is None else np.ascontiguousarray(C, dtype=np.uint8)
    kind, win = _mask_code(mask, window)
    rc = _load().stream_oracle_prune_head_rect(
        _ptr(Qh, ctypes.c_float), _ptr(Kh, ctypes.c_float), _ptr(Cc, ctypes.c_ubyte), kind, win, T, d,
        int(block), bk, int(topk), int(n_levels), _ptr(ql, ctypes.c_int), nq,
        _ptr(idx, ctypes.c_int), _ptr(cnt, ctypes.c_int), _ptr(score, ctypes.c_double),
        _ptr(trace, ctypes.c_int), _ptr(evals, ctypes.c_longlong))
    if rc != 0:
        raise ValueError("stream_oracle_prune_head: bad arguments")
    return {"idx": idx, "cnt": cnt, "score": score, "trace": trace, "evals": evals}


def block_table(cu_seqlens: Sequence[int], block: int, block_k: Optional[int] = None):
    """(sequence id, local block id) of every global query block of a packed batch (T_p / b_q
    query blocks per sequence, T_p the sequence's padded length)."""
    seq, loc = [], []
    for s in range(len(cu_seqlens) - 1):
        L = cu_seqlens[s + 1] - cu_seqlens[s]
        nb = (L + block - 1) // block if not block_k or block_k == block else padded_len(L, block, block_k) // block
        seq += [s] * nb
        loc += list(range(nb))
    return np.asarray(seq, dtype=np.int64), np.asarray(loc, dtype=np.int64)


def prune(Q, K, heads: int, kv_heads: int, block: int, topk, cu_seqlens=None,
          rows: Optional[Sequence[Sequence[int]]] = None, n_levels: int = -1,
          want_trace: bool = False, mask: str = "causal", window: int = 0,
          block_k: Optional[int] = None, C=None):
    """Stream for every (head, query block), or for the listed rows only.  C: explicit [T, T]
    mask shared by all heads (single sequence only), else the rule `mask` / `window`.

    Q [heads, T, d], K [kv_heads, T, d]; topk is an int or one int per sequence.
    rows: optional list of (head, global query block).  Output arrays are
    [heads, NB, kmax] (full) or [len(rows), kmax] (rows), block ids sequence-local.
    """
    Q, K = _f32(Q), _f32(K)
    H, T, d = Q.shape
    g = heads // kv_heads
    cu = [0, T] if cu_seqlens is None else [int(x) for x in cu_seqlens]
    nseq = len(cu) - 1
    ks = [int(topk)] * nseq if np.isscalar(topk) else [int(x) for x in topk]
    kmax = max(ks)
    bseq, bloc = block_table(cu, block, block_k)
    NB = len(bseq)
    blk_off = np.concatenate([[0], np.cumsum(np.bincount(bseq, minlength=nseq))])
    if rows is None:
        rows_arr = np.asarray([(h, gb) for h in range(H) for gb in range(NB)], dtype=np.int64)
        full = True
    else:
        rows_arr = np.asarray(rows, dtype=np.int64).reshape(-1, 2)
        full = False
    R = len(rows_arr)
    idx = np.full((R, kmax), -1, dtype=np.int32)
    cnt = np.zeros((R,), dtype=np.int32)
    score = np.full((R, kmax), -np.inf, dtype=np.float64)
    traces = [None] * R
    evals = np.zeros(2, dtype=np.int64)
    hs, ss = rows_arr[:, 0], bseq[rows_arr[:, 1]]
    for h in np.unique(hs):
        for s in np.unique(ss[hs == h]):
            sel = np.nonzero((hs == h) & (ss == s))[0]
            ql = bloc[rows_arr[sel, 1]].astype(np.int32)
            Qh = Q[h, cu[s]:cu[s + 1]]
            Kh = K[h // g, cu[s]:cu[s + 1]]
            if C is not None and nseq != 1:
                raise ValueError("an explicit mask is taken for a single sequence only")
            out = prune_head(Qh, Kh, block, ks[s], ql, n_levels=n_levels, want_trace=want_trace,
                             mask=mask, window=window, block_k=block_k, C=C)
            idx[sel, :ks[s]] = out["idx"]
            cnt[sel] = out["cnt"]
            score[sel, :ks[s]] = out["score"]
            evals += out["evals"]
            if want_trace:
                for a, r in enumerate(sel):
                    traces[r] = out["trace"][a]
    if full:
        idx = idx.reshape(H, NB, kmax)
        cnt = cnt.reshape(H, NB)
        score = score.reshape(H, NB, kmax)
    return {"idx": idx, "cnt": cnt, "score": score, "trace": traces if want_trace else None,
            "evals": evals, "rows": rows_arr, "blk_off": blk_off}


def variable_k(valid: int, keep_num: int, keep_den: int, topk_min: int, topk_max: int) -> int:
    """Sparsity constant of a row that keeps a fixed share of its valid key blocks.  The paper
    names a variable k as the remedy for the harder pruning of the bottom rows of a causal
    pattern (Section 4.2.1, Discussion; Section 6 (4)) without defining one; this is the rule the
    library implements: ceil(valid * keep_num / keep_den), clamped to [topk_min, topk_max]."""
    k = -((-valid * keep_num) // keep_den)
    return min(topk_max, max(topk_min, k))


def valid_blocks(q: int, N: int, block: int, mask: str = "causal", window: int = 0,
                 block_k: Optional[int] = None, L: Optional[int] = None, C=None) -> int:
    """Number of key blocks the mask C leaves to query block q: blocks with at least one real key
    that one real query of the block sees (C^blk of the preamble of Alg. 2).

    Square blocks under a rule: N = blocks of the sequence.  With b_q != b_k (block_k) pass the
    sequence length L; with an explicit [T, T] array C the count is read off the array (L = T)."""
    bk = int(block_k or block)
    if C is not None:
        C = np.asarray(C) != 0
        T = C.shape[0]
        Tp = padded_len(T, block, bk)
        rows = C[q * block:min((q + 1) * block, T)]              # the block's real queries
        if rows.shape[0] == 0:
            return 0
        cols = np.zeros((Tp,), dtype=bool)
        cols[:T] = rows.any(axis=0)                                # keys some query of the block sees
        return int(cols.reshape(Tp // bk, bk).any(axis=1).sum())
    if bk == block and L is None:
        if mask == "full":
            return N
        rmin = 0
        if mask == "sliding":
            lo = q * block - window + 1
            rmin = lo // block if lo > 0 else 0
        return q - rmin + 1
    if L is None:
        raise ValueError("b_q != b_k needs the sequence length L")
    t_first = q * block
    if t_first >= L:
        return 0                                                   # a query block of padding only
    t_last = min((q + 1) * block, L) - 1
    if mask == "full":
        return (L - 1) // bk + 1
    u_lo = max(0, t_first - window + 1) if mask == "sliding" else 0   # lowest key any query of the block sees
    return t_last // bk - u_lo // bk + 1


def prune_variable(Q, K, heads: int, kv_heads: int, block: int, keep_num: int, keep_den: int,
                   topk_min: int, topk_max: int, cu_seqlens=None,
                   rows: Optional[Sequence[Sequence[int]]] = None, mask: str = "causal", window: int = 0,
                   block_k: Optional[int] = None, C=None):
    """Algorithm 2 run row by row with k(row) = variable_k(valid(row), ...), valid(row) counted
    under the mask the row is pruned with (rule, rectangular blocks, or an explicit [T, T] array C
    for a single sequence).  Output arrays as prune(): [heads, NB, topk_max] (full) or
    [len(rows), topk_max]; also "k" per row."""
    Q, K = _f32(Q), _f32(K)
    H, T, d = Q.shape
    g = heads // kv_heads
    cu = [0, T] if cu_seqlens is None else [int(x) for x in cu_seqlens]
    if C is not None and len(cu) != 2:
        raise ValueError("an explicit mask is taken for a single sequence only")
    bseq, bloc = block_table(cu, block, block_k)
    NB = len(bseq)
    full = rows is None
    rows_arr = (np.asarray([(h, gb) for h in range(H) for gb in range(NB)], dtype=np.int64) if full
                else np.asarray(rows, dtype=np.int64).reshape(-1, 2))
    R = len(rows_arr)
    idx = np.full((R, topk_max), -1, dtype=np.int32)
    cnt = np.zeros((R,), dtype=np.int32)
    score = np.full((R, topk_max), -np.inf, dtype=np.float64)
    ks = np.zeros((R,), dtype=np.int32)
    valid_of = {}
    for i, (h, gb) in enumerate(rows_arr):
        s, q = int(bseq[gb]), int(bloc[gb])
        L = cu[s + 1] - cu[s]
        if (s, q) not in valid_of:
            if C is not None:
                valid_of[(s, q)] = valid_blocks(q, 0, block, block_k=block_k, C=C)
            elif block_k is not None and block_k != block:
                valid_of[(s, q)] = valid_blocks(q, 0, block, mask, window, block_k=block_k, L=L)
            else:
                valid_of[(s, q)] = valid_blocks(q, -(-L // block), block, mask, window)
        k = variable_k(valid_of[(s, q)], keep_num, keep_den, topk_min, topk_max)
        out = prune_head(Q[h, cu[s]:cu[s + 1]], K[h // g, cu[s]:cu[s + 1]], block, k, [q], mask=mask,
                         window=window, block_k=block_k, C=C)
        idx[i, :k] = out["idx"][0]
        cnt[i] = out["cnt"][0]
        score[i, :k] = out["score"][0]
        ks[i] = k
    if full:
        idx, cnt, score, ks = idx.reshape(H, NB, topk_max), cnt.reshape(H, NB), score.reshape(H, NB, topk_max), ks.reshape(H, NB)
    return {"idx": idx, "cnt": cnt, "score": score, "k": ks, "rows": rows_arr}


def sparse_attn(Q, K, V, heads: int, kv_heads: int, block: int, idx, cnt, scale: float,
                cu_seqlens=None, rows: Optional[Sequence[Sequence[int]]] = None,
                want_mass: bool = True, mask: str = "causal", window: int = 0,
                block_k: Optional[int] = None, C=None):
    """Eq. (2) over the retained blocks given by idx/cnt (query blocks of `block` tokens, key
    blocks of `block_k` tokens, default the same).  The mask C inside the retained blocks is the
    explicit [T, T] array C (single sequence only) if given, else the rule `mask` / `window`.

    idx/cnt are [heads, NB, kmax]/[heads, NB] (full) or aligned with `rows`.
    Returns dict(O [heads, T, d], lse [heads, T], mass [heads, T]) in fp64; with `rows`,
    only the tokens of the listed query blocks are written in O / lse, and mass holds
    the contribution of those rows only.
    """
    Q, K, V = _f32(Q), _f32(K), _f32(V)
    H, T, d = Q.shape
    g = heads // kv_heads
    cu = [0, T] if cu_seqlens is None else [int(x) for x in cu_seqlens]
    bseq, bloc = block_table(cu, block, block_k)
    NB = len(bseq)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    cnt = np.ascontiguousarray(cnt, dtype=np.int32)
    kmax = idx.shape[-1]
    if rows is None:
        rows_arr = np.asarray([(h, gb) for h in range(H) for gb in range(NB)], dtype=np.int64)
        idx2, cnt2 = idx.reshape(H * NB, kmax), cnt.reshape(H * NB)
    else:
        rows_arr = np.asarray(rows, dtype=np.int64).reshape(-1, 2)
        idx2, cnt2 = idx.reshape(len(rows_arr), kmax), cnt.reshape(len(rows_arr))
    O = np.zeros((H, T, d), dtype=np.float64)
    lse = np.full((H, T), np.nan, dtype=np.float64)
    mass = np.zeros((H, T), dtype=np.float64)
    hs, ss = rows_arr[:, 0], bseq[rows_arr[:, 1]]
    lib = _load()
    for h in np.unique(hs):
        for s in np.unique(ss[hs == h]):
            sel = np.nonzero((hs == h) & (ss == s))[0]
            ql = bloc[rows_arr[sel, 1]].astype(np.int32)
            a, b_ = cu[s], cu[s + 1]
            Qh, Kh, Vh = (np.ascontiguousarray(Q[h, a:b_]), np.ascontiguousarray(K[h // g, a:b_]),
                          np.ascontiguousarray(V[h // g, a:b_]))
            Oh = np.zeros((b_ - a, d), dtype=np.float64)
            lh = np.full((b_ - a,), np.nan, dtype=np.float64)
            mh = np.zeros((b_ - a,), dtype=np.float64)
            i2 = np.ascontiguousarray(idx2[sel])
            c2 = np.ascontiguousarray(cnt2[sel])
            kind, win = _mask_code(mask, window)
            Cc = None if C is None else np.ascontiguousarray(C, dtype=np.uint8)
            if Cc is not None and len(cu) != 2:
                raise ValueError("an explicit mask is taken for a single sequence only")
            rc = lib.stream_oracle_attn_head_mask(
                _ptr(Qh, ctypes.c_float), _ptr(Kh, ctypes.c_float), _ptr(Vh, ctypes.c_float),
                _ptr(Cc, ctypes.c_ubyte), kind, win, b_ - a, d, int(block), int(block_k or block), kmax, float(scale),
                _ptr(ql, ctypes.c_int), len(ql),
                _ptr(i2, ctypes.c_int), _ptr(c2, ctypes.c_int), _ptr(Oh, ctypes.c_double),
                _ptr(lh, ctypes.c_double), _ptr(mh if want_mass else None, ctypes.c_double))
            if rc != 0:
                raise ValueError("stream_oracle_attn_head: bad arguments")
            for qb in ql:
                t0, t1 = min(qb * block, b_ - a), min((qb + 1) * block, b_ - a)
                O[h, a + t0:a + t1] = Oh[t0:t1]
                lse[h, a + t0:a + t1] = lh[t0:t1]
            mass[h, a:b_] += mh
    return {"O": O, "lse": lse, "mass": mass}
