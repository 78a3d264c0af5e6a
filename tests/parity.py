"""Comparison rule GPU <-> oracle for the pruning path.

Index lists must be equal.  Where a row differs, the row is replayed level by level along the
GPU's own choices (its per-level node trace) with the oracle's fp64 block scores, and accepted
only if every level is a correct top-k up to a relative score gap of 1e-3 (fp32 accumulation
on the GPU): the kept branches are children of the previous level's nodes, as many as the
listing keeps, and no dropped valid branch beats a kept one by more than the tolerance.
"""
from __future__ import annotations

import math

import numpy as np

from oracle import stream_oracle as so

TIE_RTOL = 1e-3


def valid_range(mask, window, q, block, N, block_k=None, L=None):
    """First and last key block with a key visible to a query of block q under the mask rule
    (square blocks: N = blocks of the sequence; b_q != b_k: pass block_k and the length L)."""
    if block_k is None or block_k == block:
        rmax = N - 1 if mask == "full" else q
        rmin = 0
        if mask == "sliding":
            lo = q * block - window + 1           # first key the block's first query sees
            rmin = max(0, lo // block) if lo > 0 else 0
        return rmin, rmax
    if q * block >= L:
        return 0, -1                              # a query block of padding only
    last_q = min(L, (q + 1) * block) - 1
    rmax = (L - 1) // block_k if mask == "full" else last_q // block_k
    rmin = 0
    if mask == "sliding":
        lo = q * block - window + 1
        rmin = lo // block_k if lo > 0 else 0
    return rmin, rmax


def certify_row(Qh, Kh, block, k, q, trace_row, mask="causal", window=0, block_k=None, C=None):
    """trace_row: int array [levels, k, 2] of (f, l) kept after each GPU level (-1 = dead).
    C: explicit [T, T] mask (then `mask` / `window` are not looked at).  Returns (ok, reason)."""
    T = Qh.shape[0]
    bk = block_k or block
    N = so.padded_len(T, block, bk) // bk     # key blocks: the nodes range over these
    if C is None:
        rmin, rmax = valid_range(mask, window, q, block, N, block_k, T)
        def rep(f, l):                        # a branch's representative: its first valid block, or None
            r = max(f, rmin)
            return r if f <= l and r <= min(l, rmax) else None
    else:
        Cb = np.asarray(C) != 0
        rows = Cb[q * block:min((q + 1) * block, T)]
        cols = np.zeros((N * bk,), dtype=bool)
        if rows.shape[0]:
            cols[:T] = rows.any(axis=0)
        vblk = cols.reshape(N, bk).any(axis=1)    # C^blk[q, :]
        def rep(f, l):
            if f > l:
                return None
            hit = np.nonzero(vblk[f:l + 1])[0]
            return f + int(hit[0]) if len(hit) else None
    score = lambda r: so.block_score(Qh, Kh, block, q, r, C=C, mask=mask, window=window, block_k=block_k)
    nodes = [((j * N) // k, ((j + 1) * N) // k - 1) for j in range(k)]
    nodes = [(f, l) for (f, l) in nodes if f <= l]
    for lv in range(trace_row.shape[0]):
        children = []
        for (f, l) in nodes:
            m = (f + l + 1) // 2
            for (cf, cl) in ((f, m - 1), (m, l)):
                if rep(cf, cl) is not None:
                    children.append((cf, cl))
        kept = [(int(f), int(l)) for f, l in trace_row[lv] if f >= 0]
        if len(set(kept)) != len(kept) or kept != sorted(kept):
            return False, f"level {lv}: kept nodes not distinct/ascending"
        if not set(kept) <= set(children):
            return False, f"level {lv}: kept a branch that is not a valid child"
        if len(kept) != min(k, len(children)):
            return False, f"level {lv}: kept {len(kept)} of {len(children)} valid, k={k}"
        dropped = [c for c in children if c not in set(kept)]
        if dropped:
            s_keep = min(score(rep(f, l)) for f, l in kept)
            s_drop = max(score(rep(f, l)) for f, l in dropped)
            if s_keep < s_drop - TIE_RTOL * max(abs(s_drop), abs(s_keep)):
                return False, f"level {lv}: dropped {s_drop} > kept {s_keep}"
        nodes = kept
    if any(f != l for f, l in nodes):
        return False, "final nodes are not single blocks"
    return True, ""


def compare_variable(gpu, ref, Q, K, heads, kv_heads, block, kmax, cu_seqlens=None, mask="causal",
                     window=0, block_k=None, C=None):
    """stream_prune_variable against oracle.prune_variable.  gpu: numpy idx [H, NB, kmax], cnt,
    score (optional), trace [levels, H, NB, kmax, 2] (needed only if a row differs); ref: the
    oracle's output (all rows, or the rows it lists).  Counts must be equal, lists equal or
    certified level by level as in compare_prune.  Returns dict(rows, equal, tie_rows)."""
    g = heads // kv_heads
    T = Q.shape[1]
    cu = [0, T] if cu_seqlens is None else [int(x) for x in cu_seqlens]
    bseq, bloc = so.block_table(cu, block, block_k)
    ri = ref["idx"].reshape(-1, kmax)
    rc = ref["cnt"].reshape(-1)
    rs = ref["score"].reshape(-1, kmax)
    rk = ref["k"].reshape(-1)
    equal = ties = 0
    for i, (h, gb) in enumerate(ref["rows"]):
        gi, gc = gpu["idx"][h, gb], int(gpu["cnt"][h, gb])
        assert gc == int(rc[i]), (h, gb, gc, int(rc[i]))
        assert (gi[gc:] == -1).all(), (h, gb)
        if np.array_equal(gi, ri[i]):
            equal += 1
            if gpu.get("score") is not None and gc:
                np.testing.assert_allclose(gpu["score"][h, gb, :gc], rs[i, :gc], rtol=1e-4,
                                           atol=1e-4 * float(np.abs(rs[i, :gc]).max()))
            continue
        assert gpu.get("trace") is not None, f"row {(h, gb)} differs and no trace was taken"
        s, q = int(bseq[gb]), int(bloc[gb])
        k = int(rk[i])
        Qh, Kh = Q[h, cu[s]:cu[s + 1]], K[h // g, cu[s]:cu[s + 1]]
        n_key = so.padded_len(Qh.shape[0], block, block_k) // (block_k or block)
        n_eff = max(1, math.ceil(math.log2(math.ceil(n_key / k))))
        tr = gpu["trace"][:n_eff, h, gb, :k]
        ok, why = certify_row(Qh, Kh, block, k, q, tr, mask=mask, window=window, block_k=block_k, C=C)
        assert ok, f"row (h={h}, block={gb}, k={k}): {why}; gpu={gi[:gc]} oracle={ri[i][:gc]}"
        assert list(tr[-1][:gc, 0]) == list(gi[:gc])
        ties += 1
    return {"rows": len(ref["rows"]), "equal": equal, "tie_rows": ties}


def compare_prune(gpu, ref, Q, K, heads, kv_heads, block, topk, cu_seqlens=None, rows=None,
                  mask="causal", window=0, block_k=None):
    """gpu: dict of numpy arrays idx [H,NB,kmax], cnt [H,NB], optional score, trace
    [levels,H,NB,kmax,2].  ref: output of so.prune(...) for the same rows (or all).
    Q, K: numpy float32 (exact input values).  Returns dict with counts; raises on failure."""
    H = heads
    g = heads // kv_heads
    T = Q.shape[1]
    cu = [0, T] if cu_seqlens is None else [int(x) for x in cu_seqlens]
    nseq = len(cu) - 1
    ks = [int(topk)] * nseq if np.isscalar(topk) else [int(x) for x in topk]
    bseq, bloc = so.block_table(cu, block, block_k)
    NB = len(bseq)
    if rows is None:
        rows_arr = np.asarray([(h, gb) for h in range(H) for gb in range(NB)], dtype=np.int64)
        ridx = ref["idx"].reshape(H * NB, -1)
        rcnt = ref["cnt"].reshape(H * NB)
        rscore = ref["score"].reshape(H * NB, -1)
    else:
        rows_arr = np.asarray(rows, dtype=np.int64).reshape(-1, 2)
        ridx, rcnt, rscore = ref["idx"], ref["cnt"], ref["score"]
    equal = ties = 0
    for i, (h, gb) in enumerate(rows_arr):
        s, q = int(bseq[gb]), int(bloc[gb])
        k = ks[s]
        gi, gc = gpu["idx"][h, gb], int(gpu["cnt"][h, gb])
        Ns = -(-(cu[s + 1] - cu[s]) // block)
        rmin, rmax = valid_range(mask, window, q, block, Ns, block_k, cu[s + 1] - cu[s])
        assert gc == int(rcnt[i]) == min(k, max(0, rmax - rmin + 1)), (h, gb, gc, int(rcnt[i]))
        assert np.all(gi[gc:] == -1), (h, gb)
        assert np.all(np.diff(gi[:gc]) > 0) and (gc == 0 or (gi[0] >= rmin and gi[gc - 1] <= rmax)), (h, gb)
        Qh = Q[h, cu[s]:cu[s + 1]]
        Kh = K[h // g, cu[s]:cu[s + 1]]
        if np.array_equal(gi, ridx[i]):
            equal += 1
            if gpu.get("score") is not None:
                gs = gpu["score"][h, gb]
                if gc:
                    np.testing.assert_allclose(gs[:gc], rscore[i, :gc], rtol=1e-4,
                                               atol=1e-4 * float(np.abs(rscore[i, :gc]).max()))
                assert np.all(np.isneginf(gs[gc:]))
        else:
            assert gpu.get("trace") is not None, f"row {(h, gb)} differs and no trace was taken"
            tr = gpu["trace"][:, h, gb, :k, :]
            n_key = so.padded_len(Qh.shape[0], block, block_k) // (block_k or block)
            n_eff = max(1, math.ceil(math.log2(math.ceil(n_key / k))))
            tr = tr[:n_eff]
            ok, why = certify_row(Qh, Kh, block, k, q, tr, mask=mask, window=window, block_k=block_k)
            assert ok, f"row (h={h}, block={gb}): {why}; gpu={gi[:gc]} oracle={ridx[i][:gc]}"
            assert list(tr[-1][:gc, 0]) == list(gi[:gc])
            ties += 1
    return {"rows": len(rows_arr), "equal": equal, "tie_rows": ties}


def sample_rows(w, n, seed=0, heads=None):
    """Seeded sample of (head, global block) rows that always holds the edge rows of every sequence."""
    rng = np.random.default_rng(seed)
    heads = list(range(w.heads)) if heads is None else list(heads)
    rows = set()
    off = 0
    for s, nb in enumerate(w.blocks_per_seq):
        k = w.topk[s]
        for q in {0, 1, k - 1, k, nb // 2, nb - 1}:
            if 0 <= q < nb:
                rows.add((heads[int(rng.integers(len(heads)))], off + q))
        off += nb
    NB = off
    n = min(n, len(heads) * NB)
    while len(rows) < n:
        rows.add((heads[int(rng.integers(len(heads)))], int(rng.integers(NB))))
    return sorted(rows)


def kurtosis_gradient(x):
    """d kurt / d x_i of the excess kurtosis m4 / m2^2 - 3 (biased central moments) of the values
    x: (4 / n) * ((c_i^3 - m3) / m2^2 - m4 * c_i / m2^3), c = x - mean.  Used to turn the error of
    the block means into the error their column kurtosis may show (first order)."""
    x = np.asarray(x, dtype=np.float64)
    n = x.size
    c = x - x.mean()
    m2, m3, m4 = np.mean(c * c), np.mean(c ** 3), np.mean(c ** 4)
    return (4.0 / n) * ((c ** 3 - m3) / (m2 * m2) - m4 * c / (m2 ** 3))


def kurtosis_tolerance(x_ref, x_got, kurt_ref):
    """How far the kurtosis of x_got may lie from that of x_ref given how far the values
    themselves lie apart: twice the first-order bound sum_i |d kurt / d x_i| * |x_got_i - x_ref_i|
    (the factor covers the second-order terms while the deviations stay small) plus the rounding of
    an fp32 result."""
    g = kurtosis_gradient(x_ref)
    return 2.0 * float(np.sum(np.abs(g) * np.abs(np.asarray(x_got, np.float64) - np.asarray(x_ref, np.float64)))) + \
        2e-5 * (1.0 + abs(kurt_ref))
