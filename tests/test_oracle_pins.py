"""Pins for the CPU oracle (no GPU): what the paper and the mathematics fix.

Each test states which plausible mistake it would catch.  The oracle under test is
oracle/stream_oracle.c (through oracle/stream_oracle.py); the yardsticks are
oracle/bruteforce.py (dense T x T scores), closed forms, and hand-traced cases in
tests/golden/alg2_hand_trace.txt.
"""
import math
import os

import numpy as np
import pytest

from oracle import bruteforce as bf
from oracle import stream_oracle as so

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "alg2_hand_trace.txt")


def lists(idx, cnt):
    return [list(map(int, idx[q, :cnt[q]])) for q in range(idx.shape[0])]


def gauss(rng, T, d):
    return rng.standard_normal((T, d)).astype(np.float32)


def small_ints(rng, T, d):
    # exactly representable, many equal scores -> exercises tie-breaking with exact arithmetic
    return rng.integers(-2, 3, size=(T, d)).astype(np.float32)


# ---------------------------------------------------------------- P8: hand-traced cases
def golden_cases():
    out = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, N, k, q, scores, exp = [x.strip() for x in line.split("|")]
        out.append((name, int(N), int(k), int(q), [float(x) for x in scores.split()],
                    [int(x) for x in exp.split()]))
    return out


@pytest.mark.parametrize("case", golden_cases(), ids=lambda c: c[0])
def test_hand_traced_example(case):
    """A wrong midpoint, a 1-based j, 'best block in range' scoring, exact top-k, or ties
    resolved to the higher position all change these results."""
    name, N, k, q, A, expect = case
    b, d = 2, 4
    T = N * b
    Q = np.zeros((T, d), np.float32)
    K = np.zeros((T, d), np.float32)
    Q[:, 0] = -0.5          # other query tokens only produce negative products
    Q[q * b, 0] = 1.0       # the token of block q that realises the block score
    for r in range(N):
        K[r * b, 0] = A[r]
        K[r * b + 1, 0] = A[r] - 0.5
    out = so.prune_head(Q, K, b, k, qblocks=[q])
    assert lists(out["idx"], out["cnt"])[0] == expect
    # the reported block scores are the planted ones
    np.testing.assert_allclose(out["score"][0, :len(expect)], [A[r] for r in expect])


# ---------------------------------------------------------------- P1: brute force
@pytest.mark.parametrize("maker", [gauss, small_ints], ids=["gauss", "ints"])
def test_matches_bruteforce_all_small_shapes(maker):
    """Dense scores -> max-pool -> recursion by table look-up, in separate Python code.
    Catches index slips in the block views, the padding, validity, representative and
    selection (incl. k not dividing N and T not a multiple of b)."""
    rng = np.random.default_rng(1)
    b, d = 3, 5
    checked = 0
    for N in list(range(1, 18)) + [23, 32]:
        for k in sorted({1, 2, 3, 5, 8, N, N + 2}):
            for tail in (0, 1):
                T = N * b - tail * (b - 1)  # last block holds a single real token when tail=1
                if T <= 0:
                    continue
                Q, K = maker(rng, T, d), maker(rng, T, d)
                out = so.prune_head(Q, K, b, k)
                A, Cblk = bf.block_score_table(Q, K, b)
                ref = bf.stream_from_table(A, Cblk, k)
                got = lists(out["idx"], out["cnt"])
                assert got == ref, (N, k, T)
                for q, lst in enumerate(ref):
                    np.testing.assert_allclose(out["score"][q, :len(lst)], A[q, lst], rtol=1e-12)
                checked += 1
    assert checked > 200


def test_explicit_mask_equals_causal_predicate_and_general_masks():
    """The causal closed form for C^blk / first valid block must equal the listing's generic
    max over an explicit C; and a non-causal C (random, banded) goes through the same code."""
    rng = np.random.default_rng(2)
    b, d = 4, 6
    for N, k in [(8, 2), (13, 3), (16, 4)]:
        T = N * b - 2
        Q, K = gauss(rng, T, d), gauss(rng, T, d)
        C = bf.causal_mask(T)
        a = so.prune_head(Q, K, b, k)
        e = so.prune_head(Q, K, b, k, C=C)
        assert np.array_equal(a["idx"], e["idx"]) and np.array_equal(a["cnt"], e["cnt"])
        band = np.triu(C, -3 * b)  # sliding window
        rnd = (rng.random((T, T)) < 0.05).astype(np.uint8) * C
        for Cm in (band, rnd):
            o = so.prune_head(Q, K, b, k, C=Cm)
            A, Cblk = bf.block_score_table(Q, K, b, Cm)
            assert lists(o["idx"], o["cnt"]) == bf.stream_from_table(A, Cblk, k)


# ---------------------------------------------------------------- P2: exact top-k regime
def test_equals_exact_block_topk_when_every_block_is_scored():
    """N <= 2k: level 1 scores every block, so the heuristic is exact.  Catches a score that is
    not the masked b x b maximum (e.g. mean, unmasked max, transposed operand)."""
    rng = np.random.default_rng(3)
    b, d = 4, 8
    for N, k in [(8, 4), (8, 5), (6, 3), (16, 8), (10, 7), (5, 9)]:
        T = N * b
        Q, K = gauss(rng, T, d), gauss(rng, T, d)
        out = so.prune_head(Q, K, b, k)
        A, Cblk = bf.block_score_table(Q, K, b)
        assert lists(out["idx"], out["cnt"]) == bf.exact_block_topk(A, Cblk, k)


# ---------------------------------------------------------------- P3: count law
def test_count_law_and_canonical_form():
    rng = np.random.default_rng(4)
    b, d = 2, 4
    for N, k in [(64, 8), (50, 7), (33, 4), (9, 16)]:
        T = N * b
        out = so.prune_head(gauss(rng, T, d), gauss(rng, T, d), b, k)
        q = np.arange(N)
        assert np.array_equal(out["cnt"], np.minimum(k, q + 1))
        kk = min(k, N)
        assert out["cnt"].sum() == kk * N - kk * (kk - 1) // 2
        for row, c in zip(out["idx"], out["cnt"]):
            assert np.all(np.diff(row[:c]) > 0) and np.all(row[c:] == -1) and np.all(row[:c] >= 0)


# ---------------------------------------------------------------- P4: causality
def test_no_future_block_and_future_tokens_do_not_matter():
    rng = np.random.default_rng(5)
    b, d, N, k = 4, 8, 24, 3
    T = N * b
    Q, K = gauss(rng, T, d), gauss(rng, T, d)
    base = so.prune_head(Q, K, b, k)
    for q in range(N):
        assert np.all(base["idx"][q, :base["cnt"][q]] <= q)
    cut = 10
    Q2, K2 = Q.copy(), K.copy()
    K2[(cut + 1) * b:] = 100.0 * gauss(rng, T - (cut + 1) * b, d)
    Q2[(cut + 1) * b:] = 100.0 * gauss(rng, T - (cut + 1) * b, d)
    pert = so.prune_head(Q2, K2, b, k)
    assert np.array_equal(base["idx"][:cut + 1], pert["idx"][:cut + 1])
    # inside the diagonal block the token-level mask matters: a huge key at the last token of
    # block q is visible only to the last query token of that block
    K3 = K.copy()
    K3[cut * b + b - 1] = 0.0
    s_masked = so.block_score(Q, K3, b, cut, cut)
    A, _ = bf.block_score_table(Q, K3, b)
    assert s_masked == pytest.approx(A[cut, cut], rel=1e-12)


# ---------------------------------------------------------------- P5 (mask part) and P10
def test_topk_at_least_n_blocks_gives_full_causal_mask():
    rng = np.random.default_rng(6)
    b, d, N = 4, 8, 11
    T = N * b - 1
    Q, K = gauss(rng, T, d), gauss(rng, T, d)
    for k in (N, N + 1, 2 * N + 3):
        out = so.prune_head(Q, K, b, k)
        assert lists(out["idx"], out["cnt"]) == [list(range(q + 1)) for q in range(N)]


def test_levels_beyond_n_eff_are_no_ops():
    """n_it as printed, the productive depth ceil(log2(ceil(N/k))), and extra levels agree."""
    rng = np.random.default_rng(7)
    b, d = 2, 6
    for N, k in [(64, 4), (37, 5), (20, 3), (16, 16), (7, 2)]:
        T = N * b
        Q, K = gauss(rng, T, d), gauss(rng, T, d)
        n_eff = math.ceil(math.log2(math.ceil(N / k))) if N > k else 0
        ref = so.prune_head(Q, K, b, k)
        assert so.n_it(T, b) == (math.ceil(math.log2(N)) if N > 1 else 0)
        for lv in (n_eff, so.n_it(T, b) + 3):
            o = so.prune_head(Q, K, b, k, n_levels=lv)
            assert np.array_equal(o["idx"], ref["idx"]), (N, k, lv)
        if n_eff >= 1 and N > 2 * k:
            o = so.prune_head(Q, K, b, k, n_levels=n_eff - 1)
            assert not np.array_equal(o["idx"], ref["idx"])  # one level short is not enough


# ---------------------------------------------------------------- P6: monotone closed forms
def test_monotone_scores_closed_forms():
    """Scores decreasing in key position keep the first min(k, q+1) blocks, increasing ones keep
    the sliding window q-k+1..q.  Catches a reversed comparison or a wrong representative."""
    b, N = 2, 32
    T = N * b
    t = np.arange(T, dtype=np.float32)
    Q = np.stack([np.ones(T), np.zeros(T)], 1).astype(np.float32)
    for k in (1, 3, 4, 8):
        Kdec = np.stack([-t, np.zeros(T)], 1).astype(np.float32)
        Kinc = np.stack([t, np.zeros(T)], 1).astype(np.float32)
        dec = so.prune_head(Q, Kdec, b, k)
        inc = so.prune_head(Q, Kinc, b, k)
        for q in range(N):
            c = min(k, q + 1)
            assert list(dec["idx"][q, :c]) == list(range(c))
            if (N // k) * k == N and k <= N:
                assert list(inc["idx"][q, :c]) == list(range(q - c + 1, q + 1)), (k, q)


# ---------------------------------------------------------------- P7: invariances
def test_scale_gqa_and_head_permutation_invariance():
    rng = np.random.default_rng(8)
    b, d, N, k, H, Hkv = 4, 8, 16, 3, 4, 2
    T = N * b
    Q = rng.standard_normal((H, T, d)).astype(np.float32)
    K = rng.standard_normal((Hkv, T, d)).astype(np.float32)
    base = so.prune(Q, K, H, Hkv, b, k)
    assert np.array_equal(so.prune(4.0 * Q, K, H, Hkv, b, k)["idx"], base["idx"])
    assert np.array_equal(so.prune(Q, 0.25 * K, H, Hkv, b, k)["idx"], base["idx"])
    Krep = np.repeat(K, H // Hkv, axis=0)
    assert np.array_equal(so.prune(Q, Krep, H, H, b, k)["idx"], base["idx"])
    perm = np.array([1, 0, 3, 2])  # stays inside each group
    assert np.array_equal(so.prune(Q[perm], K, H, Hkv, b, k)["idx"], base["idx"][perm])
    # the second group really reads the second key head
    K2 = K.copy()
    K2[1] = rng.standard_normal((T, d)).astype(np.float32)
    o2 = so.prune(Q, K2, H, Hkv, b, k)
    assert np.array_equal(o2["idx"][:2], base["idx"][:2]) and not np.array_equal(o2["idx"][2:], base["idx"][2:])


def test_rows_subset_and_ragged_batch_equal_separate_sequences():
    rng = np.random.default_rng(9)
    b, d, H, Hkv = 4, 8, 2, 1
    lens = [37, 64, 9]
    ks = [3, 2, 1]
    cu = np.concatenate([[0], np.cumsum(lens)])
    T = int(cu[-1])
    Q = rng.standard_normal((H, T, d)).astype(np.float32)
    K = rng.standard_normal((Hkv, T, d)).astype(np.float32)
    packed = so.prune(Q, K, H, Hkv, b, ks, cu_seqlens=cu)
    off = 0
    for s, L in enumerate(lens):
        nb = -(-L // b)
        for h in range(H):
            one = so.prune_head(Q[h, cu[s]:cu[s + 1]], K[0, cu[s]:cu[s + 1]], b, ks[s])
            assert np.array_equal(packed["idx"][h, off:off + nb, :ks[s]], one["idx"])
            assert np.all(packed["idx"][h, off:off + nb, ks[s]:] == -1)
        off += nb
    rows = [(1, 3), (0, 0), (1, packed["idx"].shape[1] - 1)]
    sub = so.prune(Q, K, H, Hkv, b, ks, cu_seqlens=cu, rows=rows)
    for i, (h, gb) in enumerate(rows):
        assert np.array_equal(sub["idx"][i], packed["idx"][h, gb])


# ---------------------------------------------------------------- evaluation counters
def test_evaluation_counters():
    """evals[0] = finite-score branch evaluations as executed, evals[1] = those that a parent's
    score cannot supply.  With N/k a power of two the first level scores both children of every
    node; afterwards exactly one child per kept node has a new representative."""
    rng = np.random.default_rng(10)
    b, d, N, k = 2, 4, 64, 4
    T = N * b
    Q, K = gauss(rng, T, d), gauss(rng, T, d)
    q = N - 1  # every block causal
    n_eff = 4
    o = so.prune_head(Q, K, b, k, qblocks=[q], n_levels=n_eff)
    assert o["evals"][0] == 2 * k * n_eff
    assert o["evals"][1] == 2 * k + k * (n_eff - 1)
    o2 = so.prune_head(Q, K, b, k, qblocks=[q])  # n_it = 6: two no-op levels, k finite evals each
    assert o2["evals"][0] == 2 * k * n_eff + 2 * k and o2["evals"][1] == o["evals"][1]


# ---------------------------------------------------------------- attention: P5, P9
def test_attention_equals_dense_softmax_on_the_masked_pattern():
    """Eq. (2) on the retained blocks == dense softmax with the token mask M*C (numpy), for
    pruned and for full masks; lse and column sums too.  Catches a missing causal mask in the
    diagonal block, a wrong normaliser, V indexed by the wrong key."""
    rng = np.random.default_rng(11)
    b, d, N, k = 4, 8, 12, 3
    T = N * b - 2
    Q, K, V = gauss(rng, T, d), gauss(rng, T, d), gauss(rng, T, d)
    for kk in (k, N + 1):
        p = so.prune_head(Q, K, b, kk)
        o = so.sparse_attn(Q[None], K[None], V[None], 1, 1, b, p["idx"][None], p["cnt"][None], 0.3)
        M = bf.mask_from_blocks(lists(p["idx"], p["cnt"]), T, b)
        O, lse, mass = bf.dense_attention(Q, K, V, M, 0.3)
        np.testing.assert_allclose(o["O"][0], O, rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(o["lse"][0], lse, rtol=1e-12)
        np.testing.assert_allclose(o["mass"][0], mass, rtol=1e-10, atol=1e-14)
        if kk > N:
            assert np.array_equal(M, bf.causal_mask(T))


def test_full_mask_attention_equals_torch_causal_sdpa():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(12)
    b, d, N, H, Hkv = 4, 16, 8, 4, 2
    T = N * b
    Q = rng.standard_normal((H, T, d)).astype(np.float32)
    K = rng.standard_normal((Hkv, T, d)).astype(np.float32)
    V = rng.standard_normal((Hkv, T, d)).astype(np.float32)
    p = so.prune(Q, K, H, Hkv, b, N)
    o = so.sparse_attn(Q, K, V, H, Hkv, b, p["idx"], p["cnt"], 1.0 / math.sqrt(d))
    tq, tk, tv = (torch.from_numpy(x).double() for x in (Q, K, V))
    ref = torch.nn.functional.scaled_dot_product_attention(
        tq[None], tk.repeat_interleave(H // Hkv, 0)[None], tv.repeat_interleave(H // Hkv, 0)[None],
        is_causal=True)[0].numpy()
    np.testing.assert_allclose(o["O"], ref, rtol=1e-9, atol=1e-12)


def test_received_mass_invariants():
    rng = np.random.default_rng(13)
    b, d, N, k, H, Hkv = 4, 8, 16, 2, 2, 1
    T = N * b - 3
    Q = rng.standard_normal((H, T, d)).astype(np.float32)
    K = rng.standard_normal((Hkv, T, d)).astype(np.float32)
    V = rng.standard_normal((Hkv, T, d)).astype(np.float32)
    p = so.prune(Q, K, H, Hkv, b, k)
    o = so.sparse_attn(Q, K, V, H, Hkv, b, p["idx"], p["cnt"], 0.5)
    np.testing.assert_allclose(o["mass"].sum(axis=1), T, rtol=1e-12)  # every row of P sums to 1
    assert np.all(o["mass"] >= 0)
    for h in range(H):
        kept = np.zeros(N, bool)
        for q in range(N):
            kept[p["idx"][h, q, :p["cnt"][h, q]]] = True
        never = np.repeat(~kept, b)[:T]
        assert np.all(o["mass"][h, never] == 0)


def test_level_certificate_accepts_the_oracle_trace_and_rejects_planted_mistakes():
    """The checker that replays a differing GPU row level by level (tests/parity.py) is itself
    checked here on the CPU: it accepts the oracle's own per-level trace under a rule, with
    rectangular blocks and with an explicit array, and rejects a trace in which one kept branch is
    swapped for a clearly worse sibling, one with a branch too few, and one that keeps a branch
    the mask hides."""
    from tests import parity

    rng = np.random.default_rng(31)
    T, d = 4 * 37 + 2, 8
    Qh = rng.standard_normal((T, d)).astype(np.float32)
    Kh = rng.standard_normal((T, d)).astype(np.float32)
    t = np.arange(T)[:, None]
    u = np.arange(T)[None, :]
    docs = (u <= t) & ((t // 50) == (u // 50))                 # three packed documents
    cases = [dict(block=4, k=3), dict(block=4, k=3, mask="sliding", window=40),
             dict(block=4, k=2, block_k=8), dict(block=8, k=5, block_k=4, mask="full"),
             dict(block=4, k=3, C=docs), dict(block=4, k=2, block_k=8, C=docs)]
    for kw in cases:
        block, k = kw["block"], kw["k"]
        extra = {x: kw[x] for x in ("mask", "window", "block_k", "C") if x in kw}
        nq = so.padded_len(T, block, kw.get("block_k")) // block
        rejected = 0
        for q in (nq - 1, nq // 2, 1):
            r = so.prune_head(Qh, Kh, block, k, [q], want_trace=True, **extra)
            n_key = so.padded_len(T, block, kw.get("block_k")) // kw.get("block_k", block)
            n_eff = max(1, int(np.ceil(np.log2(np.ceil(n_key / k)))))
            tr = r["trace"][0][:n_eff]
            ok, why = parity.certify_row(Qh, Kh, block, k, q, tr, **extra)
            assert ok, (kw.keys(), q, why)
            # a branch too few at the first level that prunes
            for lv in range(n_eff):
                live = int((tr[lv][:, 0] >= 0).sum())
                if live >= 2:
                    bad = tr.copy()
                    bad[lv][live - 1] = -1
                    ok, _ = parity.certify_row(Qh, Kh, block, k, q, bad, **extra)
                    assert not ok
                    rejected += 1
                    break
            # the last level's best block swapped for the worst valid sibling the level dropped
            last = [(int(f), int(l)) for f, l in tr[-1] if f >= 0]
            prev = [(int(f), int(l)) for f, l in (tr[-2] if n_eff > 1 else [])]
            cands = []
            for (f, l) in prev:
                m = (f + l + 1) // 2
                for c in ((f, m - 1), (m, l)):
                    if c[0] <= c[1] and c not in last:
                        cands.append(c)
            scored = []
            for c in cands:
                rp = [x for x in range(c[0], c[1] + 1)]
                sc = [so.block_score(Qh, Kh, block, q, x, **extra) for x in rp]
                fin = [v for v in sc if np.isfinite(v)]
                if fin:
                    scored.append((sc[[i for i, v in enumerate(sc) if np.isfinite(v)][0]], c))
            if scored and last:
                kept_scores = [so.block_score(Qh, Kh, block, q, f, **extra) for f, _ in last]
                worst = min(scored)
                best_i = int(np.argmax(kept_scores))
                if worst[0] < kept_scores[best_i] - 0.5:
                    bad = tr.copy()
                    row = [c for i, c in enumerate(last) if i != best_i] + [worst[1]]
                    row.sort()
                    bad[-1][:] = -1
                    for i, c in enumerate(row):
                        bad[-1][i] = c
                    ok, _ = parity.certify_row(Qh, Kh, block, k, q, bad, **extra)
                    assert not ok
                    rejected += 1
        assert rejected >= 2, kw.keys()
    # a kept branch the mask hides (future blocks under the causal rule)
    r = so.prune_head(Qh, Kh, 4, 3, [5], want_trace=True)
    tr = r["trace"][0][:4].copy()
    tr[0][0] = (20, 24)
    ok, _ = parity.certify_row(Qh, Kh, 4, 3, 5, tr)
    assert not ok
