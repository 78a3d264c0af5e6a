"""Pins of oracle/select_update.py (CPU only): the selection/update step checked against
things that are not itself - the C oracle's per-level trace of the whole algorithm, the
hand-traced golden cases, and the definition of "the k largest, ties to the lower position"."""
import os

import numpy as np
import pytest

from oracle import bruteforce as bf
from oracle import stream_oracle as so
from oracle.select_update import select_update

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "alg2_hand_trace.txt")


def _levels_by_select(A, q, k, levels):
    """Alg. 2 for row q with the branch scores read from the table A and every level's
    selection done by select_update.  Returns the node lists after each level."""
    N = A.shape[0]
    nf = np.array([[(j * N) // k for j in range(k)]], dtype=np.int32)
    nl = np.array([[((j + 1) * N) // k - 1 for j in range(k)]], dtype=np.int32)
    nc = np.array([k], dtype=np.int32)
    out = []
    for _ in range(levels):
        sc = np.full((1, 2 * k), -np.inf)
        for j in range(int(nc[0])):
            f, l = int(nf[0, j]), int(nl[0, j])
            m = (f + l + 1) // 2
            for side, (a, b) in enumerate(((f, m - 1), (m, l))):
                if a <= b and a <= q:              # causal: the first valid block is the first block
                    sc[0, 2 * j + side] = A[q, a]
        nf, nl, nc = select_update(sc, nf, nl, nc, k)
        out.append([(int(nf[0, j]), int(nl[0, j])) for j in range(int(nc[0]))])
    return out


def _golden_cases():
    cases = []
    with open(GOLDEN) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            name, N, k, q, scores, exp = [x.strip() for x in line.split("|")]
            cases.append((name, int(N), int(k), int(q), [float(x) for x in scores.split()],
                          [int(x) for x in exp.split()]))
    return cases


@pytest.mark.parametrize("case", _golden_cases(), ids=lambda c: c[0])
def test_hand_traced_cases_through_select_update(case):
    _, N, k, q, scores, expected = case
    A = np.tile(np.asarray(scores, dtype=np.float64), (N, 1))
    levels = so.n_it(N, 1)
    final = _levels_by_select(A, q, k, levels)[-1]
    assert sorted(f for f, l in final if f == l) == expected
    assert all(f == l for f, l in final)


@pytest.mark.parametrize("T,block,k", [(96, 8, 3), (200, 8, 4), (64, 4, 5), (130, 16, 2), (77, 7, 6)])
def test_levels_equal_the_c_oracle_trace(T, block, k):
    rng = np.random.default_rng(1000 + T + k)
    d = 8
    # coarse values: many exact ties between block scores
    Q = np.round(rng.standard_normal((T, d)) * 2).astype(np.float32)
    K = np.round(rng.standard_normal((T, d)) * 2).astype(np.float32)
    A, _ = bf.block_score_table(Q, K, block)
    res = so.prune_head(Q, K, block, k, want_trace=True)
    N = A.shape[0]
    levels = res["trace"].shape[1]
    for q in range(N):
        mine = _levels_by_select(A, q, k, levels)
        for lv in range(levels):
            tr = res["trace"][q, lv]
            theirs = [(int(f), int(l)) for f, l in tr if f >= 0]
            assert mine[lv] == theirs, (q, lv)


def test_definition_of_top_k_with_ties_and_dead_branches():
    rng = np.random.default_rng(7)
    for trial in range(300):
        kmax = int(rng.integers(1, 9))
        k = int(rng.integers(1, kmax + 1))
        c = int(rng.integers(0, kmax + 1))
        # disjoint ascending ranges of sizes 1..4
        sizes = rng.integers(1, 5, size=kmax)
        starts = np.concatenate([[0], np.cumsum(sizes)[:-1]])
        nf = starts[None, :].astype(np.int32)
        nl = (starts + sizes - 1)[None, :].astype(np.int32)
        sc = rng.integers(0, 4, size=(1, 2 * kmax)).astype(np.float64)      # heavy ties
        sc[0, rng.random(2 * kmax) < 0.25] = -np.inf
        of, ol, oc = select_update(sc, nf, nl, np.array([c]), k)
        # the definition, written independently: enumerate valid branches
        valid = []
        for j in range(c):
            f, l = int(nf[0, j]), int(nl[0, j])
            m = (f + l + 1) // 2
            if m - 1 >= f and sc[0, 2 * j] > -np.inf:
                valid.append((2 * j, f, m - 1, sc[0, 2 * j]))
            if sc[0, 2 * j + 1] > -np.inf:
                valid.append((2 * j + 1, m, l, sc[0, 2 * j + 1]))
        n = int(oc[0])
        assert n == min(k, len(valid))
        kept = [(int(of[0, i]), int(ol[0, i])) for i in range(n)]
        kept_pos = [p for p, f, l, s in valid if (f, l) in kept]
        assert len(kept_pos) == n and kept == [(f, l) for p, f, l, s in valid if p in kept_pos]
        dropped = [(p, s) for p, f, l, s in valid if p not in kept_pos]
        for p, f, l, s in valid:
            if p in kept_pos:
                for pd, sd in dropped:
                    assert s > sd or (s == sd and p < pd)
        assert (of[0, n:] == -1).all() and (ol[0, n:] == -1).all()
