"""Top-k selection and node update of Algorithm 2 as a step of its own (TEST INFRASTRUCTURE ONLY).

Only tests, the smoke check and the bench's CPU-baseline leg may import this.

One level of the listing in Appendix C, after the branch scores are known: the row's live
nodes (f_j, l_j) are split at the midpoint into branches, the k best branches are kept
("top-k indices" line) and become the row's nodes for the next level ("update" line).
Readings, as in stream_oracle.c: a range is half open at the midpoint,
m = floor((f + l + 1) / 2), children [f, m - 1] and [m, l]; an empty branch or one whose
score is -inf (no valid block) is never kept; equal scores go to the lower branch position;
survivors keep their positional order.  Plain Python on purpose.
"""
from __future__ import annotations

import numpy as np


def select_update(score, node_first, node_last, node_count, k: int):
    """score [rows, 2*kmax] (branch 2j = left child of node j, 2j+1 = right child),
    node_first/node_last [rows, kmax], node_count [rows].  Returns (first, last, count) of the
    next level; slots at and after count are -1."""
    score = np.asarray(score, dtype=np.float64)
    nf = np.asarray(node_first)
    nl = np.asarray(node_last)
    nc = np.asarray(node_count)
    rows, kmax = nf.shape
    assert score.shape == (rows, 2 * kmax) and 1 <= k <= kmax
    of = np.full((rows, kmax), -1, dtype=np.int32)
    ol = np.full((rows, kmax), -1, dtype=np.int32)
    oc = np.zeros((rows,), dtype=np.int32)
    for r in range(rows):
        branches = []
        for j in range(int(nc[r])):
            f, l = int(nf[r, j]), int(nl[r, j])
            m = (f + l + 1) // 2
            branches.append((f, m - 1, score[r, 2 * j]))
            branches.append((m, l, score[r, 2 * j + 1]))
        cand = [(-s, pos) for pos, (f, l, s) in enumerate(branches) if f <= l and s > -np.inf]
        keep = sorted(pos for _, pos in sorted(cand)[:k])
        for o, pos in enumerate(keep):
            of[r, o], ol[r, o] = branches[pos][0], branches[pos][1]
        oc[r] = len(keep)
    return of, ol, oc
