"""Difference of two block-sparse masks (TEST INFRASTRUCTURE ONLY).

Only tests, the smoke check and the bench's CPU-baseline leg may import this.

Section 4.2.2 ("Exploring Information Flow") subtracts the masks estimated with k_fail from the
masks estimated with k_success, per layer and head, and weights the remaining connections by
the block scores of the k_success run.  Per (head, query block) row that is a set difference of
two index lists; written with Python sets on purpose.
"""
from __future__ import annotations

import numpy as np


def mask_diff(idx_a, cnt_a, score_a, idx_b, cnt_b):
    """idx_a [rows, ka], cnt_a [rows], score_a [rows, ka] or None: the k_success lists;
    idx_b [rows, kb], cnt_b [rows]: the k_fail lists.  Returns (idx [rows, ka] ascending, padded
    with -1; cnt [rows]; weight [rows, ka] = score_a of the kept entries, padded with -inf)."""
    idx_a, idx_b = np.asarray(idx_a), np.asarray(idx_b)
    rows, ka = idx_a.shape
    out = np.full((rows, ka), -1, dtype=np.int32)
    wt = np.full((rows, ka), -np.inf, dtype=np.float64)
    cnt = np.zeros((rows,), dtype=np.int32)
    for r in range(rows):
        a = [int(x) for x in idx_a[r, :int(cnt_a[r])]]
        b = set(int(x) for x in idx_b[r, :int(cnt_b[r])])
        keep = sorted(set(a) - b)
        for o, blk in enumerate(keep):
            out[r, o] = blk
            if score_a is not None:
                wt[r, o] = score_a[r, a.index(blk)]
        cnt[r] = len(keep)
    return out, cnt, wt
