"""Variable sparsity constant k(row): the oracle's rule pinned on the CPU, the GPU entry point
stream_prune_variable against the oracle through the C ABI."""
import math

import numpy as np
import pytest

from oracle import stream_oracle as so
from paper_2510_19875_amd import workloads as wl
from tests import parity


def gauss(rng, T, d):
    return rng.standard_normal((T, d)).astype(np.float32)


# ------------------------------------------------------------------ CPU pins of the rule
def test_rule_values_and_limits():
    assert [so.variable_k(v, 1, 10, 1, 64) for v in (1, 9, 10, 11, 20, 21, 640, 641, 10 ** 6)] == \
        [1, 1, 1, 2, 2, 3, 64, 64, 64]
    assert so.variable_k(5, 1, 1, 1, 64) == 5 and so.variable_k(5, 1, 1, 8, 64) == 8
    assert [so.valid_blocks(q, 40, 16) for q in (0, 7, 39)] == [1, 8, 40]
    assert so.valid_blocks(10, 40, 16, "full") == 40
    assert [so.valid_blocks(q, 40, 16, "sliding", 40) for q in (0, 2, 3, 10)] == [1, 3, 4, 4]


def test_reduces_to_constant_k_and_to_the_full_mask():
    rng = np.random.default_rng(4)
    b, d, N = 4, 6, 20
    T = N * b - 1
    Q, K = gauss(rng, T, d)[None], gauss(rng, T, d)[None]
    # topk_min = topk_max pins k: the constant-k algorithm
    c = so.prune(Q, K, 1, 1, b, 5)
    v = so.prune_variable(Q, K, 1, 1, b, 1, 1000, 5, 5)
    np.testing.assert_array_equal(c["idx"], v["idx"])
    np.testing.assert_array_equal(c["cnt"], v["cnt"])
    # share 1/1: every valid block is kept
    f = so.prune_variable(Q, K, 1, 1, b, 1, 1, 1, N)
    for q in range(N):
        assert list(f["idx"][0, q, :f["cnt"][0, q]]) == list(range(q + 1))


def test_keeps_the_same_share_of_every_row():
    """The point of a variable k: the retained share of the valid blocks is (nearly) the same at
    the top and at the bottom of the causal pattern, unlike with a constant k."""
    rng = np.random.default_rng(6)
    b, d, N = 4, 6, 64
    T = N * b
    Q, K = gauss(rng, T, d)[None], gauss(rng, T, d)[None]
    v = so.prune_variable(Q, K, 1, 1, b, 1, 4, 1, 16)
    for q in range(N):
        k = v["k"][0, q]
        assert k == min(16, max(1, math.ceil((q + 1) / 4)))
        assert v["cnt"][0, q] == min(k, q + 1)
        assert 0.25 <= v["cnt"][0, q] / (q + 1) <= 0.25 + 1.0 / (q + 1) + 1e-12
    c = so.prune(Q, K, 1, 1, b, 4)
    assert c["cnt"][0, N - 1] / N < 0.07 < 0.25 <= v["cnt"][0, N - 1] / N


def dense_rule_mask(T, mask, window):
    t = np.arange(T)[:, None]
    u = np.arange(T)[None, :]
    if mask == "full":
        return np.ones((T, T), bool)
    c = u <= t
    return c & (t - u < window) if mask == "sliding" else c


@pytest.mark.parametrize("bq,bk", [(4, 4), (4, 8), (8, 4), (2, 8), (8, 2)])
def test_valid_blocks_equal_the_dense_block_mask(bq, bk):
    """The closed-form counts (rules, square and rectangular blocks) and the count read off an
    explicit array both equal C^blk of the preamble of Alg. 2 written out densely: pad C with zero
    rows and columns to T_p, take the maximum over every b_q x b_k span, count the ones of a row."""
    for T in (1, 7, 8, 29, 64, 67):
        Tp = so.padded_len(T, bq, bk)
        for mask, window in (("causal", 0), ("full", 0), ("sliding", 1), ("sliding", 5), ("sliding", 13), ("sliding", 1000)):
            C = dense_rule_mask(T, mask, window)
            Cp = np.zeros((Tp, Tp), bool)
            Cp[:T, :T] = C
            dense = Cp.reshape(Tp // bq, bq, Tp // bk, bk).any(axis=(1, 3)).sum(axis=1)
            for q in range(Tp // bq):
                if bq == bk:
                    assert so.valid_blocks(q, Tp // bq, bq, mask, window) == dense[q], (T, mask, window, q)
                assert so.valid_blocks(q, 0, bq, mask, window, block_k=bk, L=T) == dense[q], (T, mask, window, q)
                assert so.valid_blocks(q, 0, bq, block_k=bk, C=C) == dense[q], (T, mask, window, q)
    # an array no rule expresses: random bits
    rng = np.random.default_rng(9)
    T = 45
    C = rng.random((T, T)) < 0.03
    Tp = so.padded_len(T, bq, bk)
    Cp = np.zeros((Tp, Tp), bool)
    Cp[:T, :T] = C
    dense = Cp.reshape(Tp // bq, bq, Tp // bk, bk).any(axis=(1, 3)).sum(axis=1)
    assert [so.valid_blocks(q, 0, bq, block_k=bk, C=C) for q in range(Tp // bq)] == list(dense)


@pytest.mark.parametrize("bq,bk", [(4, 4), (4, 8), (8, 4)])
def test_variable_k_with_rectangular_blocks_and_arrays(bq, bk):
    """prune_variable under b_q != b_k and under an explicit array: a rule written out as an array
    gives the rule's result; every row is Alg. 2 with the k the row's valid count gives; with an
    arbitrary array the kept blocks are valid ones, as many as min(k(row), valid(row))."""
    rng = np.random.default_rng(12)
    T = 8 * 11 + 3
    Q, K = gauss(rng, T, 6)[None], gauss(rng, T, 6)[None]
    for mask, window in (("causal", 0), ("sliding", 21), ("full", 0)):
        rule = so.prune_variable(Q, K, 1, 1, bq, 1, 3, 1, 6, mask=mask, window=window, block_k=bk)
        arr = so.prune_variable(Q, K, 1, 1, bq, 1, 3, 1, 6, block_k=bk, C=dense_rule_mask(T, mask, window))
        for key in ("idx", "cnt", "k"):
            np.testing.assert_array_equal(rule[key], arr[key])
        for q in range(rule["idx"].shape[1]):
            k = int(rule["k"][0, q])
            one = so.prune_head(Q[0], K[0], bq, k, [q], mask=mask, window=window, block_k=bk)
            np.testing.assert_array_equal(rule["idx"][0, q, :k], one["idx"][0])
            assert (rule["idx"][0, q, k:] == -1).all()
    C = rng.random((T, T)) < 0.02
    v = so.prune_variable(Q, K, 1, 1, bq, 1, 2, 1, 6, block_k=bk, C=C)
    Tp = so.padded_len(T, bq, bk)
    Cp = np.zeros((Tp, Tp), bool)
    Cp[:T, :T] = C
    Cblk = Cp.reshape(Tp // bq, bq, Tp // bk, bk).any(axis=(1, 3))
    for q in range(Tp // bq):
        valid = int(Cblk[q].sum())
        k = min(6, max(1, -(-valid // 2)))
        assert v["k"][0, q] == k and v["cnt"][0, q] == min(k, valid)
        kept = v["idx"][0, q, :v["cnt"][0, q]]
        assert all(Cblk[q, r] for r in kept) and list(kept) == sorted(set(kept))


# ------------------------------------------------------------------ GPU parity
def run_gpu_case(w, keep, kmin, kmax, mask="causal", window=0, n_rows=None):
    import torch

    from paper_2510_19875_amd import binding

    dev = "cuda:0"
    print(f"[vark] {w.name} b={w.block} share={keep} k in [{kmin},{kmax}] mask={mask}", flush=True)
    Q, K, _, _ = wl.make_inputs(w, with_v=False)
    cu = w.cu_seqlens if w.batch > 1 else None
    out = binding.stream_prune_variable(Q.to(dev), K.to(dev), w.heads, w.kv_heads, w.block, keep[0], keep[1],
                                        kmin, kmax, cu_seqlens=cu, want_score=True, want_trace=True,
                                        mask=mask, window=window)
    torch.cuda.synchronize()
    gpu = {x: out[x].cpu().numpy() for x in ("idx", "cnt", "score", "trace")}
    Qf, Kf = Q.float().numpy(), K.float().numpy()
    rows = parity.sample_rows(w, n_rows, seed=3) if n_rows is not None else None
    ref = so.prune_variable(Qf, Kf, w.heads, w.kv_heads, w.block, keep[0], keep[1], kmin, kmax,
                            cu_seqlens=cu, rows=rows, mask=mask, window=window)
    res = parity.compare_variable(gpu, ref, Qf, Kf, w.heads, w.kv_heads, w.block, kmax, cu_seqlens=cu,
                                  mask=mask, window=window)
    print(f"[vark] rows={res['rows']} equal={res['equal']} ties={res['tie_rows']}", flush=True)
    assert res["tie_rows"] <= max(2, res["rows"] // 100)


@pytest.mark.gpu
@pytest.mark.parametrize("block,T,keep,kmin,kmax,mask,window", [
    (64, 64 * 50 + 3, (1, 10), 1, 8, "causal", 0),
    (32, 32 * 70, (1, 4), 2, 16, "causal", 0),
    (128, 128 * 40 + 5, (1, 3), 1, 64, "causal", 0),
    (64, 64 * 64, (1, 2), 1, 64, "sliding", 1500),
    (64, 64 * 30 + 1, (1, 5), 3, 7, "full", 0),
    (64, 64 * 20, (1, 1), 1, 64, "causal", 0),
])
def test_gpu_variable_k(block, T, keep, kmin, kmax, mask, window):
    w = wl.scaled(wl.config(2), (T,), topk=kmax, heads=4, kv_heads=2, block=block, needles_per_kv_head=2)
    run_gpu_case(w, keep, kmin, kmax, mask, window)


@pytest.mark.gpu
def test_gpu_variable_k_ragged_and_config3_rows():
    w = wl.scaled(wl.config(5), (3000, 64 * 7, 1, 5000 + 13), topk=8, heads=7, kv_heads=1)
    run_gpu_case(w, (1, 8), 1, 8, n_rows=200)
    run_gpu_case(wl.config(3), (1, 64), 1, 32, n_rows=24)
