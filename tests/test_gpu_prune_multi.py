"""stream_prune_multi (Alg. 2 for a list of k over the same Q, K) through the C ABI: every
result against the CPU oracle run for that k, and against stream_prune called for that k."""
import numpy as np
import pytest
import torch

from oracle import stream_oracle as so
from paper_2510_19875_amd import binding, workloads as wl
from tests import parity

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def check(w, ks, n_rows=None, seed=0):
    print(f"[multi] {w.name} T={w.T} b={w.block} ks={ks}", flush=True)
    Q, K, _, _ = wl.make_inputs(w, with_v=False)
    cu = w.cu_seqlens if w.batch > 1 else None
    Qd, Kd = Q.to(DEV), K.to(DEV)
    out = binding.stream_prune_multi(Qd, Kd, w.heads, w.kv_heads, w.block, ks, cu_seqlens=cu,
                                     want_score=True, want_tiles=True)
    torch.cuda.synchronize()
    midx, mcnt, msc = (out[x].cpu().numpy() for x in ("idx", "cnt", "score"))
    kmax = max(ks)
    assert midx.shape == (w.heads, len(ks), w.total_blocks, kmax)
    Qf, Kf = Q.float().numpy(), K.float().numpy()
    rows = parity.sample_rows(w, n_rows, seed=seed) if n_rows is not None else None
    tiles_single = tiles_max = 0
    for i, k in enumerate(ks):
        topk = [k] * w.batch if w.batch > 1 else k
        one = binding.stream_prune(Qd, Kd, w.heads, w.kv_heads, w.block, topk, cu_seqlens=cu,
                                   want_score=True, want_trace=True, want_tiles=True)
        torch.cuda.synchronize()
        tiles_single += int(one["tiles"].item())
        tiles_max = max(tiles_max, int(one["tiles"].item()))
        g1 = {x: one[x].cpu().numpy() for x in ("idx", "cnt", "score", "trace")}
        # the sweep's result i is bit-for-bit what a call with that k alone returns
        np.testing.assert_array_equal(midx[:, i, :, :k], g1["idx"])
        np.testing.assert_array_equal(mcnt[:, i], g1["cnt"])
        np.testing.assert_array_equal(msc[:, i, :, :k], g1["score"])
        assert (midx[:, i, :, k:] == -1).all() and np.isneginf(msc[:, i, :, k:]).all()
        # and that call agrees with the oracle (ties certified along its level trace)
        ref = so.prune(Qf, Kf, w.heads, w.kv_heads, w.block, topk, cu_seqlens=cu, rows=rows)
        gm = {"idx": np.ascontiguousarray(midx[:, i, :, :k]), "cnt": np.ascontiguousarray(mcnt[:, i]),
              "score": np.ascontiguousarray(msc[:, i, :, :k]), "trace": g1["trace"]}
        res = parity.compare_prune(gm, ref, Qf, Kf, w.heads, w.kv_heads, w.block, topk,
                                   cu_seqlens=cu, rows=rows)
        print(f"[multi] k={k} rows={res['rows']} equal={res['equal']} tie_rows={res['tie_rows']}", flush=True)
        assert res["tie_rows"] <= max(2, res["rows"] // 100)
    # scores are shared between the values of k: never more evaluations than separate calls,
    # never fewer than the most expensive single call
    assert tiles_max <= int(out["tiles"].item()) <= tiles_single
    print(f"[multi] block scores: sweep {int(out['tiles'].item())}, separate calls {tiles_single}", flush=True)


def test_sweep_small_full_oracle():
    w = wl.scaled(wl.config(2), (64 * 40 + 9,), topk=8, heads=4, kv_heads=2, needles_per_kv_head=2)
    check(w, [8, 4, 2, 1, 5, 8])          # unordered, repeated, k not dividing N


def test_sweep_fp32_block32():
    w = wl.scaled(wl.config(1), (32 * 33,), topk=8, block=32)
    check(w, [16, 3, 1])


def test_sweep_block128_and_large_k():
    w = wl.scaled(wl.config(2), (128 * 70 + 1,), topk=64, heads=4, kv_heads=2, block=128, needles_per_kv_head=2)
    check(w, [64, 32, 7], n_rows=150)


def test_sweep_ragged_batch():
    w = wl.scaled(wl.config(5), (3000, 64 * 7, 1, 5000 + 13), topk=4, heads=7, kv_heads=1)
    check(w, [4, 2, 9], n_rows=200)


def test_limits():
    w = wl.scaled(wl.config(2), (64 * 8,), topk=4, heads=2, kv_heads=1, needles_per_kv_head=0)
    Q, K, _, _ = wl.make_inputs(w, with_v=False)
    Qd, Kd = Q.to(DEV), K.to(DEV)
    r = binding.stream_prune_multi(Qd, Kd, 2, 1, 64, [1] * 32)        # 32 values is the limit
    torch.cuda.synchronize()
    assert (r["cnt"].cpu().numpy() == 1).all()
    with pytest.raises(binding.StreamError):
        binding.stream_prune_multi(Qd, Kd, 2, 1, 64, [1] * 33)
