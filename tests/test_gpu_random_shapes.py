"""Seeded random valid configurations (dtype, head dim, b_q, b_k, mask rule, window, GQA ratio,
ragged batch, k per sequence) through the whole path against the oracle: Alg. 2 lists, scores and
traces over every row, then Eq. (2) (O, lse, mass) on the oracle's lists."""
import math

import numpy as np
import pytest
import torch

from oracle import stream_oracle as so
from paper_2510_19875_amd import binding, workloads as wl
from tests import parity

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL = {"bf16": 2e-2, "f32": 1e-4}


def draw(seed):
    rng = np.random.default_rng(1000 + seed)
    dtype = ["bf16", "f32"][int(rng.integers(2))]
    d = [64, 128][int(rng.integers(2))]
    bq, bk = (int(x) for x in rng.choice([32, 64, 128], size=2))
    if dtype == "f32" and d == 128 and {bq, bk} == {64, 128}:
        bk = bq                                         # the one shape the library refuses
    kv = int(rng.choice([1, 2, 3]))
    g = int(rng.choice([1, 2, 4, 7]))
    nseq = int(rng.choice([1, 1, 2, 4]))
    lens = tuple(int(x) for x in rng.integers(1, 2200, size=nseq))
    mask = ["causal", "sliding", "full"][int(rng.integers(3))]
    window = int(rng.choice([1, 17, 100, 333, 1500, 10 ** 6])) if mask == "sliding" else 0
    ks = tuple(int(x) for x in rng.integers(1, 12, size=nseq))
    return dtype, d, bq, bk, kv, g, lens, mask, window, ks


def draw_wide(seed):
    """The same, with more than 64 blocks kept per row in at least one sequence (the kernels that
    keep the lists in LDS)."""
    dtype, d, bq, bk, kv, g, lens, mask, window, ks = draw(500 + seed)
    rng = np.random.default_rng(9000 + seed)
    if bq == 128 and bk == 128 and dtype == "f32" and d == 128:
        bq = int(rng.choice([32, 64]))                  # (refused: the tile fits no wavefront)
    if dtype == "f32" and d == 128 and {bq, bk} == {64, 128}:
        bq = 32                                         # the one shape the library refuses
    ks = tuple(int(x) for x in rng.integers(1, 220, size=len(lens)))
    ks = (int(rng.integers(65, 220)),) + ks[1:]
    return dtype, d, bq, bk, kv, min(g, 2), lens, mask, window, ks


@pytest.mark.parametrize("seed", [("narrow", s) for s in range(28)] + [("wide", s) for s in range(10)] +
                         [("narrow", s) for s in range(600, 680)] + [("wide", s) for s in range(500, 520)],
                         ids=lambda x: f"{x[0]}{x[1]}")
def test_random_configuration(seed):
    cfg = draw(seed[1]) if seed[0] == "narrow" else draw_wide(seed[1])
    run_configuration(f"{seed[0]} {seed[1]}", *cfg)


def test_batches_of_many_sequences():
    """50 and 64 (the most a call takes) short sequences in one packed batch, k per sequence."""
    for n, bq, bk, dtype in ((50, 64, 64, "bf16"), (64, 32, 128, "f32")):
        rng = np.random.default_rng(n)
        lens = tuple(int(x) for x in rng.integers(1, 500, size=n))
        ks = tuple(int(x) for x in rng.integers(1, 9, size=n))
        run_configuration(f"batch of {n}", dtype, 64, bq, bk, 2, 2, lens, "causal", 0, ks)


def run_configuration(seed, dtype, d, bq, bk, kv, g, lens, mask, window, ks):
    H = kv * g
    cfg = 5 if len(lens) > 1 else 2
    kw = {"needles_per_kv_head": 1} if cfg == 2 else {"anchors_per_seq": 2}
    w = wl.scaled(wl.config(cfg), lens, topk=ks if len(lens) > 1 else ks[0], heads=H, kv_heads=kv, block=bq,
                  dtype=dtype, head_dim=d, **kw)
    print(f"[random {seed}] {dtype} d={d} b_q={bq} b_k={bk} H={H}/{kv} lens={lens} {mask}/{window} k={ks}", flush=True)
    Q, K, V, _ = wl.make_inputs(w)
    cu = w.cu_seqlens if len(lens) > 1 else None
    topk = list(ks) if len(lens) > 1 else ks[0]
    Qd, Kd, Vd = Q.to(DEV), K.to(DEV), V.to(DEV)
    out = binding.stream_prune(Qd, Kd, H, kv, bq, topk, cu_seqlens=cu, want_score=True, want_trace=True,
                               mask=mask, window=window, block_k=bk)
    torch.cuda.synchronize()
    gpu = {x: out[x].cpu().numpy() for x in ("idx", "cnt", "score", "trace")}
    Qf, Kf, Vf = Q.float().numpy(), K.float().numpy(), V.float().numpy()
    ref = so.prune(Qf, Kf, H, kv, bq, topk, cu_seqlens=cu, mask=mask, window=window, block_k=bk)
    res = parity.compare_prune(gpu, ref, Qf, Kf, H, kv, bq, topk, cu_seqlens=cu, mask=mask, window=window,
                               block_k=bk)
    assert res["tie_rows"] <= max(2, res["rows"] // 100)
    scale = 1.0 / math.sqrt(d)
    att = binding.stream_sparse_attn(Qd, Kd, Vd, H, kv, bq, torch.from_numpy(ref["idx"]).to(DEV),
                                     torch.from_numpy(ref["cnt"]).to(DEV), scale, cu_seqlens=cu, want_lse=True,
                                     want_mass=True, mask=mask, window=window, block_k=bk)
    torch.cuda.synchronize()
    ra = so.sparse_attn(Qf, Kf, Vf, H, kv, bq, ref["idx"], ref["cnt"], scale, cu_seqlens=cu, mask=mask,
                        window=window, block_k=bk)
    glse, gO = att["lse"].cpu().numpy(), att["O"].float().cpu().numpy()
    empty = np.isneginf(ra["lse"])
    assert np.isneginf(glse[empty]).all() and (gO[empty] == 0).all()
    err = np.abs(gO - ra["O"]).max()
    lerr = np.abs(np.where(empty, 0.0, glse - np.where(empty, 0.0, ra["lse"]))).max()
    mass = att["mass"].cpu().numpy().astype(np.float64)
    merr = (np.abs(mass - ra["mass"]) / np.maximum(ra["mass"], 1.0)).max()
    print(f"[random {seed}] rows={res['rows']} equal={res['equal']} max|dO|={err:.2e} max|dlse|={lerr:.2e} "
          f"mass={merr:.2e} empty={int(empty.sum())}", flush=True)
    assert err <= TOL[dtype] and lerr <= 1e-3 and merr <= 1e-3
