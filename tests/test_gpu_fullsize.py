"""Full-size workloads in the launch configuration bench.py times: sampled rows against the oracle
(rows are independent, so a sampled row is checked exactly) plus properties that hold at any size."""
import math

import numpy as np
import pytest
import torch

from oracle import stream_oracle as so
from paper_2510_19875_amd import binding, workloads as wl
from tests import parity

pytestmark = pytest.mark.gpu


def check_full(w, heads_sampled, n_rows, seed, check_sink=True, mask="causal", window=0):
    dev = torch.device("cuda:0")
    print(f"[full] {w.name}: generating inputs", flush=True)
    Q, K, V, meta = wl.make_inputs(w, device=dev)
    cu = w.cu_seqlens if w.batch > 1 else None
    topk = list(w.topk) if w.batch > 1 else w.topk[0]
    kmax = w.topk_max
    torch.cuda.reset_peak_memory_stats()
    base = torch.cuda.memory_allocated()
    print("[full] prune", flush=True)
    out = binding.stream_prune(Q, K, w.heads, w.kv_heads, w.block, topk, cu_seqlens=cu,
                               want_score=True, want_trace=True, mask=mask, window=window)
    scale = 1.0 / math.sqrt(w.head_dim)
    print("[full] attention", flush=True)
    att = binding.stream_sparse_attn(Q, K, V, w.heads, w.kv_heads, w.block, out["idx"], out["cnt"], scale,
                                     cu_seqlens=cu, want_lse=True, want_mass=True, mask=mask, window=window)
    torch.cuda.synchronize()
    extra = torch.cuda.max_memory_allocated() - base
    # O(T) memory: everything beyond the inputs is outputs + workspaces, linear in T (no T x T term)
    lin = (Q.numel() + 3 * K.numel()) * Q.element_size() + w.heads * w.T * 12 + \
        w.heads * w.total_blocks * kmax * (4 * 5 + 8 * out["levels"]) + (1 << 24)
    print(f"[full] extra device bytes {extra:,} (linear bound {lin:,})", flush=True)
    assert extra <= lin

    # ---- properties at full size
    bseq, bloc = so.block_table(w.cu_seqlens, w.block)
    qloc = torch.from_numpy(bloc).to(dev)
    kseq = torch.tensor([w.topk[s] for s in bseq], device=dev)
    cnt = out["cnt"]
    # valid key blocks of every row under the mask rule: rmin .. rmax
    nseq_blocks = torch.tensor([w.blocks_per_seq[s] for s in bseq], device=dev)
    rmax = nseq_blocks - 1 if mask == "full" else qloc
    rmin = torch.zeros_like(qloc)
    if mask == "sliding":
        lo = qloc * w.block - window + 1
        rmin = torch.where(lo > 0, torch.div(lo, w.block, rounding_mode="floor"), torch.zeros_like(lo))
    assert torch.equal(cnt, torch.minimum(kseq, rmax - rmin + 1).to(torch.int32)[None, :].expand_as(cnt))
    idx = out["idx"]
    slot = torch.arange(kmax, device=dev)[None, None, :]
    live = slot < cnt[:, :, None]
    assert bool(((idx >= rmin[None, :, None]) & (idx <= rmax[None, :, None]))[live].all()) and bool((idx[~live] == -1).all())
    assert bool((idx[:, :, 1:] > idx[:, :, :-1])[live[:, :, 1:]].all())
    if check_sink:
        assert bool((idx[:, :, 0] == 0).all())
    mass = att["mass"]
    assert bool((mass >= 0).all())
    np.testing.assert_allclose(mass.sum(dim=1).cpu().numpy(), float(w.T), rtol=2e-4)
    assert bool(torch.isfinite(att["O"].float()).all()) and bool(torch.isfinite(att["lse"]).all())

    # ---- sampled rows against the oracle
    rows = parity.sample_rows(w, n_rows, seed=seed, heads=heads_sampled)
    g = w.heads // w.kv_heads
    cuq = w.cu_seqlens
    idx_c, cnt_c = idx.cpu().numpy(), cnt.cpu().numpy()
    score_c, trace_c = out["score"].cpu().numpy(), out["trace"].cpu().numpy()
    tol = 2e-2 if w.dtype == "bf16" else 1e-4
    equal = ties = 0
    worst_o = worst_l = 0.0
    cache = {}
    for (h, gb) in rows:
        s, q = int(bseq[gb]), int(bloc[gb])
        a, e = cuq[s], cuq[s + 1]
        key = (h, s)
        if key not in cache:
            cache.clear()
            cache[key] = (Q[h, a:e].float().cpu().numpy(), K[h // g, a:e].float().cpu().numpy(),
                          V[h // g, a:e].float().cpu().numpy())
        Qh, Kh, Vh = cache[key]
        k = w.topk[s]
        r = so.prune_head(Qh, Kh, w.block, k, qblocks=[q], mask=mask, window=window)
        c = int(r["cnt"][0])
        if np.array_equal(r["idx"][0], idx_c[h, gb, :k]):
            equal += 1
            np.testing.assert_allclose(score_c[h, gb, :c], r["score"][0, :c], rtol=1e-4)
        else:
            n_eff = max(1, math.ceil(math.log2(math.ceil(-(-(e - a) // w.block) / k))))
            ok, why = parity.certify_row(Qh, Kh, w.block, k, q, trace_c[:n_eff, h, gb, :k], mask=mask, window=window)
            assert ok, (h, gb, why)
            ties += 1
        # attention of that row with the GPU's own list (checked above) against Eq. (2) in fp64
        gi = np.ascontiguousarray(idx_c[h, gb][None, :])
        gc = np.ascontiguousarray(cnt_c[h, gb][None])
        ra = so.sparse_attn(Qh[None], Kh[None], Vh[None], 1, 1, w.block, gi, gc, scale, rows=[(0, q)],
                            mask=mask, window=window)
        t0, t1 = q * w.block, min((q + 1) * w.block, e - a)
        O_g = att["O"][h, a + t0:a + t1].float().cpu().numpy()
        l_g = att["lse"][h, a + t0:a + t1].cpu().numpy()
        worst_o = max(worst_o, float(np.abs(O_g - ra["O"][0, t0:t1]).max()))
        worst_l = max(worst_l, float(np.abs(l_g - ra["lse"][0, t0:t1]).max()))
    print(f"[full] {w.name}: sampled rows={len(rows)} equal={equal} ties={ties} "
          f"max|dO|={worst_o:.3e} max|dlse|={worst_l:.3e}", flush=True)
    assert worst_o <= tol and worst_l <= 1e-3
    assert ties <= max(2, len(rows) // 20)
    return meta, att


def test_config3_attention_and_prune_sampled():
    check_full(wl.config(3), heads_sampled=[2, 17, 30], n_rows=36, seed=11)


def test_config3_sliding_window_sampled():
    """The headline shape under a sliding window of 4096 tokens (65 valid key blocks per row,
    32 kept): the local layers of the Gemma 3 models the paper traces."""
    check_full(wl.config(3), heads_sampled=[4, 21], n_rows=24, seed=14, check_sink=False,
               mask="sliding", window=4096)


def test_config3_long_lists_sampled():
    """The headline tensors keeping 100 blocks per row: the kernels with the row's lists in LDS at scale."""
    w = wl.config(3)
    check_full(wl.scaled(w, w.seq_lens, topk=100, name=w.name + "_k100"), heads_sampled=[7, 25], n_rows=12, seed=15)


def test_config4_one_million_tokens_sampled():
    """T = 1,048,576, block 128, k = 64: O(T) memory and the four-wavefront row path at scale."""
    check_full(wl.config(4), heads_sampled=[5, 26], n_rows=14, seed=12)


def test_config5_ragged_reasoning_shape_sampled():
    w = wl.config(5)
    # (k_s is 1-5 here and the anchor keys outscore the sink, so block 0 is not always kept)
    meta, att = check_full(w, heads_sampled=[0, 9, 27], n_rows=70, seed=13, check_sink=False)
    # anchors (shared direction, every query has a component along it) collect far more mass
    mass = att["mass"].cpu().numpy()
    cu = w.cu_seqlens
    ratios = []
    for s in range(w.batch):
        a = [cu[s] + t for t in meta["anchors"][s]]
        ratios.append(np.median(mass[:, a]) / max(np.median(mass[:, cu[s]:cu[s + 1]]), 1e-9))
    print("[full] anchor/typical received-mass ratio per sequence:", np.round(ratios, 1), flush=True)
    assert np.median(ratios) > 5
