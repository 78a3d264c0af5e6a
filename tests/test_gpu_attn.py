"""GPU parity of stream_sparse_attn against the CPU oracle (through the C ABI)."""
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


def run_case(w, rows=None, full_mask=False):
    print(f"[attn] {w.name} T={w.T} H={w.heads}/{w.kv_heads} d={w.head_dim} {w.dtype} b={w.block} "
          f"k={w.topk}", flush=True)
    dev = torch.device("cuda:0")
    Q, K, V, meta = wl.make_inputs(w)
    cu = w.cu_seqlens if w.batch > 1 else None
    topk = list(w.topk) if w.batch > 1 else w.topk[0]
    Qf, Kf, Vf = Q.float().numpy(), K.float().numpy(), V.float().numpy()
    ref_p = so.prune(Qf, Kf, w.heads, w.kv_heads, w.block, topk, cu_seqlens=cu)
    scale = 1.0 / math.sqrt(w.head_dim)
    # the oracle's lists feed the GPU attention, so near-ties of the prune cannot leak in here
    idx_t = torch.from_numpy(ref_p["idx"]).to(dev)
    cnt_t = torch.from_numpy(ref_p["cnt"]).to(dev)
    out = binding.stream_sparse_attn(Q.to(dev), K.to(dev), V.to(dev), w.heads, w.kv_heads, w.block,
                                     idx_t, cnt_t, scale, cu_seqlens=cu, want_lse=True, want_mass=True)
    torch.cuda.synchronize()
    ref = so.sparse_attn(Qf, Kf, Vf, w.heads, w.kv_heads, w.block, ref_p["idx"], ref_p["cnt"], scale,
                         cu_seqlens=cu)
    O = out["O"].float().cpu().numpy()
    err = np.abs(O - ref["O"]).max()
    lerr = np.abs(out["lse"].cpu().numpy() - ref["lse"]).max()
    mass = out["mass"].cpu().numpy().astype(np.float64)
    merr = (np.abs(mass - ref["mass"]) / np.maximum(ref["mass"], 1.0)).max()
    print(f"[attn] max|dO|={err:.3e} max|dlse|={lerr:.3e} mass rel err={merr:.3e}", flush=True)
    assert err <= TOL[w.dtype]
    assert lerr <= 1e-3
    assert merr <= 1e-3
    np.testing.assert_allclose(mass.sum(axis=1), w.T, rtol=1e-4)   # every real row of P sums to 1
    return out, ref, meta


def test_config1_full_fp32_sink_dominates():
    w = wl.config(1)
    out, ref, meta = run_case(w)
    mass = out["mass"].cpu().numpy()
    assert np.all(mass[:, 0] >= 0.5 * mass.max(axis=1))   # the sink column is (about) the largest


@pytest.mark.parametrize("block,k,T,dtype,d,H,Hkv", [
    (64, 8, 4096 + 37, "bf16", 128, 8, 2),
    (128, 4, 4096 + 100, "bf16", 128, 4, 2),
    (32, 8, 2048 + 5, "bf16", 128, 4, 2),
    (64, 8, 3000, "bf16", 64, 4, 4),
    (64, 4, 1500, "f32", 128, 2, 1),
    (32, 3, 1000, "f32", 64, 2, 2),
    (128, 5, 3000, "f32", 64, 2, 1),
    (64, 64, 64 * 40, "bf16", 128, 2, 1),   # k >= N: dense causal attention
])
def test_shapes(block, k, T, dtype, d, H, Hkv):
    w = wl.scaled(wl.config(2), (T,), topk=k, heads=H, kv_heads=Hkv, block=block, dtype=dtype,
                  head_dim=d, needles_per_kv_head=2)
    run_case(w)


def test_ragged_anchor_batch():
    w = wl.scaled(wl.config(5), (700, 1300, 64, 33, 2049), topk=(2, 3, 1, 4, 2), heads=14, kv_heads=2,
                  anchors_per_seq=3)
    out, ref, meta = run_case(w)
    # anchors collect far more attention than a typical key
    mass = out["mass"].cpu().numpy()
    cu = w.cu_seqlens
    for s in (1, 4):
        a = [cu[s] + t for t in meta["anchors"][s]]
        assert np.median(mass[:, a]) > 5 * np.median(mass[:, cu[s]:cu[s + 1]])


def test_full_mask_equals_torch_causal_attention_on_gpu():
    """k >= N: Eq. (2) with the full causal mask is ordinary causal attention."""
    w = wl.scaled(wl.config(2), (2048,), topk=32, heads=4, kv_heads=2, needles_per_kv_head=0)
    dev = torch.device("cuda:0")
    Q, K, V, _ = wl.make_inputs(w)
    Qd, Kd, Vd = Q.to(dev), K.to(dev), V.to(dev)
    p = binding.stream_prune(Qd, Kd, w.heads, w.kv_heads, w.block, 32)
    scale = 1.0 / math.sqrt(w.head_dim)
    a = binding.stream_sparse_attn(Qd, Kd, Vd, w.heads, w.kv_heads, w.block, p["idx"], p["cnt"], scale)
    ref = torch.nn.functional.scaled_dot_product_attention(
        Q.double()[None], K.double().repeat_interleave(2, 0)[None], V.double().repeat_interleave(2, 0)[None],
        is_causal=True)[0]
    assert (a["O"].double().cpu() - ref).abs().max() <= 2e-2


@pytest.mark.parametrize("kind", ["overflow", "vanish"])
def test_fixed_reference_falls_back_to_the_tracked_order(kind):
    """The pipelined loop keeps the softmax reference of the sub-tile before it.  Scores that
    then jump by hundreds of octaves (overflow), or a row whose first visible keys sit hundreds
    of octaves above everything else seen later under a zero reference (vanish), must come out
    right: the kernel notices the non-finite / vanished sums and recomputes the row while
    tracking the maximum."""
    dev = torch.device("cuda:0")
    H, T, d, b = 2, 64 * 8 + 5, 128, 64
    g = torch.Generator().manual_seed(5)
    V = torch.randn((H, T, d), generator=g).to(torch.bfloat16)
    Q = torch.full((H, T, d), 4.0).to(torch.bfloat16)
    K = torch.full((H, T, d), 4.0).to(torch.bfloat16)
    if kind == "overflow":
        K[:, :32] = 0.0          # first sub-tile: score 0; every later key: 2048 * scale * log2(e) = 261 octaves
    else:
        K[:, 32:] = -4.0         # first sub-tile: +261 octaves; later keys: -261
        K[:, :32] = 0.0
        Q[:, :] = 4.0
    mask, window = ("causal", 0) if kind == "overflow" else ("sliding", 100)
    Qf, Kf, Vf = Q.float().numpy(), K.float().numpy(), V.float().numpy()
    N = -(-T // b)
    ref_p = so.prune(Qf, Kf, H, H, b, N, mask=mask, window=window)
    scale = 1.0 / math.sqrt(d)
    out = binding.stream_sparse_attn(Q.to(dev), K.to(dev), V.to(dev), H, H, b, torch.from_numpy(ref_p["idx"]).to(dev),
                                     torch.from_numpy(ref_p["cnt"]).to(dev), scale, want_lse=True, want_mass=True,
                                     mask=mask, window=window)
    torch.cuda.synchronize()
    ref = so.sparse_attn(Qf, Kf, Vf, H, H, b, ref_p["idx"], ref_p["cnt"], scale, mask=mask, window=window)
    O = out["O"].float().cpu().numpy()
    assert np.isfinite(O).all() and np.isfinite(out["lse"].cpu().numpy()).all()
    assert np.abs(O - ref["O"]).max() <= TOL["bf16"]
    np.testing.assert_allclose(out["lse"].cpu().numpy(), ref["lse"], rtol=1e-5, atol=1e-3)
    mass = out["mass"].cpu().numpy().astype(np.float64)
    assert (np.abs(mass - ref["mass"]) / np.maximum(ref["mass"], 1.0)).max() <= 1e-3


def test_strided_inputs_and_output():
    """Token-major [T, H, d] storage (one fused projection buffer) viewed as [H, T, d], for Q, K,
    V and the output: same results as the contiguous call, for the attention and for the
    receiver statistics."""
    w = wl.scaled(wl.config(2), (64 * 33 + 11,), topk=4, heads=4, kv_heads=2, needles_per_kv_head=1)
    dev = torch.device("cuda:0")
    Q, K, V, _ = wl.make_inputs(w)
    Qd, Kd, Vd = Q.to(dev), K.to(dev), V.to(dev)
    T, d = w.T, w.head_dim
    fused = torch.empty((T, w.heads + 2 * w.kv_heads, d), dtype=Qd.dtype, device=dev)
    fused[:, :w.heads] = Qd.transpose(0, 1)
    fused[:, w.heads:w.heads + w.kv_heads] = Kd.transpose(0, 1)
    fused[:, w.heads + w.kv_heads:] = Vd.transpose(0, 1)
    Qs = fused[:, :w.heads].transpose(0, 1)
    Ks = fused[:, w.heads:w.heads + w.kv_heads].transpose(0, 1)
    Vs = fused[:, w.heads + w.kv_heads:].transpose(0, 1)
    assert not Qs.is_contiguous() and Qs.stride(1) == (w.heads + 2 * w.kv_heads) * d
    scale = 1.0 / math.sqrt(d)
    p = binding.stream_prune(Qs, Ks, w.heads, w.kv_heads, w.block, 4)
    a = binding.stream_sparse_attn(Qd, Kd, Vd, w.heads, w.kv_heads, w.block, p["idx"], p["cnt"], scale, want_lse=True)
    O_tok = torch.zeros((T, w.heads, d), dtype=Qd.dtype, device=dev)       # token-major output
    b = binding.stream_sparse_attn(Qs, Ks, Vs, w.heads, w.kv_heads, w.block, p["idx"], p["cnt"], scale,
                                   want_lse=True, out={"O": O_tok.transpose(0, 1), "lse": torch.empty_like(a["lse"])})
    torch.cuda.synchronize()
    assert torch.equal(a["O"], O_tok.transpose(0, 1)) and torch.equal(a["lse"], b["lse"])
    ra = binding.stream_receiver_stats(Qd, Kd, w.heads, w.kv_heads, w.block, scale)
    rb = binding.stream_receiver_stats(Qs, Ks, w.heads, w.kv_heads, w.block, scale)
    torch.cuda.synchronize()
    assert torch.equal(ra["col_mean"], rb["col_mean"]) and torch.equal(ra["head"], rb["head"])


@pytest.mark.parametrize("kmax,block", [(12, 64), (80, 32)])
def test_lists_not_ascending_or_out_of_range_never_leak_future_keys(kmax, block):
    """Lists the pruning never writes: shuffled entries, blocks after the query block, ids past the
    end of the sequence and below zero.  The kernels then mask every tile at token level: the
    result is Eq. (2) over the listed blocks' visible keys (the oracle takes a list in any
    order), ids outside the sequence add nothing, no key after a query ever counts."""
    w = wl.scaled(wl.config(2), (block * 41 + 7,), topk=4, heads=4, kv_heads=2, block=block, needles_per_kv_head=2)
    Q, K, V, _ = wl.make_inputs(w)
    N = w.blocks_per_seq[0]
    rng = np.random.default_rng(5)
    idx = np.full((w.heads, N, kmax), -1, dtype=np.int32)
    cnt = np.zeros((w.heads, N), dtype=np.int32)
    for h in range(w.heads):
        for q in range(N):
            c = int(rng.integers(1, kmax + 1))
            pool = np.arange(N + 3)                               # incl. future blocks and ids >= N
            ent = rng.choice(pool, size=min(c, len(pool)), replace=False)
            kind = (h + q) % 4
            if kind == 0:
                ent = np.sort(ent[ent <= q])                      # a list as the pruning writes it
            elif kind == 1:
                ent = np.sort(ent)                                # ascending, but with future / outside ids
            cnt[h, q] = len(ent)                                  # kinds 2, 3: shuffled as drawn
            idx[h, q, :len(ent)] = ent
    scale = 1.0 / math.sqrt(w.head_dim)
    ref = so.sparse_attn(Q.float().numpy(), K.float().numpy(), V.float().numpy(), w.heads, w.kv_heads, block,
                         idx, cnt, scale)
    it, ct = torch.from_numpy(idx).to(DEV), torch.from_numpy(cnt).to(DEV)
    a = binding.stream_sparse_attn(Q.to(DEV), K.to(DEV), V.to(DEV), w.heads, w.kv_heads, block, it, ct, scale,
                                   want_lse=True, want_mass=True)
    torch.cuda.synchronize()
    O, lse, mass = a["O"].float().cpu().numpy(), a["lse"].cpu().numpy(), a["mass"].cpu().numpy()
    seen = np.isfinite(ref["lse"])                                # queries with at least one visible listed key
    assert (np.isneginf(lse) == ~seen).all()
    np.testing.assert_allclose(lse[seen], ref["lse"][seen], atol=1e-3)
    assert np.abs(O - ref["O"]).max() <= TOL[w.dtype]
    np.testing.assert_allclose(mass, ref["mass"], rtol=1e-3, atol=1e-5)
    # ids below zero: the same result as the list without them
    idx2 = idx.copy()
    idx2[:, :, 0] = np.where(cnt > 1, -1 - (idx[:, :, 0] % 3), idx[:, :, 0])
    idx3 = idx.copy()
    cnt3 = cnt.copy()
    for h in range(w.heads):
        for q in range(N):
            if cnt[h, q] > 1:
                idx3[h, q, :cnt[h, q] - 1] = idx[h, q, 1:cnt[h, q]]
                idx3[h, q, cnt[h, q] - 1] = -1
                cnt3[h, q] -= 1
    ref3 = so.sparse_attn(Q.float().numpy(), K.float().numpy(), V.float().numpy(), w.heads, w.kv_heads, block,
                          idx3, cnt3, scale)
    b = binding.stream_sparse_attn(Q.to(DEV), K.to(DEV), V.to(DEV), w.heads, w.kv_heads, block,
                                   torch.from_numpy(idx2).to(DEV), ct, scale, want_lse=True, want_mass=True)
    torch.cuda.synchronize()
    assert np.abs(b["O"].float().cpu().numpy() - ref3["O"]).max() <= TOL[w.dtype]
    np.testing.assert_allclose(b["mass"].cpu().numpy(), ref3["mass"], rtol=1e-3, atol=1e-5)
