"""The library allocates nothing and never synchronises, so a prune + attention step with
caller-provided workspaces and outputs can be recorded into a HIP graph and replayed.  Every replay
(several, with new inputs written into the captured buffers and eager work in between) must equal
the eager result bit for bit, apart from the received mass, whose atomics have no fixed order."""
import math

import numpy as np
import pytest
import torch

from paper_2510_19875_amd import binding, workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def step(Q, K, V, w, bufs, mask="causal", window=0, block_k=0, mask_bits=None):
    cu = w.cu_seqlens if w.batch > 1 else None
    topk = list(w.topk) if w.batch > 1 else w.topk[0]
    p = binding.stream_prune(Q, K, w.heads, w.kv_heads, w.block, topk, cu_seqlens=cu, want_score=True,
                             workspace=bufs.get("wp"), out=bufs.get("op"), mask=mask, window=window,
                             block_k=block_k, mask_bits=mask_bits)
    a = binding.stream_sparse_attn(Q, K, V, w.heads, w.kv_heads, w.block, p["idx"], p["cnt"],
                                   1.0 / math.sqrt(w.head_dim), cu_seqlens=cu, want_lse=True, want_mass=True,
                                   workspace=bufs.get("wa"), out=bufs.get("oa"), mask=mask, window=window,
                                   block_k=block_k, mask_bits=mask_bits)
    bufs["wp"], bufs["op"] = p["workspace"], {"idx": p["idx"], "cnt": p["cnt"], "score": p["score"]}
    bufs["wa"], bufs["oa"] = a["workspace"], {"O": a["O"], "lse": a["lse"], "mass": a["mass"]}
    return bufs


@pytest.mark.parametrize("case", ["single", "ragged_sliding_rect", "long_lists", "mask_array"])
def test_graph_replays_equal_eager(case):
    if case == "single":
        w = wl.scaled(wl.config(2), (64 * 70 + 9,), topk=8, heads=8, kv_heads=2, needles_per_kv_head=2)
        kw = {}
    elif case == "long_lists":
        w = wl.scaled(wl.config(2), (32 * 150 + 9,), topk=80, heads=4, kv_heads=2, block=32, needles_per_kv_head=2)
        kw = {}
    elif case == "mask_array":
        T = 64 * 40 + 9
        w = wl.scaled(wl.config(2), (T,), topk=8, heads=4, kv_heads=2, needles_per_kv_head=2)
        t = np.arange(T)
        C = (t[None, :] <= t[:, None]) & ((t[:, None] // 500 == t[None, :] // 500) | (t[None, :] < 70))
        bits = np.packbits(np.pad(C, ((0, 0), (0, -T % 32))), axis=1, bitorder="little").view(np.int32)
        kw = {"mask_bits": torch.from_numpy(bits.copy()).to(DEV)}
    else:
        w = wl.scaled(wl.config(5), (900, 64, 1700), topk=(3, 1, 5), heads=7, kv_heads=1, block=32, anchors_per_seq=3)
        kw = {"mask": "sliding", "window": 400, "block_k": 64}
    inputs = [wl.make_inputs(w.with_layer(l)) for l in range(3)]
    Qs, Ks, Vs = (torch.empty_like(t, device=DEV) for t in inputs[0][:3])
    for t, src in zip((Qs, Ks, Vs), inputs[0][:3]):
        t.copy_(src)

    # eager results for every layer, with buffers of their own
    eager = []
    for (Q, K, V, _) in inputs:
        b = step(Q.to(DEV), K.to(DEV), V.to(DEV), w, {}, **kw)
        torch.cuda.synchronize()
        eager.append({k: v.clone() for k, v in {**b["op"], **b["oa"]}.items()})

    # warm-up on a side stream (allocates the static buffers), then capture
    bufs = {}
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        step(Qs, Ks, Vs, w, bufs, **kw)
    torch.cuda.current_stream().wait_stream(s)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step(Qs, Ks, Vs, w, bufs, **kw)

    for rep in range(6):
        l = rep % 3
        for t, src in zip((Qs, Ks, Vs), inputs[l][:3]):
            t.copy_(src)                                   # eager work between replays
        g.replay()
        torch.cuda.synchronize()
        got = {**bufs["op"], **bufs["oa"]}
        for key in ("idx", "cnt", "score", "O", "lse"):
            assert torch.equal(got[key], eager[l][key]), (rep, key)
        np.testing.assert_allclose(got["mass"].cpu().numpy(), eager[l]["mass"].cpu().numpy(), rtol=1e-4, atol=1e-5)
        # scribble over the outputs so that a replay that did nothing cannot pass
        for key in ("idx", "cnt"):
            got[key].fill_(-7)
        got["O"].zero_()
