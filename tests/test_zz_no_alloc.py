"""stream_prune_static (the entry point that allocates nothing: its scratch is a device array of
the library) through the C ABI against stream_prune on the same inputs: two calls in a row, the
second on a smaller input (the scratch keeps the first call's contents), then a ragged batch, a
mask array and a list of more than 64 blocks; sizes beyond the array are refused on the host."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import stream_oracle as so
from paper_2510_19875_amd import binding, workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def both(w, mask_bits=None, block_k=0):
    Q, K, _, _ = wl.make_inputs(w, with_v=False)
    Qd, Kd = Q.to(DEV), K.to(DEV)
    cu = w.cu_seqlens if w.batch > 1 else None
    topk = list(w.topk) if w.batch > 1 else w.topk[0]
    ref = binding.stream_prune(Qd, Kd, w.heads, w.kv_heads, w.block, topk, cu_seqlens=cu, want_score=True,
                               mask_bits=mask_bits, block_k=block_k)
    out = {"idx": torch.full_like(ref["idx"], -7), "cnt": torch.full_like(ref["cnt"], -7),
           "score": torch.full_like(ref["score"], 123.0)}
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated(), torch.cuda.memory_reserved()
    binding.stream_prune_static(Qd, Kd, w.heads, w.kv_heads, w.block, topk, out, cu_seqlens=cu,
                                mask_bits=mask_bits, block_k=block_k)
    torch.cuda.synchronize()
    assert (torch.cuda.memory_allocated(), torch.cuda.memory_reserved()) == before
    # integer lists and counts bit for bit; the scores are the same arithmetic on the same tiles
    assert torch.equal(out["idx"], ref["idx"]) and torch.equal(out["cnt"], ref["cnt"])
    assert torch.equal(out["score"], ref["score"])
    return Q, K, out


def test_two_calls_in_a_row_second_smaller_then_other_shapes():
    print("[static] first call: 9001 tokens, 8/2 heads, k = 8", flush=True)
    w1 = wl.scaled(wl.config(2), (9001,), topk=8, heads=8, kv_heads=2, needles_per_kv_head=2)
    both(w1)
    print("[static] second call: 1500 tokens, 4/2 heads, k = 4", flush=True)
    w2 = wl.scaled(wl.config(2), (1500,), topk=4, heads=4, kv_heads=2, needles_per_kv_head=2)
    Q, K, out = both(w2)
    # and the smaller call against the oracle itself
    ref = so.prune(Q.float().numpy(), K.float().numpy(), w2.heads, w2.kv_heads, w2.block, w2.topk[0])
    np.testing.assert_array_equal(out["cnt"].cpu().numpy(), ref["cnt"])
    same = (out["idx"].cpu().numpy() == ref["idx"]).all(axis=-1).mean()
    assert same >= 0.99, same
    print("[static] ragged batch, per-sequence k", flush=True)
    both(wl.scaled(wl.config(5), (3000, 64 * 7, 1, 1500 + 13), topk=(4, 2, 1, 5), heads=7, kv_heads=1))
    print("[static] more than 64 blocks per row, rectangular blocks", flush=True)
    both(wl.scaled(wl.config(2), (32 * 200 + 3,), topk=100, heads=2, kv_heads=1, block=32, needles_per_kv_head=2))
    both(wl.scaled(wl.config(2), (64 * 60 + 5,), topk=8, heads=4, kv_heads=2, block=64, needles_per_kv_head=2), block_k=32)
    print("[static] mask array", flush=True)
    T = 64 * 30 + 9
    t = np.arange(T)
    C = (t[None, :] <= t[:, None]) & ((t[:, None] // 700) == (t[None, :] // 700))
    padded = np.zeros((T, -(-T // 32) * 32), dtype=np.uint8)
    padded[:, :T] = C
    bits = torch.from_numpy(np.packbits(padded, axis=1, bitorder="little").view(np.int32).copy()).to(DEV)
    both(wl.scaled(wl.config(2), (T,), topk=6, heads=4, kv_heads=2, needles_per_kv_head=2), mask_bits=bits)
    print("[static] the first shape again", flush=True)
    both(w1)


def test_sizes_beyond_the_scratch_are_refused_before_any_launch():
    lib = binding.load()
    # config 2's own shape fits (its workspace is below the limit) ...
    s = binding.StreamShape()
    s.heads, s.kv_heads, s.head_dim, s.block, s.dtype, s.batch, s.T = 32, 8, 128, 64, binding.STREAM_BF16, 1, 32768
    assert lib.stream_prune_workspace_bytes(ctypes.byref(s), 16) <= binding.STATIC_SCRATCH_BYTES
    # ... the headline shape does not: refused with the workspace status, pointers never looked at
    s.T = 131072
    assert lib.stream_prune_workspace_bytes(ctypes.byref(s), 32) > binding.STATIC_SCRATCH_BYTES
    fake = ctypes.c_void_p(4096)
    rc = lib.stream_prune_static(fake, fake, ctypes.byref(s), 32, None, 32, fake, fake, None, None, None)
    assert rc == binding.STREAM_EWORKSPACE
    assert lib.stream_prune_static(None, fake, ctypes.byref(s), 32, None, 32, fake, fake, None, None, None) == binding.STREAM_EINVAL


def test_under_graph_capture():
    """What the entry point is for: recorded into a HIP graph (after one call outside the capture,
    which looks up the scratch on this device) and replayed with new inputs written into the
    captured buffers and eager work in between; every replay equals stream_prune run eagerly."""
    w = wl.scaled(wl.config(2), (64 * 50 + 9,), topk=8, heads=8, kv_heads=2, needles_per_kv_head=2)
    inputs = [wl.make_inputs(w.with_layer(l), with_v=False) for l in range(3)]
    Qs, Ks = (torch.empty_like(t, device=DEV) for t in inputs[0][:2])
    eager = []
    for (Q, K, _, _) in inputs:
        r = binding.stream_prune(Q.to(DEV), K.to(DEV), w.heads, w.kv_heads, w.block, w.topk[0], want_score=True)
        torch.cuda.synchronize()
        eager.append({k: r[k].clone() for k in ("idx", "cnt", "score")})
    out = {k: torch.empty_like(v) for k, v in eager[0].items()}
    Qs.copy_(inputs[0][0]); Ks.copy_(inputs[0][1])
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        binding.stream_prune_static(Qs, Ks, w.heads, w.kv_heads, w.block, w.topk[0], out)
    torch.cuda.current_stream().wait_stream(s)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        binding.stream_prune_static(Qs, Ks, w.heads, w.kv_heads, w.block, w.topk[0], out)
    for rep in range(5):
        l = rep % 3
        Qs.copy_(inputs[l][0]); Ks.copy_(inputs[l][1])         # eager work between replays
        g.replay()
        torch.cuda.synchronize()
        for key in ("idx", "cnt", "score"):
            assert torch.equal(out[key], eager[l][key]), (rep, key)
        out["idx"].fill_(-7)
        out["cnt"].fill_(-7)
