"""Input generators: shapes, determinism, planted structure (no GPU)."""
import numpy as np
import torch

from paper_2510_19875_amd import workloads as wl


def test_named_configs_have_the_stated_shapes():
    c = [wl.config(i) for i in range(1, 6)]
    assert (c[0].T, c[0].heads, c[0].kv_heads, c[0].head_dim, c[0].dtype, c[0].block, c[0].topk) == \
        (4096, 8, 8, 64, "f32", 64, (8,))
    assert (c[1].T, c[1].heads, c[1].kv_heads, c[1].block, c[1].topk) == (32768, 32, 8, 64, (16,))
    assert (c[2].T, c[2].topk, c[2].total_blocks) == (131072, (32,), 2048)
    assert (c[3].T, c[3].block, c[3].topk, c[3].total_blocks) == (1048576, 128, (64,), 8192)
    assert c[4].batch == 8 and all(8192 <= L <= 32768 for L in c[4].seq_lens)
    assert (c[4].heads, c[4].kv_heads) == (28, 4)
    for L, k in zip(c[4].seq_lens, c[4].topk):
        N = -(-L // 64)
        frac = (k * N - k * (k - 1) / 2) / (N * (N + 1) / 2)
        assert 0.01 <= frac <= 0.03


def test_small_variants_are_deterministic_and_structured():
    w = wl.scaled(wl.config(2), (1024,), topk=4, heads=4, kv_heads=2, needles_per_kv_head=2)
    Q, K, V, meta = wl.make_inputs(w)
    Q2, K2, V2, _ = wl.make_inputs(w)
    assert torch.equal(Q, Q2) and torch.equal(K, K2) and torch.equal(V, V2)
    assert Q.shape == (4, 1024, 128) and K.shape == (2, 1024, 128) and Q.dtype == torch.bfloat16
    Q3, _, _, _ = wl.make_inputs(w.with_layer(1))
    assert not torch.equal(Q, Q3)
    # sink: first key is 4x a typical key
    n0 = K[:, 0].float().norm(dim=-1)
    nt = K[:, 1:].float().norm(dim=-1).median()
    assert torch.all(n0 > 3 * nt)
    # needles point along their query
    for nd in meta["needles"]:
        q = Q[nd["head"], nd["t_q"]].float()
        k = K[nd["kv_head"], nd["t_n"]].float()
        assert torch.dot(q, k) / (q.norm() * k.norm()) > 0.99
        assert nd["t_n"] < nd["t_q"] - 2 * w.block


def test_ragged_anchor_workload_small():
    w = wl.scaled(wl.config(5), (300, 515), topk=(1, 2), heads=4, kv_heads=2, anchors_per_seq=3)
    Q, K, V, meta = wl.make_inputs(w)
    assert Q.shape[1] == 815 and w.total_blocks == 5 + 9
    cu = w.cu_seqlens
    for s in range(2):
        a = meta["anchors"][s]
        assert len(a) == 3
        ka = K[:, [cu[s] + t for t in a]].float()
        qs = Q[:, cu[s]:cu[s + 1]].float()
        # anchors collect a positive product from (nearly) every query of their sequence
        dots = torch.einsum("htd,had->hta", qs[:2], ka[:1].expand(2, -1, -1))
        assert (dots > 0).float().mean() > 0.95


def test_rope_is_a_rotation_of_pairs():
    x = torch.randn(16, 8, dtype=torch.float64)
    y = wl._rope_(x.clone(), torch.arange(16), 500000.0)
    np.testing.assert_allclose(y.norm(dim=-1).numpy(), x.norm(dim=-1).numpy(), rtol=1e-12)
    assert torch.equal(y[0], x[0])  # position 0 is unrotated
