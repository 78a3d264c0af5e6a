"""stream_mask_diff against oracle/mask_diff.py, bit-exact, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle.mask_diff import mask_diff
from paper_2510_19875_amd import binding, workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def lists(rng, rows, k, N):
    idx = np.full((rows, k), -1, dtype=np.int32)
    cnt = np.minimum(rng.integers(0, k + 1, size=rows), N).astype(np.int32)
    for r in range(rows):
        idx[r, :cnt[r]] = np.sort(rng.choice(N, size=int(cnt[r]), replace=False))
    return idx, cnt


def compare(ia, ca, sa, ib, cb):
    t = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    r = binding.stream_mask_diff(t(ia), t(ca), t(sa), t(ib), t(cb))
    torch.cuda.synchronize()
    eo, ec, ew = mask_diff(ia.reshape(-1, ia.shape[-1]), ca.reshape(-1),
                           None if sa is None else sa.reshape(-1, ia.shape[-1]),
                           ib.reshape(-1, ib.shape[-1]), cb.reshape(-1))
    np.testing.assert_array_equal(r["idx"].cpu().numpy().reshape(eo.shape), eo)
    np.testing.assert_array_equal(r["cnt"].cpu().numpy().reshape(ec.shape), ec)
    if sa is not None:
        np.testing.assert_array_equal(r["weight"].cpu().numpy().reshape(ew.shape), ew.astype(np.float32))
    else:
        assert r["weight"] is None


@pytest.mark.parametrize("ka,kb,N", [(1, 1, 3), (6, 3, 32), (8, 8, 10), (32, 16, 2048), (64, 64, 100), (5, 64, 70), (64, 1, 64),
                                      (65, 3, 300), (200, 512, 600), (512, 512, 513), (7, 100, 40), (300, 64, 5000)])
def test_random_lists(ka, kb, N):
    rng = np.random.default_rng(ka * 1000 + kb)
    rows = 1001
    ia, ca = lists(rng, rows, ka, N)
    ib, cb = lists(rng, rows, kb, N)
    sa = rng.standard_normal((rows, ka)).astype(np.float32)
    compare(ia, ca, sa, ib, cb)
    compare(ia, ca, None, ib, cb)


def test_degenerate():
    rng = np.random.default_rng(9)
    ia, ca = lists(rng, 64, 8, 20)
    sa = rng.standard_normal((64, 8)).astype(np.float32)
    compare(ia, ca, sa, ia.copy(), ca.copy())                        # a \\ a: empty everywhere
    compare(ia, ca, sa, ia.copy(), np.zeros_like(ca))                # a \\ {}: a
    compare(ia, np.zeros_like(ca), sa, ia.copy(), ca.copy())         # {} \\ b: empty
    e = torch.zeros((0, 8), dtype=torch.int32, device=DEV)
    c = torch.zeros((0,), dtype=torch.int32, device=DEV)
    binding.stream_mask_diff(e, c, None, e.clone(), c.clone())       # no rows: no-op


def test_on_pruned_masks_paper_sizes_and_config3_shape():
    """k_success = 6 against k_fail = 3 at T = 1000, b = 32 (the sizes of Section 4.2.2), and a
    GQA case with the sweep entry point supplying both masks; 3-D inputs [H, NB, k]."""
    for (T, b, ks, kf, H, Hkv) in ((1000, 32, 6, 3, 4, 4), (64 * 300 + 11, 64, 32, 16, 8, 2)):
        w = wl.scaled(wl.config(2), (T,), topk=ks, heads=H, kv_heads=Hkv, block=b, needles_per_kv_head=2)
        Q, K, _, _ = wl.make_inputs(w, with_v=False)
        r = binding.stream_prune_multi(Q.to(DEV), K.to(DEV), H, Hkv, b, [ks, kf], want_score=True)
        ia = r["idx"][:, 0].contiguous(); ca = r["cnt"][:, 0].contiguous(); sa = r["score"][:, 0].contiguous()
        ib = r["idx"][:, 1, :, :kf].contiguous(); cb = r["cnt"][:, 1].contiguous()
        compare(ia.cpu().numpy(), ca.cpu().numpy(), sa.cpu().numpy(), ib.cpu().numpy(), cb.cpu().numpy())
        d = binding.stream_mask_diff(ia, ca, sa, ib, cb)
        n = int(d["cnt"].sum().item())
        print(f"[diff] T={T} k={ks}\\\\{kf}: {n} of {int(ca.sum().item())} connections remain", flush=True)
        assert 0 < n < int(ca.sum().item())


def test_full_size_sampled_rows():
    rows, ka, kb, N = 1 << 21, 32, 16, 2048
    g = torch.Generator(device=DEV); g.manual_seed(7)
    # ascending distinct lists: sorted random offsets on a stride-64 grid plus a row shift
    base = torch.arange(ka, device=DEV, dtype=torch.int32) * (N // ka)
    ia = (base[None, :] + torch.randint(0, N // ka, (rows, ka), device=DEV, generator=g, dtype=torch.int32)).contiguous()
    ib = ia[:, ::2].contiguous().clone()
    flip = torch.rand((rows, kb), device=DEV, generator=g) < 0.5
    ib = torch.where(flip & (ib % (N // ka) != 0), ib - 1, ib).contiguous()    # half the entries moved off a's
    ca = torch.randint(0, ka + 1, (rows,), device=DEV, generator=g, dtype=torch.int32)
    cb = torch.randint(0, kb + 1, (rows,), device=DEV, generator=g, dtype=torch.int32)
    sa = torch.randn((rows, ka), device=DEV, generator=g)
    r = binding.stream_mask_diff(ia, ca, sa, ib, cb)
    torch.cuda.synchronize()
    pick = torch.from_numpy(np.unique(np.concatenate([[0, rows - 1], np.random.default_rng(1).integers(0, rows, 2000)]))).to(DEV)
    h = lambda t: t[pick].cpu().numpy()
    eo, ec, ew = mask_diff(h(ia), h(ca), h(sa), h(ib), h(cb))
    np.testing.assert_array_equal(h(r["idx"]), eo)
    np.testing.assert_array_equal(h(r["cnt"]), ec)
    np.testing.assert_array_equal(h(r["weight"]), ew.astype(np.float32))
    assert int((r["cnt"] > ca).sum().item()) == 0
