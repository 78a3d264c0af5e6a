"""stream_select_update (top-k selection + node update of Alg. 2 as a pass of its own) against
oracle/select_update.py, bit-exact, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle.select_update import select_update
from paper_2510_19875_amd import binding

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def make_case(rows, kmax, seed, ties=True, dead=0.2, full=False):
    """Random rows: disjoint ascending node ranges of sizes 1..6, live counts 0..kmax, scores
    on a coarse grid (many exact ties, signed zeros), a share of -inf branches."""
    rng = np.random.default_rng(seed)
    sizes = rng.integers(1, 7, size=(rows, kmax))
    starts = np.cumsum(sizes, axis=1) - sizes
    nf = starts.astype(np.int32)
    nl = (starts + sizes - 1).astype(np.int32)
    nc = (np.full(rows, kmax) if full else rng.integers(0, kmax + 1, size=rows)).astype(np.int32)
    if ties:
        sc = (rng.integers(-3, 4, size=(rows, 2 * kmax)) * 0.5).astype(np.float32)
        sc[rng.random(sc.shape) < 0.1] = -0.0
    else:
        sc = rng.standard_normal((rows, 2 * kmax)).astype(np.float32)
    sc[rng.random(sc.shape) < dead] = -np.inf
    return sc, nf, nl, nc


def run_gpu(sc, nf, nl, nc, k):
    t = [torch.from_numpy(a.copy()).to(DEV) for a in (sc, nf, nl, nc)]
    binding.stream_select_update(t[0], t[1], t[2], t[3], k)
    torch.cuda.synchronize()
    return [x.cpu().numpy() for x in t[1:]]


def compare(sc, nf, nl, nc, k):
    gf, gl, gc = run_gpu(sc, nf, nl, nc, k)
    of, ol, oc = select_update(sc, nf, nl, nc, k)
    np.testing.assert_array_equal(gc, oc)
    live = np.arange(nf.shape[1])[None, :] < oc[:, None]
    np.testing.assert_array_equal(gf[live], of[live])
    np.testing.assert_array_equal(gl[live], ol[live])
    # slots after the new count are left as they were
    np.testing.assert_array_equal(gf[~live], nf[~live])
    np.testing.assert_array_equal(gl[~live], nl[~live])


@pytest.mark.parametrize("kmax,k", [(1, 1), (2, 1), (5, 3), (8, 8), (16, 7), (32, 32), (33, 20), (64, 64), (64, 1),
                                    (65, 65), (65, 1), (200, 77), (512, 512), (512, 300), (100, 3)])
@pytest.mark.parametrize("ties", [True, False])
def test_matches_oracle(kmax, k, ties):
    rows = 1003                                     # not a multiple of the 4 rows per workgroup
    compare(*make_case(rows, kmax, seed=kmax * 100 + k + int(ties), ties=ties), k)


def test_degenerate_rows():
    kmax, k = 8, 4
    sc, nf, nl, nc = make_case(64, kmax, seed=5)
    sc[0:8] = -np.inf                               # nothing valid: count 0
    nc[8:16] = 0                                    # no live node
    sc[16:24] = 1.5                                 # all equal: the k lowest positions win
    nc[16:24] = kmax
    nf[24:32] = nl[24:32]                           # single-block nodes: left child empty
    nc[32] = 99                                     # out-of-range count is clamped
    of = nf.copy(); ol = nl.copy(); oc = nc.copy(); oc[32] = kmax
    gf, gl, gc = run_gpu(sc, nf, nl, nc, k)
    ef, el, ec = select_update(sc, of, ol, oc, k)
    np.testing.assert_array_equal(gc, ec)
    assert (gc[0:16] == 0).all()
    live = np.arange(kmax)[None, :] < ec[:, None]
    np.testing.assert_array_equal(gf[live], ef[live])
    np.testing.assert_array_equal(gl[live], el[live])


def test_empty_call_and_repeated_levels():
    z = torch.zeros((0, 16), dtype=torch.float32, device=DEV)
    zi = torch.zeros((0, 8), dtype=torch.int32, device=DEV)
    binding.stream_select_update(z, zi, zi.clone(), torch.zeros((0,), dtype=torch.int32, device=DEV), 4)
    # several levels in a row on the same node tensors, like the loop of Alg. 2
    kmax, k, rows = 16, 16, 257
    rng = np.random.default_rng(11)
    nf = np.tile((np.arange(kmax) * 64).astype(np.int32), (rows, 1))
    nl = nf + 63
    nc = np.full(rows, kmax, dtype=np.int32)
    tf, tl, tc = [torch.from_numpy(a.copy()).to(DEV) for a in (nf, nl, nc)]
    for level in range(7):
        sc = rng.standard_normal((rows, 2 * kmax)).astype(np.float32)
        sc[rng.random(sc.shape) < 0.3] = -np.inf
        binding.stream_select_update(torch.from_numpy(sc).to(DEV), tf, tl, tc, k)
        nf, nl, nc = select_update(sc, nf, nl, nc, k)
        torch.cuda.synchronize()
        gc = tc.cpu().numpy()
        np.testing.assert_array_equal(gc, nc)
        live = np.arange(kmax)[None, :] < nc[:, None]
        np.testing.assert_array_equal(tf.cpu().numpy()[live], nf[live])
        np.testing.assert_array_equal(tl.cpu().numpy()[live], nl[live])
        nf = tf.cpu().numpy().copy(); nl = tl.cpu().numpy().copy()


def test_full_size_sampled_rows():
    """The size the bench measures: 2M rows at k = kmax = 32 (1.5 GB of traffic); 2000 sampled rows."""
    rows, kmax, k = 1 << 21, 32, 32
    g = torch.Generator(device=DEV); g.manual_seed(123)
    sc = torch.randn((rows, 2 * kmax), device=DEV, generator=g)
    sc = torch.where(torch.rand(sc.shape, device=DEV, generator=g) < 0.1, torch.full_like(sc, -float("inf")), sc)
    sc = (sc * 4).round() / 4                        # ties
    nf = (torch.arange(kmax, device=DEV, dtype=torch.int32) * 64).repeat(rows, 1).contiguous()
    nl = nf + 63
    nc = torch.full((rows,), kmax, dtype=torch.int32, device=DEV)
    pick = np.unique(np.concatenate([[0, 1, rows - 1], np.random.default_rng(3).integers(0, rows, 2000)]))
    before = [t[pick].cpu().numpy() for t in (sc, nf, nl, nc)]
    binding.stream_select_update(sc, nf, nl, nc, k)
    torch.cuda.synchronize()
    of, ol, oc = select_update(*before, k)
    gf, gl, gc = [t[pick].cpu().numpy() for t in (nf, nl, nc)]
    np.testing.assert_array_equal(gc, oc)
    live = np.arange(kmax)[None, :] < oc[:, None]
    np.testing.assert_array_equal(gf[live], of[live])
    np.testing.assert_array_equal(gl[live], ol[live])
    # law at full size: count = min(k, number of valid branches)
    assert int(nc.max()) <= k and int(nc.min()) >= 0


def test_more_rows_than_one_launch_addresses():
    """A launch of the narrow kernel addresses its rows with 32-bit byte offsets (2 GiB of scores);
    the entry point takes more rows in further launches.  4.3 M rows at kmax = 64: rows on both
    sides of the seam, the last rows and random ones against the oracle."""
    kmax, k = 64, 24
    seam = (1 << 31) // (8 * kmax)                   # rows of the first launch
    rows = seam + 100_003
    g = torch.Generator(device=DEV); g.manual_seed(77)
    sc = torch.randn((rows, 2 * kmax), device=DEV, generator=g)
    sc = torch.where(torch.rand(sc.shape, device=DEV, generator=g) < 0.2, torch.full_like(sc, -float("inf")), sc)
    sc = (sc * 2).round() / 2                        # ties
    nf = (torch.arange(kmax, device=DEV, dtype=torch.int32) * 8).repeat(rows, 1).contiguous()
    nl = nf + torch.randint(0, 8, (rows, kmax), device=DEV, generator=g, dtype=torch.int32)
    nc = torch.randint(0, kmax + 1, (rows,), device=DEV, generator=g, dtype=torch.int32)
    pick = np.unique(np.concatenate([np.arange(0, 8), np.arange(seam - 40, seam + 40), np.arange(rows - 40, rows),
                                     np.random.default_rng(5).integers(0, rows, 1500)]))
    before = [t[pick].cpu().numpy() for t in (sc, nf, nl, nc)]
    print(f"[select] {rows} rows, kmax {kmax}: seam at row {seam}, {len(pick)} rows against the oracle", flush=True)
    binding.stream_select_update(sc, nf, nl, nc, k)
    torch.cuda.synchronize()
    of, ol, oc = select_update(*before, k)
    gf, gl, gc = [t[pick].cpu().numpy() for t in (nf, nl, nc)]
    np.testing.assert_array_equal(gc, oc)
    live = np.arange(kmax)[None, :] < oc[:, None]
    np.testing.assert_array_equal(gf[live], of[live])
    np.testing.assert_array_equal(gl[live], ol[live])
    np.testing.assert_array_equal(gf[~live], before[1][~live])
    assert int(nc.max()) <= k and int(nc.min()) >= 0
