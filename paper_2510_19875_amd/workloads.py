"""Seeded synthetic inputs for the Stream pruning / sparse-attention path.

This module only *makes data*: Gaussian Q/K/V, rotary position embedding applied
to them, and planted structure (an attention sink at token 0, needle keys, a
local diagonal bias, clustered anchor keys).  It holds none of the method's
arithmetic (no block scores, no top-k, no softmax) and is the only module the
CPU oracle's tests and the HIP path's tests/bench have in common.

The five named workloads stand in, by shape only, for the paper's evaluation
inputs (needle-in-a-haystack contexts of 1k-20k tokens and chain-of-thought
traces of 3k-20k tokens, Section 4); none of those datasets' items are used.

Tensors are laid out [heads, T_total, head_dim] (queries) and
[kv_heads, T_total, head_dim] (keys, values); a ragged batch is packed along the
token axis and described by `cu_seqlens`.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field, replace
from typing import Dict, List, Optional, Tuple

import torch

BASE_SEED = 251019875


@dataclass(frozen=True)
class Workload:
    name: str
    seq_lens: Tuple[int, ...]
    heads: int
    kv_heads: int
    head_dim: int
    dtype: str  # "f32" | "bf16"
    block: int
    topk: Tuple[int, ...]  # one per sequence
    seed: int
    sigma: float = 1.0  # per-component std of the Gaussian base
    rope_theta: Optional[float] = 500000.0
    sink_gain: float = 4.0
    needles_per_kv_head: int = 0
    needle_gain: float = 3.0
    needles_on_partition: bool = False  # place needle blocks at multiples of ceil(N/k)
    diag_beta: float = 0.0  # local diagonal bias strength (in units of the typical row norm)
    diag_period: int = 1024
    anchors_per_seq: int = 0
    anchor_gain: float = 3.0
    anchor_query_component: float = 2.0

    @property
    def T(self) -> int:
        return int(sum(self.seq_lens))

    @property
    def batch(self) -> int:
        return len(self.seq_lens)

    @property
    def cu_seqlens(self) -> List[int]:
        out = [0]
        for L in self.seq_lens:
            out.append(out[-1] + int(L))
        return out

    @property
    def blocks_per_seq(self) -> List[int]:
        return [(L + self.block - 1) // self.block for L in self.seq_lens]

    @property
    def total_blocks(self) -> int:
        return sum(self.blocks_per_seq)

    @property
    def topk_max(self) -> int:
        return max(self.topk)

    @property
    def torch_dtype(self) -> torch.dtype:
        return {"f32": torch.float32, "bf16": torch.bfloat16}[self.dtype]

    def with_layer(self, layer: int) -> "Workload":
        """Same shape, independently seeded (the 32-layer run of config 3)."""
        return replace(self, seed=self.seed + 1000 * layer, name=f"{self.name}/layer{layer}")


def retained_fraction_topk(n_blocks: int) -> int:
    """Per-sequence k for the reasoning-trace workload: about 1-3 % of the causal blocks.

    With k blocks kept per row, R = k*N - k(k-1)/2 of the N(N+1)/2 causal blocks
    survive (about 2k/(N+1)); k = round(N/100) keeps that inside 1.3-2.6 % for
    N in [128, 512].
    """
    return max(1, int(math.floor(n_blocks / 100.0 + 0.5)))


def config(i: int) -> Workload:
    """The five named workloads (1-based)."""
    if i == 1:
        return Workload(name="cfg1_T4096_mha8_d64_f32", seq_lens=(4096,), heads=8, kv_heads=8,
                        head_dim=64, dtype="f32", block=64, topk=(8,), seed=BASE_SEED + 1,
                        sigma=1.0 / 8.0, rope_theta=None, needles_per_kv_head=4,
                        needles_on_partition=True, diag_beta=2.0)
    if i == 2:
        return Workload(name="cfg2_T32768_gqa32x8_d128_bf16", seq_lens=(32768,), heads=32,
                        kv_heads=8, head_dim=128, dtype="bf16", block=64, topk=(16,),
                        seed=BASE_SEED + 2, needles_per_kv_head=16)
    if i == 3:
        return Workload(name="cfg3_T131072_gqa32x8_d128_bf16", seq_lens=(131072,), heads=32,
                        kv_heads=8, head_dim=128, dtype="bf16", block=64, topk=(32,),
                        seed=BASE_SEED + 3, needles_per_kv_head=16)
    if i == 4:
        return Workload(name="cfg4_T1048576_gqa32x8_d128_bf16_b128", seq_lens=(1048576,),
                        heads=32, kv_heads=8, head_dim=128, dtype="bf16", block=128, topk=(64,),
                        seed=BASE_SEED + 4, needles_per_kv_head=64)
    if i == 5:
        g = torch.Generator().manual_seed(BASE_SEED + 5)
        lens = tuple(int(x) for x in torch.randint(8192, 32768 + 1, (8,), generator=g))
        ks = tuple(retained_fraction_topk((L + 63) // 64) for L in lens)
        return Workload(name="cfg5_ragged8_gqa28x4_d128_bf16", seq_lens=lens, heads=28,
                        kv_heads=4, head_dim=128, dtype="bf16", block=64, topk=ks,
                        seed=BASE_SEED + 5, anchors_per_seq=20)
    raise ValueError(f"no config {i}")


def scaled(w: Workload, seq_lens, topk=None, **kw) -> Workload:
    """Same recipe at another size (parity cases the oracle finishes quickly)."""
    seq_lens = tuple(int(x) for x in seq_lens)
    if topk is None:
        topk = tuple(w.topk[0] for _ in seq_lens)
    elif isinstance(topk, int):
        topk = tuple(topk for _ in seq_lens)
    name = kw.pop("name", f"{w.name}@{'+'.join(map(str, seq_lens))}")
    return replace(w, seq_lens=seq_lens, topk=tuple(topk), name=name, **kw)


def _gen(device, seed: int, tensor_id: int, head: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed((seed * 1000003 + tensor_id * 7919 + head) & 0x7FFFFFFFFFFFFFFF)
    return g


def _rope_(x: torch.Tensor, pos: torch.Tensor, theta: float) -> torch.Tensor:
    """Rotary embedding, half-split pairing (dim i pairs with i + d/2), angles in fp64."""
    d = x.shape[-1]
    half = d // 2
    inv = theta ** (-2.0 * torch.arange(half, dtype=torch.float64, device=x.device) / d)
    ang = pos.to(torch.float64)[:, None] * inv[None, :]
    c, s = torch.cos(ang), torch.sin(ang)
    x1, x2 = x[:, :half].clone(), x[:, half:].clone()
    x[:, :half] = x1 * c - x2 * s
    x[:, half:] = x2 * c + x1 * s
    return x


def make_inputs(w: Workload, device="cpu", with_v: bool = True):
    """Return (Q, K, V, meta).  Values are generated in fp64, cast to the workload dtype;
    the cast values are the inputs for every consumer."""
    dev = torch.device(device)
    T, d, H, Hkv = w.T, w.head_dim, w.heads, w.kv_heads
    g_sz = H // Hkv
    dt = w.torch_dtype
    cu = w.cu_seqlens
    pos = torch.cat([torch.arange(L, device=dev) for L in w.seq_lens])
    typ_norm = w.sigma * math.sqrt(d)

    Q = torch.empty((H, T, d), dtype=dt, device=dev)
    K = torch.empty((Hkv, T, d), dtype=dt, device=dev)
    V = torch.empty((Hkv, T, d), dtype=dt, device=dev) if with_v else None
    meta: Dict[str, object] = {"needles": [], "anchors": [], "cu_seqlens": cu}

    # host-side choices (positions), independent of device
    hg = torch.Generator().manual_seed(w.seed * 31 + 17)

    # shared directions: diagonal-bias plane, per-sequence anchor direction
    plane = None
    if w.diag_beta > 0:
        a = torch.randn(2, d, generator=hg, dtype=torch.float64)
        e0 = a[0] / a[0].norm()
        e1 = a[1] - (a[1] @ e0) * e0
        e1 = e1 / e1.norm()
        ph = 2.0 * math.pi * pos.to(torch.float64).cpu() / w.diag_period
        plane = (torch.cos(ph)[:, None] * e0[None, :] + torch.sin(ph)[:, None] * e1[None, :])
        plane = (w.diag_beta * typ_norm * plane).to(dev)
    anchor_dirs, anchor_pos = [], []
    for s, L in enumerate(w.seq_lens):
        if w.anchors_per_seq > 0:
            u = torch.randn(d, generator=hg, dtype=torch.float64)
            anchor_dirs.append((u / u.norm()).to(dev))
            p = torch.randperm(L - 1, generator=hg)[: w.anchors_per_seq] + 1
            anchor_pos.append(sorted(int(x) for x in p))
    meta["anchors"] = anchor_pos

    def base(tensor_id, head):
        x = torch.randn((T, d), generator=_gen(dev, w.seed, tensor_id, head),
                        dtype=torch.float32, device=dev).to(torch.float64) * w.sigma
        return x

    # queries (kept in fp64 per head only as long as needed)
    for h in range(H):
        x = base(0, h)
        if w.rope_theta:
            _rope_(x, pos, w.rope_theta)
        if plane is not None:
            x += plane
        for s in range(w.batch):
            if w.anchors_per_seq > 0:
                x[cu[s]:cu[s + 1]] += w.anchor_query_component * w.sigma * anchor_dirs[s][None, :]
        Q[h] = x.to(dt)

    for kvh in range(Hkv):
        x = base(1, kvh)
        if w.rope_theta:
            _rope_(x, pos, w.rope_theta)
        if plane is not None:
            x += plane
        for s, L in enumerate(w.seq_lens):
            x[cu[s]] *= w.sink_gain  # attention sink: first key of every sequence
            nb = (L + w.block - 1) // w.block
            # needles: a key far in the past aligned with one later query of the group
            for _ in range(w.needles_per_kv_head):
                if L < 6 * w.block:
                    break
                t_q = int(torch.randint(L // 2, L, (1,), generator=hg))
                hi = t_q - 2 * w.block
                if w.needles_on_partition:
                    step = -(-nb // w.topk[s])  # ceil(N/k): blocks that are representatives at every level
                    cands = [r for r in range(step, nb, step) if (r + 1) * w.block - 1 < hi]
                    if not cands:
                        continue
                    r = cands[int(torch.randint(0, len(cands), (1,), generator=hg))]
                    t_n = r * w.block + int(torch.randint(0, w.block, (1,), generator=hg))
                else:
                    t_n = int(torch.randint(1, hi, (1,), generator=hg))
                h = kvh * g_sz + int(torch.randint(0, g_sz, (1,), generator=hg))
                qv = Q[h, cu[s] + t_q].to(torch.float64)
                x[cu[s] + t_n] = w.needle_gain * typ_norm * qv / qv.norm()
                meta["needles"].append({"seq": s, "kv_head": kvh, "head": h, "t_q": t_q, "t_n": t_n})
            if w.anchors_per_seq > 0:
                for t_a in anchor_pos[s]:
                    noise = torch.randn(d, generator=hg, dtype=torch.float64).to(dev) * w.sigma
                    x[cu[s] + t_a] = w.anchor_gain * typ_norm * anchor_dirs[s] + noise
        K[kvh] = x.to(dt)
        if with_v:
            V[kvh] = base(2, kvh).to(dt)
    return Q, K, V, meta
