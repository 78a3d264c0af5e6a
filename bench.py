"""Benchmark of the Stream hot path on one MI355X.

One step = one pass of the whole path over one layer's synthetic Q, K, V at the headline
workload (T = 131072, 32 query / 8 KV heads, head_dim 128, bf16, block 64, top-k 32):
stream_prune (K tile packing + the refinement levels, fused select/compaction/emit) followed by
stream_sparse_attn with the received-mass read-out.  Layers are independently seeded and
resident in HBM before the timed region; consecutive steps walk through them.

Prints ONE JSON line: whole-path throughput in query-tokens x heads per second, the roofline of
the dominant kernel (the level scorer: algorithmic FLOP of the block scores it had to compute /
its launch time, measured with HIP events recorded on the launch stream inside the timed
region, against the dense bf16 MFMA peak), and the CPU oracle timed on a bounded row sample.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_MFMA_TFLOPS = 2500.0   # MI355X dense bf16
PEAK_FP32_MFMA_TFLOPS = 157.3    # MI355X fp32 (the contraction of the fp32 workload)


def mfma_peak(dtype: str) -> float:
    return PEAK_BF16_MFMA_TFLOPS if dtype == "bf16" else PEAK_FP32_MFMA_TFLOPS
PEAK_HBM_GBS = 8000.0
# HBM-side bytes per launch of the dominant kernel come from the rocprofv3 --pmc summary under
# profiles/ (FETCH_SIZE and WRITE_SIZE runs, scaled by what the same counters read for a plain copy
# of known size).  The summary records the hash of the kernel sources it was taken with; when the
# sources on disk differ, the figure is not that of the binary being timed and `traffic` is null.
PMC_SUMMARY = os.path.join(ROOT, "profiles", "cfg3_pmc_counters.txt")
LEVEL_KERNEL_SOURCES = ["stream_prune.hip", "stream_prune.h", "stream_select.h", "stream_mfma.h", "stream_common.h"]


def kernel_source_hash(files=LEVEL_KERNEL_SOURCES) -> str:
    import hashlib

    h = hashlib.sha256()
    for f in files:
        with open(os.path.join(ROOT, "paper_2510_19875_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def level_kernel_traffic(workload: str):
    """Bytes per launch from the line `traffic level_kernel <workload> <bytes> sources <hash>` of the
    counter summary, or None when there is no such line for these sources."""
    try:
        with open(PMC_SUMMARY) as fh:
            for line in fh:
                t = line.split()
                if len(t) >= 6 and t[0] == "traffic" and t[1] == "level_kernel" and t[2] == workload:
                    return float(t[3]) if t[5] == kernel_source_hash() else None
    except OSError:
        pass
    return None


class HipEvents:
    """hipEvent_t handles for the per-level timing hooks of stream_prune (plumbing only)."""

    def __init__(self, n):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.arr = (ctypes.c_void_p * n)()
        for i in range(n):
            ev = ctypes.c_void_p()
            rc = self.hip.hipEventCreate(ctypes.byref(ev))
            assert rc == 0, f"hipEventCreate -> {rc}"
            self.arr[i] = ev

    def elapsed_ms(self, a, b):
        ms = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), ctypes.c_void_p(self.arr[a]),
                                          ctypes.c_void_p(self.arr[b]))
        assert rc == 0, f"hipEventElapsedTime -> {rc}"
        return ms.value


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=32)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=3, help="named workload (default: the headline one)")
    ap.add_argument("--layers", type=int, default=0, help="resident input layers (default min(steps, 32))")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-select", action="store_true", help="skip the standalone select-kernel measurement")
    ap.add_argument("--no-sweep", action="store_true", help="skip the k-sweep (stream_prune_multi) measurement")
    ap.add_argument("--dense-reference", action="store_true",
                    help="also time PyTorch's dense causal attention on the same tensors (context only)")
    ap.add_argument("--levels-per-launch", type=int, default=0,
                    help="refinement levels per kernel launch (0 = library default: all in one)")
    ap.add_argument("--cpu-rows", type=int, default=1536)
    ap.add_argument("--probes", action="store_true",
                    help="run only the micro-benchmarks behind the roofline statements (MFMA-only rate, "
                         "shader clock under matrix load, tile-gather bandwidth) and print them as JSON")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding code); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    if args.probes:
        print(json.dumps(probes()))
        return

    import numpy as np
    import torch

    from paper_2510_19875_amd import binding, workloads as wl

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    w = wl.config(args.config)
    if w.batch != 1:
        cu, topk = w.cu_seqlens, list(w.topk)
    else:
        cu, topk = None, w.topk[0]
    H, Hkv, b, d, T = w.heads, w.kv_heads, w.block, w.head_dim, w.T
    kmax = w.topk_max
    scale = 1.0 / math.sqrt(d)
    n_layers = args.layers or max(1, min(args.steps, 32))
    layers = [wl.make_inputs(w.with_layer(i), device=dev)[:3] for i in range(n_layers)]
    torch.cuda.synchronize()

    NB = w.total_blocks
    out_p = {"idx": torch.empty((H, NB, kmax), dtype=torch.int32, device=dev),
             "cnt": torch.empty((H, NB), dtype=torch.int32, device=dev),
             "score": torch.empty((H, NB, kmax), dtype=torch.float32, device=dev)}
    out_a = {"O": torch.empty((H, T, d), dtype=w.torch_dtype, device=dev),
             "lse": torch.empty((H, T), dtype=torch.float32, device=dev),
             "mass": torch.empty((H, T), dtype=torch.float32, device=dev)}
    ws_p = ws_a = None
    tiles = torch.zeros((1,), dtype=torch.int64, device=dev)

    lpl = args.levels_per_launch

    def step(i, events=None, count_tiles=False):
        nonlocal ws_p, ws_a
        Q, K, V = layers[i % n_layers]
        r = binding.stream_prune(Q, K, H, Hkv, b, topk, cu_seqlens=cu, want_score=True,
                                 workspace=ws_p, out=out_p, level_events=events,
                                 want_tiles=count_tiles, levels_per_launch=lpl)
        ws_p = r["workspace"]
        a = binding.stream_sparse_attn(Q, K, V, H, Hkv, b, out_p["idx"], out_p["cnt"], scale,
                                       cu_seqlens=cu, want_lse=True, want_mass=True,
                                       workspace=ws_a, out=out_a)
        ws_a = a["workspace"]
        return r

    levels = None
    for i in range(args.warmup):
        r = step(i)
        levels = r["levels"]
    if levels is None:
        levels = step(0)["levels"]
    torch.cuda.synchronize()
    torch.cuda.reset_peak_memory_stats()

    # algorithmic work: block scores the path has to compute (those no parent score supplies),
    # counted by the kernels themselves on one untimed pass per resident layer
    tile_counts = []
    for i in range(n_layers):
        r = step(i, count_tiles=True)
        torch.cuda.synchronize()
        tile_counts.append(int(r["tiles"].item()))

    K_steps = args.steps
    ev = HipEvents(2 * levels * K_steps)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(2 * K_steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(K_steps):
        Q, K, V = layers[i % n_layers]
        sub = ctypes.cast(ctypes.byref(ev.arr, 2 * levels * i * ctypes.sizeof(ctypes.c_void_p)),
                          ctypes.POINTER(ctypes.c_void_p * (2 * levels))).contents
        marks[2 * i].record()
        r = binding.stream_prune(Q, K, H, Hkv, b, topk, cu_seqlens=cu, want_score=True,
                                 workspace=ws_p, out=out_p, level_events=sub, levels_per_launch=lpl)
        marks[2 * i + 1].record()
        binding.stream_sparse_attn(Q, K, V, H, Hkv, b, out_p["idx"], out_p["cnt"], scale,
                                   cu_seqlens=cu, want_lse=True, want_mass=True,
                                   workspace=ws_a, out=out_a)
    marks[2 * K_steps].record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    total_s = t1 - t0
    ms_per_step = total_s * 1e3 / K_steps
    prune_ms = [marks[2 * i].elapsed_time(marks[2 * i + 1]) for i in range(K_steps)]
    attn_ms = [marks[2 * i + 1].elapsed_time(marks[2 * i + 2]) for i in range(K_steps)]
    n_launch = 1 if lpl <= 0 else -(-levels // lpl)              # refinement-kernel launches per step
    level_ms = np.array([[ev.elapsed_ms(2 * levels * i + 2 * l, 2 * levels * i + 2 * l + 1)
                          for l in range(n_launch)] for i in range(K_steps)])
    tok_heads = float(T) * H
    value = tok_heads / (ms_per_step * 1e-3)

    Q_BYTES = float(H) * T * d * layers[0][0].element_size()      # Q tile of every row, once per launch
    K_BYTES = float(Hkv) * T * d * layers[0][0].element_size()    # distinct K tiles: 1/64 .. 1/2 of K by level
    retained = float(out_p["cnt"].sum().item())
    attn_flop = retained * 6.0 * b * b * d                        # QK^T + PV + the QK^T of the mass pass
    tile_flop = 2.0 * b * b * d
    flops_per_step = np.array([tile_counts[i % n_layers] for i in range(K_steps)]) * tile_flop
    level_total_s = level_ms.sum() * 1e-3
    launches = n_launch * K_steps
    achieved_tflops = flops_per_step.sum() / level_total_s / 1e12
    peak_mem = torch.cuda.max_memory_allocated()
    tensor_bytes = sum(t.numel() * t.element_size() for t in layers[0]) + \
        sum(t.numel() * t.element_size() for t in list(out_p.values()) + list(out_a.values()))

    result = {
        "metric": "query-tokens·heads/s pruned at T=131k bf16 GQA; % MFMA / HBM peak",
        "value": value,
        "unit": "query-tokens*heads/s",
        "n_gpus": 1,
        "steps": K_steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic",
        "config": {"workload": w.name, "T": T, "heads": H, "kv_heads": Hkv, "head_dim": d,
                   "block": b, "topk": kmax, "resident_layers": n_layers,
                   "step": "stream_prune + stream_sparse_attn (O, lse, mass)"},
        "prune_ms": float(np.mean(prune_ms)),
        "attn_ms": float(np.mean(attn_ms)),
        # one entry per timed step; step i runs the independently seeded layer i % resident_layers
        "per_layer_prune_ms": [round(float(x), 4) for x in prune_ms],
        "per_layer_attn_ms": [round(float(x), 4) for x in attn_ms],
        "prune_only_value": tok_heads / (float(np.mean(prune_ms)) * 1e-3),
        "attn_tflops": attn_flop / (float(np.mean(attn_ms)) * 1e-3) / 1e12,
        "attn_frac_of_mfma_peak": attn_flop / (float(np.mean(attn_ms)) * 1e-3) / 1e12 / mfma_peak(w.dtype),
        "level_kernel_ms": [float(x) for x in level_ms.mean(axis=0)],
        "levels": levels, "level_kernel_launches_per_step": n_launch,
        "tiles_scored_per_step": float(np.mean(tile_counts)),
        "peak_device_bytes": int(peak_mem),
        "workspace_plus_state_bytes": int(ws_p.numel() + ws_a.numel()),
        "tensor_bytes_one_layer": int(tensor_bytes),
        "roofline": {
            "kernel": "level_kernel (branch scorer + top-k select + compaction, all levels of a row per launch)"
                      if n_launch == 1 else
                      "level_kernel (branch scorer + top-k select + in-place compaction)",
            "bound": "mfma",
            "achieved": achieved_tflops,
            "peak": mfma_peak(w.dtype),
            "unit": "TFLOP/s",
            "frac": achieved_tflops / mfma_peak(w.dtype),
            "flop_per_launch": float(flops_per_step.sum() / launches),
            "avg_launch_ms": float(level_ms.sum() / launches),
            "launches": launches,
            "traffic": level_kernel_traffic(w.name) if n_launch == 1 else None,
            "algorithmic_bytes_per_launch": float(Q_BYTES + K_BYTES + H * NB * (8 * kmax + 4)) if n_launch == 1
                                            else float(Q_BYTES + K_BYTES * 0.25 + H * NB * (24 * kmax + 4)),
        },
    }
    if w.batch == 1 and H * NB * NB <= (1 << 31):
        result["list_sharing"] = list_sharing(out_p["idx"], out_p["cnt"], Hkv)
    if not args.no_select:
        result["select_roofline"] = select_standalone(kmax)
    if not args.no_select:
        result["mask_diff_roofline"] = mask_diff_standalone(kmax)
    if not args.no_sweep and w.batch == 1:
        result["k_sweep"] = k_sweep(w, layers[0])
        result["mask_rules"] = mask_rules(w, layers[0], scale)
        result["variable_k"] = variable_k(w, layers[0])
        result["receiver_stats"] = receiver_stats(w, layers[0], scale)
        result["block_shapes"] = block_shapes(w, layers[0], scale)
        result["wide_lists"] = wide_lists(w, layers[0], scale)
        if w.T <= 262144:                                   # (T^2 / 8 bytes of mask)
            result["mask_array"] = mask_array(w, layers[0], scale)
    if args.dense_reference and w.batch == 1:
        result["dense_reference"] = dense_reference(w, layers[0])
    try:
        # what the matrix cores and the memory path deliver on their own on this very box
        result["probes"] = probes()
    except (OSError, RuntimeError) as e:
        result["probes"] = {"error": str(e)}
    if not args.no_cpu_baseline:
        # the step's own outputs for layer 0, taken again after the timed region (with the per-level
        # trace a differing row is certified from), for the row-by-row comparison with the oracle
        Q0, K0, V0 = layers[0]
        gp = binding.stream_prune(Q0, K0, H, Hkv, b, topk, cu_seqlens=cu, want_score=True, want_trace=True,
                                  workspace=ws_p)
        ga = binding.stream_sparse_attn(Q0, K0, V0, H, Hkv, b, gp["idx"], gp["cnt"], scale, cu_seqlens=cu,
                                        want_lse=True, want_mass=True, workspace=ws_a)
        torch.cuda.synchronize()
        result["cpu_baseline"] = cpu_baseline(w, layers[0], args.cpu_rows, scale, gp, ga)
    print(json.dumps(result))


def probes():
    """Micro-benchmarks of csrc/stream_probe.hip (libstream_probe.so): what the matrix cores and
    the vector-memory path deliver on their own, for the tile shapes the level kernel uses."""
    lib = ctypes.CDLL(os.path.join(ROOT, "paper_2510_19875_amd", "libstream_probe.so"))
    lib.stream_probe_run.restype = ctypes.c_int
    lib.stream_probe_run.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.c_int]
    out = (ctypes.c_double * 22)()
    rc = lib.stream_probe_run(out, 22)
    if rc != 0:
        raise RuntimeError(f"stream_probe_run -> {rc}")
    v = list(out)
    res = {"what": "micro-benchmarks: 64x64x128 bf16 tile products on register operands (mfma), shader clock "
                   "during them (shader-clock counter / 100 MHz counter), random 16 KiB tile gathers (gather)",
           "mfma": {}, "gather": []}
    for i, name in enumerate(("2_waves_per_simd_short", "2_waves_per_simd_long", "1_wave_per_simd_short",
                              "1_wave_per_simd_long")):
        res["mfma"][name] = {"tflops": v[2 * i], "frac_of_2500": v[2 * i] / PEAK_BF16_MFMA_TFLOPS,
                             "shader_clock_mhz": v[2 * i + 1]}
    res["mfma"]["2_waves_per_simd_long_zero_operands"] = {"tflops": v[18], "frac_of_2500": v[18] / PEAK_BF16_MFMA_TFLOPS,
                                                          "shader_clock_mhz": v[19]}
    res["mfma"]["2_waves_per_simd_long_16x16x32_shape"] = {"tflops": v[20], "frac_of_2500": v[20] / PEAK_BF16_MFMA_TFLOPS,
                                                           "shader_clock_mhz": v[21]}
    for i in range(5):
        tbs, ws = v[8 + 2 * i], v[9 + 2 * i]
        clk = res["mfma"]["2_waves_per_simd_long"]["shader_clock_mhz"] * 1e6
        res["gather"].append({"working_set_mib": ws / 2 ** 20, "tb_per_s": tbs,
                              "bytes_per_clk_per_cu_at_2400mhz": tbs * 1e12 / 256 / 2.4e9,
                              "bytes_per_clk_per_cu_at_sustained_clock": tbs * 1e12 / 256 / clk if clk else None})
    return res


def list_sharing(idx, cnt, kv_heads):
    """How much the retained lists overlap where the attention kernel could share K/V tiles:
    between the query heads of one key/value head at the same query block, and between adjacent
    query blocks of one head.  Fractions of all list entries."""
    import torch

    H, NB, kmax = idx.shape
    g = H // kv_heads
    live = torch.arange(kmax, device=idx.device)[None, None, :] < cnt[:, :, None]
    pres = torch.zeros((H, NB, NB + 1), dtype=torch.bool, device=idx.device)
    pres.scatter_(2, torch.where(live, idx, torch.full_like(idx, NB)).long(), True)
    pres = pres[:, :, :NB]
    total = float(cnt.sum().item())
    union = float(pres.view(kv_heads, g, NB, NB).any(dim=1).sum().item())
    adjacent = float((pres[:, 1:] & pres[:, :-1]).sum().item())
    pairs = float(((pres[:, 0::2][:, :NB // 2]) | (pres[:, 1::2][:, :NB // 2])).sum().item())
    return {"entries": total,
            "distinct_per_kv_head_and_query_block": union,
            "saved_by_sharing_within_gqa_group": 1.0 - union / total,
            "entries_also_in_previous_query_block": adjacent / total,
            "saved_by_sharing_between_two_adjacent_query_blocks": 1.0 - pairs / total}


def dense_reference(w, layer):
    """Context only: the dense causal attention the method replaces, as PyTorch's fused
    scaled_dot_product_attention computes it on the same Q, K, V (one call, after a warm-up)."""
    import torch

    Q, K, V = layer
    g = w.heads // w.kv_heads
    q, k, v = Q[None], K[None].repeat_interleave(g, 1), V[None].repeat_interleave(g, 1)
    torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=True)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=True)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1)
    flop = 4.0 * w.head_dim * w.heads * (float(w.T) * (w.T + 1) / 2)
    return {"what": "torch scaled_dot_product_attention(is_causal=True), K/V repeated per query head",
            "ms": ms, "tflops": flop / (ms * 1e-3) / 1e12}


def k_sweep(w, layer, reps=4):
    """stream_prune_multi over k, k/2, ..., 1 (the values a binary search over k visits) against
    the same values as separate stream_prune calls: time and block scores computed."""
    import torch

    from paper_2510_19875_amd import binding

    Q, K, _ = layer
    ks = []
    k = w.topk[0]
    while k >= 1:
        ks.append(k)
        k //= 2

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    st = {}

    def multi():
        r = binding.stream_prune_multi(Q, K, w.heads, w.kv_heads, w.block, ks, workspace=st.get("ws"),
                                       out=st.get("out"), want_tiles=True)
        st["ws"], st["out"], st["tiles"] = r["workspace"], {"idx": r["idx"], "cnt": r["cnt"]}, r["tiles"]

    multi_ms = timed(multi)
    multi_tiles = int(st["tiles"].item())
    sep_ms, sep_tiles = 0.0, 0
    for k in ks:
        s1 = {}

        def one():
            r = binding.stream_prune(Q, K, w.heads, w.kv_heads, w.block, k, workspace=s1.get("ws"),
                                     out=s1.get("out"), want_tiles=True)
            s1["ws"], s1["out"], s1["tiles"] = r["workspace"], {"idx": r["idx"], "cnt": r["cnt"]}, r["tiles"]

        sep_ms += timed(one)
        sep_tiles += int(s1["tiles"].item())
    return {"topk_list": ks, "sweep_ms": multi_ms, "separate_calls_ms": sep_ms,
            "speedup": sep_ms / multi_ms, "block_scores_sweep": multi_tiles,
            "block_scores_separate_calls": sep_tiles}


def mask_rules(w, layer, scale, reps=3):
    """The same step under the other mask rules C: a sliding window of 4096 tokens (a local
    layer) and no mask at all (Alg. 1), next to the causal mask; milliseconds per call."""
    import torch

    from paper_2510_19875_amd import binding

    Q, K, V = layer
    out = {}
    for name, mask, window in (("causal", "causal", 0), ("sliding_4096", "sliding", 4096), ("full", "full", 0)):
        st = {}

        def prune():
            r = binding.stream_prune(Q, K, w.heads, w.kv_heads, w.block, w.topk[0], workspace=st.get("wp"),
                                     out=st.get("op"), mask=mask, window=window)
            st["wp"], st["op"] = r["workspace"], {"idx": r["idx"], "cnt": r["cnt"]}

        def attn():
            r = binding.stream_sparse_attn(Q, K, V, w.heads, w.kv_heads, w.block, st["op"]["idx"], st["op"]["cnt"],
                                           scale, want_lse=True, want_mass=True, workspace=st.get("wa"),
                                           out=st.get("oa"), mask=mask, window=window)
            st["wa"], st["oa"] = r["workspace"], {"O": r["O"], "lse": r["lse"], "mass": r["mass"]}

        res = {}
        for key, fn in (("prune_ms", prune), ("attn_ms", attn)):
            fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            res[key] = e0.elapsed_time(e1) / reps
        res["retained_blocks"] = int(st["op"]["cnt"].sum().item())
        out[name] = res
    return out


def _timed_pair(prune, attn, reps):
    import torch

    res = {}
    for key, fn in (("prune_ms", prune), ("attn_ms", attn)):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        res[key] = e0.elapsed_time(e1) / reps
    return res


def wide_lists(w, layer, scale, reps=3):
    """More than 64 blocks kept per row (the kernels that keep the row's lists in LDS), next to
    k = 64 through the one-node-per-lane kernels: milliseconds per call and MFMA rates."""
    import torch

    from paper_2510_19875_amd import binding

    Q, K, V = layer
    out = {}
    for k in (64, 65, 128):
        st = {}

        def prune():
            r = binding.stream_prune(Q, K, w.heads, w.kv_heads, w.block, k, workspace=st.get("wp"),
                                     out=st.get("op"), want_tiles=True)
            st["wp"], st["op"], st["tiles"] = r["workspace"], {"idx": r["idx"], "cnt": r["cnt"]}, r["tiles"]

        def attn():
            r = binding.stream_sparse_attn(Q, K, V, w.heads, w.kv_heads, w.block, st["op"]["idx"], st["op"]["cnt"],
                                           scale, want_lse=True, want_mass=True, workspace=st.get("wa"),
                                           out=st.get("oa"))
            st["wa"], st["oa"] = r["workspace"], {"O": r["O"], "lse": r["lse"], "mass": r["mass"]}

        res = _timed_pair(prune, attn, reps)
        tile_flop = 2.0 * w.block * w.block * w.head_dim
        retained = int(st["op"]["cnt"].sum().item())
        res["retained_blocks"] = retained
        res["prune_tflops"] = int(st["tiles"].item()) * tile_flop / (res["prune_ms"] * 1e-3) / 1e12
        res["attn_tflops"] = retained * 3 * tile_flop / (res["attn_ms"] * 1e-3) / 1e12
        out[f"k{k}"] = res
    return out


def mask_array(w, layer, scale, reps=3):
    """The mask C as an explicit T x T bit array (here: the causal mask written out) against the
    causal rule: milliseconds per call, and whether the lists come out identical."""
    import torch

    from paper_2510_19875_amd import binding

    Q, K, V = layer
    T = w.T
    W = (T + 31) // 32
    bits = torch.empty((T, W), dtype=torch.int32, device=Q.device)
    wd = torch.arange(W, device=Q.device)[None, :]
    for t0 in range(0, T, 8192):
        t = torch.arange(t0, min(T, t0 + 8192), device=Q.device)[:, None]
        part = (torch.ones_like(t) << ((t % 32) + 1)) - 1               # bits 0 .. t % 32 (int64)
        rows = torch.where(wd < t // 32, torch.full_like(part, 0xFFFFFFFF),
                           torch.where(wd == t // 32, part, torch.zeros_like(part)))
        bits[t0:t0 + rows.shape[0]] = ((rows + (1 << 31)) % (1 << 32) - (1 << 31)).to(torch.int32)
    out = {"array_bytes": int(bits.numel() * 4)}
    lists = {}
    for name, kw in (("rule", {}), ("array", {"mask_bits": bits})):
        st = {}

        def prune():
            r = binding.stream_prune(Q, K, w.heads, w.kv_heads, w.block, w.topk[0], workspace=st.get("wp"),
                                     out=st.get("op"), **kw)
            st["wp"], st["op"] = r["workspace"], {"idx": r["idx"], "cnt": r["cnt"]}

        def attn():
            r = binding.stream_sparse_attn(Q, K, V, w.heads, w.kv_heads, w.block, st["op"]["idx"], st["op"]["cnt"],
                                           scale, want_lse=True, want_mass=True, workspace=st.get("wa"),
                                           out=st.get("oa"), **kw)
            st["wa"], st["oa"] = r["workspace"], {"O": r["O"], "lse": r["lse"], "mass": r["mass"]}

        out[name] = _timed_pair(prune, attn, reps)
        lists[name] = st["op"]["idx"].clone()
    out["lists_identical"] = bool(torch.equal(lists["rule"], lists["array"]))
    return out


def variable_k(w, layer, reps=3):
    """stream_prune_variable: every row keeps 1/64 of its valid key blocks (k from 1 at the top
    of the pattern to the headline k at the bottom), next to the constant-k call."""
    import torch

    from paper_2510_19875_amd import binding

    Q, K, _ = layer
    kmax = w.topk[0]
    st = {}

    def run():
        r = binding.stream_prune_variable(Q, K, w.heads, w.kv_heads, w.block, 1, 64, 1, kmax,
                                          workspace=st.get("ws"), out=st.get("out"), want_tiles=True)
        st["ws"], st["out"], st["tiles"] = r["workspace"], {"idx": r["idx"], "cnt": r["cnt"]}, r["tiles"]

    run()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        run()
    e1.record()
    torch.cuda.synchronize()
    return {"rule": f"k(row) = clamp(ceil(valid/64), 1, {kmax})", "prune_ms": e0.elapsed_time(e1) / reps,
            "block_scores": int(st["tiles"].item()), "retained_blocks": int(st["out"]["cnt"].sum().item())}


def block_shapes(w, layer, scale, reps=3):
    """The step with the other block shapes (b_q, b_k in 32, 64, 128) on the same Q, K, V: k scaled
    so that every shape keeps the same 2048 keys per query row as the headline shape."""
    import torch

    from paper_2510_19875_amd import binding

    Q, K, V = layer
    out = {}
    for bq, bk in ((32, 32), (128, 128), (32, 64), (64, 32), (32, 128), (128, 32), (64, 128), (128, 64)):
        k = max(1, min(64, w.topk[0] * w.block // bk))        # the library keeps at most 64 blocks per row
        st = {}

        def prune():
            r = binding.stream_prune(Q, K, w.heads, w.kv_heads, bq, k, workspace=st.get("wp"),
                                     out=st.get("op"), block_k=bk, want_tiles=True)
            st["wp"], st["op"], st["tiles"] = r["workspace"], {"idx": r["idx"], "cnt": r["cnt"]}, r["tiles"]

        def attn():
            r = binding.stream_sparse_attn(Q, K, V, w.heads, w.kv_heads, bq, st["op"]["idx"], st["op"]["cnt"],
                                           scale, want_lse=True, want_mass=True, workspace=st.get("wa"),
                                           out=st.get("oa"), block_k=bk)
            st["wa"], st["oa"] = r["workspace"], {"O": r["O"], "lse": r["lse"], "mass": r["mass"]}

        res = {"topk": k}
        for key, fn in (("prune_ms", prune), ("attn_ms", attn)):
            fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            res[key] = e0.elapsed_time(e1) / reps
        res["block_scores"] = int(st["tiles"].item())
        res["prune_tflops"] = res["block_scores"] * 2.0 * bq * bk * w.head_dim / (res["prune_ms"] * 1e-3) / 1e12
        out[f"bq{bq}_bk{bk}"] = res
    return out


def receiver_stats(w, layer, scale, reps=2):
    """stream_receiver_stats on the same Q, K: two dense passes of b x b x d tile products over the
    causal half of the pattern (row log-sum-exp, then block means and column moments)."""
    import torch

    from paper_2510_19875_amd import binding

    Q, K, _ = layer
    st = {}

    def run():
        r = binding.stream_receiver_stats(Q, K, w.heads, w.kv_heads, w.block, scale,
                                          workspace=st.get("ws"), out=st.get("out"))
        st["ws"] = r["workspace"]
        st["out"] = {k: r[k] for k in ("col_mean", "col_kurt", "head")}

    run()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        run()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    N = w.blocks_per_seq[0]
    flop = 2.0 * w.heads * (N * (N + 1) / 2) * 2.0 * w.block * w.block * w.head_dim
    return {"ms": ms, "tflops": flop / (ms * 1e-3) / 1e12, "bound": "mfma",
            "frac_of_mfma_peak": flop / (ms * 1e-3) / 1e12 / mfma_peak(w.dtype),
            "max_column_kurtosis_head0": float(st["out"]["head"][0, 0, 0].item())}


def mask_diff_standalone(kmax, rows=1 << 21, launches=12):
    """stream_mask_diff (lists of k against lists of k/2, half of the latter shared) on synthetic
    lists, against the HBM roofline.  Algorithmic bytes per row: both index lists, the scores and
    the two counts read; the difference, its weights and its count written."""
    import torch

    from paper_2510_19875_amd import binding

    dev = "cuda:0"
    ka, kb, N = kmax, max(1, kmax // 2), 2048
    g = torch.Generator(device=dev)
    g.manual_seed(2510_19875 + 1)
    step = max(1, N // ka)
    base = torch.arange(ka, device=dev, dtype=torch.int32) * step
    ia = (base[None, :] + torch.randint(0, step, (rows, ka), device=dev, generator=g, dtype=torch.int32)).contiguous()
    ib = ia[:, ::2][:, :kb].contiguous().clone()
    move = (torch.rand(ib.shape, device=dev, generator=g) < 0.5) & (ib % step != 0)
    ib = torch.where(move, ib - 1, ib).contiguous()
    ca = torch.full((rows,), ka, dtype=torch.int32, device=dev)
    cb = torch.full((rows,), ib.shape[1], dtype=torch.int32, device=dev)
    sa = torch.randn((rows, ka), device=dev, generator=g)
    r = binding.stream_mask_diff(ia, ca, sa, ib, cb)
    out = {"idx": r["idx"], "cnt": r["cnt"], "weight": r["weight"]}
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(launches):
        binding.stream_mask_diff(ia, ca, sa, ib, cb, out=out)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / launches
    bytes_per_row = 4 * ka + 4 * ka + 4 * ib.shape[1] + 8 + 8 * ka + 4
    gbs = rows * bytes_per_row / (ms * 1e-3) / 1e9
    return {"kernel": "diff_kernel (stream_mask_diff: sorted-list set difference + weights)",
            "bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
            "frac": gbs / PEAK_HBM_GBS, "rows": rows, "k_a": ka, "k_b": int(ib.shape[1]),
            "bytes_per_row": bytes_per_row, "avg_launch_ms": ms, "launches": launches}


def select_standalone(kmax, rows=1 << 21, launches=12):
    """The top-k selection + node update as a pass of its own (inside stream_prune it is fused
    into the scoring kernel and moves no bytes): stream_select_update on a synthetic score
    tensor, against the HBM roofline.  Algorithmic bytes per row: 2k scores + k node ranges +
    the count read, k node ranges + the count written = 24k + 8."""
    import torch

    from paper_2510_19875_amd import binding

    dev = "cuda:0"
    g = torch.Generator(device=dev)
    g.manual_seed(2510_19875)
    sc = torch.randn((rows, 2 * kmax), device=dev, generator=g)
    dead = torch.rand(sc.shape, device=dev, generator=g) < 0.1          # 10% invalid branches
    sc = torch.where(dead, torch.full_like(sc, -float("inf")), sc)
    span = 1 << 20                                                        # nodes stay splittable
    nf = (torch.arange(kmax, device=dev, dtype=torch.int32) * span).repeat(rows, 1).contiguous()
    nl = nf + (span - 1)
    nc = torch.full((rows,), kmax, dtype=torch.int32, device=dev)
    binding.stream_select_update(sc, nf, nl, nc, kmax)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(launches):
        binding.stream_select_update(sc, nf, nl, nc, kmax)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / launches
    bytes_per_row = 24 * kmax + 8
    gbs = rows * bytes_per_row / (ms * 1e-3) / 1e9
    return {"kernel": "select_kernel (stream_select_update: top-k select + in-place compaction)",
            "bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
            "frac": gbs / PEAK_HBM_GBS, "rows": rows, "topk": kmax, "bytes_per_row": bytes_per_row,
            "bytes_per_launch": rows * bytes_per_row, "avg_launch_ms": ms, "launches": launches}


def cpu_baseline(w, layer, n_rows, scale, gpu_prune=None, gpu_attn=None):
    """The oracle as it stands (fp64, OpenMP over rows), timed on a seeded row sample of the same
    workload: prune + attention of those rows.  A reported baseline, not a target.  The rows it
    computes are then compared with the library's outputs for the same layer (outside the timing):
    lists equal, or certified level by level within the 1e-3 tie rule; O and lse of the equal rows."""
    import numpy as np

    from oracle import stream_oracle as so

    Q, K, V = layer
    rng = np.random.default_rng(12345)
    NB = w.total_blocks
    heads = sorted(set(int(x) for x in rng.integers(0, w.heads, size=3)))
    rows = sorted(set((heads[int(rng.integers(len(heads)))], int(rng.integers(NB))) for _ in range(n_rows)))
    g = w.heads // w.kv_heads
    Qh = {h: Q[h].float().cpu().numpy() for h in heads}
    Kh = {h // g: K[h // g].float().cpu().numpy() for h in heads}
    Vh = {h // g: V[h // g].float().cpu().numpy() for h in heads}
    cu = w.cu_seqlens
    bseq, bloc = so.block_table(cu, w.block)
    t0 = time.perf_counter()
    tokens = 0
    done = []
    for h in heads:
        for s in range(w.batch):
            gbs = [gb for (hh, gb) in rows if hh == h and bseq[gb] == s]
            ql = [int(bloc[gb]) for gb in gbs]
            if not ql:
                continue
            a, e = cu[s], cu[s + 1]
            p = so.prune_head(Qh[h][a:e], Kh[h // g][a:e], w.block, w.topk[s], qblocks=ql)
            at = so.sparse_attn(Qh[h][None, a:e], Kh[h // g][None, a:e], Vh[h // g][None, a:e], 1, 1, w.block,
                                p["idx"], p["cnt"], scale, rows=[(0, qb) for qb in ql])
            tokens += sum(min(w.block, (e - a) - qb * w.block) for qb in ql)
            done.append((h, s, gbs, ql, p, at))
    dt = time.perf_counter() - t0
    res = {"value": tokens / dt, "unit": "query-tokens*heads/s", "cores": so.threads(),
           "kind": "oracle", "seconds": dt,
           "sample": f"{len(rows)} seeded (head, query block) rows of {w.name}: Alg. 2 as printed "
                     f"(n_it levels, no score reuse) + Eq. (2) on the retained blocks, fp64"}
    if gpu_prune is not None:
        from tests import parity

        gi, gc = gpu_prune["idx"].cpu().numpy(), gpu_prune["cnt"].cpu().numpy()
        gt = gpu_prune["trace"].cpu().numpy()
        equal = ties = failed = 0
        worst_o = worst_l = 0.0
        for (h, s, gbs, ql, p, at) in done:
            a, e = cu[s], cu[s + 1]
            k = w.topk[s]
            O_g = gpu_attn["O"][h, a:e].float().cpu().numpy()
            l_g = gpu_attn["lse"][h, a:e].cpu().numpy()
            for i, (gb, q) in enumerate(zip(gbs, ql)):
                if int(gc[h, gb]) == int(p["cnt"][i]) and np.array_equal(gi[h, gb, :k], p["idx"][i]):
                    equal += 1
                    t0_, t1_ = q * w.block, min((q + 1) * w.block, e - a)
                    worst_o = max(worst_o, float(np.abs(O_g[t0_:t1_] - at["O"][0, t0_:t1_]).max()))
                    worst_l = max(worst_l, float(np.abs(l_g[t0_:t1_] - at["lse"][0, t0_:t1_]).max()))
                    continue
                n_eff = max(1, math.ceil(math.log2(math.ceil(-(-(e - a) // w.block) / k))))
                ok, _ = parity.certify_row(Qh[h][a:e], Kh[h // g][a:e], w.block, k, q, gt[:n_eff, h, gb, :k])
                ties += 1 if ok else 0
                failed += 0 if ok else 1
        tol = 2e-2 if w.dtype == "bf16" else 1e-4
        res.update({"parity_rows": len(rows), "parity_equal": equal, "parity_tie_rows": ties,
                    "parity_failed_rows": failed, "parity_max_abs_dO": worst_o, "parity_max_abs_dlse": worst_l,
                    "parity_ok": bool(failed == 0 and worst_o <= tol and worst_l <= 1e-3)})
    return res


if __name__ == "__main__":
    main()
