"""ctypes binding of the C ABI in include/stream.h.

Argument marshalling only: every step of the path runs in the HIP kernels.  PyTorch supplies
device memory and the current stream.  There is no fallback: if the library has not been built
(python __graft_entry__.py) loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libstream_hip.so")

STREAM_OK, STREAM_EINVAL, STREAM_EUNSUPPORTED, STREAM_EWORKSPACE, STREAM_EDEVICE = range(5)
STREAM_F32, STREAM_BF16 = 0, 1

EXPORTS = ["stream_num_blocks", "stream_num_key_blocks", "stream_prune_levels", "stream_prune_workspace_bytes",
           "stream_prune", "stream_prune_static", "stream_sparse_attn_workspace_bytes", "stream_sparse_attn",
           "stream_prune_multi_workspace_bytes", "stream_prune_multi", "stream_prune_variable",
           "stream_select_update", "stream_mask_diff", "stream_receiver_stats_workspace_bytes",
           "stream_receiver_stats", "stream_status_str"]


class StreamShape(ctypes.Structure):
    _fields_ = [("heads", ctypes.c_int), ("kv_heads", ctypes.c_int), ("head_dim", ctypes.c_int),
                ("block", ctypes.c_int), ("dtype", ctypes.c_int), ("batch", ctypes.c_int),
                ("T", ctypes.c_longlong), ("cu_seqlens", ctypes.POINTER(ctypes.c_int)),
                ("q_stride_h", ctypes.c_longlong), ("q_stride_t", ctypes.c_longlong),
                ("k_stride_h", ctypes.c_longlong), ("k_stride_t", ctypes.c_longlong),
                ("v_stride_h", ctypes.c_longlong), ("v_stride_t", ctypes.c_longlong),
                ("o_stride_h", ctypes.c_longlong), ("o_stride_t", ctypes.c_longlong),
                ("mask", ctypes.c_int), ("window", ctypes.c_longlong), ("block_k", ctypes.c_int),
                ("mask_bits", ctypes.c_void_p), ("mask_pitch", ctypes.c_longlong)]


class StreamPruneDiag(ctypes.Structure):
    _fields_ = [("trace", ctypes.c_void_p), ("tiles_scored", ctypes.c_void_p),
                ("level_events", ctypes.POINTER(ctypes.c_void_p)), ("levels_per_launch", ctypes.c_int)]


class StreamError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = load().stream_status_str(code).decode() if _lib is not None else str(code)
        super().__init__(f"{where}: {msg} (status {code})")


_lib = None


def load():
    """Load the HIP library and declare every exported symbol (no GPU call)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python __graft_entry__.py` "
                           "(there is no fallback path)")
    lib = ctypes.CDLL(LIB_PATH)
    sp = ctypes.POINTER(StreamShape)
    vp, ip = ctypes.c_void_p, ctypes.POINTER(ctypes.c_int)
    lib.stream_num_blocks.restype = ctypes.c_longlong
    lib.stream_num_blocks.argtypes = [sp]
    lib.stream_num_key_blocks.restype = ctypes.c_longlong
    lib.stream_num_key_blocks.argtypes = [sp]
    lib.stream_prune_levels.restype = ctypes.c_int
    lib.stream_prune_levels.argtypes = [sp, ctypes.c_int, ip]
    lib.stream_prune_workspace_bytes.restype = ctypes.c_size_t
    lib.stream_prune_workspace_bytes.argtypes = [sp, ctypes.c_int]
    lib.stream_prune.restype = ctypes.c_int
    lib.stream_prune.argtypes = [vp, vp, sp, ctypes.c_int, ip, ctypes.c_int, vp, vp, vp,
                                 ctypes.POINTER(StreamPruneDiag), vp, ctypes.c_size_t, vp]
    lib.stream_prune_static.restype = ctypes.c_int
    lib.stream_prune_static.argtypes = [vp, vp, sp, ctypes.c_int, ip, ctypes.c_int, vp, vp, vp,
                                        ctypes.POINTER(StreamPruneDiag), vp]
    lib.stream_sparse_attn_workspace_bytes.restype = ctypes.c_size_t
    lib.stream_sparse_attn_workspace_bytes.argtypes = [sp, ctypes.c_int]
    lib.stream_sparse_attn.restype = ctypes.c_int
    lib.stream_sparse_attn.argtypes = [vp, vp, vp, sp, vp, vp, ctypes.c_int, ctypes.c_float,
                                       vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.stream_prune_multi_workspace_bytes.restype = ctypes.c_size_t
    lib.stream_prune_multi_workspace_bytes.argtypes = [sp, ctypes.c_int, ctypes.c_int]
    lib.stream_prune_multi.restype = ctypes.c_int
    lib.stream_prune_multi.argtypes = [vp, vp, sp, ip, ctypes.c_int, ctypes.c_int, vp, vp, vp,
                                       ctypes.POINTER(StreamPruneDiag), vp, ctypes.c_size_t, vp]
    lib.stream_prune_variable.restype = ctypes.c_int
    lib.stream_prune_variable.argtypes = [vp, vp, sp, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                          vp, vp, vp, ctypes.POINTER(StreamPruneDiag), vp, ctypes.c_size_t, vp]
    lib.stream_select_update.restype = ctypes.c_int
    lib.stream_select_update.argtypes = [vp, vp, vp, vp, ctypes.c_longlong, ctypes.c_int, ctypes.c_int, vp]
    lib.stream_mask_diff.restype = ctypes.c_int
    lib.stream_mask_diff.argtypes = [vp, vp, vp, ctypes.c_int, vp, vp, ctypes.c_int, ctypes.c_longlong,
                                     vp, vp, vp, vp]
    lib.stream_receiver_stats_workspace_bytes.restype = ctypes.c_size_t
    lib.stream_receiver_stats_workspace_bytes.argtypes = [sp]
    lib.stream_receiver_stats.restype = ctypes.c_int
    lib.stream_receiver_stats.argtypes = [vp, vp, sp, ctypes.c_float, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.stream_status_str.restype = ctypes.c_char_p
    lib.stream_status_str.argtypes = [ctypes.c_int]
    _lib = lib
    return lib


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return STREAM_F32
    if t.dtype == torch.bfloat16:
        return STREAM_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


MASKS = {"causal": 0, "full": 1, "sliding": 2, "array": 3}


def make_shape(heads, kv_heads, head_dim, block, dtype_code, T, cu_seqlens=None, Q=None, K=None,
               V=None, O=None, mask="causal", window=0, block_k=0, mask_bits=None):
    """Build a stream_shape; returns (shape, keepalive) - keepalive owns the host cu_seqlens array.
    mask_bits: int32 device tensor [T, pitch] holding the explicit mask C as bits (bit u % 32 of
    word [t, u // 32]); selects STREAM_MASK_ARRAY."""
    s = StreamShape()
    s.heads, s.kv_heads, s.head_dim, s.block, s.dtype = heads, kv_heads, head_dim, block, dtype_code
    s.T = int(T)
    s.mask = MASKS[mask] if isinstance(mask, str) else int(mask)
    s.window = int(window)
    s.block_k = int(block_k or 0)
    if mask_bits is not None:
        if not mask_bits.is_cuda or mask_bits.dtype != torch.int32 or mask_bits.dim() != 2 or mask_bits.stride(1) != 1:
            raise ValueError("mask_bits must be a device int32 tensor [T, pitch] with contiguous rows")
        s.mask = MASKS["array"]
        s.mask_bits = mask_bits.data_ptr()
        s.mask_pitch = mask_bits.stride(0)
    keep = None
    if cu_seqlens is not None:
        cu = [int(x) for x in cu_seqlens]
        keep = (ctypes.c_int * len(cu))(*cu)
        s.cu_seqlens = ctypes.cast(keep, ctypes.POINTER(ctypes.c_int))
        s.batch = len(cu) - 1
    else:
        s.batch = 1
    for name, t in (("q", Q), ("k", K), ("v", V), ("o", O)):
        if t is not None:
            if t.stride(-1) != 1:
                raise ValueError("last dimension must be contiguous")
            setattr(s, f"{name}_stride_h", t.stride(0))
            setattr(s, f"{name}_stride_t", t.stride(1))
    return s, keep


def _stream_ptr() -> int:
    return torch.cuda.current_stream().cuda_stream


def num_blocks(shape: StreamShape) -> int:
    return int(load().stream_num_blocks(ctypes.byref(shape)))


def stream_prune(Q: torch.Tensor, K: torch.Tensor, heads: int, kv_heads: int, block: int,
                 topk, cu_seqlens: Optional[Sequence[int]] = None, want_score: bool = False,
                 want_trace: bool = False, want_tiles: bool = False, workspace=None, out=None,
                 level_events=None, levels_per_launch: int = 0, mask="causal", window: int = 0,
                 block_k: int = 0, mask_bits=None):
    """Algorithm 2 for every (head, query block).  Q [H, T, d], K [Hkv, T, d] on the GPU.

    topk: int, or one int per sequence.  Returns dict(idx [H, NB, kmax] int32, cnt [H, NB] int32,
    score (optional) fp32, trace (optional) int32 [levels, H, NB, kmax, 2], tiles (optional)).
    """
    lib = load()
    if not (Q.is_cuda and K.is_cuda):
        raise ValueError("Q and K must be device tensors (the library has no CPU path)")
    H, T, d = Q.shape
    shape, keep = make_shape(heads, kv_heads, d, block, _dtype_code(Q), T, cu_seqlens, Q=Q, K=K,
                             mask=mask, window=window, block_k=block_k, mask_bits=mask_bits)
    nseq = shape.batch
    if isinstance(topk, int):
        ks, kmax, k_arr = None, int(topk), None
    else:
        ks = [int(x) for x in topk]
        kmax = max(ks)
        k_arr = (ctypes.c_int * nseq)(*ks)
    NB = num_blocks(shape)
    if NB < 0:
        raise StreamError(STREAM_EINVAL, "stream_num_blocks")
    dev = Q.device
    if out is None:
        idx = torch.empty((H, NB, kmax), dtype=torch.int32, device=dev)
        cnt = torch.empty((H, NB), dtype=torch.int32, device=dev)
        score = torch.empty((H, NB, kmax), dtype=torch.float32, device=dev) if want_score else None
    else:
        idx, cnt, score = out["idx"], out["cnt"], out.get("score")
    need = lib.stream_prune_workspace_bytes(ctypes.byref(shape), kmax)
    if workspace is None:
        workspace = torch.empty((max(need, 256),), dtype=torch.uint8, device=dev)
    diag = StreamPruneDiag()
    trace = tiles = None
    levels = lib.stream_prune_levels(ctypes.byref(shape), kmax if ks is None else 0,
                                     k_arr if k_arr is not None else None)
    if want_trace:
        trace = torch.empty((max(levels, 0), H, NB, kmax, 2), dtype=torch.int32, device=dev)
        diag.trace = trace.data_ptr()
    if want_tiles:
        tiles = torch.zeros((1,), dtype=torch.int64, device=dev)
        diag.tiles_scored = tiles.data_ptr()
    if level_events is not None:
        if len(level_events) < 2 * levels:
            raise ValueError("level_events needs 2 events per level")
        diag.level_events = ctypes.cast(level_events, ctypes.POINTER(ctypes.c_void_p))
    diag.levels_per_launch = int(levels_per_launch)
    rc = lib.stream_prune(Q.data_ptr(), K.data_ptr(), ctypes.byref(shape),
                          kmax if ks is None else 0, k_arr, kmax,
                          idx.data_ptr(), cnt.data_ptr(), score.data_ptr() if score is not None else None,
                          ctypes.byref(diag) if (want_trace or want_tiles or level_events is not None
                                                 or levels_per_launch) else None,
                          workspace.data_ptr(), workspace.numel(), _stream_ptr())
    if rc != STREAM_OK:
        raise StreamError(rc, "stream_prune")
    return {"idx": idx, "cnt": cnt, "score": score, "trace": trace, "tiles": tiles,
            "levels": levels, "workspace": workspace, "_keep": keep}


STATIC_SCRATCH_BYTES = 80 * 1024 * 1024   # STREAM_STATIC_SCRATCH_BYTES of include/stream.h


def stream_prune_static(Q: torch.Tensor, K: torch.Tensor, heads: int, kv_heads: int, block: int,
                        topk, out, cu_seqlens: Optional[Sequence[int]] = None, mask="causal",
                        window: int = 0, block_k: int = 0, mask_bits=None):
    """stream_prune through the entry point that allocates nothing: the scratch is the library's
    own device array, the outputs out["idx"] [H, NB, kmax], out["cnt"] [H, NB] and (optional)
    out["score"] come from the caller.  Raises StreamError(STREAM_EWORKSPACE) beyond the limit."""
    lib = load()
    if not (Q.is_cuda and K.is_cuda):
        raise ValueError("Q and K must be device tensors (the library has no CPU path)")
    H, T, d = Q.shape
    shape, keep = make_shape(heads, kv_heads, d, block, _dtype_code(Q), T, cu_seqlens, Q=Q, K=K,
                             mask=mask, window=window, block_k=block_k, mask_bits=mask_bits)
    if isinstance(topk, int):
        ks, kmax, k_arr = None, int(topk), None
    else:
        ks = [int(x) for x in topk]
        kmax = max(ks)
        k_arr = (ctypes.c_int * shape.batch)(*ks)
    idx, cnt, score = out["idx"], out["cnt"], out.get("score")
    rc = lib.stream_prune_static(Q.data_ptr(), K.data_ptr(), ctypes.byref(shape),
                                 kmax if ks is None else 0, k_arr, idx.shape[-1],
                                 idx.data_ptr(), cnt.data_ptr(), score.data_ptr() if score is not None else None,
                                 None, _stream_ptr())
    if rc != STREAM_OK:
        raise StreamError(rc, "stream_prune_static")
    return {"idx": idx, "cnt": cnt, "score": score, "_keep": keep}


def stream_prune_multi(Q: torch.Tensor, K: torch.Tensor, heads: int, kv_heads: int, block: int,
                       topk_list: Sequence[int], cu_seqlens: Optional[Sequence[int]] = None,
                       want_score: bool = False, want_tiles: bool = False, workspace=None, out=None,
                       mask="causal", window: int = 0, block_k: int = 0, mask_bits=None):
    """Algorithm 2 for several k over the same Q, K in one call.  Returns dict(idx
    [H, n_k, NB, kmax] int32, cnt [H, n_k, NB] int32, score (optional) fp32, tiles (optional))."""
    lib = load()
    if not (Q.is_cuda and K.is_cuda):
        raise ValueError("Q and K must be device tensors (the library has no CPU path)")
    H, T, d = Q.shape
    shape, keep = make_shape(heads, kv_heads, d, block, _dtype_code(Q), T, cu_seqlens, Q=Q, K=K,
                             mask=mask, window=window, block_k=block_k, mask_bits=mask_bits)
    ks = [int(x) for x in topk_list]
    n_k, kmax = len(ks), max(ks)
    k_arr = (ctypes.c_int * n_k)(*ks)
    NB = num_blocks(shape)
    if NB < 0:
        raise StreamError(STREAM_EINVAL, "stream_num_blocks")
    dev = Q.device
    if out is None:
        idx = torch.empty((H, n_k, NB, kmax), dtype=torch.int32, device=dev)
        cnt = torch.empty((H, n_k, NB), dtype=torch.int32, device=dev)
        score = torch.empty((H, n_k, NB, kmax), dtype=torch.float32, device=dev) if want_score else None
    else:
        idx, cnt, score = out["idx"], out["cnt"], out.get("score")
    need = lib.stream_prune_multi_workspace_bytes(ctypes.byref(shape), n_k, kmax)
    if workspace is None:
        workspace = torch.empty((max(need, 256),), dtype=torch.uint8, device=dev)
    diag = StreamPruneDiag()
    tiles = None
    if want_tiles:
        tiles = torch.zeros((1,), dtype=torch.int64, device=dev)
        diag.tiles_scored = tiles.data_ptr()
    rc = lib.stream_prune_multi(Q.data_ptr(), K.data_ptr(), ctypes.byref(shape), k_arr, n_k, kmax,
                                idx.data_ptr(), cnt.data_ptr(), score.data_ptr() if score is not None else None,
                                ctypes.byref(diag) if want_tiles else None,
                                workspace.data_ptr(), workspace.numel(), _stream_ptr())
    if rc != STREAM_OK:
        raise StreamError(rc, "stream_prune_multi")
    return {"idx": idx, "cnt": cnt, "score": score, "tiles": tiles, "workspace": workspace, "_keep": keep}


def stream_prune_variable(Q: torch.Tensor, K: torch.Tensor, heads: int, kv_heads: int, block: int,
                          keep_num: int, keep_den: int, topk_min: int, topk_max: int,
                          cu_seqlens: Optional[Sequence[int]] = None, want_score: bool = False,
                          want_trace: bool = False, want_tiles: bool = False, workspace=None, out=None,
                          mask="causal", window: int = 0, block_k: int = 0, mask_bits=None):
    """Algorithm 2 with k(row) = clamp(ceil(valid(row) * keep_num / keep_den), topk_min, topk_max).
    Returns dict(idx [H, NB, topk_max], cnt [H, NB], score, trace, tiles)."""
    lib = load()
    if not (Q.is_cuda and K.is_cuda):
        raise ValueError("Q and K must be device tensors (the library has no CPU path)")
    H, T, d = Q.shape
    shape, keep = make_shape(heads, kv_heads, d, block, _dtype_code(Q), T, cu_seqlens, Q=Q, K=K,
                             mask=mask, window=window, block_k=block_k, mask_bits=mask_bits)
    NB = num_blocks(shape)
    if NB < 0:
        raise StreamError(STREAM_EINVAL, "stream_num_blocks")
    dev = Q.device
    kmax = int(topk_max)
    if out is None:
        idx = torch.empty((H, NB, kmax), dtype=torch.int32, device=dev)
        cnt = torch.empty((H, NB), dtype=torch.int32, device=dev)
        score = torch.empty((H, NB, kmax), dtype=torch.float32, device=dev) if want_score else None
    else:
        idx, cnt, score = out["idx"], out["cnt"], out.get("score")
    need = lib.stream_prune_workspace_bytes(ctypes.byref(shape), kmax)
    if workspace is None:
        workspace = torch.empty((max(need, 256),), dtype=torch.uint8, device=dev)
    diag = StreamPruneDiag()
    trace = tiles = None
    levels = lib.stream_prune_levels(ctypes.byref(shape), int(topk_min), None)
    if want_trace:
        trace = torch.empty((max(levels, 0), H, NB, kmax, 2), dtype=torch.int32, device=dev)
        diag.trace = trace.data_ptr()
    if want_tiles:
        tiles = torch.zeros((1,), dtype=torch.int64, device=dev)
        diag.tiles_scored = tiles.data_ptr()
    rc = lib.stream_prune_variable(Q.data_ptr(), K.data_ptr(), ctypes.byref(shape), int(keep_num), int(keep_den),
                                   int(topk_min), kmax, idx.data_ptr(), cnt.data_ptr(),
                                   score.data_ptr() if score is not None else None,
                                   ctypes.byref(diag) if (want_trace or want_tiles) else None,
                                   workspace.data_ptr(), workspace.numel(), _stream_ptr())
    if rc != STREAM_OK:
        raise StreamError(rc, "stream_prune_variable")
    return {"idx": idx, "cnt": cnt, "score": score, "trace": trace, "tiles": tiles, "levels": levels,
            "workspace": workspace, "_keep": keep}


def stream_sparse_attn(Q, K, V, heads: int, kv_heads: int, block: int, idx, cnt, scale: float,
                       cu_seqlens=None, want_lse: bool = False, want_mass: bool = False,
                       workspace=None, out=None, mask="causal", window: int = 0, block_k: int = 0,
                       mask_bits=None):
    """Eq. (2) on the retained blocks.  Returns dict(O [H, T, d], lse [H, T], mass [H, T])."""
    lib = load()
    if not (Q.is_cuda and K.is_cuda and V.is_cuda):
        raise ValueError("Q, K, V must be device tensors (the library has no CPU path)")
    H, T, d = Q.shape
    dev = Q.device
    O = torch.empty_like(Q) if out is None else out["O"]
    shape, keep = make_shape(heads, kv_heads, d, block, _dtype_code(Q), T, cu_seqlens, Q=Q, K=K, V=V, O=O,
                             mask=mask, window=window, block_k=block_k, mask_bits=mask_bits)
    kmax = idx.shape[-1]
    if idx.dtype != torch.int32 or cnt.dtype != torch.int32 or not idx.is_contiguous() or not cnt.is_contiguous():
        raise ValueError("idx/cnt must be contiguous int32 device tensors")
    lse = (torch.empty((H, T), dtype=torch.float32, device=dev) if out is None else out.get("lse")) if want_lse else None
    mass = (torch.empty((H, T), dtype=torch.float32, device=dev) if out is None else out.get("mass")) if want_mass else None
    need = lib.stream_sparse_attn_workspace_bytes(ctypes.byref(shape), kmax)
    if workspace is None:
        workspace = torch.empty((max(need, 256),), dtype=torch.uint8, device=dev)
    rc = lib.stream_sparse_attn(Q.data_ptr(), K.data_ptr(), V.data_ptr(), ctypes.byref(shape),
                                idx.data_ptr(), cnt.data_ptr(), kmax, float(scale), O.data_ptr(),
                                lse.data_ptr() if lse is not None else None,
                                mass.data_ptr() if mass is not None else None,
                                workspace.data_ptr(), workspace.numel(), _stream_ptr())
    if rc != STREAM_OK:
        raise StreamError(rc, "stream_sparse_attn")
    return {"O": O, "lse": lse, "mass": mass, "workspace": workspace, "_keep": keep}


def stream_select_update(score, node_first, node_last, node_count, topk: int):
    """Top-k selection + node update of Alg. 2 on branch scores held in memory, in place.

    score [rows, 2*kmax] fp32, node_first/node_last [rows, kmax] int32, node_count [rows] int32,
    all contiguous device tensors; the node tensors are updated in place."""
    lib = load()
    for t in (score, node_first, node_last, node_count):
        if not t.is_cuda:
            raise ValueError("all arguments must be device tensors (the library has no CPU path)")
        if not t.is_contiguous():
            raise ValueError("all arguments must be contiguous")
    if score.dtype != torch.float32 or any(t.dtype != torch.int32 for t in (node_first, node_last, node_count)):
        raise ValueError("score must be float32, the node tensors int32")
    rows, kmax = node_first.shape
    if tuple(score.shape) != (rows, 2 * kmax) or tuple(node_last.shape) != (rows, kmax) or tuple(node_count.shape) != (rows,):
        raise ValueError("shape mismatch")
    rc = lib.stream_select_update(score.data_ptr(), node_first.data_ptr(), node_last.data_ptr(),
                                  node_count.data_ptr(), rows, int(topk), kmax, _stream_ptr())
    if rc != STREAM_OK:
        raise StreamError(rc, "stream_select_update")


def stream_mask_diff(idx_a, cnt_a, score_a, idx_b, cnt_b, want_weight: bool = True, out=None):
    """Entries of the lists a (k_success) absent from the lists b (k_fail), row by row.

    idx_* [..., kmax] int32, cnt_* [...] int32, score_a like idx_a (fp32) or None; leading
    dimensions are flattened to rows.  Returns dict(idx, cnt, weight) shaped like the a inputs."""
    lib = load()
    ts = [idx_a, cnt_a, idx_b, cnt_b] + ([score_a] if score_a is not None else [])
    for t in ts:
        if not t.is_cuda:
            raise ValueError("all arguments must be device tensors (the library has no CPU path)")
        if not t.is_contiguous():
            raise ValueError("all arguments must be contiguous")
    if any(t.dtype != torch.int32 for t in (idx_a, cnt_a, idx_b, cnt_b)) or \
            (score_a is not None and score_a.dtype != torch.float32):
        raise ValueError("index/count tensors must be int32, scores float32")
    ka, kb = idx_a.shape[-1], idx_b.shape[-1]
    rows = cnt_a.numel()
    if idx_a.numel() != rows * ka or idx_b.numel() != rows * kb or cnt_b.numel() != rows or \
            (score_a is not None and score_a.shape != idx_a.shape):
        raise ValueError("shape mismatch")
    want_weight = want_weight and score_a is not None
    if out is None:
        io = torch.empty_like(idx_a)
        co = torch.empty_like(cnt_a)
        wo = torch.empty(idx_a.shape, dtype=torch.float32, device=idx_a.device) if want_weight else None
    else:
        io, co, wo = out["idx"], out["cnt"], out.get("weight")
    rc = lib.stream_mask_diff(idx_a.data_ptr(), cnt_a.data_ptr(),
                              score_a.data_ptr() if score_a is not None else None, ka,
                              idx_b.data_ptr(), cnt_b.data_ptr(), kb, rows,
                              io.data_ptr(), co.data_ptr(), wo.data_ptr() if wo is not None else None,
                              _stream_ptr())
    if rc != STREAM_OK:
        raise StreamError(rc, "stream_mask_diff")
    return {"idx": io, "cnt": co, "weight": wo}


def stream_receiver_stats(Q, K, heads: int, kv_heads: int, block: int, scale: float, cu_seqlens=None,
                          want_block_mean: bool = False, workspace=None, out=None, mask="causal",
                          window: int = 0, block_k: int = 0, mask_bits=None):
    """Block means of the dense attention pattern and their vertical kurtosis (Section 4.1).

    Returns dict(block_mean [H, NB, NBk] or None, col_mean [H, NBk], col_kurt [H, NBk],
    head [H, batch, 2] = (max column kurtosis, kurtosis of the column means))."""
    lib = load()
    if not (Q.is_cuda and K.is_cuda):
        raise ValueError("Q, K must be device tensors (the library has no CPU path)")
    H, T, d = Q.shape
    dev = Q.device
    shape, keep = make_shape(heads, kv_heads, d, block, _dtype_code(Q), T, cu_seqlens, Q=Q, K=K,
                             mask=mask, window=window, block_k=block_k, mask_bits=mask_bits)
    NB = lib.stream_num_blocks(ctypes.byref(shape))
    NBk = lib.stream_num_key_blocks(ctypes.byref(shape))
    if NB < 0 or NBk < 0:
        raise StreamError(1, "stream_num_blocks")
    batch = shape.batch
    if out is None:
        bm = torch.empty((H, NB, NBk), dtype=torch.float32, device=dev) if want_block_mean else None
        cm = torch.empty((H, NBk), dtype=torch.float32, device=dev)
        ck = torch.empty((H, NBk), dtype=torch.float32, device=dev)
        hs = torch.empty((H, batch, 2), dtype=torch.float32, device=dev)
    else:
        bm, cm, ck, hs = out.get("block_mean"), out["col_mean"], out["col_kurt"], out["head"]
    need = lib.stream_receiver_stats_workspace_bytes(ctypes.byref(shape))
    if workspace is None:
        workspace = torch.empty((max(need, 256),), dtype=torch.uint8, device=dev)
    rc = lib.stream_receiver_stats(Q.data_ptr(), K.data_ptr(), ctypes.byref(shape), float(scale),
                                   bm.data_ptr() if bm is not None else None, cm.data_ptr(),
                                   ck.data_ptr(), hs.data_ptr(), workspace.data_ptr(),
                                   workspace.numel(), _stream_ptr())
    if rc != STREAM_OK:
        raise StreamError(rc, "stream_receiver_stats")
    return {"block_mean": bm, "col_mean": cm, "col_kurt": ck, "head": hs, "workspace": workspace,
            "_keep": keep}
