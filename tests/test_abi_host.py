"""Host-side checks of the C ABI (no GPU): the library loads, exports every symbol the header
declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

from paper_2510_19875_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    return B.load()


def shape(**kw):
    s = B.StreamShape()
    s.heads, s.kv_heads, s.head_dim, s.block, s.dtype, s.batch, s.T = 8, 2, 128, 64, B.STREAM_BF16, 1, 1000
    for k, v in kw.items():
        setattr(s, k, v)
    return s


def test_exports_every_declared_symbol(lib):
    hdr = open(os.path.join(ROOT, "include", "stream.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = set(re.findall(r"\b(stream_[a-z_]+)\s*\(", hdr))
    assert names == set(B.EXPORTS)
    for n in names:
        assert hasattr(lib, n), n


def test_status_strings(lib):
    for code in range(5):
        assert lib.stream_status_str(code)
    assert lib.stream_status_str(B.STREAM_OK) == b"ok"


def test_block_geometry(lib):
    assert lib.stream_num_blocks(ctypes.byref(shape())) == 16  # ceil(1000/64)
    cu = (ctypes.c_int * 4)(0, 100, 164, 1000)
    s = shape(batch=3, cu_seqlens=ctypes.cast(cu, ctypes.POINTER(ctypes.c_int)))
    assert lib.stream_num_blocks(ctypes.byref(s)) == 2 + 1 + 14
    # levels = max(1, ceil(log2(ceil(N/k))))
    assert lib.stream_prune_levels(ctypes.byref(shape(T=131072)), 32, None) == 6
    assert lib.stream_prune_levels(ctypes.byref(shape(T=1048576, block=128)), 64, None) == 7
    assert lib.stream_prune_levels(ctypes.byref(shape(T=4096)), 8, None) == 3
    assert lib.stream_prune_levels(ctypes.byref(shape(T=4096)), 64, None) == 1
    ks = (ctypes.c_int * 3)(1, 1, 2)
    assert lib.stream_prune_levels(ctypes.byref(s), 0, ks) == 3  # 14 blocks, k=2 -> ceil(log2 7)
    # b_q != b_k: sequences are padded to a multiple of lcm(b_q, b_k); NB counts query blocks,
    # the levels follow the key blocks
    assert lib.stream_num_blocks(ctypes.byref(shape(block=32, block_k=128))) == 32      # T_p = 1024
    assert lib.stream_num_blocks(ctypes.byref(shape(block=128, block_k=32))) == 8
    assert lib.stream_num_key_blocks(ctypes.byref(shape(block=128, block_k=32))) == 32
    assert lib.stream_num_key_blocks(ctypes.byref(shape())) == 16
    assert lib.stream_num_blocks(ctypes.byref(shape(block=64, block_k=64))) == 16
    s.block, s.block_k = 32, 128
    assert lib.stream_num_blocks(ctypes.byref(s)) == 4 + 4 + 28                         # 128, 128, 896
    assert lib.stream_prune_levels(ctypes.byref(shape(T=131072, block=32, block_k=128)), 16, None) == 6
    assert lib.stream_prune_levels(ctypes.byref(shape(T=131072, block=128, block_k=32)), 64, None) == 6


@pytest.mark.parametrize("kw,code", [
    (dict(heads=0), B.STREAM_EINVAL),
    (dict(kv_heads=3), B.STREAM_EINVAL),
    (dict(T=0), B.STREAM_EINVAL),
    (dict(dtype=7), B.STREAM_EINVAL),
    (dict(batch=2), B.STREAM_EINVAL),            # batch > 1 without cu_seqlens
    (dict(head_dim=96), B.STREAM_EUNSUPPORTED),
    (dict(block=48), B.STREAM_EUNSUPPORTED),
    (dict(block_k=16), B.STREAM_EUNSUPPORTED),
    (dict(block_k=256), B.STREAM_EUNSUPPORTED),
    (dict(batch=65), B.STREAM_EINVAL),
])
def test_bad_shapes_are_rejected_on_the_host(lib, kw, code):
    s = shape(**kw)
    assert lib.stream_num_blocks(ctypes.byref(s)) == -1
    assert lib.stream_prune_workspace_bytes(ctypes.byref(s), 8) == 0
    fake = ctypes.c_void_p(4096)
    rc = lib.stream_prune(fake, fake, ctypes.byref(s), 8, None, 8, fake, fake, None, None,
                          ctypes.c_void_p(256 * 16), 1 << 40, None)
    assert rc == code
    rc = lib.stream_sparse_attn(fake, fake, fake, ctypes.byref(s), fake, fake, 8, 1.0, fake, None,
                                None, ctypes.c_void_p(256 * 16), 1 << 40, None)
    assert rc == code


def test_bad_arguments_of_prune(lib):
    s = shape()
    fake = ctypes.c_void_p(4096)
    ws = ctypes.c_void_p(256 * 16)
    need = lib.stream_prune_workspace_bytes(ctypes.byref(s), 8)
    assert need > 0 and need % 256 == 0

    def call(Q=fake, K=fake, topk=8, per=None, kmax=8, idx=fake, cnt=fake, wsp=ws, wsz=need, sh=s):
        return lib.stream_prune(Q, K, ctypes.byref(sh), topk, per, kmax, idx, cnt, None, None, wsp, wsz, None)

    assert call(Q=None) == B.STREAM_EINVAL
    assert call(K=None) == B.STREAM_EINVAL
    assert call(idx=None) == B.STREAM_EINVAL
    assert call(cnt=None) == B.STREAM_EINVAL
    assert call(topk=0) == B.STREAM_EINVAL
    assert call(topk=9, kmax=8) == B.STREAM_EINVAL          # k beyond the row length of idx
    assert call(topk=513, kmax=513) == B.STREAM_EUNSUPPORTED  # beyond the LDS node lists of the wide kernel
    # fp32 rows of 128 queries at d = 128 fit no single wavefront: 64 blocks per row at most
    assert call(topk=65, kmax=65, sh=shape(block=128, dtype=B.STREAM_F32)) == B.STREAM_EUNSUPPORTED
    assert call(Q=ctypes.c_void_p(4100)) == B.STREAM_EINVAL  # not 16-byte aligned
    assert call(sh=shape(q_stride_t=100)) == B.STREAM_EINVAL  # rows shorter than head_dim
    assert call(sh=shape(q_stride_t=132)) == B.STREAM_EINVAL  # rows not 16-byte aligned
    # a query block's rows are addressed with 32-bit offsets from the block's first row: token
    # strides of 16 MiB and more are refused (anything below is fine whatever the sequence length)
    assert call(sh=shape(q_stride_t=(1 << 23))) == B.STREAM_EUNSUPPORTED
    assert call(wsp=None) == B.STREAM_EWORKSPACE
    assert call(wsp=ctypes.c_void_p(4096 + 64)) == B.STREAM_EWORKSPACE
    assert call(wsz=need - 1) == B.STREAM_EWORKSPACE
    cu = (ctypes.c_int * 3)(0, 600, 900)  # does not end at T
    bad = shape(batch=2, cu_seqlens=ctypes.cast(cu, ctypes.POINTER(ctypes.c_int)))
    assert call(sh=bad) == B.STREAM_EINVAL


def test_bad_arguments_of_the_mask_array(lib):
    fake = ctypes.c_void_p(4096)
    ws = ctypes.c_void_p(256 * 16)

    def prune(s):
        return lib.stream_prune(fake, fake, ctypes.byref(s), 8, None, 8, fake, fake, None, None, ws, 1 << 40, None)

    arr = dict(mask=B.MASKS["array"], mask_bits=8192, mask_pitch=32)          # T = 1000: 32 words per row
    assert lib.stream_prune_workspace_bytes(ctypes.byref(shape(**arr)), 8) > \
        lib.stream_prune_workspace_bytes(ctypes.byref(shape()), 8)            # + the block summaries
    assert prune(shape(**{**arr, "mask_bits": None})) == B.STREAM_EINVAL
    assert prune(shape(**{**arr, "mask_bits": 8194})) == B.STREAM_EINVAL      # words are 4-byte aligned
    assert prune(shape(**{**arr, "mask_pitch": 31})) == B.STREAM_EINVAL       # rows shorter than T bits
    cu = (ctypes.c_int * 3)(0, 600, 1000)
    two = shape(batch=2, cu_seqlens=ctypes.cast(cu, ctypes.POINTER(ctypes.c_int)), **arr)
    assert prune(two) == B.STREAM_EUNSUPPORTED                                 # single sequence only
    # the statistics take the array too (one sequence): more workspace, the same refusal of a batch
    assert lib.stream_receiver_stats_workspace_bytes(ctypes.byref(shape(**arr))) > \
        lib.stream_receiver_stats_workspace_bytes(ctypes.byref(shape()))
    rc = lib.stream_receiver_stats(fake, fake, ctypes.byref(two), 0.125, None, fake, fake, fake, ws, 1 << 40, None)
    assert rc == B.STREAM_EUNSUPPORTED


def test_bad_arguments_of_sparse_attn(lib):
    s = shape()
    fake = ctypes.c_void_p(4096)
    ws = ctypes.c_void_p(256 * 16)
    need = lib.stream_sparse_attn_workspace_bytes(ctypes.byref(s), 8)
    assert need > 0

    def call(Q=fake, V=fake, idx=fake, O=fake, kmax=8, scale=1.0, wsz=need):
        return lib.stream_sparse_attn(Q, fake, V, ctypes.byref(s), idx, fake, kmax, scale, O, None,
                                      None, ws, wsz, None)

    assert call(Q=None) == B.STREAM_EINVAL
    assert call(V=None) == B.STREAM_EINVAL
    assert call(idx=None) == B.STREAM_EINVAL
    assert call(O=None) == B.STREAM_EINVAL
    assert call(kmax=0) == B.STREAM_EINVAL
    assert call(scale=0.0) == B.STREAM_EINVAL
    assert call(scale=float("nan")) == B.STREAM_EINVAL
    assert call(wsz=need - 1) == B.STREAM_EWORKSPACE


def test_bad_arguments_of_select_update(lib):
    fake = ctypes.c_void_p(4096)

    def call(sc=fake, nf=fake, nl=fake, nc=fake, rows=8, k=4, kmax=8):
        return lib.stream_select_update(sc, nf, nl, nc, rows, k, kmax, None)

    assert call(sc=None) == B.STREAM_EINVAL
    assert call(nf=None) == B.STREAM_EINVAL
    assert call(nl=None) == B.STREAM_EINVAL
    assert call(nc=None) == B.STREAM_EINVAL
    assert call(sc=ctypes.c_void_p(4100)) == B.STREAM_EINVAL      # scores are read in pairs
    assert call(rows=-1) == B.STREAM_EINVAL
    assert call(k=0) == B.STREAM_EINVAL
    assert call(k=9) == B.STREAM_EINVAL
    assert call(k=513, kmax=513) == B.STREAM_EUNSUPPORTED
    assert call(rows=1 << 40) == B.STREAM_EUNSUPPORTED
    assert call(rows=0) == B.STREAM_OK                            # nothing to do, nothing launched


def test_bad_arguments_of_mask_diff(lib):
    fake = ctypes.c_void_p(4096)
    other = ctypes.c_void_p(8192)

    def call(ia=fake, ca=fake, sa=fake, ka=8, ib=fake, cb=fake, kb=4, rows=5, io=other, co=other, wo=other):
        return lib.stream_mask_diff(ia, ca, sa, ka, ib, cb, kb, rows, io, co, wo, None)

    assert call(ia=None) == B.STREAM_EINVAL
    assert call(cb=None) == B.STREAM_EINVAL
    assert call(io=None) == B.STREAM_EINVAL
    assert call(sa=None) == B.STREAM_EINVAL                 # weights wanted but no scores given
    assert call(io=fake) == B.STREAM_EINVAL                 # output aliases an input
    assert call(ka=0) == B.STREAM_EINVAL
    assert call(rows=-1) == B.STREAM_EINVAL
    assert call(ka=513) == B.STREAM_EUNSUPPORTED
    assert call(kb=513) == B.STREAM_EUNSUPPORTED
    assert call(rows=1 << 40) == B.STREAM_EUNSUPPORTED
    assert call(rows=0) == B.STREAM_OK


def test_bad_arguments_of_receiver_stats(lib):
    s = shape()
    fake = ctypes.c_void_p(4096)
    ws = ctypes.c_void_p(256 * 16)
    need = lib.stream_receiver_stats_workspace_bytes(ctypes.byref(s))
    assert need > 0

    def call(Q=fake, K=fake, sh=s, scale=0.125, cm=fake, ck=fake, hs=fake, wsp=ws, wsz=need):
        return lib.stream_receiver_stats(Q, K, ctypes.byref(sh), scale, None, cm, ck, hs, wsp, wsz, None)

    assert call(Q=None) == B.STREAM_EINVAL
    assert call(K=None) == B.STREAM_EINVAL
    assert call(cm=None) == B.STREAM_EINVAL
    assert call(ck=None) == B.STREAM_EINVAL
    assert call(hs=None) == B.STREAM_EINVAL
    assert call(scale=0.0) == B.STREAM_EINVAL
    assert call(scale=float("inf")) == B.STREAM_EINVAL
    assert call(Q=ctypes.c_void_p(4100)) == B.STREAM_EINVAL          # 16-byte loads
    assert call(wsz=need - 1) == B.STREAM_EWORKSPACE
    assert call(wsp=None) == B.STREAM_EWORKSPACE
    assert call(sh=shape(dtype=B.STREAM_F32, head_dim=128, block=128)) == B.STREAM_EUNSUPPORTED
    assert call(sh=shape(dtype=B.STREAM_F32, head_dim=128, block_k=128)) == B.STREAM_EUNSUPPORTED
    assert lib.stream_receiver_stats_workspace_bytes(ctypes.byref(shape(block=48))) == 0


def test_binding_refuses_cpu_tensors():
    import torch
    Q = torch.zeros(2, 64, 64)
    with pytest.raises(ValueError):
        B.stream_prune(Q, Q, 2, 2, 64, 1)
    with pytest.raises(ValueError):
        B.stream_receiver_stats(Q, Q, 2, 2, 64, 0.125)


def test_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: the header compiles as C99 with no C++ in it."""
    import shutil
    import subprocess
    cc = shutil.which("gcc") or shutil.which("cc")
    if cc is None:
        pytest.skip("no C compiler")
    src = tmp_path / "t.c"
    src.write_text('#include "stream.h"\nint main(void) { stream_shape s; (void)s; return (int)STREAM_OK; }\n')
    subprocess.check_call([cc, "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only",
                           "-I", os.path.join(ROOT, "include"), str(src)])
