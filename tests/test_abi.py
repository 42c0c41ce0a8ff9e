"""C-ABI surface: the shared object loads, exports every symbol the header declares, and
rejects bad arguments on the host without launching anything (no GPU needed)."""
import ctypes
import os
import re

import pytest

from paper_2511_19835_amd import binding as rb


@pytest.fixture(scope="module")
def lib(repo_root):
    if not os.path.exists(rb.LIB_PATH):
        from paper_2511_19835_amd.build import build_library
        build_library(verbose=False)
    return rb.load_library()


def test_header_symbols_are_exported(lib, repo_root):
    text = open(os.path.join(repo_root, "include", "rsa.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(rsa_[a-z_]+)\s*\(", text))
    assert declared == set(rb.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def _shape(**kw):
    base = dict(batch=1, heads=2, head_dim=128, block=128, t_video=1000, t_text=50,
                stride_b=2 * 1050 * 128, stride_h=1050 * 128, stride_t=128, scale=0.0)
    base.update(kw)
    return rb.rsa_shape(**base)


def test_block_counts_and_workspace(lib):
    n, m, w = rb.rsa_block_counts(_shape())
    assert (n, m, w) == (8, 9, 1)
    n, m, w = rb.rsa_block_counts(_shape(t_video=118800, t_text=256, heads=24))
    assert (n, m, w) == (929, 931, 30)
    pool_ws, attn_ws = rb.rsa_workspace_bytes(_shape())
    assert pool_ws > 0 and pool_ws % 256 == 0
    # C_n (fp32 [b][h][N][d]), the row order (one int32 per query block, padded to 256 B), then the
    # schedule of the persistent kernel: a table with room for every query block, two counters per queue
    comp, order = 1 * 2 * 8 * 128 * 4, 256
    assert attn_ws % 256 == 0 and attn_ws >= comp + order + 2 * 8 * 4 + 2 * 256
    # the headline shape fits the scratch array of the entry point that allocates nothing
    big = 118800 + 256
    _, attn_big = rb.rsa_workspace_bytes(_shape(t_video=118800, t_text=256, heads=24, stride_b=24 * big * 128,
                                                stride_h=big * 128))
    assert attn_big <= rb.RSA_STATIC_SCRATCH_BYTES


@pytest.mark.parametrize("kw,code", [
    (dict(head_dim=96), -3), (dict(block=32), -3), (dict(batch=0), -2), (dict(t_video=0), -2),
    (dict(t_text=-1), -2), (dict(stride_t=100), -2), (dict(stride_t=132), -2),
    (dict(t_video=128 * 5000), -3), (dict(scale=-1.0), -5),
    (dict(stride_t=1 << 23), -3),            # 128 rows * 2^23 elements * 2 B = 2^31: past the 32-bit row offsets
])
def test_bad_shapes_are_rejected(lib, kw, code):
    with pytest.raises(rb.RsaError) as e:
        rb.rsa_block_counts(_shape(**kw))
    assert e.value.status == code


def test_null_and_range_arguments_are_rejected_before_launch(lib):
    sh = _shape()
    one = ctypes.c_void_p(256)     # never dereferenced: validation fails first
    args = [one] * 11
    assert lib.rsa_pool(ctypes.byref(sh), *([None] + args[1:]), 1, one, 1 << 30, None) == -1
    assert lib.rsa_pool(ctypes.byref(sh), *args, 5, one, 1 << 30, None) == -5
    assert lib.rsa_pool(ctypes.byref(sh), *args, 1, one, 16, None) == -4
    assert lib.rsa_pool(ctypes.byref(sh), *args, 1, ctypes.c_void_p(8), 1 << 30, None) == -4
    assert lib.rsa_pool_values(ctypes.byref(sh), one, None, one, None) == -1
    assert lib.rsa_implicit_attention(ctypes.byref(sh), one, one, one, one, None, one, None) == -1
    sel = lambda sp, p, l=one: lib.rsa_select_blocks(ctypes.byref(sh), l, one, sp, p, None, one, one, one, one, None)
    assert sel(1.5, 0.0) == -5 and sel(0.5, -0.1) == -5 and sel(float("nan"), 0.0) == -5
    assert sel(0.5, 0.0, None) == -1
    att = lambda flags, q=one, lists=one: lib.rsa_sparse_attn_rectified(
        ctypes.byref(sh), q, one, one, lists, lists, one, one, one, one, one, flags, one, None, None, 0, None)
    assert att(8) == -5 and att(3, None) == -1 and att(3, one, None) == -1
    # RSA_COMPENSATE needs the C_n workspace: present, large enough, 256-byte aligned
    attw = lambda flags, ws, nbytes: lib.rsa_sparse_attn_rectified(
        ctypes.byref(sh), one, one, one, one, one, one, one, one, one, one, flags, one, None, ws, nbytes, None)
    assert attw(3, None, 0) == -1 and attw(2, one, 16) == -4 and attw(2, ctypes.c_void_p(8), 1 << 30) == -4
    # the entry point with built-in scratch: same checks, and shapes beyond its array are refused on the host
    atts = lambda shape, flags, q=one: lib.rsa_sparse_attn_rectified_static(
        ctypes.byref(shape), q, one, one, one, one, one, one, one, one, one, flags, one, None, None)
    assert atts(sh, 8) == -5 and atts(sh, 3, None) == -1
    t = 118800
    big = _shape(heads=48, t_video=t, t_text=0, stride_b=48 * t * 128, stride_h=t * 128)
    assert rb.rsa_workspace_bytes(big)[1] > rb.RSA_STATIC_SCRATCH_BYTES and atts(big, 3) == -4
    # adjacency mask: grid must multiply out to t_video, tile entries positive, radius in range
    i3 = lambda *v: (ctypes.c_int32 * 3)(*v)
    adj = lambda grid, tile, radius, out=one: lib.rsa_adjacency_mask(ctypes.byref(sh), grid, tile, radius, out, None)
    assert adj(i3(10, 10, 10), i3(2, 8, 8), 1, None) == -1 and adj(None, i3(2, 8, 8), 1) == -1
    assert adj(i3(10, 10, 11), i3(2, 8, 8), 1) == -2 and adj(i3(10, 10, 10), i3(2, 0, 8), 1) == -2
    assert adj(i3(10, 10, 10), i3(2, 8, 8), -1) == -5 and adj(i3(10, 10, 10), i3(2, 8, 8), 65) == -5
    reo = lambda grid, direction, src=one, dst=ctypes.c_void_p(512): lib.rsa_reorder_tokens(
        ctypes.byref(sh), grid, i3(2, 8, 8), direction, src, dst, None)
    assert reo(i3(10, 10, 10), 0, None) == -1 and reo(i3(10, 10, 11), 0) == -2
    assert reo(i3(10, 10, 10), 2) == -5 and reo(i3(10, 10, 10), 0, one, one) == -5
    assert lib.rsa_status_string(-4).decode().startswith("workspace")
    assert lib.rsa_status_string(0).decode() == "ok"


def test_binding_refuses_cpu_tensors(lib):
    import torch
    q = torch.zeros(1, 2, 1050, 128, dtype=torch.bfloat16)
    sh = rb.make_shape(q, 1000, 50, 128)
    with pytest.raises(RuntimeError, match="device tensors only"):
        rb.rsa_pool(sh, q, q, q, q, q, q, q, q, q, q, q, 1, q)
