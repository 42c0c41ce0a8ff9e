"""Thin ctypes binding of librsa.so: argument marshalling only.

The entry points carry the names of the C-ABI (include/rsa.h). Tensors are torch CUDA
(ROCm) tensors used purely as device buffers; every step of the method runs inside the
library's HIP kernels. There is no CPU fallback: if the shared object is missing or the
tensors are not on the GPU the calls raise.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librsa.so")

RSA_RECTIFY_CRITICAL = 1
RSA_COMPENSATE = 2
RSA_DENSE = 4
RSA_MAX_BLOCKS = 4096
RSA_STATIC_SCRATCH_BYTES = 16 << 20

EXPORTS = (
    "rsa_block_counts", "rsa_workspace_bytes", "rsa_pool", "rsa_pool_values", "rsa_implicit_attention", "rsa_adjacency_mask", "rsa_reorder_tokens", "rsa_select_blocks",
    "rsa_sparse_attn_rectified", "rsa_sparse_attn_rectified_static", "rsa_status_string",
)


class RsaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = _lib().rsa_status_string(status).decode() if _LIB is not None else str(status)
        super().__init__(f"{where}: {msg} ({status})")


class rsa_shape(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("block", ctypes.c_int32),
        ("t_video", ctypes.c_int64), ("t_text", ctypes.c_int64),
        ("stride_b", ctypes.c_int64), ("stride_h", ctypes.c_int64), ("stride_t", ctypes.c_int64),
        ("scale", ctypes.c_float),
    ]


_LIB: Optional[ctypes.CDLL] = None


def _lib() -> ctypes.CDLL:
    """Load librsa.so (built by ``python -m paper_2511_19835_amd.build``); never falls back."""
    global _LIB
    if _LIB is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2511_19835_amd.build` "
                "(there is no fallback path)")
        lib = ctypes.CDLL(LIB_PATH)
        vp, i64p, szp = ctypes.c_void_p, ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_size_t)
        shp = ctypes.POINTER(rsa_shape)
        lib.rsa_block_counts.argtypes = [shp, i64p, i64p, i64p]
        lib.rsa_block_counts.restype = ctypes.c_int
        lib.rsa_workspace_bytes.argtypes = [shp, szp, szp]
        lib.rsa_workspace_bytes.restype = ctypes.c_int
        lib.rsa_pool.argtypes = [shp] + [vp] * 11 + [ctypes.c_int, vp, ctypes.c_size_t, vp]
        lib.rsa_pool.restype = ctypes.c_int
        lib.rsa_pool_values.argtypes = [shp, vp, vp, vp, vp]
        lib.rsa_pool_values.restype = ctypes.c_int
        lib.rsa_implicit_attention.argtypes = [shp] + [vp] * 7
        lib.rsa_implicit_attention.restype = ctypes.c_int
        lib.rsa_select_blocks.argtypes = [shp, vp, vp, ctypes.c_double, ctypes.c_double, vp, vp, vp, vp, vp, vp]
        lib.rsa_select_blocks.restype = ctypes.c_int
        lib.rsa_sparse_attn_rectified.argtypes = [shp] + [vp] * 10 + [ctypes.c_int, vp, vp, vp, ctypes.c_size_t, vp]
        lib.rsa_sparse_attn_rectified.restype = ctypes.c_int
        lib.rsa_sparse_attn_rectified_static.argtypes = [shp] + [vp] * 10 + [ctypes.c_int, vp, vp, vp]
        lib.rsa_sparse_attn_rectified_static.restype = ctypes.c_int
        lib.rsa_adjacency_mask.argtypes = [shp, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32), ctypes.c_int, vp, vp]
        lib.rsa_adjacency_mask.restype = ctypes.c_int
        lib.rsa_reorder_tokens.argtypes = [shp, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32), ctypes.c_int, vp, vp, vp]
        lib.rsa_reorder_tokens.restype = ctypes.c_int
        lib.rsa_status_string.argtypes = [ctypes.c_int]
        lib.rsa_status_string.restype = ctypes.c_char_p
        _LIB = lib
    return _LIB


def load_library() -> ctypes.CDLL:
    return _lib()


def _check(status: int, where: str) -> None:
    if status != 0:
        raise RsaError(status, where)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise RuntimeError("librsa takes device tensors only (no CPU path)")
    return t.data_ptr()


def _stream_ptr(stream: Optional[torch.cuda.Stream]) -> int:
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream


def make_shape(q: torch.Tensor, t_video: int, t_text: int, block: int, scale: float = 0.0) -> rsa_shape:
    """Shape record for a [batch, heads, T, d] view of bf16 Q/K/V/O (any b/h/t strides)."""
    assert q.dim() == 4 and q.stride(3) == 1, "expect [batch, heads, tokens, head_dim], last dim contiguous"
    assert q.shape[2] == t_video + t_text
    return rsa_shape(q.shape[0], q.shape[1], q.shape[3], block, t_video, t_text,
                     q.stride(0), q.stride(1), q.stride(2), scale)


def rsa_block_counts(shape: rsa_shape):
    n, m, w = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
    _check(_lib().rsa_block_counts(ctypes.byref(shape), ctypes.byref(n), ctypes.byref(m), ctypes.byref(w)),
           "rsa_block_counts")
    return n.value, m.value, w.value


def rsa_workspace_bytes(shape: rsa_shape):
    a, b = ctypes.c_size_t(), ctypes.c_size_t()
    _check(_lib().rsa_workspace_bytes(ctypes.byref(shape), ctypes.byref(a), ctypes.byref(b)), "rsa_workspace_bytes")
    return a.value, b.value


def rsa_pool(shape, Q, K, V, Qp, Kp, Vp, Vt, Spool, Apool, Lmass, Mc_bits, gapr_mode, ws, stream=None):
    _check(_lib().rsa_pool(ctypes.byref(shape), _ptr(Q), _ptr(K), _ptr(V), _ptr(Qp), _ptr(Kp), _ptr(Vp), _ptr(Vt),
                           _ptr(Spool), _ptr(Apool), _ptr(Lmass), _ptr(Mc_bits), int(gapr_mode),
                           _ptr(ws), ws.numel() * ws.element_size() if ws is not None else 0,
                           _stream_ptr(stream)), "rsa_pool")


def rsa_implicit_attention(shape, K, Qp, Kp, Spool, Lmass, Apool, stream=None):
    _check(_lib().rsa_implicit_attention(ctypes.byref(shape), _ptr(K), _ptr(Qp), _ptr(Kp), _ptr(Spool), _ptr(Lmass),
                                         _ptr(Apool), _stream_ptr(stream)), "rsa_implicit_attention")


def rsa_pool_values(shape, V, Vp, Vt, stream=None):
    _check(_lib().rsa_pool_values(ctypes.byref(shape), _ptr(V), _ptr(Vp), _ptr(Vt), _stream_ptr(stream)),
           "rsa_pool_values")


def rsa_select_blocks(shape, Lmass, Apool, sparsity, p, forced_bits, mask_bits, block_idx, count, R, stream=None):
    _check(_lib().rsa_select_blocks(ctypes.byref(shape), _ptr(Lmass), _ptr(Apool), float(sparsity), float(p),
                                    _ptr(forced_bits), _ptr(mask_bits), _ptr(block_idx), _ptr(count), _ptr(R),
                                    _stream_ptr(stream)), "rsa_select_blocks")


def rsa_adjacency_mask(shape, grid, tile, radius, forced_bits, stream=None):
    g = (ctypes.c_int32 * 3)(*[int(x) for x in grid])
    t = (ctypes.c_int32 * 3)(*[int(x) for x in tile])
    _check(_lib().rsa_adjacency_mask(ctypes.byref(shape), g, t, int(radius), _ptr(forced_bits), _stream_ptr(stream)),
           "rsa_adjacency_mask")


def rsa_reorder_tokens(shape, grid, tile, direction, src, dst, stream=None):
    g = (ctypes.c_int32 * 3)(*[int(x) for x in grid])
    t = (ctypes.c_int32 * 3)(*[int(x) for x in tile])
    _check(_lib().rsa_reorder_tokens(ctypes.byref(shape), g, t, int(direction), _ptr(src), _ptr(dst),
                                     _stream_ptr(stream)), "rsa_reorder_tokens")


def rsa_sparse_attn_rectified(shape, Q, K, Vt, block_idx, count, mask_bits, R, Apool, Mc_bits, Vp, flags, O,
                              lse=None, ws=None, stream=None):
    _check(_lib().rsa_sparse_attn_rectified(
        ctypes.byref(shape), _ptr(Q), _ptr(K), _ptr(Vt), _ptr(block_idx), _ptr(count), _ptr(mask_bits), _ptr(R),
        _ptr(Apool), _ptr(Mc_bits), _ptr(Vp), int(flags), _ptr(O), _ptr(lse), _ptr(ws),
        ws.numel() * ws.element_size() if ws is not None else 0, _stream_ptr(stream)),
        "rsa_sparse_attn_rectified")


def rsa_sparse_attn_rectified_static(shape, Q, K, Vt, block_idx, count, mask_bits, R, Apool, Mc_bits, Vp, flags, O,
                                     lse=None, stream=None):
    _check(_lib().rsa_sparse_attn_rectified_static(
        ctypes.byref(shape), _ptr(Q), _ptr(K), _ptr(Vt), _ptr(block_idx), _ptr(count), _ptr(mask_bits), _ptr(R),
        _ptr(Apool), _ptr(Mc_bits), _ptr(Vp), int(flags), _ptr(O), _ptr(lse), _stream_ptr(stream)),
        "rsa_sparse_attn_rectified_static")


@dataclass
class LayerBuffers:
    """Caller-owned device buffers of one layer call, allocated once with torch."""
    shape: rsa_shape
    N: int
    M: int
    W: int
    Qp: torch.Tensor
    Kp: torch.Tensor
    Vp: torch.Tensor
    Vt: torch.Tensor
    Spool: torch.Tensor
    Apool: torch.Tensor
    Lmass: torch.Tensor
    Mc_bits: torch.Tensor
    mask_bits: torch.Tensor
    block_idx: torch.Tensor
    count: torch.Tensor
    R: torch.Tensor
    pool_ws: torch.Tensor
    attn_ws: Optional[torch.Tensor]


def allocate(q: torch.Tensor, t_video: int, t_text: int, block: int, scale: float = 0.0) -> LayerBuffers:
    shape = make_shape(q, t_video, t_text, block, scale)
    N, M, W = rsa_block_counts(shape)
    pool_ws, attn_ws = rsa_workspace_bytes(shape)
    B, H, _, d = q.shape
    dev = q.device
    f32 = dict(dtype=torch.float32, device=dev)
    i32 = dict(dtype=torch.int32, device=dev)
    return LayerBuffers(
        shape, N, M, W,
        Qp=torch.empty(B, H, N, d, **f32), Kp=torch.empty(B, H, M, d, **f32), Vp=torch.empty(B, H, M, d, **f32),
        Vt=torch.empty(B, H, M, d, block, dtype=torch.bfloat16, device=dev),
        Spool=torch.empty(B, H, N, M, **f32), Apool=torch.empty(B, H, N, M, **f32),
        Lmass=torch.empty(B, H, N, M, **f32),
        Mc_bits=torch.empty(B, H, N, W, **i32), mask_bits=torch.empty(B, H, N, W, **i32),
        block_idx=torch.empty(B, H, N, M, **i32), count=torch.empty(B, H, N, **i32), R=torch.empty(B, H, N, **f32),
        pool_ws=torch.empty(max(pool_ws, 256), dtype=torch.uint8, device=dev),
        attn_ws=torch.empty(attn_ws, dtype=torch.uint8, device=dev) if attn_ws else None,
    )


def rectified_sparse_attention(Q, K, V, O, buf: LayerBuffers, sparsity: float, p: float = 0.0,
                               gapr_mode: int = 1, forced_bits=None,
                               flags: int = RSA_RECTIFY_CRITICAL | RSA_COMPENSATE, lse=None, stream=None):
    """One layer: the three C-ABI calls back to back on one stream, no host sync."""
    rsa_pool(buf.shape, Q, K, V, buf.Qp, buf.Kp, buf.Vp, buf.Vt, buf.Spool, buf.Apool, buf.Lmass, buf.Mc_bits,
             gapr_mode, buf.pool_ws, stream)
    rsa_select_blocks(buf.shape, buf.Lmass, buf.Apool, sparsity, p, forced_bits, buf.mask_bits, buf.block_idx,
                      buf.count, buf.R, stream)
    rsa_sparse_attn_rectified(buf.shape, Q, K, buf.Vt, buf.block_idx, buf.count, buf.mask_bits, buf.R, buf.Apool,
                              buf.Mc_bits, buf.Vp, flags, O, lse, buf.attn_ws, stream)
    return O
