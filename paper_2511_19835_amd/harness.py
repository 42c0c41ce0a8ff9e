"""Host-side plumbing around the binding: upload bit patterns, run a layer, download.

No arithmetic of the method happens here; it exists so tests, the smoke check and the
benchmark drive the C-ABI the same way.
"""
from __future__ import annotations

from typing import Optional

import numpy as np
import torch

from . import binding as rb


def bits_to_device(bits: np.ndarray, device="cuda:0", layout: str = "bhtd") -> torch.Tensor:
    """uint16 bf16 bit patterns [B,H,T,d] -> bf16 device tensor viewed as [B,H,T,d].

    layout "bhtd": contiguous as given; "bthd": memory order [B,T,H,d] (heads interleaved
    per token), returned as a permuted view so the strides differ."""
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(device).view(torch.bfloat16)
    if layout == "bhtd":
        return t
    if layout == "bthd":
        return t.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    raise ValueError(layout)


def device_to_bits(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def unpack_bits(words: np.ndarray, n_bits: int) -> np.ndarray:
    """[..., W] int32/uint32 words -> [..., n_bits] bool (bit m%32 of word m/32)."""
    w = np.ascontiguousarray(words).view(np.uint32)
    bits = (w[..., :, None] >> np.arange(32, dtype=np.uint32)) & np.uint32(1)
    return bits.reshape(*w.shape[:-1], -1)[..., :n_bits].astype(bool)


def pack_bits(mask: np.ndarray) -> np.ndarray:
    """[..., M] bool -> [..., ceil(M/32)] int32 words."""
    M = mask.shape[-1]
    W = (M + 31) // 32
    padded = np.zeros(mask.shape[:-1] + (W * 32,), dtype=np.uint32)
    padded[..., :M] = mask
    words = (padded.reshape(*mask.shape[:-1], W, 32) << np.arange(32, dtype=np.uint32)).sum(axis=-1, dtype=np.uint64)
    return words.astype(np.uint32).view(np.int32)


def run_layer(Q_bits: np.ndarray, K_bits: np.ndarray, V_bits: np.ndarray, t_video: int, t_text: int,
              block: int, sparsity: float, p: float = 0.0, gapr_mode: int = 1,
              forced: Optional[np.ndarray] = None, flags: int = rb.RSA_RECTIFY_CRITICAL | rb.RSA_COMPENSATE,
              scale: float = 0.0, layout: str = "bhtd", device="cuda:0", want_lse: bool = True,
              attn_workspace: bool = True) -> dict:
    """Run the three entry points on the GPU and bring every buffer back as numpy. O starts out as
    NaN in every element, so a row that no kernel writes shows up in any comparison.
    ``attn_workspace=False`` passes ws = NULL to the attention call (legal without RSA_COMPENSATE)."""
    Q = bits_to_device(Q_bits, device, layout)
    K = bits_to_device(K_bits, device, layout)
    V = bits_to_device(V_bits, device, layout)
    O = torch.full_like(Q, float("nan"))
    buf = rb.allocate(Q, t_video, t_text, block, scale)
    if not attn_workspace:
        buf.attn_ws = None
    forced_dev = None
    if forced is not None:
        forced_dev = torch.from_numpy(pack_bits(np.asarray(forced, dtype=bool))).to(device)
    B, H, T, _ = Q.shape
    lse = torch.empty(B, H, T, dtype=torch.float32, device=device) if want_lse else None
    rb.rectified_sparse_attention(Q, K, V, O, buf, sparsity, p, gapr_mode, forced_dev, flags, lse)
    torch.cuda.synchronize()
    out = dict(
        N=buf.N, M=buf.M, W=buf.W,
        Qp=buf.Qp.cpu().numpy(), Kp=buf.Kp.cpu().numpy(), Vp=buf.Vp.cpu().numpy(),
        Vt_bits=device_to_bits(buf.Vt),
        Spool=buf.Spool.cpu().numpy(), Apool=buf.Apool.cpu().numpy(), Lmass=buf.Lmass.cpu().numpy(),
        Mc=unpack_bits(buf.Mc_bits.cpu().numpy(), buf.M), mask=unpack_bits(buf.mask_bits.cpu().numpy(), buf.M),
        Mc_words=buf.Mc_bits.cpu().numpy(), mask_words=buf.mask_bits.cpu().numpy(),
        block_idx=buf.block_idx.cpu().numpy(), count=buf.count.cpu().numpy(), R=buf.R.cpu().numpy(),
        O_bits=device_to_bits(O), lse=lse.cpu().numpy() if lse is not None else None,
    )
    return out


def adjacency_mask(t_video: int, t_text: int, block: int, head_dim: int, grid, tile, radius: int = 1,
                   batch: int = 1, heads: int = 1, device="cuda:0") -> np.ndarray:
    """rsa_adjacency_mask on the GPU, brought back as a boolean [batch, heads, N, M] array."""
    t = t_video + t_text
    shape = rb.rsa_shape(batch=batch, heads=heads, head_dim=head_dim, block=block, t_video=t_video, t_text=t_text,
                         stride_b=heads * t * head_dim, stride_h=t * head_dim, stride_t=head_dim, scale=0.0)
    n, m, w = rb.rsa_block_counts(shape)
    bits = torch.full((batch, heads, n, w), -1, dtype=torch.int32, device=device)   # must be fully overwritten
    rb.rsa_adjacency_mask(shape, grid, tile, radius, bits)
    torch.cuda.synchronize()
    words = bits.cpu().numpy().view(np.uint32)
    assert (words[..., -1] >> np.uint32((m - 1) % 32 + 1) == 0).all() or m % 32 == 0, "bits past M must be clear"
    return unpack_bits(words, m)


def reorder_tokens(X_bits: np.ndarray, t_video: int, t_text: int, block: int, grid, tile, direction: int,
                   layout: str = "bhtd", device="cuda:0") -> np.ndarray:
    """rsa_reorder_tokens on the GPU for a [B, H, T, d] tensor of bf16 bit patterns."""
    X = bits_to_device(X_bits, device, layout)
    Y = torch.full_like(X, float("nan"))                      # every row must be overwritten
    shape = rb.make_shape(X, t_video, t_text, block)
    rb.rsa_reorder_tokens(shape, grid, tile, direction, X, Y)
    torch.cuda.synchronize()
    return device_to_bits(Y)


def run_layer_from_raster(Q_bits, K_bits, V_bits, grid, tile, t_text: int, block: int, sparsity: float,
                          p: float = 0.0, use_adjacency: bool = False, device="cuda:0") -> np.ndarray:
    """The whole sequence a caller with raster-ordered tokens runs, all on the device: reorder
    Q, K, V into tile order, (optionally) generate the adjacency mask, the three layer calls, and
    reorder O back. Returns O as bf16 bit patterns in raster order."""
    t_video = int(grid[0]) * int(grid[1]) * int(grid[2])
    Qr, Kr, Vr = (bits_to_device(x, device) for x in (Q_bits, K_bits, V_bits))
    shape = rb.make_shape(Qr, t_video, t_text, block)
    Q, K, V, O, Or = (torch.full_like(Qr, float("nan")) for _ in range(5))
    for src, dst in ((Qr, Q), (Kr, K), (Vr, V)):
        rb.rsa_reorder_tokens(shape, grid, tile, 0, src, dst)
    buf = rb.allocate(Q, t_video, t_text, block)
    forced = None
    if use_adjacency:
        forced = torch.empty_like(buf.mask_bits)
        rb.rsa_adjacency_mask(buf.shape, grid, tile, 1, forced)
    rb.rectified_sparse_attention(Q, K, V, O, buf, sparsity, p, 1, forced,
                                  rb.RSA_RECTIFY_CRITICAL | rb.RSA_COMPENSATE, None)
    rb.rsa_reorder_tokens(shape, grid, tile, 1, O, Or)
    torch.cuda.synchronize()
    return device_to_bits(Or)


def run_two_steps_reusing_masks(step1, step2, t_video: int, t_text: int, block: int, sparsity: float,
                                device="cuda:0") -> dict:
    """Step 1: the whole layer on (Q1, K1, V1). Step 2: only rsa_pool_values(V2) and the attention
    call on (Q2, K2, V2), with the lists, factors, A^pool and gate bits step 1 left in the buffers.
    Returns the step-1 mask / gate / R / A^pool and both outputs (bf16 bit patterns)."""
    Q1, K1, V1 = (bits_to_device(x, device) for x in step1)
    Q2, K2, V2 = (bits_to_device(x, device) for x in step2)
    O1, O2 = torch.full_like(Q1, float("nan")), torch.full_like(Q2, float("nan"))
    buf = rb.allocate(Q1, t_video, t_text, block)
    flags = rb.RSA_RECTIFY_CRITICAL | rb.RSA_COMPENSATE
    rb.rectified_sparse_attention(Q1, K1, V1, O1, buf, sparsity, 0.0, 1, None, flags, None)
    rb.rsa_pool_values(buf.shape, V2, buf.Vp, buf.Vt)
    rb.rsa_sparse_attn_rectified(buf.shape, Q2, K2, buf.Vt, buf.block_idx, buf.count, buf.mask_bits, buf.R,
                                 buf.Apool, buf.Mc_bits, buf.Vp, flags, O2, None, buf.attn_ws)
    torch.cuda.synchronize()
    return dict(mask=unpack_bits(buf.mask_bits.cpu().numpy(), buf.M), Mc=unpack_bits(buf.Mc_bits.cpu().numpy(), buf.M),
                R=buf.R.cpu().numpy(), Apool=buf.Apool.cpu().numpy(), Vp=buf.Vp.cpu().numpy(),
                O1_bits=device_to_bits(O1), O2_bits=device_to_bits(O2))
