"""Seeded synthetic inputs for the rectified sparse-attention layer.

This module only *draws inputs*; it holds none of the method's arithmetic and is the
one piece shared by the CPU oracle's tests and the HIP path's tests/bench. It stands in
for the activations of the video DiTs the paper measures on (HunyuanVideo, Wan 2.1):
those models, their weights and their prompt sets are not available, so tensors with
the same shapes are drawn from a smooth-field-plus-noise distribution that mimics the
intra-block homogeneity of video tokens (paper Sec. 1, Sec. 3.2) and the inhomogeneity
of text tokens (paper Sec. 4.1).

Recipe (per batch item and head, generator ``numpy.random.default_rng([seed, b, h])``):
  * video tokens are enumerated tile by tile over the (T, H, W) latent grid -- tile
    (1, 8, 8) for block 64 and (2, 8, 8) for block 128, tiles in raster order, tokens in
    raster order inside a tile, coordinates outside the grid skipped;
  * four integer wave vectors f_r in {0..3}^3 (not all zero); per sinusoid r and channel
    c a phase phi ~ U[0, 2 pi) and an amplitude a ~ N(0, sigma_a);
    field_c(x) = sum_r a[r, c] sin(2 pi f_r . x / (T, H, W) + phi[r, c]);
  * Q_video = field + N(0, 0.5), K_video = field + N(0, 0.5) (same field, independent
    noise); text Q, K ~ N(0, 1.5); V ~ N(0, 1) for every token (all std);
  * values are rounded once to bf16 (round-to-nearest-even); the uint16 bit patterns are
    what both the oracle and the GPU receive.
"""
from __future__ import annotations

import hashlib
from dataclasses import dataclass, field, replace
from typing import Iterable, Optional, Tuple

import numpy as np

__all__ = [
    "LayerConfig", "CONFIGS", "default_tile", "tile_order_coords", "make_head", "make_inputs",
    "f32_to_bf16_bits", "bf16_bits_to_f32", "sha256_of",
]


@dataclass(frozen=True)
class LayerConfig:
    """Shape of one attention layer call. Token order is [video | text]."""
    name: str
    batch: int
    heads: int
    head_dim: int
    grid: Tuple[int, int, int]          # latent (T, H, W); t_video = T*H*W
    t_text: int
    block: int
    sparsity: float
    sigma_a: float = 0.5                # amplitude std of the sinusoid bank
    noise_std: float = 0.5
    text_std: float = 1.5

    @property
    def t_video(self) -> int:
        return int(self.grid[0] * self.grid[1] * self.grid[2])

    @property
    def t_total(self) -> int:
        return self.t_video + self.t_text

    @property
    def n_video_blocks(self) -> int:
        return -(-self.t_video // self.block)

    @property
    def n_text_blocks(self) -> int:
        return -(-self.t_text // self.block)

    @property
    def n_blocks(self) -> int:
        return self.n_video_blocks + self.n_text_blocks

    def with_(self, **kw) -> "LayerConfig":
        return replace(self, **kw)


CONFIGS = {
    # the small case the CPU oracle finishes in well under a second
    "tiny": LayerConfig("tiny", 1, 2, 64, (4, 16, 16), 64, 64, 0.75),
    "mid": LayerConfig("mid", 1, 24, 128, (13, 30, 52), 0, 128, 0.90),
    "wan": LayerConfig("wan", 1, 40, 128, (21, 45, 80), 0, 128, 0.90),
    "hunyuan": LayerConfig("hunyuan", 1, 24, 128, (33, 45, 80), 256, 128, 0.90),
    # a 2-D image DiT shape (one latent frame of 256 x 256 tokens, 512 text tokens): stands in for the
    # paper's 4K Flux.1-dev runs, which keep 10-25 % of the blocks
    "flux": LayerConfig("flux", 1, 24, 128, (1, 256, 256), 512, 128, 0.90),
}


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to float32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def default_tile(block: int) -> Tuple[int, int, int]:
    """Tile of the token order used for a block size: 64 tokens = (1, 8, 8), 128 = (2, 8, 8)."""
    return (1, 8, 8) if block <= 64 else (2, 8, 8)


def tile_order_coords(grid: Tuple[int, int, int], block: int,
                      tile: Optional[Tuple[int, int, int]] = None) -> np.ndarray:
    """(t, h, w) coordinate of every video token in tile order, shape [T*H*W, 3]."""
    if tile is None:
        tile = default_tile(block)
    T, H, W = grid
    out = []
    for t0 in range(0, T, tile[0]):
        for h0 in range(0, H, tile[1]):
            for w0 in range(0, W, tile[2]):
                t = np.arange(t0, min(t0 + tile[0], T))
                h = np.arange(h0, min(h0 + tile[1], H))
                w = np.arange(w0, min(w0 + tile[2], W))
                tt, hh, ww = np.meshgrid(t, h, w, indexing="ij")
                out.append(np.stack([tt.ravel(), hh.ravel(), ww.ravel()], axis=1))
    coords = np.concatenate(out, axis=0).astype(np.int32)
    assert coords.shape[0] == T * H * W
    return coords


def make_head(cfg: LayerConfig, seed: int, b: int, h: int,
              coords: Optional[np.ndarray] = None):
    """Draw Q, K, V of one (batch item, head): three uint16 [t_total, head_dim] arrays."""
    rng = np.random.default_rng([int(seed), int(b), int(h)])
    d, tv, tt = cfg.head_dim, cfg.t_video, cfg.t_text
    if coords is None:
        coords = tile_order_coords(cfg.grid, cfg.block)
    while True:
        f = rng.integers(0, 4, size=(4, 3))
        if np.all(f.any(axis=1)):
            break
    phi = rng.uniform(0.0, 2.0 * np.pi, size=(4, d))
    amp = rng.normal(0.0, cfg.sigma_a, size=(4, d))
    theta = 2.0 * np.pi * (coords.astype(np.float64) / np.asarray(cfg.grid, dtype=np.float64)) @ f.T.astype(np.float64)
    fld = (np.sin(theta) @ (amp * np.cos(phi)) + np.cos(theta) @ (amp * np.sin(phi))).astype(np.float32)

    def noise(n, std):
        return rng.standard_normal(size=(n, d), dtype=np.float32) * np.float32(std)

    q = np.empty((tv + tt, d), dtype=np.float32)
    k = np.empty((tv + tt, d), dtype=np.float32)
    q[:tv] = fld + noise(tv, cfg.noise_std)
    k[:tv] = fld + noise(tv, cfg.noise_std)
    if tt:
        q[tv:] = noise(tt, cfg.text_std)
        k[tv:] = noise(tt, cfg.text_std)
    v = noise(tv + tt, 1.0)
    return f32_to_bf16_bits(q), f32_to_bf16_bits(k), f32_to_bf16_bits(v)


def _make_head_job(job):
    cfg, seed, b, h = job
    return make_head(cfg, seed, b, h)


def make_inputs(cfg: LayerConfig, seed: int = 0, heads: Optional[Iterable[int]] = None, workers: int = 1,
                threads: bool = False):
    """Q, K, V as uint16 bf16 bit patterns, shape [batch, len(heads), t_total, head_dim].

    ``heads`` selects a subset of head indices (each head has its own generator stream,
    so a subset reproduces exactly the same bits as the full draw). ``workers`` > 1 draws
    heads in forked worker processes (call it before the process touches the GPU) or, with
    ``threads=True``, in threads of this process.
    """
    hs = list(range(cfg.heads)) if heads is None else list(heads)
    shape = (cfg.batch, len(hs), cfg.t_total, cfg.head_dim)
    Q = np.empty(shape, dtype=np.uint16)
    K = np.empty(shape, dtype=np.uint16)
    V = np.empty(shape, dtype=np.uint16)
    jobs = [(cfg, seed, b, h) for b in range(cfg.batch) for h in hs]
    if workers > 1 and len(jobs) > 1:
        import concurrent.futures
        pool = concurrent.futures.ThreadPoolExecutor if threads else concurrent.futures.ProcessPoolExecutor
        with pool(max_workers=min(workers, len(jobs))) as ex:
            results = list(ex.map(_make_head_job, jobs))
    else:
        coords = tile_order_coords(cfg.grid, cfg.block)
        results = [make_head(cfg, seed, b, h, coords) for (_, _, b, h) in jobs]
    it = iter(results)
    for b in range(cfg.batch):
        for i in range(len(hs)):
            Q[b, i], K[b, i], V[b, i] = next(it)
    return Q, K, V


def sha256_of(*arrays: np.ndarray) -> str:
    m = hashlib.sha256()
    for a in arrays:
        m.update(np.ascontiguousarray(a).tobytes())
    return m.hexdigest()
