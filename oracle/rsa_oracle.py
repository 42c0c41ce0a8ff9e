"""CPU fp64 oracle for one rectified block-sparse attention layer (Rectified SpaAttn).

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT. Only the test-suite, the smoke check and
the benchmark's CPU-baseline leg may import it. It shares no code with the HIP path and
must never be used as a fallback for it.

Everything is plain numpy in float64 on the exactly-widened bf16 inputs, one (batch,
head) at a time, written in the order and notation of the paper's Alg. 1. No blocking,
fusion or reordering beyond what the paper states. Where the paper is silent or garbled
the reading taken is stated at the function; the list of readings is:

  R1  masked scores are excluded from the softmax (Sec. 3.1: the mask sits inside the
      denominator sum and a non-critical numerator is 0), not multiplied by 0.
  R2  T_v and T_t need not be multiples of B: the last video block and the last text
      block are ragged, text always starts a block of its own (isolation, Sec. 4.1), and
      the token count c_m of a block replaces B wherever the paper writes B for it.
  R3  IPAR's denominator is the row total sum_m A_v[n,m] c_m + sum_t A_t[n,t]
      ("re-normalization", Sec. 4.1; appendix normaliser sum_m sum_{j in B_m} exp(s^pool)).
  R4  "aggregate by blocks" of the text weights is a sum, so A^pool is a distribution
      over the M blocks, as R_n = "total weight of the critical tokens" needs.
  R5  sparsity ratio rho -> kept blocks per video row k = clamp(M - floor(rho M + 1e-6), 1, M);
      ties in top-k go to the lower block index.
  R6  the kept set with a weight threshold p is the shortest prefix, in descending
      A^pool order, that has at least k blocks and cumulative A^pool > p (Alg. 1 step 13,
      Sec. 4.3, appendix "Implementations").
  R7  GAPR: as printed, the relaxed condition compares |sum_ij s^pool_ij| with
      |sum_ij Delta s_ij|, and the latter is identically zero because block means are
      subtracted (see ``gapr_signed_sums``). The absolute value is therefore taken inside
      the sums, as in the paper's un-relaxed definitions of G and E, on the two
      first-order terms separately:
         a_i = (q_i - q^pool_n) . k^pool_m / sqrt(d),  b_j = q^pool_n . (k_j - k^pool_m) / sqrt(d)
         G[n,m] = | sum_i sum_j s^pool_nm | = c_n c_m |s^pool_nm|
         E[n,m] = sum_i sum_j (|a_i| + |b_j|) = c_m sum_i |a_i| + c_n sum_j |b_j|
         M_c[n,m] = G[n,m] > E[n,m]        (strict, "exceeds")
      This keeps the cost at (tokens x pooled blocks), as "built on pooled vectors"
      requires, and is an upper bound of sum_ij |a_i + b_j| (the exact first-order L1).
      s^pool in G is the raw pooled score (no block-size reweighting); a text block is
      represented by its directly pooled key.
  R8  V^pool covers all M blocks (Alg. 1 step 3 pools V, step 21 multiplies an N x M
      matrix with it).
  R9  M_adja (Alg. 1 "Require", step 14; Sec. 4.3 "retaining spatial-temporal neighbor
      blocks") is not defined further in the paper. Reading: the video latent grid is cut
      into tiles (the tiles of the token order); a video query block and a video key block
      are neighbours when some token of one and some token of the other lie in tiles whose
      tile coordinates differ by at most `radius` (default 1) along every axis -- the
      block itself and, where blocks and tiles coincide, its 26 surrounding tiles. Text
      key blocks are never forced by it.

Parity pins live in tests/test_oracle_*.py. Unpinned (needs the paper's models): the
appendix statistic on softmax denominators, every quality table and alignment figure.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np

__all__ = [
    "bf16_bits_to_f64", "Partition", "partition", "pool", "pooled_scores", "ipar",
    "kept_count", "select_blocks", "tile_order", "reorder_tokens", "adjacency_mask", "rectification_factor", "gapr", "gapr_signed_sums",
    "sparse_attention_block", "sparse_attention", "dense_attention", "compensation", "rectified_layer_head",
    "rectified_layer",
]


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact value of bfloat16 bit patterns (uint16) as float64."""
    u = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


@dataclass(frozen=True)
class Partition:
    """Block partition of the joint [video | text] sequence (Sec. 3.1; reading R2)."""
    t_video: int
    t_text: int
    block: int
    n_video: int          # N: video blocks (query blocks that run sparse, key blocks < N)
    n_text: int           # text blocks
    starts: np.ndarray    # [M] first token of block m
    counts: np.ndarray    # [M] c_m

    @property
    def n_blocks(self) -> int:   # M
        return self.n_video + self.n_text

    def tokens(self, m: int) -> slice:
        return slice(int(self.starts[m]), int(self.starts[m] + self.counts[m]))


def partition(t_video: int, t_text: int, block: int) -> Partition:
    n = -(-t_video // block)
    nt = -(-t_text // block)
    starts = [m * block for m in range(n)] + [t_video + i * block for i in range(nt)]
    counts = [min(block, t_video - m * block) for m in range(n)] + \
             [min(block, t_text - i * block) for i in range(nt)]
    return Partition(t_video, t_text, block, n, nt,
                     np.asarray(starts, dtype=np.int64), np.asarray(counts, dtype=np.int64))


def pool(X: np.ndarray, part: Partition) -> np.ndarray:
    """Uniform pooling per block (Sec. 3.2 pooled equations; Alg. 1 step 3): [M, d] block means."""
    return np.stack([X[part.tokens(m)].mean(axis=0) for m in range(part.n_blocks)], axis=0)


def pooled_scores(Qp: np.ndarray, Kp: np.ndarray, scale: float) -> np.ndarray:
    """S^pool = Q^pool K^pool^T / sqrt(d) (Sec. 3.2)."""
    return (Qp @ Kp.T) * scale


def _softmax_rows(S: np.ndarray) -> np.ndarray:
    E = np.exp(S - S.max(axis=1, keepdims=True))
    return E / E.sum(axis=1, keepdims=True)


def ipar(Qp_video: np.ndarray, Kp_video: np.ndarray, K_text: np.ndarray,
         part: Partition, scale: float) -> np.ndarray:
    """Isolated-Pooling Attention Reallocation (Sec. 4.1; Alg. 1 steps 5-7).

    Mixed keys = [pooled video keys ; individual text tokens]; A_mix = softmax over them;
    video weights are multiplied by the block's token count, everything is re-normalised
    by the row total (R3), text-token weights are summed per text block (R4).
    Returns A^pool [N, M].
    """
    N, nt = part.n_video, part.n_text
    K_mix = np.concatenate([Kp_video, K_text], axis=0)            # [(N + T_t), d]
    A_mix = _softmax_rows((Qp_video @ K_mix.T) * scale)           # [N, N + T_t]
    A_v, A_t = A_mix[:, :N], A_mix[:, N:]
    c_video = part.counts[:N].astype(np.float64)
    weighted_v = A_v * c_video[None, :]
    denom = weighted_v.sum(axis=1, keepdims=True) + A_t.sum(axis=1, keepdims=True)
    A_hat_v = weighted_v / denom
    A_hat_t = A_t / denom
    A_pool = np.empty((N, N + nt), dtype=np.float64)
    A_pool[:, :N] = A_hat_v
    for i in range(nt):
        lo = int(part.starts[N + i]) - part.t_video
        A_pool[:, N + i] = A_hat_t[:, lo:lo + int(part.counts[N + i])].sum(axis=1)
    return A_pool


def kept_count(n_blocks: int, sparsity: float) -> int:
    """Blocks kept per video row for a sparsity ratio (reading R5)."""
    k = n_blocks - int(np.floor(sparsity * n_blocks + 1e-6))
    return max(1, min(n_blocks, k))


def select_blocks(A_pool: np.ndarray, sparsity: float, p: float = 0.0,
                  forced: Optional[np.ndarray] = None) -> np.ndarray:
    """Sparse mask (Alg. 1 steps 13-14; Sec. 4.3): top-k blocks by A^pool, extended
    until the kept weight exceeds p (R6), OR-ed with a caller-supplied forced-keep mask
    (the adjacency mask M_adja). Returns a boolean [N, M] mask."""
    N, M = A_pool.shape
    k = kept_count(M, sparsity)
    mask = np.zeros((N, M), dtype=bool)
    for n in range(N):
        order = np.argsort(-A_pool[n], kind="stable")             # descending, ties -> lower index
        keep = k
        if p > 0.0:
            csum = np.cumsum(A_pool[n][order])
            above = np.nonzero(csum > p)[0]
            k_p = int(above[0]) + 1 if above.size else M
            keep = max(k, k_p)
        mask[n, order[:keep]] = True
    if forced is not None:
        mask |= np.asarray(forced, dtype=bool)
    return mask


def tile_order(grid, tile) -> np.ndarray:
    """Raster index (t*H + h)*W + w of the video token stored at every position of the tile
    order (appendix "Implementations": tokens are reordered so that a block holds spatially
    close tokens; the order used here cuts the (T, H, W) grid into tiles, walks the tiles in
    raster order and the tokens of a tile in raster order). Returns int64 [T*H*W]."""
    T, H, W = (int(x) for x in grid)
    tt, th, tw = (int(x) for x in tile)
    order = []
    for t0 in range(0, T, tt):
        for h0 in range(0, H, th):
            for w0 in range(0, W, tw):
                for t in range(t0, min(t0 + tt, T)):
                    for h in range(h0, min(h0 + th, H)):
                        for w in range(w0, min(w0 + tw, W)):
                            order.append((t * H + h) * W + w)
    return np.asarray(order, dtype=np.int64)


def reorder_tokens(X: np.ndarray, grid, tile, direction: int) -> np.ndarray:
    """Rows of X [T, d] moved between raster order and tile order; text rows (beyond T*H*W)
    keep their place. direction 0: raster -> tile order; 1: tile order -> raster."""
    order = tile_order(grid, tile)
    tv = order.size
    Y = np.array(X, copy=True)
    if direction == 0:
        Y[:tv] = X[order]
    else:
        Y[order] = X[:tv]
    return Y


def adjacency_mask(coords: np.ndarray, tile, part: Partition, radius: int = 1) -> np.ndarray:
    """M_adja (Alg. 1 step 14; Sec. 4.3; reading R9) as a boolean [N, M] mask.

    coords [T_v, 3]: the (t, h, w) latent-grid coordinate of every video token in the order
    the tokens are stored; tile = (tile_t, tile_h, tile_w). Columns of text blocks are False.
    """
    N, M = part.n_video, part.n_blocks
    tile_of = np.asarray(coords, dtype=np.int64) // np.asarray(tile, dtype=np.int64)[None, :]
    tiles = [np.unique(tile_of[part.tokens(n)], axis=0) for n in range(N)]     # tiles block n touches
    mask = np.zeros((N, M), dtype=bool)
    for n in range(N):
        for m in range(N):
            d = np.abs(tiles[n][:, None, :] - tiles[m][None, :, :]).max(axis=2)    # Chebyshev distances
            mask[n, m] = bool((d <= radius).any())
    return mask


def rectification_factor(A_pool: np.ndarray, mask: np.ndarray) -> np.ndarray:
    """R_n = sum over critical blocks of A^pool[n, m] (Sec. 4.1; Alg. 1 step 19)."""
    return (A_pool * mask).sum(axis=1)


def gapr(Q: np.ndarray, K: np.ndarray, Qp: np.ndarray, Kp: np.ndarray,
         part: Partition, scale: float, mode: int = 1):
    """Gain-Aware Pooling Rectification gate (Sec. 4.2; Alg. 1 steps 9-11; reading R7).

    mode 0: never compensate; mode 1: gated, M_c = G > E; mode 2: always compensate.
    Returns (M_c [N, M] bool, G [N, M], E [N, M]).
    """
    N, M = part.n_video, part.n_blocks
    c = part.counts.astype(np.float64)
    s_pool = (Qp[:N] @ Kp.T) * scale                              # raw pooled scores
    G = np.abs(c[:N, None] * c[None, :] * s_pool)
    sum_abs_a = np.empty((N, M))
    for n in range(N):
        dq = Q[part.tokens(n)] - Qp[n][None, :]                   # q_i - q^pool
        sum_abs_a[n] = np.abs((dq @ Kp.T) * scale).sum(axis=0)
    sum_abs_b = np.empty((N, M))
    for m in range(M):
        dk = K[part.tokens(m)] - Kp[m][None, :]                   # k_j - k^pool
        sum_abs_b[:, m] = np.abs((Qp[:N] @ dk.T) * scale).sum(axis=1)
    E = c[None, :] * sum_abs_a + c[:N, None] * sum_abs_b
    if mode == 0:
        Mc = np.zeros((N, M), dtype=bool)
    elif mode == 2:
        Mc = np.ones((N, M), dtype=bool)
    else:
        Mc = G > E
    return Mc, G, E


def gapr_signed_sums(Q, K, Qp, Kp, part: Partition, scale: float) -> np.ndarray:
    """The relaxed condition's right-hand side exactly as printed: sum_i sum_j Delta s_ij
    with the first-order Delta s (Sec. 4.2). Diagnostic only; it vanishes identically,
    which is why reading R7 is needed."""
    N, M = part.n_video, part.n_blocks
    out = np.empty((N, M))
    for n in range(N):
        dq = Q[part.tokens(n)] - Qp[n][None, :]
        for m in range(M):
            dk = K[part.tokens(m)] - Kp[m][None, :]
            ds = ((dq @ Kp[m])[:, None] + (dk @ Qp[n])[None, :]) * scale
            out[n, m] = ds.sum()
    return out


def dense_attention(Q: np.ndarray, K: np.ndarray, V: np.ndarray, scale: float) -> np.ndarray:
    """softmax(Q K^T / sqrt(d)) V (Sec. 3.1, full attention)."""
    return _softmax_rows((Q @ K.T) * scale) @ V


def sparse_attention_block(Q: np.ndarray, K: np.ndarray, V: np.ndarray, mask_row: np.ndarray,
                           n: int, part: Partition, scale: float) -> np.ndarray:
    """Sparse attention of query block n (Sec. 3.1 sparse equation, reading R1; Alg. 1
    step 16): its tokens attend to the tokens of the key blocks with mask_row[m] = 1
    only, and the softmax is taken over those tokens. Returns [c_n, d]."""
    cols = np.concatenate([np.arange(part.starts[m], part.starts[m] + part.counts[m])
                           for m in np.nonzero(mask_row)[0]])
    return dense_attention(Q[part.tokens(n)], K[cols], V[cols], scale)


def sparse_attention(Q: np.ndarray, K: np.ndarray, V: np.ndarray, mask: np.ndarray,
                     part: Partition, scale: float) -> np.ndarray:
    """Block-sparse attention of all video queries, [T_v, d]."""
    out = np.empty((part.t_video, V.shape[1]))
    for n in range(part.n_video):
        out[part.tokens(n)] = sparse_attention_block(Q, K, V, mask[n], n, part, scale)
    return out


def compensation(A_pool: np.ndarray, mask: np.ndarray, Mc: np.ndarray, Vp: np.ndarray) -> np.ndarray:
    """O^ncri per query block (Alg. 1 step 21): (A^pool * (not mask and M_c)) V^pool, [N, d]."""
    return (A_pool * (~mask & Mc)) @ Vp


def rectified_layer_head(Q: np.ndarray, K: np.ndarray, V: np.ndarray, t_video: int, t_text: int,
                         block: int, sparsity: float, p: float = 0.0,
                         forced: Optional[np.ndarray] = None, gapr_mode: int = 1,
                         scale: Optional[float] = None, rectify: bool = True,
                         compensate: bool = True, query_blocks=None) -> dict:
    """Alg. 1 for one (batch, head). Q, K, V: float64 [T_v + T_t, d], tokens [video | text].

    ``query_blocks`` (optional iterable of query-block indices in the joint partition)
    restricts the expensive attention outputs to those blocks; all pooled quantities,
    masks and factors are always computed in full. Returns every intermediate.
    """
    T, d = Q.shape
    assert T == t_video + t_text
    scale = 1.0 / np.sqrt(d) if scale is None else float(scale)
    part = partition(t_video, t_text, block)
    N, M = part.n_video, part.n_blocks

    # steps 1-3: split, pool
    Qp, Kp, Vp = pool(Q, part), pool(K, part), pool(V, part)
    # steps 5-7: implicit full attention
    S_pool = pooled_scores(Qp[:N], Kp, scale)
    A_pool = ipar(Qp[:N], Kp[:N], K[t_video:], part, scale)
    # steps 9-11: compensation mask
    Mc, G, E = gapr(Q, K, Qp, Kp, part, scale, gapr_mode)
    # steps 13-14: sparse mask
    mask = select_blocks(A_pool, sparsity, p, forced)
    # step 19: rectification factor
    R = rectification_factor(A_pool, mask)
    # step 21 (pooled part)
    C = compensation(A_pool, mask, Mc, Vp)

    O = np.full((T, d), np.nan)
    blocks = range(M) if query_blocks is None else [int(x) for x in query_blocks]
    for n in blocks:
        rows = part.tokens(n)
        if n < N:
            # step 16 for this block, then steps 20-22
            o_spa = sparse_attention_block(Q, K, V, mask[n], n, part, scale)
            o = o_spa * R[n] if rectify else o_spa
            if compensate:
                o = o + C[n][None, :]
            O[rows] = o
        else:
            # step 17: text queries keep full attention
            O[rows] = dense_attention(Q[rows], K, V, scale)
    return dict(part=part, Qp=Qp, Kp=Kp, Vp=Vp, S_pool=S_pool, A_pool=A_pool, Mc=Mc, G=G, E=E,
                mask=mask, R=R, C=C, O=O, scale=scale)


def rectified_layer(Q_bits: np.ndarray, K_bits: np.ndarray, V_bits: np.ndarray, t_video: int,
                    t_text: int, block: int, sparsity: float, **kw) -> list:
    """All (batch, head) pairs of bf16-bit inputs [B, H, T, d]; returns a nested list [B][H] of dicts."""
    B, H = Q_bits.shape[:2]
    return [[rectified_layer_head(bf16_bits_to_f64(Q_bits[b, h]), bf16_bits_to_f64(K_bits[b, h]),
                                  bf16_bits_to_f64(V_bits[b, h]), t_video, t_text, block,
                                  sparsity, **kw)
             for h in range(H)] for b in range(B)]
