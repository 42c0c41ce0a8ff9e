"""Token-level brute force of the rectified sparse-attention layer, for tiny inputs only.

TEST INFRASTRUCTURE. A second, deliberately different way to reach what
``rsa_oracle.rectified_layer_head`` computes: instead of block-level matrices it builds,
token by token in pure-Python loops, the explicit rectified weight matrix W' of the video
queries (paper Sec. 4.1 / 4.2):

  * critical token j of query i in block n:   W'[i, j] = R_n * A^spa[i, j]
  * token j of a compensated non-critical block m:  W'[i, j] = A^pool[n, m] / c_m
    (the block weight spread uniformly over the block's keys, Sec. 4.2 remap equation)
  * every other token: 0

with A^pool from the token-expanded normaliser of the appendix (every key token j
contributes exp(s^pool_ij), where s^pool_ij uses the pooled key of j's block for video
tokens and the token itself for text tokens, Sec. 4.1), and O'_i = sum_j W'[i, j] v_j.
It imports nothing from the oracle and uses no numpy linear algebra.
"""
from __future__ import annotations

import math
from typing import List, Optional, Sequence


def _dot(a: Sequence[float], b: Sequence[float]) -> float:
    return math.fsum(x * y for x, y in zip(a, b))


def _mean_vec(rows: List[Sequence[float]]) -> List[float]:
    n = len(rows)
    return [math.fsum(r[c] for r in rows) / n for c in range(len(rows[0]))]


def brute_force_layer(Q, K, V, t_video: int, t_text: int, block: int, kept: int,
                      p: float = 0.0, gapr_mode: int = 1, scale: Optional[float] = None,
                      forced=None):
    """Q, K, V: nested lists / arrays [T, d] of Python floats. ``kept`` = blocks kept per
    video row before the p-extension. Returns dict(W=[T_v][T], O=[T][d], A_pool, mask, Mc, R)."""
    Q = [[float(x) for x in r] for r in Q]
    K = [[float(x) for x in r] for r in K]
    V = [[float(x) for x in r] for r in V]
    T, d = len(Q), len(Q[0])
    assert T == t_video + t_text
    scale = 1.0 / math.sqrt(d) if scale is None else scale

    # block membership of every token; text starts a block of its own
    blocks: List[List[int]] = []
    for s in range(0, t_video, block):
        blocks.append(list(range(s, min(s + block, t_video))))
    n_video = len(blocks)
    for s in range(t_video, T, block):
        blocks.append(list(range(s, min(s + block, T))))
    M = len(blocks)
    block_of = [0] * T
    for m, toks in enumerate(blocks):
        for j in toks:
            block_of[j] = m

    q_pool = [_mean_vec([Q[i] for i in blocks[n]]) for n in range(n_video)]
    k_pool = [_mean_vec([K[j] for j in blocks[m]]) for m in range(M)]
    v_pool = [_mean_vec([V[j] for j in blocks[m]]) for m in range(M)]

    A_pool = [[0.0] * M for _ in range(n_video)]
    mask = [[False] * M for _ in range(n_video)]
    Mc = [[False] * M for _ in range(n_video)]
    R = [0.0] * n_video
    for n in range(n_video):
        # implicit full attention, expanded to tokens
        s_tok = []
        for j in range(T):
            key = k_pool[block_of[j]] if j < t_video else K[j]
            s_tok.append(_dot(q_pool[n], key) * scale)
        top = max(s_tok)
        e_tok = [math.exp(s - top) for s in s_tok]
        total = math.fsum(e_tok)
        for m in range(M):
            A_pool[n][m] = math.fsum(e_tok[j] for j in blocks[m]) / total
        # top-k by repeated arg-max (lowest index wins ties), then extend until weight > p
        remaining = list(range(M))
        chosen: List[int] = []
        weight = 0.0
        while remaining and (len(chosen) < kept or (p > 0.0 and not weight > p)):
            best = remaining[0]
            for m in remaining[1:]:
                if A_pool[n][m] > A_pool[n][best]:
                    best = m
            remaining.remove(best)
            chosen.append(best)
            weight += A_pool[n][best]
        for m in chosen:
            mask[n][m] = True
        if forced is not None:
            for m in range(M):
                if forced[n][m]:
                    mask[n][m] = True
        R[n] = math.fsum(A_pool[n][m] for m in range(M) if mask[n][m])
        # gain / error gate, written as the double sums over (i, j)
        for m in range(M):
            if gapr_mode == 0:
                continue
            if gapr_mode == 2:
                Mc[n][m] = True
                continue
            s_nm = _dot(q_pool[n], k_pool[m]) * scale
            gain = 0.0
            err = 0.0
            for i in blocks[n]:
                a_i = _dot([Q[i][c] - q_pool[n][c] for c in range(d)], k_pool[m]) * scale
                for j in blocks[m]:
                    b_j = _dot(q_pool[n], [K[j][c] - k_pool[m][c] for c in range(d)]) * scale
                    gain += s_nm
                    err += abs(a_i) + abs(b_j)
            Mc[n][m] = abs(gain) > err

    W = [[0.0] * T for _ in range(t_video)]
    O = [[0.0] * d for _ in range(T)]
    for i in range(t_video):
        n = block_of[i]
        crit = [j for j in range(T) if mask[n][block_of[j]]]
        s = {j: _dot(Q[i], K[j]) * scale for j in crit}
        top = max(s.values())
        z = math.fsum(math.exp(v - top) for v in s.values())
        for j in crit:
            W[i][j] = R[n] * math.exp(s[j] - top) / z
        for m in range(M):
            if not mask[n][m] and Mc[n][m]:
                for j in blocks[m]:
                    W[i][j] = A_pool[n][m] / len(blocks[m])
        for c in range(d):
            O[i][c] = math.fsum(W[i][j] * V[j][c] for j in range(T))
    for i in range(t_video, T):
        s = [_dot(Q[i], K[j]) * scale for j in range(T)]
        top = max(s)
        e = [math.exp(v - top) for v in s]
        z = math.fsum(e)
        for c in range(d):
            O[i][c] = math.fsum(e[j] / z * V[j][c] for j in range(T))
    return dict(W=W, O=O, A_pool=A_pool, mask=mask, Mc=Mc, R=R, v_pool=v_pool)
