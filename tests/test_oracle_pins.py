"""Pins for the CPU oracle: what the paper and the mathematics fix, not the oracle itself.

Each test names the passage it pins. None of them needs a GPU.
"""
import math
import os

import numpy as np
import pytest
import scipy.special
import torch

from oracle import rsa_oracle as ro
from oracle.brute_force import brute_force_layer

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _read_golden(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(line.split())
    return rows


def _rand_qkv(rng, T, d, scale=1.0):
    return (rng.normal(size=(T, d)) * scale, rng.normal(size=(T, d)) * scale, rng.normal(size=(T, d)))


def _blockwise_constant(rng, part, d, amp=1.0):
    """[T, d] with all tokens of a block equal."""
    X = np.empty((part.t_video + part.t_text, d))
    for m in range(part.n_blocks):
        X[part.tokens(m)] = rng.normal(size=d) * amp
    return X


# ------------------------------------------------------------------ dense attention / rho = 0

def test_dense_attention_matches_library_routines():
    """Sec. 3.1 full attention = a library softmax-attention (torch SDPA in fp64, scipy softmax)."""
    rng = np.random.default_rng(1)
    Q, K, V = _rand_qkv(rng, 37, 16)
    scale = 1.0 / math.sqrt(16)
    got = ro.dense_attention(Q, K, V, scale)
    want = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(Q)[None], torch.from_numpy(K)[None], torch.from_numpy(V)[None]).numpy()[0]
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)
    want2 = scipy.special.softmax(Q @ K.T * scale, axis=1) @ V
    np.testing.assert_allclose(got, want2, rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("t_video,t_text,block", [(64, 0, 16), (50, 11, 16), (33, 16, 8)])
def test_sparsity_zero_is_dense_attention(t_video, t_text, block):
    """All blocks critical => R_n = 1, no compensation, output = full attention (Sec. 3.1, 4.1)."""
    rng = np.random.default_rng(2)
    Q, K, V = _rand_qkv(rng, t_video + t_text, 8)
    r = ro.rectified_layer_head(Q, K, V, t_video, t_text, block, sparsity=0.0)
    assert r["mask"].all()
    np.testing.assert_allclose(r["R"], 1.0, rtol=0, atol=1e-14)
    np.testing.assert_allclose(r["C"], 0.0, atol=0)
    want = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(Q)[None], torch.from_numpy(K)[None], torch.from_numpy(V)[None]).numpy()[0]
    np.testing.assert_allclose(r["O"], want, rtol=1e-11, atol=1e-12)


# ------------------------------------------------------------------ brute force on tiny inputs

@pytest.mark.parametrize("seed,t_video,t_text,block,kept,p,mode,use_forced", [
    (0, 16, 0, 4, 2, 0.0, 1, False),
    (1, 18, 6, 4, 2, 0.0, 1, False),       # ragged video block and ragged text block
    (2, 18, 6, 4, 3, 0.0, 2, False),
    (3, 18, 6, 4, 1, 0.0, 0, False),
    (4, 18, 5, 4, 2, 0.55, 1, False),      # weight-threshold extension
    (5, 14, 4, 4, 2, 0.0, 1, True),        # forced-keep (adjacency) mask
    (6, 12, 3, 3, 5, 0.0, 1, False),       # everything kept
])
def test_oracle_equals_token_level_brute_force(seed, t_video, t_text, block, kept, p, mode, use_forced):
    """Whole Alg. 1 against an independent token-level construction of W' (Sec. 4.1, 4.2)."""
    rng = np.random.default_rng(seed)
    d = 6
    T = t_video + t_text
    part = ro.partition(t_video, t_text, block)
    # smooth-ish video tokens so that the gate fires on some blocks and not on others
    base = _blockwise_constant(rng, part, d, amp=1.5)
    Q = base + rng.normal(size=(T, d)) * 0.15
    K = base + rng.normal(size=(T, d)) * 0.15
    Q[t_video:] = rng.normal(size=(t_text, d)) * 1.5
    K[t_video:] = rng.normal(size=(t_text, d)) * 1.5
    V = rng.normal(size=(T, d))
    M = part.n_blocks
    sparsity = (M - kept) / M
    assert ro.kept_count(M, sparsity) == kept
    forced = None
    if use_forced:
        forced = np.zeros((part.n_video, M), dtype=bool)
        forced[np.arange(part.n_video), np.arange(part.n_video)] = True   # keep the diagonal
    r = ro.rectified_layer_head(Q, K, V, t_video, t_text, block, sparsity, p=p, forced=forced, gapr_mode=mode)
    b = brute_force_layer(Q, K, V, t_video, t_text, block, kept, p=p, gapr_mode=mode, forced=forced)
    np.testing.assert_array_equal(r["mask"], np.asarray(b["mask"]))
    np.testing.assert_array_equal(r["Mc"], np.asarray(b["Mc"]))
    np.testing.assert_allclose(r["A_pool"], np.asarray(b["A_pool"]), rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(r["R"], np.asarray(b["R"]), rtol=1e-12)
    np.testing.assert_allclose(r["O"], np.asarray(b["O"]), rtol=1e-11, atol=1e-12)
    if mode == 1 and seed in (0, 1):
        # the gate must be non-trivial on these inputs or the pin proves little
        noncrit = ~r["mask"]
        assert 0 < (r["Mc"] & noncrit).sum() < noncrit.sum()
    # row-weight identity (Sec. 4.2 remap): total rectified weight = 1 - uncompensated mass
    W = np.asarray(b["W"])
    uncomp = (r["A_pool"] * (~r["mask"] & ~r["Mc"])).sum(axis=1)
    for n in range(part.n_video):
        np.testing.assert_allclose(W[part.tokens(n)].sum(axis=1), 1.0 - uncomp[n], rtol=1e-12)
    if mode == 2:
        np.testing.assert_allclose(W.sum(axis=1), 1.0, rtol=1e-12)


@pytest.mark.parametrize("rectify,compensate", [(False, False), (True, False), (False, True)])
def test_rectification_switches_against_token_level_weights(rectify, compensate):
    """Alg. 1 steps 20-22 taken apart: without step 20 the critical weights are the plain sparse softmax
    (the brute-force critical weights divided by R_n), without steps 21-22 the compensated weights are
    dropped. Built from the token-level weight matrix of the brute force, not from the oracle."""
    rng = np.random.default_rng(23)
    t_video, t_text, block, d, kept = 29, 5, 6, 4, 2
    T = t_video + t_text
    part = ro.partition(t_video, t_text, block)
    base = _blockwise_constant(rng, part, d, amp=1.5)
    Q = base + rng.normal(size=(T, d)) * 0.15
    K = base + rng.normal(size=(T, d)) * 0.15
    V = rng.normal(size=(T, d))
    M = part.n_blocks
    r = ro.rectified_layer_head(Q, K, V, t_video, t_text, block, (M - kept) / M, rectify=rectify, compensate=compensate)
    b = brute_force_layer(Q, K, V, t_video, t_text, block, kept)
    W, mask, R = np.asarray(b["W"]), np.asarray(b["mask"]), np.asarray(b["R"])
    assert (np.asarray(b["Mc"]) & ~mask).any(), "nothing is compensated: the case proves nothing"
    want = np.asarray(b["O"]).copy()
    for n in range(part.n_video):
        crit_tok = np.concatenate([np.arange(T)[part.tokens(m)] for m in range(M) if mask[n][m]])
        is_crit = np.zeros(T, dtype=bool)
        is_crit[crit_tok] = True
        Wn = W[part.tokens(n)]
        w_crit = np.where(is_crit, Wn, 0.0) / (1.0 if rectify else R[n])
        w_comp = np.where(is_crit, 0.0, Wn) if compensate else 0.0
        want[part.tokens(n)] = (w_crit + w_comp) @ V
    np.testing.assert_allclose(r["O"], want, rtol=1e-11, atol=1e-12)


# ------------------------------------------------------------------ the paper's worked numbers

def test_intro_worked_example_single_token_blocks():
    """Sec. 1: critical 0.8 -> 1.0, non-critical 0.2 -> 0.0; rectification restores 0.8 / 0.2."""
    g = {k: float(v) for k, v in _read_golden("intro_worked_example.txt")}
    d = 4
    # two one-token blocks whose full-attention weights are 0.8 and 0.2: score gap = ln 4
    q = np.array([1.0, 0.0, 0.0, 0.0])
    gap = math.log(g["full_weight_critical"] / g["full_weight_noncritical"]) * math.sqrt(d)
    K = np.array([[gap, 0.3, 0.0, 0.0], [0.0, -0.2, 0.5, 0.0]])
    K[:, 0] += 0.7                                        # non-zero pooled scores so the gain is non-zero
    Q = np.stack([q, q])
    V = np.array([[1.0, 2.0, 3.0, 4.0], [-1.0, 0.5, 0.0, 2.0]])
    full = scipy.special.softmax(Q @ K.T / math.sqrt(d), axis=1)
    np.testing.assert_allclose(full[0], [g["full_weight_critical"], g["full_weight_noncritical"]], rtol=1e-12)
    r = ro.rectified_layer_head(Q, K, V, 2, 0, 1, sparsity=0.5)
    assert r["mask"].tolist() == [[True, False], [True, False]]
    part = r["part"]
    o_spa = ro.sparse_attention(Q, K, V, r["mask"], part, r["scale"])
    np.testing.assert_allclose(o_spa[0], g["sparse_weight_critical"] * V[0] + g["sparse_weight_noncritical"] * V[1],
                               rtol=1e-13)
    np.testing.assert_allclose(r["R"], g["rectification_factor"], rtol=1e-12)
    assert r["Mc"][:, 1].all()
    np.testing.assert_allclose((r["A_pool"] * (~r["mask"] & r["Mc"])).sum(axis=1), g["compensated_weight"], rtol=1e-12)
    np.testing.assert_allclose(r["O"], full @ V, rtol=1e-12)
    b = brute_force_layer(Q, K, V, 2, 0, 1, kept=1)
    np.testing.assert_allclose(np.asarray(b["W"])[0], [g["full_weight_critical"], g["full_weight_noncritical"]], rtol=1e-12)


def test_intro_worked_example_blocks_of_identical_tokens():
    """Same numbers with real blocks: identical tokens per block make pooling exact."""
    g = {k: float(v) for k, v in _read_golden("intro_worked_example.txt")}
    d, B = 8, 4
    rng = np.random.default_rng(3)
    q = rng.normal(size=d)
    k2 = rng.normal(size=d)
    # choose k1 = k2 + t q with t such that the score gap is ln(0.8/0.2)
    t = math.log(g["full_weight_critical"] / g["full_weight_noncritical"]) * math.sqrt(d) / (q @ q)
    k1 = k2 + t * q
    Q = np.tile(q, (2 * B, 1))
    K = np.concatenate([np.tile(k1, (B, 1)), np.tile(k2, (B, 1))])
    V = rng.normal(size=(2 * B, d))
    r = ro.rectified_layer_head(Q, K, V, 2 * B, 0, B, sparsity=0.5)
    np.testing.assert_allclose(r["A_pool"], [[0.8, 0.2], [0.8, 0.2]], rtol=1e-12)
    np.testing.assert_allclose(r["R"], g["rectification_factor"], rtol=1e-12)
    # the token weights inside the critical block sum to 1.0 before and 0.8 after rectification
    o_spa = ro.sparse_attention(Q, K, V, r["mask"], r["part"], r["scale"])
    np.testing.assert_allclose(o_spa[0], V[:B].mean(axis=0), rtol=1e-12)
    # non-critical block recovered from pooled values with weight 0.2
    np.testing.assert_allclose(r["C"][0], g["compensated_weight"] * V[B:].mean(axis=0), rtol=1e-12)
    np.testing.assert_allclose(r["O"], ro.dense_attention(Q, K, V, r["scale"]), rtol=1e-12)


# ------------------------------------------------------------------ identical tokens per block => exact

@pytest.mark.parametrize("sparsity", [0.0, 0.3, 0.6, 0.85])
@pytest.mark.parametrize("t_video,t_text,block", [(40, 0, 8), (44, 12, 8)])
def test_identical_tokens_per_block_recover_dense_attention(t_video, t_text, block, sparsity):
    """Pooling is exact when every block's Q and K tokens coincide: A^pool equals the true
    block masses, the gate's error terms vanish, and the rectified output equals full
    attention at any sparsity (Sec. 3.2, 4.1, 4.2)."""
    rng = np.random.default_rng(4)
    d = 8
    part = ro.partition(t_video, t_text, block)
    Q, K = _blockwise_constant(rng, part, d), _blockwise_constant(rng, part, d)
    V = rng.normal(size=(t_video + t_text, d))       # V may vary: pooled V is the exact block average
    r = ro.rectified_layer_head(Q, K, V, t_video, t_text, block, sparsity)
    scale = r["scale"]
    A_full = scipy.special.softmax(Q @ K.T * scale, axis=1)
    masses = np.stack([A_full[part.starts[n], part.tokens(m)].sum() * np.ones(1)
                       for n in range(part.n_video) for m in range(part.n_blocks)]).reshape(part.n_video, -1)
    np.testing.assert_allclose(r["A_pool"], masses, rtol=1e-12)
    np.testing.assert_allclose(r["E"], 0.0, atol=1e-12)
    assert (r["Mc"] == (np.abs(r["S_pool"]) > 1e-12)).all()
    np.testing.assert_allclose(r["O"], A_full @ V, rtol=1e-10, atol=1e-12)


# ------------------------------------------------------------------ IPAR

def test_ipar_without_text_equal_blocks_is_plain_softmax():
    """No text and equal block sizes: reallocation cancels, A^pool = softmax(S^pool) (Sec. 3.2)."""
    rng = np.random.default_rng(5)
    Q, K, V = _rand_qkv(rng, 48, 8)
    r = ro.rectified_layer_head(Q, K, V, 48, 0, 8, 0.5)
    np.testing.assert_allclose(r["A_pool"], scipy.special.softmax(r["S_pool"], axis=1), rtol=1e-12)


def test_ipar_uniform_scores_give_token_count_shares():
    """Uniform pooled scores (all keys equal): every token weighs the same, so
    A^pool[n, m] = c_m / T and R_n = (tokens in critical blocks) / T (closed form)."""
    rng = np.random.default_rng(6)
    t_video, t_text, block, d = 29, 7, 8, 8
    T = t_video + t_text
    Q = rng.normal(size=(T, d))
    K = np.tile(rng.normal(size=d), (T, 1))
    V = rng.normal(size=(T, d))
    r = ro.rectified_layer_head(Q, K, V, t_video, t_text, block, 0.5)
    c = r["part"].counts
    np.testing.assert_allclose(r["A_pool"], np.tile(c / T, (r["part"].n_video, 1)), rtol=1e-12)
    np.testing.assert_allclose(r["R"], (r["mask"] * c[None, :]).sum(axis=1) / T, rtol=1e-12)
    # ties: the first k block indices are kept
    k = ro.kept_count(r["part"].n_blocks, 0.5)
    order = np.argsort(-(c / T), kind="stable")[:k]
    assert set(np.nonzero(r["mask"][0])[0]) == set(order)


def test_ipar_rows_sum_to_one_and_match_log_mass_form():
    """A^pool is a distribution over blocks (R4); it equals softmax of the block log-mass
    l[n,m] = s^pool + ln c_m (video) / logsumexp of the block's token scores (text)."""
    rng = np.random.default_rng(7)
    t_video, t_text, block, d = 45, 13, 8, 8
    Q, K, V = _rand_qkv(rng, t_video + t_text, d, scale=1.3)
    r = ro.rectified_layer_head(Q, K, V, t_video, t_text, block, 0.5)
    part, scale = r["part"], r["scale"]
    np.testing.assert_allclose(r["A_pool"].sum(axis=1), 1.0, rtol=1e-13)
    N = part.n_video
    lm = np.empty((N, part.n_blocks))
    lm[:, :N] = r["S_pool"][:, :N] + np.log(part.counts[:N])[None, :]
    u = r["Qp"][:N] @ K[t_video:].T * scale
    for i in range(part.n_text):
        lo = part.starts[N + i] - t_video
        lm[:, N + i] = scipy.special.logsumexp(u[:, lo:lo + part.counts[N + i]], axis=1)
    np.testing.assert_allclose(r["A_pool"], scipy.special.softmax(lm, axis=1), rtol=1e-12)


def test_ipar_differs_from_direct_pooling_of_text():
    """Isolation matters: pooling the text keys like video keys gives a different map (Sec. 4.1)."""
    rng = np.random.default_rng(8)
    t_video, t_text, block, d = 32, 16, 8, 8
    Q, K, V = _rand_qkv(rng, t_video + t_text, d, scale=1.5)
    r = ro.rectified_layer_head(Q, K, V, t_video, t_text, block, 0.5)
    direct = scipy.special.softmax(r["S_pool"] + np.log(r["part"].counts)[None, :], axis=1)
    assert np.abs(direct - r["A_pool"]).max() > 1e-3
    # Jensen: the isolated text mass is never below the directly pooled one, relative to video mass
    N = r["part"].n_video
    ratio_iso = r["A_pool"][:, N:].sum(axis=1) / r["A_pool"][:, :N].sum(axis=1)
    ratio_dir = direct[:, N:].sum(axis=1) / direct[:, :N].sum(axis=1)
    assert (ratio_iso >= ratio_dir - 1e-12).all()


# ------------------------------------------------------------------ selection

def test_kept_count_matches_hand_arithmetic():
    for M, rho, k in _read_golden("kept_blocks.txt"):
        assert ro.kept_count(int(M), float(rho)) == int(k)
    assert ro.kept_count(10, 1.0) == 1          # never fewer than one block
    assert ro.kept_count(10, 0.0) == 10


def test_select_matches_brute_force_sort_and_is_permutation_equivariant():
    rng = np.random.default_rng(9)
    N, M = 7, 23
    A = rng.random((N, M))
    A[2, 5] = A[2, 11] = A[2, 17]                # ties
    A /= A.sum(axis=1, keepdims=True)
    for rho in (0.0, 0.3, 0.9, (M - 1) / M):
        mask = ro.select_blocks(A, rho)
        k = ro.kept_count(M, rho)
        assert (mask.sum(axis=1) == k).all()
        for n in range(N):
            ranked = sorted(range(M), key=lambda m: (-A[n, m], m))[:k]
            assert set(np.nonzero(mask[n])[0]) == set(ranked)
    perm = rng.permutation(M)
    A2 = rng.random((N, M))                       # no ties
    np.testing.assert_array_equal(ro.select_blocks(A2[:, perm], 0.6), ro.select_blocks(A2, 0.6)[:, perm])


def test_select_weight_threshold_and_forced_mask():
    """Alg. 1 steps 13-14: extension until the kept weight exceeds p; OR with M_adja."""
    A = np.array([[0.05, 0.4, 0.1, 0.25, 0.2], [0.6, 0.1, 0.1, 0.1, 0.1]])
    m0 = ro.select_blocks(A, sparsity=0.8)                 # k = 1
    assert m0.tolist() == [[False, True, False, False, False], [True, False, False, False, False]]
    m1 = ro.select_blocks(A, sparsity=0.8, p=0.5)          # row 0 needs 0.4+0.25 > 0.5; row 1 already above
    assert m1.tolist() == [[False, True, False, True, False], [True, False, False, False, False]]
    m2 = ro.select_blocks(A, sparsity=0.8, p=0.65)         # 0.65 is not > 0.65 => take a third block
    assert m2[0].tolist() == [False, True, False, True, True]
    forced = np.zeros((2, 5), dtype=bool)
    forced[:, 4] = True
    m3 = ro.select_blocks(A, sparsity=0.8, forced=forced)
    assert m3.tolist() == [[False, True, False, False, True], [True, False, False, False, True]]
    m4 = ro.select_blocks(A, sparsity=0.8, p=2.0)          # unreachable threshold keeps everything
    assert m4.all()


# ------------------------------------------------------------------ rectification factor

def test_factor_with_true_block_masses_restores_full_attention_weights():
    """Sec. 4.1: R_n = A / A^spa = total full-attention weight of the critical tokens; with the
    true masses in place of A^pool, R * A^spa equals A on every critical token."""
    rng = np.random.default_rng(10)
    T, d, B = 40, 8, 8
    Q, K, V = _rand_qkv(rng, T, d)
    part = ro.partition(T, 0, B)
    scale = 1 / math.sqrt(d)
    A = scipy.special.softmax(Q @ K.T * scale, axis=1)
    mask = ro.select_blocks(rng.random((part.n_video, part.n_blocks)), 0.6)
    for n in range(part.n_video):
        cols = np.concatenate([np.arange(part.starts[m], part.starts[m] + part.counts[m]) for m in np.nonzero(mask[n])[0]])
        for i in range(part.starts[n], part.starts[n] + part.counts[n]):
            a_spa = scipy.special.softmax(Q[i] @ K[cols].T * scale)
            masses_i = np.array([A[i, part.tokens(m)].sum() for m in range(part.n_blocks)])
            R_i = ro.rectification_factor(masses_i[None, :], mask[n][None, :])[0]
            np.testing.assert_allclose(R_i * a_spa, A[i, cols], rtol=1e-12)


# ------------------------------------------------------------------ GAPR gate

def _gate_inputs(seed, eps):
    rng = np.random.default_rng(seed)
    t_video, t_text, block, d = 24, 8, 8, 8
    part = ro.partition(t_video, t_text, block)
    base_q, base_k = _blockwise_constant(rng, part, d), _blockwise_constant(rng, part, d)
    dev_q, dev_k = rng.normal(size=base_q.shape), rng.normal(size=base_k.shape)
    for m in range(part.n_blocks):                    # zero-mean deviations keep the block means fixed
        dev_q[part.tokens(m)] -= dev_q[part.tokens(m)].mean(axis=0)
        dev_k[part.tokens(m)] -= dev_k[part.tokens(m)].mean(axis=0)
    return part, base_q + eps * dev_q, base_k + eps * dev_k


def test_gate_error_vanishes_iff_blocks_are_homogeneous_and_scales_linearly():
    part, Q0, K0 = _gate_inputs(11, 0.0)
    scale = 0.35
    _, G0, E0 = ro.gapr(Q0, K0, ro.pool(Q0, part), ro.pool(K0, part), part, scale)
    np.testing.assert_allclose(E0, 0.0, atol=1e-12)
    _, G1, E1 = ro.gapr(*(lambda p, q, k: (q, k, ro.pool(q, p), ro.pool(k, p), p, scale))(*_gate_inputs(11, 0.1)))
    _, G2, E2 = ro.gapr(*(lambda p, q, k: (q, k, ro.pool(q, p), ro.pool(k, p), p, scale))(*_gate_inputs(11, 0.3)))
    assert (E1 > 0).all()
    np.testing.assert_allclose(E2, 3.0 * E1, rtol=1e-9)      # first-order terms are linear in the deviation
    np.testing.assert_allclose(G1, G0, rtol=1e-9)            # the gain only sees block means
    np.testing.assert_allclose(G2, G0, rtol=1e-9)
    c = part.counts.astype(float)
    S = ro.pool(Q0, part)[:part.n_video] @ ro.pool(K0, part).T * scale
    np.testing.assert_allclose(G0, np.abs(S) * c[:part.n_video, None] * c[None, :], rtol=1e-12)


def test_gate_error_bounds_exact_first_order_l1_and_printed_signed_sum_vanishes():
    """R7: E >= sum_ij |a_i + b_j| (triangle inequality), and the signed double sum of the
    first-order Delta s, which the relaxed condition prints, is identically zero."""
    part, Q, K = _gate_inputs(12, 0.4)
    scale = 0.35
    Qp, Kp = ro.pool(Q, part), ro.pool(K, part)
    _, G, E = ro.gapr(Q, K, Qp, Kp, part, scale)
    np.testing.assert_allclose(ro.gapr_signed_sums(Q, K, Qp, Kp, part, scale), 0.0, atol=1e-10)
    for n in range(part.n_video):
        for m in range(part.n_blocks):
            a = (Q[part.tokens(n)] - Qp[n]) @ Kp[m] * scale
            b = (K[part.tokens(m)] - Kp[m]) @ Qp[n] * scale
            exact = np.abs(a[:, None] + b[None, :]).sum()
            assert exact <= E[n, m] * (1 + 1e-12)
            np.testing.assert_allclose(E[n, m], len(b) * np.abs(a).sum() + len(a) * np.abs(b).sum(), rtol=1e-12)


def test_gate_modes():
    part, Q, K = _gate_inputs(13, 0.5)
    Qp, Kp = ro.pool(Q, part), ro.pool(K, part)
    Mc1, G, E = ro.gapr(Q, K, Qp, Kp, part, 0.35, mode=1)
    assert (Mc1 == (G > E)).all() and 0 < Mc1.sum() < Mc1.size
    assert not ro.gapr(Q, K, Qp, Kp, part, 0.35, mode=0)[0].any()
    assert ro.gapr(Q, K, Qp, Kp, part, 0.35, mode=2)[0].all()


# ------------------------------------------------------------------ invariances of the sparse path

def test_key_shift_and_in_block_permutation_invariance():
    """softmax shift: adding one vector to every key changes no attention weight, hence not
    A^pool, the mask, R or the sparse output. Permuting the tokens inside key blocks
    (K and V together) changes nothing at all."""
    rng = np.random.default_rng(14)
    t_video, t_text, block, d = 40, 8, 8, 8
    T = t_video + t_text
    Q, K, V = _rand_qkv(rng, T, d)
    r0 = ro.rectified_layer_head(Q, K, V, t_video, t_text, block, 0.6, gapr_mode=2)
    r1 = ro.rectified_layer_head(Q, K + rng.normal(size=d)[None, :], V, t_video, t_text, block, 0.6, gapr_mode=2)
    np.testing.assert_allclose(r1["A_pool"], r0["A_pool"], rtol=1e-10)
    np.testing.assert_array_equal(r1["mask"], r0["mask"])
    np.testing.assert_allclose(r1["O"], r0["O"], rtol=1e-9, atol=1e-12)
    perm = np.arange(T)
    for m in range(r0["part"].n_blocks):
        s = r0["part"].tokens(m)
        perm[s] = rng.permutation(perm[s])
    r2 = ro.rectified_layer_head(Q, K[perm], V[perm], t_video, t_text, block, 0.6, gapr_mode=1)
    r3 = ro.rectified_layer_head(Q, K, V, t_video, t_text, block, 0.6, gapr_mode=1)
    np.testing.assert_array_equal(r2["mask"], r3["mask"])
    np.testing.assert_array_equal(r2["Mc"], r3["Mc"])
    np.testing.assert_allclose(r2["O"], r3["O"], rtol=1e-10, atol=1e-12)


def test_uniform_scores_and_homogeneous_blocks_make_total_weight_one():
    """With uniform pooled scores and identical tokens per block every non-critical block is
    compensated (zero error, non-zero gain), so the rectified weights sum to exactly 1 and
    the output equals full attention."""
    rng = np.random.default_rng(15)
    t_video, block, d = 48, 8, 8
    part = ro.partition(t_video, 0, block)
    Q = _blockwise_constant(rng, part, d)
    K = np.tile(rng.normal(size=d), (t_video, 1))
    V = rng.normal(size=(t_video, d))
    r = ro.rectified_layer_head(Q, K, V, t_video, 0, block, 0.75)
    comp = (r["A_pool"] * (~r["mask"] & r["Mc"])).sum(axis=1)
    np.testing.assert_allclose(r["R"] + comp, 1.0, rtol=1e-13)
    np.testing.assert_allclose(r["O"], ro.dense_attention(Q, K, V, r["scale"]), rtol=1e-11)


def test_bf16_widening_is_exact():
    bits = np.array([0x3F80, 0xBF80, 0x4049, 0x0000, 0x8000, 0x3DCD], dtype=np.uint16)
    want = [1.0, -1.0, 3.140625, 0.0, -0.0, 0.10009765625]
    np.testing.assert_array_equal(ro.bf16_bits_to_f64(bits), want)
