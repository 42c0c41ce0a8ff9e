"""GPU parity: the HIP path behind the C-ABI against the CPU oracle, element by element,
on the same seeded inputs. Needs an MI355X: run with ``-m gpu``."""
import os

import numpy as np
import pytest

from paper_2511_19835_amd import synth
from paper_2511_19835_amd.synth import LayerConfig

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible: these tests must run on the MI355X box")
    from paper_2511_19835_amd import binding, harness
    binding.load_library()          # fails loudly if librsa.so is missing
    return harness


def _run_and_compare(harness, cfg, seed=0, heads=None, layout="bhtd", **kw):
    import parity
    Qb, Kb, Vb = synth.make_inputs(cfg, seed, heads)
    sparsity = kw.pop("sparsity", cfg.sparsity)
    p = kw.get("p", 0.0)
    gapr_mode = kw.get("gapr_mode", 1)
    forced = kw.get("forced", None)
    flags = kw.get("flags", 3)
    scale = kw.get("scale", None)                      # None: the default 1/sqrt(d) on both sides
    out = harness.run_layer(Qb, Kb, Vb, cfg.t_video, cfg.t_text, cfg.block, sparsity, p=p, gapr_mode=gapr_mode,
                            forced=forced, flags=flags, layout=layout, scale=0.0 if scale is None else scale,
                            attn_workspace=kw.get("attn_workspace", True))
    stats = []
    for b in range(Qb.shape[0]):
        for h in range(Qb.shape[1]):
            ref = parity.oracle_head(Qb[b, h], Kb[b, h], Vb[b, h], cfg.t_video, cfg.t_text, cfg.block, sparsity,
                                     p=p, gapr_mode=gapr_mode,
                                     forced=None if forced is None else forced[b, h], scale=scale,
                                     rectify=bool(flags & 1), compensate=bool(flags & 2))
            st = parity.compare_head(out, b, h, ref, Qb[b, h], Kb[b, h], Vb[b, h], p=p,
                                     forced=None if forced is None else forced[b, h],
                                     rectify=bool(flags & 1), compensate=bool(flags & 2))
            stats.append(st)
            print(f"  [{cfg.name} b{b} h{h}] {st}", flush=True)
    return out, stats, (Qb, Kb, Vb)


def test_tiny_config_full_parity(gpu):
    """The small benchmark configuration: 2 heads, d 64, 1024 video + 64 text tokens, block 64, 75 % sparsity."""
    import parity
    from oracle import rsa_oracle as ro
    cfg = synth.CONFIGS["tiny"]
    out, stats, (Qb, Kb, Vb) = _run_and_compare(gpu, cfg)
    assert (out["count"][:, :, :] == 5).all()
    # log-sum-exp of the un-rectified sparse / dense rows
    for h in range(cfg.heads):
        Q, K = ro.bf16_bits_to_f64(Qb[0, h]), ro.bf16_bits_to_f64(Kb[0, h])
        part = ro.partition(cfg.t_video, cfg.t_text, cfg.block)
        scale = 1 / np.sqrt(cfg.head_dim)
        for n in (0, 7, part.n_video):            # two video blocks and the text block
            rows = part.tokens(n)
            if n < part.n_video:
                cols = np.concatenate([np.arange(part.starts[m], part.starts[m] + part.counts[m])
                                       for m in np.nonzero(out["mask"][0, h, n])[0]])
            else:
                cols = np.arange(cfg.t_total)
            S = Q[rows] @ K[cols].T * scale
            want = np.log(np.exp(S - S.max(axis=1, keepdims=True)).sum(axis=1)) + S.max(axis=1)
            np.testing.assert_allclose(out["lse"][0, h, rows], want, atol=2e-3)


def test_mid_config_two_heads_parity(gpu):
    """The mid-size benchmark shape (20 280 video tokens, ragged last block, block 128, d 128, 90 %)."""
    cfg = synth.CONFIGS["mid"]
    out, stats, _ = _run_and_compare(gpu, cfg, heads=[0, 7])
    assert (out["count"] == 16).all()


def _random_config(rng, i):
    d = int(rng.choice([64, 128]))
    block = int(rng.choice([64, 128]))
    grid = (int(rng.integers(1, 6)), int(rng.integers(3, 14)), int(rng.integers(3, 18)))
    t_text = int(rng.choice([0, 0, 1, 17, 64, 130, 257]))
    heads = int(rng.integers(1, 4))
    sparsity = float(rng.choice([0.3, 0.5, 0.7, 0.9]))
    return LayerConfig(f"random{i}", 1, heads, d, grid, t_text, block, sparsity)


@pytest.mark.parametrize("case", range(int(os.environ.get("RSA_RANDOM_CASES", "16"))))
def test_random_shapes(gpu, case):
    """Seeded random shapes over both head dimensions and block sizes, ragged grids, odd text
    lengths, with the weight threshold and the rectification flags drawn at random too."""
    rng = np.random.default_rng(1000 + case)
    cfg = _random_config(rng, case)
    p = float(rng.choice([0.0, 0.0, 0.2, 0.4]))
    flags = int(rng.choice([3, 3, 1, 2, 0]))
    gapr_mode = int(rng.choice([1, 1, 0, 2]))
    print(f"  {cfg} p={p} flags={flags} gapr_mode={gapr_mode}", flush=True)
    if p > 0.0:
        # the extension decides on cumulative fp32 sums: compare outputs on the GPU's own masks
        import parity
        Qb, Kb, Vb = synth.make_inputs(cfg, 2000 + case)
        out = gpu.run_layer(Qb, Kb, Vb, cfg.t_video, cfg.t_text, cfg.block, cfg.sparsity, p=p, gapr_mode=gapr_mode, flags=flags)
        for h in range(cfg.heads):
            ref = parity.oracle_head(Qb[0, h], Kb[0, h], Vb[0, h], cfg.t_video, cfg.t_text, cfg.block, cfg.sparsity,
                                     p=p, gapr_mode=gapr_mode, rectify=bool(flags & 1), compensate=bool(flags & 2))
            A = ref["A_pool"]
            from oracle import rsa_oracle as ro
            _check_masks_under_weight_threshold(out["mask"][0, h], ref, p, ro.kept_count(cfg.n_blocks, cfg.sparsity),
                                                min_clear=0.5)
            gm = out["mask"][0, h].copy()
            O = _oracle_output_with_mask(ref, gm, Qb[0, h], Kb[0, h], Vb[0, h], rectify=bool(flags & 1),
                                         compensate=bool(flags & 2))
            parity.compare_head(out, 0, h, dict(ref, mask=gm, R=(A * gm).sum(axis=1), O=O), Qb[0, h], Kb[0, h], Vb[0, h],
                                p=p, rectify=bool(flags & 1), compensate=bool(flags & 2))
    else:
        _run_and_compare(gpu, cfg, seed=2000 + case, p=p, flags=flags, gapr_mode=gapr_mode)


def _check_masks_under_weight_threshold(gmask, ref, p, k, min_clear=0.0):
    """Rows whose cumulative sorted weight passes p by a clear margin (1e-5) must match the oracle bit
    for bit. For the others the fp32 sums of the kernel may cross p one block earlier or later than
    the fp64 sums: the mask must then be one of the two prefixes (of the oracle's own descending
    order) that end at the near-crossing or one block after it, never shorter than the top-k part."""
    A = ref["A_pool"]
    order = np.lexsort((np.arange(A.shape[1])[None, :].repeat(A.shape[0], 0), -A), axis=1)
    cs = np.cumsum(np.take_along_axis(A, order, axis=1), axis=1)
    near = np.abs(cs - p).argmin(axis=1)
    clear = np.abs(cs - p).min(axis=1) > 1e-5
    assert clear.mean() >= min_clear, f"only {clear.mean():.2f} of the rows are clear of the threshold"
    np.testing.assert_array_equal(gmask[clear], ref["mask"][clear])
    for n in np.nonzero(~clear)[0]:
        ok = False
        for length in (near[n] + 1, near[n] + 2):
            want = np.zeros(A.shape[1], dtype=bool)
            want[order[n, :max(k, min(length, A.shape[1]))]] = True
            ok |= np.array_equal(gmask[n], want)
        assert ok, f"row {n}: the mask is neither of the two prefixes around the crossing of p"
    return clear


def test_peaky_inputs_parity(gpu):
    """The same shape with the sinusoid amplitude doubled (pooled-score std about 4 instead of 1):
    scores span a wider range, the softmax is peakier and the lazy rescale fires more often."""
    cfg = synth.CONFIGS["mid"].with_(sigma_a=1.0)
    _run_and_compare(gpu, cfg, seed=5, heads=[3])
    _run_and_compare(gpu, cfg.with_(t_text=200), seed=6, heads=[1], sparsity=0.8)


EDGE = {
    "ragged_d64_b128": LayerConfig("ragged_d64_b128", 1, 2, 64, (5, 9, 13), 77, 128, 0.6),
    "d128_b64_text": LayerConfig("d128_b64_text", 1, 2, 128, (4, 12, 10), 100, 64, 0.7),
    "single_block": LayerConfig("single_block", 1, 1, 64, (1, 5, 7), 0, 64, 0.5),
    "video_lt_block_text": LayerConfig("video_lt_block_text", 1, 1, 128, (1, 6, 9), 30, 128, 0.5),
    "batch2": LayerConfig("batch2", 2, 3, 128, (3, 12, 16), 40, 128, 0.5),
    "text_many_blocks": LayerConfig("text_many_blocks", 1, 1, 64, (2, 8, 8), 300, 64, 0.5),
}


@pytest.mark.parametrize("name", sorted(EDGE))
def test_edge_shapes(gpu, name):
    _run_and_compare(gpu, EDGE[name], seed=3)


def test_strided_token_major_layout(gpu):
    """Q/K/V/O stored [batch, tokens, heads, d] (strides differ from the contiguous case)."""
    _run_and_compare(gpu, EDGE["batch2"], seed=4, layout="bthd")


@pytest.mark.parametrize("sparsity", [0.0, 0.5, 0.95, 1.0])
def test_sparsity_range(gpu, sparsity):
    """rho = 0 must reproduce full attention (R = 1, nothing compensated); rho = 1 keeps one block."""
    import parity
    cfg = EDGE["d128_b64_text"]
    out, stats, (Qb, Kb, Vb) = _run_and_compare(gpu, cfg, seed=5, sparsity=sparsity)
    if sparsity == 0.0:
        from oracle import rsa_oracle as ro
        assert out["mask"].all()
        np.testing.assert_allclose(out["R"], 1.0, atol=1e-5)
        for h in range(cfg.heads):
            Q, K, V = (ro.bf16_bits_to_f64(x[0, h]) for x in (Qb, Kb, Vb))
            dense = ro.dense_attention(Q, K, V, 1 / np.sqrt(cfg.head_dim))
            err = ro.bf16_bits_to_f64(out["O_bits"][0, h]) - dense
            assert np.abs(err).max() <= parity.OUT_MAX_ABS
            assert np.linalg.norm(err) / np.linalg.norm(dense) <= parity.OUT_REL_L2
    if sparsity == 1.0:
        assert (out["count"] == 1).all()


@pytest.mark.parametrize("gapr_mode", [0, 2])
def test_gate_modes(gpu, gapr_mode):
    out, _, _ = _run_and_compare(gpu, EDGE["ragged_d64_b128"], seed=6, gapr_mode=gapr_mode)
    assert out["Mc"].all() if gapr_mode == 2 else not out["Mc"].any()


@pytest.mark.parametrize("flags", [0, 1, 2])
def test_rectification_flags(gpu, flags):
    _run_and_compare(gpu, EDGE["ragged_d64_b128"], seed=7, flags=flags)


def test_non_default_softmax_scale(gpu):
    """rsa_shape.scale other than 1/sqrt(d): the pooled scores, the text log-mass, the gate and the
    attention kernel each apply it on their own."""
    _run_and_compare(gpu, EDGE["d128_b64_text"], seed=13, scale=0.05)
    _run_and_compare(gpu, EDGE["ragged_d64_b128"], seed=14, scale=0.2, sparsity=0.8)


def test_scores_far_from_the_softmax_reference(gpu):
    """Alg. 1 steps 16-17 with scores that leave any fixed window: the lists come from a selection at the
    default scale, the attention runs with a scale 40 times larger, so that the scaled scores of a row lie
    hundreds of binades apart. Queries are made non-negative and the keys of block 0 (kept by every row: a
    forced bit) non-positive, so that every score of the first block a row meets is far below 0, and later
    blocks hold scores far above them. Whatever reference the kernel keeps for its running softmax has to
    move off 0 at once and up later, and the output and the log-sum-exp must still be those of the exact
    softmax over the kept keys."""
    import torch
    import parity
    from oracle import rsa_oracle as ro
    from paper_2511_19835_amd import binding as rb
    for name, seed in (("d128_b64_text", 21), ("ragged_d64_b128", 22)):
        cfg = EDGE[name]
        Qb, Kb, Vb = synth.make_inputs(cfg, seed, [0])
        Qb = Qb & np.uint16(0x7fff)
        Kb = Kb.copy()
        Kb[0, 0, :cfg.block] |= np.uint16(0x8000)
        Q, K, V = (gpu.bits_to_device(x) for x in (Qb, Kb, Vb))
        buf = rb.allocate(Q, cfg.t_video, cfg.t_text, cfg.block)
        rb.rsa_pool(buf.shape, Q, K, V, buf.Qp, buf.Kp, buf.Vp, buf.Vt, buf.Spool, buf.Apool, buf.Lmass, buf.Mc_bits,
                    0, buf.pool_ws)
        forced = torch.zeros_like(buf.mask_bits)
        forced[..., 0] = 1
        rb.rsa_select_blocks(buf.shape, buf.Lmass, buf.Apool, 0.6, 0.0, forced, buf.mask_bits, buf.block_idx,
                             buf.count, buf.R)
        scale = 40.0 / np.sqrt(cfg.head_dim)
        big = rb.make_shape(Q, cfg.t_video, cfg.t_text, cfg.block, scale)
        O = torch.full_like(Q, float("nan"))
        lse = torch.full((1, 1, cfg.t_total), float("nan"), dtype=torch.float32, device=Q.device)
        rb.rsa_sparse_attn_rectified(big, Q, K, buf.Vt, buf.block_idx, buf.count, buf.mask_bits, buf.R, buf.Apool,
                                     buf.Mc_bits, buf.Vp, 0, O, lse, buf.attn_ws)
        torch.cuda.synchronize()
        part = ro.partition(cfg.t_video, cfg.t_text, cfg.block)
        mask = gpu.unpack_bits(buf.mask_bits[0, 0].cpu().numpy(), part.n_blocks)
        assert mask[:, 0].all()
        Qf, Kf, Vf = (ro.bf16_bits_to_f64(x[0, 0]) for x in (Qb, Kb, Vb))
        # the spread this test is about, in binades: block 0 against the best kept key of a row
        X = (Qf @ Kf.T) * scale * np.log2(np.e)
        assert X[:, :cfg.block].max() < -45.0
        kept_cols = np.repeat(mask, part.counts, axis=1)                      # [N, T]: kept keys of a query block
        block_of_token = np.repeat(np.arange(part.n_video), part.counts[:part.n_video])
        best = np.where(kept_cols[block_of_token], X[:cfg.t_video], -np.inf).max(axis=1)
        assert np.median(best - X[:cfg.t_video, :cfg.block].max(axis=1)) > 45.0
        O_ref = np.empty_like(Qf)
        O_ref[:cfg.t_video] = ro.sparse_attention(Qf, Kf, Vf, mask, part, scale)
        if cfg.t_text:
            O_ref[cfg.t_video:] = ro.dense_attention(Qf[cfg.t_video:], Kf, Vf, scale)
        O_gpu = ro.bf16_bits_to_f64(gpu.device_to_bits(O[0, 0]))
        assert np.isfinite(O_gpu).all()
        err = O_gpu - O_ref
        assert np.abs(err).max() <= parity.OUT_MAX_ABS
        assert np.linalg.norm(err) / np.linalg.norm(O_ref) <= parity.OUT_REL_L2
        for n in (0, part.n_video // 2, part.n_video - 1):
            rows = part.tokens(n)
            cols = np.nonzero(kept_cols[n])[0]
            S = Qf[rows] @ Kf[cols].T * scale
            want = np.log(np.exp(S - S.max(axis=1, keepdims=True)).sum(axis=1)) + S.max(axis=1)
            np.testing.assert_allclose(lse[0, 0, rows].cpu().numpy(), want, rtol=2e-5, atol=2e-3)


def test_attention_without_a_workspace(gpu):
    """ws = NULL is legal without RSA_COMPENSATE: the rows are then launched in index order."""
    _run_and_compare(gpu, EDGE["d128_b64_text"], seed=15, flags=1, attn_workspace=False)
    _run_and_compare(gpu, EDGE["batch2"], seed=16, flags=0, attn_workspace=False)


def _blockwise_constant_bits(rng, cfg, amp):
    """bf16 bit patterns [1, 1, T, d] with all tokens of a block equal (the block partition of the layer)."""
    from oracle import rsa_oracle as ro
    part = ro.partition(cfg.t_video, cfg.t_text, cfg.block)
    X = np.empty((cfg.t_total, cfg.head_dim), dtype=np.float32)
    for m in range(part.n_blocks):
        X[part.tokens(m)] = rng.normal(size=cfg.head_dim) * amp
    return synth.f32_to_bf16_bits(X).reshape(1, 1, cfg.t_total, cfg.head_dim).copy()


@pytest.mark.parametrize("sparsity", [0.5, 0.9])
@pytest.mark.parametrize("name", ["ragged_d64_b128", "d128_b64_text"])
def test_identical_tokens_per_block_recover_dense_attention(gpu, name, sparsity):
    """Sec. 3.2 (intra-block homogeneity): when all tokens of a block are equal the pooled scores are
    the token scores, A^pool holds the true block masses, the pooling error vanishes, and the rectified
    output equals full attention at any sparsity."""
    import parity
    from oracle import rsa_oracle as ro
    cfg = EDGE[name]
    rng = np.random.default_rng(31)
    Qb, Kb, Vb = (_blockwise_constant_bits(rng, cfg, a) for a in (1.0, 1.0, 1.0))
    out = gpu.run_layer(Qb, Kb, Vb, cfg.t_video, cfg.t_text, cfg.block, sparsity)
    Q, K, V = (ro.bf16_bits_to_f64(x[0, 0]) for x in (Qb, Kb, Vb))
    scale = 1.0 / np.sqrt(cfg.head_dim)
    part = ro.partition(cfg.t_video, cfg.t_text, cfg.block)
    N, M = part.n_video, part.n_blocks
    dense = ro.dense_attention(Q, K, V, scale)
    # true block masses of full attention (any token of the query block: they are all equal)
    first = part.starts[:N]
    W = np.exp(Q[first] @ K.T * scale)
    W /= W.sum(axis=1, keepdims=True)
    mass = np.stack([W[:, part.tokens(m)].sum(axis=1) for m in range(M)], axis=1)
    np.testing.assert_allclose(out["Apool"][0, 0], mass, rtol=3e-4, atol=1e-9)
    S = out["Spool"][0, 0]
    assert out["Mc"][0, 0][np.abs(S) > 1e-3].all(), "zero pooling error: the gate must be on wherever the gain is not 0"
    k = ro.kept_count(M, sparsity)
    assert (out["count"] == k).all() and k < M
    err = ro.bf16_bits_to_f64(out["O_bits"][0, 0]) - dense
    assert np.abs(err).max() <= parity.OUT_MAX_ABS
    assert np.linalg.norm(err) / np.linalg.norm(dense) <= parity.OUT_REL_L2
    # and the oracle says the same of these inputs
    ref = parity.oracle_head(Qb[0, 0], Kb[0, 0], Vb[0, 0], cfg.t_video, cfg.t_text, cfg.block, sparsity)
    np.testing.assert_allclose(ref["O"], dense, rtol=1e-9, atol=1e-12)


@pytest.mark.parametrize("p", [0.0, 0.5])
@pytest.mark.parametrize("name", ["ragged_d64_b128", "d128_b64_text"])
def test_uniform_pooled_scores_and_ties(gpu, name, p):
    """Sec. 4.1: with every key equal all scores of a row are equal, so A^pool[n, m] = c_m / T exactly,
    and every full video block ties. Ties go to the lower block index (the first k are kept), with and
    without the weight threshold; masks are compared bit for bit, without the threshold band."""
    import parity
    from oracle import rsa_oracle as ro
    cfg = EDGE[name].with_(heads=1)
    if cfg.t_text >= cfg.block:
        cfg = cfg.with_(t_text=cfg.block - 14)       # no text block as large as a full video block: it would tie too
    rng = np.random.default_rng(41)
    Qb, _, Vb = synth.make_inputs(cfg, 17)
    kvec = synth.f32_to_bf16_bits((rng.normal(size=cfg.head_dim) * 0.7).astype(np.float32))
    Kb = np.broadcast_to(kvec, Qb.shape).copy()
    sparsity = 0.8
    out = gpu.run_layer(Qb, Kb, Vb, cfg.t_video, cfg.t_text, cfg.block, sparsity, p=p)
    part = ro.partition(cfg.t_video, cfg.t_text, cfg.block)
    N, M = part.n_video, part.n_blocks
    np.testing.assert_allclose(out["Apool"][0, 0], np.broadcast_to(part.counts / cfg.t_total, (N, M)), rtol=2e-5)
    ref = parity.oracle_head(Qb[0, 0], Kb[0, 0], Vb[0, 0], cfg.t_video, cfg.t_text, cfg.block, sparsity, p=p)
    k = ro.kept_count(M, sparsity)
    full = np.nonzero(part.counts == cfg.block)[0]
    kept_len = k if p == 0.0 else max(k, int(np.floor(p * cfg.t_total / cfg.block)) + 1)
    assert kept_len < full.size and (p == 0.0 or kept_len > k), "the case must end inside the run of tied blocks"
    want = np.zeros((N, M), dtype=bool)
    want[:, full[:kept_len]] = True                  # the tied full blocks carry the largest mass; first ones win
    np.testing.assert_array_equal(ref["mask"], want)
    np.testing.assert_array_equal(out["mask"][0, 0], want)
    np.testing.assert_allclose(out["R"][0, 0], kept_len * cfg.block / cfg.t_total, rtol=2e-5)
    parity.compare_head(out, 0, 0, ref, Qb[0, 0], Kb[0, 0], Vb[0, 0], p=p)


def test_forced_keep_mask(gpu):
    """Caller-supplied adjacency mask M_adja is OR-ed into the sparse mask (Alg. 1 step 14)."""
    cfg = EDGE["d128_b64_text"]
    N, M = cfg.n_video_blocks, cfg.n_blocks
    forced = np.zeros((cfg.batch, cfg.heads, N, M), dtype=bool)
    idx = np.arange(N)
    forced[:, :, idx, idx] = True
    forced[:, :, idx, np.maximum(idx - 1, 0)] = True
    out, _, _ = _run_and_compare(gpu, cfg, seed=8, forced=forced)
    assert (out["mask"] & forced == forced).all()
    assert (out["count"] >= 3).all()


@pytest.mark.parametrize("name", ["d128_b64_text", "ragged_d64_b128", "batch2"])
def test_rows_of_very_different_length(gpu, name):
    """Every third video row is forced to keep all key blocks, its neighbours stay at the top-k
    minimum: query blocks that share a workgroup then walk lists of very different length."""
    cfg = EDGE[name]
    N, M = cfg.n_video_blocks, cfg.n_blocks
    forced = np.zeros((cfg.batch, cfg.heads, N, M), dtype=bool)
    forced[:, :, 0::3, :] = True
    out, _, _ = _run_and_compare(gpu, cfg, seed=12, sparsity=0.9, forced=forced)
    assert (out["count"][:, :, 0::3] == M).all()
    if N > 1:
        assert out["count"][:, :, 1::3].max() < M


def test_weight_threshold_extension(gpu):
    """p > 0 extends the kept prefix until the kept A^pool exceeds p (Alg. 1 step 13)."""
    import parity
    from oracle import rsa_oracle as ro
    cfg = EDGE["d128_b64_text"]
    p = 0.45
    Qb, Kb, Vb = synth.make_inputs(cfg, 9)
    out = gpu.run_layer(Qb, Kb, Vb, cfg.t_video, cfg.t_text, cfg.block, 0.9, p=p)
    k = ro.kept_count(cfg.n_blocks, 0.9)
    extended = 0
    for h in range(cfg.heads):
        ref = parity.oracle_head(Qb[0, h], Kb[0, h], Vb[0, h], cfg.t_video, cfg.t_text, cfg.block, 0.9, p=p)
        # rows whose cumulative weight passes p by a clear margin must match exactly
        A = ref["A_pool"]
        _check_masks_under_weight_threshold(out["mask"][0, h], ref, p, k, min_clear=0.9)
        extended += int((ref["mask"].sum(axis=1) > k).sum())
        # outputs: compare on the GPU's own masks
        parity.compare_head(out, 0, h, dict(ref, mask=out["mask"][0, h].copy(),
                                            R=(A * out["mask"][0, h]).sum(axis=1),
                                            O=_oracle_output_with_mask(ref, out["mask"][0, h], Qb[0, h], Kb[0, h], Vb[0, h])),
                            Qb[0, h], Kb[0, h], Vb[0, h], p=p)
    assert extended > 0, "the threshold never extended a row: the case proves nothing"


def _oracle_output_with_mask(ref, mask, Qb, Kb, Vb, rectify=True, compensate=True):
    from oracle import rsa_oracle as ro
    Q, K, V = (ro.bf16_bits_to_f64(x) for x in (Qb, Kb, Vb))
    part = ref["part"]
    O = ref["O"].copy()
    R = (ref["A_pool"] * mask).sum(axis=1) if rectify else np.ones(part.n_video)
    C = ro.compensation(ref["A_pool"], mask, ref["Mc"], ref["Vp"])
    for n in range(part.n_video):
        O[part.tokens(n)] = ro.sparse_attention_block(Q, K, V, mask[n], n, part, ref["scale"]) * R[n]
        if compensate:
            O[part.tokens(n)] += C[n][None, :]
    return O


def test_dense_flag_is_full_attention(gpu):
    import parity
    import torch
    from oracle import rsa_oracle as ro
    from paper_2511_19835_amd import binding as rb
    cfg = EDGE["ragged_d64_b128"]
    Qb, Kb, Vb = synth.make_inputs(cfg, 10)
    Q, K, V = (gpu.bits_to_device(x) for x in (Qb, Kb, Vb))
    buf = rb.allocate(Q, cfg.t_video, cfg.t_text, cfg.block)
    O = torch.empty_like(Q)
    rb.rsa_pool(buf.shape, Q, K, V, buf.Qp, buf.Kp, buf.Vp, buf.Vt, buf.Spool, buf.Apool, buf.Lmass, buf.Mc_bits,
                0, buf.pool_ws)
    rb.rsa_sparse_attn_rectified(buf.shape, Q, K, buf.Vt, None, None, None, None, None, None, None, rb.RSA_DENSE, O)
    torch.cuda.synchronize()
    Ob = gpu.device_to_bits(O)
    for h in range(cfg.heads):
        q, k, v = (ro.bf16_bits_to_f64(x[0, h]) for x in (Qb, Kb, Vb))
        dense = ro.dense_attention(q, k, v, 1 / np.sqrt(cfg.head_dim))
        err = ro.bf16_bits_to_f64(Ob[0, h]) - dense
        assert np.abs(err).max() <= parity.OUT_MAX_ABS
        assert np.linalg.norm(err) / np.linalg.norm(dense) <= parity.OUT_REL_L2


def test_results_are_deterministic(gpu):
    cfg = synth.CONFIGS["tiny"]
    Qb, Kb, Vb = synth.make_inputs(cfg, 11)
    a = gpu.run_layer(Qb, Kb, Vb, cfg.t_video, cfg.t_text, cfg.block, cfg.sparsity)
    b = gpu.run_layer(Qb, Kb, Vb, cfg.t_video, cfg.t_text, cfg.block, cfg.sparsity)
    for key in ("O_bits", "mask_words", "Mc_words", "R", "Apool", "Lmass", "count"):
        np.testing.assert_array_equal(a[key], b[key])


def test_full_size_hunyuan_shape_sampled(gpu):
    """The headline benchmark configuration at full size (24 heads, 118 800 video + 256 text tokens, block 128,
    90 %), in the launch configuration the benchmark times. All pooled tensors, masks, gates
    and factors of two heads are compared in full; outputs on sampled query blocks (first,
    ragged last video block, both text blocks, 12 random); cheap properties on every head."""
    import parity
    from paper_2511_19835_amd import binding as rb
    import torch
    cfg = synth.CONFIGS["hunyuan"]
    Qb, Kb, Vb = synth.make_inputs(cfg, 0, workers=8, threads=True)   # the GPU is initialised: no forking here
    out = gpu.run_layer(Qb, Kb, Vb, cfg.t_video, cfg.t_text, cfg.block, cfg.sparsity, want_lse=False)
    N, M = cfg.n_video_blocks, cfg.n_blocks
    assert (out["count"] == 94).all()
    assert (out["mask"].sum(axis=-1) == 94).all()
    assert np.all((out["R"] > 0) & (out["R"] <= 1 + 1e-5))
    np.testing.assert_allclose(out["Apool"].sum(axis=-1), 1.0, atol=2e-5)
    from oracle import rsa_oracle as ro
    assert np.isfinite(ro.bf16_bits_to_f64(out["O_bits"])).all()
    rng = np.random.default_rng(0)
    for h in (0, 17):
        blocks = sorted(set([0, N - 1, N, N + 1] + [int(x) for x in rng.integers(0, N, 12)]))
        ref = parity.oracle_head(Qb[0, h], Kb[0, h], Vb[0, h], cfg.t_video, cfg.t_text, cfg.block, cfg.sparsity,
                                 query_blocks=blocks)
        st = parity.compare_head(out, 0, h, ref, Qb[0, h], Kb[0, h], Vb[0, h], query_blocks=blocks)
        print(f"  [hunyuan h{h}] {st}", flush=True)


@pytest.mark.parametrize("grid,tile,block,t_text,radius", [
    ((4, 16, 16), (1, 8, 8), 64, 64, 1),        # tiny: blocks coincide with tiles
    ((13, 30, 52), (2, 8, 8), 128, 0, 1),       # mid: partial tiles along every axis
    ((5, 9, 17), (1, 8, 8), 64, 30, 1),         # one-token-wide partial tiles, ragged last block
    ((5, 9, 17), (2, 4, 4), 128, 0, 2),
    ((3, 20, 20), (2, 8, 8), 64, 0, 0),         # radius 0: blocks that share a tile
    ((33, 45, 80), (2, 8, 8), 128, 256, 1),     # the benchmark shape
])
def test_adjacency_mask_is_bit_exact(gpu, grid, tile, block, t_text, radius):
    """rsa_adjacency_mask against the oracle's tile-set definition, every bit, every (b, h)."""
    from oracle import rsa_oracle as ro
    tv = grid[0] * grid[1] * grid[2]
    got = gpu.adjacency_mask(tv, t_text, block, 64, grid, tile, radius, batch=1, heads=2)
    coords = synth.tile_order_coords(grid, block, tile)
    part = ro.partition(tv, t_text, block)
    ref = ro.adjacency_mask(coords, tile, part, radius)
    assert got.shape == (1, 2) + ref.shape
    assert np.array_equal(got[0, 0], ref) and np.array_equal(got[0, 1], ref)


def test_full_mask_rule_mid(gpu):
    """Alg. 1 steps 13-14 as the paper runs them: top-k, weight threshold p = 0.3 (appendix,
    parameter table) and the adjacency mask generated on the GPU, 2 heads of the mid config."""
    cfg = synth.CONFIGS["mid"]
    adja = gpu.adjacency_mask(cfg.t_video, cfg.t_text, cfg.block, cfg.head_dim, cfg.grid,
                              synth.default_tile(cfg.block), 1, batch=1, heads=2)
    out, stats, _ = _run_and_compare(gpu, cfg, heads=[0, 5], p=0.3, forced=adja)
    k = 159 - int(np.floor(0.9 * 159 + 1e-6))
    assert (out["count"] >= k).all() and (out["count"] > k).any()          # rows have different lengths now
    assert (out["mask"][:, :, :, :] >= adja).all()                         # every neighbour is kept


@pytest.mark.parametrize("grid,tile,block,t_text,d,layout", [
    ((4, 16, 16), (1, 8, 8), 64, 64, 64, "bhtd"),
    ((5, 9, 17), (2, 8, 8), 128, 30, 128, "bthd"),
    ((3, 5, 7), (2, 2, 4), 64, 0, 64, "bhtd"),
    ((33, 45, 80), (2, 8, 8), 128, 256, 128, "bhtd"),
])
def test_reorder_tokens_is_bit_exact(gpu, grid, tile, block, t_text, d, layout):
    """rsa_reorder_tokens against the oracle's enumeration of the tile order, both directions."""
    from oracle import rsa_oracle as ro
    tv = grid[0] * grid[1] * grid[2]
    rng = np.random.default_rng(11)
    X = rng.integers(0, 1 << 16, size=(1, 2, tv + t_text, d), dtype=np.uint16)
    fwd = gpu.reorder_tokens(X, tv, t_text, block, grid, tile, 0, layout)
    for h in range(2):
        assert np.array_equal(fwd[0, h], ro.reorder_tokens(X[0, h], grid, tile, 0))
    back = gpu.reorder_tokens(fwd, tv, t_text, block, grid, tile, 1, layout)
    assert np.array_equal(back, X)
    inv = gpu.reorder_tokens(X, tv, t_text, block, grid, tile, 1, layout)
    assert np.array_equal(inv[0, 1], ro.reorder_tokens(X[0, 1], grid, tile, 1))


def _sampled_shape_check(gpu, cfg, heads, seed, sparsity, n_random=8, **kw):
    """Full-size shape, a few heads: pooled tensors, masks, gates and factors in full, outputs on
    sampled query blocks (first, ragged last video block, text blocks, some random ones)."""
    import parity
    Qb, Kb, Vb = synth.make_inputs(cfg, seed, heads=heads, workers=min(8, len(heads)), threads=True)
    out = gpu.run_layer(Qb, Kb, Vb, cfg.t_video, cfg.t_text, cfg.block, sparsity, want_lse=False, **kw)
    N, M = cfg.n_video_blocks, cfg.n_blocks
    rng = np.random.default_rng(seed)
    for i, h in enumerate(heads):
        blocks = sorted(set([0, N - 1] + list(range(N, M)) + [int(x) for x in rng.integers(0, N, n_random)]))
        ref = parity.oracle_head(Qb[0, i], Kb[0, i], Vb[0, i], cfg.t_video, cfg.t_text, cfg.block, sparsity,
                                 query_blocks=blocks, **{k: v for k, v in kw.items() if k in ("p", "gapr_mode")})
        st = parity.compare_head(out, 0, i, ref, Qb[0, i], Kb[0, i], Vb[0, i], query_blocks=blocks,
                                 **{k: v for k, v in kw.items() if k in ("p",)})
        print(f"  [{cfg.name} seed {seed} sparsity {sparsity} h{h}] {st}", flush=True)
    return out


def test_wan_shape_sampled(gpu):
    """The second full-size benchmark configuration (Wan-2.1-like: 21x45x80 = 75 600 video tokens, no text, block 128, 90 %),
    three of its 40 heads."""
    cfg = synth.CONFIGS["wan"]
    out = _sampled_shape_check(gpu, cfg, [0, 19, 39], 0, cfg.sparsity)
    assert (out["count"] == 591 - int(np.floor(0.9 * 591 + 1e-6))).all()


@pytest.mark.parametrize("sparsity,seed,head", [(0.0, 0, 2), (0.5, 1, 5), (0.75, 2, 7), (0.85, 1, 11), (0.95, 2, 23)])
def test_sparsity_sweep_at_hunyuan_shape(gpu, sparsity, seed, head):
    """The sparsity sweep at the headline shape (one head per point, seeds 0-2).
    At sparsity 0 every block is critical: R = 1, nothing is compensated, output = dense attention."""
    cfg = synth.CONFIGS["hunyuan"]
    out = _sampled_shape_check(gpu, cfg, [head], seed, sparsity, n_random=4 if sparsity < 0.7 else 8)
    k = 931 - int(np.floor(sparsity * 931 + 1e-6))
    assert (out["count"] == k).all()
    if sparsity == 0.0:
        np.testing.assert_allclose(out["R"], 1.0, atol=2e-5)


def test_image_shape_with_long_text_sampled(gpu):
    """A 2-D image DiT shape (one latent frame, 256 x 256 tokens + 512 text tokens = 4 text blocks),
    paper's image setting keeps 10 % of the blocks; full mask rule on top (p = 0.3)."""
    cfg = synth.CONFIGS["flux"]
    out = _sampled_shape_check(gpu, cfg, [1, 13], 0, 0.9, p=0.3)
    assert (out["count"] >= 516 - int(np.floor(0.9 * 516 + 1e-6))).all()


def test_raster_ordered_tokens_end_to_end(gpu):
    """A caller with raster-ordered tokens: reorder in, adjacency mask, the three layer calls, reorder
    out — against the oracle run the same way (its own tile order, adjacency mask and layer)."""
    import parity
    from oracle import rsa_oracle as ro
    cfg = LayerConfig("raster", 1, 2, 64, (3, 12, 20), 40, 64, 0.6)
    tile = synth.default_tile(cfg.block)
    Qt, Kt, Vt = synth.make_inputs(cfg, 4)                       # drawn in tile order
    to_raster = lambda X: np.stack([[ro.reorder_tokens(X[0, h], cfg.grid, tile, 1) for h in range(cfg.heads)]])
    Qr, Kr, Vr = (to_raster(X) for X in (Qt, Kt, Vt))
    O_gpu = gpu.run_layer_from_raster(Qr, Kr, Vr, cfg.grid, tile, cfg.t_text, cfg.block, cfg.sparsity,
                                      p=0.3, use_adjacency=True)
    part = ro.partition(cfg.t_video, cfg.t_text, cfg.block)
    adja = ro.adjacency_mask(synth.tile_order_coords(cfg.grid, cfg.block, tile), tile, part, 1)
    for h in range(cfg.heads):
        Q, K, V = (ro.reorder_tokens(ro.bf16_bits_to_f64(X[0, h]), cfg.grid, tile, 0) for X in (Qr, Kr, Vr))
        ref = ro.rectified_layer_head(Q, K, V, cfg.t_video, cfg.t_text, cfg.block, cfg.sparsity, p=0.3, forced=adja)
        O_ref = ro.reorder_tokens(ref["O"], cfg.grid, tile, 1)
        err = ro.bf16_bits_to_f64(O_gpu[0, h]) - O_ref
        assert np.abs(err).max() <= parity.OUT_MAX_ABS
        assert np.linalg.norm(err) / np.linalg.norm(O_ref) <= parity.OUT_REL_L2


def test_masks_reused_for_a_second_call(gpu):
    """Pool and select once, attend twice: the second call sees new Q, K, V but the lists, factors,
    A^pool and gate bits of the first (rsa_pool_values + rsa_sparse_attn_rectified only)."""
    import parity
    from oracle import rsa_oracle as ro
    cfg = synth.CONFIGS["tiny"]
    s1, s2 = synth.make_inputs(cfg, 0), synth.make_inputs(cfg, 1)
    out = gpu.run_two_steps_reusing_masks(s1, s2, cfg.t_video, cfg.t_text, cfg.block, cfg.sparsity)
    part = ro.partition(cfg.t_video, cfg.t_text, cfg.block)
    scale = 1.0 / np.sqrt(cfg.head_dim)
    for h in range(cfg.heads):
        Q1, K1, V1 = (ro.bf16_bits_to_f64(x[0, h]) for x in s1)
        Q2, K2, V2 = (ro.bf16_bits_to_f64(x[0, h]) for x in s2)
        ref1 = ro.rectified_layer_head(Q1, K1, V1, cfg.t_video, cfg.t_text, cfg.block, cfg.sparsity)
        assert np.array_equal(out["mask"][0, h], ref1["mask"]) and np.array_equal(out["Mc"][0, h], ref1["Mc"])
        Vp2 = ro.pool(V2, part)
        np.testing.assert_allclose(out["Vp"][0, h], Vp2, rtol=2e-6, atol=2e-6)
        O_ref = np.empty_like(Q2)
        O_spa = ro.sparse_attention(Q2, K2, V2, ref1["mask"], part, scale)
        C = ro.compensation(ref1["A_pool"], ref1["mask"], ref1["Mc"], Vp2)
        for n in range(part.n_video):
            O_ref[part.tokens(n)] = ref1["R"][n] * O_spa[part.tokens(n)] + C[n][None, :]
        O_ref[cfg.t_video:] = ro.dense_attention(Q2[cfg.t_video:], K2, V2, scale)
        err = ro.bf16_bits_to_f64(out["O2_bits"][0, h]) - O_ref
        assert np.abs(err).max() <= parity.OUT_MAX_ABS
        assert np.linalg.norm(err) / np.linalg.norm(O_ref) <= parity.OUT_REL_L2


def test_implicit_attention_alone(gpu):
    """rsa_implicit_attention recomputes Spool, Lmass and A^pool from the pooled vectors of an earlier
    rsa_pool call: the same values as that call wrote (both run the same kernels), on a shape with a
    ragged last video block and text blocks, for both routes through the scores (rows within and beyond
    the one-pass kernel's 1024 blocks are covered by test_maximum_block_count through rsa_pool)."""
    import torch
    from paper_2511_19835_amd import binding as rb
    cfg = synth.CONFIGS["mid"].with_(heads=2, t_text=200)
    Qb, Kb, Vb = synth.make_inputs(cfg, 3)
    Q, K, V = (gpu.bits_to_device(x) for x in (Qb, Kb, Vb))
    buf = rb.allocate(Q, cfg.t_video, cfg.t_text, cfg.block)
    rb.rsa_pool(buf.shape, Q, K, V, buf.Qp, buf.Kp, buf.Vp, buf.Vt, buf.Spool, buf.Apool, buf.Lmass, buf.Mc_bits, 1,
                buf.pool_ws)
    want = [t.clone() for t in (buf.Spool, buf.Lmass, buf.Apool)]
    for t in (buf.Spool, buf.Lmass, buf.Apool):
        t.fill_(float("nan"))
    rb.rsa_implicit_attention(buf.shape, K, buf.Qp, buf.Kp, buf.Spool, buf.Lmass, buf.Apool)
    torch.cuda.synchronize()
    for got, ref in zip((buf.Spool, buf.Lmass, buf.Apool), want):
        assert torch.equal(got, ref)


def test_pooled_tensors_do_not_depend_on_the_gate_mode(gpu):
    """With the gate on, k^pool comes from the key-side deviation launch instead of the pooling kernel:
    every pooled tensor and the implicit attention must be bit for bit what gapr_mode 0 (no gate GEMMs,
    the pooling kernel for Q and K) writes. Shapes with a ragged last video block and text blocks, for
    each kernel template."""
    import torch
    from paper_2511_19835_amd import binding as rb
    for cfg in (synth.CONFIGS["mid"].with_(heads=2, t_text=200),
                synth.CONFIGS["tiny"].with_(t_text=70),
                synth.CONFIGS["mid"].with_(heads=1, head_dim=64, t_text=130),
                synth.CONFIGS["mid"].with_(heads=1, block=64, t_text=130)):
        Qb, Kb, Vb = synth.make_inputs(cfg, 5)
        Q, K, V = (gpu.bits_to_device(x) for x in (Qb, Kb, Vb))
        buf = rb.allocate(Q, cfg.t_video, cfg.t_text, cfg.block)
        names = ("Qp", "Kp", "Vp", "Vt", "Spool", "Lmass", "Apool")
        got = {}
        for mode in (0, 1):
            for name in names:
                t = getattr(buf, name)
                t.fill_(float("nan")) if t.is_floating_point() else t.zero_()
            rb.rsa_pool(buf.shape, Q, K, V, buf.Qp, buf.Kp, buf.Vp, buf.Vt, buf.Spool, buf.Apool, buf.Lmass,
                        buf.Mc_bits, mode, buf.pool_ws)
            torch.cuda.synchronize()
            got[mode] = {name: getattr(buf, name).clone() for name in names}
        for name in names:
            a, b = got[0][name], got[1][name]
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), (cfg.name, cfg.head_dim, cfg.block, name)


def test_maximum_block_count(gpu):
    """M = RSA_MAX_BLOCKS = 4096 key blocks (64 x 64 x 64 latent grid, block 64, one head of d 64):
    the selection kernel's LDS keys, the launch-order sort and the mask words at their largest."""
    cfg = LayerConfig("max", 1, 1, 64, (64, 64, 64), 0, 64, 0.99)
    assert cfg.n_blocks == 4096
    out = _sampled_shape_check(gpu, cfg, [0], 0, cfg.sparsity, n_random=6)
    assert (out["count"] == 4096 - int(np.floor(0.99 * 4096 + 1e-6))).all()
    assert out["mask_words"].shape[-1] == 128


def test_one_block_more_than_the_maximum_is_refused(gpu):
    import torch
    from paper_2511_19835_amd import binding as rb
    q = torch.zeros(1, 1, 4097 * 64, 64, dtype=torch.bfloat16, device="cuda:0")
    with pytest.raises(rb.RsaError) as e:
        rb.allocate(q, 4097 * 64, 0, 64)
    assert e.value.status == -3
