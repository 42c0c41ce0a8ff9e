"""rsa_sparse_attn_rectified_static (the entry point for callers that cannot allocate: its scratch is
a device array inside the library) against rsa_sparse_attn_rectified on the same buffers, through the
C-ABI: identical output bits, on two calls in a row, the second with a smaller input."""
import numpy as np
import pytest

from paper_2511_19835_amd import synth
from paper_2511_19835_amd.synth import LayerConfig

pytestmark = pytest.mark.gpu


def _both_entry_points(cfg, seed, sparsity, flags):
    import torch
    from paper_2511_19835_amd import binding as rb, harness
    Qb, Kb, Vb = synth.make_inputs(cfg, seed)
    Q, K, V = (harness.bits_to_device(x) for x in (Qb, Kb, Vb))
    buf = rb.allocate(Q, cfg.t_video, cfg.t_text, cfg.block)
    rb.rsa_pool(buf.shape, Q, K, V, buf.Qp, buf.Kp, buf.Vp, buf.Vt, buf.Spool, buf.Apool, buf.Lmass, buf.Mc_bits,
                1, buf.pool_ws)
    rb.rsa_select_blocks(buf.shape, buf.Lmass, buf.Apool, sparsity, 0.0, None, buf.mask_bits, buf.block_idx,
                         buf.count, buf.R)
    O_ws = torch.full_like(Q, float("nan"))
    O_st = torch.full_like(Q, float("nan"))
    lse_ws = torch.full(Q.shape[:3], float("nan"), dtype=torch.float32, device=Q.device)
    lse_st = torch.full_like(lse_ws, float("nan"))
    args = (buf.shape, Q, K, buf.Vt, buf.block_idx, buf.count, buf.mask_bits, buf.R, buf.Apool, buf.Mc_bits, buf.Vp, flags)
    rb.rsa_sparse_attn_rectified(*args, O_ws, lse_ws, buf.attn_ws)
    rb.rsa_sparse_attn_rectified_static(*args, O_st, lse_st)
    torch.cuda.synchronize()
    a, b = harness.device_to_bits(O_ws), harness.device_to_bits(O_st)
    assert not torch.isnan(O_st.float()).any(), "rows left unwritten"
    np.testing.assert_array_equal(a, b)
    np.testing.assert_array_equal(lse_ws.cpu().numpy(), lse_st.cpu().numpy())
    return Qb, Kb, Vb, b


def test_static_scratch_entry_point_matches_on_two_calls_in_a_row():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible: this test must run on the MI355X box")
    import parity
    big = LayerConfig("static_big", 1, 3, 128, (4, 16, 24), 150, 128, 0.7)      # 12 + 2 blocks, 3 heads
    small = LayerConfig("static_small", 1, 2, 64, (2, 9, 11), 20, 64, 0.5)      # ragged, fewer and shorter rows
    for cfg, seed in ((big, 21), (small, 22)):
        Qb, Kb, Vb, O_bits = _both_entry_points(cfg, seed, cfg.sparsity, 3)
        # and the shared result is the right one: head 0 against the oracle
        ref = parity.oracle_head(Qb[0, 0], Kb[0, 0], Vb[0, 0], cfg.t_video, cfg.t_text, cfg.block, cfg.sparsity)
        err = parity.bf16_bits_to_f64(O_bits[0, 0]) - ref["O"]
        assert np.abs(err).max() <= parity.OUT_MAX_ABS
        assert np.linalg.norm(err) / np.linalg.norm(ref["O"]) <= parity.OUT_REL_L2
    # without compensation and with the dense flag (scratch unused) the two entry points agree as well
    _both_entry_points(small, 23, 0.5, 1)
    _both_entry_points(small, 24, 0.5, 4)


def test_static_scratch_entry_point_refuses_shapes_beyond_its_array():
    import torch
    from paper_2511_19835_amd import binding as rb
    # 48 heads of 118 800 tokens: C_n alone is 22.8 MB > 16 MiB; refused on the host, nothing dereferenced
    t = 118800
    sh = rb.rsa_shape(batch=1, heads=48, head_dim=128, block=128, t_video=t, t_text=0,
                      stride_b=48 * t * 128, stride_h=t * 128, stride_t=128, scale=0.0)
    assert rb.rsa_workspace_bytes(sh)[1] > rb.RSA_STATIC_SCRATCH_BYTES
    x = torch.zeros(64, dtype=torch.int32, device="cuda:0")
    with pytest.raises(rb.RsaError) as e:
        rb.rsa_sparse_attn_rectified_static(sh, x, x, x, x, x, x, x, x, x, x, 3, x)
    assert e.value.status == -4
