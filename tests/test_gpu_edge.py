"""GPU parity on the degenerate inputs the method has (Section 1.1: smoothing, per-block INT8 scales, FP8
weights; Section 1.3: Top-K classification): operands whose quantisation scale is taken from an all-zero
block, rows of equal block scores, a key block that outweighs everything before it by more than the
rescaling hardware can express in one step, inputs of larger magnitude -- and the longest sequence the
library accepts.  Every case goes through the C ABI and is compared with the oracle like the ordinary cases."""
import numpy as np
import pytest
import torch

from oracle import sla_oracle as so
from paper_2512_16093_amd import binding as sla
from paper_2512_16093_amd import synth

import parity_util as pu

pytestmark = pytest.mark.gpu


def _constant_keys(q, k, v):
    """Every key the same vector: smoothing leaves all-zero keys (scale 1, codes 0), all scores and all
    pooled scores are equal (classification by index alone, uniform attention)."""
    k = k.clone()
    k[:] = k[0, 0, 0]
    return q, k, v


def _zero_blocks(q, k, v):
    """An all-zero query block (scale 1, scores 0, equal pooled scores), an all-zero and a constant channel of V
    (the first has scale 1 and codes 0), a key block that repeats one vector."""
    q, k, v = q.clone(), k.clone(), v.clone()
    q[:, :, :128] = 0
    v[..., 5] = 0
    v[..., 9] = 1.5
    k[:, :, 64:128] = k[:, :, 64:65]
    return q, k, v


def _late_dominant_block(q, k, v):
    """The last key block scores ~ 50 nats above everything before it for every query: the reference level
    jumps by more than 64 binary orders at the end of every row, beyond what one block scale expresses."""
    q, k = q.float(), k.float()
    q = q + 1.8
    N = k.shape[2]
    k[:, :, (N - 1) // 64 * 64:] += 2.4
    return q.to(torch.bfloat16), k.to(torch.bfloat16), v


def _doubled(q, k, v):
    """Q and K times two (exact in bf16): scores four times as large, sharper rows, more weights that round to 0."""
    return (q.float() * 2).to(torch.bfloat16), (k.float() * 2).to(torch.bfloat16), v


def _check_sharp_rows(gpu, ref, what):
    """The bar for inputs that make rows sharp (a few keys carry most of a row's weight).  There a single FP8
    weight (3 mantissa bits: relative step 2^-4 .. 2^-3) that rounds the other way in the kernel's fp32 than
    in the oracle's fp64 is worth several percent of the output, and the kernel knows a weight's exponent to
    ~1e-4 only (the score bias it carries through the conversion-free exponent costs that much).  Such rows are
    few and scattered; an indexing or scaling mistake moves most rows.  So: at most 1 % of the rows beyond the
    usual 2e-2, none beyond 8e-2, cosine as usual."""
    gpu = np.asarray(gpu, dtype=np.float64)
    assert np.isfinite(gpu).all(), what + ": non-finite output"
    row_err = np.abs(gpu - ref).max(axis=1)
    assert row_err.max() <= 8e-2, "%s: max-abs %.3e" % (what, row_err.max())
    assert (row_err > pu.MAX_ABS).mean() <= 0.01, "%s: %d rows beyond %.0e" % (what, (row_err > pu.MAX_ABS).sum(), pu.MAX_ABS)
    assert pu.cosine(gpu, ref) >= pu.MIN_COS, what + ": cosine"


CASES = {"constant_keys": _constant_keys, "zero_blocks": _zero_blocks, "late_dominant_block": _late_dominant_block,
         "doubled": _doubled}


@pytest.mark.parametrize("bq", [128, 64])
@pytest.mark.parametrize("name", sorted(CASES))
def test_degenerate_inputs_low_bit_forward(name, bq):
    cfg = synth.custom_config(1, 2, (5, 10, 20), block_q=bq, topk_ratio=0.25, marginal_ratio=0.5, cfg_id=700)
    q, k, v = CASES[name](*synth.make_qkv(cfg))
    W = synth.make_proj(cfg)
    qd, kd, vd, Wd = pu.to_dev(q, k, v, W)
    out = sla.sla_attention_fwd(qd, kd, vd, bq, 64, cfg.topk_ratio, cfg.marginal_ratio, proj_w=Wd).float().cpu().numpy()
    mask = sla.sla_classify_blocks(qd, kd, bq, 64, cfg.topk_ratio, cfg.marginal_ratio)[0].cpu().numpy()
    Tq, Tk, n_c, n_m = so.block_counts(cfg.N, bq, 64, cfg.topk_ratio, cfg.marginal_ratio)
    assert np.isfinite(out).all()
    qc, qs = (t.cpu().numpy() for t in sla.sla_debug_quantize_q(qd, bq))
    vc = sla.sla_debug_quantize_kv(kd, vd)[3].cpu().numpy()
    from oracle import formats
    for h in range(cfg.H):
        # the operands quantised from 16-bit inputs carry the oracle's codes exactly (zero blocks and exact ties included)
        Q8, dq = so.quantize_q(synth.as_f64(q[0, h]), bq)
        assert np.array_equal(qc[0, h].astype(np.float64), Q8) and np.allclose(qs[0, h], dq, rtol=1e-6)
        assert np.array_equal(formats.e4m3_decode(vc[0, h]), so.quantize_v(synth.as_f64(v[0, h]))[0])
        r = pu.oracle_head(cfg, q, k, v, 0, h, W)
        nbad, _, _ = pu.check_mask(mask[0, h], r["scores"], n_c, n_m, "%s head %d" % (name, h))
        if nbad:
            r = pu.oracle_head(cfg, q, k, v, 0, h, W, mask=mask[0, h])
        if name in ("doubled", "late_dominant_block"):
            _check_sharp_rows(out[0, h], r["out"], "%s head %d" % (name, h))
        else:
            pu.check_output(out[0, h], r["out"], "%s head %d" % (name, h))
    if name == "constant_keys":   # equal scores everywhere: the lowest block indices win, in every row
        assert (mask[..., :n_c] == 1).all() and (mask[..., n_c:n_c + n_m] == 0).all() and (mask[..., n_c + n_m:] == -1).all()


@pytest.mark.parametrize("name", sorted(CASES))
def test_degenerate_inputs_unquantised_forward_and_backward(name):
    """The same inputs through the 16-bit forward pass and the backward pass (bf16 products, fp32 statistics)."""
    from oracle import sla_bwd_oracle as bo
    bq = 128
    cfg = synth.custom_config(1, 1, (5, 10, 20), block_q=bq, topk_ratio=0.25, marginal_ratio=0.5, cfg_id=701)
    q, k, v = CASES[name](*synth.make_qkv(cfg))
    W = synth.make_proj(cfg)
    dout = synth.make_qkv(cfg, seed=5)[2]
    qd, kd, vd, Wd, dd = pu.to_dev(q, k, v, W, dout)
    out = sla.sla_attention_fwd(qd, kd, vd, bq, 64, cfg.topk_ratio, cfg.marginal_ratio, proj_w=Wd,
                                quant_mode=sla.QUANT_NONE).float().cpu().numpy().astype(np.float64)
    mask = sla.sla_classify_blocks(qd, kd, bq, 64, cfg.topk_ratio, cfg.marginal_ratio, want_scores=False)[0].cpu().numpy()
    Q, K, V, D = (synth.as_f64(t[0, 0]) for t in (q, k, v, dout))
    r = so.sla_forward_head(Q, K, V, bq, 64, cfg.topk_ratio, cfg.marginal_ratio, proj_w=synth.as_f64(W),
                            quant=so.QUANT_NONE, mask=mask[0, 0])
    pu.check_output(out[0, 0], r["out"], name + " unquantised forward")
    g = sla.sla_attention_bwd(qd, kd, vd, dd, bq, 64, cfg.topk_ratio, cfg.marginal_ratio, proj_w=Wd)
    ref = bo.sla_backward_head(Q, K, V, D, mask[0, 0], bq, 64, proj_w=synth.as_f64(W), has_bias=False)
    for key, got in (("dQ", g[0]), ("dK", g[1]), ("dV", g[2])):
        a = got[0, 0].float().cpu().numpy().astype(np.float64)
        b = ref[key]
        assert np.isfinite(a).all(), "%s %s: non-finite" % (name, key)
        # (with constant keys dQ is exactly 0 -- the rows of dS sum to zero -- and the bf16 path leaves rounding
        # residue of dS times |K| there: the bounds are taken relative to a magnitude of at least 1)
        scale = max(np.abs(b).max(), 1.0)
        assert np.linalg.norm(a - b) <= 1e-2 * max(np.linalg.norm(b), np.sqrt(b.size)), "%s %s: Frobenius" % (name, key)
        assert np.abs(a - b).max() <= 3e-2 * scale, "%s %s: element" % (name, key)


@pytest.mark.parametrize("bq", [128, 64])
@pytest.mark.parametrize("n_c", [2, 5, 6, 7, 8, 9, 17])
def test_every_list_length_through_the_sparse_stage(n_c, bq):
    """The attention kernel's main loop takes four list entries per round, up to three more one by one, and the
    ragged last key block apart: lists of every remainder, with and without the last block, chosen at random
    (ascending, as the classification delivers them), through sla_sparse_attn_fwd against the oracle on the same mask.
    With query blocks of 64 the kernel merges the lists of adjacent blocks (17 query blocks: the last pair has one)."""
    cfg = synth.custom_config(1, 2, (6, 7, 25), block_q=bq, topk_ratio=0.2, marginal_ratio=0.4, cfg_id=710)   # N = 1050, Tk = 17
    q, k, v = synth.make_qkv(cfg)
    Tq, Tk = -(-cfg.N // bq), -(-cfg.N // 64)
    rng = np.random.default_rng(1000 * n_c + bq)
    masks = np.full((1, cfg.H, Tq, Tk), -1, dtype=np.int8)
    for h in range(cfg.H):
        for i in range(Tq):
            pick = rng.choice(Tk, size=n_c, replace=False)
            if i % 3 == 0 and (Tk - 1) not in pick:      # a third of the rows must end in the ragged block
                pick[0] = Tk - 1
            if i % 3 == 1 and n_c < Tk:                  # a third must not
                pick = rng.choice(Tk - 1, size=n_c, replace=False)
            masks[0, h, i, pick] = 1
    crit = pu.lists_from_mask(masks)
    out, lse = sla.sla_sparse_attn_fwd(*pu.to_dev(q, k, v, crit), bq, 64)
    out, lse = out.cpu().numpy(), lse.cpu().numpy()
    for h in range(cfg.H):
        ref, ref_lse = so.sparse_branch_quant(synth.as_f64(q[0, h]), synth.as_f64(k[0, h]), synth.as_f64(v[0, h]),
                                              masks[0, h], bq, 64, return_lse=True, ref_tile=pu.REF_TILE)
        pu.check_output(out[0, h], ref, "n_c %d head %d" % (n_c, h))
        dl = np.abs(lse[0, h] - ref_lse)
        assert dl.max() < 2e-2 and np.median(dl) < 1e-5


def test_codes_of_blocks_with_tiny_maxima():
    """Blocks whose largest magnitude is far below the reciprocal's range (16-bit inputs reach 2^-133; 1 / 2^-130
    overflows fp32): the quotient is formed on a rescaled maximum, the codes are still the oracle's."""
    from oracle import formats
    cfg = synth.custom_config(1, 1, (2, 8, 16), block_q=128, topk_ratio=0.5, marginal_ratio=0.5, cfg_id=730)   # N = 256
    q, k, v = synth.make_qkv(cfg)
    q, v = q.float(), v.float()
    q[:, :, :128] *= 2.0 ** -128          # first query block: maxima near 2^-126, most values denormal in bf16
    v[..., 3] *= 2.0 ** -127
    v[..., 7] *= 2.0 ** -110
    q, v = q.to(torch.bfloat16), v.to(torch.bfloat16)
    qc, qs = (t.cpu().numpy() for t in sla.sla_debug_quantize_q(q.cuda(), 128))
    vc = sla.sla_debug_quantize_kv(k.cuda(), v.cuda())[3].cpu().numpy()
    Q8, dq = so.quantize_q(synth.as_f64(q[0, 0]), 128)
    assert np.array_equal(qc[0, 0].astype(np.float64), Q8) and np.allclose(qs[0, 0], dq, rtol=1e-6)
    assert np.array_equal(formats.e4m3_decode(vc[0, 0]), so.quantize_v(synth.as_f64(v[0, 0]))[0])
    out = sla.sla_attention_fwd(q.cuda(), k.cuda(), v.cuda(), 128, 64, 0.5, 0.5).float().cpu().numpy()
    r = pu.oracle_head(cfg, q, k, v, 0, 0, None)
    pu.check_output(out[0, 0], r["out"], "tiny maxima")
