"""GPU parity of the SLA backward pass: sla_attention_bwd (through the C ABI) against the float64
gradient oracle, element by element, on seeded synthetic inputs that span several tiles and ragged
tails.  The block mask is the library's own (its agreement with the oracle's classification is the
subject of the forward parity tests), so ties in the Top-K choice play no role here.

Tolerance.  The path computes in bf16 with fp32 accumulation: inputs are bf16 already; P, dS, the
per-block summaries H, Z, their gradients and the outputs are each rounded to bf16 once (relative
step 2^-9), the softmax statistics, delta and the normalisers stay in fp32.  A handful of
independent roundings of relative size 2^-9 per contribution, averaged over long sums, give a
relative Frobenius error well under 1e-2; single elements are held to 3e-2 of the largest
reference entry, and the direction (cosine) to 0.999 as for the forward pass."""
import numpy as np
import pytest
import torch

from oracle import sla_bwd_oracle as bo
from paper_2512_16093_amd import binding as sla
from paper_2512_16093_amd import synth

pytestmark = pytest.mark.gpu

REL_FRO, REL_MAX, COS_MIN = 1e-2, 3e-2, 0.999

CASES = [
    # (H, grid, block_q, rc, rm, proj)  -- batch 1; a batch of 2 is in test_backward_batch_of_two
    (2, (5, 10, 20), 128, 0.25, 0.0, False),   # sparse branch alone, N = 1000 (ragged in both block sizes)
    (2, (5, 10, 20), 64, 0.2, 0.0, False),
    (2, (5, 10, 20), 128, 0.25, 0.5, True),    # both branches with projection and bias gradient
    (2, (5, 10, 20), 64, 0.2, 0.4, True),
    (1, (3, 27, 27), 128, 0.1, 0.2, False),    # N = 2187 = 17*128 + 11, no projection (identity)
    (1, (1, 9, 9), 128, 0.5, 0.5, True),       # N = 81: one ragged query block, two key blocks
    (1, (1, 5, 5), 64, 1.0, 0.0, False),       # N = 25: a single short block, dense attention
    (1, (4, 16, 16), 64, 0.15, 0.85, True),    # N = 1024: whole blocks, no negligible block
    (2, (5, 10, 20), 128, 0.75, 0.25, True),   # most blocks critical: the dK/dV kernel's two-key-block variant
    (1, (3, 27, 27), 64, 0.6, 0.0, False),     # the same with an odd number of key blocks (35) and no linear term
]


def _compare(name, got, ref):
    got, ref = got.astype(np.float64), ref.astype(np.float64)
    scale = np.abs(ref).max()
    assert np.isfinite(got).all(), name
    if scale == 0.0:
        assert not got.any(), name
        return
    err = np.abs(got - ref).max()
    fro = np.linalg.norm(got - ref) / np.linalg.norm(ref)
    cos = float((got * ref).sum() / np.linalg.norm(got) / np.linalg.norm(ref))
    assert err <= REL_MAX * scale and fro <= REL_FRO and cos >= COS_MIN, (name, err / scale, fro, cos)


@pytest.mark.parametrize("H,grid,bq,rc,rm,proj", CASES)
def test_backward_matches_gradient_oracle(H, grid, bq, rc, rm, proj):
    cfg = synth.custom_config(1, H, grid, block_q=bq, topk_ratio=rc, marginal_ratio=rm, use_proj=proj, cfg_id=300)
    q, k, v = synth.make_qkv(cfg)
    dout = synth.make_qkv(cfg, seed=7)[2]          # a V-like tensor as the upstream gradient
    W = synth.make_proj(cfg) if proj else None
    dev = torch.device("cuda:0")
    qd, kd, vd, dd = (t.to(dev) for t in (q, k, v, dout))
    Wd = W.to(dev) if proj else None
    print("case", H, grid, bq, rc, rm, proj, flush=True)
    mask = sla.sla_classify_blocks(qd, kd, bq, 64, rc, rm, want_scores=False)[0].cpu().numpy()
    dq, dk, dv, dw, db = sla.sla_attention_bwd(qd, kd, vd, dd, bq, 64, rc, rm, proj_w=Wd, want_dw=proj, want_db=proj)
    torch.cuda.synchronize()
    sums_w = np.zeros((cfg.d, cfg.d))
    sums_b = np.zeros(cfg.d)
    for h in range(H):
        r = bo.sla_backward_head(synth.as_f64(q[0, h]), synth.as_f64(k[0, h]), synth.as_f64(v[0, h]),
                                 synth.as_f64(dout[0, h]), mask[0, h], bq, 64,
                                 proj_w=synth.as_f64(W) if proj else None, has_bias=proj)
        _compare("dq", dq[0, h].float().cpu().numpy(), r["dQ"])
        _compare("dk", dk[0, h].float().cpu().numpy(), r["dK"])
        _compare("dv", dv[0, h].float().cpu().numpy(), r["dV"])
        if proj:
            sums_w += r["dW"]
            sums_b += r["db"]
    if proj:
        _compare("dproj_w", dw.cpu().numpy(), sums_w)
        _compare("dproj_b", db.cpu().numpy(), sums_b)


@pytest.mark.parametrize("phi", ["elu1", "relu"])
@pytest.mark.parametrize("H,grid,bq,rc,rm", [(2, (5, 10, 20), 128, 0.25, 0.5), (1, (3, 27, 27), 64, 0.1, 0.9),
                                             (2, (5, 10, 20), 64, 0.75, 0.25)])
def test_backward_with_the_other_feature_maps(H, grid, bq, rc, rm, phi):
    """phi = elu + 1 or relu in the linear branch (the forward pass offers them; the oracle's gradient for
    them is pinned by the same finite-difference and autograd checks as the softmax's -- relu's on inputs
    kept away from its kink; the bf16 inputs here hold no exact zero that both sides would not treat
    alike, x > 0): both dK/dV variants."""
    cfg = synth.custom_config(1, H, grid, block_q=bq, topk_ratio=rc, marginal_ratio=rm, use_proj=True, cfg_id=303)
    q, k, v = synth.make_qkv(cfg)
    dout = synth.make_qkv(cfg, seed=11)[2]
    W = synth.make_proj(cfg)
    dev = torch.device("cuda:0")
    qd, kd, vd, dd, Wd = (t.to(dev) for t in (q, k, v, dout, W))
    mask = sla.sla_classify_blocks(qd, kd, bq, 64, rc, rm, want_scores=False)[0].cpu().numpy()
    dq, dk, dv, dw, db = sla.sla_attention_bwd(qd, kd, vd, dd, bq, 64, rc, rm, proj_w=Wd, want_dw=True, want_db=True,
                                               phi_kind=sla.PHI_ELU1 if phi == "elu1" else sla.PHI_RELU)
    torch.cuda.synchronize()
    sums_w, sums_b = np.zeros((cfg.d, cfg.d)), np.zeros(cfg.d)
    for h in range(H):
        r = bo.sla_backward_head(synth.as_f64(q[0, h]), synth.as_f64(k[0, h]), synth.as_f64(v[0, h]),
                                 synth.as_f64(dout[0, h]), mask[0, h], bq, 64, proj_w=synth.as_f64(W), has_bias=True,
                                 phi=phi)
        _compare("dq", dq[0, h].float().cpu().numpy(), r["dQ"])
        _compare("dk", dk[0, h].float().cpu().numpy(), r["dK"])
        _compare("dv", dv[0, h].float().cpu().numpy(), r["dV"])
        sums_w += r["dW"]
        sums_b += r["db"]
    _compare("dproj_w", dw.cpu().numpy(), sums_w)
    _compare("dproj_b", db.cpu().numpy(), sums_b)


def test_backward_batch_of_two():
    """Two batch entries with different contents: every (b, h) slice matches the oracle, and the
    projection gradients sum over both."""
    H, grid, bq, rc, rm = 2, (3, 9, 11), 128, 0.3, 0.5          # N = 297: ragged, Tq = 3 (odd), Tk = 5 (odd)
    cfg = synth.custom_config(2, H, grid, block_q=bq, topk_ratio=rc, marginal_ratio=rm, use_proj=True, cfg_id=301)
    q, k, v = synth.make_qkv(cfg)
    dout = synth.make_qkv(cfg, seed=9)[2]
    W = synth.make_proj(cfg)
    dev = torch.device("cuda:0")
    qd, kd, vd, dd, Wd = (t.to(dev) for t in (q, k, v, dout, W))
    assert not torch.equal(q[0], q[1])
    mask = sla.sla_classify_blocks(qd, kd, bq, 64, rc, rm, want_scores=False)[0].cpu().numpy()
    dq, dk, dv, dw, db = sla.sla_attention_bwd(qd, kd, vd, dd, bq, 64, rc, rm, proj_w=Wd, want_dw=True, want_db=True)
    torch.cuda.synchronize()
    sums_w, sums_b = np.zeros((cfg.d, cfg.d)), np.zeros(cfg.d)
    for b in range(2):
        for h in range(H):
            r = bo.sla_backward_head(synth.as_f64(q[b, h]), synth.as_f64(k[b, h]), synth.as_f64(v[b, h]),
                                     synth.as_f64(dout[b, h]), mask[b, h], bq, 64, proj_w=synth.as_f64(W), has_bias=True)
            _compare("dq", dq[b, h].float().cpu().numpy(), r["dQ"])
            _compare("dk", dk[b, h].float().cpu().numpy(), r["dK"])
            _compare("dv", dv[b, h].float().cpu().numpy(), r["dV"])
            sums_w += r["dW"]
            sums_b += r["db"]
    _compare("dproj_w", dw.cpu().numpy(), sums_w)
    _compare("dproj_b", db.cpu().numpy(), sums_b)


@pytest.mark.parametrize("H,grid,bq,rc,rm", [(2, (5, 10, 20), 128, 0.25, 0.5), (2, (3, 9, 11), 64, 0.3, 0.4)])
def test_backward_from_the_forward_pass_saved_state(H, grid, bq, rc, rm):
    """sla_attention_fwd_train gives the same output as the unquantised forward and a state with which
    sla_attention_bwd_saved matches the oracle to the same bar as the self-contained backward (and
    agrees with it closely: the only difference is delta formed from the bf16 O^s)."""
    cfg = synth.custom_config(1, H, grid, block_q=bq, topk_ratio=rc, marginal_ratio=rm, use_proj=True, cfg_id=302)
    q, k, v = synth.make_qkv(cfg)
    dout = synth.make_qkv(cfg, seed=5)[2]
    W = synth.make_proj(cfg)
    dev = torch.device("cuda:0")
    qd, kd, vd, dd, Wd = (t.to(dev) for t in (q, k, v, dout, W))
    out, saved = sla.sla_attention_fwd_train(qd, kd, vd, bq, 64, rc, rm, proj_w=Wd)
    ref_out = sla.sla_attention_fwd(qd, kd, vd, bq, 64, rc, rm, proj_w=Wd, quant_mode=sla.QUANT_NONE)
    assert torch.equal(out, ref_out)
    mask = sla.sla_classify_blocks(qd, kd, bq, 64, rc, rm, want_scores=False)[0].cpu().numpy()
    a = sla.sla_attention_bwd(qd, kd, vd, dd, bq, 64, rc, rm, proj_w=Wd, want_dw=True, want_db=True, saved=saved)
    b = sla.sla_attention_bwd(qd, kd, vd, dd, bq, 64, rc, rm, proj_w=Wd, want_dw=True, want_db=True)
    torch.cuda.synchronize()
    for x, y in zip(a[:3], b[:3]):
        x, y = x.float(), y.float()
        assert (x - y).abs().max() <= 2e-2 * y.abs().max()
    for h in range(H):
        r = bo.sla_backward_head(synth.as_f64(q[0, h]), synth.as_f64(k[0, h]), synth.as_f64(v[0, h]),
                                 synth.as_f64(dout[0, h]), mask[0, h], bq, 64, proj_w=synth.as_f64(W), has_bias=True)
        for name, got in (("dQ", a[0]), ("dK", a[1]), ("dV", a[2])):
            _compare(name, got[0, h].float().cpu().numpy(), r[name])


def test_backward_argument_errors():
    dev = torch.device("cuda:0")
    x = torch.zeros((1, 1, 128, 128), dtype=torch.bfloat16, device=dev)
    with pytest.raises(sla.SLAError) as e:
        sla.sla_attention_bwd(x, x, x, x, 128, 64, 0.5, 0.5, phi_kind=3)
    assert e.value.status == sla.ERR_UNSUPPORTED
    with pytest.raises(sla.SLAError) as e:
        sla.sla_attention_bwd(x, x, x, x, 128, 64, 0.5, 0.5, workspace=torch.empty(256, dtype=torch.uint8, device=dev))
    assert e.value.status == sla.ERR_WORKSPACE


def test_projection_gradients_are_deterministic_and_bias_alone_can_be_asked_for():
    """dproj_w and dproj_b are per-workgroup partial sums added in a fixed order: two calls give the same
    bits (a shape with several workgroups per head), and asking for the bias gradient alone gives the same
    bias gradient as asking for both."""
    cfg = synth.custom_config(1, 3, (8, 16, 32), block_q=128, topk_ratio=0.2, marginal_ratio=0.4, use_proj=True, cfg_id=305)
    q, k, v = synth.make_qkv(cfg)
    dout = synth.make_qkv(cfg, seed=5)[2]
    dev = torch.device("cuda:0")
    qd, kd, vd, dd, Wd = (t.to(dev) for t in (q, k, v, dout, synth.make_proj(cfg)))
    run = lambda **kw: sla.sla_attention_bwd(qd, kd, vd, dd, 128, 64, 0.2, 0.4, proj_w=Wd, **kw)
    a = run(want_dw=True, want_db=True)
    b = run(want_dw=True, want_db=True)
    c = run(want_db=True)
    torch.cuda.synchronize()
    for x, y in zip(a, b):
        assert torch.equal(x, y)
    assert c[3] is None and torch.equal(c[4], a[4])
    ref_b = dout.double().sum(dim=(0, 1, 2)).numpy()           # the bias gradient has a closed form
    assert np.abs(a[4].cpu().numpy() - ref_b).max() <= 1e-4 * np.abs(ref_b).max() + 1e-3


@pytest.mark.parametrize("bq,rc,rm", [(128, 0.25, 0.5), (64, 0.75, 0.25)])
def test_training_step_on_token_major_tensors_gives_the_same_bits(bq, rc, rm):
    """sla_attention_fwd_train_strided + sla_attention_bwd_strided on [B,N,H,d] memory (q, k, v packed in one
    [B,N,3,H,d] buffer, gradients written into another): bit-identical to the contiguous calls, which the tests
    above check against the oracle.  Both dK/dV variants (one and two key blocks per workgroup)."""
    cfg = synth.custom_config(2, 2, (5, 10, 20), block_q=bq, topk_ratio=rc, marginal_ratio=rm, use_proj=True, cfg_id=306)
    q, k, v = synth.make_qkv(cfg)
    dout = synth.make_qkv(cfg, seed=13)[2]
    dev = torch.device("cuda:0")
    qd, kd, vd, dd, Wd = (t.to(dev) for t in (q, k, v, dout, synth.make_proj(cfg)))
    out_ref, saved_ref = sla.sla_attention_fwd_train(qd, kd, vd, bq, 64, rc, rm, proj_w=Wd)
    ref = sla.sla_attention_bwd(qd, kd, vd, dd, bq, 64, rc, rm, proj_w=Wd, want_dw=True, want_db=True, saved=saved_ref)
    B, H, N, d = qd.shape
    packed = torch.stack([t.permute(0, 2, 1, 3) for t in (qd, kd, vd)], dim=2).contiguous()      # [B,N,3,H,d]
    qv, kv, vv = (packed[:, :, i].permute(0, 2, 1, 3) for i in range(3))
    dtm = dd.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    out_tm = torch.empty((B, N, H, d), dtype=torch.bfloat16, device=dev).permute(0, 2, 1, 3)
    saved = sla.sla_attention_fwd_train_strided(qv, kv, vv, out_tm, bq, 64, rc, rm, proj_w=Wd)
    assert torch.equal(out_tm, out_ref) and torch.equal(saved, saved_ref)
    grads = torch.full((B, N, 3, H, d), 7.0, dtype=torch.bfloat16, device=dev)
    gq, gk, gv = (grads[:, :, i].permute(0, 2, 1, 3) for i in range(3))
    for sv in (saved, None):                          # from the saved statistics, and recomputing them
        dw, db = sla.sla_attention_bwd_strided(qv, kv, vv, dtm, gq, gk, gv, bq, 64, rc, rm, proj_w=Wd, want_dw=True,
                                               want_db=True, saved=sv)
        torch.cuda.synchronize()
        if sv is None:
            ref = sla.sla_attention_bwd(qd, kd, vd, dd, bq, 64, rc, rm, proj_w=Wd, want_dw=True, want_db=True)
        for got, want in zip((gq, gk, gv, dw, db), ref):
            assert torch.equal(got, want)


def test_saved_state_of_another_problem_poisons_the_gradients():
    """The state a training forward pass saves names its problem; handed to a backward pass with another number of
    critical blocks per row (same sizes, so the byte count matches) every gradient comes out NaN, not plausibly wrong."""
    cfg = synth.custom_config(1, 2, (5, 10, 20), block_q=128, topk_ratio=0.25, marginal_ratio=0.5, cfg_id=330)
    q, k, v = synth.make_qkv(cfg)
    dout = synth.make_qkv(cfg, seed=7)[2]
    W = synth.make_proj(cfg)
    qd, kd, vd, dd, Wd = (t.cuda() for t in (q, k, v, dout, W))
    out, saved = sla.sla_attention_fwd_train(qd, kd, vd, 128, 64, 0.25, 0.5, proj_w=Wd)
    good = sla.sla_attention_bwd(qd, kd, vd, dd, 128, 64, 0.25, 0.5, proj_w=Wd, saved=saved)
    assert all(torch.isfinite(g.float()).all() for g in good[:3])
    bad = sla.sla_attention_bwd(qd, kd, vd, dd, 128, 64, 0.5, 0.5, proj_w=Wd, saved=saved)   # 8 critical blocks, not 4
    assert all(torch.isnan(g.float()).any() for g in bad[:3])
    junk = torch.zeros_like(saved)
    assert torch.isnan(sla.sla_attention_bwd(qd, kd, vd, dd, 128, 64, 0.25, 0.5, proj_w=Wd, saved=junk)[0].float()).any()

