"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by
element, on seeded synthetic inputs.  Sizes here finish in seconds on the CPU side and
still span several tiles plus ragged tails; the full-size sampled checks are in
test_gpu_fullsize.py."""
import math

import numpy as np
import pytest
import torch

from oracle import formats
from oracle import sla_oracle as so
from paper_2512_16093_amd import binding as sla
from paper_2512_16093_amd import synth

import parity_util as pu

pytestmark = pytest.mark.gpu

RAGGED = [
    # (H, grid, block_q, rc, rm): N = 1000 (15 full key blocks + 40), 2080+..., etc.
    (2, (5, 10, 20), 64, 0.2, 0.4),
    (2, (5, 10, 20), 128, 0.25, 0.5),
    (1, (3, 27, 27), 128, 0.1, 0.2),      # N = 2187 = 17*128 + 11 = 34*64 + 11
    (1, (1, 9, 9), 128, 0.5, 0.5),        # N = 81: one ragged query block, two key blocks
    (1, (1, 5, 5), 64, 1.0, 0.0),         # N = 25: a single short block
    (1, (3, 9, 7), 64, 0.34, 0.66),       # N = 189: three query blocks of 64 (an odd count: the last pair has one)
    (2, (6, 7, 25), 64, 0.2, 0.4),        # N = 1050: 17 query blocks of 64, ragged
]


def _cfg(H, grid, bq, rc, rm, proj=True, cid=100):
    return synth.custom_config(1, H, grid, block_q=bq, topk_ratio=rc, marginal_ratio=rm, use_proj=proj, cfg_id=cid)


def test_fp8_encoding_matches_software_e4m3():
    rng = np.random.default_rng(0)
    pos = formats.e4m3_decode(np.arange(0, 0x7F, dtype=np.uint8))
    mids = (pos[:-1] + pos[1:]) / 2
    x = np.concatenate([pos, -pos, mids, -mids, np.nextafter(mids.astype(np.float32), 1e9),
                        np.nextafter(mids.astype(np.float32), -1e9), rng.uniform(-448, 448, 50000),
                        np.exp2(rng.uniform(-14, 9, 50000)), [448.0, 449.0, 463.9, 464.0, 480.0, 1e6, -1e6, 1e30]]
                       ).astype(np.float32)
    got = sla.sla_debug_e4m3_encode(torch.from_numpy(x).cuda()).cpu().numpy()
    want = formats.e4m3_encode(x.astype(np.float64))
    # +0 and -0 are distinct codes of the same value: compare decoded values, then codes off zero
    nz = x != 0
    assert np.array_equal(got[nz], want[nz])
    assert np.array_equal(formats.e4m3_decode(got), formats.e4m3_decode(want))


@pytest.mark.parametrize("case", [None] + RAGGED[:3])
def test_quantised_operands_match_oracle(case):
    cfg = synth.CONFIGS[0] if case is None else _cfg(*case)
    q, k, v = synth.make_qkv(cfg)
    kc, ks, km, vc, vs = (t.cpu().numpy() for t in sla.sla_debug_quantize_kv(*pu.to_dev(k, v)))
    for h in range(cfg.H):
        K, V = synth.as_f64(k[0, h]), synth.as_f64(v[0, h])
        K8, dk, mu = so.quantize_k(K, 64)
        V8, dv = so.quantize_v(V)
        assert np.abs(km[0, h] - mu).max() < 2e-6
        assert np.allclose(ks[0, h], dk, rtol=1e-5)
        assert np.allclose(vs[0, h], dv, rtol=1e-6)
        # K codes: the smoothed K is formed in fp32 on the GPU and in fp64 here, so a code may differ where
        # the two differences fall on either side of a rounding boundary (about one code in 10^5)
        dkc = kc[0, h].astype(np.float64) - K8
        assert np.abs(dkc).max() <= 1 and (dkc != 0).mean() < 1e-4
        # V and Q are quantised from the 16-bit inputs themselves: the same codes, exact ties included
        assert np.array_equal(formats.e4m3_decode(vc[0, h]), V8)
    qc, qs = (t.cpu().numpy() for t in sla.sla_debug_quantize_q(q.cuda(), cfg.block_q))
    for h in range(cfg.H):
        Q8, dq = so.quantize_q(synth.as_f64(q[0, h]), cfg.block_q)
        assert np.allclose(qs[0, h], dq, rtol=1e-6)
        assert np.array_equal(qc[0, h].astype(np.float64), Q8)


@pytest.mark.parametrize("case", [None] + RAGGED)
def test_block_classification_matches_oracle(case):
    cfg = synth.CONFIGS[0] if case is None else _cfg(*case)
    q, k, v = synth.make_qkv(cfg)
    mask, crit, marg, scores = sla.sla_classify_blocks(*pu.to_dev(q, k), cfg.block_q, cfg.block_k,
                                                       cfg.topk_ratio, cfg.marginal_ratio)
    Tq, Tk, n_c, n_m = so.block_counts(cfg.N, cfg.block_q, cfg.block_k, cfg.topk_ratio, cfg.marginal_ratio)
    assert mask.shape == (1, cfg.H, Tq, Tk) and crit.shape[-1] == n_c and marg.shape[-1] == n_m
    mask, crit, marg, scores = (t.cpu().numpy() for t in (mask, crit, marg, scores))
    for h in range(cfg.H):
        s64 = so.pooled_scores(synth.as_f64(q[0, h]), synth.as_f64(k[0, h]), cfg.block_q, cfg.block_k)
        assert np.abs(scores[0, h] - s64).max() < 2e-5
        pu.check_mask(mask[0, h], s64, n_c, n_m, "head %d" % h)
        for i in range(Tq):
            assert np.array_equal(crit[0, h, i], np.flatnonzero(mask[0, h, i] == 1))
            assert np.array_equal(marg[0, h, i], np.flatnonzero(mask[0, h, i] == 0))


@pytest.mark.parametrize("case", [None] + RAGGED)
def test_sparse_branch_matches_oracle(case):
    cfg = synth.CONFIGS[0] if case is None else _cfg(*case)
    q, k, v = synth.make_qkv(cfg)
    Tq, Tk, n_c, n_m = so.block_counts(cfg.N, cfg.block_q, cfg.block_k, cfg.topk_ratio, cfg.marginal_ratio)
    masks = np.stack([so.classify(so.pooled_scores(synth.as_f64(q[0, h]), synth.as_f64(k[0, h]), cfg.block_q, 64),
                                  n_c, n_m) for h in range(cfg.H)])[None]
    crit = pu.lists_from_mask(masks)
    out, lse = sla.sla_sparse_attn_fwd(*pu.to_dev(q, k, v, crit), cfg.block_q, cfg.block_k)
    out, lse = out.cpu().numpy(), lse.cpu().numpy()
    for h in range(cfg.H):
        ref, ref_lse = so.sparse_branch_quant(synth.as_f64(q[0, h]), synth.as_f64(k[0, h]), synth.as_f64(v[0, h]),
                                              masks[0, h], cfg.block_q, 64, return_lse=True, ref_tile=pu.REF_TILE)
        # tighter than the task's 2e-2 where a row's softmax spans several blocks; with a single 64-key block
        # one weight whose 8-bit rounding falls the other way (fp32 here, fp64 there) moves an output by ~1e-2
        pu.check_output(out[0, h], ref, "sparse head %d" % h, max_abs=1e-2 if n_c > 1 else pu.MAX_ABS)
        # the row sum is a sum of FP8-rounded terms: a rounding that falls the other way moves it a little
        dl = np.abs(lse[0, h] - ref_lse)
        assert dl.max() < 2e-2 and np.median(dl) < 1e-5


# every shape with the default feature map; the alternative ones on two shapes
@pytest.mark.parametrize("case,phi", [(c, "softmax") for c in [None] + RAGGED[:4]] +
                         [(c, f) for f in ("elu1", "relu") for c in (None, RAGGED[0])])
def test_linear_branch_matches_oracle(case, phi):
    cfg = synth.CONFIGS[0] if case is None else _cfg(*case)
    q, k, v = synth.make_qkv(cfg)
    W = synth.make_proj(cfg)
    bias = (torch.arange(cfg.d, dtype=torch.float32) / 64 - 1).to(torch.bfloat16)
    Tq, Tk, n_c, n_m = so.block_counts(cfg.N, cfg.block_q, cfg.block_k, cfg.topk_ratio, cfg.marginal_ratio)
    masks = np.stack([so.classify(so.pooled_scores(synth.as_f64(q[0, h]), synth.as_f64(k[0, h]), cfg.block_q, 64),
                                  n_c, n_m) for h in range(cfg.H)])[None]
    kind = {"softmax": sla.PHI_SOFTMAX, "elu1": sla.PHI_ELU1, "relu": sla.PHI_RELU}[phi]
    dq, dk, dv, dm, dW, db = pu.to_dev(q, k, v, torch.from_numpy(masks), W, bias)
    out = sla.sla_linear_attn_fwd(dq, dk, dv, dm, cfg.block_q, cfg.block_k, proj_w=dW, proj_b=db,
                                  phi_kind=kind).cpu().numpy()
    for h in range(cfg.H):
        ol = so.linear_branch(synth.as_f64(q[0, h]), synth.as_f64(k[0, h]), synth.as_f64(v[0, h]), masks[0, h],
                              cfg.block_q, 64, phi)
        ref = ol @ synth.as_f64(W).T + synth.as_f64(bias)[None, :]
        pu.check_output(out[0, h], ref, "linear %s head %d" % (phi, h), max_abs=6e-3, min_cos=0.9999)
    # identity projection, no bias
    out = sla.sla_linear_attn_fwd(dq, dk, dv, dm, cfg.block_q, cfg.block_k, phi_kind=kind).cpu().numpy()
    ol = so.linear_branch(synth.as_f64(q[0, 0]), synth.as_f64(k[0, 0]), synth.as_f64(v[0, 0]), masks[0, 0],
                          cfg.block_q, 64, phi)
    pu.check_output(out[0, 0], ol, "linear identity", max_abs=6e-3, min_cos=0.9999)


# every shape with seed 0; a second seed on the named tiny config
@pytest.mark.parametrize("case,seed", [(c, 0) for c in [None] + RAGGED] + [(None, 1)])
def test_full_forward_matches_oracle(case, seed):
    cfg = synth.CONFIGS[0] if case is None else _cfg(*case)
    q, k, v = synth.make_qkv(cfg, seed=seed)
    W = synth.make_proj(cfg, seed=seed)
    out = sla.sla_attention_fwd(*pu.to_dev(q, k, v), cfg.block_q, cfg.block_k, cfg.topk_ratio,
                                cfg.marginal_ratio, proj_w=W.cuda()).float().cpu().numpy()
    mask = sla.sla_classify_blocks(*pu.to_dev(q, k), cfg.block_q, cfg.block_k, cfg.topk_ratio,
                                   cfg.marginal_ratio)[0].cpu().numpy()
    Tq, Tk, n_c, n_m = so.block_counts(cfg.N, cfg.block_q, cfg.block_k, cfg.topk_ratio, cfg.marginal_ratio)
    for h in range(cfg.H):
        r = pu.oracle_head(cfg, q, k, v, 0, h, W)
        nbad, _, _ = pu.check_mask(mask[0, h], r["scores"], n_c, n_m, "head %d" % h)
        if nbad:   # a tie went the other way: compare against the oracle run on the GPU's mask
            r = pu.oracle_head(cfg, q, k, v, 0, h, W, mask=mask[0, h])
        pu.check_output(out[0, h], r["out"], "full head %d" % h)


@pytest.mark.parametrize("case,seed", [(c, 0) for c in [None] + RAGGED] + [(None, 1)])
def test_full_forward_against_the_plain_reading_of_the_scheme(case, seed):
    """The same GPU output against the oracle run WITHOUT the three switches that follow the kernel's
    shape: the plain running maximum as the softmax reference (not its integer ceiling), refreshed
    once per 64-key block (not per 32 keys), and the row sum of the unrounded weights.  The two
    readings round P to the 8-bit float at different levels, so they differ from each other by what
    either differs from the exact branch (CPU test test_the_two_readings_are_equally_close_to_exact:
    up to 2.7e-2 in one element, 3e-3 rms on these shapes); the cosine bound of the task holds
    unchanged, the element bound is the task's 2e-2 plus that rounding share, and the GPU result
    must be as close to the exact (unquantised) branch as the plain reading is."""
    cfg = synth.CONFIGS[0] if case is None else _cfg(*case)
    q, k, v = synth.make_qkv(cfg, seed=seed)
    W = synth.make_proj(cfg, seed=seed)
    out = sla.sla_attention_fwd(*pu.to_dev(q, k, v), cfg.block_q, cfg.block_k, cfg.topk_ratio,
                                cfg.marginal_ratio, proj_w=W.cuda()).float().cpu().numpy().astype(np.float64)
    mask = sla.sla_classify_blocks(*pu.to_dev(q, k), cfg.block_q, cfg.block_k, cfg.topk_ratio,
                                   cfg.marginal_ratio)[0].cpu().numpy()
    for h in range(cfg.H):
        Q, K, V = (synth.as_f64(t[0, h]) for t in (q, k, v))
        kw = dict(proj_w=synth.as_f64(W), mask=mask[0, h])
        plain = so.sla_forward_head(Q, K, V, cfg.block_q, cfg.block_k, cfg.topk_ratio, cfg.marginal_ratio,
                                    reference="running", rowsum_quantized=False, ref_tile=None, **kw)["out"]
        exact = so.sla_forward_head(Q, K, V, cfg.block_q, cfg.block_k, cfg.topk_ratio, cfg.marginal_ratio,
                                    quant=so.QUANT_NONE, **kw)["out"]
        pu.check_output(out[0, h], plain, "plain reading, head %d" % h, max_abs=3.5e-2, min_cos=pu.MIN_COS)
        rms = lambda x: float(np.sqrt((x ** 2).mean()))
        assert rms(out[0, h] - exact) <= 1.15 * rms(plain - exact) + 1e-3


def test_full_forward_bias_batch_and_no_marginal():
    # B = 2, bias, and a second call with no marginal blocks (no linear term, bias dropped)
    cfg = synth.custom_config(2, 2, (2, 16, 16), block_q=128, topk_ratio=0.25, marginal_ratio=0.25, cfg_id=101)
    q, k, v = synth.make_qkv(cfg)
    W = synth.make_proj(cfg)
    bias = (torch.linspace(-0.5, 0.5, cfg.d)).to(torch.bfloat16)
    out = sla.sla_attention_fwd(*pu.to_dev(q, k, v), 128, 64, 0.25, 0.25, proj_w=W.cuda(),
                                proj_b=bias.cuda()).float().cpu().numpy()
    for b in range(2):
        for h in range(2):
            r = pu.oracle_head(cfg, q, k, v, b, h, W, bias)
            pu.check_output(out[b, h], r["out"], "b%d h%d" % (b, h))
    out0 = sla.sla_attention_fwd(*pu.to_dev(q, k, v), 128, 64, 0.25, 0.0, proj_w=W.cuda(),
                                 proj_b=bias.cuda()).float().cpu().numpy()
    cfg0 = synth.custom_config(2, 2, (2, 16, 16), block_q=128, topk_ratio=0.25, marginal_ratio=0.0, cfg_id=101)
    r = pu.oracle_head(cfg0, q, k, v, 1, 1, W, bias)
    assert r["o_linear"] is None
    pu.check_output(out0[1, 1], r["out"], "no marginal")


def test_all_critical_small_is_close_to_dense_attention():
    # the isolated dense quantised path (every block critical) at a size the CPU does in full
    cfg = synth.custom_config(1, 2, (4, 16, 32), block_q=128, topk_ratio=1.0, marginal_ratio=0.0,
                              use_proj=False, cfg_id=2)
    q, k, v = synth.make_qkv(cfg)
    out = sla.sla_attention_fwd(*pu.to_dev(q, k, v), 128, 64, 1.0, 0.0).float().cpu().numpy()
    for h in range(2):
        Q, K, V = (synth.as_f64(t[0, h]) for t in (q, k, v))
        ref = pu.oracle_head(cfg, q, k, v, 0, h)["out"]
        pu.check_output(out[0, h], ref, "dense-quant head %d" % h)
        S = Q @ K.T / math.sqrt(cfg.d)
        P = np.exp(S - S.max(1, keepdims=True))
        dense = (P / P.sum(1, keepdims=True)) @ V
        assert pu.cosine(out[0, h], dense) > 0.999


def test_deterministic_and_inputs_untouched():
    cfg = synth.CONFIGS[0]
    q, k, v = pu.to_dev(*synth.make_qkv(cfg))
    W = synth.make_proj(cfg).cuda()
    q0, k0, v0 = q.clone(), k.clone(), v.clone()
    ws = sla.alloc_workspace(1, cfg.H, cfg.N, cfg.d, 64, 64, 0.2, 0.4)
    a = sla.sla_attention_fwd(q, k, v, 64, 64, 0.2, 0.4, proj_w=W, workspace=ws).clone()
    ws.fill_(0xFF)       # workspace contents before a call are undefined: poison them
    b = sla.sla_attention_fwd(q, k, v, 64, 64, 0.2, 0.4, proj_w=W, workspace=ws)
    assert torch.equal(a, b)
    assert torch.equal(q, q0) and torch.equal(k, k0) and torch.equal(v, v0)


@pytest.mark.parametrize("case", [(2, (5, 10, 20), 64, 0.2, 0.4), (3, (3, 27, 27), 128, 0.1, 0.2)])
def test_token_major_and_packed_layouts_give_the_same_bits(case):
    """The strided entry point on [B,N,H,d] tensors and on one packed [B,N,3,H,d] buffer (what
    a fused QKV projection writes), writing a token-major output: identical, bit for bit, to
    the contiguous call on the same values -- and that one is checked against the oracle."""
    H, grid, bq, rc, rm = case
    cfg = synth.custom_config(2, H, grid, block_q=bq, topk_ratio=rc, marginal_ratio=rm, cfg_id=102)
    q, k, v = pu.make_qkv_threaded(cfg)
    W = synth.make_proj(cfg).cuda()
    qd, kd, vd = pu.to_dev(q, k, v)
    B, N, d = cfg.B, cfg.N, cfg.d
    ref = sla.sla_attention_fwd(qd, kd, vd, cfg.block_q, cfg.block_k, rc, rm, proj_w=W)
    r = pu.oracle_head(cfg, q, k, v, 1, H - 1, synth.make_proj(cfg))
    pu.check_output(ref[1, H - 1].float().cpu().numpy(), r["out"], "contiguous reference")

    # [B,N,H,d] inputs and output
    tm = [t.permute(0, 2, 1, 3).contiguous() for t in (qd, kd, vd)]
    out_tm = torch.full((B, N, H, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    sla.sla_attention_fwd_strided(*[t.permute(0, 2, 1, 3) for t in tm], out_tm.permute(0, 2, 1, 3),
                                  cfg.block_q, cfg.block_k, rc, rm, proj_w=W)
    assert torch.equal(out_tm.permute(0, 2, 1, 3), ref)

    # one packed [B,N,3,H,d] buffer; output into a wider buffer whose other columns must stay untouched
    packed = torch.stack(tm, dim=2).contiguous()
    views = [packed[:, :, i].permute(0, 2, 1, 3) for i in range(3)]
    wide = torch.full((B, N, 2, H, d), 7.0, dtype=torch.bfloat16, device="cuda")
    sla.sla_attention_fwd_strided(*views, wide[:, :, 1].permute(0, 2, 1, 3), cfg.block_q, cfg.block_k, rc, rm,
                                  proj_w=W)
    assert torch.equal(wide[:, :, 1].permute(0, 2, 1, 3), ref)
    assert (wide[:, :, 0] == 7.0).all()
    torch.cuda.synchronize()


@pytest.mark.parametrize("H,grid,bq,rc,rm,proj,phi", [
    (2, (5, 10, 20), 128, 0.25, 0.5, True, "softmax"),     # N = 1000, ragged in both block sizes
    (2, (5, 10, 20), 64, 0.2, 0.4, True, "elu1"),
    (1, (3, 27, 27), 128, 0.1, 0.2, False, "relu"),        # N = 2187, identity projection
    (1, (1, 9, 9), 128, 0.5, 0.5, True, "softmax"),        # N = 81: one ragged query block
    (1, (1, 5, 5), 64, 1.0, 0.0, False, "softmax"),        # N = 25: dense attention, no linear term
])
def test_unquantised_forward_matches_oracle(H, grid, bq, rc, rm, proj, phi):
    """quant_mode SLA_QUANT_NONE (the operator the backward pass differentiates): bf16 products with
    fp32 accumulation against the oracle's exact branch, on the library's own mask.  The bar of the
    low-bit path (max-abs 2e-2, cosine 0.999) applies; the only roundings here are P, the summaries
    and the output to bf16 (relative step 2^-9: up to 8e-3 on outputs of magnitude 4, which the bias
    brings about), so the relative Frobenius error is asserted too, at 5e-3."""
    cfg = _cfg(H, grid, bq, rc, rm, proj=proj, cid=400)
    q, k, v = synth.make_qkv(cfg)
    W = synth.make_proj(cfg) if proj else None
    bias = synth.make_qkv(cfg, seed=3)[0][0, 0, 0].contiguous() if proj else None   # 128 bf16 values
    qd, kd, vd, Wd, bd = pu.to_dev(q, k, v, W, bias)
    kind = {"softmax": sla.PHI_SOFTMAX, "elu1": sla.PHI_ELU1, "relu": sla.PHI_RELU}[phi]
    out = sla.sla_attention_fwd(qd, kd, vd, bq, 64, rc, rm, proj_w=Wd, proj_b=bd, phi_kind=kind,
                                quant_mode=sla.QUANT_NONE)
    mask = sla.sla_classify_blocks(qd, kd, bq, 64, rc, rm, want_scores=False)[0].cpu().numpy()
    torch.cuda.synchronize()
    for h in range(H):
        r = so.sla_forward_head(synth.as_f64(q[0, h]), synth.as_f64(k[0, h]), synth.as_f64(v[0, h]), bq, 64, rc, rm,
                                proj_w=None if W is None else synth.as_f64(W),
                                proj_b=None if bias is None else synth.as_f64(bias), phi=phi,
                                quant=so.QUANT_NONE, mask=mask[0, h])
        got = out[0, h].float().cpu().numpy().astype(np.float64)
        pu.check_output(got, r["out"], "unquantised forward head %d" % h)
        assert np.linalg.norm(got - r["out"]) / np.linalg.norm(r["out"]) <= 5e-3


@pytest.mark.parametrize("mode", ["none", "qk_int8"])
def test_sixteen_bit_forward_takes_token_major_layouts(mode):
    """The strided entry point with SLA_QUANT_NONE / SLA_QUANT_QK_INT8 on [B,N,H,d] memory and on one packed
    [B,N,3,H,d] buffer, token-major output: bit-identical to the contiguous call (which is oracle-checked above)."""
    cfg = _cfg(3, (3, 27, 27), 128, 0.1, 0.2, cid=411)
    cfg = synth.custom_config(2, 3, (3, 27, 27), block_q=128, topk_ratio=0.1, marginal_ratio=0.2, cfg_id=411)
    q, k, v = pu.to_dev(*pu.make_qkv_threaded(cfg))
    W = synth.make_proj(cfg).cuda()
    qm = sla.QUANT_NONE if mode == "none" else sla.QUANT_QK_INT8
    ref = sla.sla_attention_fwd(q, k, v, 128, 64, 0.1, 0.2, proj_w=W, quant_mode=qm)
    B, H, N, d = q.shape
    packed = torch.stack([t.permute(0, 2, 1, 3) for t in (q, k, v)], dim=2).contiguous()      # [B,N,3,H,d]
    views = [packed[:, :, i].permute(0, 2, 1, 3) for i in range(3)]
    out_tm = torch.full((B, N, H, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    ws = sla.alloc_workspace(B, H, N, d, 128, 64, 0.1, 0.2, quant_mode=qm)
    sla.sla_attention_fwd_strided(*views, out_tm.permute(0, 2, 1, 3), 128, 64, 0.1, 0.2, proj_w=W, quant_mode=qm, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(out_tm.permute(0, 2, 1, 3), ref)


@pytest.mark.parametrize("H,grid,bq,rc,rm,proj,phi", [
    (2, (4, 16, 16), 64, 0.2, 0.4, True, "softmax"),       # the tiny named shape
    (2, (5, 10, 20), 128, 0.25, 0.5, True, "softmax"),     # N = 1000, ragged in both block sizes
    (1, (3, 27, 27), 128, 0.1, 0.2, False, "elu1"),        # N = 2187, identity projection
    (1, (1, 9, 9), 128, 0.5, 0.5, True, "relu"),           # N = 81: one ragged query block
    (1, (1, 5, 5), 64, 1.0, 0.0, False, "softmax"),        # N = 25: every block critical, no linear term
])
def test_int8_scores_mode_matches_oracle(H, grid, bq, rc, rm, proj, phi):
    """quant_mode SLA_QUANT_QK_INT8 (INT8 Q.K^T with K-smoothing, 16-bit P and V) against the oracle's mode of
    the same name, on the library's own mask: nothing is rounded to the 8-bit float here, so what is left
    against the oracle is bf16 (P, the summaries, the output) -- the bar of the unquantised forward -- and
    the distance to the exact branch is the INT8 error alone, smaller than the full low-bit path's."""
    cfg = _cfg(H, grid, bq, rc, rm, proj=proj, cid=410)
    q, k, v = synth.make_qkv(cfg)
    W = synth.make_proj(cfg) if proj else None
    qd, kd, vd, Wd = pu.to_dev(q, k, v, W)
    kind = {"softmax": sla.PHI_SOFTMAX, "elu1": sla.PHI_ELU1, "relu": sla.PHI_RELU}[phi]
    out8 = sla.sla_attention_fwd(qd, kd, vd, bq, 64, rc, rm, proj_w=Wd, phi_kind=kind, quant_mode=sla.QUANT_QK_INT8)
    out88 = sla.sla_attention_fwd(qd, kd, vd, bq, 64, rc, rm, proj_w=Wd, phi_kind=kind)
    mask = sla.sla_classify_blocks(qd, kd, bq, 64, rc, rm, want_scores=False)[0].cpu().numpy()
    torch.cuda.synchronize()
    for h in range(H):
        args = (synth.as_f64(q[0, h]), synth.as_f64(k[0, h]), synth.as_f64(v[0, h]), bq, 64, rc, rm)
        kw = dict(proj_w=None if W is None else synth.as_f64(W), phi=phi, mask=mask[0, h])
        ref = so.sla_forward_head(*args, quant=so.QUANT_QK_INT8, **kw)["out"]
        exact = so.sla_forward_head(*args, quant=so.QUANT_NONE, **kw)["out"]
        got = out8[0, h].float().cpu().numpy().astype(np.float64)
        pu.check_output(got, ref, "INT8-scores mode, head %d" % h)
        assert np.linalg.norm(got - ref) / np.linalg.norm(ref) <= 5e-3
        full = out88[0, h].float().cpu().numpy().astype(np.float64)
        assert np.linalg.norm(got - exact) <= np.linalg.norm(full - exact)     # INT8 alone errs less than INT8 + FP8


def test_counted_copy_waits_agree_with_full_waits():
    """The attention kernel waits for its asynchronous K/V copies by hand-counted `vmcnt` values.  A
    second build of the library (-DSLA_FULL_WAITS) waits for every copy at each step instead; the two
    must agree bit for bit (tiny named shape, a ragged one with query blocks of 128, one of 64)."""
    import ctypes
    import os
    from paper_2512_16093_amd import build as b
    assert os.path.exists(b.LIB_FULL_WAITS), "run python -m paper_2512_16093_amd.build"
    L = ctypes.CDLL(b.LIB_FULL_WAITS)
    c_int, c_dbl, c_vp, c_sz = ctypes.c_int, ctypes.c_double, ctypes.c_void_p, ctypes.c_size_t
    L.sla_attention_fwd.restype = c_int
    L.sla_attention_fwd.argtypes = [c_vp] * 4 + [c_int] * 6 + [c_dbl, c_dbl, c_vp, c_vp, c_int, c_int, c_vp, c_sz, c_vp]
    for cfg in (synth.CONFIGS[0], _cfg(2, (5, 10, 20), 128, 0.25, 0.5), _cfg(1, (3, 27, 27), 128, 0.1, 0.2),
                _cfg(2, (6, 7, 25), 64, 0.2, 0.4)):
        q, k, v = pu.to_dev(*synth.make_qkv(cfg))
        W = synth.make_proj(cfg).cuda()
        ws = sla.alloc_workspace(cfg.B, cfg.H, cfg.N, cfg.d, cfg.block_q, cfg.block_k, cfg.topk_ratio, cfg.marginal_ratio)
        ref = sla.sla_attention_fwd(q, k, v, cfg.block_q, cfg.block_k, cfg.topk_ratio, cfg.marginal_ratio, proj_w=W, workspace=ws)
        out = torch.empty_like(ref)
        st = L.sla_attention_fwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), cfg.B, cfg.H, cfg.N, cfg.d,
                                 cfg.block_q, cfg.block_k, cfg.topk_ratio, cfg.marginal_ratio, W.data_ptr(), None, 0,
                                 sla.QUANT_QK_INT8_PV_FP8, ws.data_ptr(), ws.numel(),
                                 torch.cuda.current_stream().cuda_stream)
        assert st == 0
        torch.cuda.synchronize()
        assert torch.equal(out, ref), cfg.name


def test_prepass_and_attend_give_the_bits_of_the_single_call():
    """sla_fwd_prepass + sla_fwd_attend (here on token-major memory, with a bias, the second call enqueued on the
    same stream later) against sla_attention_fwd on the same values."""
    cfg = synth.custom_config(2, 3, (3, 27, 27), block_q=128, topk_ratio=0.1, marginal_ratio=0.2, cfg_id=412)
    q, k, v = pu.to_dev(*pu.make_qkv_threaded(cfg))
    W = synth.make_proj(cfg).cuda()
    bias = torch.linspace(-0.5, 0.5, cfg.d).to(torch.bfloat16).cuda()
    ref = sla.sla_attention_fwd(q, k, v, 128, 64, 0.1, 0.2, proj_w=W, proj_b=bias)
    tm = [t.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3) for t in (q, k, v)]
    out = torch.full((cfg.B, cfg.N, cfg.H, cfg.d), float("nan"), dtype=torch.bfloat16, device="cuda").permute(0, 2, 1, 3)
    ws = sla.alloc_workspace(cfg.B, cfg.H, cfg.N, cfg.d, 128, 64, 0.1, 0.2)
    ws.fill_(0xFF)
    sla.sla_fwd_prepass(*tm, 128, 64, 0.1, 0.2, ws, proj_w=W)
    torch.cuda.synchronize()                      # (anything may run in between; the workspace holds the state)
    sla.sla_fwd_attend(tm[0], out, 128, 64, 0.1, 0.2, ws, proj_b=bias)
    torch.cuda.synchronize()
    assert torch.equal(out, ref)


def test_forward_can_be_captured_in_a_graph_and_replayed():
    """The forward call only enqueues kernels (no allocation, no synchronisation, clearing by a kernel), so it can
    be recorded into a HIP graph: three replays on fresh inputs, with eager calls and synchronisations in between,
    give the bits of the eager call every time."""
    cfg = _cfg(2, (5, 10, 20), 128, 0.25, 0.5, cid=440)
    W = synth.make_proj(cfg).cuda()
    args = (cfg.block_q, cfg.block_k, cfg.topk_ratio, cfg.marginal_ratio)
    qd, kd, vd = pu.to_dev(*synth.make_qkv(cfg, seed=9))
    ws = sla.alloc_workspace(cfg.B, cfg.H, cfg.N, cfg.d, *args)
    ws_eager = sla.alloc_workspace(cfg.B, cfg.H, cfg.N, cfg.d, *args)
    out = torch.empty_like(qd)
    sla.sla_attention_fwd(qd, kd, vd, *args, proj_w=W, workspace=ws, out=out)     # (first call outside the capture)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        sla.sla_attention_fwd(qd, kd, vd, *args, proj_w=W, workspace=ws, out=out)
    for seed in (0, 1, 2):
        q, k, v = pu.to_dev(*synth.make_qkv(cfg, seed=seed))
        qd.copy_(q); kd.copy_(k); vd.copy_(v)
        out.zero_()
        graph.replay()
        torch.cuda.synchronize()
        eager = sla.sla_attention_fwd(q, k, v, *args, proj_w=W, workspace=ws_eager)
        torch.cuda.synchronize()
        assert torch.equal(out, eager), "replay %d differs from the eager call" % seed
