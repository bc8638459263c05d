"""Pins for the SLA oracle (CPU only): textbook reductions, brute force on tiny
inputs, closed-form cases and invariants.  None of these re-type the oracle's
own formula; each one is chosen so that a dropped term, wrong index, wrong sign
or transposed operand in oracle/sla_oracle.py fails it.
"""
import math

import numpy as np
import pytest
import scipy.special

from oracle import brute, formats
from oracle import sla_oracle as so
from paper_2512_16093_amd import synth


def _rand_bf16(rng, shape, scale=1.0, bias=None):
    x = rng.standard_normal(shape) * scale
    if bias is not None:
        x = x + bias
    return formats.bf16_round(x.astype(np.float32))


def _tiny(seed=0, H=1):
    cfg = synth.CONFIGS[0]
    q, k, v = synth.make_head(cfg, 0, seed % cfg.H, seed=seed)
    return cfg, synth.as_f64(q), synth.as_f64(k), synth.as_f64(v)


# ---- block counts -----------------------------------------------------------
def test_block_counts_at_named_configs():
    # Top-K ratio 0.1 must leave at least 90 % of the key blocks out (Section 2.1).
    assert so.block_counts(1024, 64, 64, 0.2, 0.4) == (16, 16, 3, 6)
    assert so.block_counts(32760, 128, 64, 0.1, 0.2) == (256, 512, 51, 102)
    assert so.block_counts(75600, 128, 64, 0.1, 0.2) == (591, 1182, 118, 236)
    assert so.block_counts(32760, 128, 64, 1.0, 0.0) == (256, 512, 512, 0)
    for N in (64, 100, 1000, 75600):
        Tq, Tk, n_c, n_m = so.block_counts(N, 128, 64, 0.1, 0.2)
        assert 1 <= n_c and n_c <= max(1, 0.1 * Tk) and n_c + n_m <= Tk
    assert so.block_counts(64, 64, 64, 0.001, 0.0)[2] == 1      # never empty
    assert so.block_counts(640, 64, 64, 0.5, 0.9)[3] == 5       # marginal clipped to what is left


# ---- dense reduction (anchor) ----------------------------------------------
@pytest.mark.parametrize("N,bq,bk", [(256, 64, 64), (300, 128, 64), (1000, 64, 32), (2048, 128, 64)])
def test_all_critical_no_quant_is_dense_softmax_attention(N, bq, bk):
    rng = np.random.default_rng(N)
    d = 32
    Q, K, V = (_rand_bf16(rng, (N, d)) for _ in range(3))
    r = so.sla_forward_head(Q, K, V, bq, bk, 1.0, 0.0, quant=so.QUANT_NONE)
    ref = scipy.special.softmax(Q @ K.T / math.sqrt(d), axis=1) @ V
    assert np.abs(r["out"] - ref).max() < 1e-12
    assert (r["mask"] == 1).all() and r["o_linear"] is None


def test_quantised_all_critical_close_to_dense():
    # Not a parity pin: the low-bit branch must still be an attention.
    rng = np.random.default_rng(5)
    N, d = 512, 128
    Q, V = _rand_bf16(rng, (N, d)), _rand_bf16(rng, (N, d))
    K = _rand_bf16(rng, (N, d), bias=2 * rng.standard_normal(d))
    ref = scipy.special.softmax(Q @ K.T / math.sqrt(d), axis=1) @ V
    for mode, tol in ((so.QUANT_QK_INT8, 1.5e-2), (so.QUANT_QK_INT8_PV_FP8, 3e-2)):
        out = so.sla_forward_head(Q, K, V, 128, 64, 1.0, 0.0, quant=mode)["out"]
        cos = (out * ref).sum() / np.linalg.norm(out) / np.linalg.norm(ref)
        assert np.abs(out - ref).max() < tol and cos > 0.999


# ---- brute force ------------------------------------------------------------
@pytest.mark.parametrize("N,d,bq,bk,rc,rm,proj", [
    (64, 8, 16, 16, 0.25, 0.5, False), (100, 8, 32, 16, 0.3, 0.3, True),
    (192, 16, 32, 32, 0.2, 0.4, True), (250, 16, 32, 16, 0.1, 0.2, False),
    (90, 8, 16, 32, 0.34, 0.66, True)])
def test_matches_scalar_brute_force(N, d, bq, bk, rc, rm, proj):
    rng = np.random.default_rng(N + d)
    Q, K, V = (_rand_bf16(rng, (N, d), 1.5) for _ in range(3))
    W = _rand_bf16(rng, (d, d), 0.3) if proj else None
    b = _rand_bf16(rng, (d,), 0.3) if proj else None
    Tq, Tk, n_c, n_m = so.block_counts(N, bq, bk, rc, rm)
    r = so.sla_forward_head(Q, K, V, bq, bk, rc, rm, proj_w=W, proj_b=b, quant=so.QUANT_NONE)
    ref, ref_mask = brute.brute_sla(Q.tolist(), K.tolist(), V.tolist(), bq, bk, n_c, n_m,
                                    None if W is None else W.tolist(), None if b is None else b.tolist())
    assert np.array_equal(r["mask"], np.array(ref_mask, dtype=np.int8))
    assert np.abs(r["out"] - np.array(ref)).max() < 1e-12


# ---- brute force of the low-bit sparse branch --------------------------------
_QCASES = [(64, 8, 16, 16, 0.25), (100, 8, 32, 16, 0.3), (192, 16, 32, 32, 0.2), (250, 16, 32, 16, 0.1),
           (90, 8, 16, 32, 0.34), (150, 128, 64, 32, 0.4)]


def _quant_case(N, d, bq, bk, rc):
    rng = np.random.default_rng(7 * N + d)
    Q, V = (_rand_bf16(rng, (N, d), 1.5) for _ in range(2))
    K = _rand_bf16(rng, (N, d), 1.5, bias=2 * rng.standard_normal(d))     # outlier channels, as K-smoothing expects
    Tq, Tk, n_c, n_m = so.block_counts(N, bq, bk, rc, 0.3)
    mask = so.classify(so.pooled_scores(Q, K, bq, bk), n_c, n_m)
    return Q, K, V, mask


@pytest.mark.parametrize("N,d,bq,bk,rc", _QCASES)
@pytest.mark.parametrize("reference", ["ceil_log2", "running"])
@pytest.mark.parametrize("ref_tile", [None, 16])
def test_quantised_branch_matches_scalar_brute_force(N, d, bq, bk, rc, reference, ref_tile):
    # Second statement of the whole low-bit branch: token by token, Python round() for the integer
    # codes, the 8-bit float as the nearest entry of its value table (ties to the even code).
    Q, K, V, mask = _quant_case(N, d, bq, bk, rc)
    for mode, fp8 in ((so.QUANT_QK_INT8_PV_FP8, True), (so.QUANT_QK_INT8, False)):
        for rq in ((True, False) if d <= 16 else (True,)):
            out, lse = so.sparse_branch_quant(Q, K, V, mask, bq, bk, mode=mode, reference=reference, ref_tile=ref_tile,
                                              rowsum_quantized=rq, return_lse=True)
            ref, ref_lse = brute.brute_sparse_quant(Q.tolist(), K.tolist(), V.tolist(), mask.tolist(), bq, bk, pv_fp8=fp8,
                                                    reference=reference, ref_tile=ref_tile, rowsum_quantized=rq)
            assert np.abs(out - np.array(ref)).max() < 1e-12
            assert np.abs(lse - np.array(ref_lse)).max() < 1e-12


def test_brute_force_notices_misplaced_rounding(monkeypatch):
    # The pin has teeth: each of these slips inside the low-bit branch moves the result far
    # beyond 1e-12 of the scalar restatement (which does not go through oracle.formats).
    Q, K, V, mask = _quant_case(100, 8, 32, 16, 0.3)
    ref = np.array(brute.brute_sparse_quant(Q.tolist(), K.tolist(), V.tolist(), mask.tolist(), 32, 16)[0])
    assert np.abs(so.sparse_branch_quant(Q, K, V, mask, 32, 16) - ref).max() < 1e-12
    # (a) V used unrounded  (b) P not rounded  (c) truncation instead of nearest-even for the integer codes
    real_round = formats.e4m3_round
    calls = {"n": 0}

    def v_unrounded(x):
        calls["n"] += 1
        return np.asarray(x, dtype=np.float64) if calls["n"] == 1 else real_round(x)   # first call = V
    monkeypatch.setattr(formats, "e4m3_round", v_unrounded)
    assert np.abs(so.sparse_branch_quant(Q, K, V, mask, 32, 16) - ref).max() > 1e-6
    calls["n"] = 0

    def p_unrounded(x):
        calls["n"] += 1
        return real_round(x) if calls["n"] == 1 else np.asarray(x, dtype=np.float64)
    monkeypatch.setattr(formats, "e4m3_round", p_unrounded)
    assert np.abs(so.sparse_branch_quant(Q, K, V, mask, 32, 16) - ref).max() > 1e-6
    monkeypatch.setattr(formats, "e4m3_round", real_round)
    monkeypatch.setattr(formats, "int8_codes",
                        lambda x, amax: np.clip(np.trunc(np.asarray(x) * 127.0 / amax), -127, 127))
    assert np.abs(so.sparse_branch_quant(Q, K, V, mask, 32, 16) - ref).max() > 1e-6


def test_brute_e4m3_is_the_published_format():
    # every table value survives, midpoints go to the even code, the top saturates
    vals = brute._E4M3
    assert len(vals) == 127 and vals[0] == 0.0 and vals[1] == 2.0 ** -9 and vals[8] == 2.0 ** -6 and vals[-1] == 448.0
    for c, v in enumerate(vals):
        assert brute.brute_e4m3(v) == v and brute.brute_e4m3(-v) == -v
    for c in range(126):
        mid = (vals[c] + vals[c + 1]) / 2
        assert brute.brute_e4m3(mid) == vals[c if c % 2 == 0 else c + 1]
    assert brute.brute_e4m3(1e9) == 448.0 and brute.brute_e4m3(-465.0) == -448.0
    xs = np.random.default_rng(0).uniform(-500, 500, 4000)
    assert np.array_equal(np.array([brute.brute_e4m3(float(x)) for x in xs]), formats.e4m3_round(xs))


# ---- classification ---------------------------------------------------------
def test_classification_closed_form_ranking():
    # Every key block is a constant multiple c_j of one vector u, every query block
    # is the vector u: the score of block j is c_j |u|^2 / sqrt(d), so the ranking
    # is the ranking of c_j (ties -> lower index).
    d, bk = 8, 4
    u = np.array([1, -2, 0.5, 3, -1, 2, 0.25, -0.5])
    c = np.array([0.5, 3.0, -1.0, 3.0, 2.0, 0.0, 2.5, -2.0])   # blocks 1 and 3 tie
    K = np.repeat(c, bk)[:, None] * u[None, :]
    Q = np.tile(u, (len(c) * bk, 1))
    mask = so.classify(so.pooled_scores(Q, K, 8, bk), 3, 2)
    expect = np.array([-1, 1, -1, 1, 0, -1, 1, -1])    # top3: 1,3 (tie, both in),6; next 2: 4, 0
    expect[0] = 0
    assert (mask == expect[None, :]).all()
    mask2 = so.classify(so.pooled_scores(Q, K, 8, bk), 1, 1)
    assert mask2[0, 1] == 1 and mask2[0, 3] == 0      # tie broken by lower index


def test_classification_invariants_on_synthetic():
    cfg, Q, K, V = _tiny()
    Tq, Tk, n_c, n_m = so.block_counts(cfg.N, cfg.block_q, cfg.block_k, cfg.topk_ratio, cfg.marginal_ratio)
    s = so.pooled_scores(Q, K, cfg.block_q, cfg.block_k)
    mask = so.classify(s, n_c, n_m)
    assert ((mask == 1).sum(1) == n_c).all() and ((mask == 0).sum(1) == n_m).all()
    for i in range(Tq):
        assert s[i][mask[i] == 1].min() >= s[i][mask[i] == 0].max()
        assert s[i][mask[i] == 0].min() >= s[i][mask[i] == -1].max()
    # the row softmax of the pooled scores is a distribution with the same ranking
    P = scipy.special.softmax(s, axis=1)
    assert np.allclose(P.sum(1), 1.0)
    assert np.array_equal(so.classify(P, n_c, n_m), mask)
    # adding one constant vector to every key shifts each row by a constant
    shift = np.linspace(-1, 1, cfg.d)
    s2 = so.pooled_scores(Q, K + shift, cfg.block_q, cfg.block_k)
    assert np.allclose((s2 - s).std(axis=1), 0, atol=1e-12)
    crit, marg = so.mask_lists(mask)
    assert crit.shape == (Tq, n_c) and marg.shape == (Tq, n_m)
    assert (np.diff(crit, axis=1) > 0).all() and (np.diff(marg, axis=1) > 0).all()


def test_ragged_pooling_divides_by_valid_count():
    X = np.arange(10, dtype=np.float64)[:, None] * np.ones((1, 3))
    p = so.pool_blocks(X, 4)
    assert np.allclose(p[:, 0], [1.5, 5.5, 8.5])


# ---- sparse branch semantics -----------------------------------------------
@pytest.mark.parametrize("quant", [so.QUANT_NONE, so.QUANT_QK_INT8_PV_FP8])
def test_skipped_blocks_contribute_nothing(quant):
    cfg, Q, K, V = _tiny()
    V = V.copy()
    V[0, :] = 8.0        # pins every channel's global scale to a token that stays put
    r = so.sla_forward_head(Q, K, V, 64, 64, 0.2, 0.4, quant=quant, linear=False)
    mask = r["mask"]
    # a key block that no row marks critical can hold anything; poison V there,
    # and (exact mode, where K has no global statistic) K too
    unused = np.flatnonzero((mask != 1).all(axis=0))
    unused = unused[unused != 0]
    assert unused.size > 0
    K2, V2 = K.copy(), V.copy()
    for j in unused:
        V2[j * 64:(j + 1) * 64] = np.nan
        if quant == so.QUANT_NONE:
            K2[j * 64:(j + 1) * 64] = np.nan
    if quant != so.QUANT_NONE:
        # V's per-channel scale is global: poison within the pinned range instead of NaN
        for j in unused:
            V2[j * 64:(j + 1) * 64] = -7.5
    r2 = so.sla_forward_head(Q, K2, V2, 64, 64, 0.2, 0.4, quant=quant, linear=False, mask=mask)
    if quant == so.QUANT_NONE:
        assert np.array_equal(r["out"], r2["out"])
    else:
        assert np.abs(V2).max(0).tolist() == np.abs(V).max(0).tolist()
        assert np.array_equal(r["out"], r2["out"])


def test_softmax_weights_sum_to_one_over_critical_keys():
    # With V = 1 in channel 0 the branch returns the sum of its softmax weights;
    # with V = indicator of one key block it returns that block's share.
    cfg, Q, K, _ = _tiny()
    mask = so.classify(so.pooled_scores(Q, K, 64, 64), 3, 6)
    V = np.zeros_like(K)
    V[:, 0] = 1.0
    V[5 * 64:6 * 64, 1] = 1.0
    o = so.sparse_branch_exact(Q, K, V, mask, 64, 64)
    assert np.allclose(o[:, 0], 1.0, atol=1e-13)
    rows_without = np.repeat(mask[:, 5] != 1, 64)
    assert (o[rows_without, 1] == 0).all() and (o[~rows_without, 1] > 0).all()
    for ref in ("ceil_log2", "running"):
        oq = so.sparse_branch_quant(Q, K, V, mask, 64, 64, so.QUANT_QK_INT8, reference=ref)
        assert np.allclose(oq[:, 0], 1.0, atol=1e-12)          # unrounded P: exact normalisation
        o8 = so.sparse_branch_quant(Q, K, V, mask, 64, 64, so.QUANT_QK_INT8_PV_FP8, reference=ref,
                                    rowsum_quantized=False)
        assert np.abs(o8[:, 0] - 1.0).max() < 2.0 ** -4          # FP8 P vs unrounded sum: one rounding step
        o8q = so.sparse_branch_quant(Q, K, V, mask, 64, 64, so.QUANT_QK_INT8_PV_FP8, reference=ref)
        assert np.allclose(o8q[:, 0], 1.0, atol=1e-12)         # sum of the rounded P: exact again


def test_key_block_permutation_invariance_exact():
    cfg, Q, K, V = _tiny()
    mask = so.classify(so.pooled_scores(Q, K, 64, 64), 3, 6)
    perm = np.random.default_rng(0).permutation(16)
    tok = (perm[:, None] * 64 + np.arange(64)[None, :]).ravel()
    o1 = so.sparse_branch_exact(Q, K, V, mask, 64, 64) + so.linear_branch(Q, K, V, mask, 64, 64)
    o2 = so.sparse_branch_exact(Q, K[tok], V[tok], mask[:, perm], 64, 64) \
        + so.linear_branch(Q, K[tok], V[tok], mask[:, perm], 64, 64)
    assert np.abs(o1 - o2).max() < 1e-12


def test_k_smoothing_is_invisible_without_rounding():
    # Subtracting a constant vector from every key shifts each query's logits by
    # a constant, which softmax removes.
    cfg, Q, K, V = _tiny()
    mask = so.classify(so.pooled_scores(Q, K, 64, 64), 3, 6)
    o1 = so.sparse_branch_exact(Q, K, V, mask, 64, 64)
    o2 = so.sparse_branch_exact(Q, K - K.mean(0), V, mask, 64, 64)
    assert np.abs(o1 - o2).max() < 1e-12


def test_k_smoothing_helps_with_channel_bias():
    cfg, Q, K, V = _tiny()
    mask = so.classify(so.pooled_scores(Q, K, 64, 64), 3, 6)
    ex = so.sparse_branch_exact(Q, K, V, mask, 64, 64)
    e_s = np.abs(so.sparse_branch_quant(Q, K, V, mask, 64, 64, so.QUANT_QK_INT8, smooth_k=True) - ex).mean()
    e_n = np.abs(so.sparse_branch_quant(Q, K, V, mask, 64, 64, so.QUANT_QK_INT8, smooth_k=False) - ex).mean()
    assert e_s < e_n


def test_online_softmax_equals_two_pass_when_nothing_is_rounded(monkeypatch):
    # Take the rounding out of the quantised branch (identity codes): what is left
    # is the online-softmax recurrence, which must equal the exact branch.
    cfg, Q, K, V = _tiny()
    mask = so.classify(so.pooled_scores(Q, K, 64, 64), 3, 6)
    monkeypatch.setattr(formats, "int8_codes", lambda x, amax: np.asarray(x) * 127.0 / amax)
    monkeypatch.setattr(formats, "e4m3_round", lambda x: np.asarray(x, dtype=np.float64))
    ex = so.sparse_branch_exact(Q, K, V, mask, 64, 64)
    for ref in ("running", "ceil_log2"):
        for rq in (False, True):
            oq, lse = so.sparse_branch_quant(Q, K, V, mask, 64, 64, so.QUANT_QK_INT8_PV_FP8, return_lse=True,
                                             reference=ref, rowsum_quantized=rq)
            assert np.abs(oq - ex).max() < 1e-11
    # log-sum-exp of the smoothed logits over the critical keys
    Kt = K - K.mean(0)
    i = 3
    keys = np.concatenate([np.arange(j * 64, (j + 1) * 64) for j in np.flatnonzero(mask[i] == 1)])
    ref = scipy.special.logsumexp(Q[i * 64:(i + 1) * 64] @ Kt[keys].T / math.sqrt(cfg.d), axis=1)
    assert np.abs(lse[i * 64:(i + 1) * 64] - ref).max() < 1e-10


def test_int8_codes_and_score_error_bound():
    cfg, Q, K, V = _tiny()
    Q8, dq = so.quantize_q(Q, 64)
    K8, dk, mu = so.quantize_k(K, 64)
    assert np.allclose(mu, K.mean(0))
    for c in (Q8, K8):
        assert (c == np.rint(c)).all() and np.abs(c).max() == 127
    Kt = K - mu
    assert np.abs(Q8 * np.repeat(dq, 64)[:, None] - Q).max() <= dq.max() / 2 + 1e-12
    assert np.abs(K8 * np.repeat(dk, 64)[:, None] - Kt).max() <= dk.max() / 2 + 1e-12
    # each block's largest magnitude maps to code +-127
    for j in range(16):
        assert np.abs(K8[j * 64:(j + 1) * 64]).max() == 127
    # |dS| <= dq/2 sum|K~| + dk/2 sum|Q| + d dq dk / 4  (row-wise, before 1/sqrt(d))
    i, j = 2, 7
    Sq = (Q8[i * 64:(i + 1) * 64] @ K8[j * 64:(j + 1) * 64].T) * dq[i] * dk[j]
    Se = Q[i * 64:(i + 1) * 64] @ Kt[j * 64:(j + 1) * 64].T
    bound = dq[i] / 2 * np.abs(Kt[j * 64:(j + 1) * 64]).sum(1)[None, :] \
        + dk[j] / 2 * np.abs(Q[i * 64:(i + 1) * 64]).sum(1)[:, None] + cfg.d * dq[i] * dk[j] / 4
    assert (np.abs(Sq - Se) <= bound + 1e-9).all()
    # integer dot products are exact in float64
    prod = Q8[i * 64:(i + 1) * 64].astype(np.int64) @ K8[j * 64:(j + 1) * 64].astype(np.int64).T
    assert np.array_equal(prod, Q8[i * 64:(i + 1) * 64] @ K8[j * 64:(j + 1) * 64].T)


def test_v_quantisation_is_per_channel_fp8():
    cfg, Q, K, V = _tiny()
    V8, dv = so.quantize_v(V)
    assert np.allclose(dv, np.abs(V).max(0) / 448)
    assert np.abs(V8).max() == 448 and np.array_equal(formats.e4m3_round(V8), V8)
    assert (np.abs(V8 * dv - V) <= 2.0 ** -4 * np.abs(V) + dv * 2.0 ** -10).all()
    Z8, dz = so.quantize_v(np.zeros((8, 4)))
    assert (dz == 1).all() and (Z8 == 0).all()


# ---- linear branch -----------------------------------------------------------
def test_linear_branch_single_marginal_block_is_textbook_linear_attention():
    # Two key blocks; the top-1 block is critical, the other is marginal for every
    # row.  Make block 1 marginal for all rows by construction and compare with
    # unblocked linear attention over exactly those keys.
    rng = np.random.default_rng(11)
    N, d = 128, 16
    Q, K, V = (_rand_bf16(rng, (N, d)) for _ in range(3))
    mask = np.array([[1, 0]] * 4, dtype=np.int8)         # 4 query blocks of 32, 2 key blocks of 64
    o = so.linear_branch(Q, K, V, mask, 32, 64)
    pq = scipy.special.softmax(Q, axis=1)
    pk = scipy.special.softmax(K[64:], axis=1)
    ref = (pq @ (pk.T @ V[64:])) / (pq @ pk.sum(0))[:, None]
    assert np.abs(o - ref).max() < 1e-13
    # all blocks marginal == linear attention over every key
    mask0 = np.zeros((4, 2), dtype=np.int8)
    pk = scipy.special.softmax(K, axis=1)
    ref0 = (pq @ (pk.T @ V)) / (pq @ pk.sum(0))[:, None]
    assert np.abs(so.linear_branch(Q, K, V, mask0, 32, 64) - ref0).max() < 1e-13


def test_linear_branch_is_a_weighted_mean_of_values():
    cfg, Q, K, V = _tiny()
    mask = so.classify(so.pooled_scores(Q, K, 64, 64), 3, 6)
    o = so.linear_branch(Q, K, V, mask, 64, 64)
    for i in range(16):
        keys = np.concatenate([np.arange(j * 64, (j + 1) * 64) for j in np.flatnonzero(mask[i] == 0)])
        lo, hi = V[keys].min(0), V[keys].max(0)
        blk = o[i * 64:(i + 1) * 64]
        assert (blk >= lo - 1e-12).all() and (blk <= hi + 1e-12).all()
    # changing a marginal block's V moves only the linear term
    j = int(np.flatnonzero((mask == 0).any(0) & (mask != 1).all(0))[0])
    V2 = V.copy()
    V2[j * 64:(j + 1) * 64] += 1.0
    assert np.array_equal(so.sparse_branch_exact(Q, K, V, mask, 64, 64), so.sparse_branch_exact(Q, K, V2, mask, 64, 64))
    assert not np.allclose(so.linear_branch(Q, K, V2, mask, 64, 64), o)
    for kind in ("softmax", "elu1", "relu"):
        assert (so.feature_map(Q, kind) >= 0).all()
    assert np.allclose(so.feature_map(Q, "softmax").sum(1), 1.0)
    x = np.array([[-1.0, 0.0, 2.0]])
    assert np.allclose(so.feature_map(x, "elu1"), [[math.exp(-1), 1.0, 3.0]])
    assert np.allclose(so.feature_map(x, "relu"), [[0.0, 0.0, 2.0]])


def test_projection_identity_zero_and_bias():
    cfg, Q, K, V = _tiny()
    kw = dict(block_q=64, block_k=64, topk_ratio=0.2, marginal_ratio=0.4, quant=so.QUANT_NONE)
    r = so.sla_forward_head(Q, K, V, **kw)
    assert np.array_equal(r["out"], r["o_sparse"] + r["o_linear"])
    rI = so.sla_forward_head(Q, K, V, proj_w=np.eye(cfg.d), **kw)
    assert np.abs(rI["out"] - r["out"]).max() < 1e-14
    r0 = so.sla_forward_head(Q, K, V, proj_w=np.zeros((cfg.d, cfg.d)), **kw)
    assert np.array_equal(r0["out"], r0["o_sparse"])
    # W is [out, in]: a W that copies input channel 1 into output channel 0
    W = np.zeros((cfg.d, cfg.d))
    W[0, 1] = 1.0
    rW = so.sla_forward_head(Q, K, V, proj_w=W, proj_b=np.arange(cfg.d, dtype=np.float64), **kw)
    assert np.allclose(rW["out"][:, 0], r["o_sparse"][:, 0] + r["o_linear"][:, 1])
    assert np.allclose(rW["out"][:, 5], r["o_sparse"][:, 5] + 5.0)
    # no marginal blocks: no linear term, no bias
    rn = so.sla_forward_head(Q, K, V, 64, 64, 0.2, 0.0, proj_b=np.ones(cfg.d), quant=so.QUANT_NONE)
    assert np.array_equal(rn["out"], rn["o_sparse"])


def test_q_block_subset_matches_full_run():
    cfg, Q, K, V = _tiny()
    W = synth.as_f64(synth.make_proj(cfg))
    full = so.sla_forward_head(Q, K, V, 64, 64, 0.2, 0.4, proj_w=W)["out"]
    part = so.sla_forward_head(Q, K, V, 64, 64, 0.2, 0.4, proj_w=W, q_blocks=[1, 15])["out"]
    assert np.array_equal(part[64:128], full[64:128]) and np.array_equal(part[-64:], full[-64:])
    assert np.isnan(part[:64]).all()


def test_quantised_sla_tracks_exact_sla_on_tiny_config():
    cfg = synth.CONFIGS[0]
    W = synth.as_f64(synth.make_proj(cfg))
    for h in range(cfg.H):
        q, k, v = (synth.as_f64(t) for t in synth.make_head(cfg, 0, h))
        ex = so.sla_forward_head(q, k, v, 64, 64, 0.2, 0.4, proj_w=W, quant=so.QUANT_NONE)["out"]
        lo = so.sla_forward_head(q, k, v, 64, 64, 0.2, 0.4, proj_w=W)["out"]
        cos = (ex * lo).sum() / np.linalg.norm(ex) / np.linalg.norm(lo)
        assert cos > 0.999 and np.abs(ex - lo).max() < 5e-2


def test_oracle_reproduces_its_stored_tiny_outputs():
    # Regression guard only (the stored values are the oracle's own, written by
    # tests/golden/make_golden.py): flags an unintended change of its arithmetic.
    import importlib.util
    import json
    import os
    here = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(here, "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    with open(os.path.join(here, "tiny_sla_oracle.json")) as f:
        stored = json.load(f)
    live = mod.build()
    for hs, hl in zip(stored["heads"], live["heads"]):
        assert hs["mask"] == hl["mask"]
        for key in (so.QUANT_NONE, so.QUANT_QK_INT8, so.QUANT_QK_INT8_PV_FP8, "scores_row0"):
            assert np.allclose(np.array(hs[key]), np.array(hl[key]), rtol=0, atol=1e-12)


def test_integer_reference_keeps_every_rescale_a_power_of_two():
    # With the ceil reference the largest scaled probability of a row is in (1/2, 1]
    # and the two reference rules agree to within the FP8 rounding they both apply.
    cfg, Q, K, V = _tiny()
    mask = so.classify(so.pooled_scores(Q, K, 64, 64), 3, 6)
    a = so.sparse_branch_quant(Q, K, V, mask, 64, 64, reference="ceil_log2")
    b = so.sparse_branch_quant(Q, K, V, mask, 64, 64, reference="running")
    assert np.abs(a - b).max() < 2e-2 and (a * b).sum() / np.linalg.norm(a) / np.linalg.norm(b) > 0.9995
    ex = so.sparse_branch_exact(Q, K, V, mask, 64, 64)
    ea, eb = np.abs(a - ex).mean(), np.abs(b - ex).mean()
    assert ea < 1.5 * eb          # no worse than the plain running maximum, on average


def test_reference_refresh_tile_changes_only_the_rounding():
    # Refreshing the running reference every 32 keys instead of once per 64-key block is the
    # same computation before rounding (online softmax is exact for any blocking) ...
    cfg, Q, K, V = _tiny()
    mask = so.classify(so.pooled_scores(Q, K, 64, 64), 3, 6)
    a = so.sparse_branch_quant(Q, K, V, mask, 64, 64, so.QUANT_QK_INT8)
    b = so.sparse_branch_quant(Q, K, V, mask, 64, 64, so.QUANT_QK_INT8, ref_tile=32)
    assert np.abs(a - b).max() < 1e-12
    c = so.sparse_branch_quant(Q, K, V, mask, 64, 64, so.QUANT_QK_INT8, ref_tile=16, reference="running")
    assert np.abs(a - c).max() < 1e-12
    # ... and with FP8 P only moves where the codes round: both stay equally close to the exact branch
    a8, la = so.sparse_branch_quant(Q, K, V, mask, 64, 64, return_lse=True)
    b8, lb = so.sparse_branch_quant(Q, K, V, mask, 64, 64, return_lse=True, ref_tile=32)
    assert np.abs(a8 - b8).max() < 2e-2 and np.abs(la - lb).max() < 2e-2
    ex = so.sparse_branch_exact(Q, K, V, mask, 64, 64)
    ea, eb = np.abs(a8 - ex).mean(), np.abs(b8 - ex).mean()
    assert eb < 1.25 * ea and ea < 1.25 * eb
    # a tile equal to the block is the default
    assert np.array_equal(a8, so.sparse_branch_quant(Q, K, V, mask, 64, 64, ref_tile=64))


def test_the_two_readings_are_equally_close_to_exact():
    # The kernel-shaped switches (integer reference level, refreshed per 32 keys, row sum of the rounded
    # weights) against the plain reading (running maximum per 64-key block, unrounded row sum): the two
    # differ only in where P is rounded to the 8-bit float, so each is as far from the exact branch as the
    # other, and they are no further from each other than from it.
    cfg = synth.CONFIGS[0]
    for h in range(cfg.H):
        q, k, v = synth.make_head(cfg, 0, h, seed=0)
        Q, K, V = synth.as_f64(q), synth.as_f64(k), synth.as_f64(v)
        args = (Q, K, V, cfg.block_q, cfg.block_k, cfg.topk_ratio, cfg.marginal_ratio)
        a = so.sla_forward_head(*args, ref_tile=32)["out"]
        b = so.sla_forward_head(*args, reference="running", rowsum_quantized=False, ref_tile=None)["out"]
        e = so.sla_forward_head(*args, quant=so.QUANT_NONE)["out"]
        rms = lambda x: float(np.sqrt((x ** 2).mean()))
        assert 0.85 < rms(a - e) / rms(b - e) < 1.15
        assert rms(a - b) <= max(rms(a - e), rms(b - e))
        assert np.abs(a - b).max() <= 3e-2 and np.abs(a - e).max() <= 3.5e-2 and np.abs(b - e).max() <= 3.5e-2
        cos = (a * b).sum() / np.linalg.norm(a) / np.linalg.norm(b)
        assert cos >= 0.9999
