"""Pins of the SLA backward oracle (CPU only).  The gradient has a definition outside the
oracle's own formulas: the derivative of the forward oracle.  It is checked here by central
finite differences of that forward pass, by autograd over a forward pass written another way
(token-level dense masking in torch, float64), against the library's dense attention in the
all-critical special case, and through identities the forward pass implies."""
import math

import numpy as np
import pytest
import torch

from oracle import sla_bwd_oracle as bo
from oracle import sla_oracle as so


def _case(N, d, bq, bk, rc, rm, seed, proj=True, bias=True, off_kink=False):
    g = np.random.default_rng(seed)
    Q, K, V, dO = (g.standard_normal((N, d)) for _ in range(4))
    Q *= 1.5   # sharper softmax rows, so P is far from uniform
    if off_kink:   # relu is not differentiable at 0: keep every entry of Q and K at least 0.05 away from it
        Q, K = (X + 0.05 * np.where(X >= 0, 1.0, -1.0) for X in (Q, K))
        Q[:, 0], K[:, 0] = np.abs(Q[:, 0]), np.abs(K[:, 0])   # and one live channel per token, so phi(Q) . Z > 0
    Tq, Tk, n_c, n_m = so.block_counts(N, bq, bk, rc, rm)
    mask = so.classify(so.pooled_scores(Q, K, bq, bk), n_c, n_m)
    W = g.standard_normal((d, d)) / math.sqrt(d) if proj else None
    b = g.standard_normal(d) if bias else None
    return Q, K, V, dO, mask, W, b


CASES = [  # N, d, bq, bk, critical, marginal
    (40, 8, 8, 4, 0.3, 0.4),      # whole blocks
    (45, 8, 16, 8, 0.34, 0.5),    # ragged last query and key block
    (30, 4, 4, 4, 0.25, 0.75),    # no negligible block
]


@pytest.mark.parametrize("phi", ["softmax", "elu1", "relu"])
@pytest.mark.parametrize("N,d,bq,bk,rc,rm", CASES)
def test_matches_central_differences_of_the_forward_oracle(N, d, bq, bk, rc, rm, phi):
    Q, K, V, dO, mask, W, b = _case(N, d, bq, bk, rc, rm, 1, off_kink=(phi == "relu"))

    def loss(Q_, K_, V_, W_, b_):
        out = so.sla_forward_head(Q_, K_, V_, bq, bk, rc, rm, proj_w=W_, proj_b=b_, phi=phi,
                                  quant=so.QUANT_NONE, mask=mask)["out"]
        return float((out * dO).sum())

    g = bo.sla_backward_head(Q, K, V, dO, mask, bq, bk, proj_w=W, has_bias=True, phi=phi)
    rng = np.random.default_rng(2)
    eps = 1e-6
    args = [Q, K, V, W, b]
    for idx, name in enumerate(["dQ", "dK", "dV", "dW", "db"]):
        grad = g[name]
        # a random direction (catches any wrong term) and a few single entries (catch wrong indices)
        probes = [rng.standard_normal(grad.shape)]
        for _ in range(4):
            e = np.zeros(grad.shape)
            e[tuple(rng.integers(0, s) for s in grad.shape)] = 1.0
            probes.append(e)
        for p in probes:
            hi = [a.copy() for a in args]
            lo = [a.copy() for a in args]
            hi[idx] = hi[idx] + eps * p
            lo[idx] = lo[idx] - eps * p
            fd = (loss(*hi) - loss(*lo)) / (2 * eps)
            an = float((grad * p).sum())
            assert abs(fd - an) <= 1e-6 * max(1.0, abs(an)) + 1e-7, (name, fd, an)


def _torch_forward(Q, K, V, mask, bq, bk, W, b, phi):
    """The forward pass once more, written with token-level masks over the whole N x N score
    matrix (no block loops), for autograd."""
    N, d = Q.shape
    rows = torch.arange(N) // bq
    cols = torch.arange(N) // bk
    tok = torch.as_tensor(mask.astype(np.int64))[rows][:, cols]           # [N, N] token-level mask
    S = Q @ K.T / math.sqrt(d)
    P = torch.softmax(S.masked_fill(tok != 1, float("-inf")), dim=1)
    Os = P @ V
    if phi == "softmax":
        fq, fk = torch.softmax(Q, dim=1), torch.softmax(K, dim=1)
    elif phi == "relu":
        fq, fk = torch.relu(Q), torch.relu(K)
    else:
        fq, fk = torch.nn.functional.elu(Q) + 1, torch.nn.functional.elu(K) + 1
    A = (fq @ fk.T) * (tok == 0)                                           # unnormalised linear attention weights
    Ol = (A @ V) / A.sum(dim=1, keepdim=True)
    return Os + Ol @ W.T + b


@pytest.mark.parametrize("phi", ["softmax", "elu1", "relu"])
@pytest.mark.parametrize("N,d,bq,bk,rc,rm", CASES)
def test_matches_autograd_of_a_dense_masked_formulation(N, d, bq, bk, rc, rm, phi):
    Q, K, V, dO, mask, W, b = _case(N, d, bq, bk, rc, rm, 3, off_kink=(phi == "relu"))
    t = [torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (Q, K, V, W, b)]
    out = _torch_forward(*t[:3], mask, bq, bk, t[3], t[4], phi)
    # the two forward passes agree, so the comparison below is about the gradient alone
    ref_out = so.sla_forward_head(Q, K, V, bq, bk, rc, rm, proj_w=W, proj_b=b, phi=phi, quant=so.QUANT_NONE,
                                  mask=mask)["out"]
    assert np.allclose(out.detach().numpy(), ref_out, rtol=1e-11, atol=1e-12)
    out.backward(torch.tensor(dO))
    g = bo.sla_backward_head(Q, K, V, dO, mask, bq, bk, proj_w=W, has_bias=True, phi=phi)
    for name, tt in zip(["dQ", "dK", "dV", "dW", "db"], t):
        ref = tt.grad.numpy()
        assert np.abs(g[name] - ref).max() <= 1e-11 * max(1.0, np.abs(ref).max()), name


def test_all_blocks_critical_is_dense_attention():
    """Every block critical, no linear term: the library's scaled-dot-product attention and its
    autograd give the same output and gradients; lse is the row log-sum-exp of the scores."""
    N, d, bq, bk = 37, 16, 8, 8
    g = np.random.default_rng(4)
    Q, K, V, dO = (g.standard_normal((N, d)) for _ in range(4))
    Tk = (N + bk - 1) // bk
    mask = np.ones(((N + bq - 1) // bq, Tk), dtype=np.int8)
    r = bo.sla_backward_head(Q, K, V, dO, mask, bq, bk, linear=False)
    t = [torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (Q, K, V)]
    out = torch.nn.functional.scaled_dot_product_attention(t[0][None], t[1][None], t[2][None])[0]
    out.backward(torch.tensor(dO))
    for name, tt in zip(["dQ", "dK", "dV"], t):
        assert np.abs(r[name] - tt.grad.numpy()).max() <= 1e-12 * max(1.0, np.abs(tt.grad.numpy()).max()), name
    S = Q @ K.T / math.sqrt(d)
    assert np.allclose(r["lse"], np.log(np.exp(S).sum(axis=1)), rtol=1e-13, atol=0)
    assert np.allclose(r["delta"], (dO * out.detach().numpy()).sum(axis=1), rtol=1e-12, atol=1e-13)
    assert r["dW"] is None and r["db"] is None


def test_identities_the_forward_pass_implies():
    N, d, bq, bk = 48, 8, 8, 4
    Q, K, V, dO, mask, W, b = _case(N, d, bq, bk, 0.25, 0.5, 5)
    # (1) sparse branch alone: adding one vector to every key shifts each score row by a constant,
    #     which softmax ignores -> the key gradients sum to zero over the tokens
    s = bo.sla_backward_head(Q, K, V, dO, mask, bq, bk, linear=False)
    assert np.abs(s["dK"].sum(axis=0)).max() <= 1e-12 * np.abs(s["dK"]).max() * N
    # (2) softmax feature map: adding a constant to all channels of one token changes nothing ->
    #     the linear branch's dQ and dK are orthogonal to the all-ones vector, token by token
    lq, lk, lv = bo.linear_branch_grad(Q, K, V, dO, mask, bq, bk, "softmax")
    assert np.abs(lq.sum(axis=1)).max() <= 1e-13 and np.abs(lk.sum(axis=1)).max() <= 1e-13
    # (3) the output minus the bias is linear in V -> <dV, V> = <dO, O - b>  (Euler)
    full = bo.sla_backward_head(Q, K, V, dO, mask, bq, bk, proj_w=W, has_bias=True)
    out = so.sla_forward_head(Q, K, V, bq, bk, 0.25, 0.5, proj_w=W, proj_b=b, quant=so.QUANT_NONE, mask=mask)["out"]
    assert abs((full["dV"] * V).sum() - (dO * (out - b)).sum()) <= 1e-11 * abs((dO * out).sum()) + 1e-11
    # (4) the linear term is linear in W, the bias enters once per row
    assert np.allclose(full["dW"], dO.T @ full["o_linear"], rtol=1e-13, atol=1e-13)
    assert np.allclose(full["db"], dO.sum(axis=0), rtol=1e-13, atol=1e-13)
    # (5) the two branches add: gradients of the whole = sparse-only + linear-only
    dOl = dO @ W
    assert np.allclose(full["dQ"], s["dQ"] + bo.linear_branch_grad(Q, K, V, dOl, mask, bq, bk)[0], rtol=1e-12, atol=1e-13)
    # (6) a query block without marginal blocks contributes nothing to the linear gradients
    m2 = mask.copy()
    m2[0][m2[0] == 0] = -1
    q2, k2, v2 = bo.linear_branch_grad(Q, K, V, dO, m2, bq, bk)
    assert not q2[:bq].any()
    dO0 = dO.copy()
    dO0[:bq] = 0.0                                  # equivalently: that block's upstream gradient zeroed
    q3, k3, v3 = bo.linear_branch_grad(Q, K, V, dO0, mask, bq, bk)
    assert np.allclose(k2, k3, rtol=1e-12, atol=1e-14) and np.allclose(v2, v3, rtol=1e-12, atol=1e-14)


def test_a_planted_mistake_is_caught():
    """The finite-difference check has teeth: a dropped delta term (a common slip in the softmax
    backward) shows up as a large mismatch."""
    N, d, bq, bk = 32, 8, 8, 4
    Q, K, V, dO, mask, _, _ = _case(N, d, bq, bk, 0.25, 0.0, 6, proj=False, bias=False)
    good = bo.sparse_branch_grad(Q, K, V, dO, mask, bq, bk)[0]

    def loss(Q_):
        return float((so.sparse_branch_exact(Q_, K, V, mask, bq, bk) * dO).sum())

    p = np.random.default_rng(7).standard_normal(Q.shape)
    fd = (loss(Q + 1e-6 * p) - loss(Q - 1e-6 * p)) / 2e-6
    assert abs(fd - (good * p).sum()) <= 1e-6 * max(1.0, abs(fd))
    # the same contraction without delta: P * dP instead of P * (dP - delta)
    qs, ks = so.block_slices(N, bq), so.block_slices(N, bk)
    bad = np.zeros_like(Q)
    for i, rows in enumerate(qs):
        keys = np.concatenate([np.arange(ks[j].start, ks[j].stop) for j in np.flatnonzero(mask[i] == 1)])
        S = Q[rows] @ K[keys].T / math.sqrt(d)
        P = np.exp(S - S.max(axis=1, keepdims=True))
        P /= P.sum(axis=1, keepdims=True)
        bad[rows] = (P * (dO[rows] @ V[keys].T)) @ K[keys] / math.sqrt(d)
    assert abs(fd - (bad * p).sum()) > 1e-3 * max(1.0, abs(fd))


def test_sampled_evaluation_equals_the_full_one_on_the_sampled_blocks():
    N, d, bq, bk = 90, 8, 8, 4
    Q, K, V, dO, mask, W, b = _case(N, d, bq, bk, 0.25, 0.5, 8)
    full = bo.sla_backward_head(Q, K, V, dO, mask, bq, bk, proj_w=W, has_bias=True)
    qb, kb = [1, 7, 11], [0, 9, 22]                      # 11 and 22: the ragged last blocks
    part = bo.sla_backward_head(Q, K, V, dO, mask, bq, bk, proj_w=W, has_bias=True, q_blocks=qb, k_blocks=kb)
    qs, ks = so.block_slices(N, bq), so.block_slices(N, bk)
    for i in range(len(qs)):
        if i in qb:
            assert np.allclose(part["dQ"][qs[i]], full["dQ"][qs[i]], rtol=1e-12, atol=1e-14)
        else:
            assert np.isnan(part["dQ"][qs[i]]).all()
    for j in range(len(ks)):
        for name in ("dK", "dV"):
            if j in kb:
                assert np.allclose(part[name][ks[j]], full[name][ks[j]], rtol=1e-12, atol=1e-14)
            else:
                assert np.isnan(part[name][ks[j]]).all()
    assert part["dW"] is None and part["db"] is None


def test_relu_derivative_switches_exactly_at_zero():
    """The finite-difference pins keep away from relu's kink, so where the derivative switches is pinned apart:
    1 for x > 0, 0 at and below 0 (the one-sided derivative from the left), to the last representable step."""
    X = np.array([[-1.0, -0.005, -np.finfo(np.float64).tiny, 0.0, np.finfo(np.float64).tiny, 0.005, 2.0]])
    dP = np.full_like(X, 3.0)
    got = bo.feature_map_grad(X, np.maximum(X, 0.0), dP, "relu")
    assert np.array_equal(got, np.array([[0.0, 0.0, 0.0, 0.0, 3.0, 3.0, 3.0]]))
    # elu + 1: exp(x) for x <= 0 (continuous at 0 with value 1), 1 above
    got = bo.feature_map_grad(X, None, dP, "elu1")
    assert np.allclose(got, 3.0 * np.array([[np.exp(-1.0), np.exp(-0.005), 1.0, 1.0, 1.0, 1.0, 1.0]]), rtol=1e-15)
