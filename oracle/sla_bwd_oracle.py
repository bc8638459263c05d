"""Float64 oracle of the backward pass of Sparse-Linear Attention (SLA), the
operator that the paper's training stage finetunes with (Section 1.2: full
attention is replaced by SLA and the model is finetuned).  TEST INFRASTRUCTURE
ONLY (see oracle/__init__.py).

The paper states no formula.  The result has a plain definition, and this file
is that definition written out: the gradient of the unquantised forward pass

    O = O^s + O^l W^T (+ b)

(sla_oracle.sparse_branch_exact and sla_oracle.linear_branch; training uses
plain SLA, the low-bit core is swapped in for inference only, Section 1.3) with
respect to Q, K, V, W and b, for a given upstream gradient dO and with the block
mask held fixed (the Top-K choice is piecewise constant in Q and K, so it passes
no gradient).  Each step below is one application of the chain rule to one line
of the forward pass; nothing is tiled, fused or reordered.

Pinned (tests/test_oracle_bwd.py): central finite differences of the forward
oracle, an autograd run over a forward pass written a different way (dense
token-level masking), the dense-attention special case against the library's
attention routine, and the identities the forward pass implies (shift
invariances of both softmaxes, linearity in V).
"""
from __future__ import annotations

import math

import numpy as np

from . import sla_oracle as so


def feature_map_grad(X, PX, dP, kind="softmax"):
    """Gradient with respect to X of phi applied row-wise, given PX = phi(X) and dP = dLoss/dPX."""
    if kind == "softmax":
        return PX * (dP - (PX * dP).sum(axis=1, keepdims=True))
    if kind == "elu1":
        return dP * np.where(X > 0, 1.0, np.exp(np.minimum(X, 0.0)))
    if kind == "relu":
        return dP * (X > 0)
    raise ValueError(kind)


def _sample_plan(mask, value, q_blocks, k_blocks):
    """Which query blocks a sampled evaluation has to visit: those asked for, plus every one whose
    mask row holds `value` at one of the key blocks asked for.  None, None = all of them."""
    if q_blocks is None and k_blocks is None:
        return None
    need = set(int(i) for i in (q_blocks or []))
    for j in (k_blocks or []):
        need.update(int(i) for i in np.flatnonzero(mask[:, j] == value))
    return need


def _keep_sampled(dQ, dK, dV, q_blocks, k_blocks, qs, ks):
    """NaN everywhere except the sampled rows (a partial sum elsewhere is not a gradient)."""
    keep_q, keep_k = np.zeros(dQ.shape[0], bool), np.zeros(dK.shape[0], bool)
    for i in (q_blocks or []):
        keep_q[qs[i]] = True
    for j in (k_blocks or []):
        keep_k[ks[j]] = True
    dQ[~keep_q] = np.nan
    dK[~keep_k] = np.nan
    dV[~keep_k] = np.nan


def sparse_branch_grad(Q, K, V, dO, mask, block_q, block_k, q_blocks=None, k_blocks=None):
    """Gradient of sparse_branch_exact: (dQ, dK, dV, lse, delta) with
    lse[n] = log sum_t exp(Q[n].K[t]/sqrt(d)) over the critical keys of n and
    delta[n] = dO[n] . O^s[n] (the two per-row statistics a tiled backward keeps).
    With q_blocks / k_blocks (lists) only dQ of those query blocks and dK, dV of those key blocks
    are evaluated (the same steps, over the query blocks that contribute to them); the rest is NaN."""
    N, d = Q.shape
    qs, ks = so.block_slices(N, block_q), so.block_slices(N, block_k)
    dQ, dK, dV = np.zeros_like(Q), np.zeros_like(K), np.zeros_like(V)
    lse, delta = np.full(N, -np.inf), np.zeros(N)
    scale = 1.0 / math.sqrt(d)
    plan = _sample_plan(mask, 1, q_blocks, k_blocks)
    for i, rows in enumerate(qs):
        if plan is not None and i not in plan:
            continue
        crit = np.flatnonzero(mask[i] == 1)
        if crit.size == 0:
            continue
        keys = np.concatenate([np.arange(ks[j].start, ks[j].stop) for j in crit])
        S = Q[rows] @ K[keys].T * scale
        m = S.max(axis=1, keepdims=True)
        E = np.exp(S - m)
        l = E.sum(axis=1, keepdims=True)
        P = E / l
        O = P @ V[keys]
        lse[rows] = (m + np.log(l))[:, 0]
        delta[rows] = (dO[rows] * O).sum(axis=1)
        dP = dO[rows] @ V[keys].T                     # O = P V
        dS = P * (dP - delta[rows][:, None])          # softmax over the keys of a row
        dQ[rows] += dS @ K[keys] * scale              # S = Q K^T / sqrt(d)
        np.add.at(dK, keys, dS.T @ Q[rows] * scale)
        np.add.at(dV, keys, P.T @ dO[rows])
    if plan is not None:
        _keep_sampled(dQ, dK, dV, q_blocks, k_blocks, qs, ks)
    return dQ, dK, dV, lse, delta


def linear_branch_grad(Q, K, V, dOl, mask, block_q, block_k, phi="softmax", q_blocks=None, k_blocks=None):
    """Gradient of linear_branch for an upstream gradient dOl = dLoss/dO^l: (dQ, dK, dV);
    q_blocks / k_blocks as in sparse_branch_grad."""
    N, d = Q.shape
    qs, ks = so.block_slices(N, block_q), so.block_slices(N, block_k)
    PQ, PK = so.feature_map(Q, phi), so.feature_map(K, phi)
    h, z = so.linear_summaries(K, V, block_k, phi)
    dh, dz = np.zeros_like(h), np.zeros_like(z)
    dPQ = np.zeros_like(PQ)
    plan = _sample_plan(mask, 0, q_blocks, k_blocks)
    for i, rows in enumerate(qs):
        if plan is not None and i not in plan:
            continue
        marg = np.flatnonzero(mask[i] == 0)
        if marg.size == 0:
            continue                                   # O^l is the constant 0 there
        H, Z = h[marg].sum(axis=0), z[marg].sum(axis=0)
        a = PQ[rows]
        num, den = a @ H, a @ Z
        Ol = num / den[:, None]
        dnum = dOl[rows] / den[:, None]                # O^l = num / den
        dden = -(dOl[rows] * Ol).sum(axis=1) / den
        dPQ[rows] = dnum @ H.T + dden[:, None] * Z[None, :]
        dh[marg] += (a.T @ dnum)[None]                 # H and Z are plain sums over the marginal blocks
        dz[marg] += (a.T @ dden)[None]
    dQ = feature_map_grad(Q, PQ, dPQ, phi)
    dPK, dV = np.zeros_like(PK), np.zeros_like(V)
    for j, rows in enumerate(ks):
        dPK[rows] = V[rows] @ dh[j].T + dz[j][None, :]  # h_j = phi(K_j)^T V_j, z_j = column sums of phi(K_j)
        dV[rows] = PK[rows] @ dh[j]
    dK = feature_map_grad(K, PK, dPK, phi)
    if plan is not None:
        _keep_sampled(dQ, dK, dV, q_blocks, k_blocks, qs, ks)
    return dQ, dK, dV


def sla_backward_head(Q, K, V, dO, mask, block_q, block_k, proj_w=None, has_bias=False, phi="softmax",
                      linear=True, q_blocks=None, k_blocks=None):
    """Backward of sla_forward_head(..., quant="none", mask=mask) for one (batch, head) slice.

    Returns a dict: dQ, dK, dV [N, d]; dW [d, d] and db [d] (zeros when the linear term is absent;
    dW is None when proj_w is None, db is None unless has_bias); lse, delta (sparse-branch row
    statistics); o_linear (what dW contracts dO with).  With q_blocks / k_blocks: dQ of those query
    blocks and dK, dV of those key blocks only (NaN elsewhere), no dW, db."""
    N, d = Q.shape
    sampled = q_blocks is not None or k_blocks is not None
    dQ, dK, dV, lse, delta = sparse_branch_grad(Q, K, V, dO, mask, block_q, block_k, q_blocks, k_blocks)
    out = {"lse": lse, "delta": delta, "dW": None, "db": None, "o_linear": None}
    if linear and bool((mask == 0).any()):
        W = None if proj_w is None else np.asarray(proj_w, dtype=np.float64)
        dOl = dO if W is None else dO @ W              # term = O^l W^T (+ b)
        if not sampled:
            Ol = so.linear_branch(Q, K, V, mask, block_q, block_k, phi)
            if W is not None:
                out["dW"] = dO.T @ Ol
            if has_bias:
                out["db"] = dO.sum(axis=0)
            out["o_linear"] = Ol
        lq, lk, lv = linear_branch_grad(Q, K, V, dOl, mask, block_q, block_k, phi, q_blocks, k_blocks)
        dQ, dK, dV = dQ + lq, dK + lk, dV + lv
    elif not sampled:
        if proj_w is not None:
            out["dW"] = np.zeros((d, d))
        if has_bias:
            out["db"] = np.zeros(d)
    out.update(dQ=dQ, dK=dK, dV=dV)
    return out
