"""Float64 oracle of the Sparse-Linear Attention (SLA) forward pass with the
low-bit sparse branch.  TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

What the paper fixes (Section 1.1, Section 1.3, Section 2.1): attention is
SLA -- a block-sparse softmax branch plus a linear-attention branch -- built
on a SageAttention2++-style low-bit core, with a Top-K ratio (0.1 in the
experiments) choosing the blocks that get exact softmax attention.  The paper
states no equation for either method; every step below follows the readings
listed in this repository's design notes (block means -> scores -> three-way
block mask -> online softmax over critical blocks with K-smoothing, per-block
INT8 QK^T and FP8 PV -> linear attention over marginal blocks -> projection).

Conventions: one (batch, head) slice at a time; Q, K, V are float64 arrays
[N, d] holding bf16-representable values; blocks are consecutive runs of
block_q / block_k tokens, the last one possibly shorter.  No tiling, fusion or
reordering beyond what the steps state.

Pins (tests/test_oracle_sla.py): all-critical + no quantisation against dense
softmax attention from a library; the exact mode and the low-bit sparse branch
(both reference rules, both refresh intervals, both row sums, both low-bit
modes) against the scalar-loop restatement in oracle/brute.py; formats against
library conversions, code rounding at exact ties against rational arithmetic
(tests/test_oracle_formats.py); closed-form rankings; textbook linear attention;
invariants.  Parity unpinned by the paper itself (no outside value exists; the
readings define them): the choice of feature map, the meaning of "marginal",
the projection form, and which of the equivalent-before-rounding variants of
the low-bit pass (reference rule, refresh interval, row sum) is "the" scheme.
"""
from __future__ import annotations

import math

import numpy as np

from . import formats

QUANT_NONE = "none"
QUANT_QK_INT8 = "qk_int8"
QUANT_QK_INT8_PV_FP8 = "qk_int8_pv_fp8"

P_SCALE = formats.E4M3_MAX  # static scale that maps P~ in [0, 1] onto the E4M3 range


# --------------------------------------------------------------------------
# Block bookkeeping
# --------------------------------------------------------------------------
def block_counts(N, block_q, block_k, topk_ratio, marginal_ratio):
    """(Tq, Tk, n_c, n_m): block grid and per-row critical / marginal counts.

    Section 2.1: a Top-K ratio of 0.1 corresponds to 90 % sparsity, so the
    critical count is the floor of ratio * Tk (never rounding sparsity below
    the stated figure), at least one so the softmax is never empty."""
    Tq = -(-N // block_q)
    Tk = -(-N // block_k)
    n_c = min(Tk, max(1, int(math.floor(topk_ratio * Tk + 1e-9))))
    n_m = min(Tk - n_c, int(math.floor(marginal_ratio * Tk + 1e-9)))
    return Tq, Tk, n_c, n_m


def block_slices(N, block):
    """Token ranges of consecutive blocks; the last may be short."""
    return [slice(s, min(s + block, N)) for s in range(0, N, block)]


# --------------------------------------------------------------------------
# Steps 1-2: pooled scores and the three-way block mask
# --------------------------------------------------------------------------
def pool_blocks(X, block):
    """Mean over the valid tokens of each block, per channel: [T, d]."""
    return np.stack([X[s].mean(axis=0) for s in block_slices(X.shape[0], block)])


def pooled_scores(Q, K, block_q, block_k):
    """s[i, j] = mean(Q block i) . mean(K block j) / sqrt(d)."""
    d = Q.shape[1]
    return pool_blocks(Q, block_q) @ pool_blocks(K, block_k).T / math.sqrt(d)


def classify(scores, n_c, n_m):
    """Mask [Tq, Tk] int8: +1 critical (top n_c scores of the row), 0 marginal
    (next n_m), -1 negligible.  Equal scores rank by ascending block index.
    (Ranking the pre-softmax score equals ranking its row softmax.)"""
    Tq, Tk = scores.shape
    mask = np.full((Tq, Tk), -1, dtype=np.int8)
    for i in range(Tq):
        order = np.lexsort((np.arange(Tk), -scores[i]))  # by -score, then index
        mask[i, order[:n_c]] = 1
        mask[i, order[n_c:n_c + n_m]] = 0
    return mask


def mask_lists(mask):
    """Ascending index lists of the critical and marginal blocks of each row."""
    crit = np.stack([np.flatnonzero(r == 1) for r in mask]).astype(np.int32)
    marg = np.stack([np.flatnonzero(r == 0) for r in mask]).astype(np.int32)
    return crit, marg


# --------------------------------------------------------------------------
# Step 3: quantisation of the sparse branch's operands
# --------------------------------------------------------------------------
def quantize_k(K, block_k, smooth=True):
    """K-smoothing then per-block symmetric INT8.

    mu = channel mean of K over all N tokens; K~ = K - mu; per block
    delta_j = max|K~_j| / 127 (1 if the block is all zero); codes are
    clip(rint(K~ / delta_j), -127, 127), the quotient taken as 127 K~ / max|K~_j|
    (formats.int8_codes: exact ties stay ties).  Returns (codes [N, d] as float64
    integers, delta [Tk], mu [d])."""
    N, d = K.shape
    mu = K.mean(axis=0) if smooth else np.zeros(d)
    Kt = K - mu
    codes = np.empty_like(Kt)
    sl = block_slices(N, block_k)
    delta = np.empty(len(sl))
    for j, s in enumerate(sl):
        amax = np.abs(Kt[s]).max()
        delta[j] = amax / formats.INT8_MAX if amax > 0 else 1.0
        codes[s] = formats.int8_codes(Kt[s], amax)
    return codes, delta, mu


def quantize_q(Q, block_q):
    """Per-block symmetric INT8 of Q (no smoothing): (codes [N, d], delta [Tq])."""
    N = Q.shape[0]
    codes = np.empty_like(Q)
    sl = block_slices(N, block_q)
    delta = np.empty(len(sl))
    for i, s in enumerate(sl):
        amax = np.abs(Q[s]).max()
        delta[i] = amax / formats.INT8_MAX if amax > 0 else 1.0
        codes[s] = formats.int8_codes(Q[s], amax)
    return codes, delta


def quantize_v(V, fp8=True):
    """Per-channel scale over all tokens, delta[c] = max_n |V[n, c]| / 448 (1 if
    zero); returns (V / delta rounded to E4M3 if fp8 else unrounded, delta [d]).
    The quotient is taken as 448 V / max|V| (the product is exact for 16-bit inputs), so
    that a value exactly half way between two E4M3 values is rounded as the tie it is
    instead of by the last bit of the rounded scale."""
    amax = np.abs(V).max(axis=0)
    delta = np.where(amax > 0, amax / formats.E4M3_MAX, 1.0)
    Vs = np.where(amax > 0, V * formats.E4M3_MAX / np.where(amax > 0, amax, 1.0), V)
    return (formats.e4m3_round(Vs) if fp8 else Vs), delta


# --------------------------------------------------------------------------
# Step 4: sparse softmax branch
# --------------------------------------------------------------------------
def sparse_branch_exact(Q, K, V, mask, block_q, block_k, q_blocks=None):
    """O^s[n] = sum over keys t in the critical blocks of n's query block of
    softmax_t(Q[n].K[t]/sqrt(d)) V[t].  Rows of blocks not in q_blocks are NaN."""
    N, d = Q.shape
    qs, ks = block_slices(N, block_q), block_slices(N, block_k)
    out = np.full((N, V.shape[1]), np.nan)
    for i in (range(len(qs)) if q_blocks is None else q_blocks):
        keys = np.concatenate([np.arange(ks[j].start, ks[j].stop) for j in np.flatnonzero(mask[i] == 1)])
        S = Q[qs[i]] @ K[keys].T / math.sqrt(d)
        P = np.exp(S - S.max(axis=1, keepdims=True))
        out[qs[i]] = (P / P.sum(axis=1, keepdims=True)) @ V[keys]
    return out


def sparse_branch_quant(Q, K, V, mask, block_q, block_k, mode=QUANT_QK_INT8_PV_FP8,
                        q_blocks=None, smooth_k=True, rowsum_quantized=True,
                        reference="ceil_log2", return_lse=False, ref_tile=None):
    """Low-bit sparse branch: one pass over the critical blocks in ascending
    block order with a running reference level per query row.

    Per query block i (scale dq_i) and critical key block j (scale dk_j), with
    t = log2(e) * S the logits in base-2 units:
      S  = (Q8_i . K8_j^T) dq_i dk_j / sqrt(d)         integer product, exact
      r' = max(r, ref(rowmax t));  a = 2^(r - r')       running reference
      P~ = 2^(t - r')  in (0, 1];  P8 = e4m3(448 P~)    (mode qk_int8: unrounded)
      l  = a l + rowsum(P8)/448;   acc = a acc + P8 . V8_j
    and O^s = acc * dv / (448 l).  The row constant Q.mu removed by K-smoothing
    cancels in the softmax, so it is never added back.

    reference = "ceil_log2": ref(x) = ceil(x), an integer, so every rescale
    factor a is a power of two and the largest P~ of a row lies in (1/2, 1];
    reference = "running": ref(x) = x, the plain running maximum (largest P~ = 1).
    rowsum_quantized = False sums the unrounded P~ instead of P8/448.
    ref_tile = T (a divisor of block_k) refreshes the running reference after
    every T keys of a critical block instead of once per block (the default,
    T = block_k): the pass then treats each run of T keys as a block of its own.
    All these alternatives give the same result before rounding."""
    if mode == QUANT_NONE:
        raise ValueError("use sparse_branch_exact for mode 'none'")
    N, d = Q.shape
    qs, ks = block_slices(N, block_q), block_slices(N, block_k)
    Q8, dq = quantize_q(Q, block_q)
    K8, dk, _ = quantize_k(K, block_k, smooth=smooth_k)
    V8, dv = quantize_v(V, fp8=(mode == QUANT_QK_INT8_PV_FP8))
    out = np.full((N, V.shape[1]), np.nan)
    lse = np.full(N, np.nan)
    log2e = 1.0 / math.log(2.0)
    for i in (range(len(qs)) if q_blocks is None else q_blocks):
        rows = qs[i].stop - qs[i].start
        r = np.full(rows, -np.inf)
        l = np.zeros(rows)
        acc = np.zeros((rows, V.shape[1]))
        for j in np.flatnonzero(mask[i] == 1):
            S_blk = (Q8[qs[i]] @ K8[ks[j]].T) * (dq[i] * dk[j] / math.sqrt(d))
            V_blk = V8[ks[j]]
            keys = S_blk.shape[1]
            tile = keys if ref_tile is None else ref_tile
            for c0 in range(0, keys, tile):
                t = S_blk[:, c0:c0 + tile] * log2e
                tmax = t.max(axis=1)
                r_new = np.maximum(r, np.ceil(tmax) if reference == "ceil_log2" else tmax)
                alpha = np.where(np.isneginf(r), 0.0, np.exp2(r - r_new))
                Pt = np.exp2(t - r_new[:, None])
                P8 = formats.e4m3_round(P_SCALE * Pt) if mode == QUANT_QK_INT8_PV_FP8 else P_SCALE * Pt
                l = alpha * l + (P8.sum(axis=1) / P_SCALE if rowsum_quantized else Pt.sum(axis=1))
                acc = alpha[:, None] * acc + P8 @ V_blk[c0:c0 + tile]
                r = r_new
        out[qs[i]] = acc * dv[None, :] / (P_SCALE * l[:, None])
        lse[qs[i]] = (r + np.log2(l)) * math.log(2.0)
    return (out, lse) if return_lse else out


# --------------------------------------------------------------------------
# Step 5: linear branch over the marginal blocks
# --------------------------------------------------------------------------
def feature_map(X, kind="softmax"):
    """phi applied to each token (row): softmax over the d channels (default),
    elu(x)+1, or relu."""
    if kind == "softmax":
        E = np.exp(X - X.max(axis=1, keepdims=True))
        return E / E.sum(axis=1, keepdims=True)
    if kind == "elu1":
        return np.where(X > 0, X + 1.0, np.exp(np.minimum(X, 0.0)))
    if kind == "relu":
        return np.maximum(X, 0.0)
    raise ValueError(kind)


def linear_summaries(K, V, block_k, phi="softmax"):
    """Per key block j: h_j = phi(K_j)^T V_j  [d, dv]  and  z_j = sum_n phi(K_j[n])  [d]."""
    ks = block_slices(K.shape[0], block_k)
    PK = feature_map(K, phi)
    h = np.stack([PK[s].T @ V[s] for s in ks])
    z = np.stack([PK[s].sum(axis=0) for s in ks])
    return h, z


def linear_branch(Q, K, V, mask, block_q, block_k, phi="softmax", q_blocks=None):
    """O^l[n] = phi(Q[n]) H_i / (phi(Q[n]) . Z_i) with H_i, Z_i the sums of h_j,
    z_j over the marginal blocks (mask == 0) of n's query block; phi sees the
    original (unsmoothed, unquantised) Q and K.  Zero where a row has no
    marginal block."""
    N = Q.shape[0]
    qs = block_slices(N, block_q)
    h, z = linear_summaries(K, V, block_k, phi)
    PQ = feature_map(Q, phi)
    out = np.full((N, V.shape[1]), np.nan)
    for i in (range(len(qs)) if q_blocks is None else q_blocks):
        marg = np.flatnonzero(mask[i] == 0)
        if marg.size == 0:
            out[qs[i]] = 0.0
            continue
        H = h[marg].sum(axis=0)
        Z = z[marg].sum(axis=0)
        out[qs[i]] = (PQ[qs[i]] @ H) / (PQ[qs[i]] @ Z)[:, None]
    return out


# --------------------------------------------------------------------------
# Step 6: whole forward pass
# --------------------------------------------------------------------------
def sla_forward_head(Q, K, V, block_q, block_k, topk_ratio, marginal_ratio,
                     proj_w=None, proj_b=None, phi="softmax", quant=QUANT_QK_INT8_PV_FP8,
                     linear=True, q_blocks=None, mask=None, ref_tile=None,
                     reference="ceil_log2", rowsum_quantized=True):
    """SLA forward of one (batch, head) slice.

    O = O^s + O^l W^T (+ b); W = identity when proj_w is None; the linear term
    (and the bias) is absent when there is no marginal block (n_m = 0) or
    linear=False.  Returns a dict with out [N, d] (NaN rows for query blocks
    outside q_blocks), mask, scores, o_sparse, o_linear.  ref_tile, reference and
    rowsum_quantized are handed to sparse_branch_quant (how often the running
    reference is refreshed, which reference rule, which row sum)."""
    N, d = Q.shape
    Tq, Tk, n_c, n_m = block_counts(N, block_q, block_k, topk_ratio, marginal_ratio)
    scores = pooled_scores(Q, K, block_q, block_k)
    if mask is None:
        mask = classify(scores, n_c, n_m)
    if quant == QUANT_NONE:
        o_s = sparse_branch_exact(Q, K, V, mask, block_q, block_k, q_blocks)
    else:
        o_s = sparse_branch_quant(Q, K, V, mask, block_q, block_k, quant, q_blocks, ref_tile=ref_tile,
                                  reference=reference, rowsum_quantized=rowsum_quantized)
    out = o_s.copy()
    o_l = None
    if linear and n_m > 0:
        o_l = linear_branch(Q, K, V, mask, block_q, block_k, phi, q_blocks)
        term = o_l if proj_w is None else o_l @ np.asarray(proj_w, dtype=np.float64).T
        if proj_b is not None:
            term = term + np.asarray(proj_b, dtype=np.float64)[None, :]
        out = out + term
    return {"out": out, "mask": mask, "scores": scores, "o_sparse": o_s, "o_linear": o_l,
            "n_c": n_c, "n_m": n_m}


def sla_forward(q, k, v, block_q, block_k, topk_ratio, marginal_ratio, **kw):
    """All (b, h) slices of [B, H, N, d] float64 inputs: out [B, H, N, d], mask [B, H, Tq, Tk]."""
    B, H = q.shape[:2]
    outs, masks = [], []
    for b in range(B):
        for h in range(H):
            r = sla_forward_head(q[b, h], k[b, h], v[b, h], block_q, block_k,
                                 topk_ratio, marginal_ratio, **kw)
            outs.append(r["out"])
            masks.append(r["mask"])
    out = np.stack(outs).reshape(B, H, *outs[0].shape)
    mask = np.stack(masks).reshape(B, H, *masks[0].shape)
    return out, mask


def dense_equiv_flops(B, H, N, d):
    """4 B H N^2 d: the flops of dense attention that the method stands in for."""
    return 4.0 * B * H * float(N) * float(N) * d
