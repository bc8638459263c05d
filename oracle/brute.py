"""Scalar-loop restatement of SLA for tiny inputs.  TEST INFRASTRUCTURE ONLY.

Independent of oracle/sla_oracle.py on purpose: tokens are visited one by one,
nothing is treated as a block matrix, and the linear branch is written in its
quadratic form (a kernel-weighted average over the marginal tokens) rather
than through per-block summaries.  Pure Python floats (IEEE double); use only
for N <= 256, d <= 16.
"""
from __future__ import annotations

import math


def _block_of(n, block):
    return n // block


def _pooled(X, block):
    N, d = len(X), len(X[0])
    T = (N + block - 1) // block
    out = []
    for b in range(T):
        lo, hi = b * block, min((b + 1) * block, N)
        out.append([sum(X[n][c] for n in range(lo, hi)) / (hi - lo) for c in range(d)])
    return out


def brute_mask(Q, K, block_q, block_k, n_c, n_m):
    """Three-way block mask by explicit ranking: block j outranks j' when its
    score is larger, or equal with j < j'."""
    d = len(Q[0])
    qb, kb = _pooled(Q, block_q), _pooled(K, block_k)
    mask = []
    for qi in qb:
        s = [sum(qi[c] * kj[c] for c in range(d)) / math.sqrt(d) for kj in kb]
        row = []
        for j in range(len(kb)):
            rank = sum(1 for jj in range(len(kb)) if s[jj] > s[j] or (s[jj] == s[j] and jj < j))
            row.append(1 if rank < n_c else (0 if rank < n_c + n_m else -1))
        mask.append(row)
    return mask


def _phi_softmax(x):
    m = max(x)
    e = [math.exp(v - m) for v in x]
    s = sum(e)
    return [v / s for v in e]


def brute_sla(Q, K, V, block_q, block_k, n_c, n_m, W=None, bias=None):
    """Exact-arithmetic SLA (no quantisation), softmax feature map.
    Q, K, V: lists of rows.  Returns (out rows, mask)."""
    N, d = len(Q), len(Q[0])
    dv = len(V[0])
    mask = brute_mask(Q, K, block_q, block_k, n_c, n_m)
    phiK = [_phi_softmax(k) for k in K]
    out = []
    for n in range(N):
        i = _block_of(n, block_q)
        # sparse branch: softmax over the tokens of critical blocks
        logits = {}
        for t in range(N):
            if mask[i][_block_of(t, block_k)] == 1:
                logits[t] = sum(Q[n][c] * K[t][c] for c in range(d)) / math.sqrt(d)
        mx = max(logits.values())
        den = sum(math.exp(v - mx) for v in logits.values())
        o = [0.0] * dv
        for t, v in logits.items():
            w = math.exp(v - mx) / den
            for c in range(dv):
                o[c] += w * V[t][c]
        # linear branch: kernel-weighted mean over the tokens of marginal blocks
        if n_m > 0:
            pq = _phi_softmax(Q[n])
            num = [0.0] * dv
            den_l = 0.0
            for t in range(N):
                if mask[i][_block_of(t, block_k)] == 0:
                    w = sum(pq[c] * phiK[t][c] for c in range(d))
                    den_l += w
                    for c in range(dv):
                        num[c] += w * V[t][c]
            ol = [x / den_l for x in num]
            if W is not None:
                ol = [sum(ol[c] * W[r][c] for c in range(dv)) for r in range(len(W))]
            if bias is not None:
                ol = [a + b for a, b in zip(ol, bias)]
            o = [a + b for a, b in zip(o, ol)]
        out.append(o)
    return out, mask
