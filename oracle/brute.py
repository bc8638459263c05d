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


# ---------------------------------------------------------------------------
# The low-bit sparse branch, scalar by scalar (Section 1.1: 8-bit integer QK^T and
# 8-bit float PV in the SageAttention2++ manner; Section 1.3: SLA on that core).
# Second statement of oracle/sla_oracle.py's quantised branch: one query token and
# one key at a time, Python's own round() for the integer codes, and the 8-bit
# float found as the nearest entry of the table of all its values.
# ---------------------------------------------------------------------------
def _e4m3_values():
    """The 127 non-negative finite values of the 1-4-3 format (exponent bias 7,
    subnormals below 2^-6, code 0x7F is NaN), in code order = ascending order."""
    vals = []
    for code in range(127):
        e, m = code >> 3, code & 7
        vals.append(m / 8.0 * 2.0 ** -6 if e == 0 else (1.0 + m / 8.0) * 2.0 ** (e - 7))
    return vals


_E4M3 = _e4m3_values()


def brute_e4m3(x):
    """Nearest table value to x (ties to the even code), saturating at the largest."""
    a = abs(x)
    if a >= _E4M3[-1]:
        r = _E4M3[-1]
    else:
        hi = next(c for c in range(127) if _E4M3[c] >= a)   # first code at or above a
        if hi == 0 or _E4M3[hi] == a:
            r = _E4M3[hi]
        else:
            lo = hi - 1
            dl, dh = a - _E4M3[lo], _E4M3[hi] - a
            r = _E4M3[lo] if dl < dh else _E4M3[hi] if dh < dl else _E4M3[lo if lo % 2 == 0 else hi]
    return -r if x < 0 else r


def _int8(x, amax):
    """Symmetric 8-bit code at the scale amax / 127, from the quotient 127 x / amax (whose numerator is
    exact for 16-bit inputs, so exact ties are ties): Python's round() is round-half-to-even."""
    return float(max(-127, min(127, round(127.0 * x / amax)))) if amax > 0 else 0.0


def brute_sparse_quant(Q, K, V, mask, block_q, block_k, pv_fp8=True, reference="ceil_log2",
                       ref_tile=None, rowsum_quantized=True, smooth_k=True):
    """Rows of O^s of the low-bit sparse branch and the log-sum-exp of every row.

    Q, K, V: lists of rows; mask: rows of +1 / 0 / -1 per (query block, key block).
    For a query token the keys of its critical blocks are visited in ascending order
    in runs of ref_tile keys (a whole block when None); before each run the
    reference level moves up to the run's largest base-2 logit (rounded up to an
    integer when reference == "ceil_log2"), the sums gathered so far are scaled
    down accordingly, and each weight 448 * 2^(logit - reference) is rounded to the
    8-bit float (pv_fp8) before it multiplies the 8-bit V and joins the row sum
    (the unrounded weight joins it when rowsum_quantized is False)."""
    N, d = len(Q), len(Q[0])
    dv_ = len(V[0])
    Tq, Tk = (N + block_q - 1) // block_q, (N + block_k - 1) // block_k
    mu = [sum(K[n][c] for n in range(N)) / N if smooth_k else 0.0 for c in range(d)]
    K8, dk = [None] * N, []
    for j in range(Tk):
        toks = range(j * block_k, min((j + 1) * block_k, N))
        amax = max(abs(K[n][c] - mu[c]) for n in toks for c in range(d))
        dk.append(amax / 127.0 if amax > 0 else 1.0)
        for n in toks:
            K8[n] = [_int8(K[n][c] - mu[c], amax) for c in range(d)]
    Q8, dq = [None] * N, []
    for i in range(Tq):
        toks = range(i * block_q, min((i + 1) * block_q, N))
        amax = max(abs(Q[n][c]) for n in toks for c in range(d))
        dq.append(amax / 127.0 if amax > 0 else 1.0)
        for n in toks:
            Q8[n] = [_int8(Q[n][c], amax) for c in range(d)]
    dv, vmax = [], []
    for c in range(dv_):
        amax = max(abs(V[n][c]) for n in range(N))
        vmax.append(amax)
        dv.append(amax / 448.0 if amax > 0 else 1.0)
    scaled = lambda n, c: 448.0 * V[n][c] / vmax[c] if vmax[c] > 0 else V[n][c]   # V / dv with an exact numerator
    V8 = [[brute_e4m3(scaled(n, c)) if pv_fp8 else scaled(n, c) for c in range(dv_)] for n in range(N)]

    log2e = 1.0 / math.log(2.0)
    out, lse = [], []
    for n in range(N):
        i = n // block_q
        r, l, acc = None, 0.0, [0.0] * dv_
        for j in range(Tk):
            if mask[i][j] != 1:
                continue
            lo, hi = j * block_k, min((j + 1) * block_k, N)
            step = (hi - lo) if ref_tile is None else ref_tile
            for t0 in range(lo, hi, step):
                run = range(t0, min(t0 + step, hi))
                logit = {t: sum(Q8[n][c] * K8[t][c] for c in range(d)) * (dq[i] * dk[j] / math.sqrt(d)) * log2e
                         for t in run}
                top = max(logit.values())
                cand = float(math.ceil(top)) if reference == "ceil_log2" else top
                r_new = cand if r is None else max(r, cand)
                a = 0.0 if r is None else 2.0 ** (r - r_new)
                l *= a
                acc = [a * x for x in acc]
                for t in run:
                    p = 2.0 ** (logit[t] - r_new)
                    p8 = brute_e4m3(448.0 * p) if pv_fp8 else 448.0 * p
                    l += p8 / 448.0 if rowsum_quantized else p
                    for c in range(dv_):
                        acc[c] += p8 * V8[t][c]
                r = r_new
        out.append([acc[c] * dv[c] / (448.0 * l) for c in range(dv_)])
        lse.append((r + math.log2(l)) * math.log(2.0))
    return out, lse
