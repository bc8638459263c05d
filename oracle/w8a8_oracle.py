"""W8A8 Linear layer with block-wise INT8 quantisation, in float64 on the CPU.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py): only tests, the smoke check
and the benchmark's cpu_baseline leg may import this module; it shares no code
with the HIP path.

What the paper fixes (Section 1.1, fourth technique; Section 1.3, "Linear layer
quantization"): weights AND activations of a Linear layer are INT8, the
quantisation granularity of both is a block of 128 x 128, and the product runs
on INT8 matrix units.  Everything else below is this build's reading, the plain
one for symmetric block-wise INT8:

  * a block of a matrix A[R, C] is rows 128 r .. 128 r + 127 and columns
    128 c .. 128 c + 127 (ragged at the edges); its scale is
    s[r, c] = max|A_block| / 127, or 1 if the block is all zero; its codes are
    rint(A_block / s[r, c]) (ties to even), which lie in [-127, 127];
  * for activations X[M, K] (tokens x input features) and weights W[N, K]
    (output x input features), with kb running over the K / 128 feature blocks,

        Y[m, n] = sum_kb  sX[m // 128, kb] * sW[n // 128, kb]
                          * sum_{k in kb} X8[m, k] * W8[n, k]      (+ bias[n]),

    the inner sum exact in integers, the outer one in floating point.
"""
from __future__ import annotations

import numpy as np

from . import formats

BLOCK = 128


def quantize_blockwise(A, block=BLOCK):
    """(codes, scales) of a 2-D array: codes as float64 integers of A's shape,
    scales [ceil(R / block), ceil(C / block)]."""
    A = np.asarray(A, dtype=np.float64)
    R, C = A.shape
    nr, nc = -(-R // block), -(-C // block)
    codes = np.empty_like(A)
    scales = np.ones((nr, nc))
    for r in range(nr):
        rs = slice(r * block, min((r + 1) * block, R))
        for c in range(nc):
            cs = slice(c * block, min((c + 1) * block, C))
            amax = np.abs(A[rs, cs]).max()
            s = amax / formats.INT8_MAX if amax > 0 else 1.0
            scales[r, c] = s
            codes[rs, cs] = formats.int8_codes(A[rs, cs], amax)   # rint(127 x / amax): exact ties stay ties
    return codes, scales


def dequantize_blockwise(codes, scales, block=BLOCK):
    """codes * (their block's scale): what the quantised matrix stands for."""
    R, C = codes.shape
    rows = np.arange(R) // block
    cols = np.arange(C) // block
    return codes * scales[np.ix_(rows, cols)]


def linear_from_codes(X8, sX, W8, sW, bias=None, block=BLOCK):
    """Y from already quantised operands (the formula of the module header)."""
    M, K = X8.shape
    N = W8.shape[0]
    assert W8.shape[1] == K
    Y = np.zeros((M, N))
    rows = np.arange(M) // block
    cols = np.arange(N) // block
    for kb in range(-(-K // block)):
        ks = slice(kb * block, min((kb + 1) * block, K))
        S = X8[:, ks] @ W8[:, ks].T          # integers below 2^53: exact in float64
        Y += S * sX[rows, kb][:, None] * sW[cols, kb][None, :]
    if bias is not None:
        Y = Y + np.asarray(bias, dtype=np.float64)[None, :]
    return Y


def w8a8_linear(X, W, bias=None, block=BLOCK):
    """Quantise X[M, K] and W[N, K] block-wise and return (Y[M, N], parts) with
    parts = dict(X8, sX, W8, sW)."""
    X8, sX = quantize_blockwise(X, block)
    W8, sW = quantize_blockwise(W, block)
    Y = linear_from_codes(X8, sX, W8, sW, bias, block)
    return Y, {"X8": X8, "sX": sX, "W8": W8, "sW": sW}


def linear_flops(M, N, K):
    """Multiply-adds of the layer counted as 2 operations each."""
    return 2.0 * M * N * K
