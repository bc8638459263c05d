"""Pins of the W8A8 Linear oracle (CPU only): what the definition and arithmetic fix,
checked by means other than the oracle's own code path -- a scalar-loop brute force,
closed forms on exactly representable inputs, the rounding error bound against the
unquantised product, and invariances a wrong index or a dropped block would break."""
import math

import numpy as np
import pytest

from oracle import w8a8_oracle as wo


def _rand(shape, seed, outliers=True):
    g = np.random.default_rng(seed)
    A = g.standard_normal(shape)
    if outliers:   # a few large entries so that block scales differ a lot
        idx = g.integers(0, A.size, size=max(1, A.size // 50))
        A.flat[idx] *= 20.0
    return A


def _brute(X, W, bias, block):
    """Scalar loops straight from the definition; Python floats and ints."""
    M, K = len(X), len(X[0])
    N = len(W)

    def scale(A, r, c):
        rows = range(r * block, min((r + 1) * block, len(A)))
        cols = range(c * block, min((c + 1) * block, len(A[0])))
        amax = max(abs(A[i][j]) for i in rows for j in cols)
        return amax / 127.0 if amax > 0 else 1.0

    def code(a, s):
        q = a / s
        f = math.floor(q)
        d = q - f
        r = f + 1 if d > 0.5 or (d == 0.5 and f % 2 == 1) else f   # ties to even
        return max(-127, min(127, int(r)))

    Y = [[0.0] * N for _ in range(M)]
    for m in range(M):
        for n in range(N):
            acc = 0.0
            for kb in range((K + block - 1) // block):
                sx, sw = scale(X, m // block, kb), scale(W, n // block, kb)
                isum = 0
                for k in range(kb * block, min((kb + 1) * block, K)):
                    isum += code(X[m][k], sx) * code(W[n][k], sw)
                acc += sx * sw * isum
            Y[m][n] = acc + (bias[n] if bias is not None else 0.0)
    return Y


@pytest.mark.parametrize("M,N,K,block", [(5, 4, 6, 2), (7, 3, 9, 4), (4, 4, 4, 4), (9, 5, 7, 3)])
def test_matches_scalar_brute_force(M, N, K, block):
    X, W = _rand((M, K), 1), _rand((N, K), 2)
    bias = np.arange(N) * 0.25 - 0.5
    Y, _ = wo.w8a8_linear(X, W, bias, block=block)
    ref = np.array(_brute(X.tolist(), W.tolist(), bias.tolist(), block))
    assert np.abs(Y - ref).max() <= 1e-12 * max(1.0, np.abs(ref).max())


def test_codes_scales_and_ragged_edges():
    A = _rand((300, 200), 3)            # 3 x 2 blocks, both edges ragged (44 rows, 72 columns)
    codes, scales = wo.quantize_blockwise(A)
    assert scales.shape == (3, 2)
    assert np.all(codes == np.rint(codes)) and np.abs(codes).max() == 127
    for r in range(3):
        for c in range(2):
            blk = A[128 * r:128 * (r + 1), 128 * c:128 * (c + 1)]
            assert scales[r, c] == np.abs(blk).max() / 127.0
            cb = codes[128 * r:128 * (r + 1), 128 * c:128 * (c + 1)]
            assert np.abs(cb).max() == 127                          # the largest entry maps to +-127
            assert np.abs(cb * scales[r, c] - blk).max() <= scales[r, c] / 2 * (1 + 1e-12)
    # zero padding to whole blocks changes nothing: edges take their scale from valid entries only
    P = np.zeros((384, 256))
    P[:300, :200] = A
    pc, ps = wo.quantize_blockwise(P)
    assert np.array_equal(ps, scales) and np.array_equal(pc[:300, :200], codes) and not pc[300:].any()
    # an all-zero block has scale 1 and zero codes
    Z = A.copy()
    Z[128:256, 0:128] = 0.0
    zc, zs = wo.quantize_blockwise(Z)
    assert zs[1, 0] == 1.0 and not zc[128:256, 0:128].any()


def test_exactly_representable_inputs_give_the_exact_product():
    """Integers in [-127, 127] times a power of two per block, every block holding a +-127:
    quantisation is lossless, so Y must equal the float64 product X W^T exactly."""
    g = np.random.default_rng(4)
    M, N, K = 200, 260, 384
    Xi = g.integers(-127, 128, size=(M, K)).astype(np.float64)
    Wi = g.integers(-127, 128, size=(N, K)).astype(np.float64)
    Xi[::128, ::128] = 127.0
    Wi[::128, ::128] = -127.0
    px = 2.0 ** g.integers(-6, 3, size=(2, 3))
    pw = 2.0 ** g.integers(-8, 1, size=(3, 3))
    X = Xi * px[np.ix_(np.arange(M) // 128, np.arange(K) // 128)]
    W = Wi * pw[np.ix_(np.arange(N) // 128, np.arange(K) // 128)]
    Y, parts = wo.w8a8_linear(X, W)
    assert np.array_equal(parts["X8"], Xi) and np.array_equal(parts["W8"], Wi)
    assert np.array_equal(parts["sX"], px) and np.array_equal(parts["sW"], pw)
    assert np.array_equal(Y, X @ W.T)
    assert np.array_equal(wo.dequantize_blockwise(parts["X8"], parts["sX"]), X)


def test_error_against_the_unquantised_product_is_within_the_rounding_bound():
    """|x - x8 sX| <= sX / 2 and |w - w8 sW| <= sW / 2 element-wise, so
    |Y - X W^T| <= sum_k |x| sW/2 + |w| sX/2 + sX sW / 4 (per element, exact bound)."""
    M, N, K = 150, 140, 300
    X, W = _rand((M, K), 5), _rand((N, K), 6)
    Y, parts = wo.w8a8_linear(X, W)
    ex = parts["sX"][np.ix_(np.arange(M) // 128, np.arange(K) // 128)] / 2
    ew = parts["sW"][np.ix_(np.arange(N) // 128, np.arange(K) // 128)] / 2
    bound = np.abs(X) @ ew.T + ex @ np.abs(W).T + ex @ ew.T
    err = np.abs(Y - X @ W.T)
    assert np.all(err <= bound * (1 + 1e-9) + 1e-12)
    assert err.max() > 0                                     # it is a lossy layer, not a no-op
    # and it is a useful approximation: about a percent on Gaussian inputs without outliers
    Xg, Wg = _rand((M, K), 5, outliers=False), _rand((N, K), 6, outliers=False)
    Yg, _ = wo.w8a8_linear(Xg, Wg)
    assert np.linalg.norm(Yg - Xg @ Wg.T) / np.linalg.norm(Xg @ Wg.T) < 0.02


def test_block_scaling_and_feature_permutation_invariances():
    M, N, K = 256, 128, 384
    X, W = _rand((M, K), 7), _rand((N, K), 8)
    Y, parts = wo.w8a8_linear(X, W)
    # scaling one activation block by a power of two scales its scale, not its codes: Y changes by
    # exactly that block's contribution times (factor - 1)
    X2 = X.copy()
    X2[128:256, 128:256] *= 8.0
    Y2, p2 = wo.w8a8_linear(X2, W)
    assert np.array_equal(p2["X8"], parts["X8"]) and p2["sX"][1, 1] == 8.0 * parts["sX"][1, 1]
    contrib = (parts["X8"][128:256, 128:256] @ parts["W8"][:, 128:256].T) * parts["sX"][1, 1] * parts["sW"][0, 1]
    assert np.allclose(Y2[128:256] - Y[128:256], 7.0 * contrib, rtol=1e-12, atol=1e-12)
    assert np.array_equal(Y2[:128], Y[:128])
    # permuting the features inside one feature block, in X and W alike, changes nothing
    perm = np.arange(K)
    perm[128:256] = 128 + np.random.default_rng(9).permutation(128)
    Yp, _ = wo.w8a8_linear(X[:, perm], W[:, perm])
    assert np.allclose(Yp, Y, rtol=1e-13, atol=1e-13)
    # moving features ACROSS blocks does change the scales, hence (slightly) the result
    roll = np.roll(np.arange(K), 64)
    Yr, _ = wo.w8a8_linear(X[:, roll], W[:, roll])
    assert not np.allclose(Yr, Y, rtol=1e-13, atol=1e-13)
    # bias is added once per output feature
    b = np.linspace(-1, 1, N)
    Yb, _ = wo.w8a8_linear(X, W, b)
    assert np.allclose(Yb - Y, b[None, :], rtol=0, atol=1e-12)


def test_identity_like_weight_returns_the_dequantised_activations():
    """W = identity: its blocks on the diagonal have scale 1/127 and codes 127 I, the others are
    zero, so Y is exactly the block-wise dequantised X."""
    K = 256
    X = _rand((130, K), 10)
    Y, parts = wo.w8a8_linear(X, np.eye(K))
    assert np.allclose(Y, wo.dequantize_blockwise(parts["X8"], parts["sX"]), rtol=1e-15, atol=0)
    assert np.abs(Y - X).max() <= parts["sX"].max() / 2 * (1 + 1e-12)
