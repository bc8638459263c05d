"""GPU parity of the W8A8 Linear layer (through the C ABI) against the CPU oracle:
the quantiser's codes and scales, the INT8 product with its block-scale accumulation
given those codes, and the whole layer from bf16 inputs."""
import numpy as np
import pytest
import torch

from oracle import w8a8_oracle as wo
from paper_2512_16093_amd import binding as sla
from paper_2512_16093_amd import synth

pytestmark = pytest.mark.gpu

# (M, K, N): one token; ragged token tails; one and many feature blocks; several output tiles
SHAPES = [(1, 128, 128), (300, 384, 256), (257, 256, 128), (1000, 1024, 512), (640, 2048, 384)]


def check_codes(gpu_codes, gpu_scales, A, what):
    codes, scales = wo.quantize_blockwise(A)
    # scales: max|block| / 127 evaluated in fp32 on the GPU, in fp64 here
    assert np.allclose(gpu_scales, scales, rtol=3e-7, atol=0), what
    # codes: the correctly rounded quotient 127 x / amax on both sides, exact ties to the even code: identical
    assert np.array_equal(gpu_codes.astype(np.float64), codes), (what, int((gpu_codes != codes).sum()))


def product_tolerance(ref, sX, sW, K):
    """bf16 rounding of the result (relative 2^-9, doubled) plus the fp32 accumulation of the block
    sums.  The kernel adds each block sum together with a constant of about 2^23.4 integer steps
    (it reads the integer accumulator as a float, see the kernel's header) and removes the
    constants every fourth block, so a running sum stays below 2^26 steps and every fma rounds by
    at most 2 steps s_X s_W: at most 2 K / 128 steps in all (a worst case; the errors are random)."""
    return 2.0 ** -8 * np.abs(ref) + (2.0 * K / 128 + 1.0) * sX.max() * sW.max()


@pytest.mark.parametrize("M,K,N", SHAPES)
def test_quantiser_matches_oracle(M, K, N):
    x, w, _ = synth.make_linear_inputs(M, K, N)
    ws = sla.w8a8_quantize_act(x.cuda())
    xc, xs = sla.w8a8_debug_unpack(ws, False, M, K)
    check_codes(xc.cpu().numpy(), xs.cpu().numpy(), synth.as_f64(x), "activations %s" % ((M, K),))
    wq = sla.w8a8_quantize_weight(w.cuda())
    wc, wsc = sla.w8a8_debug_unpack(wq, True, N, K)
    check_codes(wc.cpu().numpy(), wsc.cpu().numpy(), synth.as_f64(w), "weights %s" % ((N, K),))


@pytest.mark.parametrize("M,K,N", SHAPES)
@pytest.mark.parametrize("with_bias", [True, False])
def test_product_matches_oracle_on_the_same_codes(M, K, N, with_bias):
    x, w, b = synth.make_linear_inputs(M, K, N, seed=1, with_bias=with_bias)
    xd, wd = x.cuda(), w.cuda()
    bd = None if b is None else b.cuda()
    wq = sla.w8a8_quantize_weight(wd)
    ws = sla.w8a8_quantize_act(xd)
    y = sla.w8a8_gemm_fwd(ws, wq, M, N, K, bias=bd).float().cpu().numpy()
    xc, xs = (t.cpu().numpy().astype(np.float64) for t in sla.w8a8_debug_unpack(ws, False, M, K))
    wc, wsc = (t.cpu().numpy().astype(np.float64) for t in sla.w8a8_debug_unpack(wq, True, N, K))
    ref = wo.linear_from_codes(xc, xs, wc, wsc, None if b is None else synth.as_f64(b))
    assert np.all(np.abs(y - ref) <= product_tolerance(ref, xs, wsc, K)), np.abs(y - ref).max()


@pytest.mark.parametrize("M,K,N", SHAPES)
def test_whole_layer_matches_oracle(M, K, N):
    x, w, b = synth.make_linear_inputs(M, K, N, seed=2)
    wq = sla.w8a8_quantize_weight(w.cuda())
    y = sla.w8a8_linear_fwd(x.cuda(), wq, N, bias=b.cuda()).float().cpu().numpy()
    ref, parts = wo.w8a8_linear(synth.as_f64(x), synth.as_f64(w), synth.as_f64(b))
    # (the codes are the oracle's, see test_quantiser_matches_oracle: only the product's own tolerance applies)
    tol = product_tolerance(ref, parts["sX"], parts["sW"], K)
    assert np.all(np.abs(y - ref) <= tol), np.abs(y - ref).max()
    assert np.linalg.norm(y - ref) / np.linalg.norm(ref) < 3e-3
    # and the layer does its job: close to the unquantised product (a block's scale follows its
    # outlier features, so the other features of the block keep only a few bits: several percent)
    dense = synth.as_f64(x) @ synth.as_f64(w).T + synth.as_f64(b)
    assert np.linalg.norm(y - dense) / np.linalg.norm(dense) < 0.15


def test_exactly_representable_inputs_lose_only_the_accumulation_steps():
    """Integer codes times power-of-two scales, every block holding a 127: quantisation is lossless,
    so the only errors left are the accumulation's (at most 2 steps s_X s_W = 1/8 per block, two
    blocks here) and the bf16 rounding of the output."""
    g = np.random.default_rng(3)
    M, K, N = 300, 256, 256
    Xi = g.integers(-3, 4, size=(M, K)).astype(np.float32)
    Wi = g.integers(-2, 3, size=(N, K)).astype(np.float32)
    Xi[::128, ::128] = 127.0
    Wi[::128, ::128] = 127.0
    Xi[::128, 1::128] = 0.0
    x = torch.from_numpy(Xi * 0.25).to(torch.bfloat16)
    w = torch.from_numpy(Wi * 0.5).to(torch.bfloat16)
    xd, wd = x.cuda(), w.cuda()
    wq = sla.w8a8_quantize_weight(wd)
    ws = sla.w8a8_quantize_act(xd)
    xc, xs = sla.w8a8_debug_unpack(ws, False, M, K)
    wc, wsc = sla.w8a8_debug_unpack(wq, True, N, K)
    assert np.array_equal(xc.cpu().numpy(), Xi) and np.array_equal(wc.cpu().numpy(), Wi)      # lossless codes
    assert (xs == 0.25).all() and (wsc == 0.5).all()
    y = sla.w8a8_linear_fwd(xd, wq, N).float().cpu().numpy()
    ref = (Xi * 0.25).astype(np.float64) @ (Wi * 0.5).astype(np.float64).T
    assert np.all(np.abs(y - ref) <= 4 * 0.125 + 2.0 ** -9 * np.abs(ref))
    assert (y == ref).mean() > 0.5          # and most results are exact


def test_deterministic_and_workspace_reuse():
    x, w, b = synth.make_linear_inputs(500, 512, 256, seed=4)
    xd, bd = x.cuda(), b.cuda()
    wq = sla.w8a8_quantize_weight(w.cuda())
    ws = sla.w8a8_alloc_workspace(500, 512)
    y1 = sla.w8a8_linear_fwd(xd, wq, 256, bias=bd, workspace=ws).clone()
    sla.w8a8_linear_fwd(xd[:100].contiguous(), wq, 256, bias=bd, workspace=ws)   # a smaller call in between
    y2 = sla.w8a8_linear_fwd(xd, wq, 256, bias=bd, workspace=ws)
    assert torch.equal(y1, y2)
    assert torch.equal(x, xd.cpu())


def test_long_contraction_feed_forward_down_shape():
    """K = 13824 (108 feature blocks, the feed-forward down projection of a Wan-14B block): the
    longest accumulation of block sums the layer sees, on 1000 tokens."""
    M, K, N = 1000, 13824, 5120
    x, w, b = synth.make_linear_inputs(M, K, N, seed=5)
    wq = sla.w8a8_quantize_weight(w.cuda())
    ws = sla.w8a8_quantize_act(x.cuda())
    y = sla.w8a8_gemm_fwd(ws, wq, M, N, K, bias=b.cuda()).float().cpu().numpy()
    xc, xs = (t.cpu().numpy().astype(np.float64) for t in sla.w8a8_debug_unpack(ws, False, M, K))
    wc, wsc = (t.cpu().numpy().astype(np.float64) for t in sla.w8a8_debug_unpack(wq, True, N, K))
    ref = wo.linear_from_codes(xc, xs, wc, wsc, synth.as_f64(b))
    err = np.abs(y - ref)
    assert np.all(err <= product_tolerance(ref, xs, wsc, K)), err.max()
    # what the accumulation adds on top of the bf16 rounding of the output: in steps of the largest
    # block it stays inside the worst-case bound, and as a relative error it is smaller than the
    # output rounding itself (both are ~100x below the rounding of the INT8 codes)
    excess = (err - 2.0 ** -9 * np.abs(ref)).max() / (xs.max() * wsc.max())
    rel = np.linalg.norm(y - ref) / np.linalg.norm(ref)
    print("w8a8 K=13824: accumulation error beyond output rounding: %.1f steps (bound %d); relative error %.2e"
          % (max(excess, 0.0), 2 * K // 128 + 1, rel))
    assert rel < 3e-3


def test_full_size_attention_projection_sampled():
    """The layer at the size the benchmark times (75600 tokens, 5120 -> 5120): the oracle on whole
    quantisation row blocks -- the first, one in the middle and the ragged last one (75600 =
    590 * 128 + 80) -- against all output features."""
    M, K, N = 75600, 5120, 5120
    x, w, b = synth.make_linear_inputs(M, K, N)
    print("running the GPU layer", flush=True)
    wq = sla.w8a8_quantize_weight(w.cuda())
    y = sla.w8a8_linear_fwd(x.cuda(), wq, N, bias=b.cuda())
    torch.cuda.synchronize()
    assert torch.isfinite(y.float()).all()
    print("oracle: quantising the weight", flush=True)
    W8, sW = wo.quantize_blockwise(synth.as_f64(w))
    worst = 0.0
    for rb in (0, 295, 590):
        rows = slice(rb * 128, min((rb + 1) * 128, M))
        print("oracle on token block", rb, flush=True)
        X8, sX = wo.quantize_blockwise(synth.as_f64(x[rows]))
        ref = wo.linear_from_codes(X8, sX, W8, sW, synth.as_f64(b))
        got = y[rows].float().cpu().numpy()
        tol = product_tolerance(ref, sX, sW, K) + 127.0 * 4 * sX.max() * sW.max()
        assert np.all(np.abs(got - ref) <= tol), (rb, np.abs(got - ref).max())
        rel = np.linalg.norm(got - ref) / np.linalg.norm(ref)
        assert rel < 3e-3, (rb, rel)
        worst = max(worst, rel)
    print("w8a8 75600 x 5120 -> 5120: worst relative error of a sampled token block %.2e" % worst)
