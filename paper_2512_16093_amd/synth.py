"""Seeded synthetic Q/K/V for the SLA forward path.

This module only makes inputs. It holds none of the method's arithmetic
(no pooling, scoring, quantisation, softmax or feature map) and is the one
module that both the HIP path's tests and the CPU oracle's tests draw
inputs from.

The paper's workload is the self-attention of Wan video DiTs over the
flattened spatio-temporal token grid (Section 2.1 names the four models; their
activations need trained weights).  These inputs stand in for them: the Wan
token-grid shapes, bf16, spatio-temporally smooth (sum of low-frequency
sinusoids over (t, y, x)) plus white noise, with a large per-channel offset on
K (the outlier channels K-smoothing exists for).

Recipe, per (b, h), rng = PCG64(SeedSequence([seed, cfg_id, b, h])):
  * 8 integer frequency triples (ft, fy, fx), each entry uniform in {0,1,2,3},
    redrawn while all three are zero; shared by Q, K and V;
  * per tensor X in (Q, K, V) and channel c: amplitudes a[m,c] ~ N(0,1)/sqrt(8),
    phases th[m,c] ~ U[0, 2pi);
  * X[n,c] = sum_m a[m,c] sin(2pi(ft t/T + fy y/Hg + fx x/Wg) + th[m,c])
             + 0.5 eps[n,c],  eps ~ N(0,1);  token n = (t*Hg + y)*Wg + x;
  * K[n,c] += beta[c],  beta ~ 2 N(0,1);
  * round to bf16 (round-to-nearest-even).
The projection W ~ N(0,1)/sqrt(d) comes from SeedSequence([seed, cfg_id, 87]),
rounded to bf16.
"""
from __future__ import annotations

import dataclasses
import math

import numpy as np
import torch


@dataclasses.dataclass(frozen=True)
class SLAConfig:
    """One seeded workload: shape, token grid, block sizes and ratios."""
    cfg_id: int
    name: str
    B: int
    H: int
    grid: tuple  # (T, Hg, Wg); N = T*Hg*Wg
    d: int
    block_q: int
    block_k: int
    topk_ratio: float
    marginal_ratio: float
    use_proj: bool

    @property
    def N(self) -> int:
        t, y, x = self.grid
        return t * y * x


CONFIGS = {
    0: SLAConfig(0, "tiny", 1, 2, (4, 16, 16), 128, 64, 64, 0.2, 0.4, True),
    1: SLAConfig(1, "wan1.3b-480p", 1, 12, (21, 30, 52), 128, 128, 64, 0.1, 0.2, True),
    2: SLAConfig(2, "dense-quant", 1, 12, (21, 30, 52), 128, 128, 64, 1.0, 0.0, False),
    3: SLAConfig(3, "wan14b-480p", 1, 40, (21, 30, 52), 128, 128, 64, 0.1, 0.2, True),
    4: SLAConfig(4, "wan14b-720p", 1, 40, (21, 45, 80), 128, 128, 64, 0.1, 0.2, True),
    # The evaluation setup (Section 2.1) recommends Top-K ratios up to 0.15: that value, with the
    # other 85 % of the blocks marginal (nothing skipped but the one block per row that flooring both
    # counts leaves over), at both query block sizes
    5: SLAConfig(5, "wan14b-720p-top15-noskip", 1, 40, (21, 45, 80), 128, 128, 64, 0.15, 0.85, True),
    6: SLAConfig(6, "wan14b-720p-top15-noskip-bq64", 1, 40, (21, 45, 80), 128, 64, 64, 0.15, 0.85, True),
}


def custom_config(B, H, grid, d=128, block_q=64, block_k=64, topk_ratio=0.2,
                  marginal_ratio=0.4, use_proj=True, cfg_id=100, name="custom"):
    """A config outside the named ones (ragged tails, odd ratios ...)."""
    return SLAConfig(cfg_id, name, B, H, tuple(grid), d, block_q, block_k,
                     topk_ratio, marginal_ratio, use_proj)


def _to_bf16(x: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16)


def make_head(cfg: SLAConfig, b: int, h: int, seed: int = 0):
    """Q, K, V of one (b, h) slice as torch.bfloat16 CPU tensors [N, d]."""
    T, Hg, Wg = cfg.grid
    N, d = cfg.N, cfg.d
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, cfg.cfg_id, b, h])))
    freqs = np.zeros((8, 3), dtype=np.int64)
    for m in range(8):
        f = rng.integers(0, 4, size=3)
        while not f.any():
            f = rng.integers(0, 4, size=3)
        freqs[m] = f
    n = np.arange(N)
    x = n % Wg
    y = (n // Wg) % Hg
    t = n // (Wg * Hg)
    # phase[n, m] = 2 pi (ft t/T + fy y/Hg + fx x/Wg)
    phase = 2.0 * math.pi * (np.outer(t / T, freqs[:, 0]) + np.outer(y / Hg, freqs[:, 1])
                             + np.outer(x / Wg, freqs[:, 2]))
    sin_p, cos_p = np.sin(phase), np.cos(phase)
    out = []
    for name in ("q", "k", "v"):
        a = rng.standard_normal((8, d)) / math.sqrt(8.0)
        th = rng.uniform(0.0, 2.0 * math.pi, size=(8, d))
        # sin(p + th) = sin p cos th + cos p sin th, summed over m as two small matmuls
        X = sin_p @ (a * np.cos(th)) + cos_p @ (a * np.sin(th))
        X += 0.5 * rng.standard_normal((N, d), dtype=np.float32)
        if name == "k":
            X += 2.0 * rng.standard_normal(d)[None, :]
        out.append(_to_bf16(X))
    return tuple(out)


def make_qkv(cfg: SLAConfig, seed: int = 0, heads=None):
    """Q, K, V as torch.bfloat16 CPU tensors [B, H, N, d] (all heads, or the
    listed (b, h) pairs filled and the rest zero when `heads` is given)."""
    q = torch.zeros((cfg.B, cfg.H, cfg.N, cfg.d), dtype=torch.bfloat16)
    k = torch.zeros_like(q)
    v = torch.zeros_like(q)
    pairs = heads if heads is not None else [(b, h) for b in range(cfg.B) for h in range(cfg.H)]
    for b, h in pairs:
        q[b, h], k[b, h], v[b, h] = make_head(cfg, b, h, seed)
    return q, k, v


def make_proj(cfg: SLAConfig, seed: int = 0):
    """Projection weight W [d, d] (out, in) as torch.bfloat16, or None."""
    if not cfg.use_proj:
        return None
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, cfg.cfg_id, 87])))
    return _to_bf16(rng.standard_normal((cfg.d, cfg.d)) / math.sqrt(cfg.d))


def as_f64(x: torch.Tensor) -> np.ndarray:
    """Exact widening of a bf16 tensor to a float64 numpy array."""
    return x.to(torch.float64).numpy()


def make_linear_inputs(M: int, K: int, N: int, seed: int = 0, with_bias: bool = True):
    """Stand-in for a DiT Linear layer (no trained weights are available): activations
    X [M, K] ~ N(0, 1) with 1 % of the features carrying 10-30x the amplitude (the outlier
    channels typical of transformer activations) and a per-token amplitude in [0.5, 2];
    weights W [N, K] ~ N(0, 1 / K); bias ~ N(0, 0.1).  torch.bfloat16 CPU tensors."""
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 4242, M, K, N])))
    X = rng.standard_normal((M, K), dtype=np.float32)
    out_ch = rng.choice(K, size=max(1, K // 100), replace=False)
    X[:, out_ch] *= rng.uniform(10.0, 30.0, size=out_ch.size).astype(np.float32)
    X *= rng.uniform(0.5, 2.0, size=(M, 1)).astype(np.float32)
    W = rng.standard_normal((N, K), dtype=np.float32) / np.float32(math.sqrt(K))
    b = _to_bf16(0.1 * rng.standard_normal(N)) if with_bias else None
    return _to_bf16(X), _to_bf16(W), b
