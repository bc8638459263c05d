"""Helpers shared by the GPU parity tests: oracle runs on CPU copies of the seeded
inputs, and the comparison rules (mask ties, output tolerances)."""
import numpy as np
import torch

from oracle import sla_oracle as so
from paper_2512_16093_amd import synth

# Output tolerances against the oracle's quantised result, as the task states them.
MAX_ABS = 2e-2
MIN_COS = 0.999
TIE = 1e-4          # pooled-score band inside which a mask disagreement is excused


def cosine(a, b):
    a = np.asarray(a, dtype=np.float64).ravel()
    b = np.asarray(b, dtype=np.float64).ravel()
    return float(a @ b / (np.linalg.norm(a) * np.linalg.norm(b)))


def check_output(gpu, ref, what, max_abs=MAX_ABS, min_cos=MIN_COS):
    gpu = np.asarray(gpu, dtype=np.float64)
    ok = ~np.isnan(ref)
    assert np.isfinite(gpu[ok]).all(), what + ": non-finite output"
    err = float(np.abs(gpu[ok] - ref[ok]).max())
    cos = cosine(gpu[ok], ref[ok])
    assert err <= max_abs, "%s: max-abs %.3e > %.1e" % (what, err, max_abs)
    assert cos >= min_cos, "%s: cosine %.6f < %.4f" % (what, cos, min_cos)
    return err, cos


def check_mask(gpu_mask, scores64, n_c, n_m, what):
    """Bit-exact against the oracle's mask except where the oracle's own score is
    within TIE of a class boundary; every row must still hold exactly n_c / n_m."""
    ref = so.classify(scores64, n_c, n_m)
    gpu_mask = np.asarray(gpu_mask)
    assert gpu_mask.shape == ref.shape
    assert ((gpu_mask == 1).sum(1) == n_c).all(), what + ": wrong critical count"
    assert ((gpu_mask == 0).sum(1) == n_m).all(), what + ": wrong marginal count"
    bad = np.argwhere(gpu_mask != ref)
    srt = -np.sort(-scores64, axis=1)
    excused = 0
    for i, j in bad:
        s = scores64[i, j]
        near = abs(s - srt[i, n_c - 1]) <= TIE or (n_c < srt.shape[1] and abs(s - srt[i, n_c]) <= TIE)
        if n_m > 0 and n_c + n_m < srt.shape[1]:
            near = near or abs(s - srt[i, n_c + n_m - 1]) <= TIE or abs(s - srt[i, n_c + n_m]) <= TIE
        assert near, "%s: mask differs at row %d block %d away from any tie" % (what, i, j)
        excused += 1
    return len(bad), excused, ref


# The kernel refreshes the running reference of the softmax after every 32 keys (one MFMA key
# tile) instead of once per 64-key block; the oracle is run the same way (its ref_tile switch),
# since both sides must round P to FP8 at the same level.
REF_TILE = 32


def oracle_head(cfg, q, k, v, b, h, W=None, bias=None, q_blocks=None, mask=None, phi="softmax"):
    """Oracle forward of one (b,h) slice of CPU bf16 tensors."""
    Q, K, V = (synth.as_f64(t[b, h]) for t in (q, k, v))
    return so.sla_forward_head(Q, K, V, cfg.block_q, cfg.block_k, cfg.topk_ratio, cfg.marginal_ratio,
                               proj_w=None if W is None else synth.as_f64(W),
                               proj_b=None if bias is None else synth.as_f64(bias),
                               phi=phi, q_blocks=q_blocks, mask=mask, ref_tile=REF_TILE)


def to_dev(*ts):
    return tuple(None if t is None else t.cuda() for t in ts)


def lists_from_mask(mask_np):
    """crit_idx int32 tensor [B,H,Tq,n_c] from an int8 mask array with equal counts per row."""
    B, H, Tq, Tk = mask_np.shape
    n_c = int((mask_np[0, 0, 0] == 1).sum())
    crit = np.zeros((B, H, Tq, n_c), dtype=np.int32)
    for b in range(B):
        for h in range(H):
            crit[b, h] = so.mask_lists(mask_np[b, h])[0]
    return torch.from_numpy(crit)


def make_qkv_threaded(cfg, seed=0, workers=8):
    """All heads of a config, generated with a thread pool (numpy releases the GIL in its kernels)."""
    from concurrent.futures import ThreadPoolExecutor
    shape = (cfg.B, cfg.H, cfg.N, cfg.d)
    q, k, v = (torch.empty(shape, dtype=torch.bfloat16) for _ in range(3))

    def one(bh):
        b, h = divmod(bh, cfg.H)
        q[b, h], k[b, h], v[b, h] = synth.make_head(cfg, b, h, seed)

    with ThreadPoolExecutor(max_workers=workers) as ex:
        list(ex.map(one, range(cfg.B * cfg.H)))
    return q, k, v
