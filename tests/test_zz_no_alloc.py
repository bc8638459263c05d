"""The entry point that allocates nothing (sla_classify_blocks_static, for callers that cannot
allocate: graph capture, serving loops): through the C ABI against sla_classify_blocks on the same
inputs, bit for bit, on two calls in a row, the second smaller (the built-in scratch keeps the
first call's contents)."""
import pytest
import torch

from paper_2512_16093_amd import binding as sla
from paper_2512_16093_amd import synth

pytestmark = pytest.mark.gpu


def _both(cfg, want_scores):
    q, k, _ = synth.make_qkv(cfg)
    q, k = q.cuda(), k.cuda()
    ref = sla.sla_classify_blocks(q, k, cfg.block_q, cfg.block_k, cfg.topk_ratio, cfg.marginal_ratio,
                                  want_scores=want_scores)
    # outputs pre-filled with a pattern, so anything the call leaves unwritten shows
    outs = [torch.full_like(t, 0x55 if t.dtype != torch.float32 else float("nan")) if t is not None else None for t in ref]
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    sla.sla_classify_blocks_static(q, k, cfg.block_q, cfg.block_k, cfg.topk_ratio, cfg.marginal_ratio, *outs)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    for name, a, b in zip(("mask", "crit_idx", "marg_idx", "pooled_scores"), outs, ref):
        if b is not None:
            assert torch.equal(a, b), name


def test_static_scratch_entry_point_matches_the_workspace_one():
    big = synth.custom_config(2, 3, (3, 27, 27), block_q=128, topk_ratio=0.1, marginal_ratio=0.2, cfg_id=700)   # N = 2187, ragged
    small = synth.custom_config(1, 2, (5, 10, 20), block_q=64, topk_ratio=0.2, marginal_ratio=0.4, cfg_id=701)  # N = 1000
    _both(big, want_scores=False)       # scores in the built-in scratch
    _both(small, want_scores=False)     # a smaller problem over the first call's leftovers
    _both(small, want_scores=True)      # scores written to the caller's tensor
    _both(synth.CONFIGS[0], want_scores=False)
