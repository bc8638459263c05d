#!/usr/bin/env python3
"""Benchmark of the SLA forward hot path on one MI355X.

A "step" is one call of sla_attention_fwd (pooling/statistics -> scores + block
selection -> K/V quantisation + linear summaries -> marginal accumulation ->
fused INT8/FP8 sparse attention with the linear epilogue) on the headline
workload: the Wan-14B-720P-shaped seeded synthetic config (B=1, H=40, N=75600,
d=128, block_q=128, block_k=64, 10 % critical / 20 % marginal, random projection).
Inputs are resident in HBM before the timed region.

Prints ONE JSON line: whole-call throughput in dense-equivalent TFLOP/s
(4 B H N^2 d / t), the roofline of the dominant kernel (the sparse attention
kernel, against the INT8/FP8 MFMA peak, from HIP events recorded on the launch
stream inside the timed region) and the CPU oracle timed on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBPS = 8000.0         # MI355X HBM3E
PEAK_MFMA_8BIT_TOPS = 5000.0   # MI355X dense INT8 (POP/s) and FP8 (PFLOP/s) MFMA peak, both 5.0e15
# Bytes moved past L2 per launch of the sparse kernel (FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0, the factors
# from a 1 GiB copy in the same counter runs), by config id; source: profiles/sla_fwd_wan14b-720p.md.
SPARSE_TRAFFIC_BYTES = {4: 18.11e9}


# Linear layers of a Wan2.1-14B DiT block (hidden 5120, feed-forward 13824) on the 75600 tokens of a
# 720P clip: (M, K, N)
W8A8_SHAPES = {"attn_proj": (75600, 5120, 5120), "ffn_up": (75600, 5120, 13824), "ffn_down": (75600, 13824, 5120)}


# Bytes moved past L2 per launch of the product kernel (FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0), by shape;
# source: profiles/w8a8_linear_wan14b.md.
W8A8_TRAFFIC_BYTES = {"attn_proj": 5.30e9}
# The backward pass's dominant kernel, by (config, kernel); source: profiles/sla_bwd_wan14b-720p.md.
BWD_TRAFFIC_BYTES = {(4, "bwd_dkv_kernel"): 163.7e9}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=4, help="seeded config id (4 = Wan-14B-720P shape, the headline)")
    ap.add_argument("--layout", choices=("bhnd", "bnhd"), default="bhnd",
                    help="memory order of q, k, v and out: head-major [B,H,N,d] (default) or token-major "
                         "[B,N,H,d] through the strided entry point")
    ap.add_argument("--workload", choices=("sla", "w8a8", "sla_bwd"), default="sla",
                    help="sla: the SLA forward (the headline, default); w8a8: the W8A8 Linear layer at a Wan-14B "
                         "shape; sla_bwd: the SLA backward pass (each a JSON line of its own metric)")
    ap.add_argument("--w8a8-shape", choices=tuple(W8A8_SHAPES), default="attn_proj",
                    help="which Linear layer of a Wan-14B block, on the 75600 tokens of a 720P clip")
    ap.add_argument("--quant", choices=("int8fp8", "qk_int8", "none"), default="int8fp8",
                    help="sla workload: the paper's low-bit inference path (default), INT8 scores with a 16-bit P.V "
                         "(qk_int8), or the unquantised bf16 forward (plain SLA, the training-time operator)")
    ap.add_argument("--saved-state", action="store_true",
                    help="sla_bwd workload: hand the backward pass the statistics of a training forward pass "
                         "(sla_attention_fwd_train, run once outside the timed region) instead of recomputing them")
    ap.add_argument("--only-headline", action="store_true",
                    help="sla workload: leave out the short runs of the other two workloads (W8A8 Linear layer, SLA "
                         "backward) that the default invocation appends to its line as `other_workloads`")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=20.0, help="rough budget for the oracle sample")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy (reads 1 GiB, writes 1 GiB) a few times, so that "
                         "FETCH_SIZE / WRITE_SIZE counter runs of this command can be scaled by a kernel of known traffic")
    return ap.parse_args()


def traffic_from_profile(name, cfg_id):
    """HBM bytes per launch of the dominant kernel as the committed rocprofv3 summary of this command states them
    (profiles/<name>: the line that ends in "per launch (the `roofline.traffic` of the bench line)"); the typed-in
    constant above is used if the file cannot be read, None for configs the summary does not cover."""
    import re
    if isinstance(name, dict):        # config id -> summary file
        name = name.get(cfg_id)
    elif cfg_id != 4:
        name = None
    if name is None:
        return None, None
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", name)
    try:
        m = re.search(r"= ([0-9.]+) GB per launch \(the `roofline.traffic`", open(path).read())
        if m:
            return float(m.group(1)) * 1e9, "profiles/%s (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command)" % name
    except OSError:
        pass
    return None, None


def copy_calibration(torch, dev):
    """Three plain 1 GiB device copies (1 GiB read, 1 GiB written each): a kernel of known traffic
    for scaling the FETCH_SIZE / WRITE_SIZE counters of the same run."""
    a = torch.zeros(1 << 30, dtype=torch.uint8, device=dev)
    b = torch.empty_like(a)
    for _ in range(3):
        b.copy_(a)
    torch.cuda.synchronize()
    del a, b


def measured_rates(torch, sla, dev):
    """What this chip sustains for the bounding resource ALONE, to set beside the published peaks: the three
    matrix instructions the kernels use (every SIMD issuing nothing else, ~8 ms launches so the clock settles;
    the mean of the last two of four launches) and a plain 1 GiB device copy (bytes read + written)."""
    n_cu = torch.cuda.get_device_properties(dev).multi_processor_count
    scratch = torch.empty(2 * n_cu * 256, dtype=torch.float32, device=dev)
    out = {}
    for kind, iters, key in (("int8", 60000, "mfma_int8_TOPs"), ("fp8", 30000, "mfma_fp8_TFLOPs"), ("bf16", 60000, "mfma_bf16_TFLOPs")):
        times = []
        for _ in range(4):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            ops = sla.sla_calibrate_mfma(kind, iters, scratch)
            e1.record()
            torch.cuda.synchronize()
            times.append(e0.elapsed_time(e1))
        out[key] = round(ops / (sum(times[2:]) / 2 * 1e-3) / 1e12, 1)
    a = torch.zeros(1 << 30, dtype=torch.uint8, device=dev)
    b = torch.empty_like(a)
    times = []
    for _ in range(4):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        b.copy_(a)
        e1.record()
        torch.cuda.synchronize()
        times.append(e0.elapsed_time(e1))
    out["device_copy_GBps"] = round(2.0 * (1 << 30) / (sum(times[2:]) / 2 * 1e-3) / 1e9, 1)
    del a, b, scratch
    return out


def make_inputs(cfg, synth, torch):
    """All heads of the seeded config, generated on the host (threaded over heads), then uploaded."""
    shape = (cfg.B, cfg.H, cfg.N, cfg.d)
    q, k, v = (torch.empty(shape, dtype=torch.bfloat16, pin_memory=True) for _ in range(3))

    def one(bh):
        b, h = divmod(bh, cfg.H)
        q[b, h], k[b, h], v[b, h] = synth.make_head(cfg, b, h)

    with ThreadPoolExecutor(max_workers=8) as ex:
        list(ex.map(one, range(cfg.B * cfg.H)))
    return q, k, v


def cpu_baseline(cfg, q, k, v, W, budget_s, quant_name="int8fp8"):
    """The oracle as it stands, on the host cores, on a bounded sample of the same workload:
    head 0 in full for the per-head work (pooling, scores, classification, quantisation,
    linear summaries) and as many query blocks as the budget allows for the per-block work;
    extrapolated linearly (heads and query blocks are independent)."""
    import numpy as np
    from oracle import sla_oracle as so      # cpu_baseline leg: allowed to call the oracle
    from paper_2512_16093_amd import synth

    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [os.cpu_count() or 1])
    except Exception:
        cores = os.cpu_count() or 1
    Q, K, V = (synth.as_f64(t[0, 0]) for t in (q, k, v))
    Wd = None if W is None else synth.as_f64(W)
    Tq, Tk, n_c, n_m = so.block_counts(cfg.N, cfg.block_q, cfg.block_k, cfg.topk_ratio, cfg.marginal_ratio)
    t0 = time.perf_counter()
    scores = so.pooled_scores(Q, K, cfg.block_q, cfg.block_k)
    mask = so.classify(scores, n_c, n_m)
    if quant_name != "none":
        so.quantize_q(Q, cfg.block_q)
        so.quantize_k(K, cfg.block_k)
        so.quantize_v(V)
    quant = {"int8fp8": so.QUANT_QK_INT8_PV_FP8, "qk_int8": so.QUANT_QK_INT8, "none": so.QUANT_NONE}[quant_name]
    if n_m:
        so.linear_summaries(K, V, cfg.block_k)
    t_head = time.perf_counter() - t0
    # per-block cost: the oracle's forward recomputes the per-head work on every call, so time
    # one call on 1 block and one on 1 + nb blocks and take the difference
    t0 = time.perf_counter()
    so.sla_forward_head(Q, K, V, cfg.block_q, cfg.block_k, cfg.topk_ratio, cfg.marginal_ratio, proj_w=Wd,
                        q_blocks=[0], mask=mask, quant=quant)
    t_one = time.perf_counter() - t0
    per_block_guess = max(t_one - t_head, 1e-3)
    nb = int(max(2, min(Tq - 1, budget_s / per_block_guess)))
    blocks = [int(x) for x in np.linspace(0, Tq - 1, nb + 1).astype(int)]
    blocks = sorted(set(blocks))
    t0 = time.perf_counter()
    so.sla_forward_head(Q, K, V, cfg.block_q, cfg.block_k, cfg.topk_ratio, cfg.marginal_ratio, proj_w=Wd,
                        q_blocks=blocks, mask=mask, quant=quant)
    t_many = time.perf_counter() - t0
    per_block = max(t_many - t_one, 1e-9) / max(len(blocks) - 1, 1)
    t_full = cfg.B * cfg.H * (t_head + Tq * per_block)
    flops = so.dense_equiv_flops(cfg.B, cfg.H, cfg.N, cfg.d)
    return {"value": flops / t_full / 1e12, "unit": "TFLOP/s (dense-equivalent)", "cores": int(cores),
            "kind": "oracle",
            "sample": "head 0 of %d: per-head work in full (%.2f s) + %d of %d query blocks (%.3f s each); "
                      "extrapolated to %d heads x %d blocks = %.0f s"
                      % (cfg.H, t_head, len(blocks), Tq, per_block, cfg.B * cfg.H, Tq, t_full)}


def main_w8a8(args):
    """One step = one W8A8 Linear layer: block-wise quantisation of the bf16 activations, then the
    INT8 product with block-scale accumulation and bias, bf16 out.  Weights are quantised once,
    outside the timed region (offline in the paper's flow)."""
    import numpy as np
    import torch
    from paper_2512_16093_amd import binding as sla
    from paper_2512_16093_amd import synth

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    sla.lib()
    M, K, N = W8A8_SHAPES[args.w8a8_shape]
    t0 = time.perf_counter()
    x, w, b = synth.make_linear_inputs(M, K, N)
    print("[bench] inputs for %s generated in %.1f s" % (args.w8a8_shape, time.perf_counter() - t0), file=sys.stderr, flush=True)
    xd, wd, bd = x.cuda(), w.cuda(), b.cuda()
    wq = sla.w8a8_quantize_weight(wd)
    ws = sla.w8a8_alloc_workspace(M, K)
    y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    for _ in range(args.warmup):
        sla.w8a8_linear_fwd(xd, wq, N, bias=bd, workspace=ws, out=y)
    torch.cuda.synchronize()
    # the launches go to torch's current stream, so its events bracket them
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for e in ev:
        e[0].record()
        sla.w8a8_quantize_act(xd, workspace=ws)
        e[1].record()
        sla.w8a8_gemm_fwd(ws, wq, M, N, K, bias=bd, out=y)
        e[2].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    t_quant = sum(e[0].elapsed_time(e[1]) for e in ev) / args.steps
    t_gemm = sum(e[1].elapsed_time(e[2]) for e in ev) / args.steps
    ops = 2.0 * M * N * K
    achieved = ops / (t_gemm * 1e-3) / 1e12
    result = {
        "metric": "w8a8_linear_tops", "value": ops / (ms_per_step * 1e-3) / 1e12, "unit": "TOP/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "int8 (int32 block sums, fp32 scale accumulation, bf16 out)",
        "data": "synthetic",
        "config": {"workload": "w8a8-linear %s: M=%d tokens K=%d N=%d, 128x128 block scales, bias, seed=0"
                               % (args.w8a8_shape, M, K, N)},
        "stage_ms": {"quantize_act": round(t_quant, 4), "gemm": round(t_gemm, 4)},
        "roofline": {"kernel": "w8a8_gemm_kernel", "bound": "mfma", "achieved": achieved, "peak": PEAK_MFMA_8BIT_TOPS,
                     "unit": "TOP/s", "frac": achieved / PEAK_MFMA_8BIT_TOPS,
                     "traffic": W8A8_TRAFFIC_BYTES.get(args.w8a8_shape), "traffic_unit": "bytes per launch",
                     "launch_ms": t_gemm, "ops_per_launch": ops},
        "quantize_act_roofline": {"bound": "hbm", "achieved": 3.0 * M * K / (t_quant * 1e-3) / 1e9, "peak": 8000.0,
                                  "unit": "GB/s", "frac": 3.0 * M * K / (t_quant * 1e-3) / 1e9 / 8000.0},
        "context": "the paper reports no kernel-level number for its W8A8 Linear layers",
    }
    rates = measured_rates(torch, sla, torch.device("cuda:0"))   # what the matrix pipe and a device copy sustain by themselves
    result["measured_rates"] = rates
    result["roofline"]["mfma_alone"] = rates["mfma_int8_TOPs"]
    result["roofline"]["frac_of_mfma_alone"] = round(achieved / rates["mfma_int8_TOPs"], 4)
    if not args.no_cpu_baseline:
        from oracle import w8a8_oracle as wo      # cpu_baseline leg: allowed to call the oracle
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [os.cpu_count() or 1])
        except Exception:
            cores = os.cpu_count() or 1
        # the weight is quantised once, outside the timed part (as on the GPU); a small probe first,
        # then as many whole 128-token blocks as the time budget allows
        W8, sW = wo.quantize_blockwise(synth.as_f64(w))
        bs = synth.as_f64(b)

        def layer(nrows):
            X8, sX = wo.quantize_blockwise(synth.as_f64(x[:nrows]))
            return wo.linear_from_codes(X8, sX, W8, sW, bs)

        rows, cols = 256, N
        t0 = time.perf_counter()
        layer(rows)
        t_probe = time.perf_counter() - t0
        rows = int(min(M, max(256, args.cpu_seconds / max(t_probe, 1e-3) * 256)) // 128 * 128)
        t0 = time.perf_counter()
        layer(rows)
        t = time.perf_counter() - t0
        full = t * (M / rows) * (N / cols)
        result["cpu_baseline"] = {"value": ops / full / 1e12, "unit": "TOP/s", "cores": int(cores), "kind": "oracle",
                                  "sample": "%d tokens x %d outputs x all %d features in %.2f s; extrapolated to "
                                            "%d x %d = %.0f s" % (rows, cols, K, t, M, N, full)}
    return result


BWD_STAGE_NAMES = ("block_mask", "softmax_stats", "linear_branch", "dq", "dkv")
PEAK_MFMA_BF16_TFLOPS = 2500.0


def main_bwd(args):
    """One step = one backward pass of SLA (sla_attention_bwd): block mask, softmax
    statistics, linear-branch and projection gradients, dQ, dK and dV, for the same seeded inputs as
    the forward benchmark and a seeded upstream gradient."""
    import numpy as np
    import torch
    from paper_2512_16093_amd import binding as sla
    from paper_2512_16093_amd import synth

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    sla.lib()
    cfg = synth.CONFIGS[args.config]
    dev = torch.device("cuda:0")
    t0 = time.perf_counter()
    q, k, v = make_inputs(cfg, synth, torch)
    W = synth.make_proj(cfg)
    # the upstream gradient: the V tensor of another seed (same generator, same statistics)
    g = torch.Generator().manual_seed(11)
    dout = v[:, torch.randperm(cfg.H, generator=g)].flip(2).contiguous()
    print("[bench] inputs for %s generated in %.1f s" % (cfg.name, time.perf_counter() - t0), file=sys.stderr, flush=True)
    qd, kd, vd, dd = q.to(dev), k.to(dev), v.to(dev), dout.to(dev)
    Wd = None if W is None else W.to(dev)
    ws = sla.alloc_bwd_workspace(cfg.B, cfg.H, cfg.N, cfg.d, cfg.block_q, cfg.block_k, cfg.topk_ratio,
                                 cfg.marginal_ratio, dev)
    grads = tuple(torch.empty_like(qd) for _ in range(3))
    Tq, Tk, n_c, n_m = sla.sla_block_counts(cfg.N, cfg.block_q, cfg.block_k, cfg.topk_ratio, cfg.marginal_ratio)

    saved = None
    if args.saved_state:
        saved = sla.sla_attention_fwd_train(qd, kd, vd, cfg.block_q, cfg.block_k, cfg.topk_ratio, cfg.marginal_ratio,
                                            proj_w=Wd, workspace=ws, out=grads[0])[1]
        torch.cuda.synchronize()

    def step():
        return sla.sla_attention_bwd(qd, kd, vd, dd, cfg.block_q, cfg.block_k, cfg.topk_ratio, cfg.marginal_ratio,
                                     proj_w=Wd, want_dw=Wd is not None, want_db=Wd is not None, workspace=ws, grads=grads,
                                     saved=saved)

    if args.copy_calibration:
        copy_calibration(torch, dev)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    sla.sla_profile_enable(args.steps)
    sla.sla_profile_reset()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    stages = sla.sla_profile_read(args.steps)
    sla.sla_profile_enable(0)
    ms_per_step = dt / args.steps * 1e3
    stage_ms = [sum(r[s] for r in stages) / len(stages) for s in range(sla.N_STAGES)]
    # dense attention's backward is 2.5x its forward (five N x N x d products against two)
    flops = 10.0 * cfg.B * cfg.H * float(cfg.N) ** 2 * cfg.d
    pairs = cfg.B * cfg.H * Tq * n_c
    tile = 2.0 * cfg.block_q * cfg.block_k * cfg.d
    kernels = {"dkv": (4, stage_ms[4], "bwd_dkv_kernel"), "dq": (3, stage_ms[3], "bwd_dq_kernel")}
    dom = max(kernels, key=lambda n: kernels[n][1])
    n_prod, t_dom, kname = kernels[dom]
    ops = n_prod * tile * pairs
    achieved = ops / (t_dom * 1e-3) / 1e12
    result = {
        "metric": "sla_bwd_dense_equiv_tflops", "value": flops / (ms_per_step * 1e-3) / 1e12, "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16 (fp32 accumulate and statistics)", "data": "synthetic",
        "config": {"workload": "%s backward%s: B=%d H=%d N=%d d=%d block_q=%d block_k=%d critical=%.2f marginal=%.2f seed=0"
                               % (cfg.name, " (statistics from the forward pass)" if args.saved_state else "", cfg.B, cfg.H,
                                  cfg.N, cfg.d, cfg.block_q, cfg.block_k, cfg.topk_ratio, cfg.marginal_ratio),
                   "n_crit": n_c, "n_marg": n_m, "Tq": Tq, "Tk": Tk},
        "stage_ms": dict(zip(BWD_STAGE_NAMES, [round(x, 4) for x in stage_ms])),
        "roofline": {"kernel": kname, "bound": "mfma", "achieved": achieved, "peak": PEAK_MFMA_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": achieved / PEAK_MFMA_BF16_TFLOPS,
                     "traffic": (traffic_from_profile("sla_bwd_wan14b-720p.md", cfg.cfg_id)[0] if kname == "bwd_dkv_kernel" else None)
                                or BWD_TRAFFIC_BYTES.get((cfg.cfg_id, kname)), "traffic_unit": "bytes per launch",
                     "launch_ms": t_dom, "ops_per_launch": ops},
        "context": "the paper reports no number for its finetuning stage",
    }
    rates = measured_rates(torch, sla, dev)   # what the matrix pipe and a device copy sustain by themselves
    result["measured_rates"] = rates
    result["roofline"]["mfma_alone"] = rates["mfma_bf16_TFLOPs"]
    result["roofline"]["frac_of_mfma_alone"] = round(achieved / rates["mfma_bf16_TFLOPs"], 4)
    if not args.no_cpu_baseline:
        from oracle import sla_bwd_oracle as bo   # cpu_baseline leg: allowed to call the oracle
        from oracle import sla_oracle as so
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [os.cpu_count() or 1])
        except Exception:
            cores = os.cpu_count() or 1
        # the oracle works head by head on the whole sequence; a shorter sequence of the same
        # statistics (the first Ns tokens of head 0) is timed and scaled by the dense-equivalent work
        # (a short probe first, then a length that fills the time budget)
        def run(Ns):
            Qs, Ks, Vs, Ds = (synth.as_f64(t[0, 0, :Ns]) for t in (q, k, v, dout))
            Tq_s, Tk_s, nc_s, nm_s = so.block_counts(Ns, cfg.block_q, cfg.block_k, cfg.topk_ratio, cfg.marginal_ratio)
            mask = so.classify(so.pooled_scores(Qs, Ks, cfg.block_q, cfg.block_k), nc_s, nm_s)
            t0 = time.perf_counter()
            bo.sla_backward_head(Qs, Ks, Vs, Ds, mask, cfg.block_q, cfg.block_k,
                                 proj_w=None if W is None else synth.as_f64(W), has_bias=W is not None)
            return time.perf_counter() - t0

        t_probe = run(4096)
        Ns = int(min(cfg.N, 4096 * max(1.0, args.cpu_seconds / max(t_probe, 1e-3)) ** 0.5)) // 128 * 128
        t = run(Ns)
        full = t * cfg.B * cfg.H * (cfg.N / Ns) ** 2
        result["cpu_baseline"] = {"value": flops / full / 1e12, "unit": "TFLOP/s (dense-equivalent)", "cores": int(cores),
                                  "kind": "oracle",
                                  "sample": "one head of %d tokens (the first %d of head 0) in %.2f s; scaled by "
                                            "heads x (N / %d)^2 = %.0f s" % (Ns, Ns, t, Ns, full)}
    return result


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (heads would shard with "
              "no collective); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    if args.workload == "w8a8":
        print(json.dumps(main_w8a8(args)))
        return
    if args.workload == "sla_bwd":
        print(json.dumps(main_bwd(args)))
        return
    import torch
    from paper_2512_16093_amd import binding as sla
    from paper_2512_16093_amd import synth

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    sla.lib()   # fail loudly if the HIP library is not built
    cfg = synth.CONFIGS[args.config]
    dev = torch.device("cuda:0")
    t0 = time.perf_counter()
    q, k, v = make_inputs(cfg, synth, torch)
    W = synth.make_proj(cfg)
    print("[bench] inputs for %s generated in %.1f s" % (cfg.name, time.perf_counter() - t0), file=sys.stderr, flush=True)
    qd, kd, vd = q.to(dev), k.to(dev), v.to(dev)
    Wd = None if W is None else W.to(dev)
    if args.layout == "bnhd":
        # token-major memory, indexed [B,H,N,d] through permuted views (no copy at call time)
        qd, kd, vd = (t.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3) for t in (qd, kd, vd))
        out = torch.empty((cfg.B, cfg.N, cfg.H, cfg.d), dtype=torch.bfloat16, device=dev).permute(0, 2, 1, 3)
    else:
        out = torch.empty_like(qd)
    Tq, Tk, n_c, n_m = sla.sla_block_counts(cfg.N, cfg.block_q, cfg.block_k, cfg.topk_ratio, cfg.marginal_ratio)

    low_bit = args.quant == "int8fp8"
    qmode = {"int8fp8": sla.QUANT_QK_INT8_PV_FP8, "qk_int8": sla.QUANT_QK_INT8, "none": sla.QUANT_NONE}[args.quant]

    ws = sla.alloc_workspace(cfg.B, cfg.H, cfg.N, cfg.d, cfg.block_q, cfg.block_k, cfg.topk_ratio, cfg.marginal_ratio, dev,
                             quant_mode=qmode)

    def step():
        if args.layout == "bnhd":
            sla.sla_attention_fwd_strided(qd, kd, vd, out, cfg.block_q, cfg.block_k, cfg.topk_ratio,
                                          cfg.marginal_ratio, proj_w=Wd, workspace=ws, quant_mode=qmode)
        else:
            sla.sla_attention_fwd(qd, kd, vd, cfg.block_q, cfg.block_k, cfg.topk_ratio, cfg.marginal_ratio,
                                  proj_w=Wd, workspace=ws, out=out, quant_mode=qmode)

    if args.copy_calibration:
        copy_calibration(torch, dev)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    sla.sla_profile_enable(args.steps)
    sla.sla_profile_reset()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    stages = sla.sla_profile_read(args.steps)
    sla.sla_profile_enable(0)
    import statistics
    ms_wall_mean = dt / args.steps * 1e3
    # per call: the stages' HIP-event times on the launch stream; the step time is the MEDIAN call
    # (the mean over the wall clock of the whole timed region is reported beside it)
    call_ms = [sum(r) for r in stages]
    ms_per_step = statistics.median(call_ms) if call_ms else ms_wall_mean
    stage_mean = [sum(r[s] for r in stages) / len(stages) for s in range(sla.N_STAGES)]
    stage_ms = [statistics.median(r[s] for r in stages) for s in range(sla.N_STAGES)]

    flops = 4.0 * cfg.B * cfg.H * float(cfg.N) ** 2 * cfg.d
    value = flops / (ms_per_step * 1e-3) / 1e12
    # HBM-bound stages: algorithmic bytes (each operand once) over the stage's median time
    bhnd = float(cfg.B * cfg.H) * cfg.N * cfg.d
    hz_row = 129 * 128 * 2.0                      # one block summary: 128 x 128 + 128 bf16 values
    stage_bytes = {
        "pool_stats": 6.0 * bhnd + (1.0 * bhnd if args.quant != "none" else 0.0),  # Q, K, V read once (bf16); Q codes written
        "prep_kv": 4.0 * bhnd + (2.0 * bhnd if low_bit else 0.0) + (cfg.B * cfg.H * Tk * hz_row if n_m > 0 else 0.0),
        "lin_accumulate": cfg.B * cfg.H * (Tk + Tq) * hz_row if n_m > 0 else 0.0,  # summaries in once, sums out once
    }
    stage_hbm = {}
    for name, nbytes in stage_bytes.items():
        t = stage_ms[sla.STAGE_NAMES.index(name)]
        if nbytes > 0 and t > 0:
            gbps = nbytes / (t * 1e-3) / 1e9
            stage_hbm[name] = {"bytes": nbytes, "GBps": round(gbps, 1), "frac_of_8TBps": round(gbps / PEAK_HBM_GBPS, 4)}
    # sparse kernel: per (query block, critical key block) pair 2*bq*bk*d INT8 ops + as many FP8 flops
    pairs = cfg.B * cfg.H * Tq * n_c
    ops = 2.0 * (2.0 * cfg.block_q * cfg.block_k * cfg.d) * pairs
    t_sparse = stage_mean[4] * 1e-3           # the roofline takes the kernel's AVERAGE launch duration
    achieved = ops / t_sparse / 1e12
    peak = PEAK_MFMA_8BIT_TOPS if low_bit else PEAK_MFMA_BF16_TFLOPS
    traffic, traffic_src = traffic_from_profile({4: "sla_fwd_wan14b-720p.md", 2: "sla_fwd_dense-quant.md"}, cfg.cfg_id)
    if traffic is None and cfg.cfg_id in SPARSE_TRAFFIC_BYTES:
        traffic, traffic_src = SPARSE_TRAFFIC_BYTES[cfg.cfg_id], "constant in bench.py (from the same summary)"
    result = {
        "metric": "sla_fwd_dense_equiv_tflops", "value": value, "unit": "TFLOP/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "ms_per_step_kind": "median of the timed calls (HIP events)",
        "ms_per_step_wall_mean": ms_wall_mean, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None,
        "dtype": "int8/fp8-e4m3 (fp32 accumulate; bf16 linear branch)" if low_bit else
                 ("int8 codes carried as bf16 for Q.K^T, bf16 P.V (fp32 accumulate and softmax)" if args.quant == "qk_int8"
                  else "bf16 (fp32 accumulate and softmax)"),
        "data": "synthetic",
        "config": {"workload": "%s%s: B=%d H=%d N=%d d=%d block_q=%d block_k=%d critical=%.2f marginal=%.2f seed=0 layout=%s"
                               % (cfg.name, {"int8fp8": "", "qk_int8": " INT8 scores on the 16-bit pipe", "none": " unquantised"}[args.quant], cfg.B, cfg.H, cfg.N, cfg.d, cfg.block_q,
                                  cfg.block_k, cfg.topk_ratio, cfg.marginal_ratio,
                                  "[B,H,N,d]" if args.layout == "bhnd" else "[B,N,H,d]"),
                   "n_crit": n_c, "n_marg": n_m, "Tq": Tq, "Tk": Tk},
        "stage_ms": dict(zip(sla.STAGE_NAMES, [round(x, 4) for x in stage_ms])),
        "stage_hbm": stage_hbm,
        "roofline": {"kernel": "sparse_fwd_kernel" if low_bit else "bwd_stats_kernel<NW, true> (bf16 forward)",
                     "bound": "mfma", "achieved": achieved, "peak": peak, "unit": "TFLOP/s", "frac": achieved / peak,
                     "traffic": traffic if low_bit else None, "traffic_unit": "bytes per launch",
                     "traffic_source": traffic_src if low_bit else None,
                     "launch_ms": stage_mean[4], "launch_ms_median": stage_ms[4], "ops_per_launch": ops},
        "context": "paper: 100-200x end-to-end, 184 s -> 1.9 s on one RTX 5090 (whole pipeline; no kernel-level number)",
    }
    # beside the published peaks: what the matrix pipe and a device copy sustain on this chip by themselves
    rates = measured_rates(torch, sla, dev)
    result["measured_rates"] = rates
    if low_bit:  # half of the kernel's operations are INT8, half FP8: the harmonic mean of the two rates
        alone = 2.0 / (1.0 / rates["mfma_int8_TOPs"] + 1.0 / rates["mfma_fp8_TFLOPs"])
    else:
        alone = rates["mfma_bf16_TFLOPs"]
    result["roofline"]["mfma_alone"] = round(alone, 1)
    result["roofline"]["frac_of_mfma_alone"] = round(achieved / alone, 4)
    if not args.no_cpu_baseline:
        print("[bench] timing the CPU oracle sample ...", file=sys.stderr, flush=True)
        result["cpu_baseline"] = cpu_baseline(cfg, q, k, v, W, args.cpu_seconds, args.quant)
    if not args.only_headline and args.quant == "int8fp8" and args.layout == "bhnd" and cfg.cfg_id == 4:
        # The other two workloads of this file, timed in the same run (each is also a line of its own under
        # --workload): short runs, their own metrics; a failure there is reported and leaves the headline alone.
        del qd, kd, vd, out, ws
        torch.cuda.empty_cache()
        other = {}
        for name, fn, over in (("w8a8_linear", main_w8a8, {"workload": "w8a8", "steps": 20, "warmup": 3}),
                               ("sla_bwd", main_bwd, {"workload": "sla_bwd", "steps": 5, "warmup": 1})):
            a2 = argparse.Namespace(**vars(args))
            for key, val in over.items():
                setattr(a2, key, val)
            a2.no_cpu_baseline, a2.copy_calibration = True, False
            try:
                print("[bench] also timing %s ..." % name, file=sys.stderr, flush=True)
                r = fn(a2)
                other[name] = {k_: r[k_] for k_ in ("metric", "value", "unit", "steps", "warmup", "ms_per_step", "dtype", "config",
                                                    "stage_ms", "roofline") if k_ in r}
            except Exception as exc:   # (never takes the headline line down)
                other[name] = {"error": repr(exc)}
            torch.cuda.empty_cache()
        result["other_workloads"] = other
    print(json.dumps(result))


if __name__ == "__main__":
    main()
