"""ctypes binding of libsla.so: argument marshalling only.

Every function here has the name and the argument order of the C entry point
it calls (include/sla.h); tensors are PyTorch CUDA tensors used purely as
device memory, the stream is PyTorch's current stream.  No step of the path
runs in Python, and there is no fallback: if the library is missing or a call
returns an error status, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsla.so")

PHI_SOFTMAX, PHI_ELU1, PHI_RELU = 0, 1, 2
QUANT_NONE, QUANT_QK_INT8, QUANT_QK_INT8_PV_FP8 = 0, 1, 2

SLA_OK = 0
ERR_NULL, ERR_SHAPE, ERR_BLOCK, ERR_RATIO, ERR_WORKSPACE, ERR_UNSUPPORTED, ERR_HIP = -1, -2, -3, -4, -5, -6, -7
ERR_LAYOUT = -8
ERR_STATIC_LIMIT = -9
STATIC_SCRATCH_BYTES = 64 << 20

EXPORTS = ("sla_version", "sla_status_string", "sla_block_counts", "sla_workspace_bytes",
           "sla_attention_fwd", "sla_attention_fwd_strided", "sla_fwd_prepass", "sla_fwd_attend", "sla_classify_blocks", "sla_classify_blocks_static",
           "sla_sparse_attn_fwd",
           "sla_linear_attn_fwd", "sla_debug_e4m3_encode", "sla_debug_quantize_kv", "sla_debug_quantize_q", "sla_calibrate_mfma",
           "sla_profile_enable", "sla_profile_reset", "sla_profile_read")
W8A8_EXPORTS = ("w8a8_weight_bytes", "w8a8_quantize_weight", "w8a8_workspace_bytes", "w8a8_linear_fwd",
                "w8a8_quantize_act", "w8a8_gemm_fwd", "w8a8_debug_unpack")
BWD_EXPORTS = ("sla_bwd_workspace_bytes", "sla_attention_bwd", "sla_saved_bytes", "sla_attention_fwd_train",
               "sla_attention_bwd_saved", "sla_attention_fwd_train_strided", "sla_attention_bwd_strided")
N_STAGES = 5
STAGE_NAMES = ("pool_stats", "scores_select", "prep_kv", "lin_accumulate", "sparse_fwd")

_lib = None


class Strides(ctypes.Structure):
    """sla_strides of include/sla.h: element strides of the batch, head and token indices."""
    _fields_ = [("batch", ctypes.c_int64), ("head", ctypes.c_int64), ("token", ctypes.c_int64)]


class BwdStrides(ctypes.Structure):
    """sla_bwd_strides of include/sla_bwd.h: one layout (or NULL = contiguous) per tensor."""
    _fields_ = [(n, ctypes.POINTER(Strides)) for n in ("q", "k", "v", "dout", "dq", "dk", "dv")]


class SLAError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = lib().sla_status_string(status).decode()
        super().__init__("%s failed: %s (status %d)" % (where, msg, status))


def lib():
    """The loaded C-ABI library (opened on first use)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libsla.so is not built: run `python -m paper_2512_16093_amd.build` "
                               "(expected at %s)" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        c_int, c_dbl, c_vp, c_sz = ctypes.c_int, ctypes.c_double, ctypes.c_void_p, ctypes.c_size_t
        ip = ctypes.POINTER(ctypes.c_int)
        L.sla_version.restype = c_int
        L.sla_version.argtypes = []
        L.sla_status_string.restype = ctypes.c_char_p
        L.sla_status_string.argtypes = [c_int]
        L.sla_block_counts.restype = c_int
        L.sla_block_counts.argtypes = [c_int, c_int, c_int, c_dbl, c_dbl, ip, ip, ip, ip]
        L.sla_workspace_bytes.restype = c_sz
        L.sla_workspace_bytes.argtypes = [c_int] * 6 + [c_dbl, c_dbl, c_int]
        L.sla_attention_fwd.restype = c_int
        L.sla_attention_fwd.argtypes = [c_vp] * 4 + [c_int] * 6 + [c_dbl, c_dbl, c_vp, c_vp, c_int, c_int, c_vp, c_sz, c_vp]
        L.sla_attention_fwd_strided.restype = c_int
        L.sla_attention_fwd_strided.argtypes = ([c_vp] * 4 + [ctypes.POINTER(Strides)] * 4 + [c_int] * 6 +
                                                [c_dbl, c_dbl, c_vp, c_vp, c_int, c_int, c_vp, c_sz, c_vp])
        L.sla_fwd_prepass.restype = c_int
        L.sla_fwd_prepass.argtypes = [c_vp] * 3 + [ctypes.POINTER(Strides)] * 3 + [c_int] * 6 + [c_dbl, c_dbl, c_vp, c_int, c_vp, c_sz, c_vp]
        L.sla_fwd_attend.restype = c_int
        L.sla_fwd_attend.argtypes = [c_vp] * 2 + [ctypes.POINTER(Strides)] * 2 + [c_int] * 6 + [c_dbl, c_dbl, c_vp, c_int, c_vp, c_sz, c_vp]
        L.sla_classify_blocks.restype = c_int
        L.sla_classify_blocks.argtypes = [c_vp, c_vp] + [c_int] * 6 + [c_dbl, c_dbl] + [c_vp] * 4 + [c_vp, c_sz, c_vp]
        L.sla_classify_blocks_static.restype = c_int
        L.sla_classify_blocks_static.argtypes = [c_vp, c_vp] + [c_int] * 6 + [c_dbl, c_dbl] + [c_vp] * 4 + [c_vp]
        L.sla_sparse_attn_fwd.restype = c_int
        L.sla_sparse_attn_fwd.argtypes = [c_vp] * 4 + [c_int, c_vp, c_vp] + [c_int] * 7 + [c_vp, c_sz, c_vp]
        L.sla_linear_attn_fwd.restype = c_int
        L.sla_linear_attn_fwd.argtypes = [c_vp] * 6 + [c_int, c_vp] + [c_int] * 6 + [c_vp, c_sz, c_vp]
        L.sla_debug_e4m3_encode.restype = c_int
        L.sla_debug_e4m3_encode.argtypes = [c_vp, c_vp, c_sz, c_vp]
        L.sla_debug_quantize_q.restype = c_int
        L.sla_debug_quantize_q.argtypes = [c_vp] + [c_int] * 5 + [c_vp, c_vp] + [c_vp, c_sz, c_vp]
        L.sla_calibrate_mfma.restype = c_int
        L.sla_calibrate_mfma.argtypes = [c_int, c_int, c_vp, c_sz, ctypes.POINTER(ctypes.c_double), c_vp]
        L.sla_debug_quantize_kv.restype = c_int
        L.sla_debug_quantize_kv.argtypes = [c_vp, c_vp] + [c_int] * 5 + [c_vp] * 5 + [c_vp, c_sz, c_vp]
        L.sla_profile_enable.restype = c_int
        L.sla_profile_enable.argtypes = [c_int]
        L.sla_profile_reset.restype = c_int
        L.sla_profile_reset.argtypes = []
        L.sla_profile_read.restype = c_int
        L.sla_profile_read.argtypes = [ctypes.POINTER(ctypes.c_float), c_int, ip]
        # include/sla_bwd.h
        L.sla_bwd_workspace_bytes.restype = c_sz
        L.sla_bwd_workspace_bytes.argtypes = [c_int] * 6 + [c_dbl, c_dbl]
        L.sla_attention_bwd.restype = c_int
        L.sla_attention_bwd.argtypes = [c_vp] * 10 + [c_int] * 6 + [c_dbl, c_dbl, c_int, c_vp, c_sz, c_vp]
        L.sla_saved_bytes.restype = c_sz
        L.sla_saved_bytes.argtypes = [c_int] * 5
        L.sla_attention_fwd_train.restype = c_int
        L.sla_attention_fwd_train.argtypes = ([c_vp] * 4 + [c_int] * 6 + [c_dbl, c_dbl, c_vp, c_vp, c_int, c_vp, c_sz,
                                              c_vp, c_sz, c_vp])
        L.sla_attention_bwd_saved.restype = c_int
        L.sla_attention_bwd_saved.argtypes = ([c_vp] * 10 + [c_int] * 6 + [c_dbl, c_dbl, c_int, c_vp, c_sz, c_vp, c_sz,
                                              c_vp])
        sp = ctypes.POINTER(Strides)
        L.sla_attention_fwd_train_strided.restype = c_int
        L.sla_attention_fwd_train_strided.argtypes = ([c_vp] * 4 + [sp] * 4 + [c_int] * 6 + [c_dbl, c_dbl, c_vp, c_vp, c_int,
                                                      c_vp, c_sz, c_vp, c_sz, c_vp])
        L.sla_attention_bwd_strided.restype = c_int
        L.sla_attention_bwd_strided.argtypes = ([c_vp] * 10 + [ctypes.POINTER(BwdStrides)] + [c_int] * 6 +
                                                [c_dbl, c_dbl, c_int, c_vp, c_sz, c_vp, c_sz, c_vp])
        # include/w8a8.h
        L.w8a8_weight_bytes.restype = c_sz
        L.w8a8_weight_bytes.argtypes = [c_int, c_int]
        L.w8a8_workspace_bytes.restype = c_sz
        L.w8a8_workspace_bytes.argtypes = [c_int, c_int]
        L.w8a8_quantize_weight.restype = c_int
        L.w8a8_quantize_weight.argtypes = [c_vp, c_int, c_int, c_vp, c_vp]
        L.w8a8_linear_fwd.restype = c_int
        L.w8a8_linear_fwd.argtypes = [c_vp] * 4 + [c_int] * 3 + [c_vp, c_sz, c_vp]
        L.w8a8_quantize_act.restype = c_int
        L.w8a8_quantize_act.argtypes = [c_vp, c_int, c_int, c_vp, c_sz, c_vp]
        L.w8a8_gemm_fwd.restype = c_int
        L.w8a8_gemm_fwd.argtypes = [c_vp, c_sz, c_vp, c_vp, c_vp] + [c_int] * 3 + [c_vp]
        L.w8a8_debug_unpack.restype = c_int
        L.w8a8_debug_unpack.argtypes = [c_vp, c_int, c_int, c_int, c_vp, c_vp, c_vp]
        _lib = L
    return _lib


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(status, where):
    if status != SLA_OK:
        raise SLAError(status, where)


def _bf16_4d(*ts):
    B, H, N, d = ts[0].shape
    for t in ts:
        if t.dtype != torch.bfloat16 or not t.is_cuda or not t.is_contiguous() or tuple(t.shape) != (B, H, N, d):
            raise ValueError("expected contiguous CUDA bfloat16 tensors of one shape [B,H,N,d]")
    return B, H, N, d


def sla_version():
    return lib().sla_version()


def sla_status_string(status):
    return lib().sla_status_string(status).decode()


def sla_block_counts(N, block_q, block_k, topk_ratio, marginal_ratio):
    """(Tq, Tk, n_crit, n_marg); raises SLAError on invalid arguments."""
    vals = [ctypes.c_int(0) for _ in range(4)]
    st = lib().sla_block_counts(N, block_q, block_k, topk_ratio, marginal_ratio, *[ctypes.byref(v) for v in vals])
    _check(st, "sla_block_counts")
    return tuple(v.value for v in vals)


def sla_workspace_bytes(B, H, N, d, block_q, block_k, topk_ratio, marginal_ratio, quant_mode=QUANT_QK_INT8_PV_FP8):
    return lib().sla_workspace_bytes(B, H, N, d, block_q, block_k, topk_ratio, marginal_ratio, quant_mode)


def alloc_workspace(B, H, N, d, block_q, block_k, topk_ratio, marginal_ratio, device="cuda",
                    quant_mode=QUANT_QK_INT8_PV_FP8):
    """Device scratch of the size the library asks for (torch allocations are 256-byte aligned)."""
    nbytes = sla_workspace_bytes(B, H, N, d, block_q, block_k, topk_ratio, marginal_ratio, quant_mode)
    if nbytes == 0:
        raise ValueError("invalid problem for sla_workspace_bytes")
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def sla_attention_fwd(q, k, v, block_q, block_k, topk_ratio, marginal_ratio, proj_w=None, proj_b=None,
                      phi_kind=PHI_SOFTMAX, quant_mode=QUANT_QK_INT8_PV_FP8, workspace=None, out=None):
    B, H, N, d = _bf16_4d(q, k, v)
    if workspace is None:
        workspace = alloc_workspace(B, H, N, d, block_q, block_k, topk_ratio, marginal_ratio, q.device, quant_mode)
    if out is None:
        out = torch.empty_like(q)
    st = lib().sla_attention_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(out), B, H, N, d, block_q, block_k,
                                 topk_ratio, marginal_ratio, _ptr(proj_w), _ptr(proj_b), phi_kind, quant_mode,
                                 _ptr(workspace), workspace.numel(), _stream())
    _check(st, "sla_attention_fwd")
    return out


def sla_bwd_workspace_bytes(B, H, N, d, block_q, block_k, topk_ratio, marginal_ratio):
    return lib().sla_bwd_workspace_bytes(B, H, N, d, block_q, block_k, topk_ratio, marginal_ratio)


def alloc_bwd_workspace(B, H, N, d, block_q, block_k, topk_ratio, marginal_ratio, device="cuda"):
    nbytes = sla_bwd_workspace_bytes(B, H, N, d, block_q, block_k, topk_ratio, marginal_ratio)
    if nbytes == 0:
        raise ValueError("invalid problem for sla_bwd_workspace_bytes")
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def sla_saved_bytes(B, H, N, d, block_q):
    return lib().sla_saved_bytes(B, H, N, d, block_q)


def sla_attention_fwd_train(q, k, v, block_q, block_k, topk_ratio, marginal_ratio, proj_w=None, proj_b=None,
                            phi_kind=PHI_SOFTMAX, workspace=None, out=None, saved=None):
    """The unquantised forward pass that also keeps what the backward pass needs: returns (out, saved)."""
    B, H, N, d = _bf16_4d(q, k, v)
    if workspace is None:
        workspace = alloc_workspace(B, H, N, d, block_q, block_k, topk_ratio, marginal_ratio, q.device)
    if out is None:
        out = torch.empty_like(q)
    if saved is None:
        saved = torch.empty(sla_saved_bytes(B, H, N, d, block_q), dtype=torch.uint8, device=q.device)
    st = lib().sla_attention_fwd_train(_ptr(q), _ptr(k), _ptr(v), _ptr(out), B, H, N, d, block_q, block_k, topk_ratio,
                                       marginal_ratio, _ptr(proj_w), _ptr(proj_b), phi_kind, _ptr(saved), saved.numel(),
                                       _ptr(workspace), workspace.numel(), _stream())
    _check(st, "sla_attention_fwd_train")
    return out, saved


def sla_attention_bwd(q, k, v, dout, block_q, block_k, topk_ratio, marginal_ratio, proj_w=None, want_dw=False,
                      want_db=False, phi_kind=PHI_SOFTMAX, workspace=None, grads=None, saved=None):
    """Returns (dq, dk, dv, dproj_w or None, dproj_b or None); dq, dk, dv bf16 [B,H,N,d], the others fp32.
    `grads` may hand in preallocated (dq, dk, dv); `saved` is the state sla_attention_fwd_train returned
    for the same inputs (the statistics pass is then skipped)."""
    B, H, N, d = _bf16_4d(q, k, v, dout)
    if workspace is None:
        workspace = alloc_bwd_workspace(B, H, N, d, block_q, block_k, topk_ratio, marginal_ratio, q.device)
    dq, dk, dv = grads if grads is not None else (torch.empty_like(q), torch.empty_like(k), torch.empty_like(v))
    dw = torch.empty((d, d), dtype=torch.float32, device=q.device) if want_dw else None
    db = torch.empty((d,), dtype=torch.float32, device=q.device) if want_db else None
    if saved is None:
        st = lib().sla_attention_bwd(_ptr(q), _ptr(k), _ptr(v), _ptr(dout), _ptr(proj_w), _ptr(dq), _ptr(dk), _ptr(dv),
                                     _ptr(dw), _ptr(db), B, H, N, d, block_q, block_k, topk_ratio, marginal_ratio,
                                     phi_kind, _ptr(workspace), workspace.numel(), _stream())
    else:
        st = lib().sla_attention_bwd_saved(_ptr(q), _ptr(k), _ptr(v), _ptr(dout), _ptr(proj_w), _ptr(dq), _ptr(dk),
                                           _ptr(dv), _ptr(dw), _ptr(db), B, H, N, d, block_q, block_k, topk_ratio,
                                           marginal_ratio, phi_kind, _ptr(saved), saved.numel(), _ptr(workspace),
                                           workspace.numel(), _stream())
    _check(st, "sla_attention_bwd")
    return dq, dk, dv, dw, db


def _strides_of(t, what):
    """sla_strides of a [B,H,N,d]-indexed view (any memory order with contiguous channels)."""
    if t.dtype != torch.bfloat16 or not t.is_cuda or t.dim() != 4 or t.stride(3) != 1:
        raise ValueError("%s: expected a CUDA bfloat16 tensor indexed [B,H,N,d] with contiguous channels" % what)
    return Strides(t.stride(0), t.stride(1), t.stride(2))


def sla_attention_fwd_strided(q, k, v, out, block_q, block_k, topk_ratio, marginal_ratio, proj_w=None, proj_b=None,
                              phi_kind=PHI_SOFTMAX, quant_mode=QUANT_QK_INT8_PV_FP8, workspace=None):
    """q, k, v, out: tensors indexed [B,H,N,d] in any memory order with contiguous channels
    (e.g. `x.view(B, N, H, d).permute(0, 2, 1, 3)`); their strides are passed on as they are."""
    B, H, N, d = q.shape
    for t in (k, v, out):
        if tuple(t.shape) != (B, H, N, d):
            raise ValueError("q, k, v and out must have one shape [B,H,N,d]")
    sq, sk, sv, so_ = (_strides_of(t, n) for t, n in ((q, "q"), (k, "k"), (v, "v"), (out, "out")))
    if workspace is None:
        workspace = alloc_workspace(B, H, N, d, block_q, block_k, topk_ratio, marginal_ratio, q.device)
    st = lib().sla_attention_fwd_strided(_ptr(q), _ptr(k), _ptr(v), _ptr(out), ctypes.byref(sq), ctypes.byref(sk),
                                         ctypes.byref(sv), ctypes.byref(so_), B, H, N, d, block_q, block_k,
                                         topk_ratio, marginal_ratio, _ptr(proj_w), _ptr(proj_b), phi_kind,
                                         quant_mode, _ptr(workspace), workspace.numel(), _stream())
    _check(st, "sla_attention_fwd_strided")
    return out


def sla_classify_blocks(q, k, block_q, block_k, topk_ratio, marginal_ratio, want_scores=True, workspace=None):
    """Returns (mask int8 [B,H,Tq,Tk], crit_idx int32, marg_idx int32, pooled_scores fp32 or None)."""
    B, H, N, d = _bf16_4d(q, k)
    Tq, Tk, n_c, n_m = sla_block_counts(N, block_q, block_k, topk_ratio, marginal_ratio)
    if workspace is None:
        workspace = alloc_workspace(B, H, N, d, block_q, block_k, topk_ratio, marginal_ratio, q.device)
    dev = q.device
    mask = torch.empty((B, H, Tq, Tk), dtype=torch.int8, device=dev)
    crit = torch.empty((B, H, Tq, n_c), dtype=torch.int32, device=dev)
    marg = torch.empty((B, H, Tq, n_m), dtype=torch.int32, device=dev)
    scores = torch.empty((B, H, Tq, Tk), dtype=torch.float32, device=dev) if want_scores else None
    st = lib().sla_classify_blocks(_ptr(q), _ptr(k), B, H, N, d, block_q, block_k, topk_ratio, marginal_ratio,
                                   _ptr(mask), _ptr(crit), _ptr(marg) if n_m else None, _ptr(scores),
                                   _ptr(workspace), workspace.numel(), _stream())
    _check(st, "sla_classify_blocks")
    return mask, crit, marg, scores


def sla_classify_blocks_static(q, k, block_q, block_k, topk_ratio, marginal_ratio, mask, crit_idx, marg_idx,
                               pooled_scores=None):
    """sla_classify_blocks on the library's built-in scratch: the caller passes every output tensor
    (mask int8 [B,H,Tq,Tk], crit_idx / marg_idx int32, pooled_scores fp32 or None); nothing is allocated."""
    B, H, N, d = _bf16_4d(q, k)
    st = lib().sla_classify_blocks_static(_ptr(q), _ptr(k), B, H, N, d, block_q, block_k, topk_ratio, marginal_ratio,
                                          _ptr(mask), _ptr(crit_idx), _ptr(marg_idx), _ptr(pooled_scores), _stream())
    _check(st, "sla_classify_blocks_static")


def sla_sparse_attn_fwd(q, k, v, crit_idx, block_q, block_k, quant_mode=QUANT_QK_INT8_PV_FP8, want_lse=True,
                        workspace=None):
    """Returns (out_s fp32 [B,H,N,d], lse fp32 [B,H,N] or None)."""
    B, H, N, d = _bf16_4d(q, k, v)
    if crit_idx.dtype != torch.int32 or not crit_idx.is_contiguous() or crit_idx.dim() != 4:
        raise ValueError("crit_idx must be a contiguous int32 tensor [B,H,Tq,n_crit]")
    n_c = crit_idx.shape[-1]
    if workspace is None:
        workspace = alloc_workspace(B, H, N, d, block_q, block_k, 1.0, 0.0, q.device)
    out = torch.empty((B, H, N, d), dtype=torch.float32, device=q.device)
    lse = torch.empty((B, H, N), dtype=torch.float32, device=q.device) if want_lse else None
    st = lib().sla_sparse_attn_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(crit_idx), n_c, _ptr(out), _ptr(lse),
                                   B, H, N, d, block_q, block_k, quant_mode, _ptr(workspace), workspace.numel(),
                                   _stream())
    _check(st, "sla_sparse_attn_fwd")
    return out, lse


def sla_linear_attn_fwd(q, k, v, mask, block_q, block_k, proj_w=None, proj_b=None, phi_kind=PHI_SOFTMAX,
                        workspace=None):
    """Returns out_l fp32 [B,H,N,d] = O_l W^T (+ b)."""
    B, H, N, d = _bf16_4d(q, k, v)
    if mask.dtype != torch.int8 or not mask.is_contiguous():
        raise ValueError("mask must be a contiguous int8 tensor [B,H,Tq,Tk]")
    if workspace is None:
        workspace = alloc_workspace(B, H, N, d, block_q, block_k, 1.0, 0.0, q.device)
    out = torch.empty((B, H, N, d), dtype=torch.float32, device=q.device)
    st = lib().sla_linear_attn_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(mask), _ptr(proj_w), _ptr(proj_b), phi_kind,
                                   _ptr(out), B, H, N, d, block_q, block_k, _ptr(workspace), workspace.numel(),
                                   _stream())
    _check(st, "sla_linear_attn_fwd")
    return out


def sla_debug_e4m3_encode(x):
    """uint8 E4M3 codes of a CUDA float32 tensor."""
    x = x.contiguous()
    out = torch.empty(x.shape, dtype=torch.uint8, device=x.device)
    _check(lib().sla_debug_e4m3_encode(_ptr(x), _ptr(out), x.numel(), _stream()), "sla_debug_e4m3_encode")
    return out


MFMA_KINDS = {"int8": 0, "fp8": 1, "bf16": 2}


def sla_calibrate_mfma(kind, iters, scratch):
    """Enqueues the matrix-pipe-only loop of one instruction kind ("int8", "fp8", "bf16") on the current stream;
    returns the number of operations the launch performs (the caller times it)."""
    ops = ctypes.c_double(0.0)
    _check(lib().sla_calibrate_mfma(MFMA_KINDS[kind], iters, _ptr(scratch), scratch.numel() * scratch.element_size(),
                                    ctypes.byref(ops), _stream()), "sla_calibrate_mfma")
    return ops.value


def sla_debug_quantize_kv(k, v, block_k=64, workspace=None):
    """Returns (k_codes int8 [B,H,N,d], k_scale [B,H,Tk], k_mean [B,H,d], v_codes uint8, v_scale [B,H,d])."""
    B, H, N, d = _bf16_4d(k, v)
    Tk = -(-N // block_k)
    if workspace is None:
        workspace = alloc_workspace(B, H, N, d, 64, block_k, 1.0, 0.0, k.device)
    dev = k.device
    kc = torch.empty((B, H, N, d), dtype=torch.int8, device=dev)
    ks = torch.empty((B, H, Tk), dtype=torch.float32, device=dev)
    km = torch.empty((B, H, d), dtype=torch.float32, device=dev)
    vc = torch.empty((B, H, N, d), dtype=torch.uint8, device=dev)
    vs = torch.empty((B, H, d), dtype=torch.float32, device=dev)
    st = lib().sla_debug_quantize_kv(_ptr(k), _ptr(v), B, H, N, d, block_k, _ptr(kc), _ptr(ks), _ptr(km),
                                     _ptr(vc), _ptr(vs), _ptr(workspace), workspace.numel(), _stream())
    _check(st, "sla_debug_quantize_kv")
    return kc, ks, km, vc, vs


def sla_debug_quantize_q(q, block_q=128, workspace=None):
    """Returns (q_codes int8 [B,H,N,d], q_scale fp32 [B,H,Tq])."""
    B, H, N, d = _bf16_4d(q)
    Tq = -(-N // block_q)
    if workspace is None:
        workspace = alloc_workspace(B, H, N, d, block_q, 64, 1.0, 0.0, q.device)
    qc = torch.empty((B, H, N, d), dtype=torch.int8, device=q.device)
    qs = torch.empty((B, H, Tq), dtype=torch.float32, device=q.device)
    st = lib().sla_debug_quantize_q(_ptr(q), B, H, N, d, block_q, _ptr(qc), _ptr(qs), _ptr(workspace), workspace.numel(),
                                    _stream())
    _check(st, "sla_debug_quantize_q")
    return qc, qs


def sla_profile_enable(max_calls):
    _check(lib().sla_profile_enable(max_calls), "sla_profile_enable")


def sla_profile_reset():
    _check(lib().sla_profile_reset(), "sla_profile_reset")


def sla_profile_read(max_calls):
    """Per-call stage times in ms: list of N_STAGES-long lists (waits for the calls to finish)."""
    buf = (ctypes.c_float * (max_calls * N_STAGES))()
    n = ctypes.c_int(0)
    _check(lib().sla_profile_read(buf, max_calls, ctypes.byref(n)), "sla_profile_read")
    return [[buf[r * N_STAGES + s] for s in range(N_STAGES)] for r in range(n.value)]


# ---------------------------------------------------------------------------
# include/w8a8.h
# ---------------------------------------------------------------------------
def _bf16_2d(t, what):
    if t.dtype != torch.bfloat16 or not t.is_cuda or t.dim() != 2 or not t.is_contiguous():
        raise ValueError("%s: expected a contiguous 2-D CUDA bfloat16 tensor" % what)
    return t.shape


def w8a8_weight_bytes(N, K):
    return lib().w8a8_weight_bytes(N, K)


def w8a8_workspace_bytes(M, K):
    return lib().w8a8_workspace_bytes(M, K)


def w8a8_quantize_weight(w):
    """The quantised weight object (a uint8 tensor) of a bf16 weight [N, K]."""
    N, K = _bf16_2d(w, "w")
    nbytes = w8a8_weight_bytes(N, K)
    if nbytes == 0:
        raise ValueError("unsupported weight shape [%d, %d]" % (N, K))
    wq = torch.empty(nbytes, dtype=torch.uint8, device=w.device)
    _check(lib().w8a8_quantize_weight(_ptr(w), N, K, _ptr(wq), _stream()), "w8a8_quantize_weight")
    return wq


def w8a8_alloc_workspace(M, K, device="cuda"):
    nbytes = w8a8_workspace_bytes(M, K)
    if nbytes == 0:
        raise ValueError("unsupported activation shape [%d, %d]" % (M, K))
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def w8a8_linear_fwd(x, wq, N, bias=None, workspace=None, out=None):
    """y bf16 [M, N] = W8A8-linear(x bf16 [M, K]) with the weight object `wq` of an [N, K] weight."""
    M, K = _bf16_2d(x, "x")
    if workspace is None:
        workspace = w8a8_alloc_workspace(M, K, x.device)
    if out is None:
        out = torch.empty((M, N), dtype=torch.bfloat16, device=x.device)
    st = lib().w8a8_linear_fwd(_ptr(x), _ptr(wq), _ptr(bias), _ptr(out), M, N, K, _ptr(workspace),
                               workspace.numel(), _stream())
    _check(st, "w8a8_linear_fwd")
    return out


def w8a8_quantize_act(x, workspace=None):
    M, K = _bf16_2d(x, "x")
    if workspace is None:
        workspace = w8a8_alloc_workspace(M, K, x.device)
    _check(lib().w8a8_quantize_act(_ptr(x), M, K, _ptr(workspace), workspace.numel(), _stream()), "w8a8_quantize_act")
    return workspace


def w8a8_gemm_fwd(workspace, wq, M, N, K, bias=None, out=None):
    if out is None:
        out = torch.empty((M, N), dtype=torch.bfloat16, device=workspace.device)
    st = lib().w8a8_gemm_fwd(_ptr(workspace), workspace.numel(), _ptr(wq), _ptr(bias), _ptr(out), M, N, K, _stream())
    _check(st, "w8a8_gemm_fwd")
    return out


def w8a8_debug_unpack(q, is_weight, R, K):
    """(codes int8 [R, K], scales fp32 [ceil(R/128), K/128]) held by a weight object or a filled workspace."""
    codes = torch.empty((R, K), dtype=torch.int8, device=q.device)
    scales = torch.empty((-(-R // 128), K // 128), dtype=torch.float32, device=q.device)
    _check(lib().w8a8_debug_unpack(_ptr(q), 1 if is_weight else 0, R, K, _ptr(codes), _ptr(scales), _stream()),
           "w8a8_debug_unpack")
    return codes, scales


def _same_shape(*ts):
    B, H, N, d = ts[0].shape
    for t in ts:
        if tuple(t.shape) != (B, H, N, d):
            raise ValueError("all tensors must be indexed [B,H,N,d] with one shape")
    return B, H, N, d


def sla_attention_fwd_train_strided(q, k, v, out, block_q, block_k, topk_ratio, marginal_ratio, proj_w=None, proj_b=None,
                                    phi_kind=PHI_SOFTMAX, workspace=None, saved=None):
    """sla_attention_fwd_train on tensors indexed [B,H,N,d] in any memory order with contiguous channels;
    returns saved."""
    B, H, N, d = _same_shape(q, k, v, out)
    st_ = [_strides_of(t, n) for t, n in ((q, "q"), (k, "k"), (v, "v"), (out, "out"))]
    if workspace is None:
        workspace = alloc_workspace(B, H, N, d, block_q, block_k, topk_ratio, marginal_ratio, q.device)
    if saved is None:
        saved = torch.empty(sla_saved_bytes(B, H, N, d, block_q), dtype=torch.uint8, device=q.device)
    st = lib().sla_attention_fwd_train_strided(_ptr(q), _ptr(k), _ptr(v), _ptr(out), *[ctypes.byref(x) for x in st_],
                                               B, H, N, d, block_q, block_k, topk_ratio, marginal_ratio, _ptr(proj_w),
                                               _ptr(proj_b), phi_kind, _ptr(saved), saved.numel(), _ptr(workspace),
                                               workspace.numel(), _stream())
    _check(st, "sla_attention_fwd_train_strided")
    return saved


def sla_attention_bwd_strided(q, k, v, dout, dq, dk, dv, block_q, block_k, topk_ratio, marginal_ratio, proj_w=None,
                              want_dw=False, want_db=False, phi_kind=PHI_SOFTMAX, workspace=None, saved=None):
    """sla_attention_bwd(_saved) on tensors indexed [B,H,N,d] in any memory order with contiguous channels;
    dq, dk, dv are written in place; returns (dproj_w or None, dproj_b or None)."""
    B, H, N, d = _same_shape(q, k, v, dout, dq, dk, dv)
    names = ("q", "k", "v", "dout", "dq", "dk", "dv")
    each = [_strides_of(t, n) for t, n in zip((q, k, v, dout, dq, dk, dv), names)]
    bs = BwdStrides(*[ctypes.pointer(x) for x in each])
    if workspace is None:
        workspace = alloc_bwd_workspace(B, H, N, d, block_q, block_k, topk_ratio, marginal_ratio, q.device)
    dw = torch.empty((d, d), dtype=torch.float32, device=q.device) if want_dw else None
    db = torch.empty((d,), dtype=torch.float32, device=q.device) if want_db else None
    st = lib().sla_attention_bwd_strided(_ptr(q), _ptr(k), _ptr(v), _ptr(dout), _ptr(proj_w), _ptr(dq), _ptr(dk), _ptr(dv),
                                         _ptr(dw), _ptr(db), ctypes.byref(bs), B, H, N, d, block_q, block_k, topk_ratio,
                                         marginal_ratio, phi_kind, _ptr(saved), 0 if saved is None else saved.numel(),
                                         _ptr(workspace), workspace.numel(), _stream())
    _check(st, "sla_attention_bwd_strided")
    return dw, db


def sla_fwd_prepass(q, k, v, block_q, block_k, topk_ratio, marginal_ratio, workspace, proj_w=None, phi_kind=PHI_SOFTMAX):
    """The K/V-side part of the low-bit forward pass; leaves its results in `workspace` for sla_fwd_attend.
    Tensors indexed [B,H,N,d] in any memory order with contiguous channels."""
    B, H, N, d = _same_shape(q, k, v)
    sq, sk, sv = (_strides_of(t, n) for t, n in ((q, "q"), (k, "k"), (v, "v")))
    st = lib().sla_fwd_prepass(_ptr(q), _ptr(k), _ptr(v), ctypes.byref(sq), ctypes.byref(sk), ctypes.byref(sv), B, H, N, d,
                               block_q, block_k, topk_ratio, marginal_ratio, _ptr(proj_w), phi_kind, _ptr(workspace),
                               workspace.numel(), _stream())
    _check(st, "sla_fwd_prepass")


def sla_fwd_attend(q, out, block_q, block_k, topk_ratio, marginal_ratio, workspace, proj_b=None, phi_kind=PHI_SOFTMAX):
    """The attention kernel on a workspace sla_fwd_prepass filled for the same q and parameters."""
    B, H, N, d = _same_shape(q, out)
    sq, so_ = _strides_of(q, "q"), _strides_of(out, "out")
    st = lib().sla_fwd_attend(_ptr(q), _ptr(out), ctypes.byref(sq), ctypes.byref(so_), B, H, N, d, block_q, block_k,
                              topk_ratio, marginal_ratio, _ptr(proj_b), phi_kind, _ptr(workspace), workspace.numel(), _stream())
    _check(st, "sla_fwd_attend")
