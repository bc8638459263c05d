"""Host-side checks of the C-ABI library (no GPU needed): it loads, exports every
symbol include/sla.h declares, its host-only functions agree with the oracle's
block bookkeeping, and every argument error is reported before any launch.
"""
import ctypes
import os
import re

import pytest

from oracle import sla_oracle as so
from paper_2512_16093_amd import binding as sla

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = ctypes.c_void_p(0x1000)      # non-NULL, never dereferenced: validation fails first
WS = ctypes.c_void_p(0x10000)       # 256-byte aligned fake workspace


def _declared(header="sla.h", prefix="sla_"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(%s[a-z0-9_]+)\s*\(" % prefix, text)))


def test_library_exports_every_declared_symbol():
    L = sla.lib()
    names = _declared()
    assert set(names) == set(sla.EXPORTS)
    for n in names:
        assert hasattr(L, n), n
    assert sla.sla_version() >= 100
    names = _declared("w8a8.h", "w8a8_")
    assert set(names) == set(sla.W8A8_EXPORTS)
    for n in names:
        assert hasattr(L, n), n
    names = [n for n in _declared("sla_bwd.h") if n not in sla.EXPORTS]   # (its comments name forward entry points)
    assert set(names) == set(sla.BWD_EXPORTS)
    for n in names:
        assert hasattr(L, n), n


def test_backward_sizes_and_argument_errors():
    L = sla.lib()
    fwd = sla.sla_workspace_bytes(1, 2, 1000, 128, 128, 64, 0.25, 0.5)
    bwd = sla.sla_bwd_workspace_bytes(1, 2, 1000, 128, 128, 64, 0.25, 0.5)
    # the forward map plus the row statistics, the linear branch's fp32 share of dQ and the summaries' gradients
    assert bwd > fwd + 2 * 2 * 1024 * 4 + 2 * 1000 * 128 * 4 + 2 * 8 * 129 * 128 * 2
    assert sla.sla_bwd_workspace_bytes(1, 2, 1000, 64, 128, 64, 0.25, 0.5) == 0
    assert sla.sla_bwd_workspace_bytes(1, 2, 1000, 128, 96, 64, 0.25, 0.5) == 0
    big = 1 << 44
    args = lambda **kw: [kw.get("q", FAKE), FAKE, FAKE, kw.get("dout", FAKE), None, FAKE, FAKE, kw.get("dv", FAKE), None, None,
                         1, 2, kw.get("N", 1000), kw.get("d", 128), kw.get("bq", 128), 64, kw.get("rc", 0.25), 0.5,
                         kw.get("phi", 0), kw.get("ws", WS), kw.get("bytes", big), None]
    assert L.sla_attention_bwd(*args(q=None)) == sla.ERR_NULL
    assert L.sla_attention_bwd(*args(dout=None)) == sla.ERR_NULL
    assert L.sla_attention_bwd(*args(dv=None)) == sla.ERR_NULL
    assert L.sla_attention_bwd(*args(d=64)) == sla.ERR_SHAPE
    assert L.sla_attention_bwd(*args(bq=32)) == sla.ERR_BLOCK
    assert L.sla_attention_bwd(*args(rc=0.0)) == sla.ERR_RATIO
    assert L.sla_attention_bwd(*args(phi=3)) == sla.ERR_UNSUPPORTED          # not a feature map
    assert L.sla_attention_bwd(*args(ws=None)) == sla.ERR_WORKSPACE
    assert L.sla_attention_bwd(*args(bytes=bwd - 1)) == sla.ERR_WORKSPACE
    # the saved state: a 256-byte header, padded per-row statistics, a bf16 copy of O^s
    sv = sla.sla_saved_bytes(1, 2, 1000, 128, 128)
    assert sv == 256 + (2 * 1024 * 4 + 255) // 256 * 256 + (2 * 1000 * 128 * 2 + 255) // 256 * 256
    assert sla.sla_saved_bytes(1, 2, 1000, 64, 128) == 0 and sla.sla_saved_bytes(1, 2, 1000, 128, 96) == 0
    a = args()
    assert L.sla_attention_bwd_saved(*a[:19], WS, sv - 1, *a[19:]) == sla.ERR_WORKSPACE
    assert L.sla_attention_bwd_saved(*a[:19], ctypes.c_void_p(0x10010), sv, *a[19:]) == sla.ERR_WORKSPACE
    f = [FAKE, FAKE, FAKE, FAKE, 1, 2, 1000, 128, 128, 64, 0.25, 0.5, None, None, 0]
    assert L.sla_attention_fwd_train(*f, None, sv, WS, big, None) == sla.ERR_NULL
    assert L.sla_attention_fwd_train(*f, WS, sv - 1, WS, big, None) == sla.ERR_WORKSPACE
    assert L.sla_attention_fwd_train(*f, WS, sv, WS, 16, None) == sla.ERR_WORKSPACE
    assert L.sla_attention_fwd_train(*(f[:14] + [9]), WS, sv, WS, big, None) == sla.ERR_UNSUPPORTED


def test_strided_training_entry_points_check_layouts_on_the_host():
    L = sla.lib()
    big = 1 << 44
    bad = sla.Strides(2 * 1000 * 128, 1000 * 128, 100)            # token stride below d
    odd = sla.Strides(2 * 1000 * 128 + 4, 1000 * 128, 128)        # not a multiple of 8 elements
    sv = sla.sla_saved_bytes(1, 2, 1000, 128, 128)
    f = lambda qs: L.sla_attention_fwd_train_strided(FAKE, FAKE, FAKE, FAKE, qs, None, None, None, 1, 2, 1000, 128, 128, 64,
                                                     0.25, 0.5, None, None, 0, WS, sv, WS, big, None)
    assert f(ctypes.byref(bad)) == sla.ERR_LAYOUT and f(ctypes.byref(odd)) == sla.ERR_LAYOUT
    bs = sla.BwdStrides(None, None, None, None, None, ctypes.pointer(bad), None)
    g = lambda st, q=FAKE: L.sla_attention_bwd_strided(q, FAKE, FAKE, FAKE, None, FAKE, FAKE, FAKE, None, None, st, 1, 2, 1000,
                                                       128, 128, 64, 0.25, 0.5, 0, None, 0, WS, big, None)
    assert g(ctypes.byref(bs)) == sla.ERR_LAYOUT
    assert g(None, q=None) == sla.ERR_NULL


def test_two_call_forward_argument_errors():
    L = sla.lib()
    big = 1 << 44
    pre = lambda **kw: L.sla_fwd_prepass(kw.get("q", FAKE), FAKE, FAKE, None, None, None, 1, 2, kw.get("N", 1000), 128,
                                         kw.get("bq", 128), 64, 0.25, 0.5, None, kw.get("phi", 0), kw.get("ws", WS),
                                         kw.get("bytes", big), None)
    att = lambda **kw: L.sla_fwd_attend(FAKE, kw.get("out", FAKE), None, None, 1, 2, 1000, 128, 128, 64, kw.get("rc", 0.25),
                                        0.5, None, 0, kw.get("ws", WS), kw.get("bytes", big), None)
    assert pre(q=None) == sla.ERR_NULL and pre(N=0) == sla.ERR_SHAPE and pre(bq=96) == sla.ERR_BLOCK
    assert pre(phi=5) == sla.ERR_UNSUPPORTED and pre(ws=None) == sla.ERR_WORKSPACE and pre(bytes=64) == sla.ERR_WORKSPACE
    assert att(out=None) == sla.ERR_NULL and att(rc=2.0) == sla.ERR_RATIO and att(bytes=64) == sla.ERR_WORKSPACE


def test_static_scratch_entry_point_argument_errors():
    # sla_classify_blocks_static: every refusal happens on the host, before the GPU is touched
    L = sla.lib()
    call = lambda **kw: L.sla_classify_blocks_static(kw.get("q", FAKE), FAKE, 1, kw.get("H", 2), kw.get("N", 1000),
                                                     kw.get("d", 128), kw.get("bq", 128), 64, kw.get("rc", 0.25), 0.5,
                                                     kw.get("mask", FAKE), None, None, kw.get("scores"), None)
    assert call(q=None) == sla.ERR_NULL and call(mask=None) == sla.ERR_NULL
    assert call(d=64) == sla.ERR_SHAPE and call(bq=32) == sla.ERR_BLOCK and call(rc=1.5) == sla.ERR_RATIO
    # the Wan-14B-720P shape needs 148 MiB with the scores inside, 36 MiB with the caller holding them
    assert call(H=40, N=75600) == sla.ERR_STATIC_LIMIT
    assert call(H=80, N=75600, scores=FAKE) == sla.ERR_STATIC_LIMIT
    assert sla.STATIC_SCRATCH_BYTES == 64 << 20
    assert b"SLA_STATIC_SCRATCH_BYTES" in L.sla_status_string(sla.ERR_STATIC_LIMIT)


def test_w8a8_sizes_and_argument_errors():
    L = sla.lib()
    # weight object and workspace: one byte per code (activations padded to 256-token tiles) plus scales
    assert sla.w8a8_weight_bytes(5120, 5120) == 5120 * 5120 + 40 * 40 * 4
    assert sla.w8a8_weight_bytes(256, 128) == 256 * 128 + 256
    assert sla.w8a8_workspace_bytes(75600, 5120) == 75776 * 5120 + (592 * 40 * 4 + 255) // 256 * 256
    assert sla.w8a8_workspace_bytes(1, 128) == 256 * 128 + 256
    for bad in ((100, 128), (128, 100), (128, 64), (0, 128), (128, 1 << 17)):
        assert sla.w8a8_weight_bytes(*bad) == 0
    for bad in ((0, 128), (5, 100), (5, 0), ((1 << 22) + 1, 128)):
        assert sla.w8a8_workspace_bytes(*bad) == 0
    big = 1 << 40
    assert L.w8a8_quantize_weight(None, 128, 128, WS, None) == sla.ERR_NULL
    assert L.w8a8_quantize_weight(FAKE, 100, 128, WS, None) == sla.ERR_SHAPE
    assert L.w8a8_quantize_weight(FAKE, 128, 128, ctypes.c_void_p(0x10010), None) == sla.ERR_WORKSPACE
    assert L.w8a8_quantize_act(None, 5, 128, WS, big, None) == sla.ERR_NULL
    assert L.w8a8_quantize_act(FAKE, 5, 130, WS, big, None) == sla.ERR_SHAPE
    assert L.w8a8_quantize_act(FAKE, 5, 128, WS, 16, None) == sla.ERR_WORKSPACE
    assert L.w8a8_quantize_act(FAKE, 5, 128, None, big, None) == sla.ERR_WORKSPACE
    assert L.w8a8_gemm_fwd(WS, big, None, None, FAKE, 5, 128, 128, None) == sla.ERR_NULL
    assert L.w8a8_gemm_fwd(WS, big, WS, None, FAKE, 5, 100, 128, None) == sla.ERR_SHAPE
    assert L.w8a8_gemm_fwd(WS, 16, WS, None, FAKE, 5, 128, 128, None) == sla.ERR_WORKSPACE
    assert L.w8a8_gemm_fwd(WS, big, WS, None, ctypes.c_void_p(0x1008), 5, 128, 128, None) == sla.ERR_LAYOUT
    assert L.w8a8_linear_fwd(FAKE, WS, None, None, 5, 128, 128, WS, big, None) == sla.ERR_NULL
    assert L.w8a8_linear_fwd(FAKE, WS, None, FAKE, 5, 128, 256 + 64, WS, big, None) == sla.ERR_SHAPE
    assert L.w8a8_linear_fwd(FAKE, WS, None, FAKE, 5, 128, 128, WS, 100, None) == sla.ERR_WORKSPACE
    assert L.w8a8_debug_unpack(None, 1, 128, 128, None, None, None) == sla.ERR_NULL
    assert L.w8a8_debug_unpack(FAKE, 1, 100, 128, None, None, None) == sla.ERR_SHAPE


def test_status_strings():
    seen = set()
    for st in range(0, -9, -1):
        s = sla.sla_status_string(st)
        assert s and s != "unknown status"
        seen.add(s)
    assert len(seen) == 9 and sla.sla_status_string(-99) == "unknown status"


@pytest.mark.parametrize("N,bq,bk,rc,rm", [
    (1024, 64, 64, 0.2, 0.4), (32760, 128, 64, 0.1, 0.2), (75600, 128, 64, 0.1, 0.2),
    (32760, 128, 64, 1.0, 0.0), (100, 64, 64, 0.5, 0.5), (65, 128, 64, 0.1, 0.9),
    (75600, 128, 64, 0.15, 0.85), (4096, 64, 64, 0.3, 0.3), (1, 64, 64, 0.1, 0.0)])
def test_block_counts_match_oracle(N, bq, bk, rc, rm):
    assert sla.sla_block_counts(N, bq, bk, rc, rm) == so.block_counts(N, bq, bk, rc, rm)


def test_block_count_errors():
    L = sla.lib()
    f = L.sla_block_counts
    assert f(0, 64, 64, 0.1, 0.2, None, None, None, None) == sla.ERR_SHAPE
    assert f(64 * 8193, 64, 64, 0.1, 0.2, None, None, None, None) == sla.ERR_SHAPE
    assert f(1024, 32, 64, 0.1, 0.2, None, None, None, None) == sla.ERR_BLOCK
    assert f(1024, 64, 128, 0.1, 0.2, None, None, None, None) == sla.ERR_BLOCK
    for rc, rm in ((0.0, 0.1), (-0.1, 0.1), (1.1, 0.0), (0.5, -0.1), (0.5, 1.5), (0.7, 0.4), (float("nan"), 0.1)):
        assert f(1024, 64, 64, rc, rm, None, None, None, None) == sla.ERR_RATIO
    assert f(1024, 64, 64, 0.1, 0.2, None, None, None, None) == sla.SLA_OK


def test_workspace_bytes():
    w0 = sla.sla_workspace_bytes(1, 2, 1024, 128, 64, 64, 0.2, 0.4)
    assert w0 > 0 and w0 % 256 == 0
    # grows with the problem; at the headline shape it holds the 8-bit K/V copies and the
    # summaries, a few GB, far below the 288 GB of the device
    w4 = sla.sla_workspace_bytes(1, 40, 75600, 128, 128, 64, 0.1, 0.2)
    assert 2 * 40 * 75600 * 128 < w4 < 8e9
    assert sla.sla_workspace_bytes(1, 4, 1024, 128, 64, 64, 0.2, 0.4) > w0
    # the stage entry points accept the smallest workspace of a shape
    assert sla.sla_workspace_bytes(1, 2, 1024, 128, 64, 64, 1e-6, 0.0) <= w0
    for bad in ((0, 2, 1024, 128, 64, 64, 0.2, 0.4), (1, 2, 1024, 64, 64, 64, 0.2, 0.4),
                (1, 2, 1024, 128, 96, 64, 0.2, 0.4), (1, 2, 1024, 128, 64, 64, 0.0, 0.4)):
        assert sla.sla_workspace_bytes(*bad) == 0
    assert sla.sla_workspace_bytes(1, 2, 1024, 128, 64, 64, 0.2, 0.4, sla.QUANT_NONE) == w0   # the 16-bit path: same map
    # the INT8-scores mode adds the two 16-bit code tensors
    assert sla.sla_workspace_bytes(1, 2, 1024, 128, 64, 64, 0.2, 0.4, sla.QUANT_QK_INT8) == w0 + 2 * 2 * 1024 * 128 * 2
    assert sla.sla_workspace_bytes(1, 2, 1024, 128, 64, 64, 0.2, 0.4, 3) == 0


def _fwd(q=FAKE, k=FAKE, v=FAKE, out=FAKE, B=1, H=2, N=1024, d=128, bq=64, bk=64, rc=0.2, rm=0.4,
         phi=0, quant=2, ws=WS, wsb=1 << 40):
    return sla.lib().sla_attention_fwd(q, k, v, out, B, H, N, d, bq, bk, rc, rm, None, None, phi, quant,
                                       ws, wsb, None)


def test_attention_fwd_argument_errors_are_found_before_any_launch():
    assert _fwd(q=None) == sla.ERR_NULL and _fwd(out=None) == sla.ERR_NULL
    assert _fwd(B=0) == sla.ERR_SHAPE and _fwd(d=64) == sla.ERR_SHAPE and _fwd(N=-5) == sla.ERR_SHAPE
    assert _fwd(H=70000) == sla.ERR_SHAPE
    assert _fwd(bq=32) == sla.ERR_BLOCK and _fwd(bk=32) == sla.ERR_BLOCK
    assert _fwd(rc=0.0) == sla.ERR_RATIO and _fwd(rc=0.8, rm=0.4) == sla.ERR_RATIO
    assert _fwd(phi=7) == sla.ERR_UNSUPPORTED and _fwd(quant=3) == sla.ERR_UNSUPPORTED
    assert _fwd(quant=-1) == sla.ERR_UNSUPPORTED
    assert _fwd(quant=1, wsb=sla.sla_workspace_bytes(1, 2, 1024, 128, 64, 64, 0.2, 0.4)) == sla.ERR_WORKSPACE   # needs the larger map
    assert _fwd(quant=0, ws=None) == sla.ERR_WORKSPACE   # the 16-bit path checks its arguments the same way
    assert _fwd(ws=None) == sla.ERR_WORKSPACE
    assert _fwd(ws=ctypes.c_void_p(0x10010)) == sla.ERR_WORKSPACE          # misaligned
    need = sla.sla_workspace_bytes(1, 2, 1024, 128, 64, 64, 0.2, 0.4)
    assert _fwd(wsb=need - 1) == sla.ERR_WORKSPACE


def test_strided_entry_point_rejects_bad_layouts_before_any_launch():
    L = sla.lib()

    def call(qs=None, os_=None, q=FAKE, wsb=16):
        # the workspace is too small on purpose: a layout that passes must reach that check, not a launch
        ref = lambda s: None if s is None else ctypes.byref(sla.Strides(*s))
        return L.sla_attention_fwd_strided(q, FAKE, FAKE, FAKE, ref(qs), None, None, ref(os_), 1, 2, 1024, 128,
                                           64, 64, 0.2, 0.4, None, None, 0, 2, WS, wsb, None)

    ok = (2 * 1024 * 128, 128, 2 * 128)                                     # [B,N,H,d]
    assert call(qs=ok, os_=ok) == sla.ERR_WORKSPACE
    assert call(qs=(3 * 2 * 1024 * 128, 128, 3 * 2 * 128)) == sla.ERR_WORKSPACE   # q of a packed [B,N,3,H,d]
    assert call(qs=(0, 0, 128)) == sla.ERR_WORKSPACE                        # broadcast over batch and head
    assert call(qs=(2 * 1024 * 128, 128, 64)) == sla.ERR_LAYOUT             # token rows would overlap
    assert call(qs=(2 * 1024 * 128, 132, 256)) == sla.ERR_LAYOUT            # not a multiple of 8 elements
    assert call(qs=(-8, 128, 256)) == sla.ERR_LAYOUT
    assert call(os_=(2 * 1024 * 128, 128, 100)) == sla.ERR_LAYOUT
    assert call(qs=ok, q=ctypes.c_void_p(0x10008)) == sla.ERR_LAYOUT        # rows not 16-byte aligned
    assert call(q=None, qs=ok) == sla.ERR_NULL


def test_stage_entry_points_argument_errors():
    L = sla.lib()
    big = 1 << 40
    assert L.sla_classify_blocks(FAKE, FAKE, 1, 2, 1024, 128, 64, 64, 0.2, 0.4, None, None, None, None,
                                 WS, big, None) == sla.ERR_NULL
    assert L.sla_classify_blocks(FAKE, FAKE, 1, 2, 1024, 128, 64, 64, 1.2, 0.4, FAKE, None, None, None,
                                 WS, big, None) == sla.ERR_RATIO
    assert L.sla_classify_blocks(FAKE, FAKE, 1, 2, 1024, 128, 64, 64, 0.2, 0.4, FAKE, None, None, None,
                                 WS, 16, None) == sla.ERR_WORKSPACE
    assert L.sla_sparse_attn_fwd(FAKE, FAKE, FAKE, None, 3, FAKE, None, 1, 2, 1024, 128, 64, 64, 2,
                                 WS, big, None) == sla.ERR_NULL
    assert L.sla_sparse_attn_fwd(FAKE, FAKE, FAKE, FAKE, 0, FAKE, None, 1, 2, 1024, 128, 64, 64, 2,
                                 WS, big, None) == sla.ERR_SHAPE
    assert L.sla_sparse_attn_fwd(FAKE, FAKE, FAKE, FAKE, 17, FAKE, None, 1, 2, 1024, 128, 64, 64, 2,
                                 WS, big, None) == sla.ERR_SHAPE
    assert L.sla_sparse_attn_fwd(FAKE, FAKE, FAKE, FAKE, 3, FAKE, None, 1, 2, 1024, 128, 64, 64, 0,
                                 WS, big, None) == sla.ERR_UNSUPPORTED
    assert L.sla_linear_attn_fwd(FAKE, FAKE, FAKE, None, None, None, 0, FAKE, 1, 2, 1024, 128, 64, 64,
                                 WS, big, None) == sla.ERR_NULL
    assert L.sla_linear_attn_fwd(FAKE, FAKE, FAKE, FAKE, None, None, 5, FAKE, 1, 2, 1024, 128, 64, 64,
                                 WS, big, None) == sla.ERR_UNSUPPORTED
    assert L.sla_linear_attn_fwd(FAKE, FAKE, FAKE, FAKE, None, None, 0, FAKE, 1, 2, 1024, 128, 64, 64,
                                 None, big, None) == sla.ERR_WORKSPACE
    assert L.sla_debug_e4m3_encode(None, FAKE, 4, None) == sla.ERR_NULL
    assert L.sla_debug_quantize_q(None, 1, 2, 1024, 128, 64, None, None, WS, big, None) == sla.ERR_NULL
    assert L.sla_debug_quantize_q(FAKE, 1, 2, 1024, 128, 96, None, None, WS, big, None) == sla.ERR_BLOCK
    ops = ctypes.c_double(0.0)
    assert L.sla_calibrate_mfma(0, 10, None, big, ctypes.byref(ops), None) == sla.ERR_NULL
    assert L.sla_calibrate_mfma(0, 10, WS, big, None, None) == sla.ERR_NULL
    assert L.sla_calibrate_mfma(3, 10, WS, big, ctypes.byref(ops), None) == sla.ERR_UNSUPPORTED
    assert L.sla_calibrate_mfma(1, 0, WS, big, ctypes.byref(ops), None) == sla.ERR_SHAPE
    assert L.sla_debug_quantize_kv(None, FAKE, 1, 2, 1024, 128, 64, None, None, None, None, None,
                                   WS, big, None) == sla.ERR_NULL


def test_binding_rejects_wrong_tensors():
    import torch
    x = torch.zeros((1, 2, 64, 128), dtype=torch.bfloat16)      # CPU tensor
    with pytest.raises(ValueError):
        sla.sla_attention_fwd(x, x, x, 64, 64, 0.2, 0.4)
    with pytest.raises(sla.SLAError):
        sla.sla_block_counts(0, 64, 64, 0.1, 0.2)
