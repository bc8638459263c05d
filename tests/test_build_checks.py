"""Static check of generated code (CPU only; needs hipcc, which cross-compiles without a GPU).

The W8A8 product writes each accumulation chain (four MFMAs, the first taking its C operand as an
inline constant the compiler would otherwise hold in 16 registers) as ONE assembly statement, so the
chain accumulates in place by construction.  The compiler does not know the statement holds matrix
products and inserts no wait states before a vector instruction that reads the chain's result (the
hardware does not interlock that case); the kernel is written so that every such reader comes a
whole chain later in program order.  This test compiles the kernel to assembly and checks both: the
chains are in place, and at least 18 instructions (the wait states the longest case needs) lie
between the end of a chain and the first instruction that reads its result."""
import os
import re
import shutil
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _hipcc():
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", shutil.which("hipcc")):
        if c and os.path.exists(c):
            return c
    return None


def _regs(operand_text):
    """Register numbers named in an operand string: v12 and v[12:15] forms."""
    regs = set()
    for a, b in re.findall(r"\bv\[(\d+):(\d+)\]", operand_text):
        regs.update(range(int(a), int(b) + 1))
    regs.update(int(x) for x in re.findall(r"\bv(\d+)\b", operand_text))
    return regs


@pytest.mark.skipif(_hipcc() is None, reason="hipcc not available")
def test_w8a8_chains_are_in_place_and_read_late_enough():
    from paper_2512_16093_amd import build as b
    src = os.path.join(ROOT, "paper_2512_16093_amd", "csrc", "k_w8a8.hip")
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "k.s")
        flags = [f for f in b.FLAGS if f not in ("-fPIC",)]
        r = subprocess.run([_hipcc()] + flags + ["-S", "--cuda-device-only", src, "-o", out],
                           capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-2000:]
        text = open(out).read()
    # instructions only (no labels, directives, comments)
    ins = [l.split(";")[0].strip() for l in text.splitlines()]
    ins = [l for l in ins if l and not l.startswith(".") and not l.endswith(":") and re.match(r"[a-z]", l)]
    pat = re.compile(r"v_mfma_i32_32x32x32_i8 (v\[(\d+):(\d+)\]), v\[\d+:\d+\], v\[\d+:\d+\], (\S+)")
    starts = [i for i, l in enumerate(ins) if l.startswith("v_mfma_i32_32x32x32_i8") and l.endswith("0.15915494")]
    assert len(starts) >= 8, "expected the chains' first MFMAs to take the inline constant"
    for i in starts:
        m0 = pat.match(ins[i])
        dst, lo, hi = m0.group(1), int(m0.group(2)), int(m0.group(3))
        mine = set(range(lo, hi + 1))
        # the chain: the next three matrix products that write these registers accumulate in place
        steps, last = 0, i
        for d, l in enumerate(ins[i + 1:i + 200]):
            m = pat.match(l)
            if m and m.group(1) == dst:
                assert m.group(4) == dst, (ins[i], l)
                steps, last = steps + 1, i + 1 + d
                if steps == 3:
                    break
        assert steps == 3, ins[i]
        # the first instruction that reads the result: at least 18 wait states behind the chain's last product
        # (a matrix product that has to wait for its own chain counts as 8, s_nop n as n + 1, anything else as 1)
        waited = 0
        for l in ins[last + 1:last + 400]:
            if l.startswith("s_endpgm"):
                break
            operands = l.split(None, 1)[1] if " " in l else ""
            srcs = operands.split(",", 1)[1] if "," in operands else ""     # everything after the destination
            if _regs(srcs) & mine:
                assert waited >= 18, (ins[i], l, "result read after only %d wait states" % waited)
                break
            if _regs(operands.split(",", 1)[0]) & mine:
                break                            # overwritten before any read: nothing to wait for
            nop = re.match(r"s_nop (\d+)", l)
            waited += int(nop.group(1)) + 1 if nop else (8 if l.startswith("v_mfma") and l.split(",")[-1].strip().startswith("v[") else 1)
