"""Static check of generated code (CPU only; needs hipcc, which cross-compiles without a GPU).

The W8A8 product starts every accumulation chain with an MFMA written in inline assembly (its C
operand is an inline constant the compiler would otherwise hold in 16 registers).  The compiler
does not know that statement is an MFMA, so it inserts no wait states after it.  None are needed
as long as the next MFMA of the chain accumulates IN PLACE (same destination as its C operand,
the case the hardware forwards); a register allocation that made it accumulate into other
registers would need wait states nobody inserts.  This test compiles the kernel to assembly and
checks that every such chain is in place."""
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


@pytest.mark.skipif(_hipcc() is None, reason="hipcc not available")
def test_w8a8_chains_accumulate_in_place_after_the_assembly_mfma():
    from paper_2512_16093_amd import build as b
    src = os.path.join(ROOT, "paper_2512_16093_amd", "csrc", "k_w8a8.hip")
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "k.s")
        flags = [f for f in b.FLAGS if f not in ("-fPIC",)]
        r = subprocess.run([_hipcc()] + flags + ["-S", "--cuda-device-only", src, "-o", out],
                           capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-2000:]
        text = open(out).read()
    mfma = [l.split(";")[0].strip() for l in text.splitlines() if l.strip().startswith("v_mfma_i32_32x32x32_i8")]
    starts = [i for i, l in enumerate(mfma) if l.endswith("0.15915494")]
    assert len(starts) >= 8, "expected the chains' first MFMAs to take the inline constant"
    pat = re.compile(r"v_mfma_i32_32x32x32_i8 (v\[\d+:\d+\]), v\[\d+:\d+\], v\[\d+:\d+\], (\S+)")
    for i in starts:
        dst = pat.match(mfma[i]).group(1)
        for nxt in mfma[i + 1:i + 4]:          # the three in-place steps of the chain
            m = pat.match(nxt)
            assert m and m.group(1) == dst and m.group(2) == dst, (mfma[i], nxt)
