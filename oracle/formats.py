"""Number formats used by the quantised sparse branch, in software.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

The paper (Section 1.1) names the low-bit scheme (SageAttention2++: 8-bit
integer QK^T, 8-bit float PV) without restating the formats; the formats taken
here are the public ones: bfloat16 (1-8-7), OCP FP8 E4M3 (1-4-3, bias 7, finite
maximum 448, subnormals down to 2^-9, no infinities) and symmetric INT8 in
[-127, 127].  All rounding is round-to-nearest, ties to even.
"""
from __future__ import annotations

import numpy as np

E4M3_MAX = 448.0
INT8_MAX = 127.0


def bf16_round(x):
    """Nearest bfloat16 value (ties to even) of each float32-representable x,
    returned as float64.  Works on the float32 bit pattern: bf16 keeps the top
    16 bits, so rounding adds half of the dropped field plus the tie bit."""
    f = np.ascontiguousarray(x, dtype=np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    r = ((u + 0x7FFF + lsb) >> 16) << 16
    out = (r & 0xFFFFFFFF).astype(np.uint32).view(np.float32).astype(np.float64)
    return np.where(np.isnan(f), np.nan, out)


def e4m3_decode(code):
    """Value of each OCP E4M3 code (uint8) as float64; 0x7F / 0xFF are NaN."""
    c = np.asarray(code, dtype=np.uint8).astype(np.int64)
    sign = np.where(c & 0x80, -1.0, 1.0)
    e = (c >> 3) & 0xF
    m = (c & 0x7).astype(np.float64)
    normal = (1.0 + m / 8.0) * np.exp2((e - 7).astype(np.float64))
    sub = (m / 8.0) * 2.0 ** -6
    val = np.where(e == 0, sub, normal)
    val = np.where((e == 15) & ((c & 7) == 7), np.nan, val)
    return sign * val


def e4m3_round(x):
    """Nearest E4M3 value (ties to even), saturating at +-448, as float64.

    Within a binade [2^e, 2^(e+1)) the spacing is 2^(e-3); below 2^-6 it is the
    subnormal spacing 2^-9.  Rounding |x| to a multiple of the spacing with
    rint (ties to even) also handles the carry into the next binade."""
    x = np.asarray(x, dtype=np.float64)
    a = np.abs(x)
    with np.errstate(divide="ignore"):
        e = np.floor(np.log2(np.where(a > 0, a, 1.0)))
    e = np.maximum(e, -6.0)
    q = np.exp2(e - 3.0)
    r = np.rint(a / q) * q
    r = np.minimum(r, E4M3_MAX)
    return np.copysign(r, x)


def e4m3_encode(x):
    """E4M3 code (uint8) of e4m3_round(x)."""
    r = e4m3_round(x)
    a = np.abs(r)
    sign = (np.signbit(r)).astype(np.uint8) << 7
    with np.errstate(divide="ignore"):
        e = np.floor(np.log2(np.where(a > 0, a, 1.0)))
    is_sub = a < 2.0 ** -6
    ebits = np.where(is_sub, 0, e + 7).astype(np.int64)
    mant = np.where(is_sub, a / 2.0 ** -9, (a / np.exp2(np.where(is_sub, 0.0, e)) - 1.0) * 8.0)
    mant = np.rint(mant).astype(np.int64)
    return (sign | ((ebits << 3) | mant).astype(np.uint8)).astype(np.uint8)


def int8_quantize(x, delta):
    """Symmetric INT8 code clip(rint(x / delta), -127, 127) as float64 integers."""
    return np.clip(np.rint(np.asarray(x, dtype=np.float64) / delta), -INT8_MAX, INT8_MAX)


def int8_codes(x, amax):
    """Symmetric INT8 codes of a block whose largest magnitude is amax, i.e. with the scale amax / 127:
    clip(rint(127 x / amax), -127, 127) as float64 integers (zeros when amax is 0).  The quotient is
    formed from the product 127 x, which is exact for 16-bit inputs, so a value that lies exactly half
    way between two codes is seen as the tie it is and goes to the even code; dividing by the rounded
    scale amax / 127 instead would let that scale's last bit decide such ties."""
    x = np.asarray(x, dtype=np.float64)
    if amax <= 0:
        return np.zeros_like(x)
    return np.clip(np.rint(x * INT8_MAX / amax), -INT8_MAX, INT8_MAX)
