"""Pins for the oracle's software number formats (CPU only).

Each check is against something other than the oracle's own formula: PyTorch's
CPU bfloat16 / float8_e4m3fn conversions (an independent library), and the
constants the OCP 8-bit float specification fixes for E4M3.
"""
import numpy as np
import torch

from oracle import formats


def test_e4m3_spec_constants():
    # OCP FP8 E4M3: bias 7, max finite 448 (0x7E), min normal 2^-6 (0x08),
    # min subnormal 2^-9 (0x01), 1.0 = 0x38, no infinities, 0x7F = NaN.
    dec = formats.e4m3_decode(np.arange(256, dtype=np.uint8))
    assert dec[0x7E] == 448.0 and dec[0xFE] == -448.0
    assert dec[0x08] == 2.0 ** -6 and dec[0x01] == 2.0 ** -9
    assert dec[0x38] == 1.0 and dec[0x40] == 2.0 and dec[0x3C] == 1.5
    assert np.isnan(dec[0x7F]) and np.isnan(dec[0xFF])
    assert np.isfinite(dec[np.r_[0:0x7F, 0x80:0xFF]]).all()


def test_e4m3_decode_matches_torch_table():
    codes = torch.arange(256, dtype=torch.uint8)
    ref = codes.view(torch.float8_e4m3fn).to(torch.float64).numpy()
    dec = formats.e4m3_decode(codes.numpy())
    assert np.array_equal(np.isnan(ref), np.isnan(dec))
    ok = ~np.isnan(ref)
    assert np.array_equal(ref[ok], dec[ok])


def test_e4m3_roundtrip_all_codes():
    codes = np.array([c for c in range(256) if c & 0x7F != 0x7F], dtype=np.uint8)
    vals = formats.e4m3_decode(codes)
    assert np.array_equal(formats.e4m3_round(vals), vals)
    enc = formats.e4m3_encode(vals)
    # +0 / -0 keep their sign bit too
    assert np.array_equal(enc, codes)


def test_e4m3_round_matches_torch_in_range():
    rng = np.random.default_rng(1)
    x = np.concatenate([rng.uniform(-448, 448, 20000), rng.standard_normal(20000) * 1e-2,
                        rng.standard_normal(20000) * 1e-3, rng.uniform(0, 1, 20000) * 448,
                        np.exp2(rng.uniform(-12, 8.8, 20000))]).astype(np.float32)
    ref = torch.from_numpy(x).to(torch.float8_e4m3fn).to(torch.float64).numpy()
    got = formats.e4m3_round(x.astype(np.float64))
    assert np.array_equal(ref, got)


def test_e4m3_ties_to_even_at_every_midpoint():
    pos = np.sort(formats.e4m3_decode(np.arange(0, 0x7F, dtype=np.uint8)))
    mids = (pos[:-1] + pos[1:]) / 2.0  # exactly representable in float64
    got = formats.e4m3_round(mids)
    codes = formats.e4m3_encode(got)
    assert ((codes & 1) == 0).all()          # the even-mantissa neighbour wins
    assert ((got == pos[:-1]) | (got == pos[1:])).all()
    # just off the midpoint goes to the nearer neighbour
    assert np.array_equal(formats.e4m3_round(mids * (1 + 1e-12)), pos[1:])
    assert np.array_equal(formats.e4m3_round(mids[1:] * (1 - 1e-12)), pos[1:-1])


def test_e4m3_saturates_and_is_monotone_and_odd():
    assert formats.e4m3_round(1e9) == 448.0 and formats.e4m3_round(-1e9) == -448.0
    assert formats.e4m3_round(463.9) == 448.0 and formats.e4m3_round(480.0) == 448.0
    x = np.linspace(-500, 500, 200001)
    r = formats.e4m3_round(x)
    assert (np.diff(r) >= 0).all()
    assert np.array_equal(formats.e4m3_round(-x), -r)
    normal = np.abs(x) >= 2.0 ** -6
    inr = normal & (np.abs(x) <= 448)
    assert (np.abs(r[inr] - x[inr]) <= 2.0 ** -4 * np.abs(x[inr])).all()


def test_bf16_round_matches_torch():
    rng = np.random.default_rng(2)
    x = np.concatenate([rng.standard_normal(100000) * 3, np.exp2(rng.uniform(-30, 30, 50000)),
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.0078125, 3.3895314e38])]).astype(np.float32)
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(formats.bf16_round(x), ref)
    # ties: 1 + 2^-8 is halfway between 1 and 1 + 2^-7 -> even (1.0); 1 + 3*2^-8 -> 1 + 2^-6
    assert formats.bf16_round(np.float32(1 + 2.0 ** -8)) == 1.0
    assert formats.bf16_round(np.float32(1 + 3 * 2.0 ** -8)) == 1 + 2.0 ** -6


def test_int8_quantize_range_and_ties():
    x = np.array([-10.0, -1.0, -0.5, 0.5, 1.5, 2.5, 126.5, 127.49, 1000.0])
    q = formats.int8_quantize(x, 1.0)
    assert np.array_equal(q, [-10, -1, -0.0, 0.0, 2, 2, 126, 127, 127])
    rng = np.random.default_rng(3)
    y = rng.standard_normal(10000)
    d = np.abs(y).max() / 127
    c = formats.int8_quantize(y, d)
    assert c.min() >= -127 and c.max() <= 127 and (c == np.rint(c)).all()
    assert np.abs(c * d - y).max() <= d / 2 + 1e-15
    ref = torch.round(torch.from_numpy(y / d)).numpy()  # torch.round is half-to-even
    assert np.array_equal(c, ref)


def test_codes_at_exact_ties_follow_the_rule_not_the_rounding_of_the_scale():
    """16-bit inputs make quotients that are exactly half way between two codes common (x = amax / 2 gives
    63.5); such a value must go to the even code whatever the last bit of amax / 127 is.  Checked against
    exact rational arithmetic."""
    from fractions import Fraction
    amaxes = [1.90625, 3.0, 0.2890625, 5.5, 7.25, 100.0, 0.01171875]         # bf16 values
    for amax in amaxes:
        xs = np.array([amax * f for f in (0.5, 0.25, 0.75, 0.125, 1.0, -0.5, -0.75, 0.3125)])
        xs = formats.bf16_round(xs)
        got = formats.int8_codes(xs, amax)
        for x, c in zip(xs, got):
            t = Fraction(float(x)) * 127 / Fraction(amax)
            lo = t.numerator // t.denominator
            frac = t - lo
            want = lo + 1 if frac > Fraction(1, 2) else lo if frac < Fraction(1, 2) else lo + (lo % 2)
            assert c == want, (amax, x, c, want)
    # the case that showed it: 448 * 1.4296875 / 1.90625 is 336, half way between 320 and 352 -> 320 (even mantissa)
    from oracle import sla_oracle as so
    V = np.array([[1.90625], [1.4296875], [-1.4296875], [0.953125]])
    V8, dv = so.quantize_v(V)
    assert np.array_equal(V8[:, 0], [448.0, 320.0, -320.0, 224.0]) and dv[0] == 1.90625 / 448
    assert np.array_equal(formats.int8_codes(np.zeros(3), 0.0), np.zeros(3))

