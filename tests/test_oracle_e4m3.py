"""Pins of the oracle's number formats: OCP e4m3 encode/decode and bf16 rounding.

The oracle is compared with the format definition (exhaustive tables, exact
fractions), never with its own formula.
"""
import math
import os
from fractions import Fraction

import numpy as np
import torch

from exact_model import e4m3_code_value, e4m3_nearest_code, round_to_binary32

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _finite_codes():
    return [c for c in range(256) if (c & 0x7F) != 0x7F]


def test_textbook_values(orc):
    # values from the OFP8 specification's E4M3 table (tests/golden/e4m3_textbook.txt)
    n = 0
    for line in open(os.path.join(GOLDEN, "e4m3_textbook.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        code_s, val_s = line.split()
        code, val = int(code_s, 16), float(val_s)
        got = orc.e4m3_decode(code)
        assert got == val and math.copysign(1, got) == math.copysign(1, val), (code_s, got, val)
        assert orc.e4m3_encode(val) == code
        n += 1
    assert n >= 18
    assert math.isnan(orc.e4m3_decode(0x7F)) and math.isnan(orc.e4m3_decode(0xFF))


def test_decode_matches_format_definition_exhaustively(orc):
    for c in _finite_codes():
        assert Fraction(orc.e4m3_decode(c)) == e4m3_code_value(c), hex(c)


def test_roundtrip_all_codes(orc):
    for c in _finite_codes():
        assert orc.e4m3_encode(orc.e4m3_decode(c)) == c, hex(c)


def test_decode_monotone(orc):
    vals = [orc.e4m3_decode(c) for c in range(0x7F)]
    assert all(b > a for a, b in zip(vals, vals[1:]))
    assert vals[-1] == 448.0


def test_midpoints_round_to_even_and_neighbours_round_away(orc):
    f32 = np.float32
    for c in range(0x7E):
        lo, hi = orc.e4m3_decode(c), orc.e4m3_decode(c + 1)
        mid = f32((lo + hi) / 2)
        assert float(mid) == (lo + hi) / 2           # exactly representable in fp32
        even = c if c % 2 == 0 else c + 1
        assert orc.e4m3_encode(mid) == even, hex(c)
        below = np.nextafter(mid, f32(0))
        above = np.nextafter(mid, f32(1e9))
        assert orc.e4m3_encode(below) == c, hex(c)
        assert orc.e4m3_encode(above) == c + 1, hex(c)
        # mirrored for negative inputs
        assert orc.e4m3_encode(-mid) == (0x80 | even)
        assert orc.e4m3_encode(-below) == (0x80 | c)
        assert orc.e4m3_encode(-above) == (0x80 | (c + 1))


def test_saturation_and_signed_zero(orc):
    for v in (448.0, 448.00003, 449.0, 463.9, 464.0, 480.0, 1e4, 3.0e38, float("inf")):
        assert orc.e4m3_encode(v) == 0x7E
        assert orc.e4m3_encode(-v) == 0xFE
    assert orc.e4m3_encode(0.0) == 0x00
    assert orc.e4m3_encode(-0.0) == 0x80
    # below half the smallest subnormal -> signed zero; exactly half ties to even (zero)
    assert orc.e4m3_encode(2.0 ** -10) == 0x00
    assert orc.e4m3_encode(-(2.0 ** -10)) == 0x80
    assert orc.e4m3_encode(float(np.nextafter(np.float32(2.0 ** -10), np.float32(1)))) == 0x01
    assert orc.e4m3_encode(1e-30) == 0x00 and orc.e4m3_encode(-1e-30) == 0x80
    assert orc.e4m3_encode(float("nan")) == 0x7F


def test_encode_against_exact_nearest_search(orc):
    rng = np.random.default_rng(11)
    # log-uniform magnitudes across the whole e4m3 range plus values hugging the grid
    mags = np.exp(rng.uniform(math.log(2.0 ** -12), math.log(600.0), size=6000)).astype(np.float32)
    signs = rng.choice([-1.0, 1.0], size=mags.size).astype(np.float32)
    vals = mags * signs
    got = orc.e4m3_encode_array(vals)
    for v, g in zip(vals, got):
        want = e4m3_nearest_code(Fraction(float(v)))
        assert g == want, (float(v), hex(g), hex(want))


def test_encode_against_torch_float8_cast(orc):
    # library cross-check (PyTorch CPU float8_e4m3fn cast is RNE on the same format);
    # inputs are clamped to the finite range first because the library does not saturate.
    rng = np.random.default_rng(5)
    a = rng.standard_normal(400_000).astype(np.float32) * np.float32(60.0)
    b = np.exp(rng.uniform(math.log(1e-4), math.log(448.0), size=400_000)).astype(np.float32)
    # every bf16 bit pattern with magnitude <= 448 (these are exactly the scaled values when inv == 1)
    allb = (np.arange(65536, dtype=np.uint32) << 16).astype(np.uint32).view(np.float32)
    allb = allb[np.isfinite(allb) & (np.abs(allb) <= 448.0)]
    vals = np.clip(np.concatenate([a, b, -b, allb]), -448.0, 448.0).astype(np.float32)
    got = orc.e4m3_encode_array(vals)
    want = torch.from_numpy(vals).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(got, want)


def test_bf16_widen_and_rne_narrow(orc):
    rng = np.random.default_rng(3)
    f = (rng.standard_normal(20000) * np.exp(rng.uniform(-20, 20, 20000))).astype(np.float32)
    want = torch.from_numpy(f).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([orc.f32_to_bf16_rne(float(v)) for v in f], dtype=np.uint16)
    assert np.array_equal(got, want)
    # exact ties: x.5 ulp -> even
    for hi in (0x3F80, 0x3F81, 0x4000, 0xBF81):
        tie = np.array([(hi << 16) | 0x8000], dtype=np.uint32).view(np.float32)[0]
        assert orc.f32_to_bf16_rne(float(tie)) == (hi if hi % 2 == 0 else hi + 1)
    # widening is the exact value of the upper half
    for h in (0x0000, 0x3F80, 0xC2F7, 0x0001, 0x7F7F, 0x8000):
        u = np.array([h << 16], dtype=np.uint32).view(np.float32)[0]
        assert orc.bf16_to_f32(h) == float(u)


def test_round_to_binary32_helper_is_numpy_division():
    # keeps the test-side exact model honest: its fp32 rounding equals IEEE division
    rng = np.random.default_rng(9)
    for a in rng.uniform(1e-6, 1e6, 300).astype(np.float32):
        q = round_to_binary32(Fraction(448) / Fraction(float(a)))
        assert q == Fraction(float(np.float32(448.0) / a))
        q = round_to_binary32(Fraction(float(a)) / Fraction(448))
        assert q == Fraction(float(a / np.float32(448.0)))
