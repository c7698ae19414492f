"""Pins for the oracle's number formats (E4M3, INT4, bf16) against things other than itself:
constants the paper prints, literal hand-written values, and library casts."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_constants.txt")


def _golden():
    out = {}
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, value, _cite = [p.strip() for p in line.split("|", 2)]
        out[name] = eval(value, {"__builtins__": {}})
    return out


def test_e4m3_paper_constants():
    g = _golden()
    # smallest positive code is the smallest subnormal (App. B, Lemma B.1)
    assert oracle.e4m3_decode(0x01) == g["e4m3_min_subnormal"]
    # largest subnormal is 7 * 2^-9: sigma = max|w|/7 below it... (Lemma B.1 threshold / 7 * 7)
    assert oracle.e4m3_decode(0x07) == g["e4m3_underflow_thresh"]
    # largest finite value is the overflow threshold 1.75 * 2^8 (App. C.1)
    assert oracle.e4m3_decode(0x7E) == g["e4m3_overflow_thresh"] == 448
    finite = [oracle.e4m3_decode(c) for c in range(0x7F)]
    assert max(finite) == g["e4m3_overflow_thresh"]
    assert min(v for v in finite if v > 0) == g["e4m3_min_subnormal"]
    # Lemma B.1: sigma = max|w|/7 < 2^-9 rounds (to nearest) to zero only below half of it,
    # but anything below the smallest subnormal has no exact non-zero code:
    assert all(v == 0 or v >= g["e4m3_min_subnormal"] for v in finite)


def test_e4m3_decode_literals():
    lit = {0x00: 0.0, 0x08: 2.0 ** -6, 0x30: 0.5, 0x38: 1.0, 0x3C: 1.5, 0x40: 2.0, 0x44: 3.0,
           0x48: 4.0, 0x4A: 5.0, 0x4C: 6.0, 0x4E: 7.0, 0x50: 8.0, 0x77: 240.0, 0x78: 256.0,
           0x7D: 416.0, 0x05: 5 * 2.0 ** -9, 0x0F: 15 * 2.0 ** -9, 0xB8: -1.0, 0xD0: -8.0,
           0xFE: -448.0}
    for code, val in lit.items():
        assert oracle.e4m3_decode(code) == val, hex(code)
    assert math.isnan(oracle.e4m3_decode(0x7F)) and math.isnan(oracle.e4m3_decode(0xFF))
    assert math.copysign(1.0, oracle.e4m3_decode(0x80)) == -1.0


def test_e4m3_decode_matches_library_cast():
    codes = torch.arange(256, dtype=torch.int32).to(torch.uint8)
    lib = codes.view(torch.float8_e4m3fn).to(torch.float64).numpy()
    for c in range(256):
        mine = oracle.e4m3_decode(c)
        if math.isnan(lib[c]):
            assert math.isnan(mine)
        else:
            assert mine == lib[c], hex(c)


def test_e4m3_decode_structure():
    vals = [oracle.e4m3_decode(c) for c in range(0x7F)]
    assert all(b > a for a, b in zip(vals, vals[1:]))            # strictly increasing codes
    for c in range(0x7F):
        assert oracle.e4m3_decode(c | 0x80) == -vals[c]
    # low 16 codes are the integers 0..15 times 2^-9 (subnormals run into the first binade)
    assert [v * 512 for v in vals[:16]] == list(range(16))


def test_e4m3_encode_roundtrip_and_ties():
    for c in list(range(0x7F)) + list(range(0x81, 0xFF)):
        assert oracle.e4m3_encode_rne(oracle.e4m3_decode(c)) == c
    for c in range(0x7E):                                        # midpoints go to the even code
        mid = (Fraction(oracle.e4m3_decode(c)) + Fraction(oracle.e4m3_decode(c + 1))) / 2
        want = c if c % 2 == 0 else c + 1
        assert oracle.e4m3_encode_rne(float(mid)) == want
        assert oracle.e4m3_encode_rne(-float(mid)) == (want | 0x80)
        assert oracle.e4m3_encode_rne(np.nextafter(float(mid), 1e9)) == c + 1
        assert oracle.e4m3_encode_rne(np.nextafter(float(mid), -1e9)) == c
    # saturation, never NaN for finite input
    for x in (448.0, 449.0, 464.0, 480.0, 1e6, 3.0e38):
        assert oracle.e4m3_encode_rne(x) == 0x7E and oracle.e4m3_encode_rne(-x) == 0xFE
    assert oracle.e4m3_encode_rne(2.0 ** -10) == 0x00            # tie between 0 and 2^-9 -> even
    assert oracle.e4m3_encode_rne(3 * 2.0 ** -10) == 0x02        # tie between codes 1 and 2 -> 2
    assert oracle.e4m3_encode_rne(float("nan")) == 0x7F


def test_e4m3_encode_matches_library_cast():
    rng = np.random.default_rng(11)
    x = np.concatenate([rng.standard_normal(20000) * s for s in (1e-3, 0.05, 1.0, 30.0, 150.0)])
    x = x[np.abs(x) < 448].astype(np.float32)
    lib = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    mine = np.array([oracle.e4m3_encode_rne(float(v)) for v in x], dtype=np.uint8)
    assert np.array_equal(mine, lib)


def test_int4_decode_all_sixteen():
    g = _golden()
    want = [0, 1, 2, 3, 4, 5, 6, 7, -8, -7, -6, -5, -4, -3, -2, -1]
    got = [oracle.int4_decode(n) for n in range(16)]
    assert got == want
    assert min(got) == g["int4_lut_min_multiple"] and max(got) == g["int4_lut_max_multiple"]
    assert [oracle.int4_decode(0xA0 | n) for n in range(16)] == want   # only the low nibble counts


def test_bf16_literals_and_ties():
    assert oracle.bf16_encode_rne(1.0) == 0x3F80
    assert oracle.bf16_encode_rne(-2.5) == 0xC020
    assert oracle.bf16_encode_rne(1.0 + 2.0 ** -8) == 0x3F80     # tie -> even (1.0)
    assert oracle.bf16_encode_rne(1.0 + 3 * 2.0 ** -8) == 0x3F82  # tie -> even
    assert oracle.bf16_encode_rne(1.0 + 2.0 ** -8 + 2.0 ** -30) == 0x3F81
    assert oracle.bf16_encode_rne(0.0) == 0x0000 and oracle.bf16_encode_rne(-0.0) == 0x8000
    assert oracle.bf16_encode_rne(3.4e38) == 0x7F80              # rounds past the largest finite
    assert oracle.bf16_decode(0x3F80) == 1.0 and oracle.bf16_decode(0xC020) == -2.5
    assert oracle.bf16_ulp(1.0) == 2.0 ** -7 and oracle.bf16_ulp(1.99) == 2.0 ** -7
    assert oracle.bf16_ulp(2.0) == 2.0 ** -6 and oracle.bf16_ulp(-300.0) == 2.0
    assert oracle.bf16_ulp(0.75) == 2.0 ** -8


def test_bf16_encode_matches_library_cast():
    rng = np.random.default_rng(5)
    x = (rng.standard_normal(200000) * np.exp(rng.uniform(-30, 30, 200000))).astype(np.float32)
    lib = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    mine = oracle.bf16_round_array(x.astype(np.float64))
    assert np.array_equal(mine, lib)
    back = oracle.bf16_bits_to_f64(mine)
    assert np.all(np.abs(back - x) <= 0.5 * oracle.bf16_ulp_array(x.astype(np.float64)) * 1.0000001)
