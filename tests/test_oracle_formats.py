"""Pins for the oracle's number formats and scalar rounding rules (CPU only).

Each pin is something other than the oracle itself: PyTorch's own E4M3 / E8M0 casts,
the paper's L/G/S rounding rule evaluated on FP32 bits, or exact rational brute force.
"""
import math
import random
import struct
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import ref
from tests import bruteforce as bf


def f32_bits(x):
    return struct.unpack("<I", struct.pack("<f", x))[0]


def test_e4m3_decode_matches_torch_cast():
    codes = torch.arange(256, dtype=torch.int64).to(torch.uint8)
    want = codes.view(torch.float8_e4m3fn).float()
    for c in range(256):
        got = ref.e4m3_value(c)
        if (c & 0x7F) == 0x7F:
            assert math.isnan(got) and math.isnan(float(want[c]))
        else:
            assert got == float(want[c]), hex(c)
            assert Fraction(abs(got)) == bf.e4m3_fraction(c & 0x7F)
    assert ref.e4m3_value(0x7E) == 448.0 and ref.e4m3_value(0x01) == 2.0 ** -9


def test_e2m1_decode_is_the_format_table():
    # section 3.1: 1 sign, 2 exponent, 1 mantissa bit; subnormal drops the implicit bit
    mags = [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]
    for n in range(16):
        v = ref.e2m1_value(n)
        assert abs(v) == mags[n & 7]
        assert math.copysign(1.0, v) == (-1.0 if n & 8 else 1.0)


def lgs_round_e2m1(y):
    """The paper's bit-level rule (section 3.1) on the FP32 bits of y in [0, 6]:
    keep 1 mantissa bit; L = bit 22, G = bit 21, S = OR(bits 20..0), R = G & (S | L).
    Below 1 (E2M1 exponent field 0) the implicit bit is materialised as
    0x400000 | (mant >> 1) and the mantissa shifted right once more per binade."""
    bits = f32_bits(y)
    e, mant = (bits >> 23) & 0xFF, bits & 0x7FFFFF
    if e == 0:
        return 0
    unb = e - 127
    if unb >= 0:
        L, G, S = (mant >> 22) & 1, (mant >> 21) & 1, int((mant & 0x1FFFFF) != 0)
        code = ((unb + 1) << 1 | L) + (G & (S | L))
        return min(code, 7)
    # subnormal target: value = 0.m * 2^0 with one mantissa bit (weight 0.5)
    shift = -unb - 1                      # extra right shifts beyond the first
    sticky = 0
    m = 0x400000 | (mant >> 1)
    sticky |= mant & 1
    for _ in range(min(shift, 40)):
        sticky |= m & 1
        m >>= 1
    L, G, S = (m >> 22) & 1, (m >> 21) & 1, int((m & 0x1FFFFF) != 0 or sticky != 0)
    return L + (G & (S | L))


def test_e2m1_round_matches_paper_lgs_rule_and_brute_force():
    rng = random.Random(1)
    ys = [0.0, 0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0, 6.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0]
    for t in list(ys):
        f = np.float32(t)
        ys += [float(np.nextafter(f, np.float32(100))), float(np.nextafter(f, np.float32(-100)))]
    ys += [float(np.float32(rng.uniform(0, 6))) for _ in range(3000)]
    ys += [float(np.float32(2.0 ** rng.uniform(-30, 2.5))) for _ in range(2000)]
    for y in ys:
        if y < 0 or y > 6:
            continue
        got = ref.e2m1_round(y)
        assert got == bf.nearest_even_code(Fraction(y), bf.E2M1_GRID), y
        assert got == lgs_round_e2m1(y), y
    # ties go to the even code, anything above 6 saturates
    assert [ref.e2m1_round(t) for t in (0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0)] == [0, 2, 2, 4, 4, 6, 6]
    assert ref.e2m1_round(6.0000001) == 7 and ref.e2m1_round(1e30) == 7 and ref.e2m1_round(math.inf) == 7
    # monotone and idempotent on the grid
    for c in range(8):
        assert ref.e2m1_round(abs(ref.e2m1_value(c))) == c
    grid = np.linspace(0, 6, 2001)
    codes = [ref.e2m1_round(float(g)) for g in grid]
    assert codes == sorted(codes)


def test_e4m3_round_matches_torch_cast():
    rng = random.Random(2)
    vals = [0.0, 2.0 ** -10, 2.0 ** -9, 1.5 * 2.0 ** -9, 2.0 ** -6, 448.0, 384.0, 0.0009765625 * 2.5]
    vals += [rng.uniform(0, 448) for _ in range(3000)]
    vals += [2.0 ** rng.uniform(-14, 8.8) for _ in range(3000)]
    # every midpoint between neighbouring codes (the ties) and its float32 neighbours
    for c in range(0x7E):
        mid = (ref.e4m3_value(c) + ref.e4m3_value(c + 1)) / 2
        vals += [mid, float(np.nextafter(np.float32(mid), np.float32(1e9))),
                 float(np.nextafter(np.float32(mid), np.float32(-1)))]
    vals = [float(np.float32(v)) for v in vals if v <= 448.0]
    want = torch.tensor(vals, dtype=torch.float32).to(torch.float8_e4m3fn).view(torch.uint8).tolist()
    for v, w in zip(vals, want):
        assert ref.e4m3_round(v) == w, (v, w)


def test_scale_byte_is_smallest_power_of_two_covering_gmax_over_6():
    rng = random.Random(3)
    # exact corner cases of 2^ceil(log2(gmax/6)) (section 3.1)
    assert ref.scale_byte(6.0) == 127
    assert ref.scale_byte(float(np.nextafter(np.float32(6), np.float32(7)))) == 128
    assert ref.scale_byte(3.0) == 126
    assert ref.scale_byte(float(np.nextafter(np.float32(3), np.float32(4)))) == 127
    assert ref.scale_byte(float(np.nextafter(np.float32(6), np.float32(0)))) == 127
    assert ref.scale_byte(448.0) == 134 and ref.scale_byte(1.0) == 125 and ref.scale_byte(0.75) == 124
    # the clamps of the byte: 2^127 is the largest scale (byte 254; 255 means NaN), byte 0 the smallest.  No
    # finite FP32 maximum needs the upper one (6 * 2^127 exceeds FP32), so it is pinned on doubles.
    assert ref.scale_byte(6 * 2.0 ** 127) == 254 and ref.scale_byte(6 * 2.0 ** 128) == 254 and ref.scale_byte(2.0 ** 300) == 254
    assert ref.scale_byte(6 * 2.0 ** -127) == 0 and ref.scale_byte(2.0 ** -149) == 0 and ref.scale_byte(6 * 2.0 ** -126) == 1
    gs = [float(np.float32(2.0 ** rng.uniform(-149, 127.9))) for _ in range(4000)]
    gs += [float(np.float32(6 * 2.0 ** k)) for k in range(-130, 125)]
    gs += [float(np.nextafter(np.float32(6 * 2.0 ** k), np.float32(np.inf))) for k in range(-125, 125)]
    gs += [2.0 ** -149, 2.0 ** -126, float(np.finfo(np.float32).max)]
    for g in gs:
        if g == 0:
            continue
        b = ref.scale_byte(g)
        assert b == bf.scale_byte(Fraction(g)), g
        if 0 < b < 254:                      # unclamped: normalised maximum lies in (3, 6]
            y = Fraction(g) / bf.pow2(b - 127)
            assert 3 < y <= 6
        # same thing through floating-point log2 where it is far from an integer
        lg = math.log2(g / 6.0)
        if abs(lg - round(lg)) > 1e-6:
            assert b == min(254, max(0, math.ceil(lg) + 127))


def test_ue8m0_decode_against_torch():
    # the oracle's dequant scale output must be torch's own decode of the byte max-6
    q = np.zeros((1, 64), np.uint8)
    for b in [6, 7, 60, 127, 133, 200, 254]:
        sf = np.array([[b, 0, 0, 0]], np.uint8)
        _, xs = ref.dequant_to_fp8(q, sf)
        want = torch.tensor([b - 6], dtype=torch.uint8).view(torch.float8_e8m0fnu).float().item()
        if b - 6 == 0:
            want = 2.0 ** -127               # E8M0 byte 0 is 2^-127, an FP32 subnormal
        assert float(xs[0, 0]) == want, b
    # below byte 6 the tile scale keeps going down as an exact FP32 subnormal
    for b in range(0, 6):
        _, xs = ref.dequant_to_fp8(q, np.array([[b, 0, 0, 0]], np.uint8))
        assert float(xs[0, 0]) == 2.0 ** (b - 6 - 127)
