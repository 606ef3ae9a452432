"""Pins for the oracle's MXFP4 -> FP8 conversion (Algorithm 1, section 3.3). CPU only."""
import os
from fractions import Fraction

import numpy as np
import torch

from oracle import ref
from paper_2603_02731_amd import synth
from tests import bruteforce as bf
from tests.test_oracle_quant import unpack_nibbles

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def pack_nibbles(n):
    n = np.asarray(n, np.uint8)
    return (n[..., 0::2] | (n[..., 1::2] << 4)).astype(np.uint8)


def test_hand_worked_tile_of_algorithm_1():
    lines = [l.strip() for l in open(os.path.join(GOLDEN, "alg1_worked_tile.txt"))
             if l.strip() and not l.startswith("#")]
    sfb, scale_bits = lines[0].split("|")
    sf = np.array([[int(b) for b in sfb.split()]], np.uint8)
    nib = np.zeros((1, 128), np.uint8)
    want = {}
    for l in lines[1:]:
        blk, el, n, out = l.split()
        nib[0, int(blk) * 32 + int(el)] = int(n, 16)
        want[int(blk) * 32 + int(el)] = int(out, 16)
    x, xs = ref.dequant_to_fp8(pack_nibbles(nib), sf)
    assert xs.view(np.uint32)[0, 0] == int(scale_bits, 16)
    for k, w in want.items():
        assert x[0, k] == w, (k, hex(x[0, k]), hex(w))


def alg1_literal(nibble, sf_i, sf_max):
    """Algorithm 1, steps 1-8, literally, for one element (integers only)."""
    sf_fp8 = sf_max - 6
    e_adjust = sf_fp8 - sf_i
    sign = (nibble >> 3) & 1
    e_fp4 = (nibble >> 1) & 3
    m = nibble & 1
    e_fp8 = e_fp4 - 1 + 7
    e = e_fp8 - e_adjust
    return (sign << 7) | (e << 3) | (m << 2), e


def test_every_code_and_shift_against_algorithm_1_where_it_applies():
    # Algorithm 1 is stated for normal E2M1 codes (exponent field >= 1) and holds while
    # the resulting E4M3 exponent field stays >= 1.
    for d in range(0, 20):
        sf = np.array([[140, 140 - d, 140, 140]], np.uint8)
        nib = np.zeros((1, 128), np.uint8)
        nib[0, 32:48] = np.arange(16)
        x, xs = ref.dequant_to_fp8(pack_nibbles(nib), sf)
        assert float(xs[0, 0]) == 2.0 ** (140 - 6 - 127)
        for n in range(16):
            if (n & 7) >= 2:
                byte, e = alg1_literal(n, 140 - d, 140)
                if e >= 1:
                    assert x[0, 32 + n] == byte, (d, n)
            if (n & 7) == 0:
                assert x[0, 32 + n] == (n >> 3) << 7       # zero keeps its sign


def test_lossless_range_and_underflow_against_exact_rationals_and_torch():
    rng = np.random.default_rng(0)
    for trial in range(60):
        sf4 = rng.integers(0, 255, size=4)
        if trial % 3 == 0:                                  # close scales: the usual case
            sf4 = np.clip(int(rng.integers(0, 255)) + rng.integers(-4, 5, size=4), 0, 254)
        if trial % 7 == 0:                                  # wide spread: rounding and flush
            sf4 = np.clip(int(rng.integers(30, 255)) - rng.integers(0, 24, size=4), 0, 254)
        nib = rng.integers(0, 16, size=128).astype(np.uint8)
        nib[:16] = np.arange(16)
        x, xs = ref.dequant_to_fp8(pack_nibbles(nib[None]), sf4[None].astype(np.uint8))
        scale, want = bf.dequant_tile(nib.tolist(), [int(b) for b in sf4])
        assert Fraction(float(xs[0, 0])) == scale
        assert x[0].tolist() == want, sf4
        bmax = int(sf4.max())
        for k in range(128):
            d = bmax - int(sf4[k // 32])
            real = bf.E2M1_GRID[nib[k] & 7] * bf.pow2(int(sf4[k // 32]) - 127)
            got = bf.e4m3_fraction(int(x[0, k]) & 0x7F) * scale
            if d <= 14:                                     # "logically lossless" (section 3.2)
                assert got == real, (sf4, k)
            if d >= 19:
                assert (x[0, k] & 0x7F) == 0
            assert (x[0, k] >> 7) == (nib[k] >> 3)
        # library pin: the same division done in float32 and cast by PyTorch
        units = [float(bf.E2M1_GRID[n & 7] * bf.pow2(6 - (bmax - int(sf4[i // 32])))) for i, n in enumerate(nib)]
        cast = torch.tensor(units, dtype=torch.float32).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
        assert ((x[0] & 0x7F) == cast).all()
        assert (x[0] & 0x7F).max() <= 0x7C                  # never above 384: no saturation


def test_nan_scale_byte():
    nib = np.full((1, 128), 0x3, np.uint8)
    sf = np.array([[120, 0xFF, 125, 110]], np.uint8)
    x, xs = ref.dequant_to_fp8(pack_nibbles(nib), sf)
    assert np.isnan(xs[0, 0])
    assert (x[0, 32:64] == 0x7F).all()
    # the other blocks align to the maximum of the non-NaN bytes (125)
    sf2 = np.array([[120, 0, 125, 110]], np.uint8)
    x2, _ = ref.dequant_to_fp8(pack_nibbles(nib), sf2)
    assert (x[0, :32] == x2[0, :32]).all() and (x[0, 64:] == x2[0, 64:]).all()


def test_round_trips():
    # MXFP4 -> FP8 -> MXFP4 keeps every real value when the scales of a tile are close
    q, sf = synth.random_mxfp4(64, 512, seed=1, scale_center=120, scale_spread=5)
    q, sf = q.numpy(), sf.numpy()
    x, xs = ref.dequant_to_fp8(q, sf)
    q2, sf2 = ref.quant_from_fp8(x, xs)
    grid = np.array([0, .5, 1, 1.5, 2, 3, 4, 6])

    def real(qq, ss):
        n = unpack_nibbles(qq)
        return grid[n & 7] * np.where(n & 8, -1.0, 1.0) * np.exp2(np.repeat(ss.astype(np.float64), 32, axis=1) - 127)

    assert (real(q, sf) == real(q2, sf2)).all()
    # FP8 -> MXFP4 -> FP8: error at most half an E2M1 step (<= 1 unit) at the block scale
    x8, s = synth.tiny_roundtrip_fp8(seed=9)
    x8, s = x8.numpy(), s.numpy()
    q, sf = ref.quant_from_fp8(x8, s)
    xb, sb = ref.dequant_to_fp8(q, sf)
    dec = np.array([ref.e4m3_value(c) for c in range(256)])
    a = dec[x8] * np.repeat(s.astype(np.float64), 128, axis=1)
    b = dec[xb] * np.repeat(sb.astype(np.float64), 128, axis=1)
    step = np.exp2(np.repeat(sf.astype(np.float64), 32, axis=1) - 127)
    spread = np.repeat(sf.reshape(sf.shape[0], -1, 4).max(-1), 128, axis=1) - np.repeat(sf, 32, axis=1)
    ok = spread <= 14
    assert (np.abs(a - b)[ok] <= step[ok] * (1 + 1e-9)).all()
