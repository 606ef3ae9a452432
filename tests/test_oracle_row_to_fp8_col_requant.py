"""Pins for the oracle's row-blocked MXFP4 -> column-wise FP8 conversion under the re-quantization reading
(section 3.4: de-quantize, transpose, re-quantize with the power-of-two scale 2^ceil(log2(amax/448))). CPU only."""
import os
from fractions import Fraction

import numpy as np
import torch

from oracle import ref
from paper_2603_02731_amd import synth
from tests import bruteforce as bf
from tests.test_oracle_dequant import pack_nibbles
from tests.test_oracle_quant import unpack_nibbles

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_hand_worked_column():
    lines = [l.strip() for l in open(os.path.join(GOLDEN, "fp8_col_requant_worked_column.txt"))
             if l.strip() and not l.startswith("#")]
    head, scale_bits = lines[0].split("|")
    dbyte, dnib, dout = head.split()
    M, K = 128, 128
    nib = np.full((M, K), int(dnib, 16), np.uint8)
    sf = np.full((M, K // 32), int(dbyte), np.uint8)
    want = np.full(M, int(dout, 16), np.uint8)
    kcol = 70                                               # the worked column; it lies in k-block 2
    for l in lines[1:]:
        m, b, n, out = l.split()
        sf[int(m), kcol // 32] = int(b)
        nib[int(m), kcol // 32 * 32:kcol // 32 * 32 + 32] = 0   # the other columns of that block: zeros
        nib[int(m), kcol] = int(n, 16)
        want[int(m)] = int(out, 16)
    x, xs = ref.row_to_fp8_col(pack_nibbles(nib), sf, requant=True)
    assert xs.view(np.uint32)[kcol, 0] == int(scale_bits, 16)
    assert x[kcol].tolist() == want.tolist()
    # an untouched k-block: every value 2^-7, S = 2^-15, every element 256 = 0x78
    assert float(xs[0, 0]) == 2.0 ** -15 and (x[0] == 0x78).all()


def emax_form(nib_col, bytes_col):
    """The scale re-derived in integers: a non-zero E2M1 code is (1 + M/2) * 2^(E-1) with E its exponent
    field (0.5 = 2^-1: E = 0), and 448 = 1.75 * 2^8 lies between 1.5 and 2 times a power of two, so
    ceil(log2(v/448)) = floor(log2 v) - 8 for every such v: S = 2^(max(b + E) - 136)."""
    keys = [int(b) + ((int(n) & 7) >> 1) for n, b in zip(nib_col, bytes_col) if (int(n) & 7) != 0]
    return None if not keys else max(keys) - 136


def test_exact_rational_brute_force_library_cast_and_integer_form():
    rng = np.random.default_rng(17)
    M, K = 256, 128
    for trial in range(6):
        nib = rng.integers(0, 16, size=(M, K)).astype(np.uint8)
        nib[:16, 0] = np.arange(16)
        nib[:, 5] &= 8                                      # an all-zero column (signs only)
        nib[:, 6] = np.where(rng.random(M) < 0.97, nib[:, 6] & 8, nib[:, 6])   # a sparse column
        if trial % 3 == 0:
            sf = np.clip(int(rng.integers(8, 247)) + rng.integers(-4, 5, size=(M, K // 32)), 0, 254)
        elif trial % 3 == 1:
            sf = np.clip(int(rng.integers(30, 255)) - rng.integers(0, 24, size=(M, K // 32)), 0, 254)
        else:
            sf = rng.integers(0, 255, size=(M, K // 32))
            sf[3, 0], sf[200, 1] = 254, 0
        sf = sf.astype(np.uint8)
        x, xs = ref.row_to_fp8_col(pack_nibbles(nib), sf, requant=True)
        xa, xsa = ref.row_to_fp8_col(pack_nibbles(nib), sf)            # the alignment reading, for comparison
        for k in list(range(0, K, 7)) + [5, 6, K - 1]:
            for g in range(M // 128):
                rows = slice(g * 128, (g + 1) * 128)
                bytes_ = [int(b) for b in sf[rows, k // 32]]
                nibs = [int(n) for n in nib[rows, k]]
                S, want = bf.row_to_fp8_col_requant_column(nibs, bytes_)
                assert Fraction(float(xs[k, g])) == S, (trial, k, g)
                assert x[k, rows].tolist() == want, (trial, k, g)
                j = emax_form(nibs, bytes_)
                assert S == (1 if j is None else bf.pow2(j))
                mags = x[k, rows] & 0x7F
                if j is not None:
                    assert 0x78 <= mags.max() <= 0x7E          # the largest element lands in [256, 448]
                else:
                    assert mags.max() == 0
                # never a coarser scale than the alignment reading; equal scales give equal bytes
                ratio = Fraction(float(xsa[k, g])) / S
                assert ratio >= 1 or j is None
                if ratio == 1:
                    assert (x[k, rows] == xa[k, rows]).all()
                # library pin: the same quotient in float32 (exact or far below the E4M3 range), cast by PyTorch
                units = [float(bf.E2M1_GRID[n & 7] * bf.pow2(b - 127) / S) for n, b in zip(nibs, bytes_)]
                cast = torch.tensor(units, dtype=torch.float32).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
                assert (mags == cast).all()
                assert ((x[k, rows] >> 7) == (nib[rows, k] >> 3)).all()


def test_nan_scale_byte_and_edges():
    M, K = 128, 128
    nib = np.full((M, K), 0x3, np.uint8)
    sf = np.full((M, K // 32), 120, np.uint8)
    sf[7, 1] = 0xFF
    sf[9, 1] = 125
    x, xs = ref.row_to_fp8_col(pack_nibbles(nib), sf, requant=True)
    assert np.isnan(xs[32:64, 0]).all() and not np.isnan(xs[:32]).any() and not np.isnan(xs[64:]).any()
    assert (x[32:64, 7] == 0x7F).all()
    sf2 = sf.copy()
    sf2[7, 1] = 0                                           # the other rows see the maximum of the non-NaN rows
    x2, xs2 = ref.row_to_fp8_col(pack_nibbles(nib), sf2, requant=True)
    keep = np.ones(M, bool)
    keep[7] = False
    assert (x[:, keep] == x2[:, keep]).all()
    # both ends of the scale range: 6 * 2^127 (beyond FP32 itself) and 0.5 * 2^-127
    nib3 = np.zeros((M, K), np.uint8)
    sf3 = np.zeros((M, K // 32), np.uint8)
    nib3[0, 0], sf3[0, 0] = 7, 254
    nib3[1, 40], sf3[1, 1] = 1, 0
    x3, xs3 = ref.row_to_fp8_col(pack_nibbles(nib3), sf3, requant=True)
    assert Fraction(float(xs3[0, 0])) == Fraction(2) ** (254 + 3 - 136) and x3[0, 0] == 0x7C
    assert Fraction(float(xs3[40, 0])) == Fraction(2) ** (0 + 0 - 136) and x3[40, 1] == 0x78
    assert float(xs3[1, 0]) == 1.0 and not x3[1].any()      # an all-zero group: scale 1


def test_ragged_groups_equal_zero_padded_flat():
    K = 256
    off = np.array([0, 5, 5, 133, 389, 420, 677], np.int32)
    M = int(off[-1])
    q, sf = synth.random_mxfp4(M, K, seed=23, scale_center=118, scale_spread=9)
    q, sf = q.numpy(), sf.numpy()
    xc, xs = ref.row_to_fp8_col_grouped(q, sf, off, requant=True)
    gb = 0
    for e in range(len(off) - 1):
        lo, hi = int(off[e]), int(off[e + 1])
        T, G = hi - lo, (hi - lo + 127) // 128
        if T == 0:
            continue
        pad = G * 128 - T
        qp = np.concatenate([q[lo:hi], np.zeros((pad, K // 2), np.uint8)])
        sp = np.concatenate([sf[lo:hi], np.full((pad, K // 32), 254, np.uint8)])   # zero codes: the byte is irrelevant
        wx, ws = ref.row_to_fp8_col(qp, sp, requant=True)
        assert (xc[K * lo:K * hi].reshape(K, T) == wx[:, :T]).all(), e
        assert (xs[K * gb:K * (gb + G)].reshape(K, G).view(np.uint32) == ws.view(np.uint32)).all(), e
        gb += G
