"""Pins for the oracle's row-blocked MXFP4 -> column-wise FP8 conversion (section 3.4's fused
transposing kernel with the FP4 -> FP8 step of Algorithm 1, section 3.3, taken along m). CPU only."""
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
    lines = [l.strip() for l in open(os.path.join(GOLDEN, "fp8_col_worked_column.txt"))
             if l.strip() and not l.startswith("#")]
    head, scale_bits = lines[0].split("|")
    dbyte, dnib, dout = head.split()
    M, K = 128, 128
    nib = np.full((M, K), int(dnib, 16), np.uint8)
    sf = np.full((M, K // 32), int(dbyte), np.uint8)
    want = np.full(M, int(dout, 16), np.uint8)
    kcol = 37                                              # the worked column; it lies in k-block 1
    for l in lines[1:]:
        m, b, n, out = l.split()
        nib[int(m), kcol] = int(n, 16)
        sf[int(m), kcol // 32] = int(b)
        want[int(m)] = int(out, 16)
    x, xs = ref.row_to_fp8_col(pack_nibbles(nib), sf)
    assert xs.view(np.uint32)[kcol, 0] == int(scale_bits, 16)
    assert x[kcol].tolist() == want.tolist()
    # the other k-blocks never saw the exceptional scale bytes: all bytes 120, shift 0
    assert float(xs[0, 0]) == 2.0 ** (120 - 6 - 127)
    assert (x[0] == 0x68).all()                             # 1.0 * 2^6 = 64: E = 6 + 7 = 13


def test_exact_rational_brute_force_and_library_cast():
    rng = np.random.default_rng(11)
    M, K = 256, 128
    for trial in range(6):
        nib = rng.integers(0, 16, size=(M, K)).astype(np.uint8)
        nib[:16, 0] = np.arange(16)
        if trial % 3 == 0:      # close scales: the usual case
            sf = np.clip(int(rng.integers(8, 247)) + rng.integers(-4, 5, size=(M, K // 32)), 0, 254)
        elif trial % 3 == 1:    # wide spread: rounding through the subnormals and flush to zero
            sf = np.clip(int(rng.integers(30, 255)) - rng.integers(0, 24, size=(M, K // 32)), 0, 254)
        else:                   # anything, both ends of the byte range included
            sf = rng.integers(0, 255, size=(M, K // 32))
            sf[3, 0], sf[200, 1] = 254, 0
        sf = sf.astype(np.uint8)
        x, xs = ref.row_to_fp8_col(pack_nibbles(nib), sf)
        assert x.shape == (K, M) and xs.shape == (K, M // 128)
        for k in list(range(0, K, 9)) + [K - 1]:
            for g in range(M // 128):
                rows = slice(g * 128, (g + 1) * 128)
                bytes_ = [int(b) for b in sf[rows, k // 32]]
                S, want = bf.row_to_fp8_col_column([int(n) for n in nib[rows, k]], bytes_)
                assert Fraction(float(xs[k, g])) == S, (trial, k, g)
                assert x[k, rows].tolist() == want, (trial, k, g)
                bmax = max(bytes_)
                for e in range(128):
                    d = bmax - bytes_[e]
                    real = bf.E2M1_GRID[int(nib[g * 128 + e, k]) & 7] * bf.pow2(bytes_[e] - 127)
                    got = bf.e4m3_fraction(int(x[k, g * 128 + e]) & 0x7F) * S
                    if d <= 14:                             # lossless range of the alignment
                        assert got == real
                    if d >= 19:
                        assert (x[k, g * 128 + e] & 0x7F) == 0
                    assert (x[k, g * 128 + e] >> 7) == (nib[g * 128 + e, k] >> 3)
                # library pin: the same quotient in float32 (exact: two significant bits), cast by PyTorch
                units = [float(bf.E2M1_GRID[int(n) & 7] * bf.pow2(6 - (bmax - b)))
                         for n, b in zip(nib[rows, k], bytes_)]
                cast = torch.tensor(units, dtype=torch.float32).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
                assert ((x[k, rows] & 0x7F) == cast).all()
        assert (x & 0x7F).max() <= 0x7C                     # never above 384: no saturation


def test_reduces_to_the_row_wise_conversion_of_the_transposed_matrix():
    # When the row scales are constant over every 32 consecutive rows AND over a row's k-blocks,
    # the transposed matrix is itself a row-blocked MXFP4 matrix (blocks of 32 along m), and the
    # conversion is Algorithm 1 applied to it: the already pinned row-wise oracle function.
    rng = np.random.default_rng(3)
    M, K = 384, 256
    nib = rng.integers(0, 16, size=(M, K)).astype(np.uint8)
    per_group = np.clip(125 + rng.integers(-9, 10, size=M // 32), 0, 254).astype(np.uint8)
    per_group[5] = 100                                      # a far-away block: rounding + flush
    sf = np.repeat(per_group, 32)[:, None].repeat(K // 32, axis=1)
    x, xs = ref.row_to_fp8_col(pack_nibbles(nib), sf)
    sf_t = np.broadcast_to(per_group[None, :], (K, M // 32)).copy()
    x_t, xs_t = ref.dequant_to_fp8(pack_nibbles(nib.T.copy()), sf_t)
    assert (x == x_t).all()
    assert (xs.view(np.uint32) == xs_t.view(np.uint32)).all()


def test_uniform_scales_give_the_plain_transpose_of_the_row_wise_conversion():
    q, sf = synth.random_mxfp4(256, 256, seed=4, scale_center=131, scale_spread=0)
    q, sf = q.numpy(), sf.numpy()
    assert (sf == sf[0, 0]).all()
    x_row, xs_row = ref.dequant_to_fp8(q, sf)
    x_col, xs_col = ref.row_to_fp8_col(q, sf)
    assert (x_col == x_row.T).all()
    assert (xs_col == xs_row[0, 0]).all()


def test_nan_scale_byte_and_edges():
    M, K = 128, 128
    nib = np.full((M, K), 0x3, np.uint8)
    sf = np.full((M, K // 32), 120, np.uint8)
    sf[7, 1] = 0xFF
    sf[9, 1] = 125
    x, xs = ref.row_to_fp8_col(pack_nibbles(nib), sf)
    assert np.isnan(xs[32:64, 0]).all() and not np.isnan(xs[:32]).any() and not np.isnan(xs[64:]).any()
    assert (x[32:64, 7] == 0x7F).all()
    # the other rows align to the maximum of the non-NaN bytes (125)
    sf2 = sf.copy()
    sf2[7, 1] = 0
    x2, xs2 = ref.row_to_fp8_col(pack_nibbles(nib), sf2)
    keep = np.ones(M, bool)
    keep[7] = False
    assert (x[:, keep] == x2[:, keep]).all()
    assert float(xs2[40, 0]) == 2.0 ** (125 - 6 - 127)
    # smallest scales: an FP32 subnormal, exact
    sf3 = np.zeros((M, K // 32), np.uint8)
    sf3[0, 0] = 3
    _, xs3 = ref.row_to_fp8_col(pack_nibbles(nib), sf3)
    assert Fraction(float(xs3[0, 0])) == Fraction(2) ** (3 - 6 - 127)
    assert Fraction(float(xs3[64, 0])) == Fraction(2) ** (0 - 6 - 127)
    # empty and invalid shapes
    e_x, e_s = ref.row_to_fp8_col(np.zeros((0, 64), np.uint8), np.zeros((0, 4), np.uint8))
    assert e_x.shape == (128, 0) and e_s.shape == (128, 0)
    try:
        ref.row_to_fp8_col(np.zeros((96, 64), np.uint8), np.zeros((96, 4), np.uint8))
        assert False, "M % 128 != 0 must be rejected"
    except ValueError:
        pass


def test_grouped_equals_flat_per_expert():
    off = np.array([0, 128, 128, 512, 640], np.int32)
    q, sf = synth.random_mxfp4(640, 256, seed=8, scale_center=120, scale_spread=7)
    q, sf = q.numpy(), sf.numpy()
    xc, xs = ref.row_to_fp8_col_grouped(q, sf, off)
    K = 256
    for e in range(len(off) - 1):
        lo, hi = int(off[e]), int(off[e + 1])
        if hi == lo:
            continue
        wx, ws = ref.row_to_fp8_col(q[lo:hi], sf[lo:hi])
        assert (xc[K * lo:K * hi].reshape(K, hi - lo) == wx).all()
        assert (xs[K * lo // 128:K * hi // 128].reshape(K, (hi - lo) // 128).view(np.uint32) == ws.view(np.uint32)).all()


def test_ragged_splits_without_padding():
    # any T_e: expert e's bytes at K*off_e, its scales [K, ceil(T_e/128)] after those of the experts before
    K = 256
    off = np.array([0, 5, 5, 133, 389, 420, 676, 677], np.int32)          # T = 5 0 128 256 31 256 1
    M = int(off[-1])
    q, sf = synth.random_mxfp4(M, K, seed=21, scale_center=118, scale_spread=9)
    q, sf = q.numpy(), sf.numpy()
    sf[130, :] = 140                                                       # a maximum near a group edge
    sf[419, 2] = 0xFF                                                      # NaN in a partial group
    xc, xs = ref.row_to_fp8_col_grouped(q, sf, off)
    groups = [(int(off[e + 1] - off[e]) + 127) // 128 for e in range(len(off) - 1)]
    assert xs.shape[0] == K * sum(groups) and xc.shape[0] == K * M
    gb = 0
    nib = unpack_nibbles(q)
    for e in range(len(off) - 1):
        lo, hi = int(off[e]), int(off[e + 1])
        T, G = hi - lo, groups[e]
        if T == 0:
            continue
        got_x = xc[K * lo:K * hi].reshape(K, T)
        got_s = xs[K * gb:K * (gb + G)].reshape(K, G)
        # (a) the same rows padded with zero rows (scale byte 0) to a multiple of 128, through the flat function
        pad = G * 128 - T
        qp = np.concatenate([q[lo:hi], np.zeros((pad, K // 2), np.uint8)])
        sp = np.concatenate([sf[lo:hi], np.zeros((pad, K // 32), np.uint8)])
        wx, ws = ref.row_to_fp8_col(qp, sp)
        assert (got_x == wx[:, :T]).all(), e
        assert (got_s.view(np.uint32) == ws.view(np.uint32)).all(), e
        # (b) exact rationals on the partial last group of a few columns
        n_last = T - (G - 1) * 128
        for k in (0, 37, 70, K - 1):
            rows = slice(lo + (G - 1) * 128, hi)
            bytes_ = [int(b) for b in sf[rows, k // 32]]
            if 0xFF in bytes_:
                assert np.isnan(got_s[k, G - 1])
                continue
            S, want = bf.row_to_fp8_col_column([int(n) for n in nib[rows, k]], bytes_)
            assert Fraction(float(got_s[k, G - 1])) == S
            assert got_x[k, (G - 1) * 128:].tolist() == want and len(want) == n_last
        gb += G
    assert np.isnan(xs[K * (groups[0] + groups[1] + groups[2] + groups[3]) + 64 * groups[4]])   # k = 64, expert 4
