"""Pins for the oracle's FP8 -> MXFP4 quantizer (CPU only)."""
import os
import random
import struct

import numpy as np
import pytest

from oracle import ref
from paper_2603_02731_amd import synth
from tests import bruteforce as bf

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def bits_of(f):
    return struct.unpack("<I", struct.pack("<f", f))[0]


def f32_from_bits(b):
    return struct.unpack("<f", struct.pack("<I", b))[0]


def unpack_nibbles(q):
    q = np.asarray(q, np.uint8)
    out = np.empty(q.shape[:-1] + (q.shape[-1] * 2,), np.uint8)
    out[..., 0::2] = q & 0xF
    out[..., 1::2] = q >> 4
    return out


def quant_one_block(codes, s):
    x = np.zeros((1, 128), np.uint8)
    x[0, : len(codes)] = codes
    q, sf = ref.quant_from_fp8(x, np.array([[s]], np.float32))
    return int(sf[0, 0]), unpack_nibbles(q)[0, :32].tolist()


def test_hand_worked_blocks():
    n = 0
    for line in open(os.path.join(GOLDEN, "quant_worked_blocks.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        codes, s, byte, nibs = [p.strip() for p in line.split("|")]
        codes = [int(c, 16) for c in codes.split()]
        nibs = [int(c, 16) for c in nibs.split()]
        b, got = quant_one_block(codes, float.fromhex(s))
        assert b == int(byte), line
        assert got[: len(nibs)] == nibs, line
        assert all(g == 0 for g in got[len(nibs):])
        # the exact-rational brute force agrees with the hand derivation too
        bb, bn = bf.quant_block_from_fp8(codes + [0] * (32 - len(codes)), bits_of(float.fromhex(s)))
        assert bb == int(byte) and bn[: len(nibs)] == nibs
        n += 1
    assert n == 7


def scale_sweep():
    rng = random.Random(7)
    s = [2.0 ** k for k in (-140, -133, -126, -60, -20, -7, -1, 0, 3, 10, 60, 100, 119, 120)]
    # amax/448-style scales with random mantissas
    s += [float(np.float32(rng.uniform(0.01, 300.0)) / np.float32(448)) for _ in range(12)]
    # double-rounding witnesses (product lands on an E2M1 tie only after the FP32 rounding)
    s += [float.fromhex("0x1.aaaaacp+1"), float.fromhex("0x1.555556p+1"), float.fromhex("0x1.1c71c8p+2")]
    # scales that put a block maximum on 6*2^k and 3*2^k, and one ulp either side
    for base in (6.0, 3.0, 6.0 / 448, 3.0 / 448, 6.0 / 1.75):
        f = np.float32(base)
        s += [float(f), float(np.nextafter(f, np.float32(np.inf))), float(np.nextafter(f, np.float32(0)))]
    # subnormal scale, zero scale, scale near FLT_MAX/448 (products overflow for big codes)
    s += [2.0 ** -149, 3 * 2.0 ** -149, 0.0, float(np.finfo(np.float32).max) / 448,
          float(np.finfo(np.float32).max) / 16]
    return s


def test_all_codes_times_scale_sweep_against_exact_brute_force():
    rng = random.Random(11)
    scales = scale_sweep()
    codes = list(range(256))
    for s in scales:
        rng.shuffle(codes)
        x = np.array(codes, np.uint8).reshape(2, 128)
        q, sf = ref.quant_from_fp8(x, np.array([[s], [s]], np.float32))
        nib = unpack_nibbles(q)
        for r in range(2):
            for j in range(4):
                blk = x[r, 32 * j: 32 * j + 32].tolist()
                wb, wn = bf.quant_block_from_fp8(blk, bits_of(np.float32(s)))
                assert int(sf[r, j]) == wb, (s, r, j)
                assert nib[r, 32 * j: 32 * j + 32].tolist() == wn, (s, r, j)


def test_power_of_two_scales_every_code_under_every_block_maximum():
    # with s = 2^j the product is exact, so (code, block-max code) decides everything
    for j in (-131, -9, 0, 5, 118):
        rows = []
        for cmax in range(1, 0x7F):
            others = list(range(0, cmax + 1))
            for i in range(0, len(others), 31):
                blk = [cmax] + others[i: i + 31]
                blk += [0] * (32 - len(blk))
                sign = [0x80 if (k + cmax) % 3 == 0 else 0 for k in range(32)]
                rows.append([b | sg for b, sg in zip(blk, sign)])
        nblk = len(rows)
        pad = (-nblk) % 4
        rows += [[0] * 32] * pad
        x = np.array(rows, np.uint8).reshape(-1, 128)
        s = np.full((x.shape[0], 1), 2.0 ** j, np.float32)
        q, sf = ref.quant_from_fp8(x, s)
        nib = unpack_nibbles(q).reshape(-1, 32)
        sfl = sf.reshape(-1)
        for bi in range(0, nblk, 7):         # every 7th block through the slow checker
            wb, wn = bf.quant_block_from_fp8(rows[bi], bits_of(np.float32(2.0 ** j)))
            assert int(sfl[bi]) == wb and nib[bi].tolist() == wn, (j, bi)
        # invariants on all of them: normalised maximum in (3, 6] -> largest code is 5, 6 or 7
        for bi in range(nblk):
            if 0 < sfl[bi] < 254:
                assert (nib[bi] & 7).max() >= 5, (j, bi)


def test_invariants_zero_sign_nan_saturation():
    # a zero block gives a zero scale byte; the sign bit is always copied
    b, n = quant_one_block([0x00, 0x80, 0x00], 1.0)
    assert b == 0 and n[:3] == [0, 8, 0]
    b, n = quant_one_block([0x7E, 0xFE], 0.0)      # zero scale: zero tile
    assert b == 0 and n[:2] == [0, 8]
    # NaN poisons its own block only
    x = np.zeros((1, 128), np.uint8)
    x[0, 3] = 0x7F
    x[0, 40] = 0x38
    x[0, 70] = 0xFF
    q, sf = ref.quant_from_fp8(x, np.array([[1.0]], np.float32))
    assert sf[0].tolist() == [0xFF, 125, 0xFF, 0]
    assert not q[0, :16].any() and not q[0, 32:48].any()
    # overflowing product: byte 254, code 7, the rest scaled by 2^-127
    big = float(np.finfo(np.float32).max) / 16
    b, n = quant_one_block([0x7E, 0x08], big)       # 448*big overflows; 2^-6*big = ~2^118
    assert b == 254 and n[0] == 7 and n[1] == 0
    # sign symmetry and block independence
    x8, s = synth.tiny_roundtrip_fp8(seed=3)
    x8, s = x8.numpy(), s.numpy()
    q, sf = ref.quant_from_fp8(x8, s)
    qn, sfn = ref.quant_from_fp8(x8 ^ 0x80, s)
    assert (sf == sfn).all() and (q ^ 0x88 == qn).all()
    # sizes are the closed form of section 3.2
    M, K = x8.shape
    assert q.size + sf.size == synth.payload_bytes(M, K)["mxfp4"]
    assert x8.size + 4 * s.size == synth.payload_bytes(M, K)["fp8"]
    # error bound: |y - grid| is at most half an E2M1 step at the block scale
    nib = unpack_nibbles(q)
    val = np.array([0, .5, 1, 1.5, 2, 3, 4, 6])[nib & 7] * np.where(nib & 8, -1.0, 1.0)
    x_real = np.array([[ref.e4m3_value(c) for c in row] for row in x8[:8]]) * np.repeat(s[:8], 128, axis=1)
    y = x_real / np.exp2(np.repeat(sf[:8].astype(np.float64), 32, axis=1) - 127)
    assert np.nanmax(np.abs(y - val[:8])) <= 1.0 + 1e-6      # widest step is 2 (between 4 and 6)
    assert (np.abs(y) <= 6 * (1 + 1e-6)).all()


def test_gather_and_strides():
    x8, s = synth.tiny_roundtrip_fp8(seed=5, M=64, K=256)
    x8, s = x8.numpy(), s.numpy()
    q, sf = ref.quant_from_fp8(x8, s)
    idx = np.array([5, 5, 0, 63, 17, 2], np.int32)
    qg, sfg = ref.quant_from_fp8(x8, s, gather_idx=idx)
    assert (qg == q[idx]).all() and (sfg == sf[idx]).all()
    # interleaved records: nibbles and scales of a token back to back
    import ctypes
    M, K = x8.shape
    rec = K // 2 + K // 32
    buf = np.zeros(M * rec, np.uint8)
    L = ref.lib()
    u8p = ctypes.POINTER(ctypes.c_uint8)
    f32p = ctypes.POINTER(ctypes.c_float)
    base = buf.ctypes.data
    rc = L.mxfp4_ref_quant_from_fp8(x8.ctypes.data_as(u8p), s.ctypes.data_as(f32p), M, K, None, M,
                                    ctypes.cast(base, u8p), rec, ctypes.cast(base + K // 2, u8p), rec)
    assert rc == 0
    recs = buf.reshape(M, rec)
    assert (recs[:, : K // 2] == q).all() and (recs[:, K // 2:] == sf).all()


def test_grouped_equals_flat():
    off, counts = synth.expert_offsets(seed=2, num_experts=5, total_tokens=300, pad_to=32)
    M = int(off[-1])
    x8, s = synth.student_t_fp8(M, K=256, seed=4)
    x8, s = synth.zero_padding_rows(x8, s, off, counts)
    q, sf = ref.quant_from_fp8(x8.numpy(), s.numpy())
    qg, sfg = ref.quant_from_fp8_grouped(x8.numpy(), s.numpy(), off.numpy())
    assert (q == qg).all() and (sf == sfg).all()
    # padding rows are zero blocks: zero scale byte
    lo, hi = int(off[0]) + int(counts[0]), int(off[1])
    assert not sf[lo:hi].any() and not q[lo:hi].any()


def test_scatter_is_the_gather_turned_around():
    # each source row to 3 output rows: the gather form (pinned above) with the inverse map gives the same rows;
    # skipped entries and rows that nobody names are left alone
    rng = np.random.default_rng(4)
    x8, s = synth.tiny_roundtrip_fp8(seed=2)
    x8, s = x8.numpy()[:40], s.numpy()[:40]
    M, fan = x8.shape[0], 3
    M_out = M * fan + 7
    perm = rng.permutation(M_out)[:M * fan].reshape(M, fan).astype(np.int32)
    perm[5, 1] = -1                                          # skipped
    perm[9, 0] = M_out + 3                                   # out of range: skipped
    q0 = rng.integers(0, 256, size=(M_out, x8.shape[1] // 2)).astype(np.uint8)
    sf0 = rng.integers(0, 255, size=(M_out, x8.shape[1] // 32)).astype(np.uint8)
    q, sf = ref.quant_from_fp8_scatter(x8, s, perm, M_out, q=q0.copy(), sf=sf0.copy())
    named = np.zeros(M_out, bool)
    for i in range(M):
        for d in perm[i]:
            if 0 <= d < M_out:
                named[d] = True
    src_of = np.zeros(M_out, np.int32)
    for i in range(M):
        for d in perm[i]:
            if 0 <= d < M_out:
                src_of[d] = i
    wq, wsf = ref.quant_from_fp8(x8, s, gather_idx=src_of)
    assert named.sum() == M * fan - 2
    assert (q[named] == wq[named]).all() and (sf[named] == wsf[named]).all()
    assert (q[~named] == q0[~named]).all() and (sf[~named] == sf0[~named]).all()


def test_scales_outside_the_format_follow_ieee_products():
    """FP32 tile scales that no blockwise-FP8 producer emits.  The element value is the IEEE-754 product
    fl32(e4m3 * s), here taken with numpy's float32 multiply: NaN (a NaN scale, or an infinite scale times a zero
    code) poisons the block (byte 0xFF, codes 0); +-inf gives byte 254 and code 7 with the product's sign; a
    negative finite scale only flips the signs."""
    rng = np.random.default_rng(5)
    row = rng.integers(0, 256, 256, dtype=np.int64).astype(np.uint8)
    row[(row & 0x7F) == 0x7F] = 0x3A            # no NaN codes
    row[0:32][(row[0:32] & 0x7F) == 0] = 0x11  # block 0 of tile 0: no zeros
    row[40] = 0x00                              # block 1: a zero
    row[70] = 0x80                              # block 2: a negative zero
    row[96:128][(row[96:128] & 0x7F) == 0] = 0x95  # block 3: no zeros
    x = np.stack([row, row])
    e4m3 = np.array([(-1.0 if c & 0x80 else 1.0) * float(bf.e4m3_fraction(int(c) & 0x7F)) for c in row], np.float32)
    for s in (np.inf, -np.inf, np.nan):
        q, sf = ref.quant_from_fp8(x, np.array([[s, 1.0], [1.0, s]], np.float32))
        nib = unpack_nibbles(q)
        with np.errstate(invalid="ignore"):
            p = e4m3[:128] * np.float32(s)
        for blk in range(4):
            pv = p[32 * blk: 32 * blk + 32]
            got_sf, got = sf[0, blk], nib[0, 32 * blk: 32 * blk + 32]
            if np.isnan(pv).any():
                assert got_sf == 0xFF and (got == 0).all(), (s, blk)
            else:
                assert got_sf == 254, (s, blk)
                assert np.array_equal(got, np.where(np.signbit(pv), 0xF, 0x7)), (s, blk)
        # the other row: tile 1 carries the scale, tile 0 (scale 1) is untouched by it
        q1, sf1 = ref.quant_from_fp8(x, np.ones((2, 2), np.float32))
        assert np.array_equal(sf[1, :4], sf1[1, :4]) and np.array_equal(q[1, :64], q1[1, :64])
    qa, sfa = ref.quant_from_fp8(x, np.full((2, 2), 0.375, np.float32))
    qb, sfb = ref.quant_from_fp8(x, np.full((2, 2), -0.375, np.float32))
    assert np.array_equal(sfa, sfb)
    na, nb = unpack_nibbles(qa), unpack_nibbles(qb)
    assert np.array_equal(na ^ 8, nb)
