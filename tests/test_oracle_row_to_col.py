"""Pins for the oracle's row-blocked -> column-blocked MXFP4 conversion (section 3.4). CPU only."""
import numpy as np

from oracle import ref
from paper_2603_02731_amd import synth
from tests import bruteforce as bf
from tests.test_oracle_quant import unpack_nibbles

GRID = np.array([0, .5, 1, 1.5, 2, 3, 4, 6])


def real_rows(q, sf):
    n = unpack_nibbles(q)
    return GRID[n & 7] * np.where(n & 8, -1.0, 1.0) * np.exp2(np.repeat(sf.astype(np.float64), 32, axis=1) - 127)


def integer_form(q_row, sf_row):
    """The conversion re-derived in integers: with at most two significant bits,
    ceil(log2(x/6)) = floor(log2 x) - 2 and floor(log2 e2m1(code)) = exponent field - 1 for
    every non-zero code, so the column byte is max(0, max(b_row + field) - 3) and each
    element moves by the difference of the two bytes through an 8-entry table."""
    lut = {-3: [0, 6, 7, 7, 7, 7, 7, 7], -2: [0, 4, 6, 7, 7, 7, 7, 7], -1: [0, 2, 4, 5, 6, 7, 7, 7],
           0: [0, 1, 2, 3, 4, 5, 6, 7], 1: [0, 0, 1, 2, 2, 3, 4, 5], 2: [0, 0, 0, 1, 1, 2, 2, 3],
           3: [0, 0, 0, 0, 0, 1, 1, 2], 4: [0, 0, 0, 0, 0, 0, 0, 1]}
    nib = unpack_nibbles(q_row).astype(np.int64)
    M, K = nib.shape
    br = np.repeat(sf_row.astype(np.int64), 32, axis=1)
    field = (nib & 7) >> 1
    e = np.where((nib & 7) != 0, br + field, -10 ** 6)
    bc = np.maximum(0, e.reshape(M // 32, 32, K).max(axis=1) - 3)            # [M/32, K]
    d = np.repeat(bc, 32, axis=0) - br
    out = np.zeros_like(nib)
    for m in range(M):
        for k in range(K):
            dd = int(d[m, k])
            mag = 0 if dd >= 5 else lut[max(dd, -3)][nib[m, k] & 7]
            out[m, k] = (nib[m, k] & 8) | mag
    codes_t = out.T                                                          # [K, M]
    return (codes_t[:, 0::2] | (codes_t[:, 1::2] << 4)).astype(np.uint8), bc.T.astype(np.uint8)


def test_equals_integer_re_derivation():
    for seed, spread, center in [(0, 0, 127), (1, 3, 127), (2, 8, 100), (3, 20, 30), (4, 8, 3), (5, 6, 251)]:
        q, sf = synth.random_mxfp4(64, 128, seed=seed, scale_center=center, scale_spread=spread)
        q, sf = q.numpy(), sf.numpy()
        if seed == 2:
            q[:, :8] = 0                       # all-zero columns -> zero column scale
        qc, sc = ref.row_to_col(q, sf)
        wq, ws = integer_form(q, sf)
        assert (sc == ws).all(), seed
        assert (qc == wq).all(), seed
    assert not sc[:0].any()


def test_exact_rational_brute_force_on_tiles():
    rng = np.random.default_rng(5)
    for M, K in [(32, 128), (64, 128)]:
        q, sf = synth.random_mxfp4(M, K, seed=M, scale_center=127, scale_spread=4)
        q, sf = q.numpy(), sf.numpy()
        sf[:, 0] = rng.integers(119, 128, size=M)          # spread 0..8 inside the first tiles
        qc, sc = ref.row_to_col(q, sf)
        nib = unpack_nibbles(q)
        ncol = unpack_nibbles(qc)
        for mb in range(M // 32):
            for kb in range(0, K // 32, 3):
                tile = [[int(nib[mb * 32 + m, kb * 32 + k]) for k in range(32)] for m in range(32)]
                wsc, wcodes = bf.row_to_col_tile(tile, [int(sf[mb * 32 + m, kb]) for m in range(32)])
                for k in range(32):
                    assert int(sc[kb * 32 + k, mb]) == wsc[k]
                    assert ncol[kb * 32 + k, mb * 32: mb * 32 + 32].tolist() == wcodes[k]


def test_identity_and_idempotence():
    # equal row scales and a column whose largest code has exponent field 3: nothing changes
    q, sf = synth.random_mxfp4(64, 256, seed=8, scale_center=130, scale_spread=0)
    q, sf = q.numpy(), sf.numpy()
    nib = unpack_nibbles(q)
    nib[0::32, :] = 0x7                                     # a 6.0 in every column block
    q = (nib[:, 0::2] | (nib[:, 1::2] << 4)).astype(np.uint8)
    qc, sc = ref.row_to_col(q, sf)
    assert (sc == 130).all()
    assert (unpack_nibbles(qc) == nib.T).all()
    # applied twice the matrix comes back with the same real values where nothing was rounded
    q, sf = synth.random_mxfp4(128, 128, seed=9, scale_center=120, scale_spread=0)
    q, sf = q.numpy(), sf.numpy()
    qc, sc = ref.row_to_col(q, sf)
    qr, sr = ref.row_to_col(qc, sc)
    assert (real_rows(qr, sr) == real_rows(q, sf)).all()
    # and in general the real values move by at most half a step of the column scale
    q, sf = synth.random_mxfp4(128, 128, seed=10, scale_center=120, scale_spread=3)
    q, sf = q.numpy(), sf.numpy()
    qc, sc = ref.row_to_col(q, sf)
    a, b = real_rows(q, sf).T, real_rows(qc, sc)
    step = np.exp2(np.repeat(sc.astype(np.float64), 32, axis=1) - 127)
    assert (np.abs(a - b) <= step * (1 + 1e-12)).all()


def test_nan_row_scale_poisons_the_column_blocks_it_touches():
    q, sf = synth.random_mxfp4(64, 128, seed=11, scale_center=127, scale_spread=2)
    q, sf = q.numpy(), sf.numpy()
    sf[40, 2] = 0xFF
    qc, sc = ref.row_to_col(q, sf)
    assert (sc[64:96, 1] == 0xFF).all() and not qc[64:96, 16:32].any()
    sf[40, 2] = 127
    qc2, sc2 = ref.row_to_col(q, sf)
    mask = np.ones_like(sc, bool)
    mask[64:96, 1] = False
    assert (sc[mask] == sc2[mask]).all()


def test_grouped_equals_flat_per_expert():
    off = np.array([0, 64, 64, 160, 192], np.int32)
    q, sf = synth.random_mxfp4(192, 256, seed=12, scale_center=125, scale_spread=4)
    q, sf = q.numpy(), sf.numpy()
    K = 256
    qg, sg = ref.row_to_col_grouped(q, sf, off)
    for e in range(4):
        lo, hi = int(off[e]), int(off[e + 1])
        if hi == lo:
            continue
        wq, ws = ref.row_to_col(q[lo:hi], sf[lo:hi])
        assert (qg[K * lo // 2: K * hi // 2].reshape(K, (hi - lo) // 2) == wq).all()
        assert (sg[K * lo // 32: K * hi // 32].reshape(K, (hi - lo) // 32) == ws).all()


def test_ragged_splits_without_padding():
    # any T_e: expert e's nibbles [K, ceil(T_e/2)] and scales [K, ceil(T_e/32)] follow those of the experts
    # before it; a last block of fewer than 32 rows is quantized over the rows it has
    K = 128
    off = np.array([0, 5, 5, 37, 101, 132, 133, 197], np.int32)           # T = 5 0 32 64 31 1 64
    M = int(off[-1])
    q, sf = synth.random_mxfp4(M, K, seed=27, scale_center=120, scale_spread=6)
    q, sf = q.numpy(), sf.numpy()
    sf[110, 2] = 0xFF                                                     # NaN inside a partial block
    qc, sc = ref.row_to_col_grouped(q, sf, off)
    nib = unpack_nibbles(q)
    pb = bb = 0
    for e in range(len(off) - 1):
        lo, hi = int(off[e]), int(off[e + 1])
        T = hi - lo
        if T == 0:
            continue
        P, B = (T + 1) // 2, (T + 31) // 32
        got_q = qc[K * pb:K * (pb + P)].reshape(K, P)
        got_s = sc[K * bb:K * (bb + B)].reshape(K, B)
        # (a) the same rows padded with zero rows to a multiple of 32, through the flat function
        pad = B * 32 - T
        qp = np.concatenate([q[lo:hi], np.zeros((pad, K // 2), np.uint8)])
        sp = np.concatenate([sf[lo:hi], np.full((pad, K // 32), 200, np.uint8)])      # zero codes: byte irrelevant
        wq, ws = ref.row_to_col(qp, sp)
        assert (got_s == ws).all(), e
        codes = unpack_nibbles(wq)[:, :T]                                  # [K, T] nibble codes of the real rows
        want = np.zeros((K, 2 * P), np.uint8)
        want[:, :T] = codes
        assert (got_q == (want[:, 0::2] | (want[:, 1::2] << 4))).all(), e
        # (b) exact rationals on the partial last block of a few columns
        n_last = T - (B - 1) * 32
        rows = slice(lo + (B - 1) * 32, hi)
        for k in (0, 45, 70, K - 1):
            bytes_ = [int(b) for b in sf[rows, k // 32]]
            if 0xFF in bytes_:
                assert got_s[k, B - 1] == 0xFF
                continue
            vals = [((int(n) >> 3) & 1, bf.E2M1_GRID[int(n) & 7] * bf.pow2(b - 127)) for n, b in zip(nib[rows, k], bytes_)]
            vals += [(0, bf.Fraction(0))] * (32 - n_last)
            b_want, c_want = bf.quant_block(vals)
            assert got_s[k, B - 1] == b_want
            got_codes = unpack_nibbles(got_q[k:k + 1])[0, (B - 1) * 32:(B - 1) * 32 + n_last]
            assert got_codes.tolist() == c_want[:n_last]
        pb += P
        bb += B
    assert qc.size == K * pb and sc.size == K * bb
