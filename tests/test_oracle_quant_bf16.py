"""Pins for the oracle's BF16 -> MXFP4 quantizer, the row-wise kernel as the paper states it
(section 3.1).  CPU only."""
import numpy as np
import torch

from oracle import ref
from paper_2603_02731_amd import synth
from tests import bruteforce as bf
from tests.test_oracle_quant import unpack_nibbles


def bf16_bits(values):
    return torch.tensor(values, dtype=torch.float32).to(torch.bfloat16).view(torch.uint16).numpy()


def test_bf16_decode_matches_torch():
    # every finite pattern, through the scalar path of a block quantized with a unit-size partner:
    # decode is pinned against torch's own bfloat16 -> float32 view
    pats = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    want = torch.from_numpy(pats.view(np.int16)).view(torch.bfloat16).float().numpy()
    for h in list(range(0, 65536, 257)) + [0x0001, 0x007F, 0x0080, 0x7F7F, 0x7F80, 0xFF80, 0x8000]:
        fr = bf.bf16_fraction(h)
        if fr is None:
            assert np.isnan(want[h])
        elif fr[1] == bf.INF:
            assert np.isinf(want[h]) and (want[h] < 0) == bool(fr[0])
        else:
            assert float(fr[1]) == abs(float(want[h])) and bool(fr[0]) == bool(np.signbit(want[h]))


def test_worked_block_by_hand():
    # values 448, 1, .5, -.75, 2^-9, -0, 0, 3: group_max/6 = 74.67 -> 2^7 (byte 134); 448/128 = 3.5
    # is a tie between 3 (odd code 5) and 4 (even code 6) -> 6; the rest is below .25 -> 0, signs kept
    x = np.zeros((1, 128), np.uint16)
    x[0, :8] = bf16_bits([448.0, 1.0, 0.5, -0.75, 2.0 ** -9, -0.0, 0.0, 3.0])
    q, sf = ref.quant_from_bf16(x)
    assert sf[0, 0] == 134 and unpack_nibbles(q)[0, :8].tolist() == [6, 0, 0, 8, 0, 8, 0, 0]
    # 6, 4.5, 3, 2.25 -> byte 127, codes 7 6 5 4; one bf16 ulp above 6 (6.03125) -> byte 128, halves
    x[0, :8] = 0
    x[0, :4] = bf16_bits([6.0, 4.5, 3.0, 2.25])
    q, sf = ref.quant_from_bf16(x)
    assert sf[0, 0] == 127 and unpack_nibbles(q)[0, :4].tolist() == [7, 6, 5, 4]
    x[0, 0] = bf16_bits([6.0])[0] + 1
    q, sf = ref.quant_from_bf16(x)
    assert sf[0, 0] == 128 and unpack_nibbles(q)[0, :4].tolist() == [5, 4, 3, 2]


def test_random_and_edge_blocks_against_exact_brute_force():
    rng = np.random.default_rng(0)
    rows = []
    for t in range(96):
        if t % 4 == 0:      # arbitrary bit patterns: every exponent, NaN and inf included
            blk = rng.integers(0, 65536, size=128)
        elif t % 4 == 1:    # activations-like
            blk = bf16_bits((rng.standard_normal(128) * 10.0 ** rng.uniform(-3, 3)).tolist()).astype(np.int64)
        elif t % 4 == 2:    # subnormals and tiny values
            blk = rng.integers(0, 0x0200, size=128) | (rng.integers(0, 2, size=128) << 15)
        else:               # huge values near the top of the range
            blk = rng.integers(0x7E00, 0x7F80, size=128) | (rng.integers(0, 2, size=128) << 15)
        rows.append(blk.astype(np.uint16))
    x = np.stack(rows)
    q, sf = ref.quant_from_bf16(x)
    nib = unpack_nibbles(q)
    for r in range(x.shape[0]):
        for j in range(4):
            wb, wn = bf.quant_block_from_bf16([int(h) for h in x[r, 32 * j: 32 * j + 32]])
            assert int(sf[r, j]) == wb, (r, j)
            assert nib[r, 32 * j: 32 * j + 32].tolist() == wn, (r, j)


def test_agrees_with_the_fp8_path_where_both_are_exact():
    # an E4M3 value times a power-of-two scale is a BF16 number: both quantizers must agree
    x8, _ = synth.tiny_roundtrip_fp8(seed=4, M=64, K=512)
    x8 = x8.numpy()
    for j in (-20, -3, 0, 7, 60):
        s = np.full((64, 4), 2.0 ** j, np.float32)
        q8, sf8 = ref.quant_from_fp8(x8, s)
        vals = torch.from_numpy(x8).view(torch.float8_e4m3fn).float() * (2.0 ** j)
        xb = vals.to(torch.bfloat16)
        assert torch.equal(xb.float(), vals)              # exact in BF16
        qb, sfb = ref.quant_from_bf16(xb.view(torch.uint16).numpy())
        assert (q8 == qb).all() and (sf8 == sfb).all()


def test_invariants():
    rng = np.random.default_rng(1)
    x = bf16_bits((rng.standard_normal((32, 256)) * 3).ravel().tolist()).reshape(32, 256)
    q, sf = ref.quant_from_bf16(x)
    qn, sfn = ref.quant_from_bf16(x ^ 0x8000)                # sign symmetry
    assert (sf == sfn).all() and (q ^ 0x88 == qn).all()
    nib = unpack_nibbles(q)
    top = (nib & 7).reshape(32, 8, 32).max(-1)
    assert (top[sf > 0] >= 5).all()                          # normalised maximum in (3, 6]
    z = np.zeros((1, 128), np.uint16)
    z[0, 1] = 0x8000
    q, sf = ref.quant_from_bf16(z)
    assert sf[0, 0] == 0 and q[0, 0] == 0x80                 # zero block: byte 0, sign kept
    z[0, 40] = 0x7F80                                        # +inf: byte 254, code 7
    z[0, 41] = 0x3F80
    q, sf = ref.quant_from_bf16(z)
    assert sf[0, 1] == 254 and unpack_nibbles(q)[0, 40] == 7 and unpack_nibbles(q)[0, 41] == 0
    z[0, 70] = 0x7FC0                                        # NaN poisons its block only
    q, sf = ref.quant_from_bf16(z)
    assert sf[0, 2] == 0xFF and not q[0, 32:48].any() and sf[0, 1] == 254
