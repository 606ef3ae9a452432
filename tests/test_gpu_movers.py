"""The byte movers that serve as measured roofs: what each writes is fixed by its definition in the header
(no oracle is involved: they do no arithmetic of the method)."""
import numpy as np
import pytest
import torch

import paper_2603_02731_amd as mx

pytestmark = pytest.mark.gpu


def rnd(n, seed):
    return np.random.default_rng(seed).integers(0, 256, n, dtype=np.uint8)


@pytest.mark.parametrize("chunks", [1, 255, 1024, 4097])
@pytest.mark.parametrize("policy", [0, 1, 2, 3])
def test_stream_mixes(chunks, policy):
    a = rnd(16 * chunks, chunks + policy)
    src = torch.from_numpy(a).cuda()
    guard = 64
    # 1:1
    dst = torch.full((16 * chunks + guard,), 0xA5, dtype=torch.uint8, device="cuda")
    mx.mxfp4_stream_copy(src, dst[:16 * chunks], policy=policy)
    got = dst.cpu().numpy()
    assert np.array_equal(got[:16 * chunks], a) and (got[16 * chunks:] == 0xA5).all()
    # 2:1: every 16 bytes leave as the xor of their two halves
    dst = torch.full((8 * chunks + guard,), 0xA5, dtype=torch.uint8, device="cuda")
    mx.mxfp4_stream_mix(src, dst[:8 * chunks], 1, policy=policy)
    got = dst.cpu().numpy()
    w = a.reshape(chunks, 2, 8)
    assert np.array_equal(got[:8 * chunks], (w[:, 0] ^ w[:, 1]).reshape(-1)) and (got[8 * chunks:] == 0xA5).all()
    # 1:2: every 8 bytes leave twice
    half = src[:8 * chunks]
    dst = torch.full((16 * chunks + guard,), 0xA5, dtype=torch.uint8, device="cuda")
    mx.mxfp4_stream_mix(half, dst[:16 * chunks], 2, policy=policy)
    got = dst.cpu().numpy()
    h = a[:8 * chunks].reshape(chunks, 1, 8)
    assert np.array_equal(got[:16 * chunks], np.concatenate([h, h], 1).reshape(-1)) and (got[16 * chunks:] == 0xA5).all()
    # read only: nothing but possibly byte 0 of dst is touched
    dst = torch.full((guard,), 0xA5, dtype=torch.uint8, device="cuda")
    mx.mxfp4_stream_mix(src, dst, 3, policy=policy)
    assert (dst.cpu().numpy()[1:] == 0xA5).all()


@pytest.mark.parametrize("rows,row_bytes", [(256, 128), (512, 384), (2304, 1152), (8448, 256)])
def test_tile_copy_moves_every_piece_where_the_header_says(rows, row_bytes):
    a = rnd(rows * row_bytes, rows).reshape(rows, row_bytes)
    src = torch.from_numpy(a).cuda()
    dst = torch.full((rows * row_bytes + 64,), 0xA5, dtype=torch.uint8, device="cuda")
    mx.mxfp4_tile_copy(src, dst[:rows * row_bytes])
    got = dst.cpu().numpy()
    assert (got[rows * row_bytes:] == 0xA5).all()
    out = got[:rows * row_bytes].reshape(2 * row_bytes, rows // 2)
    tm, tk = rows // 256, row_bytes // 128
    # tile (i, j) of src, as 256 pieces of 128 bytes in reading order, lands in rows 256 j .. of dst at byte 128 i
    want = a.reshape(tm, 256, tk, 128).transpose(2, 1, 0, 3).reshape(2 * row_bytes, rows // 2)
    assert np.array_equal(out, want)


@pytest.mark.parametrize("M,fanout,rec,ld", [(1, 1, 16, 16), (37, 3, 3808, 3808), (300, 8, 3808, 7392), (5, 2, 49152, 49152)])
def test_record_fanout(M, fanout, rec, ld):
    rng = np.random.default_rng(M * fanout)
    a = rnd(M * ld, M).reshape(M, ld)
    M_out = M * fanout + 5
    perm = rng.permutation(M_out)[:M * fanout].astype(np.int32).reshape(M, fanout)
    perm[M // 2, 0] = -1          # skipped
    perm[0, fanout - 1] = M_out   # skipped
    dst = torch.full((M_out * rec,), 0xA5, dtype=torch.uint8, device="cuda")
    mx.mxfp4_record_fanout(torch.from_numpy(a).cuda(), torch.from_numpy(perm).cuda(), dst, rec_bytes=rec)
    got = dst.cpu().numpy().reshape(M_out, rec)
    want = np.full((M_out, rec), 0xA5, dtype=np.uint8)
    for i in range(M):
        for j in range(fanout):
            if 0 <= perm[i, j] < M_out:
                want[perm[i, j]] = a[i, :rec]
    assert np.array_equal(got, want)


def test_mover_argument_errors():
    z = torch.zeros(64, dtype=torch.uint8, device="cuda")
    with pytest.raises(ValueError):
        mx.mxfp4_stream_mix(z[:24], z, 0)
    with pytest.raises(ValueError):
        mx.mxfp4_stream_mix(z, z[:16], 0)
    with pytest.raises(ValueError):
        mx.mxfp4_stream_mix(z, z, 4)
    with pytest.raises(ValueError):
        mx.mxfp4_tile_copy(torch.zeros(100, 128, dtype=torch.uint8, device="cuda"), z)
    with pytest.raises(TypeError):
        mx.mxfp4_stream_mix(torch.zeros(64, dtype=torch.uint8), z, 0)
    idx = torch.zeros(4, 2, dtype=torch.int32, device="cuda")
    with pytest.raises(ValueError):
        mx.mxfp4_record_fanout(torch.zeros(4, 24, dtype=torch.uint8, device="cuda"), idx, z)
    with pytest.raises(ValueError):
        mx.mxfp4_record_fanout(torch.zeros(3, 32, dtype=torch.uint8, device="cuda"), idx, z)
    with pytest.raises(ValueError):
        mx.mxfp4_record_fanout(torch.zeros(4, 48, dtype=torch.uint8, device="cuda"), idx, z)
