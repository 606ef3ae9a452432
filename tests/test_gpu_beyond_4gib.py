"""GPU parity on buffers larger than 4 GiB: [1310720, 7168] (9.4 GB of E4M3, 4.7 GB of nibbles), where
byte offsets no longer fit 32 bits.  The rows are 128-row groups of a [65536, 7168] base drawn with
repetition, so two kinds of check cover the outputs:
  * sampled rows / row groups (the first, the last, the ones around the 2^32-byte marks of every
    buffer, random ones) against the CPU oracle, bit for bit, fed with the bytes the kernels read;
  * every byte of every output against the output of the same entry point on the base, moved to
    where the group went (the conversions are independent per row, per 32-row block and per
    128-row group); the base-sized outputs are compared with the oracle in full elsewhere."""
import numpy as np
import pytest
import torch

import paper_2603_02731_amd as mx
from oracle import ref
from paper_2603_02731_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
K = 7168
BASE_GROUPS = 512                 # 65536 rows
GROUPS = 20 * BASE_GROUPS         # 1310720 rows
M = GROUPS * 128


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def same(got, want, what):
    got, want = np.asarray(got).reshape(-1), np.asarray(want).reshape(-1)
    assert got.size == want.size, (what, got.size, want.size)
    if got.dtype == np.float32:
        got, want = got.view(np.uint32), want.view(np.uint32)
    bad = np.flatnonzero(got != want)
    assert bad.size == 0, f"{what}: {bad.size} mismatches, first at {int(bad[0])}"


def sampled_groups(rng, row_bytes):
    """First, last, random groups and the groups holding the rows at the 2^32-byte marks of row-major buffers."""
    g = {0, 1, GROUPS - 1, GROUPS - 2}
    for rb in row_bytes:
        for mark in range(1, M * rb // 2**32 + 1):
            r = mark * 2**32 // rb
            g.update({max(r // 128 - 1, 0), min(r // 128, GROUPS - 1), min(r // 128 + 1, GROUPS - 1)})
    g.update(int(v) for v in rng.integers(0, GROUPS, 6))
    return sorted(g)


@pytest.fixture(scope="module")
def big():
    rng = np.random.default_rng(77)
    x8b, sb = synth.student_t_fp8(BASE_GROUPS * 128, K, seed=7, device=DEV)
    src_group = torch.from_numpy(rng.integers(0, BASE_GROUPS, GROUPS)).to(DEV)
    x8 = torch.empty((M, K), dtype=torch.uint8, device=DEV)
    s = torch.empty((M, K // 128), dtype=torch.float32, device=DEV)
    step = 1024
    for g0 in range(0, GROUPS, step):                   # device-side copies of whole groups
        sel = src_group[g0:g0 + step]
        x8[g0 * 128:(g0 + step) * 128].view(-1, 128, K).copy_(x8b.view(BASE_GROUPS, 128, K)[sel])
        s[g0 * 128:(g0 + step) * 128].view(-1, 128, K // 128).copy_(sb.view(BASE_GROUPS, 128, K // 128)[sel])
    qb, sfb = mx.mxfp4_quant_from_fp8(x8b, sb)
    q, sf = mx.mxfp4_quant_from_fp8(x8, s)
    torch.cuda.synchronize()
    assert x8.numel() > 2**32 and q.numel() > 2**32
    return {"x8": x8, "s": s, "q": q, "sf": sf, "qb": qb, "sfb": sfb, "src_group": src_group, "rng": rng}


def rows_follow_their_groups(out, out_base, src_group, what):
    """out [M, W] against out_base [65536, W], group by group, on the device."""
    W = out.shape[1]
    for g0 in range(0, GROUPS, 1024):
        sel = src_group[g0:g0 + 1024]
        want = out_base.view(BASE_GROUPS, 128, W)[sel]
        assert torch.equal(out[g0 * 128:(g0 + 1024) * 128].view(-1, 128, W), want), f"{what}: groups {g0}.."


def columns_follow_their_groups(out, out_base, src_group, per_group, what):
    """out [K, GROUPS*per_group] against out_base [K, 512*per_group], 256 k-rows at a time."""
    for k0 in range(0, K, 256):
        want = out_base[k0:k0 + 256].view(256, BASE_GROUPS, per_group)[:, src_group, :]
        assert torch.equal(out[k0:k0 + 256].view(256, GROUPS, per_group), want), f"{what}: k-rows {k0}.."


def test_quant_beyond_4gib(big):
    for g in sampled_groups(big["rng"], (K, K // 2)):
        r = slice(g * 128, (g + 1) * 128)
        wq, wsf = ref.quant_from_fp8(host(big["x8"][r]), host(big["s"][r]))
        same(host(big["sf"][r]), wsf, f"scale bytes of rows {r}")
        same(host(big["q"][r]), wq, f"nibbles of rows {r}")
    rows_follow_their_groups(big["q"], big["qb"], big["src_group"], "nibbles")
    rows_follow_their_groups(big["sf"], big["sfb"], big["src_group"], "scale bytes")


def test_dequant_beyond_4gib(big):
    x, xs = mx.mxfp4_dequant_to_fp8(big["q"], big["sf"])
    xb, xsb = mx.mxfp4_dequant_to_fp8(big["qb"], big["sfb"])
    for g in sampled_groups(big["rng"], (K, K // 2)):
        r = slice(g * 128, (g + 1) * 128)
        wx, wxs = ref.dequant_to_fp8(host(big["q"][r]), host(big["sf"][r]))
        same(host(xs[r]), wxs, f"tile scales of rows {r}")
        same(host(x[r]), wx, f"E4M3 bytes of rows {r}")
    rows_follow_their_groups(x, xb, big["src_group"], "E4M3 bytes")
    rows_follow_their_groups(xs.view(torch.int32), xsb.view(torch.int32), big["src_group"], "tile scales")


def test_row_to_col_beyond_4gib(big):
    qc, sc = mx.mxfp4_row_to_col(big["q"], big["sf"])
    qcb, scb = mx.mxfp4_row_to_col(big["qb"], big["sfb"])
    assert qc.shape == (K, M // 2) and qc.numel() > 2**32
    for g in sampled_groups(big["rng"], (K // 2,)):
        r = slice(g * 128, (g + 1) * 128)
        wqc, wsc = ref.row_to_col(host(big["q"][r]), host(big["sf"][r]))
        same(host(sc[:, g * 4:(g + 1) * 4]), wsc, f"column scale bytes of rows {r}")
        same(host(qc[:, g * 64:(g + 1) * 64]), wqc, f"column nibbles of rows {r}")
    columns_follow_their_groups(qc, qcb, big["src_group"], 64, "column nibbles")
    columns_follow_their_groups(sc, scb, big["src_group"], 4, "column scale bytes")


@pytest.mark.parametrize("requant", [False, True])
def test_row_to_fp8_col_beyond_4gib(big, requant):
    x, xs = mx.mxfp4_row_to_fp8_col(big["q"], big["sf"], requant=requant)
    xb, xsb = mx.mxfp4_row_to_fp8_col(big["qb"], big["sfb"], requant=requant)
    assert x.shape == (K, M) and x.numel() > 2**32
    for g in sampled_groups(big["rng"], (K // 2,)):
        r = slice(g * 128, (g + 1) * 128)
        wx, wxs = ref.row_to_fp8_col(host(big["q"][r]), host(big["sf"][r]), requant=requant)
        same(host(xs[:, g:g + 1]), wxs, f"group scales of rows {r}, requant={requant}")
        same(host(x[:, r]), wx, f"E4M3 bytes of rows {r}, requant={requant}")
    columns_follow_their_groups(x, xb, big["src_group"], 128, f"E4M3 bytes, requant={requant}")
    columns_follow_their_groups(xs.view(torch.int32), xsb.view(torch.int32), big["src_group"], 1,
                                f"group scales, requant={requant}")
