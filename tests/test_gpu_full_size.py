"""GPU parity at the full sizes of the five configurations and of the benchmark workload,
in the launch configuration bench.py times.  Outputs are compared with the CPU oracle bit
for bit: completely where the oracle finishes in seconds (it runs over row ranges in a thread
pool), the 524288-row dispatch payload included (65536 records at a time)."""
import numpy as np
import pytest
import torch

import paper_2603_02731_amd as mx
from oracle import parallel as par
from oracle import ref
from paper_2603_02731_amd import synth
from tests.test_gpu_parity import assert_same, host

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def target():
    """The benchmark workload: [65536, 7168] Student-t activations, generated on the GPU."""
    x8, s = synth.student_t_fp8(65536, 7168, seed=0, device=DEV)
    q, sf = mx.mxfp4_quant_from_fp8(x8, s)
    torch.cuda.synchronize()
    return {"x8": x8, "s": s, "q": q, "sf": sf}


def test_config2_quant_dequant_4096x7168():
    x8, s = synth.student_t_fp8(4096, 7168, seed=1, device=DEV)
    q, sf = mx.mxfp4_quant_from_fp8(x8, s)
    wq, wsf = par.quant(host(x8), host(s))
    assert q.shape == (4096, 3584) and sf.shape == (4096, 224)
    assert_same(host(sf), wsf, "cfg2 scale bytes")
    assert_same(host(q), wq, "cfg2 nibbles")
    x, xs = mx.mxfp4_dequant_to_fp8(q, sf)
    wx, wxs = par.dequant(wq, wsf)
    assert_same(host(xs), wxs, "cfg2 tile scales")
    assert_same(host(x), wx, "cfg2 E4M3 bytes")


def test_config3_row_to_col_16384x2048():
    x8, s = synth.swiglu_fp8(16384, 2048, seed=2, device=DEV)
    wq, wsf = par.quant(host(x8), host(s))            # the input of this config comes from the oracle
    qc, sc = mx.mxfp4_row_to_col(torch.from_numpy(wq).to(DEV), torch.from_numpy(wsf).to(DEV))
    wqc, wsc = par.row_to_col(wq, wsf)
    assert qc.shape == (2048, 8192) and sc.shape == (2048, 512)
    assert_same(host(sc), wsc, "cfg3 column scale bytes")
    assert_same(host(qc), wqc, "cfg3 column nibbles")


def test_config4_grouped_32_experts():
    off, counts = synth.expert_offsets(seed=3, num_experts=32, total_tokens=65536, pad_to=128)
    M = int(off[-1])
    offd = off.to(DEV)
    # quant path: FP8 [sum T_e, 7168], padding rows zero
    x8, s = synth.student_t_fp8(M, 7168, seed=4, device=DEV)
    x8, s = synth.zero_padding_rows(x8, s, off, counts)
    q, sf = mx.mxfp4_quant_from_fp8_grouped(x8, s, offd)
    wq, wsf = par.quant(host(x8), host(s))             # grouped == flat, pinned on the CPU
    assert_same(host(sf), wsf, "cfg4 quant scale bytes")
    assert_same(host(q), wq, "cfg4 quant nibbles")
    del x8, s, q, sf, wq, wsf
    # row->col path: MXFP4 [sum T_e, 2048]
    y8, ys = synth.swiglu_fp8(M, 2048, seed=5, device=DEV)
    y8, ys = synth.zero_padding_rows(y8, ys, off, counts)
    rq, rsf = par.quant(host(y8), host(ys))
    qc, sc = mx.mxfp4_row_to_col_grouped(torch.from_numpy(rq).to(DEV), torch.from_numpy(rsf).to(DEV), offd)
    qc, sc = host(qc), host(sc)
    K = 2048
    for e in range(32):                                # per expert against the flat oracle routine
        lo, hi = int(off[e]), int(off[e + 1])
        wqc, wsc = par.row_to_col(rq[lo:hi], rsf[lo:hi], workers=4)
        assert_same(sc[K * lo // 32: K * hi // 32].reshape(K, (hi - lo) // 32), wsc, f"cfg4 expert {e} scales")
        assert_same(qc[K * lo // 2: K * hi // 2].reshape(K, (hi - lo) // 2), wqc, f"cfg4 expert {e} nibbles")


def test_target_quant_65536x7168(target):
    wq, wsf = par.quant(host(target["x8"]), host(target["s"]))
    assert_same(host(target["sf"]), wsf, "target scale bytes")
    assert_same(host(target["q"]), wq, "target nibbles")


def test_target_dequant_65536x7168(target):
    x, xs = mx.mxfp4_dequant_to_fp8(target["q"], target["sf"])
    wx, wxs = par.dequant(host(target["q"]), host(target["sf"]))
    assert_same(host(xs), wxs, "target tile scales")
    assert_same(host(x), wx, "target E4M3 bytes")


def test_target_row_to_col_65536x7168(target):
    qc, sc = mx.mxfp4_row_to_col(target["q"], target["sf"])
    wqc, wsc = par.row_to_col(host(target["q"]), host(target["sf"]))
    assert_same(host(sc), wsc, "target column scale bytes")
    assert_same(host(qc), wqc, "target column nibbles")


def test_target_row_to_fp8_col_65536x7168(target):
    x, xs = mx.mxfp4_row_to_fp8_col(target["q"], target["sf"])
    wx, wxs = par.row_to_fp8_col(host(target["q"]), host(target["sf"]))
    assert x.shape == (7168, 65536) and xs.shape == (7168, 512)
    assert_same(host(xs), wxs, "target FP8 column group scales")
    assert_same(host(x), wx, "target FP8 column bytes")


def test_target_row_to_fp8_col_requant_65536x7168(target):
    x, xs = mx.mxfp4_row_to_fp8_col(target["q"], target["sf"], requant=True)
    wx, wxs = par.row_to_fp8_col(host(target["q"]), host(target["sf"]), requant=True)
    assert_same(host(xs), wxs, "target FP8 column group scales (requant)")
    assert_same(host(x), wx, "target FP8 column bytes (requant)")


def test_config4_grouped_row_to_fp8_col_32_experts():
    off, counts = synth.expert_offsets(seed=3, num_experts=32, total_tokens=65536, pad_to=128)
    M, K = int(off[-1]), 2048
    y8, ys = synth.swiglu_fp8(M, K, seed=5, device=DEV)
    y8, ys = synth.zero_padding_rows(y8, ys, off, counts)
    rq, rsf = par.quant(host(y8), host(ys))
    x, xs = mx.mxfp4_row_to_fp8_col_grouped(torch.from_numpy(rq).to(DEV), torch.from_numpy(rsf).to(DEV), off.to(DEV))
    x, xs = host(x), host(xs)
    for e in range(32):                                # per expert against the flat oracle routine
        lo, hi = int(off[e]), int(off[e + 1])
        wx, wxs = par.row_to_fp8_col(rq[lo:hi], rsf[lo:hi], workers=4)
        assert_same(xs[K * lo // 128: K * hi // 128].reshape(K, (hi - lo) // 128), wxs, f"cfg4 expert {e} FP8 scales")
        assert_same(x[K * lo: K * hi].reshape(K, hi - lo), wx, f"cfg4 expert {e} FP8 bytes")


def test_config5_dispatch_payload_round_trip(target):
    x8, s = target["x8"], target["s"]
    M, K, top_k = 65536, 7168, 8
    idx = synth.routing_indices(seed=6, num_tokens=M, top_k=top_k, device=DEV)
    Mo = M * top_k
    rec = K // 2 + K // 32                                   # 3808-byte records: nibbles then scales
    buf = torch.empty(Mo * rec, dtype=torch.uint8, device=DEV)
    mx.mxfp4_quant_from_fp8(x8, s, gather_idx=idx, q=buf, sf=buf[K // 2:], ld_q=rec, ld_sf=rec)
    recs = buf.view(Mo, rec)
    # property that holds at any size: every output row is the planar quantization of its source row
    qsrc, sfsrc = target["q"], target["sf"]
    li = idx.long()
    for lo in range(0, Mo, 65536):
        sl = slice(lo, lo + 65536)
        assert torch.equal(recs[sl, : K // 2], qsrc[li[sl]])
        assert torch.equal(recs[sl, K // 2:], sfsrc[li[sl]])
    # the same payload by the scatter form (every token quantized once): byte for byte the same records
    dst = torch.argsort(li, stable=True).to(torch.int32).view(M, top_k).contiguous()
    buf2 = torch.zeros(Mo * rec, dtype=torch.uint8, device=DEV)
    mx.mxfp4_quant_from_fp8_scatter(x8, s, dst, Mo, q=buf2, sf=buf2[K // 2:], ld_q=rec, ld_sf=rec)
    assert torch.equal(buf2, buf)
    del buf2, dst
    # the oracle's own gathered form on sampled rows (the routine with the index argument)
    g = torch.Generator().manual_seed(7)
    rows = torch.randperm(Mo, generator=g)[:4096].sort().values
    xs_h, s_h, idx_h = host(x8), host(s), host(idx)
    wq, wsf = ref.quant_from_fp8(xs_h, s_h, gather_idx=idx_h[rows.numpy()])
    got = host(recs[rows.to(DEV)])
    assert_same(got[:, : K // 2], wq, "cfg5 sampled record nibbles")
    assert_same(got[:, K // 2:], wsf, "cfg5 sampled record scales")
    # and back: dequantize the whole payload from the records
    x = torch.empty((Mo, K), dtype=torch.uint8, device=DEV)
    xsc = torch.empty((Mo, K // 128), dtype=torch.float32, device=DEV)
    mx.mxfp4_dequant_to_fp8(buf, buf[K // 2:], M=Mo, K=K, ld_q=rec, ld_sf=rec, x=x, x_scale=xsc)
    # ALL 524288 records and all their de-quantized rows against the oracle, 65536 records at a time: the oracle
    # quantizes the routed rows themselves (gathered on the host) and de-quantizes its own result
    for lo in range(0, Mo, 65536):
        sl = slice(lo, lo + 65536)
        src = idx_h[sl]
        wq, wsf = par.quant(xs_h[src], s_h[src])
        got = host(recs[sl])
        assert_same(got[:, : K // 2], wq, f"cfg5 record nibbles, records {lo}..")
        assert_same(got[:, K // 2:], wsf, f"cfg5 record scales, records {lo}..")
        wx, wxs = par.dequant(wq, wsf)
        assert_same(host(xsc[sl]), wxs, f"cfg5 de-quantized tile scales, records {lo}..")
        assert_same(host(x[sl]), wx, f"cfg5 de-quantized bytes, records {lo}..")
        print(f"cfg5: records {lo}..{lo + 65535} equal the oracle", flush=True)
    del wq, wsf, wx, wxs, got
    # sizes: the closed-form payloads
    assert buf.numel() == synth.payload_bytes(Mo, K)["mxfp4"]
    assert x.numel() + 4 * xsc.numel() == synth.payload_bytes(Mo, K)["fp8"]


def test_ragged_32_experts_without_padding_65536x7168(target):
    """The un-padded 32-expert split bench.py times (Zipf counts, any T_e): the three transposing
    entry points against the oracle, expert by expert, with guard bytes around every output."""
    from concurrent.futures import ThreadPoolExecutor
    K = 7168
    off, _ = synth.expert_offsets(seed=0, num_experts=32, total_tokens=65536 - 32 * 128, pad_to=1)
    Mr = int(off[-1])
    T = np.diff(off.numpy().astype(np.int64))
    assert (T % 32 != 0).any() and (T % 2 != 0).any()
    q, sf = target["q"][:Mr], target["sf"][:Mr]
    qh, sfh = host(q), host(sf)
    offd = off.to(DEV)
    guard = 4096

    def guarded(n, dtype, fill):
        buf = torch.full((guard + n + guard,), fill, dtype=dtype, device=DEV)
        return buf, buf[guard:guard + n]

    def unguard(buf, n, fill, what):
        b = host(buf)
        assert (b[:guard] == fill).all() and (b[guard + n:] == fill).all(), f"{what}: written outside the output"
        return b[guard:guard + n]

    def per_expert(fn):
        """fn on each expert's slice as a one-expert split, experts over the host threads."""
        def one(e):
            lo, hi = int(off[e]), int(off[e + 1])
            return fn(qh[lo:hi], sfh[lo:hi], np.array([0, hi - lo], np.int32))
        with ThreadPoolExecutor(16) as pool:
            parts = list(pool.map(one, range(32)))
        return np.concatenate([p[0] for p in parts]), np.concatenate([p[1] for p in parts])

    wqc, wsc = per_expert(ref.row_to_col_grouped)
    qbuf, qv = guarded(wqc.size, torch.uint8, 0xA5)
    sbuf, sv = guarded(wsc.size, torch.uint8, 0x5A)
    mx.mxfp4_row_to_col_grouped(q, sf, offd, q_col=qv, sf_col=sv, offsets_host=off)
    assert_same(unguard(sbuf, wsc.size, 0x5A, "sf_col"), wsc, "ragged row->col scale bytes")
    assert_same(unguard(qbuf, wqc.size, 0xA5, "q_col"), wqc, "ragged row->col nibbles")
    del qbuf, sbuf, wqc, wsc

    for requant in (False, True):
        wx, wxs = per_expert(lambda a, b, o: ref.row_to_fp8_col_grouped(a, b, o, requant=requant))
        xbuf, xv = guarded(wx.size, torch.uint8, 0xA5)
        fbuf, fv = guarded(wxs.size, torch.float32, -7.0)
        mx.mxfp4_row_to_fp8_col_grouped(q, sf, offd, x_col=xv, x_col_scale=fv, requant=requant, offsets_host=off)
        assert_same(unguard(fbuf, wxs.size, -7.0, "x_col_scale"), wxs, f"ragged FP8 column scales, requant={requant}")
        assert_same(unguard(xbuf, wx.size, 0xA5, "x_col"), wx, f"ragged FP8 column bytes, requant={requant}")
        del xbuf, fbuf, wx, wxs


def test_large_grids_with_inputs_on_4_byte_boundaries():
    """[16384, 8192] is 2048 tiles, where full tiles fetch their nibbles with 16-byte loads; an input that only
    has the 4-byte alignment the entry points ask for must take the dword loads instead, with the same result."""
    M, K = 16384, 8192
    q, sf = synth.random_mxfp4(M, K, seed=21, scale_center=120, scale_spread=7, nan_scale_frac=0.0005)
    qh, sfh = q.numpy(), sf.numpy()
    buf = torch.empty(M * K // 2 + 16, dtype=torch.uint8, device=DEV)
    for shift in (0, 4):
        qd = buf[shift:shift + M * K // 2].view(M, K // 2)
        qd.copy_(q.to(DEV))
        assert qd.data_ptr() % 16 == shift
        sfd = sf.to(DEV)
        qc, sc = mx.mxfp4_row_to_col(qd, sfd)
        wqc, wsc = par.row_to_col(qh, sfh)
        assert_same(host(sc), wsc, f"column scale bytes, input at +{shift}")
        assert_same(host(qc), wqc, f"column nibbles, input at +{shift}")
        for requant in (False, True):
            x, xs = mx.mxfp4_row_to_fp8_col(qd, sfd, requant=requant)
            wx, wxs = par.row_to_fp8_col(qh, sfh, requant=requant)
            assert_same(host(xs), wxs, f"FP8 column scales, input at +{shift}, requant={requant}")
            assert_same(host(x), wx, f"FP8 column bytes, input at +{shift}, requant={requant}")


@pytest.mark.parametrize("M,K", [(32768, 4224), (32768, 4352), (32768, 4480), (24576 + 64, 5760)])
def test_large_grids_with_odd_numbers_of_column_tiles(M, K):
    """Grids of more than 2048 tiles (the launch form with 16-byte loads) whose K leaves an odd number of
    256-column tiles, a 128-column tile at the end, or both, the last with a row count that is not a multiple
    of the tile; scale bytes that force the integer path and NaN scales are strewn in.  Dense, and the same rows
    as 24 experts of unequal length."""
    q, sf = synth.random_mxfp4(M, K, seed=M + K, scale_center=118, scale_spread=9, nan_scale_frac=0.0003)
    sf[5::997, 3::7] = 254
    sf[11::1499, K // 32 - 1] = 253
    sfd, qd = sf.to(DEV), q.to(DEV)
    qc, sc = mx.mxfp4_row_to_col(qd, sfd)
    wqc, wsc = par.row_to_col(q.numpy(), sf.numpy())
    assert_same(host(sc), wsc, f"column scale bytes [{M},{K}]")
    assert_same(host(qc), wqc, f"column nibbles [{M},{K}]")
    # the same rows as 24 experts of unequal length (each a multiple of 32 rows)
    cuts = np.sort(np.random.default_rng(K).choice(np.arange(1, M // 32), 23, replace=False)) * 32
    off = np.concatenate([[0], cuts, [M]]).astype(np.int32)
    gq, gs = mx.mxfp4_row_to_col_grouped(qd, sfd, torch.from_numpy(off).to(DEV), offsets_host=off)
    gq, gs = host(gq), host(gs)
    for e in range(24):  # whole 32-row blocks per expert: its matrix is its columns of the flat result
        lo, hi = int(off[e]), int(off[e + 1])
        assert_same(gs[K * lo // 32: K * hi // 32].reshape(K, (hi - lo) // 32), wsc[:, lo // 32: hi // 32],
                    f"expert {e} column scale bytes [{M},{K}]")
        assert_same(gq[K * lo // 2: K * hi // 2].reshape(K, (hi - lo) // 2), wqc[:, lo // 2: hi // 2],
                    f"expert {e} column nibbles [{M},{K}]")
