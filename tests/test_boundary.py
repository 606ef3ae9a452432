"""Host-side checks that need no GPU: the C-ABI library loads, exports every symbol the
header declares, and rejects bad arguments before anything is launched."""
import ctypes
import os
import re

import pytest
import torch

import paper_2603_02731_amd as mx
from paper_2603_02731_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "mxfp4.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mxfp4_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert set(names) == set(binding.EXPORTS)
    L = mx.lib()
    for n in names:
        assert getattr(L, n) is not None


def test_status_strings():
    for st in range(-5, 1):
        assert mx.status_string(st) and mx.status_string(st) != "unknown status"
    assert mx.status_string(-99) == "unknown status"


def test_argument_validation_without_a_gpu():
    L = mx.lib()
    a16 = ctypes.c_void_p(0x1000)          # never dereferenced: validation fails first
    odd = ctypes.c_void_p(0x1001)
    # shape errors
    assert L.mxfp4_quant_from_fp8(a16, a16, 4, 100, None, 4, a16, 50, a16, 3, None) == binding.ERR_SHAPE
    assert L.mxfp4_quant_from_fp8(a16, a16, 4, 128, None, 5, a16, 64, a16, 4, None) == binding.ERR_SHAPE
    assert L.mxfp4_quant_from_fp8(a16, a16, 4, 128, None, 4, a16, 63, a16, 4, None) == binding.ERR_SHAPE
    assert L.mxfp4_quant_from_fp8(a16, a16, -1, 128, None, -1, a16, 64, a16, 4, None) == binding.ERR_SHAPE
    assert L.mxfp4_dequant_to_fp8(a16, 64, a16, 4, 4, 130, a16, a16, None) == binding.ERR_SHAPE
    assert L.mxfp4_row_to_col(a16, a16, 48, 128, a16, a16, None) == binding.ERR_SHAPE
    assert L.mxfp4_row_to_fp8_col(a16, a16, 96, 128, a16, a16, None) == binding.ERR_SHAPE
    assert L.mxfp4_row_to_fp8_col(a16, a16, 128, 1 << 25, a16, a16, None) == binding.ERR_SHAPE
    assert L.mxfp4_row_to_fp8_col_requant(a16, a16, 96, 128, a16, a16, None) == binding.ERR_SHAPE
    assert L.mxfp4_row_to_fp8_col_requant_grouped(a16, a16, a16, 0, 128, 128, a16, a16, None) == binding.ERR_OFFSETS
    assert L.mxfp4_row_to_fp8_col_requant(None, None, 0, 128, None, None, None) == binding.OK
    assert L.mxfp4_row_to_fp8_col(a16, a16, (1 << 24) + 128, 128, a16, a16, None) == binding.ERR_SHAPE
    assert L.mxfp4_quant_from_fp8_scatter(a16, a16, 4, 128, a16, 0, 4, a16, 64, a16, 4, None) == binding.ERR_SHAPE
    assert L.mxfp4_quant_from_fp8_scatter(a16, a16, 4, 128, None, 2, 8, a16, 64, a16, 4, None) == binding.ERR_NULL
    assert L.mxfp4_quant_from_fp8_scatter(a16, a16, 0, 128, None, 2, 8, None, 64, None, 4, None) == binding.OK
    # null pointers
    assert L.mxfp4_quant_from_fp8(None, a16, 4, 128, None, 4, a16, 64, a16, 4, None) == binding.ERR_NULL
    assert L.mxfp4_dequant_to_fp8(a16, 64, None, 4, 4, 128, a16, a16, None) == binding.ERR_NULL
    assert L.mxfp4_row_to_col(a16, a16, 32, 128, None, a16, None) == binding.ERR_NULL
    assert L.mxfp4_row_to_col_grouped(a16, a16, None, 2, 32, 128, a16, a16, None) == binding.ERR_NULL
    assert L.mxfp4_row_to_fp8_col(a16, None, 128, 128, a16, a16, None) == binding.ERR_NULL
    assert L.mxfp4_row_to_fp8_col_grouped(a16, a16, None, 2, 128, 128, a16, a16, None) == binding.ERR_NULL
    # alignment
    assert L.mxfp4_quant_from_fp8(odd, a16, 4, 128, None, 4, a16, 64, a16, 4, None) == binding.ERR_ALIGN
    assert L.mxfp4_quant_from_fp8(a16, a16, 4, 128, None, 4, a16, 68, a16, 4, None) == binding.ERR_ALIGN
    assert L.mxfp4_dequant_to_fp8(a16, 72, a16, 4, 4, 128, a16, a16, None) == binding.ERR_ALIGN
    assert L.mxfp4_row_to_col(a16, a16, 32, 128, odd, a16, None) == binding.ERR_ALIGN
    assert L.mxfp4_row_to_fp8_col(a16, a16, 128, 128, odd, a16, None) == binding.ERR_ALIGN
    assert L.mxfp4_row_to_fp8_col(a16, a16, 128, 128, a16, odd, None) == binding.ERR_ALIGN
    # expert count
    assert L.mxfp4_row_to_col_grouped(a16, a16, a16, 0, 32, 128, a16, a16, None) == binding.ERR_OFFSETS
    assert L.mxfp4_quant_from_fp8_grouped(a16, a16, a16, 5000, 32, 128, a16, a16, None) == binding.ERR_OFFSETS
    assert L.mxfp4_quant_from_fp8_grouped(a16, a16, odd, 2, 32, 128, a16, a16, None) == binding.ERR_ALIGN
    assert L.mxfp4_row_to_col_grouped(a16, a16, odd, 2, 32, 128, a16, a16, None) == binding.ERR_ALIGN
    # empty inputs are fine and launch nothing
    assert L.mxfp4_quant_from_fp8(None, None, 0, 128, None, 0, None, 64, None, 4, None) == binding.OK
    assert L.mxfp4_dequant_to_fp8(None, 64, None, 4, 0, 128, None, None, None) == binding.OK
    assert L.mxfp4_row_to_col(None, None, 0, 128, None, None, None) == binding.OK
    assert L.mxfp4_row_to_fp8_col(None, None, 0, 128, None, None, None) == binding.OK
    assert L.mxfp4_row_to_fp8_col_grouped(a16, a16, a16, 1025, 128, 128, a16, a16, None) == binding.ERR_OFFSETS


class _NoLaunch:
    """Stands in for the loaded library: any entry point reached through it fails the test."""
    def __getattr__(self, name):
        raise AssertionError(f"{name} was reached with arguments the binding had to reject")


@pytest.fixture
def no_launch(monkeypatch):
    monkeypatch.setattr(binding, "lib", lambda: _NoLaunch())


def _t(shape, dtype=torch.uint8, device="cpu"):
    return torch.zeros(shape, dtype=dtype, device=device)


def test_binding_rejects_host_tensors_before_any_launch(no_launch):
    """A tensor in host memory must never have its address handed to a kernel: every wrapper raises TypeError
    on well-shaped CPU tensors, inputs and caller-supplied outputs alike."""
    M, K = 128, 256
    x, s = _t((M, K)), _t((M, K // 128), torch.float32)
    q, sf = _t((M, K // 2)), _t((M, K // 32))
    off = torch.tensor([0, 64, 128], dtype=torch.int32)
    calls = [
        lambda: mx.mxfp4_quant_from_fp8(x, s),
        lambda: mx.mxfp4_quant_from_fp8(x, s, gather_idx=torch.zeros(4, dtype=torch.int32)),
        lambda: mx.mxfp4_quant_from_fp8_scatter(x, s, torch.zeros((M, 2), dtype=torch.int32), 2 * M),
        lambda: mx.mxfp4_quant_from_bf16(_t((M, K), torch.bfloat16)),
        lambda: mx.mxfp4_dequant_to_fp8(q, sf),
        lambda: mx.mxfp4_dequant_to_fp8(q.view(-1), sf.view(-1), M=M, K=K, ld_q=K // 2, ld_sf=K // 32),
        lambda: mx.mxfp4_row_to_col(q, sf),
        lambda: mx.mxfp4_quant_from_fp8_grouped(x, s, off),
        lambda: mx.mxfp4_row_to_col_grouped(q, sf, off),
        lambda: mx.mxfp4_row_to_fp8_col(q, sf),
        lambda: mx.mxfp4_row_to_fp8_col(q, sf, requant=True),
        lambda: mx.mxfp4_row_to_fp8_col_grouped(q, sf, off),
    ]
    for i, call in enumerate(calls):
        with pytest.raises(TypeError, match="HIP device tensor"):
            call()
    with pytest.raises(TypeError):
        mx.mxfp4_row_to_col(q.numpy(), sf)


def test_binding_rejects_wrong_dtypes_shapes_and_short_buffers(no_launch):
    """dtype, contiguity, exact scale shapes and the extent of every caller-supplied output are checked before
    the device is, so the checks themselves are exercised without a GPU; nothing reaches the library."""
    M, K = 128, 256
    x, s = _t((M, K)), _t((M, K // 128), torch.float32)
    q, sf = _t((M, K // 2)), _t((M, K // 32))
    off = torch.tensor([0, 60, 128], dtype=torch.int32)
    rec = K // 2 + K // 32
    bad = [
        (TypeError, lambda: mx.mxfp4_quant_from_fp8(x.to(torch.int8), s)),
        (TypeError, lambda: mx.mxfp4_quant_from_fp8(x, s.double())),
        (ValueError, lambda: mx.mxfp4_quant_from_fp8(x, s[:, :1])),                      # scale not contiguous
        (ValueError, lambda: mx.mxfp4_quant_from_fp8(x, _t((M, 1), torch.float32))),     # wrong scale shape
        (ValueError, lambda: mx.mxfp4_quant_from_fp8(x, _t((M - 1, 2), torch.float32))),
        (ValueError, lambda: mx.mxfp4_quant_from_fp8(_t((M, 100)), s)),                  # K % 128
        (ValueError, lambda: mx.mxfp4_quant_from_fp8(x.view(-1), s)),                    # not 2-D
        (TypeError, lambda: mx.mxfp4_quant_from_fp8(x, s, gather_idx=torch.zeros(4, dtype=torch.int64))),
        (ValueError, lambda: mx.mxfp4_quant_from_fp8(x, s, q=_t((M, K // 2 - 1)))),      # short output
        (ValueError, lambda: mx.mxfp4_quant_from_fp8(x, s, sf=_t((M - 1, K // 32)))),
        (TypeError, lambda: mx.mxfp4_quant_from_fp8(x, s, q=_t((M, K // 2), torch.int8))),
        (ValueError, lambda: mx.mxfp4_quant_from_fp8(x, s, q=_t((M, K))[:, :K // 2])),   # strided output view
        # per-token records: the views must reach the end of the last record
        (ValueError, lambda: mx.mxfp4_quant_from_fp8(x, s, q=_t(M * rec - K // 32 - 1), sf=_t(M * rec)[K // 2:], ld_q=rec,
                                                     ld_sf=rec)),
        (ValueError, lambda: mx.mxfp4_quant_from_fp8(x, s, q=_t(M * rec), sf=_t(M * rec)[K // 2 + 1:], ld_q=rec,
                                                     ld_sf=rec)),
        (ValueError, lambda: mx.mxfp4_quant_from_fp8(x, s, q=_t(M * rec), sf=_t(M * rec), ld_q=K // 2 - 8, ld_sf=rec)),
        (ValueError, lambda: mx.mxfp4_quant_from_fp8(x, s, ld_q=rec)),                   # stride without a buffer
        (ValueError, lambda: mx.mxfp4_quant_from_fp8(x, s, gather_idx=torch.zeros(2 * M, dtype=torch.int32), q=q)),
        (ValueError, lambda: mx.mxfp4_quant_from_fp8_scatter(x, s, torch.zeros((M - 1, 2), dtype=torch.int32), M)),
        (ValueError, lambda: mx.mxfp4_quant_from_fp8_scatter(x, s, torch.zeros(2 * M, dtype=torch.int32), M)),
        (ValueError, lambda: mx.mxfp4_quant_from_fp8_scatter(x, s, torch.zeros((M, 2), dtype=torch.int32), 2 * M, q=q)),
        (TypeError, lambda: mx.mxfp4_quant_from_bf16(_t((M, K), torch.float16))),
        (ValueError, lambda: mx.mxfp4_quant_from_bf16(_t((M, K), torch.bfloat16), sf=_t((M, K // 32 - 1)))),
        (TypeError, lambda: mx.mxfp4_dequant_to_fp8(q.to(torch.int8), sf)),
        (ValueError, lambda: mx.mxfp4_dequant_to_fp8(q, _t((M, K // 32 + 1)))),
        (ValueError, lambda: mx.mxfp4_dequant_to_fp8(q, sf, x=_t((M, K - 1)))),
        (ValueError, lambda: mx.mxfp4_dequant_to_fp8(q, sf, x_scale=_t((M, K // 128 - 1), torch.float32))),
        (TypeError, lambda: mx.mxfp4_dequant_to_fp8(q, sf, x_scale=_t((M, K // 128), torch.float64))),
        (ValueError, lambda: mx.mxfp4_dequant_to_fp8(q, sf, M=M)),
        (ValueError, lambda: mx.mxfp4_dequant_to_fp8(_t(M * rec - K // 32 - 1), _t(M * rec)[K // 2:], M=M, K=K, ld_q=rec, ld_sf=rec)),
        (ValueError, lambda: mx.mxfp4_dequant_to_fp8(_t(M * rec), _t(M * rec)[K // 2:], M=M + 1, K=K, ld_q=rec, ld_sf=rec)),
        (ValueError, lambda: mx.mxfp4_dequant_to_fp8(_t(M * rec), _t(M * rec)[K // 2:], M=M, K=K + 1, ld_q=rec, ld_sf=rec)),
        (ValueError, lambda: mx.mxfp4_row_to_col(q, _t((M, K // 32 - 1)))),
        (ValueError, lambda: mx.mxfp4_row_to_col(q[:48], sf[:48])),                      # M % 32
        (ValueError, lambda: mx.mxfp4_row_to_col(q, sf, q_col=_t((K, M // 2 - 1)))),
        (ValueError, lambda: mx.mxfp4_row_to_col(q, sf, sf_col=_t((K, M // 32 - 1)))),
        (TypeError, lambda: mx.mxfp4_row_to_col(q, sf, sf_col=_t((K, M // 32), torch.int32))),
        (ValueError, lambda: mx.mxfp4_row_to_fp8_col(q[:96], sf[:96])),                  # M % 128
        (ValueError, lambda: mx.mxfp4_row_to_fp8_col(q, sf, x_col=_t((K, M - 1)))),
        (ValueError, lambda: mx.mxfp4_row_to_fp8_col(q, sf, x_col_scale=_t(K * M // 128 - 1, torch.float32))),
        (TypeError, lambda: mx.mxfp4_row_to_fp8_col(q, sf, x_col_scale=_t(K * M // 128))),
        (TypeError, lambda: mx.mxfp4_row_to_col_grouped(q, sf, off.long())),
        (ValueError, lambda: mx.mxfp4_row_to_col_grouped(q, sf, off[:1])),
        # grouped outputs without host offsets need the documented upper bounds; exact sizes need the offsets
        (ValueError, lambda: mx.mxfp4_row_to_col_grouped(q, sf, off, q_col=_t(K * M // 2), sf_col=_t(K * (M // 32 + 2)))),
        (ValueError, lambda: mx.mxfp4_row_to_col_grouped(q, sf, off, q_col=_t(K * (M // 2 + 2)), sf_col=_t(K * M // 32))),
        (ValueError, lambda: mx.mxfp4_row_to_col_grouped(q, sf, off, q_col=_t(K * M // 2), sf_col=_t(K * 5 - 1),
                                                         offsets_host=[0, 60, 128])),   # ceil(60/32)+ceil(68/32) = 5
        (ValueError, lambda: mx.mxfp4_row_to_col_grouped(q, sf, off, offsets_host=[0, 60, 127])),
        (ValueError, lambda: mx.mxfp4_row_to_col_grouped(q, sf, off, offsets_host=[0, 130, 128])),
        (ValueError, lambda: mx.mxfp4_row_to_col_grouped(q, sf, off, offsets_host=[0, 128])),
        (ValueError, lambda: mx.mxfp4_row_to_fp8_col_grouped(q, sf, off, x_col=_t(M * K - 1))),
        (ValueError, lambda: mx.mxfp4_row_to_fp8_col_grouped(q, sf, off, x_col_scale=_t(K * 2, torch.float32))),
        (ValueError, lambda: mx.mxfp4_row_to_fp8_col_grouped(q, sf, off, x_col_scale=_t(K * 2 - 1, torch.float32),
                                                             offsets_host=[0, 60, 128])),
        (ValueError, lambda: mx.mxfp4_quant_from_fp8_grouped(x, s, off, q=_t((M, K // 2 - 1)))),
    ]
    for i, (exc, call) in enumerate(bad):
        with pytest.raises(exc):
            call()
        try:
            call()
        except (TypeError, ValueError) as e:
            assert "HIP device tensor" not in str(e), f"case {i} passed every check up to the device check: {e}"


def test_binding_accepts_exact_grouped_sizes_with_host_offsets(no_launch):
    """With the offsets also given as host integers the exact output sizes pass every size check (the call then
    stops at the device check, these being CPU tensors)."""
    M, K = 128, 256
    q, sf = _t((M, K // 2)), _t((M, K // 32))
    off = torch.tensor([0, 60, 128], dtype=torch.int32)
    with pytest.raises(TypeError, match="HIP device tensor"):
        mx.mxfp4_row_to_col_grouped(q, sf, off, q_col=_t(K * 64), sf_col=_t(K * 5), offsets_host=off)
    with pytest.raises(TypeError, match="HIP device tensor"):
        mx.mxfp4_row_to_fp8_col_grouped(q, sf, off, x_col=_t(K * M), x_col_scale=_t(K * 2, torch.float32),
                                        offsets_host=off)


def test_bench_refuses_more_than_one_gpu():
    """The build runs on one GPU: bench.py --gpus N with N > 1 exits with a message and touches no GPU."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2", "--steps", "1"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_nothing_in_the_product_path_touches_the_oracle():
    """oracle/ is test infrastructure: the package and the kernels never import, link or read it."""
    pkg = os.path.join(ROOT, "paper_2603_02731_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "mxfp4_ref" not in text, f"{f} names the oracle's library"
                assert not re.search(r"^\s*(from|import)\s+oracle\b", text, flags=re.M), f"{f} imports the oracle"
