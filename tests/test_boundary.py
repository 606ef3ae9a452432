"""Host-side checks that need no GPU: the C-ABI library loads, exports every symbol the
header declares, and rejects bad arguments before anything is launched."""
import ctypes
import os
import re

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
    # empty inputs are fine and launch nothing
    assert L.mxfp4_quant_from_fp8(None, None, 0, 128, None, 0, None, 64, None, 4, None) == binding.OK
    assert L.mxfp4_dequant_to_fp8(None, 64, None, 4, 0, 128, None, None, None) == binding.OK
    assert L.mxfp4_row_to_col(None, None, 0, 128, None, None, None) == binding.OK
    assert L.mxfp4_row_to_fp8_col(None, None, 0, 128, None, None, None) == binding.OK
    assert L.mxfp4_row_to_fp8_col_grouped(a16, a16, a16, 1025, 128, 128, a16, a16, None) == binding.ERR_OFFSETS


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
