"""ctypes binding of libmxfp4 (include/mxfp4.h): argument marshalling only.

Every step of the conversions runs in the HIP kernels of the library.  PyTorch is used for
device memory and streams, nothing else; there is no CPU or eager fallback: if the library
is missing or cannot be loaded the calls raise.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmxfp4.so")

OK, ERR_NULL, ERR_SHAPE, ERR_ALIGN, ERR_OFFSETS, ERR_LAUNCH = 0, -1, -2, -3, -4, -5

EXPORTS = ("mxfp4_quant_from_fp8", "mxfp4_quant_from_fp8_scatter", "mxfp4_quant_from_bf16", "mxfp4_dequant_to_fp8", "mxfp4_row_to_col",
           "mxfp4_quant_from_fp8_grouped", "mxfp4_row_to_col_grouped", "mxfp4_row_to_fp8_col",
           "mxfp4_row_to_fp8_col_grouped", "mxfp4_row_to_fp8_col_requant", "mxfp4_row_to_fp8_col_requant_grouped",
           "mxfp4_status_string")

_lib = None
_vp, _i64, _i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32


class Mxfp4Error(RuntimeError):
    def __init__(self, name, status, text):
        super().__init__(f"{name}: {text} (status {status})")
        self.status = status


def lib():
    """Load libmxfp4.so (built in-tree by paper_2603_02731_amd/build.py)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            from . import build as _build
            _build.build(force=True)
        L = ctypes.CDLL(LIB_PATH)  # raises OSError if it cannot be loaded: no fallback
        L.mxfp4_quant_from_fp8.argtypes = [_vp, _vp, _i64, _i64, _vp, _i64, _vp, _i64, _vp, _i64, _vp]
        L.mxfp4_quant_from_fp8_scatter.argtypes = [_vp, _vp, _i64, _i64, _vp, _i32, _i64, _vp, _i64, _vp, _i64, _vp]
        L.mxfp4_quant_from_bf16.argtypes = [_vp, _i64, _i64, _vp, _i64, _vp, _i64, _vp]
        L.mxfp4_dequant_to_fp8.argtypes = [_vp, _i64, _vp, _i64, _i64, _i64, _vp, _vp, _vp]
        L.mxfp4_row_to_col.argtypes = [_vp, _vp, _i64, _i64, _vp, _vp, _vp]
        L.mxfp4_quant_from_fp8_grouped.argtypes = [_vp, _vp, _vp, _i32, _i64, _i64, _vp, _vp, _vp]
        L.mxfp4_row_to_col_grouped.argtypes = [_vp, _vp, _vp, _i32, _i64, _i64, _vp, _vp, _vp]
        L.mxfp4_row_to_fp8_col.argtypes = [_vp, _vp, _i64, _i64, _vp, _vp, _vp]
        L.mxfp4_row_to_fp8_col_grouped.argtypes = [_vp, _vp, _vp, _i32, _i64, _i64, _vp, _vp, _vp]
        L.mxfp4_row_to_fp8_col_requant.argtypes = L.mxfp4_row_to_fp8_col.argtypes
        L.mxfp4_row_to_fp8_col_requant_grouped.argtypes = L.mxfp4_row_to_fp8_col_grouped.argtypes
        for n in EXPORTS[:-1]:
            getattr(L, n).restype = ctypes.c_int
        L.mxfp4_status_string.argtypes = [ctypes.c_int]
        L.mxfp4_status_string.restype = ctypes.c_char_p
        _lib = L
    return _lib


def status_string(status):
    return lib().mxfp4_status_string(int(status)).decode()


def _check(name, status):
    if status != OK:
        raise Mxfp4Error(name, status, status_string(status))


def _dev(t, dtype, name):
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name} must be a CUDA/HIP tensor")
    if t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return t


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream if hasattr(s, "cuda_stream") else int(s)


def mxfp4_quant_from_fp8(x, x_scale, gather_idx=None, q=None, sf=None, ld_q=None, ld_sf=None, stream=None):
    """x uint8 [M_src,K] (E4M3), x_scale float32 [M_src,K/128] -> (q uint8 [M_out,K/2], sf uint8 [M_out,K/32]).
    gather_idx: optional int32 [M_out].  q/sf may be preallocated; with ld_q/ld_sf they may be views
    into a record buffer (row strides in bytes)."""
    _dev(x, torch.uint8, "x")
    _dev(x_scale, torch.float32, "x_scale")
    M_src, K = x.shape
    if gather_idx is not None:
        _dev(gather_idx, torch.int32, "gather_idx")
        M_out = gather_idx.shape[0]
    else:
        M_out = M_src
    if q is None:
        q = torch.empty((M_out, K // 2), dtype=torch.uint8, device=x.device)
    if sf is None:
        sf = torch.empty((M_out, K // 32), dtype=torch.uint8, device=x.device)
    ld_q = K // 2 if ld_q is None else ld_q
    ld_sf = K // 32 if ld_sf is None else ld_sf
    st = lib().mxfp4_quant_from_fp8(x.data_ptr(), x_scale.data_ptr(), M_src, K,
                                    None if gather_idx is None else gather_idx.data_ptr(), M_out,
                                    q.data_ptr(), ld_q, sf.data_ptr(), ld_sf, _stream(stream))
    _check("mxfp4_quant_from_fp8", st)
    return q, sf


def mxfp4_quant_from_fp8_scatter(x, x_scale, dst_idx, M_out, q=None, sf=None, ld_q=None, ld_sf=None, stream=None):
    """Source row i of x -> output rows dst_idx[i, :] (int32 [M_src, fanout]; entries outside [0, M_out) are
    skipped).  Newly allocated q/sf are zero-filled, since rows that no entry names are not written."""
    _dev(x, torch.uint8, "x")
    _dev(x_scale, torch.float32, "x_scale")
    _dev(dst_idx, torch.int32, "dst_idx")
    M_src, K = x.shape
    if q is None:
        q = torch.zeros((M_out, K // 2), dtype=torch.uint8, device=x.device)
    if sf is None:
        sf = torch.zeros((M_out, K // 32), dtype=torch.uint8, device=x.device)
    ld_q = K // 2 if ld_q is None else ld_q
    ld_sf = K // 32 if ld_sf is None else ld_sf
    st = lib().mxfp4_quant_from_fp8_scatter(x.data_ptr(), x_scale.data_ptr(), M_src, K, dst_idx.data_ptr(),
                                            dst_idx.shape[1], M_out, q.data_ptr(), ld_q, sf.data_ptr(), ld_sf,
                                            _stream(stream))
    _check("mxfp4_quant_from_fp8_scatter", st)
    return q, sf


def mxfp4_quant_from_bf16(x, q=None, sf=None, ld_q=None, ld_sf=None, stream=None):
    """x bfloat16 [M,K] -> (q uint8 [M,K/2], sf uint8 [M,K/32])."""
    _dev(x, torch.bfloat16, "x")
    M, K = x.shape
    if q is None:
        q = torch.empty((M, K // 2), dtype=torch.uint8, device=x.device)
    if sf is None:
        sf = torch.empty((M, K // 32), dtype=torch.uint8, device=x.device)
    ld_q = K // 2 if ld_q is None else ld_q
    ld_sf = K // 32 if ld_sf is None else ld_sf
    st = lib().mxfp4_quant_from_bf16(x.data_ptr(), M, K, q.data_ptr(), ld_q, sf.data_ptr(), ld_sf, _stream(stream))
    _check("mxfp4_quant_from_bf16", st)
    return q, sf


def mxfp4_dequant_to_fp8(q, sf, M=None, K=None, ld_q=None, ld_sf=None, x=None, x_scale=None, stream=None):
    """q uint8 [M,K/2], sf uint8 [M,K/32] -> (x uint8 [M,K] E4M3, x_scale float32 [M,K/128])."""
    if M is None:
        M, K = q.shape[0], q.shape[1] * 2
    if x is None:
        x = torch.empty((M, K), dtype=torch.uint8, device=q.device)
    if x_scale is None:
        x_scale = torch.empty((M, K // 128), dtype=torch.float32, device=q.device)
    ld_q = K // 2 if ld_q is None else ld_q
    ld_sf = K // 32 if ld_sf is None else ld_sf
    st = lib().mxfp4_dequant_to_fp8(q.data_ptr(), ld_q, sf.data_ptr(), ld_sf, M, K,
                                    x.data_ptr(), x_scale.data_ptr(), _stream(stream))
    _check("mxfp4_dequant_to_fp8", st)
    return x, x_scale


def mxfp4_row_to_col(q_row, sf_row, q_col=None, sf_col=None, stream=None):
    """[M,K/2] + [M,K/32] row-blocked -> column-blocked, stored transposed ([K,M/2], [K,M/32])."""
    _dev(q_row, torch.uint8, "q_row")
    _dev(sf_row, torch.uint8, "sf_row")
    M, K = q_row.shape[0], q_row.shape[1] * 2
    if q_col is None:
        q_col = torch.empty((K, M // 2), dtype=torch.uint8, device=q_row.device)
    if sf_col is None:
        sf_col = torch.empty((K, M // 32), dtype=torch.uint8, device=q_row.device)
    st = lib().mxfp4_row_to_col(q_row.data_ptr(), sf_row.data_ptr(), M, K, q_col.data_ptr(),
                                sf_col.data_ptr(), _stream(stream))
    _check("mxfp4_row_to_col", st)
    return q_col, sf_col


def mxfp4_quant_from_fp8_grouped(x, x_scale, expert_offsets, q=None, sf=None, stream=None):
    _dev(x, torch.uint8, "x")
    _dev(x_scale, torch.float32, "x_scale")
    _dev(expert_offsets, torch.int32, "expert_offsets")
    M, K = x.shape
    if q is None:
        q = torch.empty((M, K // 2), dtype=torch.uint8, device=x.device)
    if sf is None:
        sf = torch.empty((M, K // 32), dtype=torch.uint8, device=x.device)
    st = lib().mxfp4_quant_from_fp8_grouped(x.data_ptr(), x_scale.data_ptr(), expert_offsets.data_ptr(),
                                            expert_offsets.shape[0] - 1, M, K, q.data_ptr(), sf.data_ptr(),
                                            _stream(stream))
    _check("mxfp4_quant_from_fp8_grouped", st)
    return q, sf


def mxfp4_row_to_col_grouped(q_row, sf_row, expert_offsets, q_col=None, sf_col=None, stream=None):
    """Outputs are flat byte buffers: expert e's [K,ceil(T_e/2)] at K*sum_{j<e} ceil(T_j/2), its [K,ceil(T_e/32)]
    at K*sum_{j<e} ceil(T_j/32) (K*off_e/2 and K*off_e/32 for multiples of 32); any T_e.  Buffers allocated here
    have the upper-bound sizes K*(M//2 + num_experts) and K*(M//32 + num_experts)."""
    _dev(q_row, torch.uint8, "q_row")
    _dev(sf_row, torch.uint8, "sf_row")
    _dev(expert_offsets, torch.int32, "expert_offsets")
    M, K = q_row.shape[0], q_row.shape[1] * 2
    E = expert_offsets.shape[0] - 1
    if q_col is None:
        q_col = torch.empty(K * (M // 2 + E), dtype=torch.uint8, device=q_row.device)
    if sf_col is None:
        sf_col = torch.empty(K * (M // 32 + E), dtype=torch.uint8, device=q_row.device)
    st = lib().mxfp4_row_to_col_grouped(q_row.data_ptr(), sf_row.data_ptr(), expert_offsets.data_ptr(),
                                        expert_offsets.shape[0] - 1, M, K, q_col.data_ptr(), sf_col.data_ptr(),
                                        _stream(stream))
    _check("mxfp4_row_to_col_grouped", st)
    return q_col, sf_col


def mxfp4_row_to_fp8_col(q_row, sf_row, x_col=None, x_col_scale=None, stream=None, requant=False):
    """[M,K/2] + [M,K/32] row-blocked MXFP4 -> the transposed matrix as FP8: (E4M3 [K,M], float32 [K,M/128]).
    requant=True calls mxfp4_row_to_fp8_col_requant (scale from the group maximum)."""
    _dev(q_row, torch.uint8, "q_row")
    _dev(sf_row, torch.uint8, "sf_row")
    M, K = q_row.shape[0], q_row.shape[1] * 2
    if x_col is None:
        x_col = torch.empty((K, M), dtype=torch.uint8, device=q_row.device)
    if x_col_scale is None:
        x_col_scale = torch.empty((K, M // 128), dtype=torch.float32, device=q_row.device)
    fn = lib().mxfp4_row_to_fp8_col_requant if requant else lib().mxfp4_row_to_fp8_col
    st = fn(q_row.data_ptr(), sf_row.data_ptr(), M, K, x_col.data_ptr(), x_col_scale.data_ptr(), _stream(stream))
    _check("mxfp4_row_to_fp8_col_requant" if requant else "mxfp4_row_to_fp8_col", st)
    return x_col, x_col_scale


def mxfp4_row_to_fp8_col_grouped(q_row, sf_row, expert_offsets, x_col=None, x_col_scale=None, stream=None,
                                 requant=False):
    """Outputs are flat buffers: expert e's [K,T_e] at K*off_e, its float32 [K,ceil(T_e/128)] at
    K*sum_{j<e} ceil(T_j/128); any T_e.  A scale buffer allocated here has the upper-bound size
    K*(M//128 + num_experts)."""
    _dev(q_row, torch.uint8, "q_row")
    _dev(sf_row, torch.uint8, "sf_row")
    _dev(expert_offsets, torch.int32, "expert_offsets")
    M, K = q_row.shape[0], q_row.shape[1] * 2
    if x_col is None:
        x_col = torch.empty(M * K, dtype=torch.uint8, device=q_row.device)
    if x_col_scale is None:
        x_col_scale = torch.empty(K * (M // 128 + expert_offsets.shape[0] - 1), dtype=torch.float32,
                                  device=q_row.device)
    fn = lib().mxfp4_row_to_fp8_col_requant_grouped if requant else lib().mxfp4_row_to_fp8_col_grouped
    st = fn(q_row.data_ptr(), sf_row.data_ptr(), expert_offsets.data_ptr(), expert_offsets.shape[0] - 1, M, K,
            x_col.data_ptr(), x_col_scale.data_ptr(), _stream(stream))
    _check("mxfp4_row_to_fp8_col_requant_grouped" if requant else "mxfp4_row_to_fp8_col_grouped", st)
    return x_col, x_col_scale
