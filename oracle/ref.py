"""ctypes front end of the CPU oracle (oracle/mxfp4_ref.c).  numpy arrays in and out.

TEST INFRASTRUCTURE: only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline
leg may import this module.  It holds no arithmetic of its own; every value comes from
the C file.  It imports nothing from the GPU package.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_LIB = None

_u8p = ctypes.POINTER(ctypes.c_uint8)
_f32p = ctypes.POINTER(ctypes.c_float)
_i32p = ctypes.POINTER(ctypes.c_int32)
_i64 = ctypes.c_int64


def lib():
    global _LIB
    if _LIB is None:
        path = _build.LIB
        if not os.path.exists(path):
            _build.build(force=True)
        L = ctypes.CDLL(path)
        L.mxfp4_ref_quant_from_fp8.argtypes = [_u8p, _f32p, _i64, _i64, _i32p, _i64, _u8p, _i64, _u8p, _i64]
        L.mxfp4_ref_quant_from_fp8_scatter.argtypes = [_u8p, _f32p, _i64, _i64, _i32p, ctypes.c_int32, _i64, _u8p, _i64, _u8p, _i64]
        L.mxfp4_ref_quant_from_fp8_scatter.restype = ctypes.c_int
        L.mxfp4_ref_quant_from_bf16.argtypes = [ctypes.POINTER(ctypes.c_uint16), _i64, _i64, _u8p, _i64, _u8p, _i64]
        L.mxfp4_ref_quant_from_bf16.restype = ctypes.c_int
        L.mxfp4_ref_dequant_to_fp8.argtypes = [_u8p, _i64, _u8p, _i64, _i64, _i64, _u8p, _f32p]
        L.mxfp4_ref_row_to_col.argtypes = [_u8p, _u8p, _i64, _i64, _u8p, _u8p]
        L.mxfp4_ref_quant_from_fp8_grouped.argtypes = [_u8p, _f32p, _i32p, ctypes.c_int32, _i64, _i64, _u8p, _u8p]
        L.mxfp4_ref_row_to_col_grouped.argtypes = [_u8p, _u8p, _i32p, ctypes.c_int32, _i64, _i64, _u8p, _u8p]
        L.mxfp4_ref_row_to_fp8_col.argtypes = [_u8p, _u8p, _i64, _i64, _u8p, _f32p]
        L.mxfp4_ref_row_to_fp8_col_grouped.argtypes = [_u8p, _u8p, _i32p, ctypes.c_int32, _i64, _i64, _u8p, _f32p]
        L.mxfp4_ref_row_to_fp8_col.restype = ctypes.c_int
        L.mxfp4_ref_row_to_fp8_col_requant.argtypes = L.mxfp4_ref_row_to_fp8_col.argtypes
        L.mxfp4_ref_row_to_fp8_col_requant_grouped.argtypes = L.mxfp4_ref_row_to_fp8_col_grouped.argtypes
        L.mxfp4_ref_row_to_fp8_col_requant.restype = ctypes.c_int
        L.mxfp4_ref_row_to_fp8_col_requant_grouped.restype = ctypes.c_int
        L.mxfp4_ref_row_to_fp8_col_grouped.restype = ctypes.c_int
        for f in (L.mxfp4_ref_quant_from_fp8, L.mxfp4_ref_dequant_to_fp8, L.mxfp4_ref_row_to_col,
                  L.mxfp4_ref_quant_from_fp8_grouped, L.mxfp4_ref_row_to_col_grouped):
            f.restype = ctypes.c_int
        L.mxfp4_ref_e4m3_value.argtypes = [ctypes.c_uint]
        L.mxfp4_ref_e4m3_value.restype = ctypes.c_double
        L.mxfp4_ref_e2m1_value.argtypes = [ctypes.c_uint]
        L.mxfp4_ref_e2m1_value.restype = ctypes.c_double
        L.mxfp4_ref_e2m1_round.argtypes = [ctypes.c_double]
        L.mxfp4_ref_e2m1_round.restype = ctypes.c_uint
        L.mxfp4_ref_e4m3_round.argtypes = [ctypes.c_double]
        L.mxfp4_ref_e4m3_round.restype = ctypes.c_uint
        L.mxfp4_ref_scale_byte.argtypes = [ctypes.c_double]
        L.mxfp4_ref_scale_byte.restype = ctypes.c_int
        _LIB = L
    return _LIB


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def _p(a, ptype):
    return a.ctypes.data_as(ptype)


def _check(rc, name):
    if rc != 0:
        raise ValueError(f"{name}: argument error ({rc})")


def quant_from_fp8(x, x_scale, gather_idx=None):
    """x uint8 [M,K] (E4M3 bytes), x_scale float32 [M,K/128] -> (q [Mo,K/2], sf [Mo,K/32])."""
    x = _c(x, np.uint8)
    x_scale = _c(x_scale, np.float32)
    M, K = x.shape
    if gather_idx is None:
        Mo, gp = M, None
    else:
        gather_idx = _c(gather_idx, np.int32)
        Mo, gp = gather_idx.shape[0], _p(gather_idx, _i32p)
    q = np.empty((Mo, K // 2), np.uint8)
    sf = np.empty((Mo, K // 32), np.uint8)
    rc = lib().mxfp4_ref_quant_from_fp8(_p(x, _u8p), _p(x_scale, _f32p), M, K, gp, Mo,
                                        _p(q, _u8p), K // 2, _p(sf, _u8p), K // 32)
    _check(rc, "quant_from_fp8")
    return q, sf


def quant_from_fp8_scatter(x, x_scale, dst_idx, M_out, q=None, sf=None):
    """Source row i -> output rows dst_idx[i, :] (entries outside [0, M_out) skipped).  q/sf: existing
    [M_out,K/2] / [M_out,K/32] arrays to write into (rows not named keep their contents), else zeros."""
    x = _c(x, np.uint8)
    x_scale = _c(x_scale, np.float32)
    dst_idx = _c(dst_idx, np.int32)
    M, K = x.shape
    q = np.zeros((M_out, K // 2), np.uint8) if q is None else q
    sf = np.zeros((M_out, K // 32), np.uint8) if sf is None else sf
    rc = lib().mxfp4_ref_quant_from_fp8_scatter(_p(x, _u8p), _p(x_scale, _f32p), M, K, _p(dst_idx, _i32p),
                                                dst_idx.shape[1], M_out, _p(q, _u8p), K // 2, _p(sf, _u8p), K // 32)
    _check(rc, "quant_from_fp8_scatter")
    return q, sf


def quant_from_bf16(x):
    """x uint16 [M,K] (BF16 bit patterns) -> (q [M,K/2], sf [M,K/32])."""
    x = _c(x, np.uint16)
    M, K = x.shape
    q = np.empty((M, K // 2), np.uint8)
    sf = np.empty((M, K // 32), np.uint8)
    rc = lib().mxfp4_ref_quant_from_bf16(_p(x, ctypes.POINTER(ctypes.c_uint16)), M, K,
                                         _p(q, _u8p), K // 2, _p(sf, _u8p), K // 32)
    _check(rc, "quant_from_bf16")
    return q, sf


def dequant_to_fp8(q, sf):
    """q uint8 [M,K/2], sf uint8 [M,K/32] -> (x uint8 [M,K], x_scale float32 [M,K/128])."""
    q = _c(q, np.uint8)
    sf = _c(sf, np.uint8)
    M, K = q.shape[0], q.shape[1] * 2
    x = np.empty((M, K), np.uint8)
    xs = np.empty((M, K // 128), np.float32)
    rc = lib().mxfp4_ref_dequant_to_fp8(_p(q, _u8p), K // 2, _p(sf, _u8p), K // 32, M, K,
                                        _p(x, _u8p), _p(xs, _f32p))
    _check(rc, "dequant_to_fp8")
    return x, xs


def row_to_col(q_row, sf_row):
    """[M,K/2] + [M,K/32] -> column-blocked, stored transposed: ([K,M/2], [K,M/32])."""
    q_row = _c(q_row, np.uint8)
    sf_row = _c(sf_row, np.uint8)
    M, K = q_row.shape[0], q_row.shape[1] * 2
    qc = np.empty((K, M // 2), np.uint8)
    sc = np.empty((K, M // 32), np.uint8)
    rc = lib().mxfp4_ref_row_to_col(_p(q_row, _u8p), _p(sf_row, _u8p), M, K, _p(qc, _u8p), _p(sc, _u8p))
    _check(rc, "row_to_col")
    return qc, sc


def row_to_fp8_col(q_row, sf_row, requant=False):
    """[M,K/2] + [M,K/32] -> the transposed matrix as FP8: (E4M3 [K,M], float32 [K,M/128]).
    requant=False: Algorithm 1's scale alignment along m; True: re-quantization from the group maximum."""
    q_row = _c(q_row, np.uint8)
    sf_row = _c(sf_row, np.uint8)
    M, K = q_row.shape[0], q_row.shape[1] * 2
    xc = np.empty((K, M), np.uint8)
    xs = np.empty((K, M // 128), np.float32)
    fn = lib().mxfp4_ref_row_to_fp8_col_requant if requant else lib().mxfp4_ref_row_to_fp8_col
    rc = fn(_p(q_row, _u8p), _p(sf_row, _u8p), M, K, _p(xc, _u8p), _p(xs, _f32p))
    _check(rc, "row_to_fp8_col")
    return xc, xs


def row_to_fp8_col_grouped(q_row, sf_row, expert_offsets, requant=False):
    """Flat buffers: expert e's [K,T_e] at K*off_e, its float32 [K,ceil(T_e/128)] at K*sum_{j<e} ceil(T_j/128).
    Any T_e >= 0 (ragged splits without padding)."""
    q_row = _c(q_row, np.uint8)
    sf_row = _c(sf_row, np.uint8)
    off = _c(expert_offsets, np.int32)
    M, K = q_row.shape[0], q_row.shape[1] * 2
    groups = int(((np.diff(off.astype(np.int64)) + 127) // 128).sum())
    xc = np.empty(M * K, np.uint8)
    xs = np.empty(groups * K, np.float32)
    fn = lib().mxfp4_ref_row_to_fp8_col_requant_grouped if requant else lib().mxfp4_ref_row_to_fp8_col_grouped
    rc = fn(_p(q_row, _u8p), _p(sf_row, _u8p), _p(off, _i32p), off.shape[0] - 1, M, K, _p(xc, _u8p), _p(xs, _f32p))
    _check(rc, "row_to_fp8_col_grouped")
    return xc, xs


def quant_from_fp8_grouped(x, x_scale, expert_offsets):
    x = _c(x, np.uint8)
    x_scale = _c(x_scale, np.float32)
    off = _c(expert_offsets, np.int32)
    M, K = x.shape
    q = np.empty((M, K // 2), np.uint8)
    sf = np.empty((M, K // 32), np.uint8)
    rc = lib().mxfp4_ref_quant_from_fp8_grouped(_p(x, _u8p), _p(x_scale, _f32p), _p(off, _i32p),
                                                off.shape[0] - 1, M, K, _p(q, _u8p), _p(sf, _u8p))
    _check(rc, "quant_from_fp8_grouped")
    return q, sf


def row_to_col_grouped(q_row, sf_row, expert_offsets):
    """Flat byte buffers: expert e's [K,ceil(T_e/2)] at K*sum_{j<e} ceil(T_j/2), its [K,ceil(T_e/32)] at
    K*sum_{j<e} ceil(T_j/32) (K*off_e/2 and K*off_e/32 for multiples of 32).  Any T_e >= 0."""
    q_row = _c(q_row, np.uint8)
    sf_row = _c(sf_row, np.uint8)
    off = _c(expert_offsets, np.int32)
    M, K = q_row.shape[0], q_row.shape[1] * 2
    T = np.diff(off.astype(np.int64))
    qc = np.empty(int(((T + 1) // 2).sum()) * K, np.uint8)
    sc = np.empty(int(((T + 31) // 32).sum()) * K, np.uint8)
    rc = lib().mxfp4_ref_row_to_col_grouped(_p(q_row, _u8p), _p(sf_row, _u8p), _p(off, _i32p),
                                            off.shape[0] - 1, M, K, _p(qc, _u8p), _p(sc, _u8p))
    _check(rc, "row_to_col_grouped")
    return qc, sc


def e4m3_value(byte):
    return lib().mxfp4_ref_e4m3_value(int(byte))


def e2m1_value(nibble):
    return lib().mxfp4_ref_e2m1_value(int(nibble))


def e2m1_round(y):
    return lib().mxfp4_ref_e2m1_round(float(y))


def e4m3_round(r):
    return lib().mxfp4_ref_e4m3_round(float(r))


def scale_byte(gmax):
    return lib().mxfp4_ref_scale_byte(float(gmax))
