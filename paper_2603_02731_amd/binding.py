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
           "mxfp4_stream_copy", "mxfp4_stream_mix", "mxfp4_tile_copy", "mxfp4_record_fanout", "mxfp4_status_string")

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
        L.mxfp4_stream_copy.argtypes = [_vp, _vp, _i64, _i32, _vp]
        L.mxfp4_stream_mix.argtypes = [_vp, _vp, _i64, _i32, _i32, _vp]
        L.mxfp4_tile_copy.argtypes = [_vp, _vp, _i64, _i64, _vp]
        L.mxfp4_record_fanout.argtypes = [_vp, _i64, _vp, _i64, _i32, _i64, _i64, _vp, _vp]
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


def _buf(t, dtype, name, *, shape=None, min_bytes=None):
    """Check one tensor argument before its address goes to the library: type, dtype, contiguity, exact shape
    or extent in bytes from its first element.  The C ABI sees addresses only, so nothing behind this check can
    tell a short buffer from a good one.  Where the tensor lives is checked by _on_device, after every argument of
    the call has passed here.  Raises TypeError / ValueError; nothing is launched."""
    if not isinstance(t, torch.Tensor):
        raise TypeError(f"{name} must be a torch.Tensor, got {type(t).__name__}")
    if t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} must have shape {tuple(shape)}, got {tuple(t.shape)}")
    if min_bytes is not None and t.numel() * t.element_size() < min_bytes:
        raise ValueError(f"{name} holds {t.numel() * t.element_size()} bytes, the call needs {min_bytes}")
    return t


def _on_device(**tensors):
    """Last check before a launch: every tensor of the call is a HIP device tensor, all on one device (a host
    address handed to a kernel is a GPU memory fault, not an exception).  Returns that device's index."""
    dev = -1
    for name, t in tensors.items():
        if t is None:
            continue
        if not t.is_cuda:
            raise TypeError(f"{name} must be a HIP device tensor, got one on {t.device}")
        d = t.get_device()
        if dev < 0:
            dev = d
        elif d != dev:
            raise ValueError(f"{name} is on device {d}, the other arguments on device {dev}")
    return dev


def _matrix(t, dtype, name, k_multiple):
    """A 2-D input [M, C] whose column count is a multiple of `k_multiple`; returns (M, C)."""
    if isinstance(t, torch.Tensor) and t.dim() != 2:
        raise ValueError(f"{name} must be 2-D, got {t.dim()}-D")
    _buf(t, dtype, name)
    M, C = t.shape
    if C % k_multiple != 0:
        raise ValueError(f"{name} must have a multiple of {k_multiple} columns, got {C}")
    return M, C


def _strided_out(t, name, rows, row_bytes, ld):
    """A caller's output of `rows` rows of `row_bytes` bytes, `ld` bytes apart, starting at t's first byte."""
    if ld < row_bytes:
        raise ValueError(f"row stride of {name} is {ld} bytes, a row has {row_bytes}")
    need = (rows - 1) * ld + row_bytes if rows > 0 else 0
    return _buf(t, torch.uint8, name, min_bytes=need)


# the raw handle of the current stream of a device, without building a torch.cuda.Stream object (2.7 us a call)
_raw_current_stream = getattr(torch._C, "_cuda_getCurrentRawStream", None)


def _stream(stream, dev):
    """The hipStream_t to launch on: the caller's (a torch.cuda.Stream or a raw handle), else the current stream
    of the tensors' device."""
    if stream is None:
        if _raw_current_stream is not None:
            return _raw_current_stream(dev)
        return torch.cuda.current_stream(dev).cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _quant_outputs(x, M_out, K, q, sf, ld_q, ld_sf, fill):
    ld_q = K // 2 if ld_q is None else int(ld_q)
    ld_sf = K // 32 if ld_sf is None else int(ld_sf)
    if q is None:
        if ld_q != K // 2:
            raise ValueError("ld_q needs a caller-supplied q")
        q = fill((M_out, K // 2), dtype=torch.uint8, device=x.device)
    else:
        _strided_out(q, "q", M_out, K // 2, ld_q)
    if sf is None:
        if ld_sf != K // 32:
            raise ValueError("ld_sf needs a caller-supplied sf")
        sf = fill((M_out, K // 32), dtype=torch.uint8, device=x.device)
    else:
        _strided_out(sf, "sf", M_out, K // 32, ld_sf)
    return q, sf, ld_q, ld_sf


def mxfp4_quant_from_fp8(x, x_scale, gather_idx=None, q=None, sf=None, ld_q=None, ld_sf=None, stream=None):
    """x uint8 [M_src,K] (E4M3), x_scale float32 [M_src,K/128] -> (q uint8 [M_out,K/2], sf uint8 [M_out,K/32]).
    gather_idx: optional int32 [M_out].  q/sf may be preallocated; with ld_q/ld_sf they may be views
    into a record buffer (row strides in bytes) that reach from their first byte to the end of the last row."""
    M_src, K = _matrix(x, torch.uint8, "x", 128)
    _buf(x_scale, torch.float32, "x_scale", shape=(M_src, K // 128))
    if gather_idx is not None:
        _buf(gather_idx, torch.int32, "gather_idx")
        if gather_idx.dim() != 1:
            raise ValueError("gather_idx must be 1-D")
        M_out = gather_idx.shape[0]
    else:
        M_out = M_src
    q, sf, ld_q, ld_sf = _quant_outputs(x, M_out, K, q, sf, ld_q, ld_sf, torch.empty)
    dev = _on_device(x=x, x_scale=x_scale, gather_idx=gather_idx, q=q, sf=sf)
    st = lib().mxfp4_quant_from_fp8(x.data_ptr(), x_scale.data_ptr(), M_src, K,
                                    None if gather_idx is None else gather_idx.data_ptr(), M_out,
                                    q.data_ptr(), ld_q, sf.data_ptr(), ld_sf, _stream(stream, dev))
    _check("mxfp4_quant_from_fp8", st)
    return q, sf


def mxfp4_quant_from_fp8_scatter(x, x_scale, dst_idx, M_out, q=None, sf=None, ld_q=None, ld_sf=None, stream=None):
    """Source row i of x -> output rows dst_idx[i, :] (int32 [M_src, fanout]; entries outside [0, M_out) are
    skipped).  Newly allocated q/sf are zero-filled, since rows that no entry names are not written."""
    M_src, K = _matrix(x, torch.uint8, "x", 128)
    _buf(x_scale, torch.float32, "x_scale", shape=(M_src, K // 128))
    _buf(dst_idx, torch.int32, "dst_idx")
    if dst_idx.dim() != 2 or dst_idx.shape[0] != M_src or dst_idx.shape[1] < 1:
        raise ValueError(f"dst_idx must be [M_src, fanout >= 1], got {tuple(dst_idx.shape)}")
    M_out = int(M_out)
    if M_out < 0:
        raise ValueError("M_out must not be negative")
    q, sf, ld_q, ld_sf = _quant_outputs(x, M_out, K, q, sf, ld_q, ld_sf, torch.zeros)
    dev = _on_device(x=x, x_scale=x_scale, dst_idx=dst_idx, q=q, sf=sf)
    st = lib().mxfp4_quant_from_fp8_scatter(x.data_ptr(), x_scale.data_ptr(), M_src, K, dst_idx.data_ptr(),
                                            dst_idx.shape[1], M_out, q.data_ptr(), ld_q, sf.data_ptr(), ld_sf,
                                            _stream(stream, dev))
    _check("mxfp4_quant_from_fp8_scatter", st)
    return q, sf


def mxfp4_quant_from_bf16(x, q=None, sf=None, ld_q=None, ld_sf=None, stream=None):
    """x bfloat16 [M,K] -> (q uint8 [M,K/2], sf uint8 [M,K/32])."""
    M, K = _matrix(x, torch.bfloat16, "x", 128)
    q, sf, ld_q, ld_sf = _quant_outputs(x, M, K, q, sf, ld_q, ld_sf, torch.empty)
    dev = _on_device(x=x, q=q, sf=sf)
    st = lib().mxfp4_quant_from_bf16(x.data_ptr(), M, K, q.data_ptr(), ld_q, sf.data_ptr(), ld_sf, _stream(stream, dev))
    _check("mxfp4_quant_from_bf16", st)
    return q, sf


def mxfp4_dequant_to_fp8(q, sf, M=None, K=None, ld_q=None, ld_sf=None, x=None, x_scale=None, stream=None):
    """q uint8 [M,K/2], sf uint8 [M,K/32] -> (x uint8 [M,K] E4M3, x_scale float32 [M,K/128]).
    With M, K, ld_q, ld_sf the inputs may be views into a record buffer (row strides in bytes) that reach
    from their first byte to the end of the last row."""
    if M is None or K is None:
        if M is not None or K is not None or ld_q is not None or ld_sf is not None:
            raise ValueError("M and K go together; row strides need both")
        M, C = _matrix(q, torch.uint8, "q", 64)
        K = 2 * C
        _buf(sf, torch.uint8, "sf", shape=(M, K // 32))
        ld_q, ld_sf = K // 2, K // 32
    else:
        M, K = int(M), int(K)
        if M < 0 or K < 0 or K % 128 != 0:
            raise ValueError(f"bad shape M={M}, K={K}")
        ld_q = K // 2 if ld_q is None else int(ld_q)
        ld_sf = K // 32 if ld_sf is None else int(ld_sf)
        _strided_out(q, "q", M, K // 2, ld_q)
        _strided_out(sf, "sf", M, K // 32, ld_sf)
    if x is None:
        x = torch.empty((M, K), dtype=torch.uint8, device=q.device)
    else:
        _buf(x, torch.uint8, "x", min_bytes=M * K)
    if x_scale is None:
        x_scale = torch.empty((M, K // 128), dtype=torch.float32, device=q.device)
    else:
        _buf(x_scale, torch.float32, "x_scale", min_bytes=M * (K // 128) * 4)
    dev = _on_device(q=q, sf=sf, x=x, x_scale=x_scale)
    st = lib().mxfp4_dequant_to_fp8(q.data_ptr(), ld_q, sf.data_ptr(), ld_sf, M, K,
                                    x.data_ptr(), x_scale.data_ptr(), _stream(stream, dev))
    _check("mxfp4_dequant_to_fp8", st)
    return x, x_scale


def _row_blocked(q_row, sf_row):
    M, C = _matrix(q_row, torch.uint8, "q_row", 64)
    K = 2 * C
    _buf(sf_row, torch.uint8, "sf_row", shape=(M, K // 32))
    return M, K


def _out(t, dtype, name, like, shape, min_elems=None):
    """A caller's output buffer (at least `min_elems` elements, default those of `shape`) or a new one."""
    if t is None:
        return torch.empty(shape, dtype=dtype, device=like.device)
    n = 1
    for d in (shape if isinstance(shape, tuple) else (shape,)):
        n *= d
    n = n if min_elems is None else min_elems
    return _buf(t, dtype, name, min_bytes=n * torch.empty((), dtype=dtype).element_size())


def _experts(expert_offsets, M, offsets_host, units):
    """Check the offsets array of a grouped call.  Returns (E, [sum_e ceil(T_e / u) for u in units]): exact when
    the caller also passes the offsets as host values (`offsets_host`, which are then checked: off_0 = 0,
    off_E = M, non-decreasing), otherwise the upper bounds M // u + E of the C ABI."""
    _buf(expert_offsets, torch.int32, "expert_offsets")
    if expert_offsets.dim() != 1 or expert_offsets.shape[0] < 2:
        raise ValueError("expert_offsets must be int32 [num_experts + 1] with at least one expert")
    E = expert_offsets.shape[0] - 1
    if offsets_host is None:
        return E, [M // u + E for u in units]
    off = [int(v) for v in offsets_host]
    if len(off) != E + 1 or off[0] != 0 or off[-1] != M or any(b < a for a, b in zip(off, off[1:])):
        raise ValueError("offsets_host must be the E+1 non-decreasing offsets from 0 to M_total")
    return E, [sum(-(-(b - a) // u) for a, b in zip(off, off[1:])) for u in units]


def mxfp4_row_to_col(q_row, sf_row, q_col=None, sf_col=None, stream=None):
    """[M,K/2] + [M,K/32] row-blocked -> column-blocked, stored transposed ([K,M/2], [K,M/32])."""
    M, K = _row_blocked(q_row, sf_row)
    if M % 32 != 0:
        raise ValueError(f"M must be a multiple of 32, got {M}")
    q_col = _out(q_col, torch.uint8, "q_col", q_row, (K, M // 2))
    sf_col = _out(sf_col, torch.uint8, "sf_col", q_row, (K, M // 32))
    dev = _on_device(q_row=q_row, sf_row=sf_row, q_col=q_col, sf_col=sf_col)
    st = lib().mxfp4_row_to_col(q_row.data_ptr(), sf_row.data_ptr(), M, K, q_col.data_ptr(),
                                sf_col.data_ptr(), _stream(stream, dev))
    _check("mxfp4_row_to_col", st)
    return q_col, sf_col


def mxfp4_quant_from_fp8_grouped(x, x_scale, expert_offsets, q=None, sf=None, stream=None):
    M, K = _matrix(x, torch.uint8, "x", 128)
    _buf(x_scale, torch.float32, "x_scale", shape=(M, K // 128))
    _experts(expert_offsets, M, None, ())
    q, sf, _, _ = _quant_outputs(x, M, K, q, sf, None, None, torch.empty)
    dev = _on_device(x=x, x_scale=x_scale, expert_offsets=expert_offsets, q=q, sf=sf)
    st = lib().mxfp4_quant_from_fp8_grouped(x.data_ptr(), x_scale.data_ptr(), expert_offsets.data_ptr(),
                                            expert_offsets.shape[0] - 1, M, K, q.data_ptr(), sf.data_ptr(),
                                            _stream(stream, dev))
    _check("mxfp4_quant_from_fp8_grouped", st)
    return q, sf


def mxfp4_row_to_col_grouped(q_row, sf_row, expert_offsets, q_col=None, sf_col=None, stream=None, offsets_host=None):
    """Outputs are flat byte buffers: expert e's [K,ceil(T_e/2)] at K*sum_{j<e} ceil(T_j/2), its [K,ceil(T_e/32)]
    at K*sum_{j<e} ceil(T_j/32) (K*off_e/2 and K*off_e/32 for multiples of 32); any T_e.  Buffers allocated here,
    and buffers passed without `offsets_host` (the same offsets as host integers), must have the upper-bound
    sizes K*(M//2 + num_experts) and K*(M//32 + num_experts); with `offsets_host` the exact sizes are enough."""
    M, K = _row_blocked(q_row, sf_row)
    E, (n2, n32) = _experts(expert_offsets, M, offsets_host, (2, 32))
    q_col = _out(q_col, torch.uint8, "q_col", q_row, K * n2)
    sf_col = _out(sf_col, torch.uint8, "sf_col", q_row, K * n32)
    dev = _on_device(q_row=q_row, sf_row=sf_row, expert_offsets=expert_offsets, q_col=q_col, sf_col=sf_col)
    st = lib().mxfp4_row_to_col_grouped(q_row.data_ptr(), sf_row.data_ptr(), expert_offsets.data_ptr(),
                                        E, M, K, q_col.data_ptr(), sf_col.data_ptr(), _stream(stream, dev))
    _check("mxfp4_row_to_col_grouped", st)
    return q_col, sf_col


def mxfp4_row_to_fp8_col(q_row, sf_row, x_col=None, x_col_scale=None, stream=None, requant=False):
    """[M,K/2] + [M,K/32] row-blocked MXFP4 -> the transposed matrix as FP8: (E4M3 [K,M], float32 [K,M/128]).
    requant=True calls mxfp4_row_to_fp8_col_requant (scale from the group maximum)."""
    M, K = _row_blocked(q_row, sf_row)
    if M % 128 != 0:
        raise ValueError(f"M must be a multiple of 128, got {M}")
    x_col = _out(x_col, torch.uint8, "x_col", q_row, (K, M))
    x_col_scale = _out(x_col_scale, torch.float32, "x_col_scale", q_row, (K, M // 128))
    dev = _on_device(q_row=q_row, sf_row=sf_row, x_col=x_col, x_col_scale=x_col_scale)
    fn = lib().mxfp4_row_to_fp8_col_requant if requant else lib().mxfp4_row_to_fp8_col
    st = fn(q_row.data_ptr(), sf_row.data_ptr(), M, K, x_col.data_ptr(), x_col_scale.data_ptr(), _stream(stream, dev))
    _check("mxfp4_row_to_fp8_col_requant" if requant else "mxfp4_row_to_fp8_col", st)
    return x_col, x_col_scale


def mxfp4_row_to_fp8_col_grouped(q_row, sf_row, expert_offsets, x_col=None, x_col_scale=None, stream=None,
                                 requant=False, offsets_host=None):
    """Outputs are flat buffers: expert e's [K,T_e] at K*off_e, its float32 [K,ceil(T_e/128)] at
    K*sum_{j<e} ceil(T_j/128); any T_e.  A scale buffer allocated here, or passed without `offsets_host` (the
    same offsets as host integers), must have the upper-bound size K*(M//128 + num_experts)."""
    M, K = _row_blocked(q_row, sf_row)
    E, (n128,) = _experts(expert_offsets, M, offsets_host, (128,))
    x_col = _out(x_col, torch.uint8, "x_col", q_row, M * K)
    x_col_scale = _out(x_col_scale, torch.float32, "x_col_scale", q_row, K * n128)
    dev = _on_device(q_row=q_row, sf_row=sf_row, expert_offsets=expert_offsets, x_col=x_col, x_col_scale=x_col_scale)
    fn = lib().mxfp4_row_to_fp8_col_requant_grouped if requant else lib().mxfp4_row_to_fp8_col_grouped
    st = fn(q_row.data_ptr(), sf_row.data_ptr(), expert_offsets.data_ptr(), E, M, K,
            x_col.data_ptr(), x_col_scale.data_ptr(), _stream(stream, dev))
    _check("mxfp4_row_to_fp8_col_requant_grouped" if requant else "mxfp4_row_to_fp8_col_grouped", st)
    return x_col, x_col_scale


def mxfp4_stream_copy(src, dst, policy=1, stream=None):
    """Plain 16-byte-per-lane copy of src into dst (uint8, same size, a multiple of 16 bytes): the measured
    roof of the conversion kernels.  policy bit 0 = non-temporal loads, bit 1 = non-temporal stores."""
    return mxfp4_stream_mix(src, dst, 0, policy=policy, stream=stream)


def mxfp4_stream_mix(src, dst, mix, policy=3, stream=None):
    """Byte mover without arithmetic in a read : write mix.  mix 0: copy src -> dst; 1: 2:1 (dst holds half of
    src's bytes); 2: 1:2 (dst holds twice src's bytes); 3: read src only (dst any non-empty uint8 device tensor)."""
    mix = int(mix)
    if mix not in (0, 1, 2, 3):
        raise ValueError("mix is 0 (1:1), 1 (2:1), 2 (1:2) or 3 (read only)")
    _buf(src, torch.uint8, "src")
    wide = 2 * src.numel() if mix == 2 else src.numel()
    if wide % 16 != 0:
        raise ValueError("the mover works in whole 16-byte chunks")
    need = {0: wide, 1: wide // 2, 2: wide, 3: 1}[mix]
    _buf(dst, torch.uint8, "dst", min_bytes=need)
    dev = _on_device(src=src, dst=dst)
    st = lib().mxfp4_stream_mix(src.data_ptr(), dst.data_ptr(), wide, int(policy), mix, _stream(stream, dev))
    _check("mxfp4_stream_mix", st)
    return dst


def mxfp4_tile_copy(src, dst, stream=None):
    """src uint8 [rows, row_bytes] moved tile by tile into dst (uint8, at least rows * row_bytes bytes) in the
    access pattern of mxfp4_row_to_col, without the conversion (rows % 256 == 0, row_bytes % 128 == 0)."""
    _buf(src, torch.uint8, "src")
    if src.dim() != 2 or src.shape[0] % 256 != 0 or src.shape[1] % 128 != 0:
        raise ValueError("src must be [rows % 256 == 0, row_bytes % 128 == 0]")
    _buf(dst, torch.uint8, "dst", min_bytes=src.numel())
    dev = _on_device(src=src, dst=dst)
    st = lib().mxfp4_tile_copy(src.data_ptr(), dst.data_ptr(), src.shape[0], src.shape[1], _stream(stream, dev))
    _check("mxfp4_tile_copy", st)
    return dst


def mxfp4_record_fanout(src, dst_idx, dst, rec_bytes=None, stream=None):
    """Record i of src (uint8 [M_src, ld_src]; its first rec_bytes bytes, default the whole row) written to the
    records dst_idx[i, j] of dst (uint8, a whole number of records of rec_bytes): the write traffic of
    mxfp4_quant_from_fp8_scatter without the quantizer."""
    _buf(src, torch.uint8, "src")
    if src.dim() != 2:
        raise ValueError("src must be [M_src, ld_src]")
    M_src, ld = src.shape
    rec = ld if rec_bytes is None else int(rec_bytes)
    if rec <= 0 or rec % 16 != 0 or ld % 16 != 0 or rec > ld or rec > 48 * 1024:
        raise ValueError("records are multiples of 16 bytes up to 48 KiB, no longer than a row of src")
    _buf(dst_idx, torch.int32, "dst_idx")
    if dst_idx.dim() != 2 or dst_idx.shape[0] != M_src or dst_idx.shape[1] < 1:
        raise ValueError("dst_idx must be int32 [M_src, fanout]")
    _buf(dst, torch.uint8, "dst")
    if dst.numel() % rec != 0:
        raise ValueError("dst must hold a whole number of records")
    dev = _on_device(src=src, dst_idx=dst_idx, dst=dst)
    st = lib().mxfp4_record_fanout(src.data_ptr(), ld, dst_idx.data_ptr(), M_src, dst_idx.shape[1], rec,
                                   dst.numel() // rec, dst.data_ptr(), _stream(stream, dev))
    _check("mxfp4_record_fanout", st)
    return dst
