"""TEST INFRASTRUCTURE (see ref.py).  Run the (single-threaded) oracle over row ranges in a thread pool.  Rows are independent
for quant / dequant, 32-row groups for row->col; ctypes releases the GIL during the calls."""
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

from . import ref

WORKERS = max(1, min(16, os.cpu_count() or 1))


def _ranges(M, step_multiple, workers=WORKERS):
    per = max(step_multiple, ((M + workers - 1) // workers + step_multiple - 1) // step_multiple * step_multiple)
    return [(lo, min(M, lo + per)) for lo in range(0, M, per)]


def quant(x, s, workers=WORKERS):
    x, s = np.ascontiguousarray(x), np.ascontiguousarray(s)
    rs = _ranges(x.shape[0], 1, workers)
    with ThreadPoolExecutor(workers) as ex:
        outs = list(ex.map(lambda r: ref.quant_from_fp8(x[r[0]:r[1]], s[r[0]:r[1]]), rs))
    return np.concatenate([o[0] for o in outs]), np.concatenate([o[1] for o in outs])


def quant_bf16(x, workers=WORKERS):
    x = np.ascontiguousarray(x)
    rs = _ranges(x.shape[0], 1, workers)
    with ThreadPoolExecutor(workers) as ex:
        outs = list(ex.map(lambda r: ref.quant_from_bf16(x[r[0]:r[1]]), rs))
    return np.concatenate([o[0] for o in outs]), np.concatenate([o[1] for o in outs])


def dequant(q, sf, workers=WORKERS):
    q, sf = np.ascontiguousarray(q), np.ascontiguousarray(sf)
    rs = _ranges(q.shape[0], 1, workers)
    with ThreadPoolExecutor(workers) as ex:
        outs = list(ex.map(lambda r: ref.dequant_to_fp8(q[r[0]:r[1]], sf[r[0]:r[1]]), rs))
    return np.concatenate([o[0] for o in outs]), np.concatenate([o[1] for o in outs])


def row_to_col(q, sf, workers=WORKERS):
    q, sf = np.ascontiguousarray(q), np.ascontiguousarray(sf)
    rs = _ranges(q.shape[0], 32, workers)
    with ThreadPoolExecutor(workers) as ex:
        outs = list(ex.map(lambda r: ref.row_to_col(q[r[0]:r[1]], sf[r[0]:r[1]]), rs))
    return np.concatenate([o[0] for o in outs], axis=1), np.concatenate([o[1] for o in outs], axis=1)


def row_to_fp8_col(q, sf, workers=WORKERS, requant=False):
    q, sf = np.ascontiguousarray(q), np.ascontiguousarray(sf)
    rs = _ranges(q.shape[0], 128, workers)
    with ThreadPoolExecutor(workers) as ex:
        outs = list(ex.map(lambda r: ref.row_to_fp8_col(q[r[0]:r[1]], sf[r[0]:r[1]], requant=requant), rs))
    return np.concatenate([o[0] for o in outs], axis=1), np.concatenate([o[1] for o in outs], axis=1)
