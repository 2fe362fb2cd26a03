"""Run the (single-threaded, per-call) oracle functions over contiguous block ranges of a large input in Python threads
and stitch the results together.  TEST INFRASTRUCTURE ONLY, like the rest of this package.

Blocks are independent, so cutting at block boundaries changes nothing: every chunk goes through the unchanged C
function, the outlier lists of the chunks are concatenated with their flat offsets, which keeps them ascending."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np

from . import OK, dequantize as _dequantize, quantize as _quantize

WORKERS = 16


def _bounds(n, block, chunks):
    nb = n // block
    return [(nb * c // chunks) * block for c in range(chunks + 1)]


def quantize(wb, block, cb, signed, T=0.0, chunks=None, workers=WORKERS):
    """Returns (codes, scales, out_idx, out_val, n_outliers) of oracle.quantize over all of wb."""
    n = wb.size
    chunks = workers if chunks is None else chunks
    bnd = _bounds(n, block, chunks)

    def run(c):
        lo, hi = bnd[c], bnd[c + 1]
        if hi == lo:
            return None
        return _quantize(wb[lo:hi], block, cb, signed, opq_T=T)

    with ThreadPoolExecutor(workers) as ex:
        parts = list(ex.map(run, range(chunks)))
    codes, scales, oidx, oval, nout = [], [], [], [], 0
    for c, p in enumerate(parts):
        if p is None:
            continue
        assert p[0] == OK
        codes.append(p[1]); scales.append(p[2]); oidx.append(p[3] + bnd[c]); oval.append(p[4]); nout += p[5]
    return (np.concatenate(codes), np.concatenate(scales), np.concatenate(oidx), np.concatenate(oval), nout)


def dequantize(codes, scales, n, block, cb, oidx=None, oval=None, chunks=None, workers=WORKERS):
    """Returns the decoded bf16 bit patterns of oracle.dequantize over all n weights."""
    chunks = workers if chunks is None else chunks
    bnd = _bounds(n, block, chunks)

    def run(c):
        lo, hi = bnd[c], bnd[c + 1]
        if hi == lo:
            return np.zeros(0, np.uint16)
        if oidx is not None and oidx.size:
            a, b = np.searchsorted(oidx, [lo, hi])
            st, d = _dequantize(codes[lo // 2:hi // 2], scales[lo // block:hi // block], hi - lo, block, cb,
                                oidx[a:b] - lo, oval[a:b])
        else:
            st, d = _dequantize(codes[lo // 2:hi // 2], scales[lo // block:hi // block], hi - lo, block, cb)
        assert st == OK
        return d

    with ThreadPoolExecutor(workers) as ex:
        return np.concatenate(list(ex.map(run, range(chunks))))
