"""Run the (single-threaded, per-call) oracle over contiguous chunks of a large input in Python threads and stitch
the results together.  Blocks are independent, so chunking at block boundaries changes nothing; the outlier lists
of the chunks are concatenated with their flat offsets, which keeps them ascending."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np

import oracle

WORKERS = 16


def _bounds(n, block, chunks):
    nb = n // block
    return [(nb * c // chunks) * block for c in range(chunks + 1)]


def quantize(wb, block, cb, signed, T=0.0, chunks=WORKERS):
    n = wb.size
    bnd = _bounds(n, block, chunks)

    def run(c):
        lo, hi = bnd[c], bnd[c + 1]
        if hi == lo:
            return None
        return oracle.quantize(wb[lo:hi], block, cb, signed, opq_T=T)

    with ThreadPoolExecutor(WORKERS) as ex:
        parts = list(ex.map(run, range(chunks)))
    codes, scales, oidx, oval, nout = [], [], [], [], 0
    for c, p in enumerate(parts):
        if p is None:
            continue
        assert p[0] == oracle.OK
        codes.append(p[1]); scales.append(p[2]); oidx.append(p[3] + bnd[c]); oval.append(p[4]); nout += p[5]
    return (np.concatenate(codes), np.concatenate(scales), np.concatenate(oidx), np.concatenate(oval), nout)


def dequantize(codes, scales, n, block, cb, oidx=None, oval=None, chunks=WORKERS):
    bnd = _bounds(n, block, chunks)

    def run(c):
        lo, hi = bnd[c], bnd[c + 1]
        if hi == lo:
            return np.zeros(0, np.uint16)
        if oidx is not None and oidx.size:
            a, b = np.searchsorted(oidx, [lo, hi])
            st, d = oracle.dequantize(codes[lo // 2:hi // 2], scales[lo // block:hi // block], hi - lo, block, cb,
                                      oidx[a:b] - lo, oval[a:b])
        else:
            st, d = oracle.dequantize(codes[lo // 2:hi // 2], scales[lo // block:hi // block], hi - lo, block, cb)
        assert st == oracle.OK
        return d

    with ThreadPoolExecutor(WORKERS) as ex:
        return np.concatenate(list(ex.map(run, range(chunks))))
