"""ctypes front end of the C oracle (oracle/bof4_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by bench.py's cpu_baseline leg.
The product package never imports this module and this module never imports the product package.

All arrays are numpy: weights / dequantised weights / scales / outlier values as uint16 bit patterns
(bfloat16 or binary16), codes as uint8, outlier indices as int64, codebooks as float64[16].
"""
import ctypes
import os

import numpy as np

from . import build as _build

OK, ERR_ARG, ERR_CAPACITY = 0, -1, -2
_lib = None


class LloydStats(ctypes.Structure):
    _fields_ = [("num", ctypes.c_double * 16), ("den", ctypes.c_double * 16), ("cnt", ctypes.c_uint64 * 16),
                ("sse", ctypes.c_double), ("n_used", ctypes.c_uint64), ("n_outliers", ctypes.c_uint64)]

    def as_dict(self):
        return {"num": np.array(self.num[:], dtype=np.float64), "den": np.array(self.den[:], dtype=np.float64),
                "cnt": np.array(self.cnt[:], dtype=np.uint64), "sse": float(self.sse),
                "n_used": int(self.n_used), "n_outliers": int(self.n_outliers)}


class ErrorStats(ctypes.Structure):
    _fields_ = [("sse", ctypes.c_double), ("sae", ctypes.c_double), ("max_abs", ctypes.c_double),
                ("n_outliers", ctypes.c_uint64), ("n", ctypes.c_uint64)]

    def as_dict(self):
        return {"sse": self.sse, "sae": self.sae, "max_abs": self.max_abs, "n_outliers": int(self.n_outliers),
                "n": int(self.n)}


class MaeStats(ctypes.Structure):
    _fields_ = [("median", ctypes.c_double * 16), ("den", ctypes.c_double * 16), ("cnt", ctypes.c_uint64 * 16),
                ("sae", ctypes.c_double), ("n_used", ctypes.c_uint64), ("n_outliers", ctypes.c_uint64)]

    def as_dict(self):
        return {"median": np.array(self.median[:], dtype=np.float64), "den": np.array(self.den[:], dtype=np.float64),
                "cnt": np.array(self.cnt[:], dtype=np.uint64), "sae": float(self.sae),
                "n_used": int(self.n_used), "n_outliers": int(self.n_outliers)}


def lib():
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path) or os.path.getmtime(path) < os.path.getmtime(_build.SRC):
            _build.build()
        L = ctypes.CDLL(path)
        u16p, u8p, i64p = (ctypes.POINTER(ctypes.c_uint16), ctypes.POINTER(ctypes.c_uint8),
                           ctypes.POINTER(ctypes.c_int64))
        f64p, u64p = ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_uint64)
        L.oracle_opq_threshold.restype = ctypes.c_double
        L.oracle_opq_threshold.argtypes = [ctypes.c_double, ctypes.c_uint32]
        L.oracle_quantize.restype = ctypes.c_int
        L.oracle_quantize.argtypes = [u16p, ctypes.c_uint64, ctypes.c_uint32, f64p, ctypes.c_int, ctypes.c_double,
                                      u8p, u16p, i64p, u16p, ctypes.c_uint64, u64p]
        L.oracle_dequantize.restype = ctypes.c_int
        L.oracle_dequantize.argtypes = [u8p, u16p, ctypes.c_uint64, ctypes.c_uint32, f64p, i64p, u16p,
                                        ctypes.c_uint64, u16p]
        L.oracle_quant_error.restype = ctypes.c_int
        L.oracle_quant_error.argtypes = [u16p, ctypes.c_uint64, ctypes.c_uint32, f64p, ctypes.c_int, ctypes.c_double,
                                         ctypes.POINTER(ErrorStats)]
        L.oracle_gemv.restype = ctypes.c_int
        L.oracle_gemv.argtypes = [u8p, u16p, ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint32, f64p, i64p, u16p,
                                  ctypes.c_uint64, u16p, ctypes.c_uint32, f64p, f64p]
        L.oracle_gemm.restype = ctypes.c_int
        L.oracle_gemm.argtypes = L.oracle_gemv.argtypes
        L.oracle_lloyd_step.restype = ctypes.c_int
        L.oracle_lloyd_step.argtypes = [u16p, ctypes.c_uint64, ctypes.c_uint32, f64p, ctypes.c_int,
                                        ctypes.c_double, ctypes.c_int, ctypes.POINTER(LloydStats)]
        L.oracle_codebook_update.restype = ctypes.c_int
        L.oracle_codebook_update.argtypes = [ctypes.POINTER(LloydStats), ctypes.c_uint16, f64p]
        L.oracle_lloyd_step_mae.restype = ctypes.c_int
        L.oracle_lloyd_step_mae.argtypes = [u16p, ctypes.c_uint64, ctypes.c_uint32, f64p, ctypes.c_int,
                                            ctypes.c_double, ctypes.c_int, ctypes.POINTER(MaeStats)]
        L.oracle_codebook_update_mae.restype = ctypes.c_int
        L.oracle_codebook_update_mae.argtypes = [ctypes.POINTER(MaeStats), ctypes.c_uint16, f64p]
        L.oracle_f32_to_f16.restype = ctypes.c_uint16
        L.oracle_f32_to_f16.argtypes = [ctypes.c_float]
        L.oracle_f16_to_f32.restype = ctypes.c_float
        L.oracle_f16_to_f32.argtypes = [ctypes.c_uint16]
        L.oracle_f32_to_bf16.restype = ctypes.c_uint16
        L.oracle_f32_to_bf16.argtypes = [ctypes.c_float]
        L.oracle_bf16_to_f32.restype = ctypes.c_float
        L.oracle_bf16_to_f32.argtypes = [ctypes.c_uint16]
        L.oracle_num_threads.restype = ctypes.c_int
        _lib = L
    return _lib


def _p(a, ct):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ct))


def _cb(cb):
    cb = np.ascontiguousarray(cb, dtype=np.float64)
    assert cb.shape == (16,)
    return cb


def _w(w):
    w = np.ascontiguousarray(w)
    assert w.dtype == np.uint16 and w.ndim == 1
    return w


def opq_threshold(q, block):
    return float(lib().oracle_opq_threshold(q, block))


def quantize(w, block, cb, signed, opq_T=0.0, capacity=None):
    """Returns (status, codes u8[n/2], scales u16[n/block], out_idx i64[k], out_val u16[k], n_outliers)."""
    w, cb = _w(w), _cb(cb)
    n = w.size
    if capacity is None:
        capacity = n if opq_T > 0 else 0
    codes = np.zeros(max(n // 2, 1), dtype=np.uint8)
    scales = np.zeros(max(n // max(block, 1), 1), dtype=np.uint16)
    oidx = np.zeros(max(capacity, 1), dtype=np.int64)
    oval = np.zeros(max(capacity, 1), dtype=np.uint16)
    nout = ctypes.c_uint64(0)
    st = lib().oracle_quantize(_p(w, ctypes.c_uint16), n, block, _p(cb, ctypes.c_double), int(signed),
                               float(opq_T), _p(codes, ctypes.c_uint8), _p(scales, ctypes.c_uint16),
                               _p(oidx, ctypes.c_int64), _p(oval, ctypes.c_uint16), capacity, ctypes.byref(nout))
    k = min(int(nout.value), capacity)
    return st, codes[: n // 2], scales[: n // max(block, 1)], oidx[:k].copy(), oval[:k].copy(), int(nout.value)


def dequantize(codes, scales, n, block, cb, out_idx=None, out_val=None):
    """Returns (status, bf16 bit patterns u16[n])."""
    cb = _cb(cb)
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    scales = np.ascontiguousarray(scales, dtype=np.uint16)
    k = 0 if out_idx is None else int(out_idx.size)
    if k:
        out_idx = np.ascontiguousarray(out_idx, dtype=np.int64)
        out_val = np.ascontiguousarray(out_val, dtype=np.uint16)
    out = np.zeros(max(n, 1), dtype=np.uint16)
    st = lib().oracle_dequantize(_p(codes, ctypes.c_uint8), _p(scales, ctypes.c_uint16), n, block,
                                 _p(cb, ctypes.c_double), _p(out_idx, ctypes.c_int64) if k else None,
                                 _p(out_val, ctypes.c_uint16) if k else None, k, _p(out, ctypes.c_uint16))
    return st, out[:n]


def quant_error(w, block, cb, signed, opq_T=0.0):
    """Returns (status, dict: sse, sae, max_abs of w - Q(w) over all weights, n_outliers, n)."""
    w, cb = _w(w), _cb(cb)
    st_ = ErrorStats()
    st = lib().oracle_quant_error(_p(w, ctypes.c_uint16), w.size, block, _p(cb, ctypes.c_double), int(signed),
                                  float(opq_T), ctypes.byref(st_))
    return st, st_.as_dict()


def gemv(codes, scales, rows, cols, block, cb, x, out_idx=None, out_val=None):
    """x: bf16 bit patterns u16[n_tokens, cols].  Returns (status, y f64[n_tokens, rows], sum |w~ x| f64[same])."""
    cb = _cb(cb)
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    scales = np.ascontiguousarray(scales, dtype=np.uint16)
    x = np.ascontiguousarray(x, dtype=np.uint16)
    if x.ndim == 1:
        x = x[None, :]
    assert x.shape[1] == cols
    k = 0 if out_idx is None else int(out_idx.size)
    if k:
        out_idx = np.ascontiguousarray(out_idx, dtype=np.int64)
        out_val = np.ascontiguousarray(out_val, dtype=np.uint16)
    y = np.zeros((x.shape[0], rows), dtype=np.float64)
    a = np.zeros((x.shape[0], rows), dtype=np.float64)
    st = lib().oracle_gemv(_p(codes, ctypes.c_uint8), _p(scales, ctypes.c_uint16), rows, cols, block,
                           _p(cb, ctypes.c_double), _p(out_idx, ctypes.c_int64) if k else None,
                           _p(out_val, ctypes.c_uint16) if k else None, k, _p(x, ctypes.c_uint16), x.shape[0],
                           _p(y, ctypes.c_double), _p(a, ctypes.c_double))
    return st, y, a


def gemm(codes, scales, rows, cols, block, cb, x, out_idx=None, out_val=None):
    """As gemv, over the decoded bfloat16 matrix (every weight rounded as oracle_dequantize rounds it)."""
    cb = _cb(cb)
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    scales = np.ascontiguousarray(scales, dtype=np.uint16)
    x = np.ascontiguousarray(x, dtype=np.uint16)
    if x.ndim == 1:
        x = x[None, :]
    assert x.shape[1] == cols
    k = 0 if out_idx is None else int(out_idx.size)
    if k:
        out_idx = np.ascontiguousarray(out_idx, dtype=np.int64)
        out_val = np.ascontiguousarray(out_val, dtype=np.uint16)
    y = np.zeros((x.shape[0], rows), dtype=np.float64)
    a = np.zeros((x.shape[0], rows), dtype=np.float64)
    st = lib().oracle_gemm(_p(codes, ctypes.c_uint8), _p(scales, ctypes.c_uint16), rows, cols, block,
                           _p(cb, ctypes.c_double), _p(out_idx, ctypes.c_int64) if k else None,
                           _p(out_val, ctypes.c_uint16) if k else None, k, _p(x, ctypes.c_uint16), x.shape[0],
                           _p(y, ctypes.c_double), _p(a, ctypes.c_double))
    return st, y, a


def lloyd_step(w, block, cb, signed, opq_T=0.0, weight_by_max2=True):
    """Returns (status, dict with num, den, cnt, sse, n_used, n_outliers)."""
    w, cb = _w(w), _cb(cb)
    s = LloydStats()
    st = lib().oracle_lloyd_step(_p(w, ctypes.c_uint16), w.size, block, _p(cb, ctypes.c_double), int(signed),
                                 float(opq_T), int(bool(weight_by_max2)), ctypes.byref(s))
    return st, s.as_dict()


def codebook_update(stats, pinned_mask, cb):
    """Returns the updated float64[16] codebook (input is not modified)."""
    cb = _cb(cb).copy()
    s = LloydStats()
    for l in range(16):
        s.num[l] = float(stats["num"][l])
        s.den[l] = float(stats["den"][l])
        s.cnt[l] = int(stats["cnt"][l])
    s.sse = float(stats["sse"])
    s.n_used = int(stats["n_used"])
    s.n_outliers = int(stats["n_outliers"])
    st = lib().oracle_codebook_update(ctypes.byref(s), pinned_mask, _p(cb, ctypes.c_double))
    assert st == OK
    return cb


def lloyd_step_mae(w, block, cb, signed, opq_T=0.0, weight_by_max=True):
    """MAE criterion (weighted medians; weight_by_max=False: plain medians of the normalised weights).  Returns
    (status, dict with median, den, cnt, sae, n_used, n_outliers)."""
    w, cb = _w(w), _cb(cb)
    s = MaeStats()
    st = lib().oracle_lloyd_step_mae(_p(w, ctypes.c_uint16), w.size, block, _p(cb, ctypes.c_double), int(signed),
                                     float(opq_T), int(bool(weight_by_max)), ctypes.byref(s))
    return st, s.as_dict()


def codebook_update_mae(stats, pinned_mask, cb):
    """Returns the updated float64[16] codebook (input is not modified)."""
    cb = _cb(cb).copy()
    s = MaeStats()
    for l in range(16):
        s.median[l] = float(stats["median"][l])
        s.den[l] = float(stats["den"][l])
        s.cnt[l] = int(stats["cnt"][l])
    st = lib().oracle_codebook_update_mae(ctypes.byref(s), pinned_mask, _p(cb, ctypes.c_double))
    assert st == OK
    return cb


def num_threads():
    return int(lib().oracle_num_threads())


def f32_to_f16(x):
    return int(lib().oracle_f32_to_f16(float(x)))


def f16_to_f32(h):
    return float(lib().oracle_f16_to_f32(int(h)))


def f32_to_bf16(x):
    return int(lib().oracle_f32_to_bf16(float(x)))


def bf16_to_f32(b):
    return float(lib().oracle_bf16_to_f32(int(b)))
