"""Thin ctypes binding of include/bof4.h: argument marshalling only, every step of the path runs in the HIP library.

torch supplies device memory (tensors) and the stream; nothing is computed here.  The functions carry the names of
the C entry points.  A missing library is an error (there is no fallback of any kind).
"""
import ctypes
import os

import numpy as np
import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libbof4_hip.so")

BOF4_OK, BOF4_ERR_ARG, BOF4_ERR_CAPACITY, BOF4_ERR_WORKSPACE, BOF4_ERR_HIP = 0, -1, -2, -3, -4
EXPORTS = ("bof4_workspace_bytes", "bof4_opq_threshold", "bof4_thresholds", "bof4_bin_table", "bof4_lloyd_step",
           "bof4_codebook_update", "bof4_lloyd_step_mae", "bof4_codebook_update_mae", "bof4_quantize",
           "bof4_dequantize", "bof4_quantize_begin", "bof4_quantize_finish", "bof4_lloyd_step_begin", "bof4_wait_result",
           "bof4_lloyd_step_static", "bof4_quantize_lloyd", "bof4_quantize_lloyd_begin", "bof4_quantize_lloyd_finish",
           "bof4_quant_error", "bof4_gemv", "bof4_gemv_outlier_table",
           "bof4_gemv_outlier_table_bytes", "bof4_gemm", "bof4_gemm_pack", "bof4_gemm_packed_bytes",
           "bof4_gemm_outlier_table", "bof4_gemm_workspace_bytes",
           "bof4_theory_centroids", "bof4_theory_workspace_bytes", "bof4_time_next_call", "bof4_last_error",
           "bof4_last_hip_error")


class Bof4Error(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"bof4 error {code}: {msg}")
        self.code = code


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


_lib = None


def lib():
    """Load libbof4_hip.so (built by `python -m paper_2505_06653_amd.build`); raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} not built - run `python -m paper_2505_06653_amd.build` "
                              "(there is no CPU fallback)")
        L = ctypes.CDLL(LIB_PATH)
        vp, f64p = ctypes.c_void_p, ctypes.POINTER(ctypes.c_double)
        L.bof4_workspace_bytes.restype = ctypes.c_size_t
        L.bof4_workspace_bytes.argtypes = [ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint64]
        L.bof4_opq_threshold.restype = ctypes.c_double
        L.bof4_opq_threshold.argtypes = [ctypes.c_double, ctypes.c_uint32]
        L.bof4_thresholds.restype = ctypes.c_int
        L.bof4_thresholds.argtypes = [f64p, ctypes.POINTER(ctypes.c_float)]
        L.bof4_bin_table.restype = ctypes.c_int
        L.bof4_bin_table.argtypes = [f64p, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_uint32),
                                     ctypes.POINTER(ctypes.c_int)]
        L.bof4_lloyd_step.restype = ctypes.c_int
        L.bof4_lloyd_step.argtypes = [vp, ctypes.c_uint64, ctypes.c_uint32, f64p, ctypes.c_int, ctypes.c_double,
                                      ctypes.c_int, ctypes.POINTER(LloydStats), vp, ctypes.c_size_t, vp]
        L.bof4_codebook_update.restype = ctypes.c_int
        L.bof4_codebook_update.argtypes = [ctypes.POINTER(LloydStats), ctypes.c_uint16, vp]
        L.bof4_lloyd_step_mae.restype = ctypes.c_int
        L.bof4_lloyd_step_mae.argtypes = [vp, ctypes.c_uint64, ctypes.c_uint32, f64p, ctypes.c_int, ctypes.c_double,
                                          ctypes.c_int, ctypes.c_uint16, ctypes.POINTER(MaeStats), vp, ctypes.c_size_t,
                                          vp]
        L.bof4_codebook_update_mae.restype = ctypes.c_int
        L.bof4_codebook_update_mae.argtypes = [ctypes.POINTER(MaeStats), ctypes.c_uint16, vp]
        L.bof4_quantize.restype = ctypes.c_int
        L.bof4_quantize.argtypes = [vp, ctypes.c_uint64, ctypes.c_uint32, f64p, ctypes.c_int, ctypes.c_double,
                                    vp, vp, vp, vp, ctypes.c_uint64, ctypes.POINTER(ctypes.c_uint64), vp,
                                    ctypes.c_size_t, vp]
        for name in ("bof4_quantize_begin", "bof4_quantize_finish"):
            getattr(L, name).restype = ctypes.c_int
            getattr(L, name).argtypes = L.bof4_quantize.argtypes
        for name in ("bof4_quantize_lloyd", "bof4_quantize_lloyd_begin", "bof4_quantize_lloyd_finish"):
            getattr(L, name).restype = ctypes.c_int
            getattr(L, name).argtypes = [vp, ctypes.c_uint64, ctypes.c_uint32, f64p, ctypes.c_int, ctypes.c_double,
                                         ctypes.c_int, vp, vp, vp, vp, ctypes.c_uint64, ctypes.POINTER(ctypes.c_uint64),
                                         ctypes.POINTER(LloydStats), vp, ctypes.c_size_t, vp]
        L.bof4_lloyd_step_begin.restype = ctypes.c_int
        L.bof4_lloyd_step_begin.argtypes = L.bof4_lloyd_step.argtypes
        L.bof4_lloyd_step_static.restype = ctypes.c_int
        L.bof4_lloyd_step_static.argtypes = [vp, ctypes.c_uint64, ctypes.c_uint32, f64p, ctypes.c_int, ctypes.c_double,
                                             ctypes.c_int, ctypes.POINTER(LloydStats), vp]
        L.bof4_wait_result.restype = ctypes.c_int
        L.bof4_wait_result.argtypes = [vp, vp]
        L.bof4_dequantize.restype = ctypes.c_int
        L.bof4_dequantize.argtypes = [vp, vp, ctypes.c_uint64, ctypes.c_uint32, f64p, vp, vp, ctypes.c_uint64, vp, vp]
        L.bof4_quant_error.restype = ctypes.c_int
        L.bof4_quant_error.argtypes = [vp, ctypes.c_uint64, ctypes.c_uint32, f64p, ctypes.c_int, ctypes.c_double,
                                       ctypes.POINTER(ErrorStats), vp, ctypes.c_size_t, vp]
        L.bof4_gemv.restype = ctypes.c_int
        L.bof4_gemv.argtypes = [vp, vp, ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint32, f64p, vp, ctypes.c_uint64,
                                vp, ctypes.c_uint32, vp, vp]
        L.bof4_gemv_outlier_table.restype = ctypes.c_int
        L.bof4_gemv_outlier_table.argtypes = [vp, vp, ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint32, f64p, vp, vp,
                                              ctypes.c_uint64, vp, ctypes.c_size_t, vp]
        L.bof4_gemv_outlier_table_bytes.restype = ctypes.c_size_t
        L.bof4_gemv_outlier_table_bytes.argtypes = [ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint64]
        L.bof4_gemm.restype = ctypes.c_int
        L.bof4_gemm.argtypes = [vp, ctypes.c_uint64, ctypes.c_uint64, f64p, vp, ctypes.c_uint64, vp, ctypes.c_uint32,
                                vp, vp, ctypes.c_size_t, vp]
        L.bof4_gemm_pack.restype = ctypes.c_int
        L.bof4_gemm_pack.argtypes = [vp, vp, ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint32, vp, ctypes.c_size_t, vp]
        L.bof4_gemm_packed_bytes.restype = ctypes.c_size_t
        L.bof4_gemm_packed_bytes.argtypes = [ctypes.c_uint64, ctypes.c_uint64]
        L.bof4_gemm_outlier_table.restype = ctypes.c_int
        L.bof4_gemm_outlier_table.argtypes = L.bof4_gemv_outlier_table.argtypes
        L.bof4_gemm_workspace_bytes.restype = ctypes.c_size_t
        L.bof4_gemm_workspace_bytes.argtypes = [ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint32]
        L.bof4_theory_workspace_bytes.restype = ctypes.c_size_t
        L.bof4_theory_workspace_bytes.argtypes = [ctypes.c_uint32]
        L.bof4_theory_centroids.restype = ctypes.c_int
        L.bof4_theory_centroids.argtypes = [f64p, f64p, ctypes.c_uint32, ctypes.c_double, ctypes.c_uint32, f64p,
                                            ctypes.c_uint16, ctypes.c_int, f64p, vp, ctypes.c_size_t, vp]
        L.bof4_time_next_call.restype = ctypes.c_int
        L.bof4_time_next_call.argtypes = [vp, vp]
        L.bof4_last_error.restype = ctypes.c_char_p
        L.bof4_last_hip_error.restype = ctypes.c_int
        _lib = L
    return _lib


def _check(code, allow=()):
    if code != BOF4_OK and code not in allow:
        raise Bof4Error(code, lib().bof4_last_error().decode())
    return code


_F64P = ctypes.POINTER(ctypes.c_double)
_cb_cache = {}  # id(array) -> (array, pointer); holding the array keeps its id from being reused


def _cb(cb):
    """Codebook as a contiguous float64[16] array plus its ctypes pointer.  Arrays that already have that form are
    passed through, and their pointer object is kept (building one costs more than the rest of a call's marshalling)."""
    hit = _cb_cache.get(id(cb))
    if hit is not None and hit[0] is cb:
        return cb, hit[1]
    arr = cb if (type(cb) is np.ndarray and cb.dtype == np.float64 and cb.flags.c_contiguous) \
        else np.ascontiguousarray(cb, dtype=np.float64)
    if arr.shape != (16,):
        raise ValueError("codebook must have 16 levels")
    ptr = arr.ctypes.data_as(_F64P)
    if arr is cb:
        if len(_cb_cache) >= 16:
            _cb_cache.clear()
        _cb_cache[id(cb)] = (cb, ptr)
    return arr, ptr


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


try:
    _raw_stream = torch._C._cuda_getCurrentRawStream  # the current stream's handle without building a Stream object
except AttributeError:  # pragma: no cover
    _raw_stream = None


def _stream(stream):
    if stream is not None:
        return ctypes.c_void_p(stream.cuda_stream)
    if _raw_stream is not None:
        return ctypes.c_void_p(_raw_stream(torch.cuda.current_device()))
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def bof4_workspace_bytes(n, block, out_capacity=0):
    return int(lib().bof4_workspace_bytes(n, block, out_capacity))


def bof4_opq_threshold(q, block):
    return float(lib().bof4_opq_threshold(q, block))


def bof4_thresholds(cb):
    cb, cbp = _cb(cb)
    thr = np.zeros(15, dtype=np.float32)
    _check(lib().bof4_thresholds(cbp, thr.ctypes.data_as(ctypes.POINTER(ctypes.c_float))))
    return thr


def bof4_bin_table(cb):
    """Returns (thr float32[33], base uint32[33], fast bool)."""
    cb, cbp = _cb(cb)
    thr = np.zeros(33, dtype=np.float32)
    base = np.zeros(33, dtype=np.uint32)
    fast = ctypes.c_int(0)
    _check(lib().bof4_bin_table(cbp, thr.ctypes.data_as(ctypes.POINTER(ctypes.c_float)),
                                base.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32)), ctypes.byref(fast)))
    return thr, base, bool(fast.value)


def bof4_codebook_update(stats, pinned_mask, cb):
    """stats: LloydStats (as returned by bof4_lloyd_step(..., raw=True)) or its dict form.  Returns new float64[16]."""
    out = np.array(cb, dtype=np.float64)  # a copy: the C function updates in place
    if out.shape != (16,):
        raise ValueError("codebook must have 16 levels")
    if not isinstance(stats, LloydStats):
        s = LloydStats()
        for l in range(16):
            s.num[l], s.den[l], s.cnt[l] = float(stats["num"][l]), float(stats["den"][l]), int(stats["cnt"][l])
        s.sse, s.n_used, s.n_outliers = float(stats["sse"]), int(stats["n_used"]), int(stats["n_outliers"])
        stats = s
    _check(lib().bof4_codebook_update(ctypes.byref(stats), pinned_mask, out.ctypes.data))
    return out


def bof4_theory_centroids(pdf, cdf, u_max, block, cb, pinned_mask, signed, ws=None, stream=None, device="cuda"):
    """One theoretical maximisation step for the distribution tabulated in pdf / cdf (float64 arrays over [0, u_max]).
    Returns the new float64[16] codebook."""
    pdf = np.ascontiguousarray(pdf, dtype=np.float64)
    cdf = np.ascontiguousarray(cdf, dtype=np.float64)
    if pdf.shape != cdf.shape or pdf.ndim != 1:
        raise ValueError("pdf and cdf must be 1-d arrays of one length")
    cb, cbp = _cb(cb)
    n = int(pdf.size)
    if ws is None:
        ws = torch.empty(int(lib().bof4_theory_workspace_bytes(n)), dtype=torch.uint8, device=device)
    out = np.zeros(16, dtype=np.float64)
    _check(lib().bof4_theory_centroids(pdf.ctypes.data_as(_F64P), cdf.ctypes.data_as(_F64P), n, float(u_max), block,
                                       cbp, int(pinned_mask), int(signed), out.ctypes.data_as(_F64P), _ptr(ws),
                                       ws.numel(), _stream(stream)))
    return out


def bof4_time_next_call(start_event, stop_event):
    """start_event / stop_event: torch.cuda.Event(enable_timing=True) that have been recorded once (so that their
    HIP handles exist); the next call records them around its main kernel."""
    _check(lib().bof4_time_next_call(ctypes.c_void_p(start_event.cuda_event), ctypes.c_void_p(stop_event.cuda_event)))


def alloc_workspace(n, block, out_capacity=0, device="cuda"):
    nbytes = max(bof4_workspace_bytes(n, block, out_capacity), 256)
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def pinned_lloyd_stats():
    """A LloydStats record in pinned host memory (the GPU then writes results in place).  Returns (struct, keepalive)."""
    buf = torch.zeros(ctypes.sizeof(LloydStats), dtype=torch.uint8).pin_memory()
    return LloydStats.from_address(buf.data_ptr()), buf


def pinned_mae_stats():
    """A MaeStats record in pinned host memory.  Returns (struct, keepalive)."""
    buf = torch.zeros(ctypes.sizeof(MaeStats), dtype=torch.uint8).pin_memory()
    return MaeStats.from_address(buf.data_ptr()), buf


def pinned_counter():
    """A uint64 outlier counter in pinned host memory.  Returns (ctypes.c_uint64, keepalive)."""
    buf = torch.zeros(1, dtype=torch.int64).pin_memory()
    return ctypes.c_uint64.from_address(buf.data_ptr()), buf


def pinned_error_stats():
    """An ErrorStats record in pinned host memory.  Returns (struct, keepalive)."""
    buf = torch.zeros(ctypes.sizeof(ErrorStats), dtype=torch.uint8).pin_memory()
    return ErrorStats.from_address(buf.data_ptr()), buf


def bof4_quant_error(w, block, cb, signed, opq_T=0.0, ws=None, stream=None, out=None):
    """Quantisation error of the flat bf16 device tensor w: dict with sse, sae, max_abs, n_outliers, n."""
    cb, cbp = _cb(cb)
    n = w.numel()
    if ws is None:
        ws = alloc_workspace(n, block, 0, w.device)
    rec = out if out is not None else ErrorStats()
    _check(lib().bof4_quant_error(_ptr(w), n, block, cbp, int(signed), float(opq_T), ctypes.byref(rec), _ptr(ws),
                                  ws.numel(), _stream(stream)))
    return rec.as_dict()


def bof4_gemv_outlier_table_bytes(rows, cols, n_outliers):
    return int(lib().bof4_gemv_outlier_table_bytes(rows, cols, n_outliers))


def bof4_gemv_outlier_table(codes, scales, rows, cols, block, cb, out_idx, out_val, n_outliers=None, out=None,
                            stream=None):
    """The outlier list of one quantised matrix in the form bof4_gemv reads (uint8 device tensor; made once)."""
    cb, cbp = _cb(cb)
    k = 0 if out_idx is None else int(out_idx.numel())
    if n_outliers is not None:
        if n_outliers > k:
            raise ValueError("n_outliers exceeds the list")
        k = int(n_outliers)
    if out is None:
        out = torch.empty(bof4_gemv_outlier_table_bytes(rows, cols, k), dtype=torch.uint8, device=codes.device)
    _check(lib().bof4_gemv_outlier_table(_ptr(codes), _ptr(scales), rows, cols, block, cbp,
                                         _ptr(out_idx) if k else None, _ptr(out_val) if k else None, k, _ptr(out),
                                         out.numel(), _stream(stream)))
    return out


def bof4_gemv(codes, scales, rows, cols, block, cb, x, table=None, n_outliers=0, out=None, stream=None):
    """y = x W~^T for the quantised row-major [rows, cols] matrix; x is bf16 [n_tokens, cols] (or [cols]) on the
    device, the result float32 [n_tokens, rows].  `table` (bof4_gemv_outlier_table) brings n_outliers outliers in."""
    cb, cbp = _cb(cb)
    x2 = x if x.dim() == 2 else x[None, :]
    if x2.dtype != torch.bfloat16 or x2.shape[1] != cols or not x2.is_contiguous():
        raise ValueError("x must be a contiguous bfloat16 tensor of [n_tokens, cols]")
    n_tokens = int(x2.shape[0])
    if out is None:
        out = torch.empty((n_tokens, rows), dtype=torch.float32, device=x.device)
    k = int(n_outliers)
    if k and table is None:
        raise ValueError("outliers need their table (bof4_gemv_outlier_table)")
    _check(lib().bof4_gemv(_ptr(codes), _ptr(scales), rows, cols, block, cbp, _ptr(table) if k else None, k,
                           _ptr(x2), n_tokens, _ptr(out), _stream(stream)))
    return out


def bof4_gemm_workspace_bytes(rows, cols, n_tokens):
    return int(lib().bof4_gemm_workspace_bytes(rows, cols, n_tokens))


def bof4_gemm_outlier_table(codes, scales, rows, cols, block, cb, out_idx, out_val, n_outliers=None, out=None,
                            stream=None):
    """The outlier list of one quantised matrix in the form bof4_gemm reads (uint8 device tensor; made once)."""
    cb, cbp = _cb(cb)
    k = 0 if out_idx is None else int(out_idx.numel())
    if n_outliers is not None:
        if n_outliers > k:
            raise ValueError("n_outliers exceeds the list")
        k = int(n_outliers)
    if out is None:
        out = torch.empty(bof4_gemv_outlier_table_bytes(rows, cols, k), dtype=torch.uint8, device=codes.device)
    _check(lib().bof4_gemm_outlier_table(_ptr(codes), _ptr(scales), rows, cols, block, cbp,
                                         _ptr(out_idx) if k else None, _ptr(out_val) if k else None, k, _ptr(out),
                                         out.numel(), _stream(stream)))
    return out


def bof4_gemm_packed_bytes(rows, cols):
    return int(lib().bof4_gemm_packed_bytes(rows, cols))


def bof4_gemm_pack(codes, scales, rows, cols, block, out=None, stream=None):
    """Codes and block constants of one quantised matrix in the order bof4_gemm reads them (uint8 device tensor;
    made once)."""
    if out is None:
        out = torch.empty(bof4_gemm_packed_bytes(rows, cols), dtype=torch.uint8, device=codes.device)
    _check(lib().bof4_gemm_pack(_ptr(codes), _ptr(scales), rows, cols, block, _ptr(out), out.numel(), _stream(stream)))
    return out


def bof4_gemm(packed, rows, cols, cb, x, table=None, n_outliers=0, out=None, ws=None, stream=None):
    """y = x W^^T for the decoded (bfloat16) form of the quantised row-major [rows, cols] matrix, given as
    bof4_gemm_pack made it; x is bf16 [n_tokens, cols] on the device, the result float32 [n_tokens, rows].  `table`
    (bof4_gemm_outlier_table) brings n_outliers outliers in; `ws`: optional uint8 device tensor of
    bof4_gemm_workspace_bytes(...) bytes."""
    cb, cbp = _cb(cb)
    x2 = x if x.dim() == 2 else x[None, :]
    if x2.dtype != torch.bfloat16 or x2.shape[1] != cols or not x2.is_contiguous():
        raise ValueError("x must be a contiguous bfloat16 tensor of [n_tokens, cols]")
    if packed.numel() < bof4_gemm_packed_bytes(rows, cols):
        raise ValueError("packed matrix too small for rows x cols (bof4_gemm_pack)")
    n_tokens = int(x2.shape[0])
    if out is None:
        out = torch.empty((n_tokens, rows), dtype=torch.float32, device=x.device)
    k = int(n_outliers)
    if k and table is None:
        raise ValueError("outliers need their table (bof4_gemm_outlier_table)")
    if ws is None:
        ws = torch.empty(bof4_gemm_workspace_bytes(rows, cols, n_tokens), dtype=torch.uint8, device=x.device)
    _check(lib().bof4_gemm(_ptr(packed), rows, cols, cbp, _ptr(table) if k else None, k, _ptr(x2), n_tokens,
                           _ptr(out), _ptr(ws), ws.numel(), _stream(stream)))
    return out


def bof4_lloyd_step(w, block, cb, signed, opq_T=0.0, weight_by_max2=True, ws=None, stream=None, raw=False, out=None):
    """w: flat bf16 device tensor.  Returns the statistics as a dict (or the ctypes struct with raw=True).
    `out`: optional LloydStats to fill (e.g. from pinned_lloyd_stats())."""
    assert w.dtype == torch.bfloat16 and w.is_cuda and w.is_contiguous()
    n = w.numel()
    cb, cbp = _cb(cb)
    if ws is None:
        ws = alloc_workspace(n, block, 0, w.device)
    if out is None:
        out = LloydStats()
    _check(lib().bof4_lloyd_step(_ptr(w), n, block, cbp, int(signed), float(opq_T), int(bool(weight_by_max2)),
                                 ctypes.byref(out), _ptr(ws), ws.numel(), _stream(stream)))
    return out if raw else out.as_dict()


def bof4_lloyd_step_mae(w, block, cb, signed, opq_T=0.0, skip_mask=0, ws=None, stream=None, raw=False, out=None,
                        weight_by_max=True):
    """MAE criterion: per-region weighted medians (weight_by_max=False: plain medians of the normalised weights).
    w: flat bf16 device tensor.  skip_mask: regions (pinned levels) whose median is not wanted.  Returns the statistics as a dict (or the ctypes struct with raw=True)."""
    assert w.dtype == torch.bfloat16 and w.is_cuda and w.is_contiguous()
    n = w.numel()
    cb, cbp = _cb(cb)
    if ws is None:
        ws = alloc_workspace(n, block, 0, w.device)
    if out is None:
        out = MaeStats()
    _check(lib().bof4_lloyd_step_mae(_ptr(w), n, block, cbp, int(signed), float(opq_T), int(bool(weight_by_max)),
                                     int(skip_mask),
                                     ctypes.byref(out), _ptr(ws), ws.numel(), _stream(stream)))
    return out if raw else out.as_dict()


def bof4_codebook_update_mae(stats, pinned_mask, cb):
    """stats: MaeStats or its dict form.  Returns new float64[16]."""
    out = np.array(cb, dtype=np.float64)
    if out.shape != (16,):
        raise ValueError("codebook must have 16 levels")
    if not isinstance(stats, MaeStats):
        s = MaeStats()
        for l in range(16):
            s.median[l], s.den[l], s.cnt[l] = float(stats["median"][l]), float(stats["den"][l]), int(stats["cnt"][l])
        s.sae, s.n_used, s.n_outliers = float(stats["sae"]), int(stats["n_used"]), int(stats["n_outliers"])
        stats = s
    _check(lib().bof4_codebook_update_mae(ctypes.byref(stats), pinned_mask, out.ctypes.data))
    return out


def bof4_quantize(w, block, cb, signed, opq_T=0.0, out_capacity=0, codes=None, scales=None, out_idx=None,
                  out_val=None, ws=None, stream=None, allow_overflow=False, counter=None, trim=True):
    """w: flat bf16 device tensor.  Returns (codes u8[n/2], scales f16[n/block], out_idx i64[k], out_val f16[k],
    n_outliers).  Output tensors are allocated here unless passed in; trim=False returns the outlier buffers whole
    (the first n_outliers entries are the list)."""
    assert w.dtype == torch.bfloat16 and w.is_cuda and w.is_contiguous()
    n = w.numel()
    dev = w.device
    cb, cbp = _cb(cb)
    if codes is None:
        codes = torch.empty(max(n // 2, 1), dtype=torch.uint8, device=dev)
    if scales is None:
        scales = torch.empty(max(n // max(block, 1), 1), dtype=torch.float16, device=dev)
    if opq_T > 0:
        if out_idx is None:
            out_idx = torch.empty(max(out_capacity, 1), dtype=torch.int64, device=dev)
        if out_val is None:
            out_val = torch.empty(max(out_capacity, 1), dtype=torch.float16, device=dev)
        if ws is None:
            ws = alloc_workspace(n, block, out_capacity, dev)
    nout = counter if counter is not None else ctypes.c_uint64(0)
    code = lib().bof4_quantize(_ptr(w), n, block, cbp, int(signed), float(opq_T), _ptr(codes), _ptr(scales),
                               _ptr(out_idx), _ptr(out_val), out_capacity, ctypes.byref(nout), _ptr(ws),
                               0 if ws is None else ws.numel(), _stream(stream))
    _check(code, allow=(BOF4_ERR_CAPACITY,) if allow_overflow else ())
    if not trim:
        return codes, scales, out_idx, out_val, int(nout.value)
    k = min(int(nout.value), out_capacity)
    return (codes, scales, None if out_idx is None else out_idx[:k], None if out_val is None else out_val[:k],
            int(nout.value))


def bof4_quantize_lloyd(w, block, cb, signed, opq_T=0.0, out_capacity=0, weight_by_max2=True, codes=None, scales=None,
                        out_idx=None, out_val=None, ws=None, stream=None, allow_overflow=False, counter=None,
                        stats=None, trim=True, raw=False):
    """bof4_quantize and bof4_lloyd_step in one pass.  Returns (codes, scales, out_idx, out_val, n_outliers, stats):
    the first five as bof4_quantize returns them, stats as bof4_lloyd_step does (dict, or the struct with raw=True)."""
    assert w.dtype == torch.bfloat16 and w.is_cuda and w.is_contiguous()
    n = w.numel()
    dev = w.device
    cb, cbp = _cb(cb)
    if codes is None:
        codes = torch.empty(max(n // 2, 1), dtype=torch.uint8, device=dev)
    if scales is None:
        scales = torch.empty(max(n // max(block, 1), 1), dtype=torch.float16, device=dev)
    if opq_T > 0:
        if out_idx is None:
            out_idx = torch.empty(max(out_capacity, 1), dtype=torch.int64, device=dev)
        if out_val is None:
            out_val = torch.empty(max(out_capacity, 1), dtype=torch.float16, device=dev)
    if ws is None:
        ws = alloc_workspace(n, block, out_capacity, dev)
    nout = counter if counter is not None else ctypes.c_uint64(0)
    st = stats if stats is not None else LloydStats()
    code = lib().bof4_quantize_lloyd(_ptr(w), n, block, cbp, int(signed), float(opq_T), int(bool(weight_by_max2)),
                                     _ptr(codes), _ptr(scales), _ptr(out_idx), _ptr(out_val), out_capacity,
                                     ctypes.byref(nout), ctypes.byref(st), _ptr(ws), ws.numel(), _stream(stream))
    _check(code, allow=(BOF4_ERR_CAPACITY,) if allow_overflow else ())
    stats_out = st if raw else st.as_dict()
    if not trim:
        return codes, scales, out_idx, out_val, int(nout.value), stats_out
    k = min(int(nout.value), out_capacity)
    return (codes, scales, None if out_idx is None else out_idx[:k], None if out_val is None else out_val[:k],
            int(nout.value), stats_out)


class QuantizeLloydInFlight:
    """bof4_quantize_lloyd_begin has been called with these arguments; finish() waits for the outlier count and
    returns it (the sums: bof4_wait_result(stats))."""

    def __init__(self, args, counter, keep):
        self.args, self.counter, self.keep = args, counter, keep

    def finish(self, allow_overflow=False):
        code = lib().bof4_quantize_lloyd_finish(*self.args)
        _check(code, allow=(BOF4_ERR_CAPACITY,) if allow_overflow else ())
        return int(self.counter.value)


def bof4_quantize_lloyd_begin(w, block, cb, signed, opq_T, out_capacity, codes, scales, out_idx, out_val, ws, counter,
                              stats, weight_by_max2=True, stream=None):
    """Enqueues bof4_quantize_lloyd into caller-owned buffers (counter: pinned_counter(), stats:
    pinned_lloyd_stats()) and returns a QuantizeLloydInFlight."""
    n = w.numel()
    cb, cbp = _cb(cb)
    args = (_ptr(w), n, block, cbp, int(signed), float(opq_T), int(bool(weight_by_max2)), _ptr(codes), _ptr(scales),
            _ptr(out_idx), _ptr(out_val), out_capacity, ctypes.byref(counter), ctypes.byref(stats), _ptr(ws),
            0 if ws is None else ws.numel(), _stream(stream))
    _check(lib().bof4_quantize_lloyd_begin(*args))
    return QuantizeLloydInFlight(args, counter, (w, cb, codes, scales, out_idx, out_val, ws, stats))


class QuantizeInFlight:
    """bof4_quantize_begin has been called with these arguments; finish() waits for the outlier count and returns it."""

    def __init__(self, args, counter, keep):
        self.args, self.counter, self.keep = args, counter, keep

    def finish(self, allow_overflow=False):
        code = lib().bof4_quantize_finish(*self.args)
        _check(code, allow=(BOF4_ERR_CAPACITY,) if allow_overflow else ())
        return int(self.counter.value)


def bof4_quantize_begin(w, block, cb, signed, opq_T, out_capacity, codes, scales, out_idx, out_val, ws, counter,
                        stream=None):
    """Enqueues bof4_quantize into caller-owned buffers (counter: from pinned_counter()) and returns a
    QuantizeInFlight; other work may be enqueued on the stream before its finish() is called."""
    n = w.numel()
    cb, cbp = _cb(cb)
    args = (_ptr(w), n, block, cbp, int(signed), float(opq_T), _ptr(codes), _ptr(scales), _ptr(out_idx),
            _ptr(out_val), out_capacity, ctypes.byref(counter), _ptr(ws), 0 if ws is None else ws.numel(),
            _stream(stream))
    _check(lib().bof4_quantize_begin(*args))
    return QuantizeInFlight(args, counter, (w, cb, codes, scales, out_idx, out_val, ws))


def bof4_lloyd_step_begin(w, block, cb, signed, out, opq_T=0.0, weight_by_max2=True, ws=None, stream=None):
    """Enqueues bof4_lloyd_step; `out` is a LloydStats in pinned host memory (pinned_lloyd_stats()), complete after
    bof4_wait_result(out)."""
    n = w.numel()
    cb, cbp = _cb(cb)
    if ws is None:
        ws = alloc_workspace(n, block, 0, w.device)
    _check(lib().bof4_lloyd_step_begin(_ptr(w), n, block, cbp, int(signed), float(opq_T), int(bool(weight_by_max2)),
                                       ctypes.byref(out), _ptr(ws), ws.numel(), _stream(stream)))
    return out


def bof4_lloyd_step_static(w, block, cb, signed, out, opq_T=0.0, weight_by_max2=True, stream=None, n=None):
    """bof4_lloyd_step without a workspace argument (the library's own fixed device array holds the partial sums; no
    allocation anywhere in the call).  `out`: a LloydStats in pinned host memory (pinned_lloyd_stats()).  `n`: number
    of weights, if not all of w."""
    n = w.numel() if n is None else int(n)
    cb, cbp = _cb(cb)
    _check(lib().bof4_lloyd_step_static(_ptr(w), n, block, cbp, int(signed), float(opq_T), int(bool(weight_by_max2)),
                                        ctypes.byref(out), _stream(stream)))
    return out


def bof4_wait_result(stats, stream=None):
    """Waits until the GPU has written the record `stats` (LloydStats / MaeStats: word n_used; ErrorStats: word n)."""
    field = "n" if isinstance(stats, ErrorStats) else "n_used"
    addr = ctypes.addressof(stats) + getattr(type(stats), field).offset
    _check(lib().bof4_wait_result(ctypes.c_void_p(addr), _stream(stream)))
    return stats


def bof4_dequantize(codes, scales, n, block, cb, out_idx=None, out_val=None, out=None, stream=None, n_outliers=None):
    """Returns the flat bf16 device tensor of n dequantised weights.  The outlier list is the first n_outliers
    entries of out_idx / out_val (all of them if n_outliers is None)."""
    cb, cbp = _cb(cb)
    if out is None:
        out = torch.empty(n, dtype=torch.bfloat16, device=codes.device)
    k = 0 if out_idx is None else int(out_idx.numel())
    if n_outliers is not None:
        if n_outliers > k:
            raise ValueError("n_outliers exceeds the list")
        k = int(n_outliers)
    _check(lib().bof4_dequantize(_ptr(codes), _ptr(scales), n, block, cbp, _ptr(out_idx) if k else None,
                                 _ptr(out_val) if k else None, k, _ptr(out), _stream(stream)))
    return out
