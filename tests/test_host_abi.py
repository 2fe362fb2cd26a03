"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol, and its pure host functions and
argument validation behave as the header says.  No compute call is made (no GPU here)."""
import ctypes
import os
import re

import numpy as np
import pytest
from scipy.stats import norm

import oracle
from paper_2505_06653_amd import binding, codebooks

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CB = codebooks.array(codebooks.BOF4S_MSE[64])


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "bof4.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(bof4_[a-z0-9_]+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    L = binding.lib()
    syms = declared_symbols()
    assert set(syms) == set(binding.EXPORTS)
    for s in syms:
        assert hasattr(L, s), s


def test_thresholds_are_round_down_midpoints():
    rng = np.random.default_rng(0)
    for cb in (CB, codebooks.array(codebooks.BOF4_MSE_64), np.sort(rng.uniform(-1, 1, 16))):
        thr = binding.bof4_thresholds(cb)
        mid = 0.5 * (cb[:-1] + cb[1:])
        assert np.all(thr.astype(np.float64) <= mid)
        assert np.all(np.nextafter(thr, np.float32(np.inf)).astype(np.float64) > mid)
        # for every binary32 x around a threshold the kernel's compare equals the binary64 mid-point compare
        for k in range(15):
            x = thr[k]
            for _ in range(4):
                x = np.nextafter(x, np.float32(-np.inf))
            for _ in range(9):
                assert (x > thr[k]) == (float(x) > mid[k])
                x = np.nextafter(x, np.float32(np.inf))


def test_opq_threshold_matches_closed_form_and_oracle():
    for block in (32, 64, 128, 256):
        for q in (0.9, 0.95, 0.97, 0.99):
            t = binding.bof4_opq_threshold(q, block)
            assert abs(t - norm.ppf((1 + q ** (1.0 / block)) / 2)) < 1e-10
            assert abs(t - oracle.opq_threshold(q, block)) < 1e-11
    assert np.isnan(binding.bof4_opq_threshold(1.5, 64))


def test_codebook_update_matches_oracle_and_respects_pins():
    rng = np.random.default_rng(1)
    stats = {"num": rng.standard_normal(16), "den": rng.uniform(0.5, 2, 16), "cnt": rng.integers(1, 100, 16),
             "sse": 1.0, "n_used": 100, "n_outliers": 0}
    stats["den"][3] = 0.0  # empty region keeps its level
    for mask in (0, codebooks.PIN_BOF4, codebooks.PIN_BOF4S, 0xFFFF):
        got = binding.bof4_codebook_update(stats, mask, CB)
        assert np.array_equal(got, oracle.codebook_update(stats, mask, CB))
        for l in range(16):
            if (mask >> l) & 1 or l == 3:
                assert got[l] == CB[l]
            else:
                assert got[l] == stats["num"][l] / stats["den"][l]


def test_workspace_bytes():
    assert binding.bof4_workspace_bytes(0, 64) == 0
    assert binding.bof4_workspace_bytes(100, 64) == 0
    assert binding.bof4_workspace_bytes(1 << 20, 48) == 0
    small = binding.bof4_workspace_bytes(1 << 20, 64, 0)
    big = binding.bof4_workspace_bytes(1 << 30, 64, 1 << 24)
    assert small > 0 and big > small and big >= (1 << 24) * 10


def test_argument_validation_returns_error_codes_without_touching_the_gpu():
    L = binding.lib()
    cbp = CB.ctypes.data_as(ctypes.POINTER(ctypes.c_double))
    bad_cb = CB[::-1].copy()
    bad_cbp = bad_cb.ctypes.data_as(ctypes.POINTER(ctypes.c_double))
    nout = ctypes.c_uint64(0)
    fake, odd = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x1002)
    q = lambda w, n, blk, c, T, codes, scales: L.bof4_quantize(w, n, blk, c, 1, T, codes, scales, None, None, 0,
                                                                ctypes.byref(nout), None, 0, None)
    assert q(None, 1024, 64, cbp, 0.0, fake, fake) == binding.BOF4_ERR_ARG        # null weights
    assert q(fake, 1000, 64, cbp, 0.0, fake, fake) == binding.BOF4_ERR_ARG        # n not a multiple of block
    assert q(fake, 0, 64, cbp, 0.0, fake, fake) == binding.BOF4_ERR_ARG           # empty input
    assert q(fake, 1024, 48, cbp, 0.0, fake, fake) == binding.BOF4_ERR_ARG        # unsupported block size
    assert q(fake, 1024, 64, bad_cbp, 0.0, fake, fake) == binding.BOF4_ERR_ARG    # unsorted codebook
    assert q(fake, 1024, 64, cbp, -1.0, fake, fake) == binding.BOF4_ERR_ARG       # negative threshold
    assert q(odd, 1024, 64, cbp, 0.0, fake, fake) == binding.BOF4_ERR_ARG         # misaligned weights
    assert q(fake, 1024, 64, cbp, 3.0, fake, fake) == binding.BOF4_ERR_ARG        # OPQ without workspace
    assert b"workspace" in L.bof4_last_error()
    st = binding.LloydStats()
    assert L.bof4_lloyd_step(fake, 1024, 64, cbp, 1, 0.0, 1, ctypes.byref(st), ctypes.c_void_p(0x1010), 1 << 30, None) == binding.BOF4_ERR_ARG
    ws = ctypes.c_void_p(0x10000)
    assert L.bof4_lloyd_step(fake, 1024, 64, cbp, 1, 0.0, 1, ctypes.byref(st), ws, 16, None) == binding.BOF4_ERR_WORKSPACE
    assert L.bof4_dequantize(fake, fake, 1024, 64, cbp, None, None, 5, fake, None) == binding.BOF4_ERR_ARG
    assert L.bof4_dequantize(fake, fake, 1024, 64, bad_cbp, None, None, 0, fake, None) == binding.BOF4_ERR_ARG
    nan_cb = CB.copy()
    nan_cb[4] = np.nan
    assert L.bof4_thresholds(nan_cb.ctypes.data_as(ctypes.POINTER(ctypes.c_double)),
                             (ctypes.c_float * 15)()) == binding.BOF4_ERR_ARG


def test_argument_validation_of_the_later_entry_points_without_touching_the_gpu():
    """bof4_lloyd_step_mae, bof4_quant_error, bof4_gemv and bof4_gemv_outlier_table refuse bad arguments before any
    GPU call; the table size is a host formula."""
    L = binding.lib()
    cbp = CB.ctypes.data_as(ctypes.POINTER(ctypes.c_double))
    bad_cb = CB[::-1].copy()
    bad_cbp = bad_cb.ctypes.data_as(ctypes.POINTER(ctypes.c_double))
    fake, odd, ws = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x1004), ctypes.c_void_p(0x10000)
    ms, es = binding.MaeStats(), binding.ErrorStats()
    assert L.bof4_lloyd_step_mae(fake, 1000, 64, cbp, 1, 0.0, 1, 0, ctypes.byref(ms), ws, 1 << 30, None) == binding.BOF4_ERR_ARG
    assert L.bof4_lloyd_step_mae(fake, 1024, 64, bad_cbp, 1, 0.0, 1, 0, ctypes.byref(ms), ws, 1 << 30, None) == binding.BOF4_ERR_ARG
    assert L.bof4_lloyd_step_mae(fake, 1024, 64, cbp, 1, 0.0, 0, 0, ctypes.byref(ms), ws, 64, None) == binding.BOF4_ERR_WORKSPACE
    assert L.bof4_quant_error(fake, 1024, 48, cbp, 1, 0.0, ctypes.byref(es), ws, 1 << 30, None) == binding.BOF4_ERR_ARG
    assert L.bof4_quant_error(fake, 1024, 64, cbp, 1, -2.0, ctypes.byref(es), ws, 1 << 30, None) == binding.BOF4_ERR_ARG
    assert L.bof4_quant_error(fake, 1024, 64, cbp, 1, 0.0, ctypes.byref(es), ws, 64, None) == binding.BOF4_ERR_WORKSPACE
    g = lambda codes, rows, cols, blk, c, table, k, x, nt: L.bof4_gemv(codes, fake, rows, cols, blk, c, table, k, x, nt, fake, None)
    assert g(None, 4, 128, 64, cbp, None, 0, fake, 1) == binding.BOF4_ERR_ARG        # null codes
    assert g(fake, 4, 96, 64, cbp, None, 0, fake, 1) == binding.BOF4_ERR_ARG         # cols not a multiple of block
    assert g(fake, 4, 128, 64, cbp, None, 0, fake, 0) == binding.BOF4_ERR_ARG        # no tokens
    assert g(fake, 4, 128, 64, bad_cbp, None, 0, fake, 1) == binding.BOF4_ERR_ARG    # unsorted codebook
    assert g(fake, 4, 128, 64, cbp, None, 3, fake, 1) == binding.BOF4_ERR_ARG        # outliers without their table
    assert g(odd, 4, 128, 64, cbp, None, 0, fake, 1) == binding.BOF4_ERR_ARG         # codes not 16-byte aligned
    assert g(fake, 4, 32768 + 64, 64, cbp, None, 0, fake, 1) == binding.BOF4_ERR_ARG  # too wide
    assert b"32768" in L.bof4_last_error()
    t = lambda rows, cols, k, tab, nbytes: L.bof4_gemv_outlier_table(fake, fake, rows, cols, 64, cbp, fake, fake, k, tab, nbytes, None)
    need = binding.bof4_gemv_outlier_table_bytes(10, 4096 + 64, 7)
    assert need == (10 * 3 + 1 + 1) // 2 * 8 + 7 * 8 and binding.bof4_gemv_outlier_table_bytes(0, 64, 0) == 0
    assert t(10, 4096 + 64, 7, ws, need - 8) == binding.BOF4_ERR_WORKSPACE
    assert t(10, 4096 + 32, 7, ws, need) == binding.BOF4_ERR_ARG
    assert t(10, 4096 + 64, 7, None, need) == binding.BOF4_ERR_ARG


def test_argument_validation_and_size_formulas_of_the_matrix_product_without_touching_the_gpu():
    """bof4_gemm, bof4_gemm_pack and bof4_gemm_outlier_table refuse bad arguments before any GPU call; the sizes of the
    packed matrix and of the workspace are host formulas."""
    L = binding.lib()
    cbp = CB.ctypes.data_as(ctypes.POINTER(ctypes.c_double))
    bad_cb = CB[::-1].copy()
    bad_cbp = bad_cb.ctypes.data_as(ctypes.POINTER(ctypes.c_double))
    fake, odd, ws = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x1004), ctypes.c_void_p(0x10000)
    # tiles of 32 rows (an even number of them) x chunks of 64 columns, 1024 bytes of codes + 64 constants each
    assert binding.bof4_gemm_packed_bytes(64, 128) == 2 * 2 * 1152
    assert binding.bof4_gemm_packed_bytes(65, 96) == 4 * 2 * 1152
    assert binding.bof4_gemm_packed_bytes(4096, 11008) == 128 * 172 * 1152
    # x twice, token slots in 32s; partial results only where the rows alone do not give 192 workgroups
    assert binding.bof4_gemm_workspace_bytes(32768, 4096, 7) == 2 * 32 * 4096 * 2
    assert binding.bof4_gemm_workspace_bytes(4096, 4096, 40) == 2 * 64 * 4096 * 2 + 2 * 64 * 4096 * 4
    assert binding.bof4_gemm_workspace_bytes(0, 64, 1) == 0
    pk = lambda codes, rows, cols, blk, out, nbytes: L.bof4_gemm_pack(codes, fake, rows, cols, blk, out, nbytes, None)
    assert pk(None, 64, 128, 64, ws, 1 << 20) == binding.BOF4_ERR_ARG
    assert pk(fake, 64, 96, 64, ws, 1 << 20) == binding.BOF4_ERR_ARG          # cols not a multiple of block
    assert pk(odd, 64, 128, 64, ws, 1 << 20) == binding.BOF4_ERR_ARG           # codes not 16-byte aligned
    assert pk(fake, 64, 128, 64, ws, 4 * 1152 - 1) == binding.BOF4_ERR_WORKSPACE
    assert pk(fake, 64, 32768 + 64, 64, ws, 1 << 30) == binding.BOF4_ERR_ARG
    g = lambda packed, rows, cols, c, table, k, x, nt, w, wb: L.bof4_gemm(packed, rows, cols, c, table, k, x, nt, fake,
                                                                           w, wb, None)
    assert g(None, 64, 128, cbp, None, 0, fake, 1, ws, 1 << 20) == binding.BOF4_ERR_ARG
    assert g(fake, 64, 80, cbp, None, 0, fake, 1, ws, 1 << 20) == binding.BOF4_ERR_ARG      # cols not a multiple of 32
    assert g(fake, 64, 128, cbp, None, 0, fake, 0, ws, 1 << 20) == binding.BOF4_ERR_ARG     # no tokens
    assert g(fake, 64, 128, bad_cbp, None, 0, fake, 1, ws, 1 << 20) == binding.BOF4_ERR_ARG
    assert g(fake, 64, 128, cbp, None, 3, fake, 1, ws, 1 << 20) == binding.BOF4_ERR_ARG     # outliers without table
    assert g(odd, 64, 128, cbp, None, 0, fake, 1, ws, 1 << 20) == binding.BOF4_ERR_ARG      # misaligned
    assert g(fake, 64, 128, cbp, None, 0, fake, 1, None, 1 << 20) == binding.BOF4_ERR_ARG   # no workspace
    assert g(fake, 64, 128, cbp, None, 0, fake, 1, ws, 100) == binding.BOF4_ERR_WORKSPACE
    assert g(fake, 64, 128, cbp, None, 0, fake, 70000, ws, 1 << 40) == binding.BOF4_ERR_ARG  # too many tokens
    t = lambda rows, cols, k, tab, nbytes: L.bof4_gemm_outlier_table(fake, fake, rows, cols, 64, cbp, fake, fake, k, tab, nbytes, None)
    need = binding.bof4_gemv_outlier_table_bytes(10, 4096 + 64, 7)
    assert t(10, 4096 + 64, 7, ws, need - 8) == binding.BOF4_ERR_WORKSPACE
    assert t(10, 4096 + 32, 7, ws, need) == binding.BOF4_ERR_ARG
