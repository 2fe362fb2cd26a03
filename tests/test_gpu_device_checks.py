"""Exhaustive GPU checks of the kernels' arithmetic shortcuts against the plain definitions they replace."""
import ctypes
import os

import numpy as np
import pytest
import torch

from paper_2505_06653_amd import binding, codebooks

pytestmark = pytest.mark.gpu
HERE = os.path.dirname(os.path.abspath(__file__))


def run_check(cb):
    path = os.path.join(HERE, "libbof4_device_checks.so")
    assert os.path.exists(path), "run `python tests/build_checks.py` first"
    L = ctypes.CDLL(path)
    thr = binding.bof4_thresholds(cb)
    bthr, bbase, fast = binding.bof4_bin_table(cb)
    assert fast
    lv = cb.astype(np.float32)
    out = torch.zeros(8, dtype=torch.int64, device="cuda")
    fp = ctypes.POINTER(ctypes.c_float)
    rc = L.bof4_check_pairs(thr.ctypes.data_as(fp), lv.ctypes.data_as(fp), bthr.ctypes.data_as(fp),
                            bbase.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32)), ctypes.c_void_p(out.data_ptr()),
                            ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == 0
    torch.cuda.synchronize()
    return out.cpu().numpy()


@pytest.mark.parametrize("name", ["bof4s_32", "bof4s_64", "bof4s_128", "bof4s_256", "bof4_mse", "bof4_mae", "init"])
def test_shortcut_division_and_bin_table_equal_the_plain_definitions(name):
    """Every (block constant, weight) pair that can reach the shortcut path: all bfloat16 constants inside binary16's
    normal range, both signs, times all bfloat16 weights not larger in magnitude (about 0.5e9 pairs)."""
    cb = {"bof4s_32": codebooks.array(codebooks.BOF4S_MSE[32]), "bof4s_64": codebooks.array(codebooks.BOF4S_MSE[64]),
          "bof4s_128": codebooks.array(codebooks.BOF4S_MSE[128]), "bof4s_256": codebooks.array(codebooks.BOF4S_MSE[256]),
          "bof4_mse": codebooks.array(codebooks.BOF4_MSE_64), "bof4_mae": codebooks.array(codebooks.BOF4_MAE_64),
          "init": codebooks.gaussian_quantile_init()}[name]
    bad_q, bad_tiny, bad_code, bad_range, n = run_check(cb)[:5]
    assert n > 200_000_000
    assert bad_q == 0            # correctly rounded quotient for every |w| >= 2^-60 (and w = 0)
    assert bad_range == 0        # |x| <= 1 always
    assert bad_code == 0         # same level as the 15-compare search on the IEEE quotient, tiny weights included
    print(f"{name}: {n} pairs, quotient differs for {bad_tiny} weights below 2^-60 (codes equal)")


def test_dot2_error_stays_inside_the_allowance_of_the_opq_statistics():
    """The approximate OPQ statistics allow DOT2_ROUNDINGS (= 6) * 2^-24 * (|a.lo b.lo| + |a.hi b.hi| + |c|) of error
    per v_dot2c_f32_bf16; the instruction's measured error (3.0 at worst, as of three truncations) must stay
    well below that."""
    L = ctypes.CDLL(os.path.join(HERE, "libbof4_device_checks.so"))
    L.bof4_check_dot2.argtypes = [ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint32, ctypes.c_void_p, ctypes.c_void_p]
    out = torch.zeros(8, dtype=torch.int64, device="cuda")
    rc = L.bof4_check_dot2(20250506653, 4096, 256, ctypes.c_void_p(out.data_ptr()),
                           ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == 0
    torch.cuda.synchronize()
    o = out.cpu().numpy()
    ratios = o[:4].view(np.float64)
    print("dot2 error / (2^-24 * sum of magnitudes), worst per regime:", ratios, "samples", o[4:])
    assert o[4:].sum() == 4096 * 256 * 256 and (o[4:] > 10_000_000).all()
    assert (ratios <= 3.5).all()


def test_wave_prefix_sum_with_dpp_moves_equals_the_serial_sum():
    L = ctypes.CDLL(os.path.join(HERE, "libbof4_device_checks.so"))
    L.bof4_check_scan.argtypes = [ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint32, ctypes.c_void_p, ctypes.c_void_p]
    out = torch.zeros(2, dtype=torch.int64, device="cuda")
    rc = L.bof4_check_scan(7, 512, 64, ctypes.c_void_p(out.data_ptr()),
                           ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == 0
    torch.cuda.synchronize()
    bad, n = out.cpu().numpy()
    assert n == 512 * 256 * 64 and bad == 0


def test_packed_binary16_maximum_orders_bfloat16_patterns_like_their_values():
    """The block-maximum search takes the largest and smallest of packed 16-bit patterns with the three-operand
    binary16 maximum / minimum: on all 2^32 pairs of patterns it must pick by sign and magnitude (+0 above -0,
    subnormal patterns not flushed) and turn every pair with a binary16 NaN pattern into a NaN pattern."""
    L = ctypes.CDLL(os.path.join(HERE, "libbof4_device_checks.so"))
    L.bof4_check_pkmax.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
    out = torch.zeros(4, dtype=torch.int64, device="cuda")
    rc = L.bof4_check_pkmax(ctypes.c_void_p(out.data_ptr()), ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == 0
    torch.cuda.synchronize()
    bad_max, bad_min, bad_nan, n = out.cpu().numpy()
    assert n == 1 << 32
    assert bad_max == 0 and bad_min == 0 and bad_nan == 0
