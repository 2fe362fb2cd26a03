"""bof4_quantize_lloyd (quantiser and Lloyd sums in one pass over the weights) against the CPU oracle: the quantiser's
outputs bit for bit, the sums to the bars of the Lloyd step, on every variant; and in two halves with other work
enqueued between them."""
import numpy as np
import pytest
import torch

import oracle
from paper_2505_06653_amd import binding, codebooks, inputs
from test_gpu_parity import RTOL, assert_stats_close, cb_for, make_weights, to_np_u16

pytestmark = pytest.mark.gpu
DEV = "cuda"


def check_fused(w_cpu, block, cb, signed, T, w2=True, cap_extra=7):
    wb = inputs.bits(w_cpu)
    st, codes, scales, oidx, oval, nout = oracle.quantize(wb, block, cb, signed, opq_T=T)
    assert st == oracle.OK
    st, o = oracle.lloyd_step(wb, block, cb, signed, opq_T=T, weight_by_max2=w2)
    assert st == oracle.OK
    w = w_cpu.to(DEV)
    g_codes, g_scales, g_idx, g_val, g_nout, g = binding.bof4_quantize_lloyd(
        w, block, cb, signed, opq_T=T, out_capacity=max(nout, 1) + cap_extra if T > 0 else 0, weight_by_max2=w2)
    torch.cuda.synchronize()
    assert g_nout == nout
    assert np.array_equal(to_np_u16(g_scales), scales)
    assert np.array_equal(g_codes.cpu().numpy(), codes)
    if T > 0:
        assert np.array_equal(g_idx.cpu().numpy(), oidx)
        assert np.array_equal(to_np_u16(g_val), oval)
    assert_stats_close(g, o)
    return nout


@pytest.mark.parametrize("block", [32, 64, 128, 256])
@pytest.mark.parametrize("signed", [0, 1])
@pytest.mark.parametrize("opq", [0, 1])
@pytest.mark.parametrize("w2", [1, 0])
def test_fused_pass_equals_the_oracle(block, signed, opq, w2):
    # 301 x 1024 weights: several tiles per wave of a small grid, a ragged last tile
    w = make_weights(301, 1024, seed=700 + block)
    T = oracle.opq_threshold(0.95, block) if opq else 0.0
    nout = check_fused(w, block, cb_for(block, signed), signed, T, bool(w2))
    assert (nout > 0) == bool(opq)


@pytest.mark.parametrize("rows", [1, 3, 64, 65])
def test_fused_pass_small_and_ragged(rows):
    """From a single block row up: fewer tiles than waves, tiles whose last lanes lie past the end."""
    w = make_weights(rows, 256, seed=720 + rows, outliers=rows > 3)
    T = oracle.opq_threshold(0.95, 64)
    check_fused(w, 64, cb_for(64, 1), 1, T)
    check_fused(w, 256, cb_for(256, 1), 1, 0.0)


def test_fused_pass_generic_search_and_degenerate_blocks():
    """A codebook whose levels are closer than a bin (the 15-compare search), blocks of zeros, a block of equal large
    numbers but one, a constant that binary16 holds only as a subnormal (division by the IEEE instruction)."""
    w = make_weights(40, 1024, seed=731).clone()
    w[:128] = 0.0
    w[128:192] = 3.0e-6
    w[192:256] = torch.tensor([0.75] * 63 + [0.01]).to(torch.bfloat16)
    w[256:320] = -0.75
    cb = np.array(sorted([-1.0, -0.7, -0.52, -0.5, -0.3, -0.2, -0.1, 0.0, 0.01, 0.02, 0.2, 0.3, 0.5, 0.6, 0.8, 1.0]))
    assert not binding.bof4_bin_table(cb)[2]
    T = oracle.opq_threshold(0.95, 64)
    for cbk in (cb, cb_for(64, 1)):
        check_fused(w, 64, cbk, 1, T)
        check_fused(w, 64, cbk, 0, 0.0)


def test_fused_pass_in_two_halves():
    w_cpu = make_weights(301, 1024, seed=741)
    wb = inputs.bits(w_cpu)
    w = w_cpu.to(DEV)
    n = w.numel()
    cb = cb_for(64, 1)
    T = oracle.opq_threshold(0.95, 64)
    st, codes, scales, oidx, oval, nout = oracle.quantize(wb, 64, cb, 1, opq_T=T)
    st, o = oracle.lloyd_step(wb, 64, cb, 1, opq_T=T)
    cap = nout + 5
    g_codes = torch.empty(n // 2, dtype=torch.uint8, device=DEV)
    g_scales = torch.empty(n // 64, dtype=torch.float16, device=DEV)
    g_idx = torch.empty(cap, dtype=torch.int64, device=DEV)
    g_val = torch.empty(cap, dtype=torch.float16, device=DEV)
    ws = binding.alloc_workspace(n, 64, cap, DEV)
    counter, k1 = binding.pinned_counter()
    stats, k2 = binding.pinned_lloyd_stats()
    flight = binding.bof4_quantize_lloyd_begin(w, 64, cb, 1, T, cap, g_codes, g_scales, g_idx, g_val, ws, counter, stats)
    other = torch.ones(1 << 20, device=DEV).sum()  # unrelated work on the same stream between the halves
    k = flight.finish()
    binding.bof4_wait_result(stats)
    torch.cuda.synchronize()
    assert k == nout and float(other) == float(1 << 20)
    assert np.array_equal(g_codes.cpu().numpy(), codes) and np.array_equal(to_np_u16(g_scales), scales)
    assert np.array_equal(g_idx[:k].cpu().numpy(), oidx) and np.array_equal(to_np_u16(g_val[:k]), oval)
    assert_stats_close(stats.as_dict(), o)
    # a record in ordinary memory cannot be written from the GPU in the background
    with pytest.raises(binding.Bof4Error):
        binding.bof4_quantize_lloyd_begin(w, 64, cb, 1, T, cap, g_codes, g_scales, g_idx, g_val, ws, counter,
                                          binding.LloydStats())


def test_fused_pass_outliers_piled_up_and_capacity_error():
    """All outliers in one stretch overflow a wave's staging region (the extraction is repeated on the general path, the
    sums stay); too small a capacity is an error with the required count."""
    w = make_weights(64, 1024, seed=751, outliers=False).clone()
    w[5000:5000 + 4096:8] = 30.0
    cb = cb_for(64, 1)
    T = oracle.opq_threshold(0.95, 64)
    nout = check_fused(w, 64, cb, 1, T, cap_extra=0)
    assert nout > 300  # far more than the 68 entries of one wave's staging region, all inside two waves
    g = binding.bof4_quantize_lloyd(w.to(DEV), 64, cb, 1, opq_T=T, out_capacity=nout - 1, allow_overflow=True)
    assert g[4] == nout


@pytest.mark.parametrize("block", [32, 64, 256])
def test_fused_pass_tile_with_more_outliers_than_lanes(block):
    """The one-pass call reads an outlier's value again from memory, one lane per outlier of the tile; a tile of 4096
    weights (2048 at block 32) with more than 64 outliers takes the loop that handles them one by one instead.  With a
    capacity large enough for every wave's staging region to hold such a tile, that loop's entries are the result."""
    w = make_weights(301, 1024, seed=761, outliers=False).clone()
    w[3 * 4096 + 5:4 * 4096:40] = 25.0      # 103 outliers in one tile (52 per tile at block 32)
    w[9 * 4096 + 1:10 * 4096:16] = -31.0    # 256 in another (128 per tile at block 32)
    cb = cb_for(block, 1)
    T = oracle.opq_threshold(0.95, block)
    nout = check_fused(w, block, cb, 1, T, cap_extra=1 << 20)
    assert nout >= 103 + 256
