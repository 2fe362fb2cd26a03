"""bof4_lloyd_step_static (the entry point that allocates nothing: partial sums in the library's own device array)
against bof4_lloyd_step on the same inputs, through the C ABI.  Same kernels, same grid, same order of additions:
every field must be equal bit for bit (counts exact, sums identical), which is stricter than the 1e-9 of the parity
tests.  Two calls in a row share the array; the second is smaller, so records of the first are still lying there."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2505_06653_amd import binding, codebooks, inputs

pytestmark = pytest.mark.gpu


def _same(a, b):
    for f in ("num", "den"):
        assert np.array_equal(np.array(getattr(a, f)[:]).view(np.uint64), np.array(getattr(b, f)[:]).view(np.uint64)), f
    assert list(a.cnt[:]) == list(b.cnt[:])
    assert np.float64(a.sse).view(np.uint64) == np.float64(b.sse).view(np.uint64)
    assert (a.n_used, a.n_outliers) == (b.n_used, b.n_outliers)


def test_static_entry_point_two_calls_second_smaller():
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    cb = codebooks.array(codebooks.BOF4S_MSE[64])
    T = binding.bof4_opq_threshold(0.95, 64)
    big = inputs.student_t_matrix(3072, 4096, 5.0, 0.02, 0.3, seed=901, device=dev).reshape(-1)  # fills the whole grid
    small = inputs.student_t_matrix(24, 1088, 4.0, 0.015, 0.0, seed=902, device=dev).reshape(-1)  # a few workgroups
    rec, keep = binding.pinned_lloyd_stats()
    for w, block, opq_T in ((big, 64, T), (small, 64, T), (big, 128, 0.0), (small, 32, 0.0)):
        ref = binding.bof4_lloyd_step(w, block, cb, 1, opq_T=opq_T, raw=True)
        ctypes.memset(ctypes.addressof(rec), 0xEE, ctypes.sizeof(rec))
        got = binding.bof4_lloyd_step_static(w, block, cb, 1, rec, opq_T=opq_T)
        assert got.n_used + got.n_outliers == w.numel()
        _same(got, ref)


def test_static_entry_point_rejects():
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    cb = codebooks.array(codebooks.BOF4S_MSE[64])
    w = torch.zeros(4096, dtype=torch.bfloat16, device=dev)
    rec, keep = binding.pinned_lloyd_stats()
    with pytest.raises(binding.Bof4Error) as e:  # beyond the stated maximum: refused before anything is launched
        binding.bof4_lloyd_step_static(w, 64, cb, 1, rec, n=(1 << 36) + 64)
    assert e.value.code == binding.BOF4_ERR_ARG and "BOF4_STATIC_MAX_N" in str(e.value)
    with pytest.raises(binding.Bof4Error) as e:  # a record in ordinary memory would need a copy
        binding.bof4_lloyd_step_static(w, 64, cb, 1, binding.LloydStats())
    assert e.value.code == binding.BOF4_ERR_ARG


@pytest.mark.parametrize("k", range(254, 270))
def test_static_entry_point_on_the_sweeps_inputs(k):
    """The same comparison on inputs of the seeded sweep (tests/test_gpu_random_sweep.py): sizes around the tile
    edges, all block sizes, both normalisations, with and without the outlier rule, both weightings."""
    from test_gpu_parity import cb_for
    from test_gpu_random_sweep import sweep_case
    w, block, signed, T, name = sweep_case(k)
    if float(w.float().abs().max()) > 65504.0:
        w = w.float().clamp(-6.0e4, 6.0e4).to(torch.bfloat16)
    print(name, flush=True)
    cb = cb_for(block, signed)
    wd = w.to("cuda:0")
    rec, keep = binding.pinned_lloyd_stats()
    w2 = bool(k % 2)
    ref = binding.bof4_lloyd_step(wd, block, cb, signed, opq_T=T, weight_by_max2=w2, raw=True)
    ctypes.memset(ctypes.addressof(rec), 0xEE, ctypes.sizeof(rec))
    got = binding.bof4_lloyd_step_static(wd, block, cb, signed, rec, opq_T=T, weight_by_max2=w2)
    _same(got, ref)
