"""A seeded sweep over sizes, block sizes, normalisations, outlier thresholds and input structure that the fixed cases
do not name: every entry point of the hot path against the CPU oracle on the same input, to the bars of the fixed
tests (codes, constants, outlier lists, decoded weights, counts and medians bit for bit; sums to relative 1e-9)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2505_06653_amd import binding, codebooks, inputs
import test_gpu_gemm
import test_gpu_gemv
from test_gpu_error import assert_error_close
from test_gpu_fused import check_fused
from test_gpu_mae import assert_mae_close, mae_cb
from test_gpu_parity import assert_stats_close, cb_for, compare_quantize

import os

pytestmark = pytest.mark.gpu
DEV = "cuda"
# BOF4_SWEEP_SHIFT=<integer> in the environment moves every case of the sweep to other seeds (for a longer hunt than
# the committed cases; the default run is the committed one).
SHIFT = 1000003 * int(os.environ.get("BOF4_SWEEP_SHIFT", "0"))
# BOF4_SWEEP_BIG=<factor> multiplies the sizes of the cases with many tiles (default 1).
BIG = int(os.environ.get("BOF4_SWEEP_BIG", "1"))


def structured_weights(n_blocks, block, shape, rng, g):
    """n_blocks * block float weights of one of five structures."""
    n = n_blocks * block
    if shape == 0:  # Gaussian
        w = torch.randn(n, generator=g) * 0.02
    elif shape == 1:  # heavy tails
        w = torch.randn(n, generator=g) * 0.02 / torch.sqrt(torch.randn(n, 4, generator=g).square().mean(dim=1))
    elif shape == 2:  # block scales spread over many octaves, some blocks all zero
        s = torch.exp2(torch.randint(-30, 12, (n_blocks, 1), generator=g).float())
        s[torch.rand(n_blocks, 1, generator=g) < 0.05] = 0.0
        w = (torch.randn(n_blocks, block, generator=g) * s).reshape(-1)
    elif shape == 3:  # few distinct values: ties in the block maximum, weights on level mid-points
        w = torch.randint(-8, 9, (n,), generator=g).float() * 0.0625
    else:  # the bottom of bfloat16's range (subnormal and smallest normal numbers) next to ordinary blocks
        s = torch.where(torch.rand(n_blocks, 1, generator=g) < 0.5, torch.tensor(2.0 ** -132), torch.tensor(0.02))
        w = (torch.randn(n_blocks, block, generator=g) * s).reshape(-1)
    if rng.random() < 0.5 and n >= 64:  # a pile of large values in one stretch, others spread out
        a = int(rng.integers(0, n - 32))
        w[a:a + int(rng.integers(1, 33))] *= 50.0
        w[torch.randint(0, n, (max(1, n // 500),), generator=g)] *= 30.0
    return w


def sweep_case(k):
    """Case k of the sweep: weights (bf16, flat), block, signed, outlier threshold T, and a word that names it."""
    rng = np.random.default_rng(77000 + k + SHIFT)
    block = int(rng.choice([32, 64, 128, 256]))
    signed = int(rng.integers(0, 2))
    # sizes around the edges the kernels have: a few blocks, just under / over a wave tile (64 segments of up to 64
    # weights), several tiles with a ragged tail, more tiles than the grid has waves
    kind = int(rng.integers(0, 5))
    seg = min(block, 64)
    tile_blocks = 64 * seg // block
    n_blocks = [int(rng.integers(1, 9)), tile_blocks - 1 + int(rng.integers(0, 3)),
                int(rng.integers(2, 40)) * tile_blocks + int(rng.integers(0, tile_blocks)),
                4096 * 4 * tile_blocks // 16 + int(rng.integers(0, 3 * tile_blocks)),
                int(rng.integers(1, 3000))][kind]
    if kind >= 2:
        n_blocks = n_blocks * BIG + (BIG - 1) * int(rng.integers(0, 7))
    n = n_blocks * block
    g = torch.Generator().manual_seed(88000 + k + SHIFT)
    shape = int(rng.integers(0, 5))
    w = structured_weights(n_blocks, block, shape, rng, g)
    T = 0.0 if rng.random() < 0.35 else float(oracle.opq_threshold(float(rng.choice([0.2, 0.5, 0.9, 0.95, 0.99])), block))
    return w.to(torch.bfloat16), block, signed, T, f"block {block} signed {signed} n {n} kind {kind} shape {shape} T {T:.3f}"


@pytest.mark.parametrize("k", range(80))
def test_sweep_quantize_dequantize_lloyd_fused(k):
    w, block, signed, T, name = sweep_case(k)
    print(name, flush=True)
    cb = cb_for(block, signed)
    compare_quantize(w, block, cb, signed, T)
    if float(w.float().abs().max()) > 65504.0:
        return  # some block constant is infinite in binary16: the sums are out of contract (not finite either way)
    w2 = k % 3 != 0  # every third case: the sums of the normalised error (appendix D) instead of eq. 6's
    st, o = oracle.lloyd_step(inputs.bits(w), block, cb, signed, opq_T=T, weight_by_max2=w2)
    assert st == oracle.OK
    assert_stats_close(binding.bof4_lloyd_step(w.to(DEV), block, cb, signed, opq_T=T, weight_by_max2=w2), o)
    check_fused(w, block, cb, signed, T, w2=w2, cap_extra=int(k % 5))


@pytest.mark.parametrize("k", range(80, 120))
def test_sweep_mae_step(k):
    w, block, signed, T, name = sweep_case(k)
    print(name, flush=True)
    cb = mae_cb(block, signed)
    weighted = bool(k % 2)
    if float(w.float().abs().max()) > 65504.0:
        w = w.float().clamp(-6.0e4, 6.0e4).to(torch.bfloat16)  # keep the block constants finite in binary16
    st, o = oracle.lloyd_step_mae(inputs.bits(w), block, cb, signed, opq_T=T, weight_by_max=weighted)
    if st != oracle.OK:  # block constants too large for exact 64-bit sums: the library must refuse as well
        with pytest.raises(binding.Bof4Error):
            binding.bof4_lloyd_step_mae(w.to(DEV), block, cb, signed, opq_T=T, weight_by_max=weighted)
        return
    assert_mae_close(binding.bof4_lloyd_step_mae(w.to(DEV), block, cb, signed, opq_T=T, weight_by_max=weighted), o)
    skip = int(np.random.default_rng(66000 + k + SHIFT).integers(1, 1 << 16))  # medians of some regions not wanted
    got = binding.bof4_lloyd_step_mae(w.to(DEV), block, cb, signed, opq_T=T, weight_by_max=weighted, skip_mask=skip)
    wanted = np.array([not ((skip >> l) & 1) for l in range(16)])
    assert np.array_equal(got["median"][wanted], o["median"][wanted], equal_nan=True)
    assert np.all(np.isnan(got["median"][~wanted]))
    assert np.array_equal(got["den"], o["den"]) and np.array_equal(got["cnt"], o["cnt"])


@pytest.mark.parametrize("k", range(120, 150))
def test_sweep_error_pass(k):
    w, block, signed, T, name = sweep_case(k)
    print(name, flush=True)
    if float(w.float().abs().max()) > 65504.0:
        w = w.float().clamp(-6.0e4, 6.0e4).to(torch.bfloat16)  # keep the block constants finite in binary16
    cb = cb_for(block, signed)
    st, o = oracle.quant_error(inputs.bits(w), block, cb, signed, T)
    assert st == oracle.OK
    assert_error_close(binding.bof4_quant_error(w.to(DEV), block, cb, signed, opq_T=T), o)


@pytest.mark.parametrize("k", range(150, 180))
def test_sweep_decoder_inside_the_matrix_products(k):
    """bof4_gemv and bof4_gemm on matrices of the sweep's structures (codes, constants and list from the oracle's
    quantiser), random shapes and token counts, to the error bounds of their own test files."""
    rng = np.random.default_rng(99000 + k + SHIFT)
    block = int(rng.choice([32, 64, 128, 256]))
    signed = int(rng.integers(0, 2))
    cols = block * int(rng.integers(1, max(2, min(32768 // block, 8192 // block) + 1)))
    rows = int(rng.integers(1, 1 + max(1, min(300, 600000 // cols))))
    shape = int(rng.integers(0, 5))
    g = torch.Generator().manual_seed(99500 + k + SHIFT)
    w = structured_weights(rows * cols // block, block, shape, rng, g).clamp(-6.0e4, 6.0e4).to(torch.bfloat16)
    T = 0.0 if rng.random() < 0.4 else float(oracle.opq_threshold(float(rng.choice([0.5, 0.95])), block))
    print(f"block {block} signed {signed} rows {rows} cols {cols} shape {shape} T {T:.3f}", flush=True)
    cb = cb_for(block, signed) if k % 2 else random_codebook(rng)
    st, codes, scales, oi, ov, n_out = oracle.quantize(inputs.bits(w), block, cb, signed, opq_T=T)
    assert st == oracle.OK
    lst = (oi, ov) if n_out > 0 else (None, None)
    xg = torch.Generator().manual_seed(99900 + k + SHIFT)
    x1 = torch.randn((int(rng.integers(1, 6)), cols), generator=xg).to(torch.bfloat16)
    test_gpu_gemv.check(cb, codes, scales, lst[0], lst[1], rows, cols, block, x1)
    x2 = torch.randn((int(rng.choice([1, 31, 32, 33, 64, 100, 128, 129, 200])), cols), generator=xg).to(torch.bfloat16)
    test_gpu_gemm.check(cb, codes, scales, lst[0], lst[1], rows, cols, block, x2)


def random_codebook(rng):
    """16 ascending levels that are not the paper's: anywhere in [-1.2, 1.2], with or without a zero, sometimes with
    two levels closer together than a bin of the kernels' search table is wide (that switches them to the general
    search), sometimes with the outermost levels at -1 and 1."""
    lv = np.sort(rng.uniform(-1.2, 1.2, 16))
    if rng.random() < 0.5:
        lv[int(np.argmin(np.abs(lv)))] = 0.0
    if rng.random() < 0.5:
        lv[0], lv[15] = -1.0, 1.0
    if rng.random() < 0.4:
        j = int(rng.integers(1, 14))
        lv[j + 1] = lv[j] + rng.uniform(1e-4, 4e-3)
    lv = np.sort(lv)
    for j in range(1, 16):  # strictly ascending
        if lv[j] <= lv[j - 1]:
            lv[j] = np.nextafter(lv[j - 1], 2.0)
    return lv.astype(np.float64)


@pytest.mark.parametrize("k", range(180, 230))
def test_sweep_other_codebooks(k):
    w, block, signed, T, name = sweep_case(k)
    if float(w.float().abs().max()) > 65504.0:
        w = w.float().clamp(-6.0e4, 6.0e4).to(torch.bfloat16)  # keep the block constants finite in binary16
    cb = random_codebook(np.random.default_rng(55000 + k + SHIFT))
    print(name, " ".join(f"{v:.5f}" for v in cb), flush=True)
    wb = inputs.bits(w)
    compare_quantize(w, block, cb, signed, T)
    check_fused(w, block, cb, signed, T, w2=bool(k % 2))
    st, o = oracle.lloyd_step_mae(wb, block, cb, signed, opq_T=T)
    assert st == oracle.OK
    assert_mae_close(binding.bof4_lloyd_step_mae(w.to(DEV), block, cb, signed, opq_T=T), o)
    st, e = oracle.quant_error(wb, block, cb, signed, T)
    assert st == oracle.OK
    assert_error_close(binding.bof4_quant_error(w.to(DEV), block, cb, signed, opq_T=T), e)


@pytest.mark.parametrize("shape,signed,T_q", [(2, 1, 0.0), (3, 0, 0.0), (3, 1, 0.95), (1, 0, 0.9)])
def test_mae_one_pass_search_on_structured_weights(shape, signed, T_q):
    """The sampled one-pass search of the MAE step (from 2^26 weights) on inputs whose keys do not spread like a
    Gaussian's: block scales over 42 octaves (most blocks' constants below or near binary16's normal range), 17
    distinct values (a region's elements share a handful of keys, so a window takes in all of them and the list runs
    full: the step must fall back to scanning), heavy tails.  Whichever way it goes, the medians are the oracle's."""
    block = 64
    n_blocks = (16384 + 9) * 64 + 3
    rng = np.random.default_rng(4711 + shape)
    w = structured_weights(n_blocks, block, shape, rng, torch.Generator().manual_seed(4712 + shape))
    w = w.clamp(-6.0e4, 6.0e4).to(torch.bfloat16)
    T = float(oracle.opq_threshold(T_q, block)) if T_q else 0.0
    cb = mae_cb(block, signed)
    pin = codebooks.PIN_BOF4S if signed else codebooks.PIN_BOF4
    st, o = oracle.lloyd_step_mae(inputs.bits(w), block, cb, signed, opq_T=T)
    assert st == oracle.OK
    got = binding.bof4_lloyd_step_mae(w.to(DEV), block, cb, signed, opq_T=T, skip_mask=pin)
    wanted = np.array([not ((pin >> l) & 1) for l in range(16)])
    assert np.array_equal(got["median"][wanted], o["median"][wanted], equal_nan=True)
    assert np.array_equal(got["den"], o["den"]) and np.array_equal(got["cnt"], o["cnt"])
    assert got["n_used"] == o["n_used"] and got["n_outliers"] == o["n_outliers"]
    assert abs(got["sae"] - o["sae"]) <= 1e-9 * o["sae"]


@pytest.mark.parametrize("k", range(230, 254))
def test_sweep_theory_centroids(k):
    """The general centroid of section 3.2 eq. 5 on the GPU for weight distributions that are mixtures of zero-mean
    Gaussians of random widths (even densities, as the recipe requires), random grids, block sizes, both
    normalisations and codebooks around the paper's: every level as the oracle's evaluation of the same recipe."""
    from scipy.special import ndtr
    from oracle import theory_general
    rng = np.random.default_rng(31000 + k + SHIFT)
    sig = rng.uniform(0.3, 3.0, int(rng.integers(1, 4)))
    wt = rng.dirichlet(np.ones(sig.size))
    pdf_f = lambda u: sum(a * np.exp(-0.5 * (u / s) ** 2) / (s * np.sqrt(2.0 * np.pi)) for a, s in zip(wt, sig))
    cdf_f = lambda u: sum(a * ndtr(u / s) for a, s in zip(wt, sig))
    u_max = float(rng.uniform(6.0, 14.0) * sig.max())
    n_grid = 2 * int(rng.integers(200, 40000)) + 1
    pdf, cdf = theory_general.tables(pdf_f, cdf_f, u_max, n_grid)
    block = int(rng.choice([32, 64, 128, 256]))
    signed = int(rng.integers(0, 2))
    pin = codebooks.PIN_BOF4S if signed else codebooks.PIN_BOF4
    cb = (codebooks.array(codebooks.BOF4S_MSE[block]) if signed else codebooks.array(codebooks.BOF4_MSE_64)).copy()
    free = np.array([not ((pin >> l) & 1) for l in range(16)])
    cb[free] = np.sort(cb[free] + rng.uniform(-0.02, 0.02, int(free.sum())))  # stays ascending between the pins
    assert np.all(np.diff(cb) > 0)
    print(f"block {block} signed {signed} grid {n_grid} u_max {u_max:.2f} widths {sig}", flush=True)
    want = theory_general.centroid_update(cb, block, pin, signed, pdf, cdf, u_max)
    got = binding.bof4_theory_centroids(pdf, cdf, u_max, block, cb, pin, signed)
    assert np.all(np.abs(got - want) <= 1e-10 * np.maximum(np.abs(want), 1e-3))


@pytest.mark.parametrize("shape,block,signed,T_q", [(2, 64, 1, 0.9), (1, 128, 0, 0.9), (4, 32, 1, 0.95)])
def test_quantiser_chain_on_large_structured_tensors(shape, block, signed, T_q):
    """Quantiser, decoder and the one-pass variant at 2^26 weights (every wave of the persistent grids busy for many
    tiles, outlier lists of 10^5 to 10^6 entries) on the sweep's less ordinary structures: outputs as the oracle's."""
    n_blocks = (1 << 26) // block + 7
    rng = np.random.default_rng(5200 + shape)
    w = structured_weights(n_blocks, block, shape, rng, torch.Generator().manual_seed(5201 + shape))
    w = w.clamp(-6.0e4, 6.0e4).to(torch.bfloat16)
    T = float(oracle.opq_threshold(T_q, block))
    cb = cb_for(block, signed)
    nout = compare_quantize(w, block, cb, signed, T)
    print(f"shape {shape} block {block}: {nout} outliers", flush=True)
    check_fused(w, block, cb, signed, T)
