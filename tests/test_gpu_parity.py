"""GPU parity: the HIP library (called through its C ABI) against the CPU oracle, element by element, on seeded
inputs small enough for the oracle yet spanning several tiles and a ragged last tile.

Bars: codes, scales, outlier lists, dequantised bf16 and Lloyd counts bit-exact; Lloyd sums, updated levels and
MSE within relative 1e-9 (binary64 sums whose terms are exact products, added in a different order)."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from paper_2505_06653_amd import binding, codebooks, inputs

pytestmark = pytest.mark.gpu
DEV = "cuda"
RTOL = 1e-9


def cb_for(block, signed):
    if signed:
        return codebooks.array(codebooks.BOF4S_MSE[block])
    return codebooks.array(codebooks.BOF4_MSE_64)


def to_np_u16(t):
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def make_weights(rows, cols, seed, outliers=True):
    wm = inputs.student_t_matrix(rows, cols, 5.0, 0.02, 0.3, seed=seed)
    if outliers:
        inputs.plant_outliers(wm, seed=seed + 1, frac=0.002)
    return wm.reshape(-1)


def compare_quantize(w_cpu, block, cb, signed, T):
    wb = inputs.bits(w_cpu)
    st, codes, scales, oidx, oval, nout = oracle.quantize(wb, block, cb, signed, opq_T=T)
    assert st == oracle.OK
    w = w_cpu.to(DEV)
    g_codes, g_scales, g_idx, g_val, g_nout = binding.bof4_quantize(w, block, cb, signed, opq_T=T,
                                                                    out_capacity=max(nout, 1) + 7 if T > 0 else 0)
    torch.cuda.synchronize()
    assert g_nout == nout
    assert np.array_equal(g_scales.view(torch.int16).cpu().numpy().view(np.uint16), scales)
    assert np.array_equal(g_codes.cpu().numpy(), codes)
    if T > 0:
        assert np.array_equal(g_idx.cpu().numpy(), oidx)
        assert np.array_equal(to_np_u16(g_val), oval)
    # decoder: same inputs (they are equal), same bits out
    st, deq = oracle.dequantize(codes, scales, wb.size, block, cb, oidx if T > 0 else None, oval if T > 0 else None)
    assert st == oracle.OK
    g_deq = binding.bof4_dequantize(g_codes, g_scales, wb.size, block, cb, g_idx if T > 0 else None,
                                    g_val if T > 0 else None)
    torch.cuda.synchronize()
    assert np.array_equal(to_np_u16(g_deq), deq)
    return nout


def assert_stats_close(g, o):
    assert np.array_equal(g["cnt"], o["cnt"])
    assert g["n_used"] == o["n_used"] and g["n_outliers"] == o["n_outliers"]
    assert np.allclose(g["den"], o["den"], rtol=RTOL, atol=0.0)
    # a region's numerator may cancel (zero level); compare against the region's mass instead of itself
    scale = np.maximum(np.abs(o["num"]), o["den"] * 1e-3)
    assert np.all(np.abs(g["num"] - o["num"]) <= RTOL * scale)
    assert abs(g["sse"] - o["sse"]) <= RTOL * o["sse"]


@pytest.mark.parametrize("block", [32, 64, 128, 256])
@pytest.mark.parametrize("signed", [0, 1])
@pytest.mark.parametrize("opq", [0, 1])
def test_quantize_dequantize_bit_exact(block, signed, opq):
    # 13 x 1024 weights: 6.5 tiles of 2048, ragged tail
    w = make_weights(13, 1024, seed=100 + block + signed)
    T = oracle.opq_threshold(0.95, block) if opq else 0.0
    nout = compare_quantize(w, block, cb_for(block, signed), signed, T)
    assert (nout > 0) == bool(opq)


@pytest.mark.parametrize("block", [32, 64, 128, 256])
@pytest.mark.parametrize("signed", [0, 1])
@pytest.mark.parametrize("opq", [0, 1])
@pytest.mark.parametrize("w2", [1, 0])
def test_lloyd_step_parity(block, signed, opq, w2):
    # 301 x 1024 = 308224 weights: more segments than one pass of a small grid, ragged tail in the last round
    w = make_weights(301, 1024, seed=200 + block)
    cb = cb_for(block, signed)
    T = oracle.opq_threshold(0.95, block) if opq else 0.0
    st, o = oracle.lloyd_step(inputs.bits(w), block, cb, signed, opq_T=T, weight_by_max2=bool(w2))
    assert st == oracle.OK
    g = binding.bof4_lloyd_step(w.to(DEV), block, cb, signed, opq_T=T, weight_by_max2=bool(w2))
    assert_stats_close(g, o)
    pins = codebooks.PIN_BOF4S if signed else codebooks.PIN_BOF4
    assert np.allclose(binding.bof4_codebook_update(g, pins, cb), oracle.codebook_update(o, pins, cb), rtol=RTOL, atol=0)


def test_config0_twenty_lloyd_iterations_then_quantize():
    """Workload 0: 1024 x 1024 N(0, 0.02^2), block 64, signed absmax, 20 EM iterations from the quantile start,
    every step compared; then quantise + pack + dequantise with the final codebook."""
    w = inputs.gaussian_matrix(1024, 1024, 0.02, seed=0).reshape(-1)
    wb, wd = inputs.bits(w), w.to(DEV)
    cb = codebooks.gaussian_quantile_init()
    ws = binding.alloc_workspace(w.numel(), 64)
    mse = []
    for it in range(20):
        st, o = oracle.lloyd_step(wb, 64, cb, 1)
        g = binding.bof4_lloyd_step(wd, 64, cb, 1, ws=ws)
        assert_stats_close(g, o)
        mse.append(g["sse"] / g["n_used"])
        cb_o = oracle.codebook_update(o, codebooks.PIN_BOF4S, cb)
        cb_g = binding.bof4_codebook_update(g, codebooks.PIN_BOF4S, cb)
        assert np.allclose(cb_g, cb_o, rtol=RTOL, atol=0.0)
        cb = cb_o
    assert all(b <= a for a, b in zip(mse, mse[1:]))
    compare_quantize(w, 64, cb, 1, 0.0)


def test_lloyd_is_bit_reproducible():
    w = make_weights(64, 1024, seed=5).to(DEV)
    cb = cb_for(64, 1)
    T = oracle.opq_threshold(0.95, 64)
    runs = [binding.bof4_lloyd_step(w, 64, cb, 1, opq_T=T) for _ in range(3)]
    for r in runs[1:]:
        assert np.array_equal(r["num"], runs[0]["num"]) and np.array_equal(r["den"], runs[0]["den"])
        assert r["sse"] == runs[0]["sse"] and np.array_equal(r["cnt"], runs[0]["cnt"])


def bf16(vals):
    return torch.tensor(vals, dtype=torch.float32).to(torch.bfloat16)


@pytest.mark.parametrize("signed", [0, 1])
def test_degenerate_blocks(signed):
    """All-zero block, -0.0, equal magnitudes of opposite sign (lowest index wins), exact mid-point values,
    a constant block, tiny (subnormal-range) and large block constants, a single block as the whole input."""
    blocks = []
    blocks.append(torch.zeros(64))                                        # all zero
    z = torch.zeros(64); z[3] = -0.0; z[10] = -0.0; blocks.append(z)      # negative zeros only
    t = torch.zeros(64); t[5] = -1.0; t[9] = 1.0; t[20] = 0.5; blocks.append(t)   # +-tie, negative first
    t = torch.zeros(64); t[5] = 1.0; t[9] = -1.0; t[20] = -0.5; blocks.append(t)  # +-tie, positive first
    blocks.append(torch.full((64,), 0.75))                                # constant block
    blocks.append(torch.linspace(-1, 1, 64) * 3e-6)                       # constant below binary16 normal range
    blocks.append(torch.linspace(-1, 1, 64) * 2e-8)                       # rounds to zero or one binary16 ulp
    blocks.append(torch.linspace(-1, 1, 64) * 6.0e4)                      # near binary16 maximum
    blocks.append(torch.linspace(-1, 1, 64) * 1e-30)                      # constant flushes to zero in binary16
    g = torch.Generator().manual_seed(1)
    blocks.append(torch.randn(64, generator=g) * torch.exp2(torch.randint(-40, 10, (64,), generator=g).float()))
    w = torch.cat(blocks).to(torch.bfloat16)
    cb = cb_for(64, signed)
    compare_quantize(w, 64, cb, signed, 0.0)
    compare_quantize(w, 64, cb, signed, oracle.opq_threshold(0.95, 64))
    compare_quantize(w[:64], 64, cb, signed, 0.0)
    st, o = oracle.lloyd_step(inputs.bits(w), 64, cb, signed)
    assert_stats_close(binding.bof4_lloyd_step(w.to(DEV), 64, cb, signed), o)
    # dyadic codebook whose mid-points are bf16 numbers: exact ties go to the lower level on both sides
    dy = np.array([-1, -.75, -.5, -.375, -.25, -.125, -.0625, 0, .0625, .125, .25, .375, .5, .625, .75, 1.0])
    mids = 0.5 * (dy[:-1] + dy[1:])
    t = torch.zeros(64)
    t[:15] = torch.tensor(mids, dtype=torch.float32)
    t[63] = 1.0
    compare_quantize(t.to(torch.bfloat16), 64, dy, signed, 0.0)


def test_outliers_piled_up_in_one_stretch():
    """Blocks of a constant plus tiny noise make every element an outlier by the paper's rule (|w| >> sigma_b T).
    A few hundred such blocks in a row exceed what one wave may stage and send the call down its general path;
    the result must be the same list."""
    w = make_weights(301, 1024, seed=31, outliers=False)
    g = torch.Generator().manual_seed(32)
    n_flat = 64 * 200
    w[4096:4096 + n_flat] = (1.0 + 0.004 * torch.randn(n_flat, generator=g)).to(torch.bfloat16)
    for block in (64, 256):
        T = oracle.opq_threshold(0.95, block)
        wb = inputs.bits(w)
        st, codes, scales, oidx, oval, nout = oracle.quantize(wb, block, cb_for(block, 1), 1, opq_T=T)
        assert nout > 5000
        gc, gs, gi, gv, gn = binding.bof4_quantize(w.to(DEV), block, cb_for(block, 1), 1, opq_T=T, out_capacity=nout + 100)
        assert gn == nout and np.array_equal(gi.cpu().numpy(), oidx) and np.array_equal(to_np_u16(gv), oval)
        assert np.array_equal(gc.cpu().numpy(), codes) and np.array_equal(to_np_u16(gs), scales)
        st, o = oracle.lloyd_step(wb, block, cb_for(block, 1), 1, opq_T=T)
        assert_stats_close(binding.bof4_lloyd_step(w.to(DEV), block, cb_for(block, 1), 1, opq_T=T), o)


def test_dequantize_arbitrary_codes_and_scales():
    g = torch.Generator().manual_seed(9)
    n, block = 64 * 333, 64
    codes = torch.randint(0, 256, (n // 2,), generator=g, dtype=torch.int32).to(torch.uint8)
    sc = (torch.randn(n // block, generator=g) * torch.exp2(torch.randint(-30, 14, (n // block,), generator=g).float()))
    scales = sc.to(torch.float16)
    cb = cb_for(64, 1)
    st, deq = oracle.dequantize(codes.numpy(), scales.view(torch.int16).numpy().view(np.uint16), n, block, cb)
    got = binding.bof4_dequantize(codes.to(DEV), scales.to(DEV), n, block, cb)
    torch.cuda.synchronize()
    assert np.array_equal(to_np_u16(got), deq)


@pytest.mark.parametrize("block", [32, 64, 128, 256])
def test_dequantize_outlier_write_back_clusters(block):
    """Outliers packed several to a 16-weight group, on both sides of group and block boundaries, at the first and
    last weight, and one index listed twice (the later value wins in both implementations)."""
    g = torch.Generator().manual_seed(19 + block)
    n = block * 97
    codes = torch.randint(0, 256, (n // 2,), generator=g, dtype=torch.int32).to(torch.uint8)
    scales = (torch.randn(n // block, generator=g) * 0.05).to(torch.float16)
    idx = sorted(set([0, 1, 2, 15, 16, 17, 31, 32, block - 1, block, block + 1, 5 * block + 7, 5 * block + 8,
                      5 * block + 9, 5 * block + 15, n - 17, n - 16, n - 2, n - 1]
                     + torch.randint(0, n, (300,), generator=g).tolist()))
    idx.insert(idx.index(17), 17)
    idx = np.array(idx, dtype=np.int64)
    val = (torch.randn(idx.size, generator=g) * 3).to(torch.float16)
    cb = cb_for(block, 1)
    val_np = val.view(torch.int16).numpy().view(np.uint16)
    st, deq = oracle.dequantize(codes.numpy(), scales.view(torch.int16).numpy().view(np.uint16), n, block, cb, idx,
                                val_np)
    got = binding.bof4_dequantize(codes.to(DEV), scales.to(DEV), n, block, cb, torch.from_numpy(idx).to(DEV),
                                  val.to(DEV))
    torch.cuda.synchronize()
    assert np.array_equal(to_np_u16(got), deq)


def test_dequantize_skips_list_entries_outside_the_tensor():
    """Entries below 0 or at/after n (the oracle rejects such a list) are ignored; the rest is written as usual."""
    g = torch.Generator().manual_seed(23)
    n, block = 64 * 150, 64  # one full decoder tile and a ragged second one
    codes = torch.randint(0, 256, (n // 2,), generator=g, dtype=torch.int32).to(torch.uint8)
    scales = (torch.randn(n // block, generator=g) * 0.05).to(torch.float16)
    good = np.array(sorted(set(torch.randint(0, n, (40,), generator=g).tolist() + [0, n - 1])), dtype=np.int64)
    idx = np.concatenate([np.array([-7, -1], dtype=np.int64), good, np.array([n, n + 5, 2 ** 40], dtype=np.int64)])
    val = (torch.randn(idx.size, generator=g) * 3).to(torch.float16)
    cb = cb_for(block, 1)
    val_np = val.view(torch.int16).numpy().view(np.uint16)
    st, deq = oracle.dequantize(codes.numpy(), scales.view(torch.int16).numpy().view(np.uint16), n, block, cb, good,
                                val_np[2:2 + good.size])
    assert st == oracle.OK
    out = torch.full((n + 64,), 7.0, dtype=torch.bfloat16, device=DEV)  # guard band behind the tensor
    binding.bof4_dequantize(codes.to(DEV), scales.to(DEV), n, block, cb, torch.from_numpy(idx).to(DEV), val.to(DEV),
                            out=out[:n])
    torch.cuda.synchronize()
    assert np.array_equal(to_np_u16(out[:n]), deq)
    assert bool((out[n:] == 7.0).all())


def test_capacity_overflow_and_workspace_errors():
    w = make_weights(16, 1024, seed=77)
    T = oracle.opq_threshold(0.95, 64)
    cb = cb_for(64, 1)
    full = oracle.quantize(inputs.bits(w), 64, cb, 1, opq_T=T)
    assert full[5] > 3
    wd = w.to(DEV)
    r = binding.bof4_quantize(wd, 64, cb, 1, opq_T=T, out_capacity=3, allow_overflow=True)
    assert r[4] == full[5]                                   # required count reported
    assert np.array_equal(r[0].cpu().numpy(), full[1])       # codes and scales still complete
    with pytest.raises(binding.Bof4Error) as e:
        binding.bof4_quantize(wd, 64, cb, 1, opq_T=T, out_capacity=3)
    assert e.value.code == binding.BOF4_ERR_CAPACITY
    with pytest.raises(binding.Bof4Error) as e:
        binding.bof4_quantize(wd, 64, cb, 1, opq_T=T, out_capacity=64, ws=torch.empty(256, dtype=torch.uint8, device=DEV))
    assert e.value.code == binding.BOF4_ERR_WORKSPACE
    with pytest.raises(binding.Bof4Error) as e:
        binding.bof4_lloyd_step(wd, 64, cb, 1, ws=torch.empty(256, dtype=torch.uint8, device=DEV))
    assert e.value.code == binding.BOF4_ERR_WORKSPACE


def test_results_in_pinned_host_memory_are_written_in_place():
    """Result records in pinned host memory are filled by the GPU directly; same numbers as the copy path."""
    w = make_weights(64, 1024, seed=91)
    cb = cb_for(64, 1)
    T = oracle.opq_threshold(0.95, 64)
    wd = w.to(DEV)
    ref = binding.bof4_lloyd_step(wd, 64, cb, 1, opq_T=T)
    rec, keep = binding.pinned_lloyd_stats()
    got = binding.bof4_lloyd_step(wd, 64, cb, 1, opq_T=T, out=rec)
    assert np.array_equal(got["num"], ref["num"]) and np.array_equal(got["cnt"], ref["cnt"])
    assert got["sse"] == ref["sse"] and got["n_used"] == ref["n_used"] and got["n_outliers"] == ref["n_outliers"]
    ctr, keep2 = binding.pinned_counter()
    a = binding.bof4_quantize(wd, 64, cb, 1, opq_T=T, out_capacity=4096)
    b = binding.bof4_quantize(wd, 64, cb, 1, opq_T=T, out_capacity=4096, counter=ctr)
    assert a[4] == b[4] == ctr.value and a[4] > 0
    assert torch.equal(a[2], b[2]) and torch.equal(a[0], b[0])


@pytest.mark.parametrize("pinned", [False, True])
def test_calls_on_a_side_stream(pinned):
    """The whole path on a stream of the caller's (not the default one), with results in ordinary and in pinned host
    memory; many calls back to back so that a result read too early, or work that escaped the stream's order, would
    show.  Compared with the oracle."""
    side = torch.cuda.Stream()
    cb = cb_for(64, 1)
    T = oracle.opq_threshold(0.95, 64)
    rec, keep = binding.pinned_lloyd_stats() if pinned else (None, None)
    ctr, keep2 = binding.pinned_counter() if pinned else (None, None)
    for rep in range(6):
        w = make_weights(96 + 8 * rep, 1024, seed=400 + rep)
        wb = inputs.bits(w)
        st, o_codes, o_scales, o_idx, o_val, o_n = oracle.quantize(wb, 64, cb, 1, opq_T=T)
        st, o_deq = oracle.dequantize(o_codes, o_scales, wb.size, 64, cb, o_idx, o_val)
        st, o_stats = oracle.lloyd_step(wb, 64, cb, 1, opq_T=T)
        wd = w.to(DEV)
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            gc, gs, gi, gv, gn = binding.bof4_quantize(wd, 64, cb, 1, opq_T=T, out_capacity=o_n + 8, stream=side,
                                                       counter=ctr)
            gd = binding.bof4_dequantize(gc, gs, wb.size, 64, cb, gi, gv, stream=side)
            g_stats = binding.bof4_lloyd_step(wd, 64, cb, 1, opq_T=T, stream=side, out=rec)
        side.synchronize()
        assert gn == o_n and np.array_equal(gi.cpu().numpy(), o_idx) and np.array_equal(to_np_u16(gv), o_val)
        assert np.array_equal(gc.cpu().numpy(), o_codes) and np.array_equal(to_np_u16(gs), o_scales)
        assert np.array_equal(to_np_u16(gd), o_deq)
        assert_stats_close(g_stats, o_stats)


def test_calls_in_two_halves_give_the_results_of_the_plain_calls():
    """bof4_quantize_begin / _finish and bof4_lloyd_step_begin / bof4_wait_result with other work enqueued in between
    (the order the benchmark uses: quantise, Lloyd step, then the count, the decoder, then the sums) against the
    plain calls; also the errors of the first halves when their result cannot go to pinned memory."""
    w = make_weights(48, 1024, seed=77).to(DEV)
    n = w.numel()
    cb = cb_for(64, 1)
    T = oracle.opq_threshold(0.95, 64)
    cap = n // 16
    ref_codes, ref_scales, ref_idx, ref_val, ref_k = binding.bof4_quantize(w, 64, cb, 1, opq_T=T, out_capacity=cap)
    ref_stats = binding.bof4_lloyd_step(w, 64, cb, 1)
    ref_deq = binding.bof4_dequantize(ref_codes, ref_scales, n, 64, cb, ref_idx, ref_val)
    codes = torch.empty(n // 2, dtype=torch.uint8, device=DEV)
    scales = torch.empty(n // 64, dtype=torch.float16, device=DEV)
    oidx = torch.empty(cap, dtype=torch.int64, device=DEV)
    oval = torch.empty(cap, dtype=torch.float16, device=DEV)
    ws_q = binding.alloc_workspace(n, 64, cap, DEV)
    ws_l = binding.alloc_workspace(n, 64, 0, DEV)
    counter, keep1 = binding.pinned_counter()
    rec, keep2 = binding.pinned_lloyd_stats()
    for _ in range(3):
        flight = binding.bof4_quantize_begin(w, 64, cb, 1, T, cap, codes, scales, oidx, oval, ws_q, counter)
        binding.bof4_lloyd_step_begin(w, 64, cb, 1, rec, ws=ws_l)
        k = flight.finish()
        deq = binding.bof4_dequantize(codes, scales, n, 64, cb, oidx, oval, n_outliers=k)
        stats = binding.bof4_wait_result(rec).as_dict()
        torch.cuda.synchronize()
        assert k == ref_k and torch.equal(codes, ref_codes) and torch.equal(scales, ref_scales)
        assert torch.equal(oidx[:k], ref_idx) and torch.equal(oval[:k], ref_val) and torch.equal(deq, ref_deq)
        assert np.array_equal(stats["cnt"], ref_stats["cnt"]) and np.array_equal(stats["num"], ref_stats["num"])
        assert stats["sse"] == ref_stats["sse"] and stats["n_used"] == n
    # without outlier extraction the first half needs no counter in pinned memory; with it, it does
    plain = ctypes.c_uint64(7)
    flight = binding.bof4_quantize_begin(w, 64, cb, 1, 0.0, 0, codes, scales, None, None, None, plain)
    assert flight.finish() == 0
    with pytest.raises(binding.Bof4Error) as e:
        binding.bof4_quantize_begin(w, 64, cb, 1, T, cap, codes, scales, oidx, oval, ws_q, plain)
    assert e.value.code == binding.BOF4_ERR_ARG
    with pytest.raises(binding.Bof4Error) as e:
        binding.bof4_lloyd_step_begin(w, 64, cb, 1, binding.LloydStats(), ws=ws_l)
    assert e.value.code == binding.BOF4_ERR_ARG
    # too small a list: the second half reports it like the plain call
    flight = binding.bof4_quantize_begin(w, 64, cb, 1, T, 8, codes, scales, oidx, oval, ws_q, counter)
    with pytest.raises(binding.Bof4Error) as e:
        flight.finish()
    assert e.value.code == binding.BOF4_ERR_CAPACITY and counter.value == ref_k


@pytest.mark.parametrize("block", [32, 64, 256])
@pytest.mark.parametrize("signed", [0, 1])
def test_lloyd_sums_of_blocks_whose_constant_binary16_stores_with_fewer_bits(block, signed):
    """A block maximum below binary16's normal range loses bits when it is stored (1.4375 x 2^-24 becomes 2^-24), so
    the weights of such a block normalise to more than 1 in magnitude, here to -1.4375 and +1.4375.  They are counted
    with that x, in the outermost regions: counts as the oracle's, sums to 1e-9, for the Lloyd step alone and in one
    pass with the quantiser (a sum of x + 1 kept as a nonnegative integer would lose a count here)."""
    g = torch.Generator().manual_seed(31 + block)
    n_blocks = 3 * 64 * min(block, 64) // block + 5  # three wave tiles and a ragged tail
    w = (torch.randn(n_blocks, block, generator=g) * 0.02)
    tiny = 1.4375 * 2.0 ** -24
    for b in range(0, n_blocks, 3):  # every third block: tiny, its extreme elements of both signs, the largest first
        w[b] = torch.randn(block, generator=g) * 0.3 * tiny
        w[b, 1], w[b, 5], w[b, 7] = tiny, -tiny, -tiny
    w = w.reshape(-1).to(torch.bfloat16)
    cb = cb_for(block, signed)
    st, o = oracle.lloyd_step(inputs.bits(w), block, cb, signed)
    assert st == oracle.OK and o["cnt"][0] >= 2 * (n_blocks // 3)  # the -1.4375s sit in the lowest region
    assert_stats_close(binding.bof4_lloyd_step(w.to(DEV), block, cb, signed), o)
    got = binding.bof4_quantize_lloyd(w.to(DEV), block, cb, signed)
    assert_stats_close(got[5], o)
    compare_quantize(w, block, cb, signed, 0.0)


@pytest.mark.parametrize("signed", [0, 1])
@pytest.mark.parametrize("weightless", [0, 1])
def test_lloyd_sums_of_a_zero_region_that_holds_only_outliers(signed, weightless):
    """One block in which no weight lies near zero; its one outlier is zeroed, runs through the sums as x = 0 and is
    taken out again.  The region of the zero level is then empty: count 0 and mass exactly 0 (not the rounding residue
    of adding and subtracting the same amount in floating point), so that an update leaves its level alone.  With
    `weightless` a second block of numbers too small for a binary16 constant (constant 0, every x = 0, weight 0) puts
    64 elements into that region that weigh nothing: count 64, mass still exactly 0."""
    w = torch.full((64,), 0.02)
    w[1::2] = -0.02
    w[::7] *= 0.7
    w[9] = 3.0  # the outlier
    if weightless:
        w = torch.cat([w, torch.full((64,), 2.0 ** -132) * torch.arange(-32, 32)])
    w = w.to(torch.bfloat16)
    cb = cb_for(64, signed)
    T = oracle.opq_threshold(0.95, 64)
    st, o = oracle.lloyd_step(inputs.bits(w), 64, cb, signed, opq_T=T)
    assert st == oracle.OK and o["n_outliers"] == 1 and o["cnt"][7] == 64 * weightless and o["den"][7] == 0.0
    g = binding.bof4_lloyd_step(w.to(DEV), 64, cb, signed, opq_T=T)
    assert g["den"][7] == 0.0 and g["num"][7] == 0.0
    assert_stats_close(g, o)
    got = binding.bof4_quantize_lloyd(w.to(DEV), 64, cb, signed, opq_T=T, out_capacity=8)
    assert got[5]["den"][7] == 0.0 and got[5]["num"][7] == 0.0
    assert_stats_close(got[5], o)
    new_g, new_o = binding.bof4_codebook_update(g, 0, cb), oracle.codebook_update(o, 0, cb)
    assert new_g[7] == cb[7] and np.allclose(new_g, new_o, rtol=RTOL, atol=0)


def test_calls_in_flight_on_three_streams_at_once_do_not_disturb_each_other():
    """Two Lloyd steps (each with its own workspace and its own pinned record) and a decoder call enqueued on three
    streams before any of them is waited for, several rounds: every result equals that of the same call made alone.
    The library keeps no device state between calls other than what the caller hands it."""
    cb = cb_for(64, 1)
    T = oracle.opq_threshold(0.95, 64)
    wa = make_weights(1536, 1024, seed=811).to(DEV)   # long enough for the calls to overlap
    wb_ = make_weights(1300, 1024, seed=812).to(DEV)
    n = wa.numel()
    codes, scales, oi, ov, k = binding.bof4_quantize(wa, 64, cb, 1, opq_T=T, out_capacity=n // 32)
    ref_a = binding.bof4_lloyd_step(wa, 64, cb, 1, opq_T=T, raw=True)
    ref_b = binding.bof4_lloyd_step(wb_, 64, cb, 1, raw=True)
    ref_d = binding.bof4_dequantize(codes, scales, n, 64, cb, oi, ov, n_outliers=int(k))
    ws_a, ws_b = binding.alloc_workspace(n, 64, 0, DEV), binding.alloc_workspace(wb_.numel(), 64, 0, DEV)
    rec_a, keep_a = binding.pinned_lloyd_stats()
    rec_b, keep_b = binding.pinned_lloyd_stats()
    out_d = torch.empty(n, dtype=torch.bfloat16, device=DEV)
    s1, s2, s3 = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    for rep in range(4):
        out_d.zero_()
        torch.cuda.synchronize()
        binding.bof4_lloyd_step_begin(wa, 64, cb, 1, rec_a, opq_T=T, ws=ws_a, stream=s1)
        binding.bof4_lloyd_step_begin(wb_, 64, cb, 1, rec_b, ws=ws_b, stream=s2)
        binding.bof4_dequantize(codes, scales, n, 64, cb, oi, ov, n_outliers=int(k), out=out_d, stream=s3)
        binding.bof4_wait_result(rec_b, stream=s2)
        binding.bof4_wait_result(rec_a, stream=s1)
        s3.synchronize()
        for got, ref in ((rec_a, ref_a), (rec_b, ref_b)):
            assert list(got.cnt[:]) == list(ref.cnt[:]) and (got.n_used, got.n_outliers) == (ref.n_used, ref.n_outliers)
            assert list(got.num[:]) == list(ref.num[:]) and list(got.den[:]) == list(ref.den[:]) and got.sse == ref.sse
        assert torch.equal(out_d.view(torch.int16), ref_d.view(torch.int16))
