"""GPU parity of the decoder inside a matrix-vector product (bof4_gemv) against the oracle.

The oracle sums in binary64; the kernel multiplies and adds in binary32 in a fixed order: 16 fused multiply-adds per
accumulator, one addition of the two accumulators, the product with the block constant, 6 additions across the
wave, at most 16 across the strips and the outlier wave - under 64 roundings of relative size 2^-24 against the sum
of the magnitudes of the terms.  An outlier's correction (value - decoded placeholder) * x brings the placeholder's
magnitude in as well, so the bound uses the magnitudes with and without the list."""
import numpy as np
import pytest
import torch

import oracle
from paper_2505_06653_amd import binding, codebooks, inputs
from test_gpu_parity import cb_for, make_weights

pytestmark = pytest.mark.gpu
DEV = "cuda"
U = 2.0 ** -24


def quantized(rows, cols, block, signed, opq, seed):
    """Codes, constants and list from the oracle's quantiser (host arrays)."""
    w = make_weights(rows, cols, seed=seed, outliers=rows * cols >= 10000)
    cb = cb_for(block, signed)
    T = oracle.opq_threshold(0.95, block) if opq else 0.0
    st, codes, scales, oi, ov, k = oracle.quantize(inputs.bits(w), block, cb, signed, opq_T=T)
    assert st == oracle.OK and ((k > 0) == bool(opq) or rows * cols < 10000)
    return cb, codes, scales, oi, ov


def rand_x(n_tokens, cols, seed):
    g = torch.Generator().manual_seed(seed)
    return torch.randn((n_tokens, cols), generator=g).to(torch.bfloat16)


def dev_i64(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int64)).to(DEV)


def dev_u16(a):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(DEV)


def run_gpu(cb, codes, scales, oi, ov, rows, cols, block, x):
    cd = torch.from_numpy(codes).to(DEV)
    sd = dev_u16(scales)
    k = 0 if oi is None else int(oi.size)
    if k:
        tab = binding.bof4_gemv_outlier_table(cd, sd, rows, cols, block, cb, dev_i64(oi), dev_u16(ov))
        y = binding.bof4_gemv(cd, sd, rows, cols, block, cb, x.to(DEV), tab, k)
    else:
        y = binding.bof4_gemv(cd, sd, rows, cols, block, cb, x.to(DEV))
    torch.cuda.synchronize()
    return y.cpu().numpy().astype(np.float64)


def check(cb, codes, scales, oi, ov, rows, cols, block, x):
    xb = inputs.bits(x).reshape(x.shape)
    st, y_o, a = oracle.gemv(codes, scales, rows, cols, block, cb, xb, oi, ov)
    assert st == oracle.OK
    if oi is not None and oi.size:
        st, _, a0 = oracle.gemv(codes, scales, rows, cols, block, cb, xb)
        a = a + a0
    y_g = run_gpu(cb, codes, scales, oi, ov, rows, cols, block, x)
    assert y_g.shape == y_o.shape
    err = np.abs(y_g - y_o)
    assert np.all(err <= 64 * U * a + 1e-37), float(np.max(err / (a + 1e-300)))
    return y_g, y_o


@pytest.mark.parametrize("block", [32, 64, 128, 256])
@pytest.mark.parametrize("opq", [0, 1])
@pytest.mark.parametrize("n_tokens", [1, 2, 5])
def test_gemv_parity(block, opq, n_tokens):
    rows, cols = 37, 2304  # ragged row chunks; two strips, the second one 256 columns wide
    cb, codes, scales, oi, ov = quantized(rows, cols, block, 1, opq, seed=900 + block)
    check(cb, codes, scales, oi if opq else None, ov if opq else None, rows, cols, block, rand_x(n_tokens, cols, 7))


@pytest.mark.parametrize("rows,cols", [(1, 32), (3, 64), (130, 6144), (65, 4096 + 2048 + 1024), (21, 20480 + 512),
                                       (9, 32768)])
def test_gemv_shapes(rows, cols):
    """Up to eight strips of 2048 columns a workgroup has one wave per strip; wider matrices (the last two: 11 and 16
    strips) make a wave take several strips in turn."""
    cb, codes, scales, oi, ov = quantized(rows, cols, 32, 0, 1, seed=31 + rows)
    check(cb, codes, scales, oi, ov, rows, cols, 32, rand_x(2, cols, 11))


def _random_cases(count, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(count):
        block = int(rng.choice([32, 64, 128, 256]))
        top = 32768 if i % 4 == 3 else 6144  # every fourth case may be many strips wide
        cols = block * int(rng.integers(1, top // block + 1))
        rows = int(rng.integers(1, 24 if cols > 8192 else 150))
        cases.append((rows, cols, block, int(rng.integers(1, 6)), int(rng.integers(0, 2)), int(rng.integers(0, 2))))
    return cases


@pytest.mark.parametrize("rows,cols,block,n_tokens,signed,opq", _random_cases(16, seed=2024))
def test_gemv_random_shapes(rows, cols, block, n_tokens, signed, opq):
    """Shapes, block sizes and token counts drawn once from a seeded generator: ragged last strips and row chunks."""
    w = make_weights(rows, cols, seed=rows * 5 + cols, outliers=False)
    cb = cb_for(block, signed)
    T = oracle.opq_threshold(0.9, block) if opq else 0.0
    st, codes, scales, oi, ov, k = oracle.quantize(inputs.bits(w), block, cb, signed, opq_T=T)
    assert st == oracle.OK
    lst = (oi, ov) if (opq and k) else (None, None)
    check(cb, codes, scales, lst[0], lst[1], rows, cols, block, rand_x(n_tokens, cols, seed=cols + n_tokens))


def test_gemv_dense_outlier_rows_take_several_rounds_and_empty_rows_none():
    """A hand-made list: a third of the weights of rows 4..11 (thousands of entries per row chunk), nothing elsewhere,
    values unrelated to the codes; a codebook without a zero level, so every placeholder decodes to something."""
    rows, cols, block = 40, 6144, 64
    cb, codes, scales, _, _ = quantized(rows, cols, block, 1, 0, seed=77)
    cb = cb + 0.013 * np.linspace(-1, 1, 16) ** 2 + 0.004
    rng = np.random.default_rng(5)
    mask = np.zeros((rows, cols), dtype=bool)
    mask[4:12] = rng.random((8, cols)) < 0.33
    mask[20, 17] = True
    mask[39, cols - 1] = True
    oi = np.flatnonzero(mask.reshape(-1)).astype(np.int64)
    ov = (rng.standard_normal(oi.size).astype(np.float32) * 0.3).astype(np.float16).view(np.uint16)
    y_g, y_o = check(cb, codes, scales, oi, ov, rows, cols, block, rand_x(2, cols, 3))
    st, y_plain, _ = oracle.gemv(codes, scales, rows, cols, block, cb, inputs.bits(rand_x(2, cols, 3)).reshape(2, cols))
    assert np.max(np.abs(y_o[:, 4:12] - y_plain[:, 4:12])) > 1e-3  # the list matters


def test_gemv_rows_without_entries_equal_the_call_without_a_list():
    rows, cols, block = 24, 2048, 128
    cb, codes, scales, _, _ = quantized(rows, cols, block, 1, 0, seed=78)
    oi = np.array([5 * cols + 3, 5 * cols + 900, 17 * cols], dtype=np.int64)
    ov = np.array([0.5, -0.25, 1.0], dtype=np.float16).view(np.uint16)
    x = rand_x(1, cols, 4)
    y_list = run_gpu(cb, codes, scales, oi, ov, rows, cols, block, x)
    y_none = run_gpu(cb, codes, scales, None, None, rows, cols, block, x)
    other = np.ones(rows, dtype=bool)
    other[[5, 17]] = False
    assert np.array_equal(y_list[:, other], y_none[:, other])
    assert np.all(y_list[:, ~other] != y_none[:, ~other])


def test_gemv_unit_vectors_and_zero_input():
    rows, cols, block = 9, 2304, 64
    cb, codes, scales, oi, ov = quantized(rows, cols, block, 1, 1, seed=79)
    x = torch.zeros((2, cols), dtype=torch.bfloat16)
    x[1, 2049] = 1.0  # second strip, an odd element: a high nibble
    y_g, y_o = check(cb, codes, scales, oi, ov, rows, cols, block, x)
    assert np.array_equal(y_g[0], np.zeros(rows))
    assert np.array_equal(y_g[1], y_o[1].astype(np.float32).astype(np.float64))  # a single product: one rounding


def test_gemv_is_bit_reproducible_and_respects_out_and_stream():
    rows, cols, block = 130, 4096, 64
    cb, codes, scales, oi, ov = quantized(rows, cols, block, 1, 1, seed=80)
    cd, sd, oid, ovd = torch.from_numpy(codes).to(DEV), dev_u16(scales), dev_i64(oi), dev_u16(ov)
    tab = binding.bof4_gemv_outlier_table(cd, sd, rows, cols, block, cb, oid, ovd)
    x = rand_x(3, cols, 5).to(DEV)
    y1 = binding.bof4_gemv(cd, sd, rows, cols, block, cb, x, tab, oi.size)
    out = torch.full((3, rows), float("nan"), device=DEV)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        y2 = binding.bof4_gemv(cd, sd, rows, cols, block, cb, x, tab, oi.size, out=out)
    side.synchronize()
    torch.cuda.synchronize()
    assert y2 is out and torch.equal(y1, y2)
    # one token alone gives the same numbers as inside a batch
    y3 = binding.bof4_gemv(cd, sd, rows, cols, block, cb, x[2], tab, oi.size)
    assert torch.equal(y3[0], y1[2])


def test_outlier_table_offsets_and_entries():
    """The table's first part counts the entries below the start of every row and every stretch of 2048 columns; its
    second part holds column and (value - decoded placeholder) per entry, rounded once to binary32."""
    rows, cols, block = 1000, 4096 + 1024, 64  # three stretches, the last one half as wide
    cb, codes, scales, _, _ = quantized(rows, cols, block, 1, 0, seed=82)
    rng = np.random.default_rng(1)
    oi = np.sort(rng.choice(rows * cols, 50_000, replace=False)).astype(np.int64)
    oi = oi[(oi // cols) % 7 != 3]  # rows without entries
    ov = (rng.standard_normal(oi.size).astype(np.float32) * 0.2).astype(np.float16)
    nbytes = binding.bof4_gemv_outlier_table_bytes(rows, cols, oi.size)
    assert nbytes == (rows * 3 + 1 + 1) // 2 * 8 + 8 * oi.size
    cd, sd = torch.from_numpy(codes).to(DEV), dev_u16(scales)
    tab = binding.bof4_gemv_outlier_table(cd, sd, rows, cols, block, cb, dev_i64(oi), dev_u16(ov.view(np.uint16)))
    raw = tab.cpu().numpy()
    n_off = rows * 3 + 1
    offs = raw[: 4 * n_off].view(np.uint32)
    starts = (np.arange(rows, dtype=np.int64)[:, None] * cols + np.arange(3, dtype=np.int64)[None, :] * 2048).reshape(-1)
    assert np.array_equal(offs, np.searchsorted(oi, np.concatenate([starts, [rows * cols]]), side="left"))
    ent = raw[(n_off + 1) // 2 * 8:].view(np.uint32).reshape(-1, 2)
    assert np.array_equal(ent[:, 0], (oi % cols).astype(np.uint32))
    code = (codes[oi >> 1] >> ((oi & 1) * 4).astype(np.uint8)) & 15
    old = scales.view(np.float16)[oi // block].astype(np.float64) * cb.astype(np.float32).astype(np.float64)[code]
    delta = ov.astype(np.float64) - old  # exact product; the difference is exact or off by far less than 2^-24
    assert np.all(np.abs(ent[:, 1].view(np.float32).astype(np.float64) - delta) <= 2.0 ** -24 * np.abs(delta))
    with pytest.raises(binding.Bof4Error) as e:
        binding.bof4_gemv_outlier_table(cd, sd, rows, cols, block, cb, dev_i64(oi), dev_u16(ov.view(np.uint16)),
                                        out=torch.empty(nbytes - 8, dtype=torch.uint8, device=DEV))
    assert e.value.code == binding.BOF4_ERR_WORKSPACE


def test_gemv_argument_errors():
    rows, cols, block = 4, 128, 64
    cb, codes, scales, oi, ov = quantized(rows, cols, block, 1, 1, seed=81)
    cd, sd = torch.from_numpy(codes).to(DEV), dev_u16(scales)
    x = rand_x(1, cols, 1).to(DEV)
    with pytest.raises(binding.Bof4Error) as e:
        binding.bof4_gemv(cd, sd, rows, 96, 64, cb, x[:, :96].contiguous())
    assert e.value.code == binding.BOF4_ERR_ARG
    with pytest.raises(binding.Bof4Error) as e:
        binding.bof4_gemv(cd, sd, rows, cols, 48, cb, x)
    assert e.value.code == binding.BOF4_ERR_ARG
    with pytest.raises(binding.Bof4Error) as e:  # codes not 16-byte aligned
        binding.bof4_gemv(cd[4:], sd, rows - 1, cols, block, cb, x)
    assert e.value.code == binding.BOF4_ERR_ARG
    with pytest.raises(ValueError):
        binding.bof4_gemv(cd, sd, rows, cols, block, cb, x, None, 3)  # outliers without their table
    with pytest.raises(ValueError):
        binding.bof4_gemv(cd, sd, rows, cols, block, cb, x.float())
    big = 32768 + 2048
    with pytest.raises(binding.Bof4Error) as e:
        binding.bof4_gemv(cd, sd, 1, big, 64, cb, torch.zeros((1, big), dtype=torch.bfloat16, device=DEV))
    assert e.value.code == binding.BOF4_ERR_ARG
    bad_cb = cb.copy()
    bad_cb[3] = bad_cb[4]
    with pytest.raises(binding.Bof4Error):
        binding.bof4_gemv(cd, sd, rows, cols, block, bad_cb, x)


@pytest.mark.parametrize("rows,cols", [(4096, 4096), (4096, 11008), (11008, 4096), (8192, 28672)])
def test_gemv_llama_matrices_with_opq(rows, cols):
    """The three matrix shapes of workload 1 and the widest one of workload 4 at full size, signed constants, block 64,
    OPQ q = 0.95, two tokens: every output against the oracle."""
    wm = inputs.student_t_matrix(rows, cols, 5.0, 0.02, 0.3, seed=rows + cols)
    cb = cb_for(64, 1)
    T = oracle.opq_threshold(0.95, 64)
    st, codes, scales, oi, ov, k = oracle.quantize(inputs.bits(wm.reshape(-1)), 64, cb, 1, opq_T=T)
    assert st == oracle.OK and k > 1000
    check(cb, codes, scales, oi, ov, rows, cols, 64, rand_x(2, cols, 9))
