"""GPU parity of the decoder inside a matrix product for many tokens (bof4_gemm) against the oracle, which multiplies
the decoded bfloat16 matrix with x in binary64.

Every product of two bfloat16 numbers is exact in binary32, so the kernel's only roundings are those of its binary32
additions: at most one per column inside the matrix cores' accumulation chain, a few across the waves and the column
splits, and the outlier corrections - under (cols + 64) roundings of relative size 2^-24 against the sum of the
magnitudes of the terms.  An outlier's correction (value - decoded placeholder) * x brings the placeholder's magnitude
in as well, so the bound uses the magnitudes with and without the list.  Where every partial sum is a binary32 number
(small integers times powers of two) the result must equal the oracle's bit for bit: that case catches a term that is
dropped, doubled or paired with the wrong x, however small."""
import numpy as np
import pytest
import torch

import oracle
from paper_2505_06653_amd import binding, inputs
from test_gpu_parity import cb_for, make_weights
from test_gpu_gemv import dev_i64, dev_u16, quantized, rand_x

pytestmark = pytest.mark.gpu
DEV = "cuda"
U = 2.0 ** -24


def run_gpu(cb, codes, scales, oi, ov, rows, cols, block, x):
    cd = torch.from_numpy(codes).to(DEV)
    sd = dev_u16(scales)
    k = 0 if oi is None else int(oi.size)
    packed = binding.bof4_gemm_pack(cd, sd, rows, cols, block)
    if k:
        tab = binding.bof4_gemm_outlier_table(cd, sd, rows, cols, block, cb, dev_i64(oi), dev_u16(ov))
        y = binding.bof4_gemm(packed, rows, cols, cb, x.to(DEV), tab, k)
    else:
        y = binding.bof4_gemm(packed, rows, cols, cb, x.to(DEV))
    torch.cuda.synchronize()
    return y.cpu().numpy().astype(np.float64)


def check(cb, codes, scales, oi, ov, rows, cols, block, x):
    xb = inputs.bits(x).reshape(x.shape)
    st, y_o, a = oracle.gemm(codes, scales, rows, cols, block, cb, xb, oi, ov)
    assert st == oracle.OK
    if oi is not None and oi.size:
        st, _, a0 = oracle.gemm(codes, scales, rows, cols, block, cb, xb)
        a = a + a0
    y_g = run_gpu(cb, codes, scales, oi, ov, rows, cols, block, x)
    assert y_g.shape == y_o.shape
    err = np.abs(y_g - y_o)
    assert np.all(err <= (cols + 64) * U * a + 1e-37), float(np.max(err / (a + 1e-300)))
    return y_g, y_o


@pytest.mark.parametrize("block", [32, 64, 128, 256])
@pytest.mark.parametrize("opq", [0, 1])
@pytest.mark.parametrize("n_tokens", [1, 7, 32, 40, 96, 130, 224])
def test_gemm_parity(block, opq, n_tokens):
    # two row tiles, the second with 5 rows; 36 chunks of 64 columns over 4 workgroups each; token tiles (of 32) taken
    # four, two or one at a time
    rows, cols = 37, 2304
    cb, codes, scales, oi, ov = quantized(rows, cols, block, 1, opq, seed=900 + block)
    check(cb, codes, scales, oi if opq else None, ov if opq else None, rows, cols, block, rand_x(n_tokens, cols, 7))


@pytest.mark.parametrize("rows,cols", [(1, 32), (3, 64), (130, 6144), (65, 4096 + 2048 + 1024), (33, 32768),
                                       (16390, 128), (16390, 32)])
def test_gemm_shapes(rows, cols):
    """Half a chunk, one chunk, many; the last two have hundreds of row tiles, so that one workgroup takes all columns of
    its rows and writes the result itself."""
    cb, codes, scales, oi, ov = quantized(rows, cols, 32, 0, 1, seed=31 + rows)
    packed_x = 32 * ((cols + 63) // 64 * 64) * 2 + cols * 32 * 2  # in product order and transposed, 32 token slots
    extra = binding.bof4_gemm_workspace_bytes(rows, cols, 5) - packed_x
    assert 0 <= extra < 512 if (rows > 16000 or cols < 1024) else extra >= 2 * 32 * rows * 4
    check(cb, codes, scales, oi, ov, rows, cols, 32, rand_x(5, cols, 11))


def _random_cases(count, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(count):
        block = int(rng.choice([32, 64, 128, 256]))
        wide = i % 4 == 3  # every fourth case has 8192 or more columns: two tiles of rows per wave above 32 tokens
        cols = block * int(rng.integers(8192 // block, 8192 // block + 6) if wide else rng.integers(1, 3072 // block + 1))
        rows = int(rng.integers(1, 40 if wide else 200))
        n_tokens = int(rng.choice([1, 2, 31, 32, 33, 63, 64, 65, 95, 96, 97, 127, 128, 129, 200]))
        cases.append((rows, cols, block, n_tokens, int(rng.integers(0, 2)), int(rng.integers(0, 2))))
    return cases


@pytest.mark.parametrize("rows,cols,block,n_tokens,signed,opq", _random_cases(24, seed=2025))
def test_gemm_random_shapes(rows, cols, block, n_tokens, signed, opq):
    """Shapes, block sizes and token counts drawn once from a seeded generator: ragged row tiles, half chunks, every
    number of token tiles per launch."""
    w = make_weights(rows, cols, seed=rows * 7 + cols, outliers=False)
    cb = cb_for(block, signed)
    T = oracle.opq_threshold(0.9, block) if opq else 0.0
    st, codes, scales, oi, ov, k = oracle.quantize(inputs.bits(w), block, cb, signed, opq_T=T)
    assert st == oracle.OK
    lst = (oi, ov) if (opq and k) else (None, None)
    check(cb, codes, scales, lst[0], lst[1], rows, cols, block, rand_x(n_tokens, cols, seed=cols + n_tokens))


@pytest.mark.parametrize("rows,cols,n_tokens", [(33, 32768, 40), (70, 8192, 130), (16390, 128, 70)])
def test_gemm_with_two_tiles_of_rows_per_wave(rows, cols, n_tokens):
    """More than 32 tokens on a matrix with 8192 or more rows or columns: a wave multiplies two tiles of 32 rows with
    every word of x it reads.  Row counts that leave the second tile nearly empty, absent (an odd number of tiles)
    or ragged."""
    cb, codes, scales, oi, ov = quantized(rows, cols, 64, 1, 1, seed=41 + rows)
    check(cb, codes, scales, oi, ov, rows, cols, 64, rand_x(n_tokens, cols, 13))
    check(cb, codes, scales, None, None, rows, cols, 64, rand_x(n_tokens, cols, 14))


@pytest.mark.parametrize("rows,cols,n_tokens", [(70, 1536, 33), (16390, 128, 9), (16390, 128, 45), (70, 8192, 33)])
def test_gemm_is_exact_where_every_partial_sum_is_a_binary32_number(rows, cols, n_tokens):
    """Levels k / 8, constants 2^e, x small integers, list values multiples of 1 / 8: every product and every sum of
    them is a multiple of 2^-9 below 2^15, so no addition rounds, in any order.  (The last two cases take two tiles
    of rows per wave.)"""
    block = 32
    rng = np.random.default_rng(rows)
    cb = (np.arange(16) - 8) / 8.0
    codes = rng.integers(0, 256, rows * cols // 2, dtype=np.uint8)
    top, xmax = (3, 4) if cols <= 2048 else (1, 2)  # |product| <= 2^(top - 1) * xmax, times cols below 2^15
    scales = (2.0 ** rng.integers(-6, top, rows * cols // block)).astype(np.float16).view(np.uint16)
    x = torch.from_numpy(rng.integers(-xmax, xmax + 1, (n_tokens, cols)).astype(np.float32)).to(torch.bfloat16)
    xb = inputs.bits(x).reshape(x.shape)
    oi = np.sort(rng.choice(rows * cols, rows * cols // 300, replace=False)).astype(np.int64)
    ov = (rng.integers(-32, 33, oi.size) / 8.0).astype(np.float16).view(np.uint16)
    for lst in ((None, None), (oi, ov)):
        st, y_o, _ = oracle.gemm(codes, scales, rows, cols, block, cb, xb, *lst)
        assert st == oracle.OK
        y_g = run_gpu(cb, codes, scales, lst[0], lst[1], rows, cols, block, x)
        assert np.array_equal(y_g, y_o)


@pytest.mark.parametrize("n_tokens", [7, 100])
def test_gemm_dense_outlier_rows_take_several_rounds_and_empty_rows_none(n_tokens):
    """A hand-made list: a third of the weights of rows 4..11 (thousands of entries per row), single entries in the
    first and last column elsewhere, nothing in most rows; values unrelated to the codes; a codebook without a zero
    level, so every placeholder decodes to something."""
    rows, cols, block = 40, 6144, 64
    cb, codes, scales, _, _ = quantized(rows, cols, block, 1, 0, seed=77)
    cb = cb + 0.013 * np.linspace(-1, 1, 16) ** 2 + 0.004
    rng = np.random.default_rng(5)
    mask = np.zeros((rows, cols), dtype=bool)
    mask[4:12] = rng.random((8, cols)) < 0.33
    mask[20, 0] = True
    mask[39, cols - 1] = True
    oi = np.flatnonzero(mask.reshape(-1)).astype(np.int64)
    ov = (rng.standard_normal(oi.size).astype(np.float32) * 0.3).astype(np.float16).view(np.uint16)
    x = rand_x(n_tokens, cols, 3)
    y_g, y_o = check(cb, codes, scales, oi, ov, rows, cols, block, x)
    y_none = run_gpu(cb, codes, scales, None, None, rows, cols, block, x)
    touched = np.zeros(rows, dtype=bool)
    touched[4:12] = touched[20] = touched[39] = True
    assert np.array_equal(y_g[:, ~touched], y_none[:, ~touched])  # rows without entries: the dense result, bit for bit
    assert np.max(np.abs(y_g[:, 4:12] - y_none[:, 4:12])) > 1e-3  # the list matters


@pytest.mark.parametrize("opq", [0, 1])
def test_gemm_a_token_that_is_not_finite_stays_on_its_own(opq):
    """One token carries an infinity: its own results are not finite (every row multiplies it), every other token's are
    what they are without it - nothing leaks through padding, clamped list slots or shared registers."""
    rows, cols, block = 70, 2304, 64
    cb, codes, scales, oi, ov = quantized(rows, cols, block, 1, opq, seed=91)
    lst = (oi, ov) if opq else (None, None)
    x = rand_x(37, cols, 17)
    y_clean = run_gpu(cb, codes, scales, lst[0], lst[1], rows, cols, block, x)
    x[5, 1000] = float("inf")
    x[33, 3] = float("nan")
    y = run_gpu(cb, codes, scales, lst[0], lst[1], rows, cols, block, x)
    bad = np.zeros(37, dtype=bool)
    bad[[5, 33]] = True
    assert not np.isfinite(y[bad]).any()
    assert np.array_equal(y[~bad], y_clean[~bad])


def test_gemm_unit_vectors_pick_single_decoded_weights():
    """x = a unit vector per token: the product returns one column of the decoded matrix, exactly."""
    rows, cols, block = 45, 2304, 64
    cb, codes, scales, oi, ov = quantized(rows, cols, block, 1, 1, seed=79)
    picks = [0, 1, 7, 8, 31, 32, 63, 64, 65, 2049, 2303]
    x = torch.zeros((len(picks), cols), dtype=torch.bfloat16)
    for t, c in enumerate(picks):
        x[t, c] = 1.0
    y_g, y_o = check(cb, codes, scales, oi, ov, rows, cols, block, x)
    st, deq = oracle.dequantize(codes, scales, rows * cols, block, cb, oi, ov)
    assert st == oracle.OK
    w_hat = (deq.astype(np.uint32) << 16).view(np.float32).reshape(rows, cols).astype(np.float64)
    assert np.array_equal(y_g, w_hat[:, picks].T)


def test_gemm_on_the_quantisers_output_equals_the_product_over_the_decoders_output():
    rows, cols, block = 257, 4096, 64
    w = inputs.student_t_matrix(rows, cols, 5.0, 0.02, 0.3, seed=5).reshape(-1).to(DEV)
    cb = cb_for(block, 1)
    T = oracle.opq_threshold(0.95, block)
    codes, scales, oi, ov, k = binding.bof4_quantize(w, block, cb, 1, opq_T=T, out_capacity=w.numel() // 20)
    assert k > 0
    tab = binding.bof4_gemm_outlier_table(codes, scales, rows, cols, block, cb, oi, ov, n_outliers=k)
    packed = binding.bof4_gemm_pack(codes, scales, rows, cols, block)
    x = rand_x(48, cols, 21).to(DEV)
    y = binding.bof4_gemm(packed, rows, cols, cb, x, tab, k)
    deq = binding.bof4_dequantize(codes, scales, w.numel(), block, cb, oi, ov, n_outliers=k).reshape(rows, cols)
    ref = x.double() @ deq.double().T
    mag = x.double().abs() @ deq.double().abs().T
    assert torch.all((y.double() - ref).abs() <= (cols + 64) * U * 2 * mag)


def test_gemm_is_bit_reproducible_and_respects_out_workspace_and_stream():
    rows, cols, block = 130, 4096, 64
    cb, codes, scales, oi, ov = quantized(rows, cols, block, 1, 1, seed=80)
    cd, sd, oid, ovd = torch.from_numpy(codes).to(DEV), dev_u16(scales), dev_i64(oi), dev_u16(ov)
    tab = binding.bof4_gemm_outlier_table(cd, sd, rows, cols, block, cb, oid, ovd)
    packed = binding.bof4_gemm_pack(cd, sd, rows, cols, block)
    x = rand_x(35, cols, 5).to(DEV)
    y1 = binding.bof4_gemm(packed, rows, cols, cb, x, tab, oi.size)
    out = torch.full((35, rows), float("nan"), device=DEV)
    ws = torch.empty(binding.bof4_gemm_workspace_bytes(rows, cols, 35), dtype=torch.uint8, device=DEV)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        y2 = binding.bof4_gemm(packed, rows, cols, cb, x, tab, oi.size, out=out, ws=ws)
    side.synchronize()
    torch.cuda.synchronize()
    assert y2 is out and torch.equal(y1, y2)
    # one token alone gives the same numbers as inside a batch
    y3 = binding.bof4_gemm(packed, rows, cols, cb, x[33:34].contiguous(), tab, oi.size)
    assert torch.equal(y3[0], y1[33])


def test_gemm_pack_layout():
    """Per tile of 32 rows and 64 columns: 64 words of 16 bytes (row lane % 32, columns 32 (lane / 32) .. + 31), then
    64 constants; zeros past the last row and the last column."""
    rows, cols, block = 45, 2304 + 32, 32  # a ragged row tile and half a chunk at the end
    cb, codes, scales, _, _ = quantized(rows, cols, block, 1, 0, seed=83)
    packed = binding.bof4_gemm_pack(torch.from_numpy(codes).to(DEV), dev_u16(scales), rows, cols, block).cpu().numpy()
    n_chunks = (cols + 63) // 64
    assert packed.size == binding.bof4_gemm_packed_bytes(rows, cols) == 2 * n_chunks * (1024 + 128)
    tiles = packed.reshape(2, n_chunks, 1152)
    code_rows = codes.reshape(rows, cols // 2)
    scale_rows = scales.reshape(rows, cols // block)
    for rt, ch, lane in [(0, 0, 0), (0, 0, 33), (0, 5, 63), (1, 7, 12), (1, 36, 3), (1, 36, 35), (1, 2, 13), (1, 2, 45)]:
        row, c = rt * 32 + lane % 32, ch * 64 + 32 * (lane // 32)
        got_q = tiles[rt, ch, 16 * lane: 16 * lane + 16]
        got_m = tiles[rt, ch, 1024 + 2 * lane: 1024 + 2 * lane + 2].view(np.uint16)[0]
        if row < rows and c < cols:
            assert np.array_equal(got_q, code_rows[row, c // 2: c // 2 + 16]) and got_m == scale_rows[row, c // block]
        else:
            assert not got_q.any() and got_m == 0


def test_gemm_argument_errors():
    rows, cols, block = 64, 2048, 64
    cb, codes, scales, oi, ov = quantized(rows, cols, block, 1, 1, seed=81)
    cd, sd = torch.from_numpy(codes).to(DEV), dev_u16(scales)
    x = rand_x(3, cols, 1).to(DEV)
    with pytest.raises(binding.Bof4Error) as e:
        binding.bof4_gemm_pack(cd, sd, rows, 96, 64)
    assert e.value.code == binding.BOF4_ERR_ARG
    with pytest.raises(binding.Bof4Error) as e:
        binding.bof4_gemm_pack(cd, sd, rows, cols, 48)
    assert e.value.code == binding.BOF4_ERR_ARG
    with pytest.raises(binding.Bof4Error) as e:  # codes not 16-byte aligned
        binding.bof4_gemm_pack(cd[4:], sd, rows - 1, cols, block)
    assert e.value.code == binding.BOF4_ERR_ARG
    with pytest.raises(binding.Bof4Error) as e:
        binding.bof4_gemm_pack(cd, sd, rows, cols, block, out=torch.empty(1152 * 63, dtype=torch.uint8, device=DEV))
    assert e.value.code == binding.BOF4_ERR_WORKSPACE
    packed = binding.bof4_gemm_pack(cd, sd, rows, cols, block)
    need = binding.bof4_gemm_workspace_bytes(rows, cols, 3)
    # x twice (in product order and transposed, 32 token slots), then the partial results of four workgroups per row
    # tile (32 chunks of 64 columns, eight waves each)
    assert need == 2 * 32 * cols * 2 + 4 * 32 * rows * 4
    with pytest.raises(binding.Bof4Error) as e:
        binding.bof4_gemm(packed, rows, cols, cb, x, ws=torch.empty(need - 256, dtype=torch.uint8, device=DEV))
    assert e.value.code == binding.BOF4_ERR_WORKSPACE
    with pytest.raises(ValueError):
        binding.bof4_gemm(packed, rows, cols, cb, x, None, 3)  # outliers without their table
    with pytest.raises(ValueError):
        binding.bof4_gemm(packed, rows, cols, cb, x.float())
    with pytest.raises(ValueError):
        binding.bof4_gemm(packed, rows + 1, cols, cb, x)  # a packed copy of fewer row tiles
    big = 32768 + 2048
    with pytest.raises(binding.Bof4Error) as e:
        binding.bof4_gemm(torch.zeros(binding.bof4_gemm_packed_bytes(1, big), dtype=torch.uint8, device=DEV), 1, big, cb,
                          torch.zeros((1, big), dtype=torch.bfloat16, device=DEV))
    assert e.value.code == binding.BOF4_ERR_ARG
    bad_cb = cb.copy()
    bad_cb[3] = bad_cb[4]
    with pytest.raises(binding.Bof4Error):
        binding.bof4_gemm(packed, rows, cols, bad_cb, x)


@pytest.mark.parametrize("rows,cols,n_tokens", [(4096, 4096, 32), (4096, 11008, 32), (11008, 4096, 64),
                                                (8192, 28672, 8)])
def test_gemm_llama_matrices_with_opq(rows, cols, n_tokens):
    """The three matrix shapes of workload 1 and the widest one of workload 4 at full size, signed constants, block 64,
    OPQ q = 0.95: every output against the oracle."""
    wm = inputs.student_t_matrix(rows, cols, 5.0, 0.02, 0.3, seed=rows + cols)
    cb = cb_for(64, 1)
    T = oracle.opq_threshold(0.95, 64)
    st, codes, scales, oi, ov, k = oracle.quantize(inputs.bits(wm.reshape(-1)), 64, cb, 1, opq_T=T)
    assert st == oracle.OK and k > 1000
    check(cb, codes, scales, oi, ov, rows, cols, 64, rand_x(n_tokens, cols, 9))
