"""Benchmark of the BOF4 hot path on one MI355X.

Default workload (`--config 4`): layers of the Llama-70B-shaped stack (855,638,016 bf16 weights each, Student-t(4),
std 0.015), block 64, signed absmax (BOF4-S) + OPQ at q = 0.95.  A "step" is one pass of the whole hot path over
`--layers` distinct resident layers, one after the other:
    bof4_quantize_lloyd (one pass: OPQ statistics, outlier extraction, absmax, normalise, assign, pack, and the
        per-level sums of eq. 6 on the same normalised weights, outliers excluded)  ->  bof4_codebook_update (host)
    bof4_dequantize (decode + outlier write-back)
(`--unfused` takes bof4_quantize and bof4_lloyd_step as two passes instead.)
Inputs are resident in HBM before the timed region; a layer (1.7 GB) is far larger than the last-level cache, and
successive calls walk different layers.  `--config 0..3` run the other workloads (see WORKLOADS below); `--config 2`
is the 13 GB Lloyd loop.

Prints ONE JSON line: whole-path throughput in GB/s of bf16 weights, per-call kernel times (HIP events recorded by
the library right around each main kernel, inside the timed region) with their fraction of the 8 TB/s data sheet
peak and of the measured plain-streaming ceiling of the same read:write mix, the roofline record of the kernel with
the longest duration, and the CPU oracle timed on a bounded sample (one thread and all cores, per call).
"""
import argparse
import ctypes
import json
import os
import subprocess
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2505_06653_amd import binding, codebooks, inputs  # noqa: E402

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
CEIL_SRC = os.path.join(ROOT, "bench_ceilings.hip")
CEIL_LIB = os.path.join(ROOT, "libbench_ceilings.so")

# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command (each counter scaled by what
# it reads for the plain copy at the end of the run); keyed by (config, block, kernel).  Filled in from the summaries
# under profiles/ named beside each entry; a workload or kernel without a profile reports null.
PROFILED_TRAFFIC = {
    (4, 64, "quantize_lloyd"): (1_907_670_111 + 584_580_390, "profiles/bench_config4_block64_opq_hbm_traffic.md: "
                                "seg_pass_kernel<64, true, true, true, true>, fetched + written per launch"),
    (4, 64, "dequantize"): (538_325_903 + 1_710_990_916, "profiles/bench_config4_block64_opq_hbm_traffic.md: "
                            "dequantize_kernel<64>, fetched + written per launch"),
}


def build_ceilings():
    """Compile bench_ceilings.hip (plain streaming kernels, benchmark-only) for gfx950."""
    cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC", "-Xclang", "-target-feature",
           "-Xclang", "-packed-fp32-ops", "-o", CEIL_LIB, CEIL_SRC]
    subprocess.run(cmd, check=True)
    return CEIL_LIB


CEILING_KINDS = (("read", 0, 1, 0), ("write", 1, 0, 1), ("copy_1_1", 2, 1, 1), ("read4_write1", 3, 4, 1),
                 ("read1_write4", 4, 1, 4))


def measure_ceilings(n_weights, dev, grids=(1024, 2048, 4096, 8192, 0), reps=5, full=False):
    """Plain streaming kernels on buffers of the workload's size (a read stream of 2 bytes per weight, or a write
    stream of that size for the write-heavy mixes): GB/s of total traffic, best over the launch shapes tried."""
    if not os.path.exists(CEIL_LIB):
        raise ImportError(f"{CEIL_LIB} not built - run `python -c 'import __graft_entry__ as g; g.build()'`")
    L = ctypes.CDLL(CEIL_LIB)
    L.bench_ceiling.restype = ctypes.c_int
    L.bench_ceiling.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint32,
                                ctypes.c_int, ctypes.c_void_p, ctypes.POINTER(ctypes.c_float)]
    big = 2 * n_weights // 4096 * 4096  # bytes of the larger stream
    a = torch.empty(big, dtype=torch.uint8, device=dev)
    b = torch.empty(big, dtype=torch.uint8, device=dev)
    a.fill_(1)
    out, table = {}, {}
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    for name, kind, r, w in CEILING_KINDS:
        n_groups = big // (4096 * max(r, w))
        total = (r + w) * 4096 * n_groups
        best = 0.0
        for g in grids:
            grid = n_groups if g == 0 else min(g, n_groups)
            ms = ctypes.c_float(0.0)
            if L.bench_ceiling(kind, a.data_ptr(), b.data_ptr(), n_groups, grid, reps, stream, ctypes.byref(ms)) != 0:
                raise RuntimeError("bench_ceiling failed")
            rate = total / (ms.value * 1e-3) / 1e9
            table[f"{name}@grid{grid}"] = rate
            best = max(best, rate)
        out[name] = best
    torch.cuda.synchronize()
    del a, b
    if full:
        out["by_launch_shape"] = table
    return out


# ------------------------------------------------------------------------------------------------ workloads
def step_calls(args):
    return ("quantize", "lloyd_step", "dequantize") if args.unfused else ("quantize_lloyd", "dequantize")


def step_text(args):
    return "quantize + lloyd_step" if args.unfused else "quantize_lloyd (quantiser and Lloyd sums in one pass)"


def make_workload(cfg, args, dev):
    """Returns dict: tensors (flat bf16, resident), block, signed, T (OPQ threshold or 0), cb, pin, calls (which of
    quantize / lloyd_step / dequantize a step runs), lloyd_T, per_step (tensors walked per step), desc, matrices."""
    block = args.block
    if cfg == 0:
        ts = [inputs.gaussian_matrix(1024, 1024, 0.02, seed=0, device=dev).reshape(-1)]
        return dict(tensors=ts, block=64, signed=1, T=0.0, lloyd_T=0.0, cb=codebooks.gaussian_quantile_init(),
                    pin=codebooks.PIN_BOF4S, calls=step_calls(args), per_step=1, move_cb=True, matrices=None,
                    desc="configs[0]: 1024x1024 N(0,0.02^2), block 64, signed absmax; step = " + step_text(args) +
                         " + codebook_update + dequantize (cache-resident, launch-bound)")
    if cfg in (1, 3):
        ts = []
        for r in range(args.replicas):
            mats = inputs.llama7b_block(seed=50 + r, device=dev)
            if cfg == 3:
                for k, (_, m) in enumerate(mats):
                    inputs.plant_outliers(m, seed=300 + 16 * r + k)
            ts.append(inputs.flatten(mats))
        signed = args.signed
        cbk = codebooks.BOF4S_MSE[block] if signed else codebooks.BOF4_MSE_64
        T = binding.bof4_opq_threshold(0.95, block) if cfg == 3 else 0.0
        return dict(tensors=ts, block=block, signed=signed, T=T, lloyd_T=T, cb=codebooks.array(cbk),
                    pin=codebooks.PIN_BOF4S if signed else codebooks.PIN_BOF4, calls=("quantize", "dequantize"),
                    per_step=1, move_cb=False, matrices=(("qkv", 3 * 4096, 4096), ("o", 4096, 4096),
                                                          ("gate_up", 2 * 11008, 4096), ("down", 4096, 11008)),
                    desc=(f"configs[{cfg}]: one Llama-7B-shaped block, 202,375,168 bf16 weights, Student-t(5) std 0.02 "
                          f"with log-normal(0,0.3) row scale" + (", 0.1% planted outliers, OPQ q=0.95" if cfg == 3 else "")
                          + f", block {block}, {'signed' if signed else 'absolute'} absmax, fixed codebook; step = "
                            f"quantize + dequantize on one of {args.replicas} rotating copies"))
    if cfg == 2:
        parts = [inputs.flatten(inputs.llama7b_block(seed=1000 + b, device=dev)) for b in range(args.blocks)]
        w = torch.cat(parts)
        del parts
        return dict(tensors=[w], block=64, signed=1, T=0.0, lloyd_T=0.0, cb=codebooks.gaussian_quantile_init(),
                    pin=codebooks.PIN_BOF4S, calls=("lloyd_step",), per_step=1, move_cb=True, matrices=None,
                    desc=f"configs[2]: {args.blocks} Llama-7B-shaped blocks resident ({w.numel()} bf16 weights, "
                         f"{2 * w.numel() / 1e9:.2f} GB), block 64, signed absmax; step = one Lloyd/EM iteration "
                         f"(bof4_lloyd_step over all weights + codebook_update), codebook from the quantile start")
    if cfg == 4:
        ts = [inputs.flatten(inputs.llama70b_layer(seed=4000 + k, device=dev)) for k in range(args.layers)]
        T = binding.bof4_opq_threshold(0.95, block)
        return dict(tensors=ts, block=block, signed=1, T=T, lloyd_T=T, cb=codebooks.array(codebooks.BOF4S_MSE[block]),
                    pin=codebooks.PIN_BOF4S, calls=step_calls(args), per_step=args.layers,
                    move_cb=True, matrices=(("qkv", 8192 + 2 * 1024, 8192), ("o", 8192, 8192),
                                            ("gate_up", 2 * 28672, 8192), ("down", 8192, 28672)),
                    desc=f"configs[4]: Llama-70B-shaped layers (855,638,016 bf16 weights each, Student-t(4) std 0.015), "
                         f"block {block}, signed absmax (BOF4-S) + OPQ q=0.95; step = {step_text(args)} (outliers "
                         f"excluded from the sums) + codebook_update + dequantize on each of {args.layers} distinct "
                         f"resident layers in turn")
    raise ValueError("config must be 0..4")


def alg_bytes_per_weight(call, block, rho):
    """Algorithmic bytes per weight of one launch (one launch processes all weights of the call)."""
    if call == "lloyd_step":
        return 2.0
    return 2.0 + 0.5 + 2.0 / block + 10.0 * rho  # quantize: read 2, write the rest; dequantize: the reverse


CEILING_OF_CALL = {"quantize": "read4_write1", "quantize_lloyd": "read4_write1", "dequantize": "read1_write4",
                   "lloyd_step": "read"}


# ------------------------------------------------------------------------------------------------ decoder in use
def _matrix_views(mats_spec, codes, scales, oidx, oval, k_all, block, dev):
    off, idx_all = 0, oidx[:k_all] if k_all else None
    for name, r, c in mats_spec:
        nw = r * c
        if k_all:
            a, b = (int(v) for v in torch.searchsorted(idx_all, torch.tensor([off, off + nw], device=dev)))
        else:
            a = b = 0
        yield name, r, c, codes[off // 2:(off + nw) // 2], scales[off // block:(off + nw) // block], \
            ((idx_all[a:b] - off).contiguous() if b > a else None), (oval[a:b].contiguous() if b > a else None), b - a
        off += nw


def gemv_pass(mats_spec, codes, scales, oidx, oval, k_all, cb, block, dev, passes=20):
    """The decoder in use (not part of the timed step): one token through the quantised matrices as the last step left
    them, y = W~ x per matrix with bof4_gemv, outliers included.  Projections that read the same input are one matrix
    (adjacent in the flat tensor)."""
    mats = []
    for name, r, c, mc, ms, mi, mv, k in _matrix_views(mats_spec, codes, scales, oidx, oval, k_all, block, dev):
        tab = binding.bof4_gemv_outlier_table(mc, ms, r, c, block, cb, mi, mv, n_outliers=k) if k else None
        x = torch.randn((1, c), device=dev).to(torch.bfloat16)
        y = torch.empty((1, r), dtype=torch.float32, device=dev)
        mats.append((r, c, mc, ms, tab, k, x, y))

    def one_pass():
        for r, c, mc, ms, tab, k, x, y in mats:
            binding.bof4_gemv(mc, ms, r, c, block, cb, x, tab, k, out=y)
    for _ in range(3):
        one_pass()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(passes):
        one_pass()
    e1.record()
    torch.cuda.synchronize()
    ms_ = e0.elapsed_time(e1) / passes
    nbytes = sum((0.5 + 2.0 / block) * m[0] * m[1] + 8.0 * m[5] for m in mats)
    return {"ms": ms_, "GBps_algorithmic": nbytes / (ms_ * 1e-3) / 1e9, "hbm_frac": nbytes / (ms_ * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "outliers": int(sum(m[5] for m in mats)),
            "note": "bof4_gemv per matrix (qkv, o, gate+up, down; one token, fp32 accumulation), back to back on one "
                    "stream, outside the timed step"}


def gemm_pass(mats_spec, codes, scales, oidx, oval, k_all, cb, block, dev, n_tokens=128, passes=10):
    """As gemv_pass, for 128 tokens at once with bof4_gemm (matrix cores; the matrices packed once)."""
    mats = []
    for name, r, c, mc, ms, mi, mv, k in _matrix_views(mats_spec, codes, scales, oidx, oval, k_all, block, dev):
        packed = binding.bof4_gemm_pack(mc, ms, r, c, block)
        tab = binding.bof4_gemm_outlier_table(mc, ms, r, c, block, cb, mi, mv, n_outliers=k) if k else None
        x = torch.randn((n_tokens, c), device=dev).to(torch.bfloat16)
        y = torch.empty((n_tokens, r), dtype=torch.float32, device=dev)
        ws = torch.empty(binding.bof4_gemm_workspace_bytes(r, c, n_tokens), dtype=torch.uint8, device=dev)
        mats.append((r, c, packed, tab, k, x, y, ws))

    def one_pass():
        for r, c, packed, tab, k, x, y, ws in mats:
            binding.bof4_gemm(packed, r, c, cb, x, tab, k, out=y, ws=ws)
    for _ in range(3):
        one_pass()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(passes):
        one_pass()
    e1.record()
    torch.cuda.synchronize()
    ms_ = e0.elapsed_time(e1) / passes
    flops = sum(2.0 * m[0] * m[1] * n_tokens for m in mats)
    return {"ms": ms_, "tokens": n_tokens, "TFLOPs": flops / (ms_ * 1e-3) / 1e12,
            "mfma_frac": flops / (ms_ * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, "outliers": int(sum(m[4] for m in mats)),
            "note": "bof4_gemm per matrix (packed once; bf16 weights decoded in registers, fp32 accumulation on the "
                    "matrix cores), back to back on one stream, outside the timed step"}


def gemv_shapes(dev, calls=50):
    """bof4_gemv on the matrix shapes of workloads 1 and 4 (Student-t weights, block 64, signed, with and without the
    OPQ outliers, one and two tokens): microseconds per call from HIP events around `calls` back-to-back calls."""
    block = 64
    cb = codebooks.array(codebooks.BOF4S_MSE[block])
    T = binding.bof4_opq_threshold(0.95, block)
    rows_out = []
    for rows, cols in ((4096, 4096), (12288, 4096), (22016, 4096), (4096, 11008), (8192, 28672), (28672, 8192)):
        w = inputs.student_t_matrix(rows, cols, 5.0, 0.02, 0.3, seed=rows + cols, device=dev).reshape(-1)
        n = rows * cols
        for opq in (0, 1):
            codes, scales, oi, ov, k = binding.bof4_quantize(w, block, cb, 1, opq_T=T if opq else 0.0,
                                                             out_capacity=n // 50 if opq else 0)
            tab = binding.bof4_gemv_outlier_table(codes, scales, rows, cols, block, cb, oi, ov, n_outliers=k) if opq else None
            for nt in (1, 2):
                x = torch.randn((nt, cols), device=dev).to(torch.bfloat16)
                y = torch.empty((nt, rows), dtype=torch.float32, device=dev)
                for _ in range(5):
                    binding.bof4_gemv(codes, scales, rows, cols, block, cb, x, tab, k if opq else 0, out=y)
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(calls):
                    binding.bof4_gemv(codes, scales, rows, cols, block, cb, x, tab, k if opq else 0, out=y)
                e1.record()
                torch.cuda.synchronize()
                us = e0.elapsed_time(e1) * 1e3 / calls
                nbytes = (0.5 + 2.0 / block) * n + 8.0 * (k if opq else 0)
                rows_out.append({"rows": rows, "cols": cols, "outliers": int(k) if opq else 0, "tokens": nt,
                                 "us_per_call": us, "GBps_algorithmic": nbytes / us / 1e3,
                                 "hbm_frac": nbytes / us / 1e3 / HBM_PEAK_GBS})
        del w
    return rows_out


def gemm_shapes(dev, calls=30):
    """bof4_gemm on the matrix shapes of workloads 1 and 4 (Student-t weights, block 64, signed, with and without the
    OPQ outliers, 32 and 128 tokens): microseconds per call (all its kernels) from HIP events around `calls`
    back-to-back calls; next to it, on the same decoded matrix, bof4_dequantize and the library's bfloat16 product
    (torch.matmul), the path the fused call replaces."""
    block = 64
    cb = codebooks.array(codebooks.BOF4S_MSE[block])
    T = binding.bof4_opq_threshold(0.95, block)

    def timed(f):
        for _ in range(3):
            f()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(calls):
            f()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / calls

    rows_out = []
    for rows, cols in ((4096, 4096), (12288, 4096), (22016, 4096), (4096, 11008), (8192, 28672), (28672, 8192)):
        w = inputs.student_t_matrix(rows, cols, 5.0, 0.02, 0.3, seed=rows + cols, device=dev).reshape(-1)
        n = rows * cols
        for opq in (0, 1):
            codes, scales, oi, ov, k = binding.bof4_quantize(w, block, cb, 1, opq_T=T if opq else 0.0,
                                                             out_capacity=n // 50 if opq else 0)
            k = int(k) if opq else 0
            packed = binding.bof4_gemm_pack(codes, scales, rows, cols, block)
            tab = binding.bof4_gemm_outlier_table(codes, scales, rows, cols, block, cb, oi, ov, n_outliers=k) if k else None
            deq = torch.empty(n, dtype=torch.bfloat16, device=dev)
            us_deq = timed(lambda: binding.bof4_dequantize(codes, scales, n, block, cb, oi, ov, n_outliers=k, out=deq))
            wm = deq.reshape(rows, cols)
            for nt in (32, 128):
                x = torch.randn((nt, cols), device=dev).to(torch.bfloat16)
                y = torch.empty((nt, rows), dtype=torch.float32, device=dev)
                ws = torch.empty(binding.bof4_gemm_workspace_bytes(rows, cols, nt), dtype=torch.uint8, device=dev)
                us = timed(lambda: binding.bof4_gemm(packed, rows, cols, cb, x, tab, k, out=y, ws=ws))
                us_mm = timed(lambda: torch.matmul(x, wm.T))
                nbytes = (0.5 + 2.0 / 32) * n * ((nt + 127) // 128) + 8.0 * k
                rows_out.append({"rows": rows, "cols": cols, "outliers": k, "tokens": nt, "us_per_call": us,
                                 "GBps_algorithmic": nbytes / us / 1e3, "hbm_frac": nbytes / us / 1e3 / HBM_PEAK_GBS,
                                 "TFLOPs": 2.0 * n * nt / us / 1e6,
                                 "mfma_frac": 2.0 * n * nt / us / 1e6 / MFMA_BF16_PEAK_TFLOPS,
                                 "us_dequantize": us_deq, "us_bf16_matmul_on_decoded": us_mm})
            del deq, wm, packed
        del w
    return rows_out


# ------------------------------------------------------------------------------------------------ CPU oracle
def cpu_baseline(w_dev, wl, sample_weights):
    """The oracle as it stands on a bounded sample of the workload (the first `sample_weights` weights of one resident
    tensor), each call of the step timed on one thread and on all host threads.  quantize / dequantize of the oracle
    are single-threaded loops over independent blocks: the all-threads figure runs them on contiguous block ranges in
    Python threads (oracle.parallel); its Lloyd step has its own OpenMP loop, limited through omp_set_num_threads."""
    import oracle
    from oracle import parallel as opar
    block, cb, signed, T = wl["block"], wl["cb"], wl["signed"], wl["T"]
    n = min(int(w_dev.numel()), sample_weights) // 4096 * 4096
    wb = inputs.bits(w_dev[:n])
    threads = oracle.num_threads()
    gomp = ctypes.CDLL("libgomp.so.1")

    def run(workers):
        gomp.omp_set_num_threads(workers)
        t = {}
        t0 = time.perf_counter()
        codes, scales, oidx, oval, nout = opar.quantize(wb, block, cb, signed, T, workers=workers)
        t["quantize"] = time.perf_counter() - t0
        t0 = time.perf_counter()
        opar.dequantize(codes, scales, n, block, cb, oidx if T > 0 else None, oval if T > 0 else None, workers=workers)
        t["dequantize"] = time.perf_counter() - t0
        t0 = time.perf_counter()
        oracle.lloyd_step(wb, block, cb, signed, opq_T=wl["lloyd_T"])
        t["lloyd_step"] = time.perf_counter() - t0
        return t
    one, many = run(1), run(threads)
    gomp.omp_set_num_threads(threads)
    # the oracle has no fused call: its step is the same work as two functions
    calls = [c for call in wl["calls"] for c in (("quantize", "lloyd_step") if call == "quantize_lloyd" else (call,))]

    def table(t):
        d = {c: {"seconds": t[c], "weights_per_s": n / t[c], "GBps_bf16": 2.0 * n / t[c] / 1e9} for c in calls}
        d["step_GBps_bf16"] = 2.0 * n / sum(t[c] for c in calls) / 1e9
        return d
    return {"value": 2.0 * n / sum(many[c] for c in calls) / 1e9, "unit": "GB/s", "cores": threads, "kind": "oracle",
            "sample": f"the first {n} weights of one resident tensor of the workload (same block size, codebook, OPQ "
                      f"threshold); every call of the step timed once on 1 thread and once on {threads} threads; "
                      f"value = all-threads rate of the whole step; no extrapolation: rates are per weight",
            "single_thread": table(one), "all_threads": table(many)}


# ------------------------------------------------------------------------------------------------ config 4, whole
def stack_run(dev, layers=80, blocks=(64, 128, 256)):
    """The Llama-70B-shaped stack (80 layers, 68,451,041,280 weights, 136.9 GB) does not fit beside its decoded copy,
    so the layers are generated (seed 4000 + layer), quantised with the Lloyd sums taken in the same pass, and
    decoded one at a time into the same buffers; the sums are added up over the stack (fixed layer order) and give
    one codebook update.  GPU time = HIP events around the calls of a layer, generation excluded."""
    n = 855_638_016
    out = {"workload": "configs[4] whole: 80 layers x 855,638,016 weights, signed absmax + OPQ q=0.95, "
                       "quantize_lloyd + dequantize per layer", "per_block": {}}
    for block in blocks:
        T = binding.bof4_opq_threshold(0.95, block)
        cb = codebooks.array(codebooks.BOF4S_MSE[block])
        cap = n // 32
        codes = torch.empty(n // 2, dtype=torch.uint8, device=dev)
        scales = torch.empty(n // block, dtype=torch.float16, device=dev)
        oidx = torch.empty(cap, dtype=torch.int64, device=dev)
        oval = torch.empty(cap, dtype=torch.float16, device=dev)
        deq = torch.empty(n, dtype=torch.bfloat16, device=dev)
        ws = binding.alloc_workspace(n, block, cap, dev)
        tot = {"num": np.zeros(16), "den": np.zeros(16), "cnt": np.zeros(16, dtype=np.uint64), "sse": 0.0}
        n_out, gpu_ms = 0, 0.0
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for layer in range(layers):
            w = inputs.flatten(inputs.llama70b_layer(seed=4000 + layer, device=dev))
            e0.record()
            k, g = binding.bof4_quantize_lloyd(w, block, cb, 1, opq_T=T, out_capacity=cap, codes=codes, scales=scales,
                                               out_idx=oidx, out_val=oval, ws=ws, trim=False)[4:6]
            binding.bof4_dequantize(codes, scales, n, block, cb, oidx, oval, out=deq, n_outliers=k)
            e1.record()
            torch.cuda.synchronize()
            gpu_ms += e0.elapsed_time(e1)
            n_out += k
            for f in ("num", "den", "cnt"):
                tot[f] += g[f]
            tot["sse"] += g["sse"]
            del w
        used = layers * n - n_out
        new_cb = binding.bof4_codebook_update({**tot, "n_used": used, "n_outliers": n_out}, codebooks.PIN_BOF4S, cb)
        out["per_block"][str(block)] = {
            "weights": layers * n, "outliers": n_out, "outlier_fraction": n_out / (layers * n),
            "mse": tot["sse"] / used, "gpu_ms_total": gpu_ms, "GBps_bf16": 2.0 * layers * n / (gpu_ms * 1e-3) / 1e9,
            "levels_after_one_step": [float(v) for v in new_cb]}
    return out


# ------------------------------------------------------------------------------------------------ main
def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--config", type=int, default=4, help="workload: index into BASELINE.json's configs (default 4: "
                    "Llama-70B-shaped layers, the largest single-GPU workload with the whole path)")
    ap.add_argument("--layers", type=int, default=8, help="config 4: distinct resident layers walked per step")
    ap.add_argument("--blocks", type=int, default=32, help="config 2: Llama-7B-shaped blocks resident")
    ap.add_argument("--replicas", type=int, default=3, help="configs 1, 3: rotating copies of the block")
    ap.add_argument("--block", type=int, default=64, help="block size I (configs 1, 3, 4)")
    ap.add_argument("--signed", type=int, default=1, help="configs 1: signed (1) or absolute (0) absmax")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the calls timed outside the step (MAE step, error "
                    "pass, decoder inside the products)")
    ap.add_argument("--cpu-sample", type=int, default=1 << 27, help="weights in the CPU oracle's sample")
    ap.add_argument("--unfused", action="store_true", help="bof4_quantize and bof4_lloyd_step as two passes over the "
                    "weights instead of bof4_quantize_lloyd")
    ap.add_argument("--serial", action="store_true",
                    help="every call waits for its result before the next is enqueued (default: the Lloyd kernels are "
                         "enqueued behind the quantiser before the host waits for the outlier count)")
    ap.add_argument("--stack", action="store_true",
                    help="instead of the benchmark step: config 4 taken whole - all 80 layers (one resident at a time, each "
                         "from its own seed) x block sizes 64, 128, 256 through quantize_lloyd + dequantize, totals "
                         "summed; one JSON line")
    ap.add_argument("--ceilings", action="store_true",
                    help="instead of the benchmark step: the plain streaming kernels over all launch shapes, one JSON line")
    ap.add_argument("--gemv-shapes", action="store_true",
                    help="instead of the benchmark step: bof4_gemv on a table of matrix shapes, one JSON line")
    ap.add_argument("--gemm-shapes", action="store_true",
                    help="instead of the benchmark step: bof4_gemm (32 and 128 tokens) on the same table, one JSON line")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is single-GPU; run with --gpus 1 (how the path would shard is part of the design notes)",
              file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.gemv_shapes:
        print(json.dumps({"bof4_gemv": gemv_shapes(dev)}))
        return
    if args.gemm_shapes:
        print(json.dumps({"bof4_gemm": gemm_shapes(dev)}))
        return
    if args.ceilings:
        n = 855_638_016
        print(json.dumps({"ceilings_GBps": measure_ceilings(n, dev, reps=10, full=True), "n_weights": n,
                          "note": "plain 16-byte nontemporal streaming kernels (bench_ceilings.hip), total traffic "
                                  "(read + written) per second; per mix the best launch shape"}))
        return
    binding.lib()
    if args.stack:
        print(json.dumps(stack_run(dev)))
        return
    if args.steps is None:
        args.steps = {0: 200, 1: 50, 2: 100, 3: 50, 4: 20}[args.config]
    if args.warmup is None:
        args.warmup = {0: 50, 1: 20, 2: 5, 3: 20, 4: 5}[args.config]

    wl = make_workload(args.config, args, dev)
    tensors, block, signed, T, pin = wl["tensors"], wl["block"], wl["signed"], wl["T"], wl["pin"]
    calls, per_step = wl["calls"], wl["per_step"]
    cb = wl["cb"]
    n = tensors[0].numel()
    assert all(t.numel() == n for t in tensors)
    do_f = "quantize_lloyd" in calls
    do_q, do_l, do_d = "quantize" in calls or do_f, "lloyd_step" in calls or do_f, "dequantize" in calls
    cap = n // 64 if T > 0 else 0
    if do_q:
        codes = torch.empty(n // 2, dtype=torch.uint8, device=dev)
        scales = torch.empty(n // block, dtype=torch.float16, device=dev)
        oidx = torch.empty(max(cap, 1), dtype=torch.int64, device=dev)
        oval = torch.empty(max(cap, 1), dtype=torch.float16, device=dev)
        ws = binding.alloc_workspace(n, block, cap, dev)
    if do_d:
        deq = torch.empty(n, dtype=torch.bfloat16, device=dev)
    ws_lloyd = binding.alloc_workspace(n, block, 0, dev)  # the Lloyd kernels run between the halves of the quantiser
    stats_rec, _keep1 = binding.pinned_lloyd_stats()     # results land in pinned host memory: no copy
    counter, _keep2 = binding.pinned_counter()
    # Kernel-level HIP events, recorded by the library right around the main kernel of a call (bof4_time_next_call).
    # An event record costs a few microseconds of stream time, so every tensor of a timed step brackets one kernel
    # only: the kernels of the enabled calls in turn.
    n_items = args.steps * per_step
    kev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(n_items)]
    for row in kev:
        for e in row:
            e.record()  # creates the HIP handle
    state = {"cb": cb, "k": 0, "mse": []}

    def item(j, timed_call=None, events=None, serial=False):
        """The calls of the step on tensor j.  Pipelined (default): quantiser kernels, Lloyd kernels (they do not
        depend on the quantiser), then the host collects the outlier count, enqueues the decoder, collects the sums and
        updates the codebook while the decoder runs.  serial: each call waits for its result."""
        w = tensors[j % len(tensors)]
        cb = state["cb"]
        k = 0
        if events:
            events[0].record()
        if do_f:
            if timed_call == "quantize_lloyd":
                binding.bof4_time_next_call(kev[j][0], kev[j][1])
            if serial:
                k = binding.bof4_quantize_lloyd(w, block, cb, signed, opq_T=T, out_capacity=cap, codes=codes,
                                                scales=scales, out_idx=oidx, out_val=oval, ws=ws, counter=counter,
                                                stats=stats_rec, trim=False, raw=True)[4]
            else:
                flight = binding.bof4_quantize_lloyd_begin(w, block, cb, signed, T, cap, codes, scales, oidx, oval, ws,
                                                           counter, stats_rec)
        elif do_q:
            if timed_call == "quantize":
                binding.bof4_time_next_call(kev[j][0], kev[j][1])
            if serial:
                k = binding.bof4_quantize(w, block, cb, signed, opq_T=T, out_capacity=cap, codes=codes, scales=scales,
                                          out_idx=oidx, out_val=oval, ws=ws, counter=counter, trim=False)[4]
            else:
                flight = binding.bof4_quantize_begin(w, block, cb, signed, T, cap, codes, scales, oidx, oval, ws, counter)
        if events:
            events[1].record()
        if do_l and not do_f:
            if timed_call == "lloyd_step":
                binding.bof4_time_next_call(kev[j][0], kev[j][1])
            if serial:
                binding.bof4_lloyd_step(w, block, cb, signed, opq_T=wl["lloyd_T"], ws=ws_lloyd, raw=True, out=stats_rec)
            else:
                binding.bof4_lloyd_step_begin(w, block, cb, signed, stats_rec, opq_T=wl["lloyd_T"], ws=ws_lloyd)
        if events:
            events[2].record()
        if do_q and not serial:
            k = flight.finish()
        if do_d:
            if timed_call == "dequantize":
                binding.bof4_time_next_call(kev[j][0], kev[j][1])
            binding.bof4_dequantize(codes, scales, n, block, cb, oidx if k else None, oval if k else None, out=deq,
                                    n_outliers=k)
        if events:
            events[3].record()
        if do_l:
            if not serial:
                binding.bof4_wait_result(stats_rec)
            if wl["move_cb"]:
                state["cb"] = binding.bof4_codebook_update(stats_rec, pin, cb)
            state["mse"].append(stats_rec.sse / max(stats_rec.n_used, 1))
        state["k"] = k

    for i in range(args.warmup * per_step):
        item(i, serial=args.serial)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for j in range(n_items):
        item(j, timed_call=calls[j % len(calls)], serial=args.serial)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    mse_last = state["mse"][-1] if state["mse"] else None
    mse_trace = state["mse"][args.warmup * per_step:] if args.config == 2 else None

    # per-call times (kernels, helper kernels and host waits of one call), from a few extra serial items outside the
    # timed region so that their event records do not slow the timed one
    n_extra = 6
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(n_extra)]
    for i in range(n_extra):
        item(n_items + i, events=ev[i], serial=True)
    torch.cuda.synchronize()
    call_ms = {nm: float(np.mean([ev[i][k].elapsed_time(ev[i][k + 1]) for i in range(n_extra)]))
               for k, nm in enumerate(("quantize_lloyd" if do_f else "quantize", "lloyd_step", "dequantize")) if nm in calls}
    kms = {}
    for c, nm in enumerate(calls):
        samples = [kev[j][0].elapsed_time(kev[j][1]) for j in range(n_items) if j % len(calls) == c]
        kms[nm] = float(np.mean(samples)) if samples else float("nan")
    rho = state["k"] / n
    ceilings = measure_ceilings(n, dev) if n >= (1 << 24) else None
    per_call = {}
    for nm in calls:
        ab = alg_bytes_per_weight(nm, block, rho) * n
        rate = ab / (kms[nm] * 1e-3) / 1e9
        per_call[nm] = {"call_ms": call_ms[nm], "kernel_ms": kms[nm], "GBps_bf16": 2.0 * n / (kms[nm] * 1e-3) / 1e9,
                        "weights_per_s": n / (kms[nm] * 1e-3), "GBps_algorithmic": rate, "hbm_frac": rate / HBM_PEAK_GBS}
        if ceilings:
            per_call[nm]["ceiling"] = CEILING_OF_CALL[nm]
            per_call[nm]["ceiling_frac"] = rate / ceilings[CEILING_OF_CALL[nm]]
    dominant = max(calls, key=lambda c: kms[c] if kms[c] == kms[c] else -1.0)
    achieved = per_call[dominant]["GBps_algorithmic"]
    prof = PROFILED_TRAFFIC.get((args.config, block, dominant))
    out = {
        "metric": "GB/s bf16 weights quantized & weights/s per Lloyd step; % of HBM peak",
        "value": 2.0 * n * n_items / dt / 1e9, "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": dt / args.steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16 in, f32 normalise/assign, f64 sums", "data": "synthetic",
        "config": {"workload": wl["desc"], "n_weights_per_tensor": n, "tensors_per_step": per_step,
                   "resident_tensors": len(tensors), "block": block, "outlier_fraction": rho,
                   "enqueue_order": "one call after the other, each waiting for its result" if args.serial else
                                    "per tensor: pass kernels, outlier count, dequantize, lloyd sums + codebook update "
                                    "(one stream; the host never lets the GPU wait)"},
        "per_call": per_call,
        "roofline": {"bound": "hbm", "kernel": dominant, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": prof[0] if prof else None,
                     "traffic_source": prof[1] if prof else None},
    }
    if ceilings:
        out["ceilings_GBps"] = ceilings
    if do_l:
        out["lloyd_weights_per_s"] = n / (kms["quantize_lloyd" if do_f else "lloyd_step"] * 1e-3)
        out["mse_last"] = mse_last
    if mse_trace is not None:
        out["mse_per_iteration"] = mse_trace

    if not args.no_extras and n >= (1 << 24):
        w0 = tensors[0]
        # the MAE-criterion expectation step (weighted medians; not part of the timed step): wall time of a few calls
        mae_rec, _keep3 = binding.pinned_mae_stats()
        mae_cb = codebooks.array(codebooks.BOF4S_MAE_64 if signed else codebooks.BOF4_MAE_64)
        ws_mae = binding.alloc_workspace(n, block, 0, dev)
        binding.bof4_lloyd_step_mae(w0, block, mae_cb, signed, skip_mask=pin, ws=ws_mae, out=mae_rec)
        torch.cuda.synchronize()
        t_mae = time.perf_counter()
        for r in range(3):
            binding.bof4_lloyd_step_mae(tensors[r % len(tensors)], block, mae_cb, signed, skip_mask=pin, ws=ws_mae,
                                        out=mae_rec)
        torch.cuda.synchronize()
        t_mae = (time.perf_counter() - t_mae) / 3
        out["mae_step"] = {"call_ms": t_mae * 1e3, "weights_per_s": n / t_mae,
                           "note": "bof4_lloyd_step_mae (exact weighted medians of the free levels: a sampling pass over one "
                                   "tile in 16, one full pass over the weights that also writes the candidate "
                                   "list, the remaining passes over that list), outside the timed step"}
        # the error pass (MSE / MAE of the tensor against its quantised form; not part of the timed step)
        err_rec, _keep4 = binding.pinned_error_stats()
        err_ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        for e in err_ev:
            e.record()
        cbq = wl["cb"]
        binding.bof4_quant_error(w0, block, cbq, signed, opq_T=T, ws=ws_mae, out=err_rec)
        torch.cuda.synchronize()
        t_err = time.perf_counter()
        for r in range(3):
            if r == 2:
                binding.bof4_time_next_call(err_ev[0], err_ev[1])
            err = binding.bof4_quant_error(tensors[r % len(tensors)], block, cbq, signed, opq_T=T, ws=ws_mae, out=err_rec)
        torch.cuda.synchronize()
        t_err = (time.perf_counter() - t_err) / 3
        k_err = err_ev[0].elapsed_time(err_ev[1])
        out["quant_error"] = {"call_ms": t_err * 1e3, "kernel_ms": k_err,
                              "GBps_algorithmic": 2.0 * n / (k_err * 1e-3) / 1e9,
                              "hbm_frac": 2.0 * n / (k_err * 1e-3) / 1e9 / HBM_PEAK_GBS, "mse": err["sse"] / err["n"],
                              "mae": err["sae"] / err["n"],
                              "note": "bof4_quant_error (quantise, decode and compare in registers: 2 bytes per weight), "
                                      "outside the timed step"}
        del ws_mae
        if do_q and wl["matrices"]:
            # the decoder in use on the last quantised tensor (quantised once more with the fixed codebook)
            cbq = wl["cb"]
            k = binding.bof4_quantize(w0, block, cbq, signed, opq_T=T, out_capacity=cap, codes=codes, scales=scales,
                                      out_idx=oidx, out_val=oval, ws=ws, counter=counter, trim=False)[4]
            out["gemv_pass"] = gemv_pass(wl["matrices"], codes, scales, oidx, oval, k, cbq, block, dev)
            out["gemm_pass"] = gemm_pass(wl["matrices"], codes, scales, oidx, oval, k, cbq, block, dev)
    if do_d:
        # one plain device copy of known size (2 n bytes read, 2 n written), outside the timed region: the reference
        # against which a counter profile of this same command scales FETCH_SIZE / WRITE_SIZE
        deq.copy_(tensors[0])
        torch.cuda.synchronize()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(tensors[0], wl, args.cpu_sample)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
