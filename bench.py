"""Benchmark of the BOF4 hot path on one MI355X.

A "step" is one pass of the whole hot path over one Llama-7B-shaped transformer block of synthetic bf16 weights
(workload 1: 202,375,168 weights, block 64, signed absmax / BOF4-S codebook, OPQ at q = 0.95):
    bof4_quantize (outlier extraction, absmax, normalise, assign, pack)  ->  bof4_dequantize (decode + outlier
    scatter)  ->  bof4_lloyd_step (normalise, assign, per-level sums; as in the paper the codebook statistics are
    taken without outlier removal)  ->  bof4_codebook_update (host).
Inputs are resident in HBM before the timed region.  Successive steps rotate over several independently seeded
copies of the workload so that no step finds its input in the last-level cache.

Prints ONE JSON line: whole-path throughput in GB/s of bf16 weights, with per-call rates, the roofline record of
the dominant kernel (HIP-event timed) and the CPU oracle timed on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2505_06653_amd import binding, codebooks, inputs  # noqa: E402

HBM_PEAK_GBS = 8000.0
BLOCK = 64
# measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE on this command (see profiles/), bytes per launch
PROFILED_TRAFFIC_BYTES = {"lloyd_step": 405.4e6, "quantize": 530.1e6, "dequantize": 526.2e6}


def gemv_block_pass(codes, scales, oidx, oval, k_all, cb, dev, passes=20):
    """The decoder in use (not part of the timed step): one token through the quantised matrices of the block, as the
    last benchmark step left them (codes, constants and the outlier list of the flat tensor), y = W~ x per matrix with
    bof4_gemv, outliers included.  Projections that read the same input are one matrix, as an inference engine
    stores them (q, k, v are adjacent in the flat block, and so are gate and up).  Returns the time of one pass over
    the block and the rate on the algorithmic bytes (codes, constants, 8 bytes per outlier table entry)."""
    mats, off = [], 0
    idx_all = oidx[:k_all]
    for name, r, c in (("qkv", 3 * 4096, 4096), ("o", 4096, 4096), ("gate_up", 2 * 11008, 4096), ("down", 4096, 11008)):
        nw = r * c
        a, b = (int(v) for v in torch.searchsorted(idx_all, torch.tensor([off, off + nw], device=dev)))
        k = b - a
        mc, ms = codes[off // 2:(off + nw) // 2], scales[off // BLOCK:(off + nw) // BLOCK]
        tab = binding.bof4_gemv_outlier_table(mc, ms, r, c, BLOCK, cb, (idx_all[a:b] - off).contiguous(),
                                              oval[a:b].contiguous(), n_outliers=k) if k else None
        off += nw
        x = torch.randn((1, c), device=dev).to(torch.bfloat16)
        y = torch.empty((1, r), dtype=torch.float32, device=dev)
        mats.append((name, r, c, mc, ms, tab, k, x, y))
    def one_pass():
        for name, r, c, codes, scales, tab, k, x, y in mats:
            binding.bof4_gemv(codes, scales, r, c, BLOCK, cb, x, tab, k, out=y)
    for _ in range(3):
        one_pass()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(passes):
        one_pass()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / passes
    nbytes = sum((0.5 + 2.0 / BLOCK) * r * c + 8.0 * k for _, r, c, _, _, _, k, _, _ in mats)
    return {"ms": ms, "GBps_algorithmic": nbytes / (ms * 1e-3) / 1e9, "hbm_frac": nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "outliers": int(sum(m[6] for m in mats)),
            "note": "four bof4_gemv calls (qkv, o, gate+up, down of the block: all 202,375,168 weights; one token, "
                    "fp32 accumulation), back to back on one stream, outside the timed step"}


def gemm_block_pass(codes, scales, oidx, oval, k_all, cb, dev, n_tokens=128, passes=10):
    """As gemv_block_pass, for 128 tokens at once with bof4_gemm (matrix cores; the matrices packed once)."""
    mats, off = [], 0
    idx_all = oidx[:k_all]
    for name, r, c in (("qkv", 3 * 4096, 4096), ("o", 4096, 4096), ("gate_up", 2 * 11008, 4096), ("down", 4096, 11008)):
        nw = r * c
        a, b = (int(v) for v in torch.searchsorted(idx_all, torch.tensor([off, off + nw], device=dev)))
        k = b - a
        mc, ms = codes[off // 2:(off + nw) // 2], scales[off // BLOCK:(off + nw) // BLOCK]
        packed = binding.bof4_gemm_pack(mc, ms, r, c, BLOCK)
        tab = binding.bof4_gemm_outlier_table(mc, ms, r, c, BLOCK, cb, (idx_all[a:b] - off).contiguous(),
                                              oval[a:b].contiguous(), n_outliers=k) if k else None
        off += nw
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
    ms = e0.elapsed_time(e1) / passes
    flops = sum(2.0 * r * c * n_tokens for r, c, *_ in mats)
    return {"ms": ms, "tokens": n_tokens, "TFLOPs": flops / (ms * 1e-3) / 1e12,
            "mfma_frac": flops / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
            "outliers": int(sum(m[4] for m in mats)),
            "note": "four bof4_gemm calls (qkv, o, gate+up, down of the block, packed once; bf16 weights decoded "
                    "in registers, fp32 accumulation on the matrix cores), back to back on one stream, outside the "
                    "timed step"}


def gemv_shapes(dev, calls=50):
    """bof4_gemv on the matrix shapes of workloads 1 and 4 (Student-t weights, block 64, signed, with and without the
    OPQ outliers, one and two tokens): microseconds per call from HIP events around `calls` back-to-back calls."""
    cb = codebooks.array(codebooks.BOF4S_MSE[BLOCK])
    T = binding.bof4_opq_threshold(0.95, BLOCK)
    rows_out = []
    for rows, cols in ((4096, 4096), (12288, 4096), (22016, 4096), (4096, 11008), (8192, 28672), (28672, 8192)):
        w = inputs.student_t_matrix(rows, cols, 5.0, 0.02, 0.3, seed=rows + cols, device=dev).reshape(-1)
        n = rows * cols
        for opq in (0, 1):
            codes, scales, oi, ov, k = binding.bof4_quantize(w, BLOCK, cb, 1, opq_T=T if opq else 0.0,
                                                             out_capacity=n // 50 if opq else 0)
            tab = binding.bof4_gemv_outlier_table(codes, scales, rows, cols, BLOCK, cb, oi, ov, n_outliers=k) if opq else None
            for nt in (1, 2):
                x = torch.randn((nt, cols), device=dev).to(torch.bfloat16)
                y = torch.empty((nt, rows), dtype=torch.float32, device=dev)
                for _ in range(5):
                    binding.bof4_gemv(codes, scales, rows, cols, BLOCK, cb, x, tab, k if opq else 0, out=y)
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(calls):
                    binding.bof4_gemv(codes, scales, rows, cols, BLOCK, cb, x, tab, k if opq else 0, out=y)
                e1.record()
                torch.cuda.synchronize()
                us = e0.elapsed_time(e1) * 1e3 / calls
                nbytes = (0.5 + 2.0 / BLOCK) * n + 8.0 * (k if opq else 0)
                rows_out.append({"rows": rows, "cols": cols, "outliers": int(k) if opq else 0, "tokens": nt,
                                 "us_per_call": us, "GBps_algorithmic": nbytes / us / 1e3,
                                 "hbm_frac": nbytes / us / 1e3 / HBM_PEAK_GBS})
        del w
    return rows_out


MFMA_BF16_PEAK_TFLOPS = 2500.0


def gemm_shapes(dev, calls=30):
    """bof4_gemm on the matrix shapes of workloads 1 and 4 (Student-t weights, block 64, signed, with and without the
    OPQ outliers, 32 and 128 tokens): microseconds per call (all its kernels) from HIP events around `calls`
    back-to-back calls; next to it, on the same decoded matrix, bof4_dequantize and the library's bfloat16 product
    (torch.matmul), the path the fused call replaces."""
    cb = codebooks.array(codebooks.BOF4S_MSE[BLOCK])
    T = binding.bof4_opq_threshold(0.95, BLOCK)

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
            codes, scales, oi, ov, k = binding.bof4_quantize(w, BLOCK, cb, 1, opq_T=T if opq else 0.0,
                                                             out_capacity=n // 50 if opq else 0)
            k = int(k) if opq else 0
            packed = binding.bof4_gemm_pack(codes, scales, rows, cols, BLOCK)
            tab = binding.bof4_gemm_outlier_table(codes, scales, rows, cols, BLOCK, cb, oi, ov, n_outliers=k) if k else None
            deq = torch.empty(n, dtype=torch.bfloat16, device=dev)
            us_deq = timed(lambda: binding.bof4_dequantize(codes, scales, n, BLOCK, cb, oi, ov, n_outliers=k, out=deq))
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


def cpu_baseline(w_samples, cb, T):
    """Oracle (as it stands) on a bounded sample of the same workload; reported baseline only."""
    import oracle
    tq = td = tl = 0.0
    n_total = 0
    for w_sample in w_samples:
        wb = inputs.bits(w_sample)
        n = wb.size
        t0 = time.perf_counter()
        st, codes, scales, oidx, oval, nout = oracle.quantize(wb, BLOCK, cb, 1, opq_T=T)
        t1 = time.perf_counter()
        oracle.dequantize(codes, scales, n, BLOCK, cb, oidx, oval)
        t2 = time.perf_counter()
        oracle.lloyd_step(wb, BLOCK, cb, 1, opq_T=0.0)
        t3 = time.perf_counter()
        tq, td, tl, n_total = tq + t1 - t0, td + t2 - t1, tl + t3 - t2, n_total + n
    return {"value": 2.0 * n_total / (tq + td + tl) / 1e9, "unit": "GB/s", "cores": oracle.num_threads(),
            "kind": "oracle",
            "sample": f"{len(w_samples)} steps (one per replica of the workload, {n_total} weights in all); quantize "
                      f"{tq:.2f}s and dequantize {td:.2f}s run on 1 thread, lloyd_step {tl:.2f}s on "
                      f"{oracle.num_threads()} OpenMP threads",
            "lloyd_weights_per_s": n_total / tl}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--replicas", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--opq", type=int, default=1, help="0 runs the path without outlier extraction (not the headline)")
    ap.add_argument("--serial", action="store_true",
                    help="every call waits for its result before the next is enqueued (default: the Lloyd kernels are "
                         "enqueued behind the quantiser before the host waits for the outlier count)")
    ap.add_argument("--two-streams", action="store_true",
                    help="enqueue the Lloyd kernels on a second stream, so that they overlap with the quantiser and the "
                         "decoder (not the default: the kernel times of the roofline record are taken without overlap)")
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
    if args.gemv_shapes:
        torch.cuda.set_device(dev)
        print(json.dumps({"bof4_gemv": gemv_shapes(dev)}))
        return
    if args.gemm_shapes:
        torch.cuda.set_device(dev)
        print(json.dumps({"bof4_gemm": gemm_shapes(dev)}))
        return
    torch.cuda.set_device(dev)
    binding.lib()

    cb = codebooks.array(codebooks.BOF4S_MSE[BLOCK])
    T = binding.bof4_opq_threshold(0.95, BLOCK) if args.opq else 0.0
    ws_list = [inputs.flatten(inputs.llama7b_block(seed=50 + r, device=dev)) for r in range(args.replicas)]
    n = ws_list[0].numel()
    cap = n // 64
    codes = torch.empty(n // 2, dtype=torch.uint8, device=dev)
    scales = torch.empty(n // BLOCK, dtype=torch.float16, device=dev)
    oidx = torch.empty(cap, dtype=torch.int64, device=dev)
    oval = torch.empty(cap, dtype=torch.float16, device=dev)
    deq = torch.empty(n, dtype=torch.bfloat16, device=dev)
    ws = binding.alloc_workspace(n, BLOCK, cap, dev)
    ws_lloyd = binding.alloc_workspace(n, BLOCK, 0, dev)  # the Lloyd kernels run between the halves of the quantiser
    stats_rec, _keep1 = binding.pinned_lloyd_stats()   # results land in pinned host memory: no copy
    counter, _keep2 = binding.pinned_counter()
    names = ("quantize", "dequantize", "lloyd_step")
    # Kernel-level HIP events, recorded by the library right around the main kernel of a call (bof4_time_next_call).
    # An event record costs about 5 us of stream time, so timed step i brackets only the kernel of call i % 3: every
    # kernel is sampled over the whole timed region at two records per step.
    kev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(args.steps)]
    for row in kev:
        for e in row:
            e.record()  # creates the HIP handle
    n_out_seen = 0

    def step(i, timed_call=None, events=None):
        """One step, every call waiting for its result before the next is enqueued."""
        nonlocal n_out_seen
        w = ws_list[i % len(ws_list)]
        if events:
            events[0].record()
        if timed_call == 0:
            binding.bof4_time_next_call(kev[i][0], kev[i][1])
        k = binding.bof4_quantize(w, BLOCK, cb, 1, opq_T=T, out_capacity=cap, codes=codes, scales=scales,
                                  out_idx=oidx, out_val=oval, ws=ws, counter=counter, trim=False)[4]
        if events:
            events[1].record()
        if timed_call == 1:
            binding.bof4_time_next_call(kev[i][0], kev[i][1])
        binding.bof4_dequantize(codes, scales, n, BLOCK, cb, oidx if k else None, oval if k else None, out=deq,
                                n_outliers=k)
        if events:
            events[2].record()
        if timed_call == 2:
            binding.bof4_time_next_call(kev[i][0], kev[i][1])
        st = binding.bof4_lloyd_step(w, BLOCK, cb, 1, opq_T=0.0, ws=ws, raw=True, out=stats_rec)
        if events:
            events[3].record()
        binding.bof4_codebook_update(st, codebooks.PIN_BOF4S, cb)
        n_out_seen = k

    def step_pipelined(i, timed_call=None):
        """The same calls on the same stream, enqueued so that the GPU always has the next kernel waiting: quantiser,
        Lloyd kernels (they do not depend on the quantiser), then the host collects the outlier count, enqueues the
        decoder, collects the sums and updates the codebook while the decoder runs."""
        nonlocal n_out_seen
        w = ws_list[i % len(ws_list)]
        if timed_call == 0:
            binding.bof4_time_next_call(kev[i][0], kev[i][1])
        flight = binding.bof4_quantize_begin(w, BLOCK, cb, 1, T, cap, codes, scales, oidx, oval, ws, counter)
        if timed_call == 2:
            binding.bof4_time_next_call(kev[i][0], kev[i][1])
        binding.bof4_lloyd_step_begin(w, BLOCK, cb, 1, stats_rec, ws=ws_lloyd, stream=side)
        k = flight.finish()
        if timed_call == 1:
            binding.bof4_time_next_call(kev[i][0], kev[i][1])
        binding.bof4_dequantize(codes, scales, n, BLOCK, cb, oidx if k else None, oval if k else None, out=deq,
                                n_outliers=k)
        binding.bof4_wait_result(stats_rec, stream=side)
        binding.bof4_codebook_update(stats_rec, codebooks.PIN_BOF4S, cb)
        n_out_seen = k

    # --two-streams: the Lloyd kernels (which read only the weights) go to a stream of their own
    side = torch.cuda.Stream() if args.two_streams else None
    timed_step = step if args.serial else step_pipelined
    for i in range(args.warmup):
        timed_step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        timed_step(i, timed_call=i % 3)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    # per-call times (kernels, helper kernels and host waits of one call), from a few extra steps outside the timed
    # region so that their event records do not slow the timed one
    n_extra = min(args.steps, 6)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(n_extra)]
    for i in range(n_extra):
        step(args.steps + i, events=ev[i])
    torch.cuda.synchronize()
    # the MAE-criterion expectation step (weighted medians; not part of the timed step): wall time of a few calls
    mae_rec, _keep3 = binding.pinned_mae_stats()
    mae_cb = codebooks.array(codebooks.BOF4S_MAE_64)
    binding.bof4_lloyd_step_mae(ws_list[0], BLOCK, mae_cb, 1, skip_mask=codebooks.PIN_BOF4S, ws=ws, out=mae_rec)
    torch.cuda.synchronize()
    t_mae = time.perf_counter()
    for r in range(3):
        binding.bof4_lloyd_step_mae(ws_list[r % len(ws_list)], BLOCK, mae_cb, 1, skip_mask=codebooks.PIN_BOF4S, ws=ws,
                                    out=mae_rec)
    torch.cuda.synchronize()
    t_mae = (time.perf_counter() - t_mae) / 3
    # the error pass (MSE / MAE of the tensor against its quantised form; not part of the timed step)
    err_rec, _keep4 = binding.pinned_error_stats()
    err_ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    for e in err_ev:
        e.record()
    binding.bof4_quant_error(ws_list[0], BLOCK, cb, 1, opq_T=T, ws=ws, out=err_rec)
    torch.cuda.synchronize()
    t_err = time.perf_counter()
    for r in range(3):
        if r == 2:
            binding.bof4_time_next_call(err_ev[0], err_ev[1])
        err = binding.bof4_quant_error(ws_list[r % len(ws_list)], BLOCK, cb, 1, opq_T=T, ws=ws, out=err_rec)
    torch.cuda.synchronize()
    t_err = (time.perf_counter() - t_err) / 3
    k_err = err_ev[0].elapsed_time(err_ev[1])
    gemv = gemv_block_pass(codes, scales, oidx, oval, n_out_seen, cb, dev)
    gemm = gemm_block_pass(codes, scales, oidx, oval, n_out_seen, cb, dev)
    # one plain device copy of known size (2 * n bytes read, 2 * n written), outside the timed region: the reference
    # against which a counter profile of this same command scales FETCH_SIZE / WRITE_SIZE
    deq.copy_(ws_list[0])
    torch.cuda.synchronize()

    ms = {nm: float(np.mean([ev[i][k].elapsed_time(ev[i][k + 1]) for i in range(n_extra)]))
          for k, nm in enumerate(names)}
    kms = {}
    for c, nm in enumerate(names):
        samples = [kev[i][0].elapsed_time(kev[i][1]) for i in range(args.steps) if i % 3 == c]
        if not samples:  # fewer than three timed steps: no sample of this kernel
            samples = [float("nan")]
        kms[nm] = float(np.mean(samples))
    rho = n_out_seen / n
    # algorithmic bytes per launch = bytes per weight x n (one launch processes the whole tensor)
    alg_bytes = {"quantize": (2.0 + 0.5 + 2.0 / BLOCK + 10.0 * rho) * n,
                 "dequantize": (0.5 + 2.0 / BLOCK + 2.0 + 10.0 * rho) * n,
                 "lloyd_step": 2.0 * n}
    dominant = max(names, key=lambda k: kms[k] if kms[k] == kms[k] else -1.0)
    achieved = alg_bytes[dominant] / (kms[dominant] * 1e-3) / 1e9
    per_call = {nm: {"call_ms": ms[nm], "kernel_ms": kms[nm], "GBps_bf16": 2.0 * n / (kms[nm] * 1e-3) / 1e9,
                     "GBps_algorithmic": alg_bytes[nm] / (kms[nm] * 1e-3) / 1e9,
                     "hbm_frac": alg_bytes[nm] / (kms[nm] * 1e-3) / 1e9 / HBM_PEAK_GBS} for nm in names}
    # HBM bytes per launch from the FETCH_SIZE / WRITE_SIZE counter profiles of this command, scaled by the plain
    # copy in the same profile (profiles/bench_configs1_opq_hbm_traffic.md); only valid for the default workload
    traffic = PROFILED_TRAFFIC_BYTES.get(dominant) if args.opq else None
    out = {
        "metric": "GB/s bf16 weights quantized & weights/s per Lloyd step; % of HBM peak",
        "value": 2.0 * n * args.steps / dt / 1e9, "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": dt / args.steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16 in, f32 normalise/assign, f64 sums", "data": "synthetic",
        "config": {"workload": "configs[1]: one Llama-7B-shaped block, 202,375,168 bf16 weights, Student-t(5) std 0.02 "
                               "with log-normal(0,0.3) row scale, block 64, signed absmax (BOF4-S), OPQ q=0.95" + ("" if args.opq else " OFF") + "; "
                               "step = quantize + dequantize + lloyd_step + codebook_update",
                   "n_weights": n, "block": BLOCK, "outlier_fraction": rho, "replicas": len(ws_list),
                   "enqueue_order": "one call after the other, each waiting for its result" if args.serial else
                                    "quantize kernels, lloyd kernels, outlier count, dequantize, lloyd sums (" +
                                    ("lloyd kernels on a second stream: kernel times include the overlap)"
                                     if args.two_streams else "one stream)")},
        "lloyd_weights_per_s": n / (kms["lloyd_step"] * 1e-3),
        "mae_step": {"call_ms": t_mae * 1e3, "weights_per_s": n / t_mae,
                     "note": "bof4_lloyd_step_mae (exact weighted medians of the 14 free levels: two passes over the weights, one over a candidate list), outside the "
                             "timed step"},
        "quant_error": {"call_ms": t_err * 1e3, "kernel_ms": k_err, "GBps_algorithmic": 2.0 * n / (k_err * 1e-3) / 1e9,
                        "hbm_frac": 2.0 * n / (k_err * 1e-3) / 1e9 / HBM_PEAK_GBS, "mse": err["sse"] / err["n"],
                        "mae": err["sae"] / err["n"],
                        "note": "bof4_quant_error (quantise, decode and compare in registers: 2 bytes per weight), outside "
                                "the timed step"},
        "gemv_block_pass": gemv,
        "gemm_block_pass": gemm,
        "per_call": per_call,
        "roofline": {"bound": "hbm", "kernel": dominant, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline([w.cpu() for w in ws_list], cb, T)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
