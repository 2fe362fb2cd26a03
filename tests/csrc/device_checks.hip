// Exhaustive device-side checks of the arithmetic shortcuts in paper_2505_06653_amd/csrc/bof4_device.h.
// Test infrastructure: built into tests/libbof4_device_checks.so and called from tests/test_gpu_device_checks.py.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "bof4_device.h"

using namespace bof4;

// For every ordinary block constant pattern m (index mi into the ordinary range, both signs) and every bfloat16
// pattern w with |w| <= |m|:  compare the shortcut division with the hardware's IEEE division and the bin-table
// nearest-level search with the 15-compare search.  out[0] quotient mismatches for |w| >= 2^-60 (or w = 0),
// out[1] quotient mismatches for tiny |w|, out[2] code mismatches, out[3] |x| > 1, out[4] pairs checked.
__global__ __launch_bounds__(256) void check_pairs_kernel(CodebookArgs cb, BinTable bt, unsigned long long* out) {
    __shared__ uint2 tab[40];
    if (threadIdx.x < 33) tab[threadIdx.x] = make_uint2(__float_as_uint(bt.thr[threadIdx.x]), bt.base[threadIdx.x]);
    __syncthreads();
    const uint32_t mi = blockIdx.x;  // 0 .. 2*(0x477F-0x3880+1)-1
    const uint32_t span = 0x477Fu - 0x3880u + 1u;
    const uint32_t mabs = 0x3880u + (mi % span);
    const uint32_t mbits = mabs | ((mi / span) << 15);
    const float m = bf16_bits_to_f32(mbits);
    const float m_eff = f16_bits_to_f32(f32_to_f16_bits(m));
    const BlockDiv dv = make_block_div(m_eff);
    unsigned long long bad_q = 0, bad_tiny = 0, bad_code = 0, bad_range = 0, n = 0;
    for (uint32_t wb = threadIdx.x; wb < 65536u; wb += 256) {
        const uint32_t wabs = wb & 0x7fffu;
        if (wabs > mabs) continue;  // cannot occur: m is the block maximum
        const float w = bf16_bits_to_f32(wb);
        const float x_ref = w / m_eff;
        const float x = div_fast(w, dv);
        ++n;
        const bool tiny = wabs != 0 && wabs < 0x2180u;  // |w| < 2^-60
        const bool same = (__float_as_uint(x) == __float_as_uint(x_ref)) || (x == 0.0f && x_ref == 0.0f);
        if (!same) (tiny ? bad_tiny : bad_q)++;
        if (!(x >= -1.0f && x <= 1.0f)) ++bad_range;
        const uint32_t off = __float_as_uint(__builtin_fmaf(x, BIN_SCALE, BIN_MAGIC)) & BIN_MASK;
        const uint2 en = *reinterpret_cast<const uint2*>(reinterpret_cast<const char*>(tab) + off);
        const uint32_t code = en.y + (x > __uint_as_float(en.x) ? 1u : 0u);
        if (code != (uint32_t)assign_code_generic(x_ref, cb)) ++bad_code;
    }
    atomicAdd(&out[0], bad_q);
    atomicAdd(&out[1], bad_tiny);
    atomicAdd(&out[2], bad_code);
    atomicAdd(&out[3], bad_range);
    atomicAdd(&out[4], n);
}

extern "C" int bof4_check_pairs(const float* thr15, const float* lv16, const float* bin_thr33,
                                const uint32_t* bin_base33, unsigned long long* out_dev, void* stream) {
    CodebookArgs cb;
    BinTable bt;
    for (int k = 0; k < 15; ++k) cb.thr[k] = thr15[k];
    cb.thr[15] = __builtin_inff();
    for (int l = 0; l < 16; ++l) {
        cb.lv32[l] = lv16[l];
        cb.cb64[l] = lv16[l];
    }
    for (int b = 0; b < 33; ++b) {
        bt.thr[b] = bin_thr33[b];
        bt.base[b] = bin_base33[b];
    }
    bt.code_of_zero = 0;
    bt.fast = 1;
    const uint32_t span = 0x477Fu - 0x3880u + 1u;
    hipLaunchKernelGGL(check_pairs_kernel, dim3(2 * span), dim3(256), 0, (hipStream_t)stream, cb, bt, out_dev);
    return (int)hipGetLastError();
}
