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
    __shared__ uint2 tab[BIN_TABLE_ENTRIES];
    bin_table_fill(tab, bt, threadIdx.x, blockDim.x);
    __syncthreads();
    const uint32_t lane_off = bin_lane_offset(threadIdx.x & 63u);
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
        const uint2 en = bin_lookup(tab, x, lane_off);
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

// ------------------------------------------------------------------------------------------------ dot2 error
// Measures the error of dot2_bf16 (one v_dot2c_f32_bf16) against the exact value of a.lo b.lo + a.hi b.hi + c on
// pseudo-random operands, in units of 2^-24 (|a.lo b.lo| + |a.hi b.hi| + |c|) - the quantity the OPQ statistics'
// error allowance is stated in.  Regimes: 0 general, 1 products that nearly cancel, 2 b = (1, 1) with a running sum,
// 3 a = b (squares) with a non-negative running sum.  out[r] = bit pattern of the largest ratio seen in regime r
// (non-negative doubles order like their bit patterns), out[4 + r] = samples.
__device__ __forceinline__ uint64_t mix64(uint64_t z) {
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
__device__ __forceinline__ uint32_t bf16_pattern(uint64_t r, int exp_lo, int exp_span) {  // sign, exponent, mantissa
    const uint32_t sign = (uint32_t)(r & 1u), man = (uint32_t)((r >> 1) & 0x7fu);
    const uint32_t e = (uint32_t)(127 + exp_lo + (int)((r >> 8) % (uint64_t)exp_span));
    return (sign << 15) | (e << 7) | man;
}
__global__ __launch_bounds__(256) void check_dot2_kernel(uint64_t seed, uint32_t per_thread,
                                                         unsigned long long* out) {
    const uint64_t tid = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    double worst[4] = {0.0, 0.0, 0.0, 0.0};
    for (uint32_t it = 0; it < per_thread; ++it) {
        const uint64_t r0 = mix64(seed + tid * 0x100000001B3ull + it), r1 = mix64(r0), r2 = mix64(r1);
        const uint32_t regime = (uint32_t)(r2 >> 62);
        uint32_t a0 = bf16_pattern(r0, -9, 19), a1 = bf16_pattern(r0 >> 20, -9, 19);
        uint32_t b0 = bf16_pattern(r1, -9, 19), b1 = bf16_pattern(r1 >> 20, -9, 19);
        float c = __uint_as_float((uint32_t)((r2 & 0x807fffffu) | ((uint32_t)(127 - 20 + (int)((r2 >> 32) % 41u)) << 23)));
        if (regime == 1) {  // second product close to minus the first
            a1 = a0 ^ 0x8000u;
            b1 = (b0 & 0xff80u) | ((b0 + (uint32_t)((r2 >> 40) & 3u)) & 0x7fu);
            if ((r2 >> 50) & 1u) c = 0.0f;
        } else if (regime == 2) {
            b0 = b1 = 0x3f80u;
        } else if (regime == 3) {
            b0 = a0;
            b1 = a1;
            c = fabsf(c);
        }
        const double p0 = (double)bf16_bits_to_f32(a0) * (double)bf16_bits_to_f32(b0);  // exact: 16-bit products
        const double p1 = (double)bf16_bits_to_f32(a1) * (double)bf16_bits_to_f32(b1);
        const double s = p0 + p1;  // exact: the operands' exponents differ by at most 36
        const double hi = s + (double)c, bb = hi - s;  // hi + lo = s + c exactly (two-sum)
        const double lo = (s - (hi - bb)) + ((double)c - bb);
        const float h = dot2_bf16(a0 | (a1 << 16), b0 | (b1 << 16), c);
        const double err = fabs(((double)h - hi) - lo);
        const double allowance = 0x1p-24 * (fabs(p0) + fabs(p1) + fabs((double)c));
        const double ratio = err / allowance;
        if (ratio > worst[regime]) worst[regime] = ratio;
        atomicAdd(&out[4 + regime], 1ull);
    }
    for (int r = 0; r < 4; ++r) atomicMax(&out[r], (unsigned long long)__double_as_longlong(worst[r]));
}
extern "C" int bof4_check_dot2(uint64_t seed, uint32_t blocks, uint32_t per_thread, unsigned long long* out_dev,
                               void* stream) {
    hipLaunchKernelGGL(check_dot2_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, seed, per_thread, out_dev);
    return (int)hipGetLastError();
}

// ------------------------------------------------------------------------------------------------ wave scan
// wave_inclusive_scan_u32 against a serial prefix sum over the wave's values (read back through LDS).
// out[0] = mismatching lanes, out[1] = lanes checked.
__global__ __launch_bounds__(256) void check_scan_kernel(uint64_t seed, uint32_t rounds, unsigned long long* out) {
    __shared__ uint32_t vals[256];
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    unsigned long long bad = 0, n = 0;
    for (uint32_t it = 0; it < rounds; ++it) {
        const uint64_t r = mix64(seed + ((uint64_t)blockIdx.x * 256 + threadIdx.x) * 0x100000001B3ull + it);
        // small counts (as in the kernels), now and then large values whose sums wrap around
        const uint32_t x = (r & 0x300) ? (uint32_t)(r & 7u) : (uint32_t)(r >> 32);
        vals[threadIdx.x] = x;
        __syncthreads();
        uint32_t ref = 0;
        for (uint32_t j = 0; j <= lane; ++j) ref += vals[wave * 64 + j];
        __syncthreads();
        if (wave_inclusive_scan_u32(x) != ref) ++bad;
        ++n;
    }
    atomicAdd(&out[0], bad);
    atomicAdd(&out[1], n);
}
extern "C" int bof4_check_scan(uint64_t seed, uint32_t blocks, uint32_t rounds, unsigned long long* out_dev,
                               void* stream) {
    hipLaunchKernelGGL(check_scan_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, seed, rounds, out_dev);
    return (int)hipGetLastError();
}

// ------------------------------------------------------------------------------------------------ packed max / min
// pk_max3_f16 / pk_min3_f16 on all 2^32 pairs (a, b) of 16-bit patterns against the order the block-maximum search
// relies on: sign first, then magnitude, +0 above -0, subnormal patterns compared like any other.  Pairs with a
// pattern that binary16 reads as NaN (magnitude field above 0x7C00) must come out as such a pattern (the kernels test
// for that and repeat the search with integer compares).  out[0] wrong maxima, out[1] wrong minima, out[2] NaN inputs
// that did not give a NaN pattern, out[3] pairs checked.
__device__ __forceinline__ int pattern_rank(uint32_t p) {  // value order of a non-NaN pattern
    return (p & 0x8000u) ? -(int)(p & 0x7fffu) - 1 : (int)(p & 0x7fffu);
}
__global__ __launch_bounds__(256) void check_pkmax_kernel(unsigned long long* out) {
    const uint32_t a = blockIdx.x;  // 0 .. 65535
    unsigned long long bad_max = 0, bad_min = 0, bad_nan = 0, n = 0;
    for (uint32_t b = threadIdx.x; b < 65536u; b += 256) {
        const uint32_t ab = a | (b << 16), ba = b | (a << 16);
        // three-operand form as the kernels use it: running value, then two new registers
        const uint32_t mx = pk_max3_f16(ab, ba, ab), mn = pk_min3_f16(ab, ba, ab);
        const bool nan_in = (a & 0x7fffu) > 0x7C00u || (b & 0x7fffu) > 0x7C00u;
        ++n;
        if (nan_in) {
            if ((mx & 0x7fffu) <= 0x7C00u || (mx >> 16 & 0x7fffu) <= 0x7C00u || (mn & 0x7fffu) <= 0x7C00u ||
                (mn >> 16 & 0x7fffu) <= 0x7C00u)
                ++bad_nan;
            continue;
        }
        const uint32_t want_max = pattern_rank(a) >= pattern_rank(b) ? a : b;
        const uint32_t want_min = pattern_rank(a) <= pattern_rank(b) ? a : b;
        if ((mx & 0xffffu) != want_max || (mx >> 16) != want_max) ++bad_max;
        if ((mn & 0xffffu) != want_min || (mn >> 16) != want_min) ++bad_min;
    }
    atomicAdd(&out[0], bad_max);
    atomicAdd(&out[1], bad_min);
    atomicAdd(&out[2], bad_nan);
    atomicAdd(&out[3], n);
}
extern "C" int bof4_check_pkmax(unsigned long long* out_dev, void* stream) {
    hipLaunchKernelGGL(check_pkmax_kernel, dim3(65536), dim3(256), 0, (hipStream_t)stream, out_dev);
    return (int)hipGetLastError();
}
