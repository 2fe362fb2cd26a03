// bof4_error.h - the quantisation error of a tensor in one pass over the weights: sum (w - Q(w))^2, sum |w - Q(w)| and
// the largest |w - Q(w)|, the quantities behind the MSE / MAE columns of the paper's error table (section 5) and the
// decomposition of appendix B.3.  Q(w) is what the decoder returns for what the quantiser stores: the bfloat16
// rounding of constant * level[code], or the outlier as kept in binary16 (section 3.3).
//
// Same front end as the quantiser (one lane, one segment): OPQ statistics, block constant, shortcut division, bin
// table.  Instead of packing the code the lane decodes it again (16-entry LDS table of levels, one binary32 product,
// hardware rounding to bfloat16), subtracts in binary32 (exact whenever the two numbers lie within 2^16 of each other,
// which is every case where the difference matters) and adds the square and the magnitude up in binary64.  Nothing
// is written but one record per workgroup: 2 bytes of HBM traffic per weight.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

#include "bof4_device.h"
#include "bof4_segment.h"

namespace bof4 {

constexpr int ERR_PART = 4;  // per workgroup: sse, sae, max (binary64), outlier count (integer bits)

typedef __bf16 err_bf16x2 __attribute__((ext_vector_type(2)));
typedef float err_f32x2 __attribute__((ext_vector_type(2)));
// Two binary32 numbers rounded to bfloat16 (nearest even, the decoder's conversion) and widened again.
__device__ __forceinline__ void round_pair_to_bf16(float a, float b, float& ra, float& rb) {
    err_f32x2 v = {a, b};
    err_bf16x2 r = __builtin_convertvector(v, err_bf16x2);
    uint32_t u;
    __builtin_memcpy(&u, &r, 4);
    ra = __uint_as_float(u << 16);
    rb = __uint_as_float(u & 0xffff0000u);
}

template <int I, bool FAST, bool OPQ>
__global__ __launch_bounds__(256, 2) void seg_error_kernel(const uint4* __restrict__ w, uint64_t n_seg, CodebookArgs cb,
                                                         BinTable bt, int signed_norm, double T2,
                                                         double* __restrict__ partials) {
    using C = SegCfg<I>;
    struct Shared {  // one object, so that the tables sit at the start of LDS (reachable by immediate offsets)
        uint2 tab[BIN_TABLE_ENTRIES];
        float lv[16];
        char stage[WAVES_PER_WG * C::STAGE_BYTES];
        uint16_t tie[WAVES_PER_WG * TIE_BUF_HALFWORDS] __attribute__((aligned(16)));
    };
    __shared__ __attribute__((aligned(16))) Shared sh;
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    bin_table_fill(sh.tab, bt, tid, blockDim.x);
    if (tid < 16) sh.lv[tid] = cb.lv32[tid];
    __syncthreads();
    const uint2* tab = sh.tab;
    const uint32_t lane_off = bin_lane_offset(threadIdx.x & 63u);
    const float* lv = sh.lv;
    char* stage = sh.stage + wave * C::STAGE_BYTES;
    uint16_t* tie_buf = sh.tie + wave * TIE_BUF_HALFWORDS;
    const uint64_t n_vec = n_seg * C::NV;
    const uint64_t n_tiles = (n_seg + 63) / 64;
    const uint64_t n_waves = (uint64_t)gridDim.x * WAVES_PER_WG;
    const uint64_t gw = (uint64_t)blockIdx.x * WAVES_PER_WG + wave;
    const uint64_t t0 = n_tiles * gw / n_waves, t1 = n_tiles * (gw + 1) / n_waves;

    double sse = 0.0, sae = 0.0;
    double mx = 0.0;
    uint32_t kout = 0;
    uint4 G[C::NV];
    uint32_t R[C::NR];
    if (t0 < t1) tile_issue_loads<I>(w, t0 * 64 * C::NV, n_vec, lane, G);
    for (uint64_t t = t0; t < t1; ++t) {
        wave_lds_fence();
        tile_stage<I>(stage, lane, G);
        if (t + 1 < t1) tile_issue_loads<I>(w, (t + 1) * 64 * C::NV, n_vec, lane, G);
        wave_lds_fence();
        tile_fetch<I>(stage, lane, R);
        const uint64_t seg = t * 64 + lane;
        const bool active = seg < n_seg;
        uint32_t k_out = 0, omap[2] = {0, 0};
        if (OPQ) {
            opq_zero_outliers<I>(R, opq_theta<I>(R, T2), omap);
            k_out = opq_count(omap);
        }
        uint32_t maxabs, sign;
        block_constant<I>(R, lane, signed_norm != 0, maxabs, sign, tie_buf);
        const float m = bf16_bits_to_f32(maxabs | (sign << 15));
        const float m_eff = f16_bits_to_f32(f32_to_f16_bits(m));
        // what a zeroed outlier's placeholder decodes to (0 for every codebook with a zero level)
        float ph, ph_unused;
        round_pair_to_bf16(m_eff * lv[bt.code_of_zero], 0.0f, ph, ph_unused);
        // Placeholders that decode to something would count as errors of zeros: such waves take the loop that
        // looks at every element's outlier bit.
        const bool placeholders = OPQ && __builtin_amdgcn_ballot_w64(k_out != 0 && ph != 0.0f) != 0;
        const bool fast = FAST && !placeholders && __builtin_amdgcn_ballot_w64(!maxabs_is_ordinary(maxabs)) == 0;
        if (active) {
            if (fast) {
                const BlockDiv dv = make_block_div(m_eff);
#pragma unroll
                for (int b0 = 0; b0 < C::SEG; b0 += 8) {
                    float f[8], x[8], q[8];
                    uint2 en[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) {  // eight table reads in flight
                        f[e] = seg_f32(R, b0 + e);
                        x[e] = div_fast(f[e], dv);
                        en[e] = bin_lookup(tab, x[e], lane_off);
                    }
#pragma unroll
                    for (int e = 0; e < 8; ++e) {  // then eight level reads
                        const uint32_t code = en[e].y + (x[e] > __uint_as_float(en[e].x) ? 1u : 0u);
                        q[e] = m_eff * lv[code];
                    }
#pragma unroll
                    for (int e = 0; e < 8; e += 2) {
                        float q0, q1;
                        round_pair_to_bf16(q[e], q[e + 1], q0, q1);
                        // the difference in binary64: in binary32 it rounds where the two numbers lie
                        // more than 2^16 apart (a weight next to nothing against a level that is not zero)
                        const double dd0 = (double)f[e] - (double)q0, dd1 = (double)f[e + 1] - (double)q1;
                        sse = fma(dd0, dd0, sse);
                        sse = fma(dd1, dd1, sse);
                        sae += fabs(dd0);
                        sae += fabs(dd1);
                        mx = fmax(mx, fmax(fabs(dd0), fabs(dd1)));
                    }
                }
            } else {
#pragma unroll 4
                for (int e = 0; e < C::SEG; ++e) {
                    if (OPQ && ((omap[(e >> 1) >> 4] >> (((e >> 1) & 15) + 16 * (e & 1))) & 1u)) continue;  // an outlier
                    const float f = seg_f32(R, e);
                    const float x = (m_eff == 0.0f) ? 0.0f : f / m_eff;
                    const uint32_t code = (uint32_t)assign_code_generic(x, cb);
                    float q0, q1;
                    round_pair_to_bf16(m_eff * lv[code], 0.0f, q0, q1);
                    const double dd = (double)f - (double)q0;
                    sse = fma(dd, dd, sse);
                    sae += fabs(dd);
                    mx = fmax(mx, fabs(dd));
                }
            }
            if (OPQ && k_out != 0) {
                // the outliers themselves: kept in binary16, decoded to bfloat16 (exact inside binary16's normal range)
                const char* myseg = stage + lane * C::PITCH;  // the staged tile still holds the original values
                uint32_t left[2] = {omap[0], omap[1]};
                while ((left[0] | left[1]) != 0u) {
                    const uint32_t e = opq_pop_lowest(left);
                    const float f = bf16_bits_to_f32(*reinterpret_cast<const uint16_t*>(myseg + 2 * e));
                    float back, unused;
                    round_pair_to_bf16(f16_bits_to_f32(f32_to_f16_bits(f)), 0.0f, back, unused);
                    const double dd = (double)f - (double)back;
                    sse = fma(dd, dd, sse);
                    sae += fabs(dd);
                    mx = fmax(mx, fabs(dd));
                }
                kout += k_out;
            }
        }
    }
    // fixed-order butterfly inside the wave, then the four waves of the workgroup in wave order
    double mxd = mx;
    unsigned long long kc = kout;
#pragma unroll
    for (int mk = 32; mk >= 1; mk >>= 1) {
        sse += __shfl_xor(sse, mk, 64);
        sae += __shfl_xor(sae, mk, 64);
        mxd = fmax(mxd, __shfl_xor(mxd, mk, 64));
        kc += (unsigned long long)__shfl_xor((long long)kc, mk, 64);
    }
    __shared__ double wave_totals[WAVES_PER_WG][ERR_PART];
    if (lane == 0) {
        wave_totals[wave][0] = sse;
        wave_totals[wave][1] = sae;
        wave_totals[wave][2] = mxd;
        wave_totals[wave][3] = __longlong_as_double((long long)kc);
    }
    __syncthreads();
    if (tid == 0) {
        double s0 = 0.0, s1 = 0.0, s2 = 0.0;
        unsigned long long s3 = 0ull;
        for (int k = 0; k < WAVES_PER_WG; ++k) {
            s0 += wave_totals[k][0];
            s1 += wave_totals[k][1];
            s2 = fmax(s2, wave_totals[k][2]);
            s3 += (unsigned long long)__double_as_longlong(wave_totals[k][3]);
        }
        double* p = partials + (uint64_t)blockIdx.x * ERR_PART;
        p[0] = s0;
        p[1] = s1;
        p[2] = s2;
        p[3] = __longlong_as_double((long long)s3);
    }
}

// Adds the per-workgroup records in index order (sixteen partial sums per quantity, then those in order) and writes
// the result in the layout of bof4_error_stats: [0] sse, [1] sae, [2] max, [3] outliers, [4] n (integers).  Word 4 is
// stored last, at system scope, so that a host watching it may read the record as soon as it changes.
__global__ __launch_bounds__(64) void error_final_kernel(const double* __restrict__ partials, uint32_t n_part,
                                                         uint64_t n, double* __restrict__ out) {
    const uint32_t lane = threadIdx.x, q = lane & 3, part = lane >> 2;  // 16 lanes per quantity
    double s = 0.0;
    unsigned long long si = 0ull;
    for (uint32_t p = part; p < n_part; p += 16) {
        const double v = partials[(uint64_t)p * ERR_PART + q];
        if (q == 3) si += (unsigned long long)__double_as_longlong(v);
        else if (q == 2) s = fmax(s, v);
        else s += v;
    }
    __shared__ double red[16][4];
    red[part][q] = q == 3 ? __longlong_as_double((long long)si) : s;
    __syncthreads();
    if (lane == 0) {
        double t0 = 0.0, t1 = 0.0, t2 = 0.0;
        unsigned long long t3 = 0ull;
        for (int k = 0; k < 16; ++k) {
            t0 += red[k][0];
            t1 += red[k][1];
            t2 = fmax(t2, red[k][2]);
            t3 += (unsigned long long)__double_as_longlong(red[k][3]);
        }
        out[0] = t0;
        out[1] = t1;
        out[2] = t2;
        out[3] = __longlong_as_double((long long)t3);
        __hip_atomic_store(reinterpret_cast<unsigned long long*>(&out[4]), (unsigned long long)n, __ATOMIC_RELEASE,
                           __HIP_MEMORY_SCOPE_SYSTEM);
    }
}

}  // namespace bof4
