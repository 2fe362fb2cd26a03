// bof4_segment.h - the "one lane, one segment" kernels: quantise and Lloyd step.
//
// Work layout.  The flat weight array is cut into segments of SEG = min(I, 64) consecutive bfloat16 weights; a
// block of I weights is I/SEG (1, 2 or 4) neighbouring segments.  A wave processes tiles of 64 consecutive
// segments: it loads the tile with fully coalesced 16-byte loads, parks it in a wave-private, padded LDS buffer and
// reads it back transposed, so that every lane ends up holding one whole segment in registers.  All per-block work
// (maximum search of section 2.1 eq. 1 / section 3.1 eq. 4, normalisation eq. 2, nearest-level search of section
// 3.2, the sums of eq. 6) then runs inside a lane without cross-lane traffic.  Every wave owns a contiguous range
// of tiles.
#pragma once
#include "bof4_device.h"

namespace bof4 {

template <int I>
struct SegCfg {
    static constexpr int SEG = I < 64 ? I : 64;    // weights per lane and tile row
    static constexpr int LPB = I / SEG;            // lanes per block
    static constexpr int NV = SEG / 8;             // 16-byte vectors per segment
    static constexpr int NR = SEG / 2;             // packed registers per segment
    static constexpr int PITCH = SEG * 2 + 16;     // staged bytes per segment (16 bytes of padding: conflict-free)
    static constexpr int STAGE_BYTES = 64 * PITCH; // wave-private staging buffer
    static constexpr int TILE = 64 * SEG;          // weights per wave tile
};

constexpr int WAVES_PER_WG = 4;
constexpr int LLOYD_PART = 56;  // doubles per per-wave partial: A[16] den15[16] cnt15[16] sxx kout_g kout nout (+pad)

// ---------------------------------------------------------------------------------------------- tile movement
template <int I>
__device__ __forceinline__ void tile_issue_loads(const uint4* __restrict__ w, uint64_t first_vec, uint64_t n_vec,
                                                 uint32_t lane, uint4 (&G)[SegCfg<I>::NV]) {
#pragma unroll
    for (int k = 0; k < SegCfg<I>::NV; ++k) {
        uint64_t v = first_vec + (uint64_t)(64 * k) + lane;
        G[k] = v < n_vec ? load_stream(&w[v]) : make_uint4(0, 0, 0, 0);
    }
}
template <int I>
__device__ __forceinline__ void tile_stage(char* stage, uint32_t lane, const uint4 (&G)[SegCfg<I>::NV]) {
    using C = SegCfg<I>;
#pragma unroll
    for (int k = 0; k < C::NV; ++k) {
        uint32_t c = 64 * k + lane;  // chunk index inside the tile
        uint32_t j = c / C::NV, i = c % C::NV;
        *reinterpret_cast<uint4*>(stage + j * C::PITCH + i * 16) = G[k];
    }
}
template <int I>
__device__ __forceinline__ void tile_fetch(const char* stage, uint32_t lane, uint32_t (&R)[SegCfg<I>::NR]) {
    using C = SegCfg<I>;
#pragma unroll
    for (int i = 0; i < C::NV; ++i) {
        uint4 q = *reinterpret_cast<const uint4*>(stage + lane * C::PITCH + i * 16);
        R[4 * i] = q.x;
        R[4 * i + 1] = q.y;
        R[4 * i + 2] = q.z;
        R[4 * i + 3] = q.w;
    }
}
// LDS traffic between the lanes of one wave: the LDS unit serves a wave's requests in order, the fences only
// keep the compiler from moving the accesses across each other.
__device__ __forceinline__ void wave_lds_fence() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int WIDTH>
__device__ __forceinline__ int group_max_i32(int v) {
#pragma unroll
    for (int m = 1; m < WIDTH; m <<= 1) v = max(v, __shfl_xor(v, m, 64));
    return v;
}
template <int WIDTH>
__device__ __forceinline__ uint32_t group_min_u32(uint32_t v) {
#pragma unroll
    for (int m = 1; m < WIDTH; m <<= 1) v = min(v, (uint32_t)__shfl_xor((int)v, m, 64));
    return v;
}

__device__ __forceinline__ uint32_t seg_bits(const uint32_t* R, int e) {
    return (e & 1) ? (R[e >> 1] >> 16) : (R[e >> 1] & 0xffffu);
}
__device__ __forceinline__ float seg_f32(const uint32_t* R, int e) {
    return __uint_as_float((e & 1) ? (R[e >> 1] & 0xffff0000u) : (R[e >> 1] << 16));
}

// ---------------------------------------------------------------------------------------------- block constant
// Largest magnitude of the block and the sign of its first occurrence (lowest index).  Packed 16-bit maxima give
// P = largest positive pattern (signed compare) and N = largest negative pattern (unsigned compare); only when +a
// and -a are both present at the maximum does the order matter, and only then the segment is scanned.
template <int I>
__device__ __forceinline__ void block_constant(const uint32_t (&R)[SegCfg<I>::NR], uint32_t lane, bool signed_norm,
                                               uint32_t& maxabs, uint32_t& sign) {
    using C = SegCfg<I>;
    uint32_t P = R[0], N = R[0];
#pragma unroll
    for (int d = 1; d < C::NR; ++d) {
        P = pk_max_i16(P, R[d]);
        N = pk_max_u16(N, R[d]);
    }
    int p = max((int)(short)(P & 0xffffu), (int)P >> 16);  // >= 0 iff a non-negative pattern exists
    uint32_t n = max(N & 0xffffu, N >> 16);                // >= 0x8000 iff a negative pattern exists
    int absP = p >= 0 ? p : -1;
    int absN = n >= 0x8000u ? (int)(n & 0x7fffu) : -1;
    absP = group_max_i32<C::LPB>(absP);
    absN = group_max_i32<C::LPB>(absN);
    maxabs = (uint32_t)max(absP, absN);
    sign = absN > absP ? 1u : 0u;
    if (!signed_norm) {
        sign = 0;
        return;
    }
    bool tie = (absP == absN);
    if (__builtin_amdgcn_ballot_w64(tie) != 0) {  // wave-uniform: rare
        uint32_t key = 0xffffffffu;
        if (tie) {
            const uint32_t lane_in_block = lane & (C::LPB - 1);
#pragma unroll
            for (int e = C::SEG - 1; e >= 0; --e) {
                uint32_t b = seg_bits(R, e);
                if ((b & 0x7fffu) == maxabs) key = ((lane_in_block * C::SEG + e) << 1) | (b >> 15);
            }
        }
        key = group_min_u32<C::LPB>(key);
        if (tie) sign = key & 1u;
    }
}

// ================================================================================================ quantise
template <int I, bool FAST>
__global__ __launch_bounds__(256) void seg_quantize_kernel(const uint4* __restrict__ w, uint64_t n_seg,
                                                            CodebookArgs cb, BinTable bt, int signed_norm,
                                                            uint32_t* __restrict__ codes,
                                                            uint16_t* __restrict__ scales) {
    using C = SegCfg<I>;
    __shared__ __attribute__((aligned(16))) char stage_all[WAVES_PER_WG * C::STAGE_BYTES];
    __shared__ uint2 tab[33];
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid < 33) tab[tid] = make_uint2(__float_as_uint(bt.thr[tid]), bt.base[tid]);
    __syncthreads();
    char* stage = stage_all + wave * C::STAGE_BYTES;
    const uint64_t n_vec = n_seg * C::NV;
    const uint64_t n_tiles = (n_seg + 63) / 64;
    const uint64_t n_waves = (uint64_t)gridDim.x * WAVES_PER_WG;
    const uint64_t gw = (uint64_t)blockIdx.x * WAVES_PER_WG + wave;
    const uint64_t t0 = n_tiles * gw / n_waves, t1 = n_tiles * (gw + 1) / n_waves;
    if (t0 >= t1) return;
    uint4 G[C::NV];
    uint32_t R[C::NR];
    tile_issue_loads<I>(w, t0 * 64 * C::NV, n_vec, lane, G);
    for (uint64_t t = t0; t < t1; ++t) {
        wave_lds_fence();
        tile_stage<I>(stage, lane, G);
        if (t + 1 < t1) tile_issue_loads<I>(w, (t + 1) * 64 * C::NV, n_vec, lane, G);
        wave_lds_fence();
        tile_fetch<I>(stage, lane, R);
        const uint64_t seg = t * 64 + lane;
        const bool active = seg < n_seg;
        uint32_t maxabs, sign;
        block_constant<I>(R, lane, signed_norm != 0, maxabs, sign);
        const float m = bf16_bits_to_f32(maxabs | (sign << 15));
        const uint32_t s16 = f32_to_f16_bits(m);
        const float m_eff = f16_bits_to_f32(s16);
        uint32_t out[C::SEG / 8];
        bool fast = FAST && __builtin_amdgcn_ballot_w64(!maxabs_is_ordinary(maxabs)) == 0;
        if (fast) {
            const BlockDiv dv = make_block_div(m_eff);
#pragma unroll
            for (int j = 0; j < C::SEG / 8; ++j) {
                uint32_t acc = 0;
#pragma unroll
                for (int e = 7; e >= 0; --e) {
                    float x = div_fast(seg_f32(R, 8 * j + e), dv);
                    uint32_t off = __float_as_uint(__builtin_fmaf(x, BIN_SCALE, BIN_MAGIC)) & BIN_MASK;
                    uint2 en = *reinterpret_cast<const uint2*>(reinterpret_cast<const char*>(tab) + off);
                    uint32_t code = en.y + (x > __uint_as_float(en.x) ? 1u : 0u);
                    acc = (acc << 4) + code;
                }
                out[j] = acc;
            }
        } else {
#pragma unroll
            for (int j = 0; j < C::SEG / 8; ++j) {
                uint32_t acc = 0;
#pragma unroll
                for (int e = 7; e >= 0; --e) {
                    float f = seg_f32(R, 8 * j + e);
                    float x = (m_eff == 0.0f) ? 0.0f : f / m_eff;
                    acc = (acc << 4) + (uint32_t)assign_code_generic(x, cb);
                }
                out[j] = acc;
            }
        }
        if (active) {
            uint4* dst = reinterpret_cast<uint4*>(codes + seg * (C::SEG / 8));
#pragma unroll
            for (int q = 0; q < C::SEG / 32; ++q) dst[q] = make_uint4(out[4 * q], out[4 * q + 1], out[4 * q + 2], out[4 * q + 3]);
            if ((lane & (C::LPB - 1)) == 0) scales[seg / C::LPB] = (uint16_t)s16;
        }
    }
}

// ================================================================================================ Lloyd step
// Per-level sums of the current block live in lane-private LDS columns acc[level][lane] (conflict-free).  One 64-bit
// LDS add per weight carries both the count and the sum of x of its level: the increment is the bit pattern of the
// binary64 number 2^-1008 + (x + 1) 2^-1020, i.e. exponent field 15 and mantissa (x + 1) 2^40 rounded to an
// integer.  Adding up to 256 of these as integers gives 15 K 2^52 + sum (x + 1) 2^40 with the second term below
// 2^52, so count K and sum separate again exactly.  Once per block the 16 columns are folded, with the block
// weight g, into binary64 registers:  A += g sum(x + 1),  den15 += g 15 K,  cnt15 += 15 K.
constexpr double LLOYD_INC_MUL = 0x1p-1020;
constexpr double LLOYD_INC_ADD = 0x1p-1008 + 0x1p-1020;

template <int I, bool FAST>
__global__ __launch_bounds__(256) void seg_lloyd_kernel(const uint4* __restrict__ w, uint64_t n_seg, CodebookArgs cb,
                                                         BinTable bt, int signed_norm, int weight_by_max2,
                                                         double* __restrict__ partials) {
    using C = SegCfg<I>;
    __shared__ __attribute__((aligned(16))) char stage_all[WAVES_PER_WG * C::STAGE_BYTES];
    __shared__ unsigned long long acc_all[WAVES_PER_WG * 16 * 64];
    __shared__ uint2 tab[33];
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid < 33) tab[tid] = make_uint2(__float_as_uint(bt.thr[tid]), bt.base[tid]);
    unsigned long long* acc = acc_all + wave * 16 * 64;
#pragma unroll
    for (int l = 0; l < 16; ++l) acc[l * 64 + lane] = 0ull;
    __syncthreads();
    char* stage = stage_all + wave * C::STAGE_BYTES;
    const uint32_t acc_lane = (uint32_t)(uintptr_t)(acc + lane);  // LDS byte address of this lane's column
    (void)acc_lane;
    const uint64_t n_vec = n_seg * C::NV;
    const uint64_t n_tiles = (n_seg + 63) / 64;
    const uint64_t n_waves = (uint64_t)gridDim.x * WAVES_PER_WG;
    const uint64_t gw = (uint64_t)blockIdx.x * WAVES_PER_WG + wave;
    const uint64_t t0 = n_tiles * gw / n_waves, t1 = n_tiles * (gw + 1) / n_waves;

    double A[16], den15[16], sxx_g = 0.0;
    uint32_t cnt15[16];
#pragma unroll
    for (int l = 0; l < 16; ++l) {
        A[l] = 0.0;
        den15[l] = 0.0;
        cnt15[l] = 0;
    }
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
        uint32_t maxabs, sign;
        block_constant<I>(R, lane, signed_norm != 0, maxabs, sign);
        const float m = bf16_bits_to_f32(maxabs | (sign << 15));
        const float m_eff = f16_bits_to_f32(f32_to_f16_bits(m));
        const double g = weight_by_max2 ? (double)m_eff * (double)m_eff : 1.0;
        double sxx = 0.0;
        bool fast = FAST && __builtin_amdgcn_ballot_w64(!maxabs_is_ordinary(maxabs)) == 0;
        if (active) {
            if (fast) {
                const BlockDiv dv = make_block_div(m_eff);
#pragma unroll
                for (int e = 0; e < C::SEG; ++e) {
                    float x = div_fast(seg_f32(R, e), dv);
                    uint32_t off = __float_as_uint(__builtin_fmaf(x, BIN_SCALE, BIN_MAGIC)) & BIN_MASK;
                    uint2 en = *reinterpret_cast<const uint2*>(reinterpret_cast<const char*>(tab) + off);
                    uint32_t code = en.y + (x > __uint_as_float(en.x) ? 1u : 0u);
                    double xd = (double)x;
                    double inc = fma(xd, LLOYD_INC_MUL, LLOYD_INC_ADD);
                    atomicAdd(&acc[code * 64 + lane], (unsigned long long)__double_as_longlong(inc));
                    sxx = fma(xd, xd, sxx);
                }
            } else {
#pragma unroll
                for (int e = 0; e < C::SEG; ++e) {
                    float f = seg_f32(R, e);
                    float x = (m_eff == 0.0f) ? 0.0f : f / m_eff;
                    uint32_t code = (uint32_t)assign_code_generic(x, cb);
                    double xd = (double)x;
                    double inc = fma(xd, LLOYD_INC_MUL, LLOYD_INC_ADD);
                    atomicAdd(&acc[code * 64 + lane], (unsigned long long)__double_as_longlong(inc));
                    sxx = fma(xd, xd, sxx);
                }
            }
            const double gs = g * 0x1p-40;
#pragma unroll
            for (int l = 0; l < 16; ++l) {
                unsigned long long v = atomicExch(&acc[l * 64 + lane], 0ull);
                uint32_t hi = (uint32_t)(v >> 32), lo = (uint32_t)v;
                uint32_t k15 = hi >> 20;
                double D = __hiloint2double((int)((hi & 0xFFFFFu) | 0x43300000u), (int)lo) - 0x1p52;  // sum (x+1) 2^40
                A[l] = fma(gs, D, A[l]);
                den15[l] = fma(g, (double)k15, den15[l]);
                cnt15[l] += k15;
            }
            sxx_g = fma(g, sxx, sxx_g);
        }
    }
    // fixed-order butterfly inside the wave; lane 0 stores the wave's partial
    double* dst = partials + gw * LLOYD_PART;
#pragma unroll
    for (int l = 0; l < 16; ++l) {
        double a = A[l], d = den15[l];
        unsigned long long c = cnt15[l];
#pragma unroll
        for (int mk = 32; mk >= 1; mk >>= 1) {
            a += __shfl_xor(a, mk, 64);
            d += __shfl_xor(d, mk, 64);
            c += (unsigned long long)__shfl_xor((long long)c, mk, 64);
        }
        if (lane == 0) {
            dst[l] = a;
            dst[16 + l] = d;
            dst[32 + l] = __longlong_as_double((long long)c);
        }
    }
    {
        double a = sxx_g;
#pragma unroll
        for (int mk = 32; mk >= 1; mk >>= 1) a += __shfl_xor(a, mk, 64);
        if (lane == 0) {
            dst[48] = a;
            dst[49] = 0.0;                       // sum of g * (outliers per block): none without OPQ
            dst[50] = __longlong_as_double(0ll); // outlier count
        }
    }
}

// Reduce the per-wave partials in a fixed order and turn them into the statistics of the C ABI:
//   num = A - den,  sse = sum g x^2 - 2 sum_l c_l num_l + sum_l c_l^2 den_l   (the three sums of the expanded square).
// out[0..15] num, [16..31] den, [32..47] cnt (as integer bits), [48] sse, [49] n_outliers (integer bits).
__global__ __launch_bounds__(1024) void seg_lloyd_final_kernel(const double* __restrict__ partials, uint32_t n_part,
                                                                CodebookArgs cb, uint32_t code_of_zero,
                                                                double* __restrict__ out) {
    __shared__ double tot[LLOYD_PART];
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (uint32_t q = wave; q < 51; q += 16) {
        const bool is_int = (q >= 32 && q < 48) || q == 50;
        double s = 0.0;
        unsigned long long si = 0;
        for (uint32_t p = lane; p < n_part; p += 64) {
            double v = partials[(uint64_t)p * LLOYD_PART + q];
            if (is_int) si += (unsigned long long)__double_as_longlong(v);
            else s += v;
        }
#pragma unroll
        for (int mk = 32; mk >= 1; mk >>= 1) {
            s += __shfl_xor(s, mk, 64);
            si += (unsigned long long)__shfl_xor((long long)si, mk, 64);
        }
        if (lane == 0) tot[q] = is_int ? __longlong_as_double((long long)si) : s;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        double sse = tot[48];
        const double koutg = tot[49];
        const unsigned long long kout = (unsigned long long)__double_as_longlong(tot[50]);
        for (int l = 0; l < 16; ++l) {
            double den = tot[16 + l] / 15.0;
            double a = tot[l];
            unsigned long long c = (unsigned long long)__double_as_longlong(tot[32 + l]) / 15ull;
            if ((uint32_t)l == code_of_zero) {  // zeroed outliers were counted as x = 0: take them out again
                den -= koutg;
                a -= koutg;
                c -= kout;
            }
            double num = a - den;
            out[l] = num;
            out[16 + l] = den;
            out[32 + l] = __longlong_as_double((long long)c);
            sse += cb.cb64[l] * (cb.cb64[l] * den - 2.0 * num);
        }
        out[48] = sse;
        out[49] = __longlong_as_double((long long)kout);
    }
}

}  // namespace bof4
