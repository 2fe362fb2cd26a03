// bof4_gemv.h - the decoder inside a matrix-vector product (section 2.1 eq. 3 used in a linear layer, with the outlier
// list of section 3.3; the inference setting of the appendix on the runtime overhead of OPQ).
//
//   y[t][r] = sum_c w~[r][c] x[t][c],   w~ = m_b * level[code]  (exact product of eq. 3), outliers as stored.
//
// The matrix is read once as 4-bit codes (0.5 + 2/I bytes per weight): the kernel is a streaming scan bounded by HBM,
// not a dense contraction worth matrix cores at one or two tokens.  One wave owns a strip of 2048 columns (32 per
// lane, one 16-byte load per lane and row) and keeps its slice of x in registers as binary32; it walks the rows of its
// workgroup's chunk, looks the 32 levels up in a 16-entry LDS table (conflict-free: 16 words in 16 banks), multiplies
// the row-and-lane sum by the block constant once and adds the 64 lanes up with six DPP additions.  The strips of one
// row meet in LDS (a workgroup has at most eight waves; on matrices wider than 16384 columns a wave takes several
// strips in turn).  With an outlier list, a table made once per matrix holds per entry its column and
// value - m * level[code], and where the entries of each row and strip begin; they go one to a lane, and
// (value - m * level[code]) * x[col] joins that lane's sum before the wave adds up.
// Every sum has a fixed order, so y is bit-reproducible.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

#include "bof4_device.h"
#include "bof4_segment.h"

namespace bof4 {

constexpr uint32_t GEMV_STRIP = 2048;   // columns per wave
constexpr uint32_t GEMV_MAX_RC = 64;    // rows per workgroup at most: the last step has one lane per row
constexpr uint32_t GEMV_MAX_TOKENS = 2;    // tokens per launch: their slices of x live in registers
constexpr uint32_t GEMV_MAX_STRIPS = 16;  // up to 32768 columns
constexpr uint32_t GEMV_MAX_WAVES = 8;    // waves per workgroup: two per SIMD, so that several workgroups pack a CU

// Sum over the 64 lanes, delivered in lane 63 (other lanes hold prefixes).  Fixed tree: shifts by 1, 2, 4, 8 inside
// rows of 16 lanes, then lane 15 of each row into the next odd row, then lane 31 into the upper half.
__device__ __forceinline__ float wave_sum_lane63(float x) {
#define BOF4_DPP_F32(v, ctrl, row_mask, bound) \
    __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), ctrl, row_mask, 0xf, bound))
    x += BOF4_DPP_F32(x, 0x111, 0xf, true);
    x += BOF4_DPP_F32(x, 0x112, 0xf, true);
    x += BOF4_DPP_F32(x, 0x114, 0xf, true);
    x += BOF4_DPP_F32(x, 0x118, 0xf, true);
    x += BOF4_DPP_F32(x, 0x142, 0xa, false);
    x += BOF4_DPP_F32(x, 0x143, 0xc, false);
#undef BOF4_DPP_F32
    return x;
}

// strip_ptr[r * n_strips + s] = number of list entries with index < r * cols + s * GEMV_STRIP (the list is
// ascending), for every row and strip, and one closing entry: rows * n_strips + 1 values.
__global__ __launch_bounds__(256) void outlier_strip_offsets_kernel(const int64_t* __restrict__ out_idx,
                                                                    uint32_t n_out, uint64_t rows, uint64_t cols,
                                                                    uint32_t n_strips,
                                                                    uint32_t* __restrict__ strip_ptr) {
    const uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    if (i > rows * n_strips) return;
    const uint64_t r = i / n_strips, sidx = i - r * n_strips;
    const int64_t target = (int64_t)(r * cols + sidx * GEMV_STRIP);
    uint32_t lo = 0, hi = n_out;  // first entry >= target
    while (lo < hi) {
        const uint32_t mid = lo + (hi - lo) / 2;
        if (out_idx[mid] < target) lo = mid + 1; else hi = mid;
    }
    strip_ptr[i] = lo;
}

// The list in the form the product wants it: per entry its column and (value - m * level[code]), what the entry adds
// to its row's sum per unit of x.  An entry outside the matrix adds nothing.
__global__ __launch_bounds__(256) void outlier_delta_kernel(const uint8_t* __restrict__ codes8,
                                                            const uint16_t* __restrict__ scales, uint64_t n,
                                                            uint64_t cols, uint32_t log2_block, CodebookArgs cb,
                                                            const int64_t* __restrict__ out_idx,
                                                            const uint16_t* __restrict__ out_val, uint32_t n_out,
                                                            uint32_t rounded, uint2* __restrict__ entries) {
    const uint32_t k = blockIdx.x * 256 + threadIdx.x;
    if (k >= n_out) return;
    const uint64_t idx = (uint64_t)out_idx[k];
    uint2 e = make_uint2(0u, 0u);
    if (idx < n) {
        const uint32_t code = (codes8[idx >> 1] >> ((idx & 1u) * 4)) & 15u;
        e.x = (uint32_t)(idx % cols);
        const float msc = f16_bits_to_f32(scales[idx >> log2_block]), val = f16_bits_to_f32(out_val[k]);
        if (rounded)  // both as the decoder stores them in bfloat16: for products over the decoded matrix
            e.y = __float_as_uint(bf16_bits_to_f32(f32_to_bf16_rne(val)) -
                                  bf16_bits_to_f32(f32_to_bf16_rne(msc * cb.lv32[code])));
        else
            e.y = __float_as_uint(fmaf(-msc, cb.lv32[code], val));  // one rounding
    }
    entries[k] = e;
}

// Byte j of v (one instruction; written out so that the compiler does not fold it back into a shift and a mask of the
// packed codes, which costs two per weight).
template <int J>
__device__ __forceinline__ uint32_t byte_of(uint32_t v) {
    uint32_t r;
    asm("v_bfe_u32 %0, %1, %2, 8" : "=v"(r) : "v"(v), "n"(8 * J));
    return r;
}

// One workgroup: rows [blockIdx.x * rc, ...) of the matrix; wave w takes strips w, w + waves, ... one after the other.
// U rows are in flight per wave.
template <int T, bool OUTLIERS>
__global__ __launch_bounds__(64 * GEMV_MAX_WAVES, 4) void gemv_kernel(const uint4* __restrict__ codes, const uint16_t* __restrict__ scales,
                                                    uint32_t rows, uint32_t cols, uint32_t log2_block, uint32_t rc,
                                                    uint32_t n_strips, CodebookArgs cb,
                                                    const uint32_t* __restrict__ strip_ptr,
                                                    const uint2* __restrict__ entries, uint32_t n_out,
                                                    const uint16_t* __restrict__ x, float* __restrict__ y) {
    constexpr uint32_t U = T == 2 ? 1 : (OUTLIERS ? 2 : 4);  // measured best for each variant
    struct Shared {  // one object, so that the table sits at LDS offset 0 (reachable by an immediate offset)
        float tab[16];
        float part[GEMV_MAX_WAVES * GEMV_MAX_RC * T];
    };
    __shared__ __attribute__((aligned(16))) Shared sh;
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, n_waves = blockDim.x >> 6;
    if (tid < 16) sh.tab[tid] = cb.lv32[tid];
    const uint32_t r0 = blockIdx.x * rc;
    const uint32_t r1 = min(rows, r0 + rc);
    __syncthreads();
    const char* tab = reinterpret_cast<const char*>(sh.tab);

    for (uint32_t strip = wave; strip < n_strips; strip += n_waves) {
    const uint32_t col0 = strip * GEMV_STRIP + lane * 32;
    const bool active = col0 < cols;
    // with a list, the wave also keeps its slice of x as bfloat16 in LDS, where an entry's column can be looked up
    extern __shared__ __attribute__((aligned(16))) uint16_t x_lds[];
    if (OUTLIERS) wave_lds_fence();  // the previous strip's slice has been read
    float xr[T][32];
#pragma unroll
    for (int t = 0; t < T; ++t) {
        const uint4* xp = reinterpret_cast<const uint4*>(x + (uint64_t)t * cols + col0);
        uint4* xl = reinterpret_cast<uint4*>(x_lds + ((uint32_t)t * n_waves + wave) * GEMV_STRIP + lane * 32);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const uint4 v = active ? xp[k] : make_uint4(0u, 0u, 0u, 0u);
            if (OUTLIERS) xl[k] = v;
            const uint32_t u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                xr[t][8 * k + 2 * i] = __uint_as_float(u[i] << 16);
                xr[t][8 * k + 2 * i + 1] = __uint_as_float(u[i] & 0xffff0000u);
            }
        }
    }
    // where this strip's entries of the chunk's rows begin and end: lane j holds row r0 + j
    uint32_t p_lo = 0, p_hi = 0;
    if (OUTLIERS) {
        if (lane < r1 - r0) {
            p_lo = min(strip_ptr[(uint64_t)(r0 + lane) * n_strips + strip], n_out);
            p_hi = min(strip_ptr[(uint64_t)(r0 + lane) * n_strips + strip + 1], n_out);
        }
        wave_lds_fence();
    }
    // what one list entry adds: (value - decoded placeholder) * x
    auto correction = [&](uint2 e, float* c) {
        const uint32_t col = (e.x - strip * GEMV_STRIP) & (GEMV_STRIP - 1);  // inside the strip by construction
#pragma unroll
        for (int t = 0; t < T; ++t)
            c[t] = fmaf(__uint_as_float(e.y),
                        bf16_bits_to_f32(x_lds[((uint32_t)t * n_waves + wave) * GEMV_STRIP + col]), c[t]);
    };
    struct Group {  // U rows at a time: codes, block constants, and the rows' first 64 list entries
        uint4 q[U];
        float m[U];
        uint32_t pa[U], pb[U];
        uint2 oe[U];
    };
    auto issue = [&](uint32_t r, Group& g) {
#pragma unroll
        for (uint32_t u = 0; u < U; ++u) {
            const uint32_t rr = min(r + u, r1 - 1);  // rows past the chunk repeat its last row and are dropped
            const uint64_t e = (uint64_t)rr * cols + col0;
            g.q[u] = active ? load_stream(&codes[e >> 5]) : make_uint4(0u, 0u, 0u, 0u);
            g.m[u] = active ? f16_bits_to_f32(__builtin_nontemporal_load(&scales[e >> log2_block])) : 0.0f;
            if (OUTLIERS) {
                g.pa[u] = (uint32_t)__builtin_amdgcn_readlane((int)p_lo, (int)(rr - r0));
                g.pb[u] = (uint32_t)__builtin_amdgcn_readlane((int)p_hi, (int)(rr - r0));
                g.oe[u] = g.pa[u] + lane < g.pb[u] ? entries[g.pa[u] + lane] : make_uint2(0u, 0u);
            }
        }
    };
    auto compute = [&](uint32_t r, const Group& g) {
#pragma unroll
        for (uint32_t u = 0; u < U; ++u) {
            if (r + u >= r1) break;  // wave-uniform: the chunk's last group may be short
            const uint32_t w[4] = {g.q[u].x, g.q[u].y, g.q[u].z, g.q[u].w};
            float acc[T][2];
#pragma unroll
            for (int t = 0; t < T; ++t) acc[t][0] = acc[t][1] = 0.0f;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                // byte j of `even` = 4 * code of element 2 j, of `odd` = 4 * code of element 2 j + 1
                const uint32_t even = (w[k] << 2) & 0x3c3c3c3cu, odd = (w[k] >> 2) & 0x3c3c3c3cu;
                const uint32_t ae[4] = {byte_of<0>(even), byte_of<1>(even), byte_of<2>(even), byte_of<3>(even)};
                const uint32_t ao[4] = {byte_of<0>(odd), byte_of<1>(odd), byte_of<2>(odd), byte_of<3>(odd)};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float le = *reinterpret_cast<const float*>(tab + ae[j]);
                    const float lo = *reinterpret_cast<const float*>(tab + ao[j]);
#pragma unroll
                    for (int t = 0; t < T; ++t) {
                        acc[t][0] = fmaf(le, xr[t][8 * k + 2 * j], acc[t][0]);
                        acc[t][1] = fmaf(lo, xr[t][8 * k + 2 * j + 1], acc[t][1]);
                    }
                }
            }
            float c[T];
#pragma unroll
            for (int t = 0; t < T; ++t) c[t] = 0.0f;
            if (OUTLIERS) {
                correction(g.oe[u], c);  // no entry: delta 0 (a non-finite x makes every row non-finite anyway)
            }
#pragma unroll
            for (int t = 0; t < T; ++t) {
                const float s = wave_sum_lane63(fmaf(acc[t][0] + acc[t][1], g.m[u], c[t]));
                if (lane == 63) {  // the wave's strips add up in its own slot
                    float* slot = &sh.part[(wave * rc + (r + u - r0)) * T + t];
                    *slot = strip == wave ? s : *slot + s;
                }
            }
        }
    };
    // No second buffer of rows in flight: it was tried (with and without a list) and the registers it takes cost more
    // occupancy than the overlap gains; other waves cover the loads.
    for (uint32_t r = r0; r < r1; r += U) {
        Group g;
        issue(r, g);
        compute(r, g);
    }
    if (OUTLIERS) {
        // Rows with more than 64 list entries inside this strip: the loop above took the first 64 (one per lane); the
        // rest is added here, outside the hot loop (a loop of unknown length inside it cost 30 registers).
        unsigned long long many = __builtin_amdgcn_ballot_w64(lane < r1 - r0 && p_hi > p_lo && p_hi - p_lo > 64u);
        while (many != 0ull) {  // wave-uniform
            const uint32_t j = (uint32_t)__builtin_ctzll(many);
            many &= many - 1ull;
            const uint32_t a = (uint32_t)__builtin_amdgcn_readlane((int)p_lo, (int)j) + 64u;
            const uint32_t b = (uint32_t)__builtin_amdgcn_readlane((int)p_hi, (int)j);
            float c[T];
#pragma unroll
            for (int t = 0; t < T; ++t) c[t] = 0.0f;
            for (uint32_t k = a + lane; k < b; k += 64) correction(entries[k], c);
#pragma unroll
            for (int t = 0; t < T; ++t) {
                const float s = wave_sum_lane63(c[t]);
                if (lane == 63) sh.part[(wave * rc + j) * T + t] += s;
            }
        }
    }
    }  // strips of this wave
    __syncthreads();
    if (wave == 0 && lane < r1 - r0) {
#pragma unroll
        for (int t = 0; t < T; ++t) {
            float s = 0.0f;
            for (uint32_t p = 0; p < n_waves; ++p) s += sh.part[(p * rc + lane) * T + t];  // waves in order
            y[(uint64_t)t * rows + r0 + lane] = s;
        }
    }
}

}  // namespace bof4
