// bof4_gemv.h - the decoder inside a matrix-vector product (section 2.1 eq. 3 used in a linear layer, with the outlier
// list of section 3.3; the inference setting of the appendix on the runtime overhead of OPQ).
//
//   y[t][r] = sum_c w~[r][c] x[t][c],   w~ = m_b * level[code]  (exact product of eq. 3), outliers as stored.
//
// The matrix is read once as 4-bit codes (0.5 + 2/I bytes per weight): the kernel is a streaming scan bounded by HBM,
// not a dense contraction worth matrix cores at one to four tokens.  One wave owns a strip of 2048 columns (32 per
// lane, one 16-byte load per lane and row) and keeps its slice of x in registers as binary32; it walks the rows of its
// workgroup's chunk, looks the 32 levels up in a 16-entry LDS table (conflict-free: 16 words in 16 banks), multiplies
// the row-and-lane sum by the block constant once and adds the 64 lanes up with six DPP additions.  The strips of one
// row meet in LDS; where an outlier list is given one more wave of the workgroup turns the chunk's entries into
// corrections (value - m * level[code]) * x[col], one entry per lane, and adds them per row in list order.  Every sum
// has a fixed order, so y is bit-reproducible.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

#include "bof4_device.h"
#include "bof4_segment.h"

namespace bof4 {

constexpr uint32_t GEMV_STRIP = 2048;   // columns per wave
constexpr uint32_t GEMV_MAX_RC = 64;    // rows per workgroup at most: the last step has one lane per row
constexpr uint32_t GEMV_CORR = 1024;    // list entries the outlier wave handles per round
constexpr uint32_t GEMV_MAX_TOKENS = 2;    // tokens per launch: their slices of x live in registers
constexpr uint32_t GEMV_UNROLL = 4;     // rows in flight per wave

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

// row_ptr[r] = number of list entries with index < r * cols, r = 0 .. rows (the list is ascending).
__global__ __launch_bounds__(256) void outlier_row_offsets_kernel(const int64_t* __restrict__ out_idx, uint32_t n_out,
                                                                  uint64_t rows, uint64_t cols,
                                                                  uint32_t* __restrict__ row_ptr) {
    const uint64_t r = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    if (r > rows) return;
    const int64_t target = (int64_t)(r * cols);
    uint32_t lo = 0, hi = n_out;  // first entry >= target
    while (lo < hi) {
        const uint32_t mid = lo + (hi - lo) / 2;
        if (out_idx[mid] < target) lo = mid + 1; else hi = mid;
    }
    row_ptr[r] = lo;
}

// Dynamic LDS: 16 levels | part[(S + OUTLIERS) * rc * T] | (OUTLIERS) row offsets [rc + 1] | corr[GEMV_CORR * T].
template <int T, bool OUTLIERS>
__global__ __launch_bounds__(1024) void gemv_kernel(const uint4* __restrict__ codes, const uint16_t* __restrict__ scales,
                                                    uint32_t rows, uint32_t cols, uint32_t log2_block, uint32_t rc,
                                                    uint32_t n_strips, CodebookArgs cb,
                                                    const int64_t* __restrict__ out_idx,
                                                    const uint16_t* __restrict__ out_val, uint32_t n_out,
                                                    const uint32_t* __restrict__ row_ptr,
                                                    const uint16_t* __restrict__ x, float* __restrict__ y) {
    extern __shared__ __attribute__((aligned(16))) float lds[];
    float* tab = lds;
    float* part = lds + 16;
    const uint32_t n_parts = n_strips + (OUTLIERS ? 1u : 0u);
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid < 16) tab[tid] = cb.lv32[tid];
    const uint32_t r0 = blockIdx.x * rc;
    const uint32_t r1 = min(rows, r0 + rc);
    __syncthreads();

    if (wave < n_strips) {
        const uint32_t col0 = wave * GEMV_STRIP + lane * 32;
        const bool active = col0 < cols;
        float xr[T][32];
#pragma unroll
        for (int t = 0; t < T; ++t) {
            const uint4* xp = reinterpret_cast<const uint4*>(x + (uint64_t)t * cols + col0);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const uint4 v = active ? xp[k] : make_uint4(0u, 0u, 0u, 0u);
                const uint32_t u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    xr[t][8 * k + 2 * i] = __uint_as_float(u[i] << 16);
                    xr[t][8 * k + 2 * i + 1] = __uint_as_float(u[i] & 0xffff0000u);
                }
            }
        }
        for (uint32_t r = r0; r < r1; r += GEMV_UNROLL) {
            uint4 q[GEMV_UNROLL];
            float m[GEMV_UNROLL];
#pragma unroll
            for (uint32_t u = 0; u < GEMV_UNROLL; ++u) {
                const uint32_t rr = min(r + u, r1 - 1);  // rows past the chunk repeat its last row and are dropped
                const uint64_t e = (uint64_t)rr * cols + col0;
                q[u] = active ? load_stream(&codes[e >> 5]) : make_uint4(0u, 0u, 0u, 0u);
                m[u] = active ? f16_bits_to_f32(__builtin_nontemporal_load(&scales[e >> log2_block])) : 0.0f;
            }
#pragma unroll
            for (uint32_t u = 0; u < GEMV_UNROLL; ++u) {
                const uint32_t w[4] = {q[u].x, q[u].y, q[u].z, q[u].w};
                float acc[T][2];
#pragma unroll
                for (int t = 0; t < T; ++t) acc[t][0] = acc[t][1] = 0.0f;
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    // byte j of `even` = 4 * code of element 2 j, of `odd` = 4 * code of element 2 j + 1
                    const uint32_t even = (w[k] << 2) & 0x3c3c3c3cu, odd = (w[k] >> 2) & 0x3c3c3c3cu;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const float le = *reinterpret_cast<const float*>(reinterpret_cast<const char*>(tab) +
                                                                         ((even >> (8 * j)) & 0xffu));
                        const float lo = *reinterpret_cast<const float*>(reinterpret_cast<const char*>(tab) +
                                                                         ((odd >> (8 * j)) & 0xffu));
#pragma unroll
                        for (int t = 0; t < T; ++t) {
                            acc[t][0] = fmaf(le, xr[t][8 * k + 2 * j], acc[t][0]);
                            acc[t][1] = fmaf(lo, xr[t][8 * k + 2 * j + 1], acc[t][1]);
                        }
                    }
                }
#pragma unroll
                for (int t = 0; t < T; ++t) {
                    const float s = wave_sum_lane63((acc[t][0] + acc[t][1]) * m[u]);
                    if (lane == 63 && r + u < r1) part[(wave * rc + (r + u - r0)) * T + t] = s;
                }
            }
        }
    } else if (OUTLIERS) {
        // the outlier wave: corrections of the chunk's list entries, one entry per lane, summed per row in list order
        uint32_t* rp = reinterpret_cast<uint32_t*>(part + n_parts * rc * T);
        float* corr = reinterpret_cast<float*>(rp + rc + 1);
        const uint32_t n_rows = r1 - r0;
        for (uint32_t j = lane; j <= n_rows; j += 64) rp[j] = min(row_ptr[r0 + j], n_out);
        wave_lds_fence();
        const uint32_t e0 = rp[0], e1 = rp[n_rows];
        const uint32_t my_lo = lane < n_rows ? rp[lane] : 0u, my_hi = lane < n_rows ? rp[lane + 1] : 0u;
        const uint64_t n = (uint64_t)rows * cols;
        const uint64_t first = (uint64_t)r0 * cols;
        const uint8_t* codes8 = reinterpret_cast<const uint8_t*>(codes);
        float rowcorr[T];
#pragma unroll
        for (int t = 0; t < T; ++t) rowcorr[t] = 0.0f;
        for (uint32_t base = e0; base < e1; base += GEMV_CORR) {
            const uint32_t cnt = min(GEMV_CORR, e1 - base);
            for (uint32_t k = lane; k < cnt; k += 64) {
                const uint64_t idx = (uint64_t)out_idx[base + k];
                float c[T];
#pragma unroll
                for (int t = 0; t < T; ++t) c[t] = 0.0f;
                if (idx >= first && idx < n) {  // an entry outside the matrix changes nothing
                    const uint32_t col = (uint32_t)(idx - first) % cols;  // the chunk spans fewer than 2^32 weights
                    const uint32_t code = (codes8[idx >> 1] >> ((idx & 1u) * 4)) & 15u;
                    const float old = f16_bits_to_f32(scales[idx >> log2_block]) * tab[code];
                    const float d = f16_bits_to_f32(out_val[base + k]) - old;
#pragma unroll
                    for (int t = 0; t < T; ++t) c[t] = d * bf16_bits_to_f32(x[(uint64_t)t * cols + col]);
                }
#pragma unroll
                for (int t = 0; t < T; ++t) corr[k * T + t] = c[t];
            }
            wave_lds_fence();
            const uint32_t lo = max(my_lo, base), hi = min(my_hi, base + cnt);
            for (uint32_t k = lo; k < hi; ++k) {
#pragma unroll
                for (int t = 0; t < T; ++t) rowcorr[t] += corr[(k - base) * T + t];
            }
            wave_lds_fence();
        }
        if (lane < n_rows) {
#pragma unroll
            for (int t = 0; t < T; ++t) part[(n_strips * rc + lane) * T + t] = rowcorr[t];
        }
    }
    __syncthreads();
    if (wave == 0 && lane < r1 - r0) {
#pragma unroll
        for (int t = 0; t < T; ++t) {
            float s = 0.0f;
            for (uint32_t p = 0; p < n_parts; ++p) s += part[(p * rc + lane) * T + t];  // strips in order, outliers last
            y[(uint64_t)t * rows + r0 + lane] = s;
        }
    }
}

}  // namespace bof4
