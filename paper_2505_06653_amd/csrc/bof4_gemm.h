// bof4_gemm.h - the decoder inside a matrix product for many tokens (the paper's inference path decodes the matrix to
// bfloat16 and multiplies in bfloat16; section 2.1 eq. 3, outliers of section 3.3):
//
//   y[t][r] = sum_c W^[r][c] x[t][c],   W^ = bfloat16(m_b * level[code]), outliers as stored - what bof4_dequantize
//   returns, never written to memory.
//
// The codes are still read once (0.5 + 2/I bytes per weight) and decoded once per 32 tokens, so per weight the cost is
// that of the matrix-vector kernel (extract, look the level up, one multiply, one conversion); the 32 multiply-adds
// per weight that follow are a dense contraction and go to the matrix cores: v_mfma_f32_32x32x16_bf16, A = 32 rows x
// 16 columns of decoded weights, B = the same 16 columns of 32 tokens, binary32 accumulators.  Lane l supplies
// row l % 32 of A and token l % 32 of B, eight consecutive columns each; which eight is the same for both (half
// l / 32 of a 64-column chunk takes its columns 32 (l / 32) + 8 j .. + 7 in the j-th of four products), so a lane
// decodes one 16-byte load of its row per chunk.
// A workgroup owns 32 rows; its waves take the 64-column chunks in turn and their 32 x 32 partial results are added
// in wave order through LDS.  Outliers: the decoded placeholder went through the product, so what is added per list
// entry is (value - bfloat16(m * level[code])) * x[t][col], from the table bof4_gemv_outlier_table makes in its
// rounded form, in list order, by a second small kernel; the same kernel adds the partial results when the columns
// of a matrix with few rows are split over several workgroups to fill the chip.  Every order is fixed: the result is
// bit-reproducible.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

#include "bof4_device.h"
#include "bof4_segment.h"
#include "bof4_gemv.h"

namespace bof4 {

constexpr uint32_t GEMM_ROWS = 32;    // rows per workgroup (M of the matrix-core product)
constexpr uint32_t GEMM_TOKENS = 32;  // tokens per launch (N)
constexpr uint32_t GEMM_CHUNK = 64;   // columns per wave and step: four products of K = 16
constexpr uint32_t GEMM_MAX_WAVES = 8;
constexpr uint32_t GEMM_TARGET_WGS = 512;  // two workgroups on each of the 256 compute units

typedef __bf16 gemm_bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 gemm_bf16x2 __attribute__((ext_vector_type(2)));
typedef float gemm_f32x2 __attribute__((ext_vector_type(2)));
typedef float gemm_f32x16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ uint32_t gemm_pack_bf16(float lo, float hi) {
    gemm_f32x2 v = {lo, hi};
    gemm_bf16x2 r = __builtin_convertvector(v, gemm_bf16x2);
    uint32_t u;
    __builtin_memcpy(&u, &r, 4);
    return u;
}

// Workgroup (t, s): rows 32 t .. 32 t + 31, the chunks s * waves + wave, + n_split * waves, ... of the row.  Its sum
// goes to dst[(s * n_tokens + token) * rows + row]: the result itself when n_split is 1, else one of n_split partial
// results that gemm_finish_kernel adds.
__global__ __launch_bounds__(64 * GEMM_MAX_WAVES) void gemm_kernel(
    const uint4* __restrict__ codes, const uint16_t* __restrict__ scales, uint32_t rows, uint32_t cols,
    uint32_t log2_block, CodebookArgs cb, const uint16_t* __restrict__ x, uint32_t n_tokens, float* __restrict__ dst) {
    struct Shared {
        float tab[16];
        float red[GEMM_MAX_WAVES * 16 * 64];  // per wave: accumulator register i of lane l at [i * 64 + l]
    };
    __shared__ __attribute__((aligned(16))) Shared sh;
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, n_waves = blockDim.x >> 6;
    if (tid < 16) sh.tab[tid] = cb.lv32[tid];
    __syncthreads();
    const char* tab = reinterpret_cast<const char*>(sh.tab);
    const uint32_t r0 = blockIdx.x * GEMM_ROWS;
    const uint32_t m = lane & 31, kh = lane >> 5;
    const uint32_t row = min(r0 + m, rows - 1);  // rows past the matrix repeat its last row and are dropped
    const bool tok_ok = m < n_tokens;            // lane l also supplies token l % 32
    const uint16_t* xrow = x + (uint64_t)min(m, n_tokens - 1) * cols;
    const uint32_t n_chunks = (cols + GEMM_CHUNK - 1) / GEMM_CHUNK;

    gemm_f32x16 acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.0f;
    for (uint32_t ch = blockIdx.y * n_waves + wave; ch < n_chunks; ch += gridDim.y * n_waves) {
        const uint32_t c = ch * GEMM_CHUNK + 32 * kh;  // this lane's 32 columns of the chunk
        const bool valid = c < cols;
        const uint64_t e = (uint64_t)row * cols + c;
        const uint4 q = valid ? load_stream(&codes[e >> 5]) : make_uint4(0u, 0u, 0u, 0u);
        const float msc = valid ? f16_bits_to_f32(__builtin_nontemporal_load(&scales[e >> log2_block])) : 0.0f;
        uint4 xb[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
            xb[j] = (valid && tok_ok) ? *reinterpret_cast<const uint4*>(xrow + c + 8 * j) : make_uint4(0u, 0u, 0u, 0u);
        const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            // byte i of `even` = 4 * code of element 2 i of the word, of `odd` = 4 * code of element 2 i + 1
            const uint32_t even = (w[j] << 2) & 0x3c3c3c3cu, odd = (w[j] >> 2) & 0x3c3c3c3cu;
            uint32_t a[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float le = *reinterpret_cast<const float*>(tab + ((even >> (8 * i)) & 0xffu));
                const float lo = *reinterpret_cast<const float*>(tab + ((odd >> (8 * i)) & 0xffu));
                a[i] = gemm_pack_bf16(msc * le, msc * lo);  // the decoder's product and rounding
            }
            gemm_bf16x8 A, B;
            const uint32_t bw[4] = {xb[j].x, xb[j].y, xb[j].z, xb[j].w};
            __builtin_memcpy(&A, a, 16);
            __builtin_memcpy(&B, bw, 16);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A, B, acc, 0, 0, 0);
        }
    }
    float* mine = sh.red + wave * 16 * 64;
#pragma unroll
    for (int i = 0; i < 16; ++i) mine[i * 64 + lane] = acc[i];
    __syncthreads();
    // The waves' results in wave order.  Accumulator i of lane l: row 8 (i / 4) + 4 (l / 32) + i % 4, token l % 32.
    float* out = dst + (uint64_t)blockIdx.y * n_tokens * rows;
    for (uint32_t idx = tid; idx < 16 * 64; idx += blockDim.x) {
        float s = 0.0f;
        for (uint32_t wv = 0; wv < n_waves; ++wv) s += sh.red[wv * 16 * 64 + idx];
        const uint32_t i = idx >> 6, l = idx & 63;
        const uint32_t mr = 8 * (i >> 2) + 4 * (l >> 5) + (i & 3u), n = l & 31;
        if (r0 + mr < rows && n < n_tokens) out[(uint64_t)n * rows + r0 + mr] = s;
    }
}

// y[token][row] = the n_split partial results in order, then the row's outlier entries in list order, each
// fma(delta, x[token][column], .) on a sum of their own that is added last.  part may be y itself when n_split is 1.
__global__ __launch_bounds__(256) void gemm_finish_kernel(const float* part, uint32_t n_split, uint32_t rows,
                                                          uint32_t cols, uint32_t n_tokens,
                                                          const uint32_t* __restrict__ strip_ptr,
                                                          const uint2* __restrict__ entries, uint32_t n_out,
                                                          uint32_t n_strips, const uint16_t* __restrict__ x,
                                                          float* y) {
    const uint64_t idx = (uint64_t)blockIdx.x * 256 + threadIdx.x, total = (uint64_t)n_tokens * rows;
    if (idx >= total) return;
    const uint32_t n = (uint32_t)(idx / rows), r = (uint32_t)(idx % rows);
    float s = 0.0f;
    for (uint32_t k = 0; k < n_split; ++k) s += part[k * total + idx];
    if (n_out != 0) {
        const uint32_t ea = min(strip_ptr[(uint64_t)r * n_strips], n_out);
        const uint32_t eb = min(strip_ptr[(uint64_t)(r + 1) * n_strips], n_out);
        float c = 0.0f;
        for (uint32_t k = ea; k < eb; ++k) {
            const uint2 en = entries[k];
            c = fmaf(__uint_as_float(en.y), bf16_bits_to_f32(x[(uint64_t)n * cols + min(en.x, cols - 1)]), c);
        }
        s += c;
    }
    y[idx] = s;
}

}  // namespace bof4
