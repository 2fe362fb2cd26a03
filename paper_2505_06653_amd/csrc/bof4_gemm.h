// bof4_gemm.h - the decoder inside a matrix product for many tokens (the paper's inference path decodes the matrix to
// bfloat16 and multiplies in bfloat16; section 2.1 eq. 3, outliers of section 3.3):
//
//   y[t][r] = sum_c W^[r][c] x[t][c],   W^ = bfloat16(m_b * level[code]), outliers as stored - what bof4_dequantize
//   returns, never written to memory.
//
// The codes are still read once (0.5 + 2/I bytes per weight) and decoded once per 32 tokens, so per weight the cost is
// that of the matrix-vector kernel (extract, look the level up, one multiply, one conversion); the 32 multiply-adds
// per weight that follow are a dense contraction and go to the matrix cores: v_mfma_f32_32x32x16_bf16, A = 32 rows x
// 16 columns of decoded weights, B = the same 16 columns of 32 tokens, binary32 accumulators; up to four tiles of
// 32 tokens share one decoded A.  Codes, constants and x are read in that order from copies laid out for it (the
// matrix once, x per call), so that every load of a wave is one run of consecutive bytes.  Lane l supplies
// row l % 32 of A and token l % 32 of B, eight consecutive columns each; which eight is the same for both (half
// l / 32 of a 64-column chunk takes its columns 32 (l / 32) + 8 j .. + 7 in the j-th of four products), so a lane
// decodes one 16-byte load of its row per chunk.
// A workgroup owns 32 or 64 rows (one or two tiles per wave: with two, every word of x read serves both); its waves
// take the 64-column chunks in turn and their 32 x 32 partial results are added in wave order through LDS.  Outliers: the decoded placeholder went through the product, so what is added per list
// entry is (value - bfloat16(m * level[code])) * x[t][col], from the table bof4_gemv_outlier_table makes in its
// rounded form.  When the columns of a matrix with few rows are split over several workgroups to fill the chip, a
// second small kernel adds their partial results.  Every order is fixed: the result is bit-reproducible.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

#include "bof4_device.h"
#include "bof4_segment.h"
#include "bof4_gemv.h"

namespace bof4 {

constexpr uint32_t GEMM_ROWS = 32;    // rows per tile (M of the matrix-core product)
constexpr uint32_t GEMM_MAX_R = 2;    // tiles of rows per workgroup: each word of x read serves up to 64 rows
constexpr uint32_t GEMM_TOKENS = 32;  // tokens per tile (N of the matrix-core product)
constexpr uint32_t GEMM_MAX_TILES = 4;  // token tiles per launch: the codes are decoded once per 128 tokens
constexpr uint32_t GEMM_CHUNK = 64;   // columns per wave and step: four products of K = 16
constexpr uint32_t GEMM_MAX_WAVES = 8;
// Workgroups wanted before the columns are also split over workgroups: three quarters of the 256 compute units.
// Measured: splitting further (to 256, 512 or 1024 workgroups) costs more in partial results and in the epilogue per
// workgroup than the fuller chip gains; fewer than 192 leave too much of it idle.
constexpr uint32_t GEMM_TARGET_WGS = 192;

typedef __bf16 gemm_bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 gemm_bf16x2 __attribute__((ext_vector_type(2)));
typedef float gemm_f32x2 __attribute__((ext_vector_type(2)));
typedef float gemm_f32x16 __attribute__((ext_vector_type(16)));

// Sum over each row of 16 lanes, delivered in its lane 15 (the other lanes hold prefixes): shifts by 1, 2, 4, 8.
__device__ __forceinline__ float row16_sum_lane15(float x) {
#define BOF4_ROW_SHR_F32(v, ctrl) __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), ctrl, 0xf, 0xf, true))
    x += BOF4_ROW_SHR_F32(x, 0x111);
    x += BOF4_ROW_SHR_F32(x, 0x112);
    x += BOF4_ROW_SHR_F32(x, 0x114);
    x += BOF4_ROW_SHR_F32(x, 0x118);
#undef BOF4_ROW_SHR_F32
    return x;
}

__device__ __forceinline__ uint32_t gemm_pack_bf16(float lo, float hi) {
    gemm_f32x2 v = {lo, hi};
    gemm_bf16x2 r = __builtin_convertvector(v, gemm_bf16x2);
    uint32_t u;
    __builtin_memcpy(&u, &r, 4);
    return u;
}

// The codes and block constants in the order the products read them, made once per matrix: per tile of 32 rows and
// chunk of 64 columns GEMM_TILE_BYTES consecutive bytes - one 16-byte word of codes per lane (row = lane % 32 of the
// tile, columns 32 (lane / 32) .. + 31 of the chunk), then one binary16 constant per lane (that of the lane's 32
// columns).  Rows past the matrix and columns past its width hold code 0 and constant 0: they add nothing.
constexpr uint32_t GEMM_TILE_BYTES = 64 * 16 + 64 * 2;
__global__ __launch_bounds__(256) void gemm_pack_weights_kernel(const uint4* __restrict__ codes,
                                                                const uint16_t* __restrict__ scales, uint32_t rows,
                                                                uint32_t cols, uint32_t log2_block, uint32_t n_chunks,
                                                                uint64_t n_tiles, char* __restrict__ packed) {
    const uint64_t idx = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= n_tiles * 64) return;
    const uint32_t lane = (uint32_t)(idx & 63);
    const uint64_t tile = idx >> 6;
    const uint32_t ch = (uint32_t)(tile % n_chunks), rt = (uint32_t)(tile / n_chunks);
    const uint32_t row = rt * GEMM_ROWS + (lane & 31), c = ch * GEMM_CHUNK + 32 * (lane >> 5);
    uint4 q = make_uint4(0u, 0u, 0u, 0u);
    uint16_t m = 0;
    if (row < rows && c < cols) {
        const uint64_t e = (uint64_t)row * cols + c;
        q = codes[e >> 5];
        m = scales[e >> log2_block];
    }
    char* out = packed + tile * GEMM_TILE_BYTES;
    reinterpret_cast<uint4*>(out)[lane] = q;
    reinterpret_cast<uint16_t*>(out + 1024)[lane] = m;
}

// x in the order the products read it, made once per call: for every tile of 32 tokens, chunk of 64 columns and
// product j one 16-byte word per lane (token = lane % 32 of the tile, columns 32 (lane / 32) + 8 j .. + 7 of the
// chunk), so that a wave's load is 1 KiB of consecutive memory; zeros past the last token and the last column.
// With a list also x transposed, xt[column][token] (n_pad tokens per column), for the outlier entries.
__global__ __launch_bounds__(256) void gemm_pack_x_kernel(const uint16_t* __restrict__ x, uint32_t n_tokens,
                                                          uint32_t cols, uint32_t n_chunks, uint32_t n_pad,
                                                          uint4* __restrict__ xp, uint16_t* __restrict__ xt) {
    const uint64_t idx = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    const uint64_t total = (uint64_t)(n_pad / 32) * n_chunks * 256;
    if (idx >= total) return;
    const uint32_t lane = (uint32_t)(idx & 63), j = (uint32_t)((idx >> 6) & 3);
    const uint64_t tc = idx >> 8;
    const uint32_t ch = (uint32_t)(tc % n_chunks), tile = (uint32_t)(tc / n_chunks);
    const uint32_t n = tile * 32 + (lane & 31), c = ch * GEMM_CHUNK + 32 * (lane >> 5) + 8 * j;
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (n < n_tokens && c < cols) v = *reinterpret_cast<const uint4*>(x + (uint64_t)n * cols + c);
    xp[idx] = v;
    if (xt != nullptr && c < cols) {
        const uint32_t wv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 8; ++i)
            xt[(uint64_t)(c + i) * n_pad + n] = (uint16_t)(wv[i >> 1] >> (16 * (i & 1)));
    }
}

// Workgroup (b, s): R tiles of 32 rows (32 R b ..), the chunks s * waves + wave, + n_split * waves, ... of the row,
// NT tiles of 32 tokens (tile0 ..).  Its sum goes to dst[(s * n_tokens + token) * rows + row], token counted from
// the first of tile0: the result itself when n_split is 1, else one of n_split partial results that gemm_sum_kernel
// adds.  The outlier entries of a row are added by one of the workgroups that share it, to that workgroup's sum.
// The packed matrix holds a multiple of GEMM_MAX_R row tiles.
template <int R, int NT, bool OUTLIERS>
__global__ __launch_bounds__(64 * GEMM_MAX_WAVES) void gemm_kernel(
    const char* __restrict__ packed, uint32_t rows, uint32_t cols, CodebookArgs cb,
    const uint32_t* __restrict__ strip_ptr, const uint2* __restrict__ entries, uint32_t n_out, uint32_t n_strips,
    const uint4* __restrict__ xp, const uint16_t* __restrict__ xt, uint32_t n_pad, uint32_t tile0, uint32_t n_tokens,
    float* __restrict__ dst) {
    struct Shared {
        float tab[16];
        float red[GEMM_MAX_WAVES * 16 * 64];         // per wave: accumulator register i of lane l at [i * 64 + l]
        float corr[OUTLIERS ? NT * 32 * 32 : 1];     // [token tile][row][token] of one tile of rows
    };
    __shared__ __attribute__((aligned(16))) Shared sh;
    const uint32_t tid = threadIdx.x, lane = tid & 63, n_waves = blockDim.x >> 6;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    if (tid < 16) sh.tab[tid] = cb.lv32[tid];
    __syncthreads();
    const char* tab = reinterpret_cast<const char*>(sh.tab);
    const uint32_t n_chunks = (cols + GEMM_CHUNK - 1) / GEMM_CHUNK;
    const uint32_t stride = gridDim.y * n_waves;

    gemm_f32x16 acc[R][NT];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[r][t][i] = 0.0f;

    // What the chunk after this one needs (codes, constants and - where the registers allow it - x) is on its way
    // while this one is decoded and multiplied, in two sets of registers used in turn.  Past the last chunk the last
    // one is read again and not used.
    constexpr bool X_AHEAD = R * NT <= 2;
    struct Operands {
        uint4 q[R], xb[NT][4];
        uint16_t m[R];
    };
    auto fetch_x = [&](Operands& o, uint32_t chunk) {
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                o.xb[t][j] = xp[((uint64_t)(tile0 + t) * n_chunks + chunk) * 256 + j * 64 + lane];
    };
    const char* my_tiles = packed + (uint64_t)blockIdx.x * R * n_chunks * GEMM_TILE_BYTES;
    auto fetch = [&](Operands& o, uint32_t chunk) {  // this lane's 32 columns of the chunk, in each tile of rows
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const char* tile = my_tiles + ((uint64_t)r * n_chunks + chunk) * GEMM_TILE_BYTES;
            o.q[r] = load_stream(reinterpret_cast<const uint4*>(tile) + lane);
            o.m[r] = __builtin_nontemporal_load(reinterpret_cast<const uint16_t*>(tile + 1024) + lane);
        }
        if (X_AHEAD) fetch_x(o, chunk);
    };
    auto multiply = [&](Operands& o, uint32_t chunk) {
        if (!X_AHEAD) {
            fetch_x(o, chunk);
            __builtin_amdgcn_sched_barrier(0);  // x is on its way while the first tile of rows is decoded
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const float msc = f16_bits_to_f32(o.m[r]);
            const uint32_t w[4] = {o.q[r].x, o.q[r].y, o.q[r].z, o.q[r].w};
            gemm_bf16x8 A[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                // byte i of `even` = 4 * code of element 2 i of the word, of `odd` = 4 * code of element 2 i + 1
                const uint32_t even = (w[j] << 2) & 0x3c3c3c3cu, odd = (w[j] >> 2) & 0x3c3c3c3cu;
                const uint32_t oe[4] = {byte_of<0>(even), byte_of<1>(even), byte_of<2>(even), byte_of<3>(even)};
                const uint32_t oo[4] = {byte_of<0>(odd), byte_of<1>(odd), byte_of<2>(odd), byte_of<3>(odd)};
                uint32_t a[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float le = *reinterpret_cast<const float*>(tab + oe[i]);
                    const float lo = *reinterpret_cast<const float*>(tab + oo[i]);
                    a[i] = gemm_pack_bf16(msc * le, msc * lo);  // the decoder's product and rounding
                }
                __builtin_memcpy(&A[j], a, 16);
            }
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    gemm_bf16x8 B;
                    const uint32_t bw[4] = {o.xb[t][j].x, o.xb[t][j].y, o.xb[t][j].z, o.xb[t][j].w};
                    __builtin_memcpy(&B, bw, 16);
                    acc[r][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[j], B, acc[r][t], 0, 0, 0);
                }
        }
    };
    Operands o0, o1;
    uint32_t ch = blockIdx.y * n_waves + wave;
    const uint32_t last = n_chunks - 1;
    const uint32_t n_iter = ch < n_chunks ? (last - ch) / stride + 1 : 0;
    fetch(o0, min(ch, last));
    if (n_iter & 1u) {  // an odd one first, so that the rest goes in pairs
        multiply(o0, ch);
        ch += stride;
        fetch(o0, min(ch, last));
    }
    for (uint32_t it = n_iter >> 1; it > 0; --it) {  // o0 holds chunk ch
        fetch(o1, ch + stride);
        __builtin_amdgcn_sched_barrier(0);  // the loads first, then the arithmetic
        multiply(o0, ch);
        fetch(o0, min(ch + 2 * stride, last));
        __builtin_amdgcn_sched_barrier(0);
        multiply(o1, ch + stride);
        ch += 2 * stride;
    }

    const uint32_t lists = min(gridDim.y, GEMM_ROWS);
    const bool with_list = OUTLIERS && blockIdx.y < lists;
    float* mine = sh.red + wave * 16 * 64;
    float* out = dst + (uint64_t)blockIdx.y * n_tokens * rows;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const uint32_t r0 = (blockIdx.x * R + r) * GEMM_ROWS;
        // The list: row mr of the tile belongs to the workgroup with s = mr % (number of workgroups sharing the
        // tile), whose waves take their rows in turn.  Per row the wave works as 16 slots of 4 lanes (lane = 16 g +
        // slot): slot e takes the entries e, e + 16, ... of the row in that order, its lane g the tokens 8 g .. 8 g + 7
        // of every token tile (runs of 16 bytes of x transposed): c[token] = fma(delta, x[token][column], c[token]);
        // then the 16 slots' sums are added inside their row of 16 lanes (shifts by 1, 2, 4, 8: no LDS traffic).
        if (with_list) {
            if (r > 0) __syncthreads();  // the corrections of the tile of rows before have been read
            const uint32_t slot = lane & 15, g = lane >> 4;
            for (uint32_t mr = blockIdx.y + lists * wave; mr < GEMM_ROWS; mr += lists * n_waves) {
                uint32_t ea = 0, eb = 0;
                if (r0 + mr < rows) {
                    ea = min(strip_ptr[(uint64_t)(r0 + mr) * n_strips], n_out);
                    eb = min(strip_ptr[(uint64_t)(r0 + mr + 1) * n_strips], n_out);
                }
                float c[NT][8];
#pragma unroll
                for (int t = 0; t < NT; ++t)
#pragma unroll
                    for (int i = 0; i < 8; ++i) c[t][i] = 0.0f;
                const uint16_t* xg = xt + tile0 * 32 + 8 * g;
                constexpr int U = 8 / NT;  // entries per lane and round: 8 loads of x in flight per lane
                for (uint32_t kb = ea; kb < eb; kb += 16 * U) {  // kb: the round's first entry (the same in all lanes)
                    const uint32_t k0 = kb + slot;
                    uint2 en[U];
#pragma unroll
                    for (int u = 0; u < U; ++u)
                        if (kb + 16 * u < eb) en[u] = entries[min(k0 + 16 * u, eb - 1)];  // past the row: not used
                    uint4 xv[U][NT];
#pragma unroll
                    for (int u = 0; u < U; ++u)
                        if (kb + 16 * u < eb) {
#pragma unroll
                            for (int t = 0; t < NT; ++t)
                                xv[u][t] = *reinterpret_cast<const uint4*>(
                                    xg + (uint64_t)min(en[u].x, cols - 1) * n_pad + 32 * t);
                        }
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        if (kb + 16 * u >= eb) break;  // no slot has an entry from here on
                        // Past the row's last entry that entry is read again and counts with delta 0.  (Where its
                        // x is not finite the sum is not finite already.)
                        const float delta = k0 + 16 * u < eb ? __uint_as_float(en[u].y) : 0.0f;
#pragma unroll
                        for (int t = 0; t < NT; ++t) {
                            const uint32_t wv[4] = {xv[u][t].x, xv[u][t].y, xv[u][t].z, xv[u][t].w};
#pragma unroll
                            for (int i = 0; i < 4; ++i) {
                                c[t][2 * i] = fmaf(delta, __uint_as_float(wv[i] << 16), c[t][2 * i]);
                                c[t][2 * i + 1] = fmaf(delta, __uint_as_float(wv[i] & 0xffff0000u), c[t][2 * i + 1]);
                            }
                        }
                    }
                }
#pragma unroll
                for (int t = 0; t < NT; ++t) {
#pragma unroll
                    for (int i = 0; i < 8; ++i) c[t][i] = row16_sum_lane15(c[t][i]);
                    if (slot == 15) {
#pragma unroll
                        for (int i = 0; i < 8; ++i) sh.corr[(t * 32 + mr) * 32 + 8 * g + i] = c[t][i];
                    }
                }
            }
        }
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            if (r > 0 || t > 0) __syncthreads();  // the sums of the round before have been read
#pragma unroll
            for (int i = 0; i < 16; ++i) mine[i * 64 + lane] = acc[r][t][i];
            __syncthreads();
            // The waves' results in wave order.  Accumulator i of lane l: row 8 (i / 4) + 4 (l / 32) + i % 4 of the
            // tile, token l % 32.
            for (uint32_t idx = tid; idx < 16 * 64; idx += blockDim.x) {
                float s = 0.0f;
                for (uint32_t wv = 0; wv < n_waves; ++wv) s += sh.red[wv * 16 * 64 + idx];
                const uint32_t i = idx >> 6, l = idx & 63;
                const uint32_t mr = 8 * (i >> 2) + 4 * (l >> 5) + (i & 3u), n = 32 * t + (l & 31);
                if (with_list && mr % lists == blockIdx.y) s += sh.corr[(t * 32 + mr) * 32 + (l & 31)];
                if (r0 + mr < rows && n < n_tokens) out[(uint64_t)n * rows + r0 + mr] = s;
            }
        }
    }
}

// y = the n_split partial results in order (count elements each).
__global__ __launch_bounds__(256) void gemm_sum_kernel(const float* __restrict__ part, uint32_t n_split, uint64_t count,
                                                       float* __restrict__ y) {
    const uint64_t idx = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= count) return;
    float s = 0.0f;
    for (uint32_t k = 0; k < n_split; ++k) s += part[k * count + idx];
    y[idx] = s;
}

}  // namespace bof4
