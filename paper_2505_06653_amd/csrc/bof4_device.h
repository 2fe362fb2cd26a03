// bof4_device.h - device-side building blocks shared by the gfx950 kernels of the BOF4 hot path.
//
// Everything here is exact integer / IEEE arithmetic; the comments state why each shortcut returns the same bits
// as the plain definition it replaces (block maximum: section 2.1 eq. 1 / section 3.1 eq. 4; normalisation:
// eq. 2; nearest level: section 3.2).
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace bof4 {

// ---------------------------------------------------------------------------------------------- kernel arguments
// Codebook-derived constants handed to the kernels by value (kernel argument segment, no device allocation).
struct CodebookArgs {
    float thr[16];    // 15 decision thresholds (+inf pad): code(x) = #{k : x > thr[k]}
    float lv32[16];   // levels rounded to binary32 (decoder)
    double cb64[16];  // levels in binary64 (Lloyd error term)
};

// Bin table for the branch-free nearest-level search.  x in [-1, 1] is mapped to one of 33 bins of width 1/16 by
// bin(x) = (bits(fma(x, 16, BIN_MAGIC)) & BIN_MASK) >> BIN_SHIFT (monotone in x): BIN_MAGIC = 2^(23 - BIN_SHIFT) + 16
// has an ulp of 2^-BIN_SHIFT, so the mantissa of the sum holds 16 (1 + x) in fixed point with the integer part - the
// bin - from bit BIN_SHIFT up.  The host puts at most one threshold into each bin: code(x) = base[bin] + (x >
// thr[bin]).  `fast` is 0 if some bin would need two thresholds or a threshold is too close to zero for the shortcut
// division; the kernels then use the 15-compare search.
struct BinTable {
    float thr[33];
    uint32_t base[33];
    uint32_t code_of_zero;
    uint32_t fast;
};
#ifndef BOF4_BIN_SHIFT
#define BOF4_BIN_SHIFT 3
#endif
constexpr int BIN_SHIFT = BOF4_BIN_SHIFT;
constexpr float BIN_SCALE = 16.0f;
constexpr float BIN_MAGIC = (float)(1u << (23 - BIN_SHIFT)) + 16.0f;
constexpr uint32_t BIN_MASK = 0x3Fu << BIN_SHIFT;
// In LDS a bin's entry (threshold, base code: 8 bytes) is repeated BIN_COPIES times, filling the 2^BIN_SHIFT bytes
// between two bin addresses; lane l reads copy l mod BIN_COPIES.  With 16 copies the 16 lanes that the LDS unit serves
// together always read from 16 different bank pairs, whatever their bins.
constexpr int BIN_COPIES = (1 << BIN_SHIFT) / 8;
constexpr int BIN_TABLE_ENTRIES = 33 * BIN_COPIES;

// ---------------------------------------------------------------------------------------------- bit helpers
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}
__device__ __forceinline__ uint32_t f32_to_f16_bits(float f) {
    _Float16 h = (_Float16)f;  // v_cvt_f16_f32, round to nearest even
    unsigned short s;
    __builtin_memcpy(&s, &h, 2);
    return s;
}
__device__ __forceinline__ float f16_bits_to_f32(uint32_t b) {
    unsigned short s = (unsigned short)b;
    _Float16 h;
    __builtin_memcpy(&h, &s, 2);
    return (float)h;
}

// Fill the LDS copy of the bin table (every lane of the workgroup takes part; the caller synchronises afterwards).
__device__ __forceinline__ void bin_table_fill(uint2* tab, const BinTable& bt, uint32_t tid, uint32_t n_threads) {
    for (uint32_t i = tid; i < (uint32_t)BIN_TABLE_ENTRIES; i += n_threads)
        tab[i] = make_uint2(__float_as_uint(bt.thr[i / BIN_COPIES]), bt.base[i / BIN_COPIES]);
}
// Byte offset of the lane's copy inside a bin's stretch of the table.
__device__ __forceinline__ uint32_t bin_lane_offset(uint32_t lane) { return (lane & (uint32_t)(BIN_COPIES - 1)) * 8u; }
// The (threshold, base code) entry of the bin that x falls into.
__device__ __forceinline__ uint2 bin_lookup(const uint2* tab, float x, uint32_t lane_off) {
    const uint32_t off = (__float_as_uint(__builtin_fmaf(x, BIN_SCALE, BIN_MAGIC)) & BIN_MASK) | lane_off;
    return *reinterpret_cast<const uint2*>(reinterpret_cast<const char*>(tab) + off);
}

// 16-byte load of data that is read exactly once (streaming: do not keep it in the caches).
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_stream(const uint4* p) {
    u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void store_stream(uint4* p, uint4 q) {
    u32x4 v = {q.x, q.y, q.z, q.w};
    __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(p));
}

typedef short s16x2 __attribute__((ext_vector_type(2)));
typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pk_max_i16(uint32_t a, uint32_t b) {
    s16x2 x, y;
    __builtin_memcpy(&x, &a, 4);
    __builtin_memcpy(&y, &b, 4);
    s16x2 r = __builtin_elementwise_max(x, y);
    uint32_t o;
    __builtin_memcpy(&o, &r, 4);
    return o;
}
__device__ __forceinline__ uint32_t pk_max_u16(uint32_t a, uint32_t b) {
    u16x2 x, y;
    __builtin_memcpy(&x, &a, 4);
    __builtin_memcpy(&y, &b, 4);
    u16x2 r = __builtin_elementwise_max(x, y);
    uint32_t o;
    __builtin_memcpy(&o, &r, 4);
    return o;
}

// Largest / smallest of three packed pairs of 16-bit patterns in binary16 order (one instruction each).  For
// patterns that are not binary16 NaNs (magnitude field <= 0x7C00) that order is the order of the bfloat16 values with
// the same patterns: sign first, then magnitude, +0 above -0; subnormal patterns are compared, not flushed.  A NaN
// pattern among the inputs comes out as a NaN pattern (callers test for it and fall back on integer compares).
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pk_max3_f16(uint32_t a, uint32_t b, uint32_t c) {
    f16x2 x, y, z;
    __builtin_memcpy(&x, &a, 4);
    __builtin_memcpy(&y, &b, 4);
    __builtin_memcpy(&z, &c, 4);
    f16x2 r = __builtin_elementwise_maximum(__builtin_elementwise_maximum(x, y), z);
    uint32_t o;
    __builtin_memcpy(&o, &r, 4);
    return o;
}
__device__ __forceinline__ uint32_t pk_min3_f16(uint32_t a, uint32_t b, uint32_t c) {
    f16x2 x, y, z;
    __builtin_memcpy(&x, &a, 4);
    __builtin_memcpy(&y, &b, 4);
    __builtin_memcpy(&z, &c, 4);
    f16x2 r = __builtin_elementwise_minimum(__builtin_elementwise_minimum(x, y), z);
    uint32_t o;
    __builtin_memcpy(&o, &r, 4);
    return o;
}

__device__ __forceinline__ uint32_t pk_sub_i16(uint32_t a, uint32_t b) {
    s16x2 x, y;
    __builtin_memcpy(&x, &a, 4);
    __builtin_memcpy(&y, &b, 4);
    s16x2 r = x - y;
    uint32_t o;
    __builtin_memcpy(&o, &r, 4);
    return o;
}
__device__ __forceinline__ uint32_t pk_sub_u16(uint32_t a, uint32_t b) {  // per-half wrap-around difference
    u16x2 x, y;
    __builtin_memcpy(&x, &a, 4);
    __builtin_memcpy(&y, &b, 4);
    u16x2 r = x - y;
    uint32_t o;
    __builtin_memcpy(&o, &r, 4);
    return o;
}
__device__ __forceinline__ uint32_t pk_sign_mask_i16(uint32_t a) {  // 0xFFFF in every half that is negative
    s16x2 x;
    __builtin_memcpy(&x, &a, 4);
    s16x2 r = x >> 15;
    uint32_t o;
    __builtin_memcpy(&o, &r, 4);
    return o;
}

// a.lo * b.lo + a.hi * b.hi + c for packed bfloat16 pairs, accumulated in binary32 (one instruction).  The rounding
// of the intermediate results is not specified; users allow DOT2_ROUNDINGS * 2^-24 * (|a.lo b.lo| + |a.hi b.hi| + |c|)
// of error per call: twice what the instruction was observed to reach at worst (3.0; the GPU tests repeat that
// measurement).
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
constexpr float DOT2_ROUNDINGS = 6.0f;
__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float c) {
    bf16x2 x, y;
    __builtin_memcpy(&x, &a, 4);
    __builtin_memcpy(&y, &b, 4);
    return __builtin_amdgcn_fdot2_f32_bf16(x, y, c, false);
}

// Inclusive prefix sum over the 64 lanes of a wave with data-parallel-primitive moves (6 additions): shifts by
// 1, 2, 4, 8 inside each row of 16 lanes (lanes shifted in from outside the row read 0), then lane 15 of every row
// is added to the whole next odd row, then lane 31 to the upper half.  All 64 lanes must be active.
__device__ __forceinline__ uint32_t wave_inclusive_scan_u32(uint32_t x) {
    int v = (int)x;
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, true);   // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, true);   // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, true);   // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, true);   // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);  // row_bcast:15 into rows 1 and 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);  // row_bcast:31 into rows 2 and 3
    return (uint32_t)v;
}

// Slow, always-valid nearest-level search.
__device__ __forceinline__ int assign_code_generic(float x, const CodebookArgs& cb) {
    int code = 0;
#pragma unroll
    for (int k = 0; k < 15; ++k) code += (x > cb.thr[k]) ? 1 : 0;
    return code;
}

// ---------------------------------------------------------------------------------------------- shortcut division
// x = w / m for a bfloat16 w and a block constant m that is a bfloat16 number inside binary16's normal range
// (so the stored binary16 constant equals m), in two operations per weight.  Per block: rh = rcp(m), within 1 ulp
// of 1/m; d = 1 - m rh, exact (the product has 32 significant bits of which the leading ~23 cancel); rl = fl(d rh).
// Then rh + rl = (1/m)(1 + e) with |e| < 2^-44.  Per weight: t = fl(w rl), x = fl(w rh + t) (one fused
// multiply-add): the rounding of a number within 2^-43 (relative) of w / m.  w and m have 8 significant bits each,
// so w / m lies at least 2^-33 (relative) away from every rounding boundary of binary32 and never on one: x is the
// correctly rounded quotient.  (Checked exhaustively against the hardware's IEEE division in the GPU tests.)  For
// |w| < 2^-60 the product w rl can fall among the subnormals and the result may differ in the last bits of a number
// below 2^-45; the host only enables this path when no threshold is that small.
struct BlockDiv {
    float rh;  // rcp(m) (0 for a zero block, which makes every quotient +-0)
    float rl;  // the correction (1/m - rh) to within 2^-23 of itself
};
__device__ __forceinline__ BlockDiv make_block_div(float m_eff) {
    BlockDiv d;
    const bool zero = (m_eff == 0.0f);
    const float r = __builtin_amdgcn_rcpf(zero ? 1.0f : m_eff);
    const float e = __builtin_fmaf(-m_eff, r, 1.0f);
    d.rh = zero ? 0.0f : r;
    d.rl = zero ? 0.0f : e * r;
    return d;
}
__device__ __forceinline__ float div_fast(float w, const BlockDiv& d) {
    return __builtin_fmaf(w, d.rh, w * d.rl);
}

// A block constant qualifies for the shortcut path if it is zero or a bfloat16 inside binary16's normal range
// [2^-14, 65280]: then binary16 storage is exact, |x| <= 1 and the division argument above applies.
__device__ __forceinline__ bool maxabs_is_ordinary(uint32_t maxabs_bits) {
    return maxabs_bits == 0u || (maxabs_bits >= 0x3880u && maxabs_bits <= 0x477Fu);
}

}  // namespace bof4
