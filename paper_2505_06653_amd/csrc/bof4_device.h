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
// bin(x) = (bits(fma(x, 16, 2^20 + 16)) & 0x1F8) / 8 (monotone in x).  The host puts at most one threshold into each
// bin: code(x) = base[bin] + (x > thr[bin]).  `fast` is 0 if some bin would need two thresholds or a threshold is
// too close to zero for the shortcut division; the kernels then use the 15-compare search.
struct BinTable {
    float thr[33];
    uint32_t base[33];
    uint32_t code_of_zero;
    uint32_t fast;
};
constexpr float BIN_SCALE = 16.0f;
constexpr float BIN_MAGIC = 1048576.0f + 16.0f;  // 2^20 + 16: ulp 1/8, mantissa = round(128 (x + 1))
constexpr uint32_t BIN_MASK = 0x1F8u;

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
// (so the stored binary16 constant equals m).  r = rcp(m) is within 1 ulp of 1/m; q0 = fl(w r) is within a few
// ulp of w/m; rem = w - q0 m is exact (fma, no underflow for |w| >= 2^-60); q1 = fl(q0 + rem r) is the rounding of
// a number within 2^-21 ulp of w/m.  w has 8 and m 8 significant bits, so w/m lies at least 2^-12 ulp away from
// every rounding boundary of binary32 and never on one: q1 is the correctly rounded quotient.  (Checked
// exhaustively against the hardware's IEEE division in the GPU tests.)  For |w| < 2^-60 the result may differ in
// the last bits of a number below 2^-45; the host only enables this path when no threshold is that small.
struct BlockDiv {
    float m;     // divisor (1 for a zero block)
    float rinv;  // rcp(m) (0 for a zero block, which makes every quotient +-0)
};
__device__ __forceinline__ BlockDiv make_block_div(float m_eff) {
    BlockDiv d;
    bool zero = (m_eff == 0.0f);
    d.m = zero ? 1.0f : m_eff;
    d.rinv = zero ? 0.0f : __builtin_amdgcn_rcpf(m_eff);
    return d;
}
__device__ __forceinline__ float div_fast(float w, const BlockDiv& d) {
    float q0 = w * d.rinv;
    float rem = __builtin_fmaf(-q0, d.m, w);
    return __builtin_fmaf(rem, d.rinv, q0);
}

// A block constant qualifies for the shortcut path if it is zero or a bfloat16 inside binary16's normal range
// [2^-14, 65280]: then binary16 storage is exact, |x| <= 1 and the division argument above applies.
__device__ __forceinline__ bool maxabs_is_ordinary(uint32_t maxabs_bits) {
    return maxabs_bits == 0u || (maxabs_bits >= 0x3880u && maxabs_bits <= 0x477Fu);
}

}  // namespace bof4
