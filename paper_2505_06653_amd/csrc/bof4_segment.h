// bof4_segment.h - the "one lane, one segment" kernels: quantise and Lloyd step.
//
// Work layout.  The flat weight array is cut into segments of SEG = min(I, 64) consecutive bfloat16 weights; a
// block of I weights is I/SEG (1, 2 or 4) neighbouring segments.  A wave processes tiles of 64 consecutive
// segments: it loads the tile with fully coalesced 16-byte loads, parks it in a wave-private, padded LDS buffer and
// reads it back transposed, so that every lane ends up holding one whole segment in registers.  All per-block work
// (maximum search of section 2.1 eq. 1 / section 3.1 eq. 4, normalisation eq. 2, nearest-level search of section
// 3.2, the sums of eq. 6) then runs inside a lane without cross-lane traffic.  A wave that writes an outlier list
// owns a contiguous range of tiles; otherwise the tiles are dealt out to the waves in turn.
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
constexpr int LLOYD_PART = 56;  // doubles per per-wave partial: A[16] den15[16] cnt15[16] sxx (unused) kout nout (+pad)

// ---------------------------------------------------------------------------------------------- tile movement
template <int I>
__device__ __forceinline__ void tile_issue_loads(const uint4* __restrict__ w, uint64_t first_vec, uint64_t n_vec,
                                                 uint32_t lane, uint4 (&G)[SegCfg<I>::NV]) {
    constexpr int NV = SegCfg<I>::NV;
    if (first_vec + 64 * NV <= n_vec) {  // wave-uniform: a whole tile, one address and constant offsets
        const uint4* p = w + first_vec + lane;
#pragma unroll
        for (int k = 0; k < NV; ++k) G[k] = load_stream(p + 64 * k);
    } else {
#pragma unroll
        for (int k = 0; k < NV; ++k) {
            uint64_t v = first_vec + (uint64_t)(64 * k) + lane;
            G[k] = v < n_vec ? load_stream(&w[v]) : make_uint4(0, 0, 0, 0);
        }
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
// Largest magnitude of the block and the sign of its first occurrence (lowest index).  P = largest pattern in value
// order, N = smallest: if the segment holds a non-negative number P is the largest of them, if it holds a negative
// number N is the one of largest magnitude.  The packed three-operand binary16 maximum / minimum does two registers
// (four weights) per instruction; if a pattern that binary16 reads as NaN turns up (a bfloat16 beyond 2^121: never in
// the ordinary range) the wave repeats the search with integer compares.
// Only when +a and -a are both present at the maximum does the order of the elements matter.  Such blocks (a few in a
// thousand for bfloat16 weights, i.e. one in every third tile) are settled one at a time by the whole wave: the
// block's lanes write their segments to `tie_buf` (wave-private LDS, I halfwords), every lane looks at I / 64 of the
// elements, and two ballots give the first element of that magnitude and its sign.
constexpr int TIE_BUF_HALFWORDS = 256;  // per wave: the largest block
template <int I>
__device__ __forceinline__ void block_constant(const uint32_t (&R)[SegCfg<I>::NR], uint32_t lane, bool signed_norm,
                                               uint32_t& maxabs, uint32_t& sign, uint16_t* tie_buf) {
    using C = SegCfg<I>;
    static_assert(C::NR % 2 == 0, "registers are taken in pairs");
    uint32_t P = pk_max3_f16(R[0], R[1], R[1]), N = pk_min3_f16(R[0], R[1], R[1]);
#pragma unroll
    for (int d = 2; d < C::NR; d += 2) {
        P = pk_max3_f16(P, R[d], R[d + 1]);
        N = pk_min3_f16(N, R[d], R[d + 1]);
    }
    const uint32_t nan_test = ((P & 0x7fffu) > 0x7C00u) | ((P & 0x7fff0000u) > 0x7C000000u) |
                              ((N & 0x7fffu) > 0x7C00u) | ((N & 0x7fff0000u) > 0x7C000000u);
    if (__builtin_amdgcn_ballot_w64(nan_test != 0) != 0) {  // wave-uniform: out-of-range input only
        P = R[0];
        N = R[0];
#pragma unroll
        for (int d = 1; d < C::NR; ++d) {
            P = pk_max_i16(P, R[d]);
            N = pk_max_u16(N, R[d]);
        }
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
    unsigned long long ties = __builtin_amdgcn_ballot_w64(absP == absN);
    constexpr int K = I >= 64 ? I / 64 : 1;  // elements of the block a lane looks at
    while (ties != 0ull) {  // wave-uniform: one block per turn
        const uint32_t first_lane = (uint32_t)__builtin_ctzll(ties) & ~(uint32_t)(C::LPB - 1);
        const bool mine = (lane & ~(uint32_t)(C::LPB - 1)) == first_lane;
        wave_lds_fence();  // the readers of the previous turn are done
        if (mine) {
            uint4* dst = reinterpret_cast<uint4*>(tie_buf + (lane - first_lane) * C::SEG);
#pragma unroll
            for (int k = 0; k < C::NV; ++k) dst[k] = make_uint4(R[4 * k], R[4 * k + 1], R[4 * k + 2], R[4 * k + 3]);
        }
        wave_lds_fence();
        const uint32_t a = (uint32_t)__builtin_amdgcn_readlane((int)maxabs, (int)first_lane);
        uint32_t best = 0xffffffffu, best_sign = 0;  // uniform: lowest element index of magnitude a, and its sign bit
#pragma unroll
        for (int j = 0; j < K; ++j) {
            const uint32_t e = lane * K + j;
            const uint32_t b = (I >= 64 || lane < 32) ? (uint32_t)tie_buf[e] : 0xffffu;
            const bool hit = (b & 0x7fffu) == a && (I >= 64 || lane < 32);
            const unsigned long long hits = __builtin_amdgcn_ballot_w64(hit);
            const unsigned long long negs = __builtin_amdgcn_ballot_w64(hit && (b >> 15) != 0u);
            if (hits != 0ull) {
                const uint32_t l0 = (uint32_t)__builtin_ctzll(hits);
                const uint32_t idx = l0 * K + j;
                if (idx < best) {
                    best = idx;
                    best_sign = (uint32_t)((negs >> l0) & 1ull);
                }
            }
        }
        if (mine) sign = best_sign;
        ties &= ~(((C::LPB == 64 ? 0ull : (1ull << C::LPB)) - 1ull) << first_lane);
    }
}

// ---------------------------------------------------------------------------------------------- OPQ (section 3.3)
// Outlier rule of eq. 9 with the corrected sample deviation of appendix E.1, in the square-root-free binary64 form
//   w^2 I (I-1) > T^2 V,   V = I sum w^2 - (sum w)^2 = fma(-S, S, I Q).
// Both sides are monotone in |w|, so per block there is one bfloat16 pattern theta with: outlier <=> |w| > theta.
// 0x7FFF means "no outliers".

// theta for a given right-hand side rhs = T^2 V > 0: from an approximate square root, settled with the exact
// binary64 test on its neighbours, so that (v v) I (I-1) > rhs holds exactly for the patterns above theta.
template <int I>
__device__ __forceinline__ bool opq_is_out(uint32_t b, double rhs) {
    constexpr double II1 = (double)I * (double)(I - 1);
    const double v = (double)bf16_bits_to_f32(b);
    return (v * v) * II1 > rhs;
}
template <int I, bool F32_ROOT = false>
__device__ __forceinline__ uint32_t opq_theta_of(double rhs) {
    constexpr double II1 = (double)I * (double)(I - 1);
    // the root only has to land within one bfloat16 pattern of tau = sqrt(rhs / (I (I - 1))): the exact tests below
    // settle the rest.  The binary64 root never under- or overflows; the binary32 one (an instruction instead of a
    // dozen) is for callers that keep rhs / (I (I - 1)) inside binary32's normal range.
    const float t = F32_ROOT ? __builtin_amdgcn_sqrtf((float)(rhs * (1.0 / II1))) : (float)__builtin_sqrt(rhs * (1.0 / II1));
    uint32_t b0 = __float_as_uint(t) >> 16;
    b0 = min(max(b0, 1u), 0x7F7Eu);
    uint32_t theta = b0 - 1;
    if (!opq_is_out<I>(b0, rhs)) theta = b0;
    if (!opq_is_out<I>(b0 + 1, rhs)) theta = b0 + 1;
    return theta;
}
// The plain evaluation: S and Q in binary64 (every term is exact).
template <int I>
__device__ __forceinline__ uint32_t opq_theta_exact(const uint32_t (&R)[SegCfg<I>::NR], double T2) {
    using C = SegCfg<I>;
    double S = 0.0, Q = 0.0;
#pragma unroll
    for (int e = 0; e < C::SEG; ++e) {
        double d = (double)seg_f32(R, e);
        S += d;
        Q = fma(d, d, Q);
    }
#pragma unroll
    for (int m = 1; m < C::LPB; m <<= 1) {
        S += __shfl_xor(S, m, 64);
        Q += __shfl_xor(Q, m, 64);
    }
    const double V = fma(-S, S, (double)I * Q);
    return V > 0.0 ? opq_theta_of<I>(T2 * V) : 0x7FFFu;
}
// The same theta at a quarter of the instructions.  S~ and Q~ come from packed binary32 dot products (one per two
// weights, no unpacking), four chains per lane.  Each chain of L = NR / 4 products with non-negative terms is off by
// at most DOT2_ROUNDINGS u (L + 1) times its sum (u = 2^-24); joining chains and lanes adds less than 6 u, so
//   |Q~ - Q| <= eps Q,   |S~ - S| <= eps A,   A = sum |w| <= sqrt(I Q),   eps = (DOT2_ROUNDINGS (L + 1) + 6) u,
// and V~ = I Q~ - S~^2 is within E = 3.05 eps I Q~ of V.  theta is monotone in V: if theta(V~ - E) also holds at
// V~ + E it is the exact one.  Otherwise (about one block in 500), or if Q~ is too small or too large for binary32
// products to be trusted, the wave takes the plain evaluation.
template <int I>
__device__ __forceinline__ uint32_t opq_theta(const uint32_t (&R)[SegCfg<I>::NR], double T2) {
    using C = SegCfg<I>;
    constexpr uint32_t ONES = 0x3F803F80u;  // (1.0, 1.0)
    constexpr double EPS = ((double)DOT2_ROUNDINGS * (C::NR / 4 + 1) + 6.0) * 0x1p-24;
    float q[4] = {0.0f, 0.0f, 0.0f, 0.0f}, s[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int d = 0; d < C::NR; ++d) {
        q[d & 3] = dot2_bf16(R[d], R[d], q[d & 3]);
        s[d & 3] = dot2_bf16(R[d], ONES, s[d & 3]);
    }
    float Qf = (q[0] + q[1]) + (q[2] + q[3]), Sf = (s[0] + s[1]) + (s[2] + s[3]);
#pragma unroll
    for (int m = 1; m < C::LPB; m <<= 1) {
        Qf += __shfl_xor(Qf, m, 64);
        Sf += __shfl_xor(Sf, m, 64);
    }
    const double IQ = (double)I * (double)Qf;
    const double V = fma(-(double)Sf, (double)Sf, IQ), E = (3.05 * EPS) * IQ;
    bool settled = false;
    uint32_t theta = 0x7FFFu;
    // (the bounds on T^2 (V - E) keep the argument of the binary32 root inside [2^-100, 2^120])
    const double rhs_lo = T2 * (V - E);
    if (Qf > 0x1p-80f && Qf < 0x1p100f && rhs_lo > 0x1p-100 * ((double)I * (double)(I - 1)) &&
        rhs_lo < 0x1p120 * ((double)I * (double)(I - 1))) {
        theta = opq_theta_of<I, true>(rhs_lo);
        settled = opq_is_out<I>(theta + 1, T2 * (V + E));
    }
    if (__builtin_amdgcn_ballot_w64(!settled) != 0) theta = opq_theta_exact<I>(R, T2);  // wave-uniform
    return theta;
}

// Replace the outliers of the segment by +0 (they then count as x = 0) and mark them: packed register d of the
// segment sets bit (d & 15) of map[d >> 4] for its low half (element 2 d) and bit 16 + (d & 15) for its high half
// (element 2 d + 1).
template <int I>
__device__ __forceinline__ void opq_zero_outliers(uint32_t (&R)[SegCfg<I>::NR], uint32_t theta, uint32_t (&map)[2]) {
    using C = SegCfg<I>;
    const uint32_t th2 = theta * 0x10001u;
    map[0] = map[1] = 0;
#pragma unroll
    for (int d = 0; d < C::NR; ++d) {
        uint32_t a = R[d] & 0x7fff7fffu;
        uint32_t mask = pk_sign_mask_i16(pk_sub_i16(th2, a));  // 0xFFFF in every half with |w| > theta
        R[d] &= ~mask;
        map[d >> 4] |= mask & (0x00010001u << (d & 15));
    }
}
__device__ __forceinline__ uint32_t opq_count(const uint32_t (&map)[2]) {
    return (uint32_t)__builtin_popcount(map[0]) + (uint32_t)__builtin_popcount(map[1]);
}
// Takes the lowest marked element out of the map and returns its index in the segment (map must not be empty).
__device__ __forceinline__ uint32_t opq_pop_lowest(uint32_t (&map)[2]) {
    const bool first = map[0] != 0u;
    const uint32_t m = first ? map[0] : map[1];
    const uint32_t lo = m & 0xffffu, hi = m >> 16;
    const uint32_t klo = lo ? (uint32_t)__builtin_ctz(lo) : 16u, khi = hi ? (uint32_t)__builtin_ctz(hi) : 16u;
    const bool take_lo = klo <= khi;  // element 2 k before element 2 k + 1
    const uint32_t k = take_lo ? klo : khi;
    const uint32_t cleared = m & ~((take_lo ? 1u : 0x10000u) << k);
    if (first) map[0] = cleared;
    else map[1] = cleared;
    return (first ? 0u : 32u) + 2u * k + (take_lo ? 0u : 1u);
}

// ================================================================================================ the pass
// One kernel streams over the weights and does the quantiser's work (codes, block constants, outlier list: sections
// 2.1, 3.1, 3.3), the Lloyd step's (per-region sums of section 3.2 eq. 6), or both on the same normalised weights.
//
// Loads.  Every lane loads its own segment straight from memory (16-byte loads at a stride of one segment; the lines
// a wave touches are consumed completely by its next loads, so the caches see every byte once) and requests the next
// tile's pieces as it uses this one up: a lane never holds two whole tiles.
//
// Outlier staging of the quantiser: every wave appends the outliers of its (contiguous, ascending) tile range to a
// region of its own, in ascending flat index, and reports how many it found.  A later pass turns the per-wave counts
// into offsets and copies the regions into the caller's list.  A wave that finds more than its region holds keeps
// counting (the count stays exact); the scan pass notices it and the host repeats the call on the general path.
// The outliers' original values (the registers hold zeros in their place by then): the quantiser on its own reads
// them back from the tile it has staged in LDS anyway.  The one-pass variant has no such copy, and making one (the
// tile parked on the Lloyd columns, which then have to be cleared again) cost 14 % of the kernel: there every lane
// writes (lane, element) of its outliers to a short wave-private list in LDS, one lane per entry reads the value
// again from memory (the line was fetched a moment ago: a cache hit) and keeps it in a register, and the entries are
// stored - neighbouring lanes to neighbouring places - at the end of the tile, when the value has long arrived.
//
// Lloyd sums.  Per-level sums of the current block live in lane-private LDS columns acc[level][lane]
// (conflict-free).  One 64-bit LDS add per weight carries both the count and the sum of x of its level: the increment
// is the bit pattern of the binary64 number 2^-1008 + (x + 2) 2^-1020, i.e. exponent field 15 and mantissa
// (x + 2) 2^40 rounded to an integer.  Adding up to 256 of these as integers gives 15 K 2^52 + sum (x + 2) 2^40 with
// the second term below 2^52, so count K and sum separate again exactly.  (x + 2, not x + 1: a block constant below
// binary16's normal range is stored with fewer bits than it has, and the weights of such a block normalise to up to
// 1.5 in magnitude; the addend must stay positive, or the increment leaves its binade and the count loses a unit.)
// Once per tile the columns are folded, with the block weights g, into binary64 registers:
// A += g sum(x + 2) 2^40,  den15 += g 15 K,  cnt15 += 15 K.
// The fold is shared inside every quad of lanes: lane 4q + p takes levels 4p .. 4p+3 of the four blocks of its quad
// (the weights g of the other three arrive by quad permutes), so a lane carries 4 and not 16 sets of accumulators -
// the registers this frees are what lets four waves share a SIMD.  At any step the 64 lanes read 64 different
// columns of one level each: conflict-free again.  The two increment constants are passed as kernel arguments (not
// literals) so that the increment is one three-operand fused multiply-add whose addend register pair is not
// overwritten.
struct OutlierStage {
    int64_t* idx;          // [n_waves * region_cap]
    uint16_t* val;         // [n_waves * region_cap]
    uint32_t* wave_count;  // [n_waves]
    uint32_t region_cap;
};
constexpr double LLOYD_INC_MUL = 0x1p-1020;
constexpr double LLOYD_INC_ADD = 0x1p-1008 + 0x1p-1019;

// Waves per SIMD a variant of the pass is compiled for (the launch bound holds its registers to 512 / that many).
__host__ __device__ constexpr int pass_waves_per_simd(bool opq, bool quant, bool lloyd) {
    return (quant && lloyd) ? 3 : lloyd ? (opq ? 3 : 4) : 4;
}

// Where lane `lane` finds its segment of tile `t`.  A lane whose segment lies past the end of the tensor (ragged last
// tile) is pointed at the tensor's last segment instead: it loads valid memory and contributes nothing.
template <int I>
__device__ __forceinline__ const uint4* own_segment(const uint4* __restrict__ w, uint64_t t, uint64_t n_seg,
                                                    uint32_t lane) {
    const uint64_t seg = t * 64 + lane;
    return w + (seg < n_seg ? seg : n_seg - 1) * SegCfg<I>::NV;
}
// The value of lane (l ^ C) of the same quad, C = 1, 2, 3 (all lanes active).
template <int C>
__device__ __forceinline__ float quad_xor(float v) {
    constexpr int ctrl = C == 1 ? 0xB1 : C == 2 ? 0x4E : 0x1B;  // quad_perm [1,0,3,2] / [2,3,0,1] / [3,2,1,0]
    return __uint_as_float((uint32_t)__builtin_amdgcn_update_dpp(0, (int)__float_as_uint(v), ctrl, 0xf, 0xf, true));
}
// STAGED (the quantiser on its own, which is bound by memory traffic and not by instruction issue): the wave loads
// whole tiles with fully coalesced 16-byte loads, parks them in a padded LDS buffer and reads them back transposed;
// the staged tile also serves the outlier values.
__host__ __device__ constexpr bool pass_staged(bool quant, bool lloyd) { return quant && !lloyd; }

template <int I, bool FAST, bool OPQ, bool QUANT, bool LLOYD>
__global__ __launch_bounds__(256, pass_waves_per_simd(OPQ, QUANT, LLOYD)) void seg_pass_kernel(
    const uint4* __restrict__ w, uint64_t n_seg, CodebookArgs cb, BinTable bt, int signed_norm, int weight_by_max2,
    double T2, double inc_mul, double inc_add, uint32_t* __restrict__ codes, uint16_t* __restrict__ scales,
    OutlierStage os, double* __restrict__ partials) {
    using C = SegCfg<I>;
    static_assert(QUANT || LLOYD, "a pass does something");
    constexpr bool STAGED = pass_staged(QUANT, LLOYD);
    constexpr bool EXTRACT = QUANT && OPQ;     // outliers go to the wave's staging region
    constexpr bool RELOAD = EXTRACT && !STAGED;  // no copy of the tile in LDS: outlier values are read again from memory
    constexpr bool COLS = LLOYD;                 // 8 KB per wave: the Lloyd columns
    struct Shared {  // one object, so that the table sits at LDS offset 0 (reachable by an immediate offset)
        uint2 tab[BIN_TABLE_ENTRIES];
        unsigned long long cols[COLS ? WAVES_PER_WG * 16 * 64 : 1];
        char stage[STAGED ? WAVES_PER_WG * C::STAGE_BYTES : 16];
        uint16_t tie[WAVES_PER_WG * TIE_BUF_HALFWORDS] __attribute__((aligned(16)));
    };
    __shared__ __attribute__((aligned(16))) Shared sh;
    const uint32_t tid = threadIdx.x, lane = tid & 63;
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(tid >> 6));  // scalar: tile ranges on the SALU
    uint16_t* tie_buf = sh.tie + wave * TIE_BUF_HALFWORDS;
    bin_table_fill(sh.tab, bt, tid, blockDim.x);
    const uint2* tab = sh.tab;
    const uint32_t lane_off = bin_lane_offset(lane);
    unsigned long long* acc = sh.cols + (COLS ? wave * 16 * 64 : 0);
    if (LLOYD) {
#pragma unroll
        for (int l = 0; l < 16; ++l) acc[l * 64 + lane] = 0ull;
    }
    __syncthreads();
    const uint64_t n_tiles = (n_seg + 63) / 64;
    const uint64_t n_waves = (uint64_t)gridDim.x * WAVES_PER_WG;
    const uint64_t gw = (uint64_t)blockIdx.x * WAVES_PER_WG + wave;
    // Which tiles the wave takes.  With an outlier list to write, a contiguous range (the wave appends to its staging
    // region in ascending order of the flat index).  Otherwise the tiles are dealt out in turn, wave g taking tiles
    // g, g + n_waves, ...: at any moment the chip then works on one compact stretch of the tensor instead of
    // thousands of far-apart ones, which the memory system takes 4 to 7 % faster where codes are written; the
    // assignment is still a fixed function of the launch, so the sums stay bit-reproducible.
    constexpr bool DEAL = !(QUANT && OPQ);
    const uint64_t t0 = DEAL ? gw : n_tiles * gw / n_waves, t1 = DEAL ? n_tiles : n_tiles * (gw + 1) / n_waves;
    const uint64_t t_step = DEAL ? n_waves : 1;
    // fold: levels 4 p + k (k = 0 .. 3) of the blocks of lanes lane ^ c (c = 0 .. 3)
    const uint32_t p4 = (lane & 3u) * 4u;
    unsigned long long* fold_col[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) fold_col[c] = acc + p4 * 64 + (lane ^ (uint32_t)c);
    char* stage = sh.stage + (STAGED ? wave * C::STAGE_BYTES : 0);
    const uint64_t n_vec = n_seg * C::NV;

    double A[4], den15[4], sxx_g = 0.0;
    uint32_t cnt15[4], kout = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        A[k] = 0.0;
        den15[k] = 0.0;
        cnt15[k] = 0;
    }
    uint32_t wcount = 0;  // outliers this wave has found so far (wave-uniform)
    // R holds the lane's segment of the current tile; Rn takes over the registers R gives up.
    uint32_t R[C::NR], Rn[C::NR];
    uint4 G[C::NV];
    if constexpr (STAGED) {
        if (t0 < t1) tile_issue_loads<I>(w, t0 * 64 * C::NV, n_vec, lane, G);
    } else if (t0 < t1) {
        const uint4* p = own_segment<I>(w, t0, n_seg, lane);
#pragma unroll
        for (int k = 0; k < C::NV; ++k) {
            const uint4 q = p[k];
            R[4 * k] = q.x;
            R[4 * k + 1] = q.y;
            R[4 * k + 2] = q.z;
            R[4 * k + 3] = q.w;
        }
    }
    for (uint64_t t = t0; t < t1; t += t_step) {
        // (after the wave's last tile this requests that tile once more: cached, and never used)
        const uint4* pn = own_segment<I>(w, t + t_step < t1 ? t + t_step : t, n_seg, lane);
        if constexpr (STAGED) {
            wave_lds_fence();
            tile_stage<I>(stage, lane, G);
            if (t + t_step < t1) tile_issue_loads<I>(w, (t + t_step) * 64 * C::NV, n_vec, lane, G);
            wave_lds_fence();
            tile_fetch<I>(stage, lane, R);
        }
        const uint64_t seg = t * 64 + lane;
        const bool active = seg < n_seg;
        uint32_t k_out = 0, omap[2] = {0, 0};
        if (OPQ) {
            opq_zero_outliers<I>(R, opq_theta<I>(R, T2), omap);
            k_out = active ? opq_count(omap) : 0u;
        }
        // entries whose value is on its way from memory: lane l < pend_n stores entry pend_first + l at the tile's end
        uint32_t pend_n = 0, pend_first = 0, pend_entry = 0, pend_raw = 0;
        if (EXTRACT) {
            // inclusive prefix of the per-lane counts = order of the flat indices
            const uint32_t incl = wave_inclusive_scan_u32(k_out);
            const uint32_t total = (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
            wave_lds_fence();
            if (total != 0) {  // wave-uniform
                const uint64_t region = gw * (uint64_t)os.region_cap;
                if (!active) omap[0] = omap[1] = 0;
                if (RELOAD && total <= 64u) {  // wave-uniform: the ordinary case
                    // (lane, element) of every outlier of the tile, in order, in the wave's tie buffer (free here)
                    uint32_t slot = incl - k_out;
                    while ((omap[0] | omap[1]) != 0u) tie_buf[slot++] = (uint16_t)(opq_pop_lowest(omap) | (lane << 6));
                    wave_lds_fence();
                    if (lane < total) {
                        pend_entry = tie_buf[lane];
                        const uint64_t flat = (t * 64 + (pend_entry >> 6)) * C::SEG + (pend_entry & 63u);
                        pend_raw = reinterpret_cast<const uint16_t*>(w)[flat];
                    }
                    pend_n = total;
                    pend_first = wcount;
                    wave_lds_fence();  // the buffer is read: the search for the block constants may use it again
                } else {
                    uint32_t pos = wcount + incl - k_out;
                    while ((omap[0] | omap[1]) != 0u) {  // lanes run dry at different times
                        const uint32_t e = opq_pop_lowest(omap);
                        const uint32_t b = STAGED ? *reinterpret_cast<const uint16_t*>(stage + lane * C::PITCH + 2 * e)
                                                  : reinterpret_cast<const uint16_t*>(w)[seg * C::SEG + e];
                        if (pos < os.region_cap) {
                            os.idx[region + pos] = (int64_t)(seg * C::SEG + e);
                            os.val[region + pos] = (uint16_t)f32_to_f16_bits(bf16_bits_to_f32(b));
                        }
                        ++pos;
                    }
                }
                wcount += total;
            }
        }
        uint32_t maxabs, sign;
        block_constant<I>(R, lane, signed_norm != 0, maxabs, sign, tie_buf);
        const float m = bf16_bits_to_f32(maxabs | (sign << 15));
        const uint32_t s16 = f32_to_f16_bits(m);
        const float m_eff = f16_bits_to_f32(s16);
        // the square of a binary16 number has 22 significant bits and an exponent in [-48, 32]: exact in binary32
        const float g = weight_by_max2 ? m_eff * m_eff : 1.0f;
        double sxx = 0.0;
        uint32_t out[QUANT ? C::SEG / 8 : 1];
        const bool fast = FAST && __builtin_amdgcn_ballot_w64(!maxabs_is_ordinary(maxabs)) == 0;
        // (lanes past the end of the tensor work on a copy of its last segment; what they produce is dropped below)
        if (fast) {
            const BlockDiv dv = make_block_div(m_eff);
#pragma unroll
            for (int b0 = 0; b0 < C::SEG; b0 += 8) {
                float x[8];
                uint2 en[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {  // table reads of a whole batch in flight ...
                    x[e] = div_fast(seg_f32(R, b0 + e), dv);
                    en[e] = bin_lookup(tab, x[e], lane_off);
                }
                if (!STAGED) {  // these four registers of R are free now: the next tile's piece moves in
                    const uint4 q = pn[b0 / 8];
                    Rn[b0 / 2] = q.x;
                    Rn[b0 / 2 + 1] = q.y;
                    Rn[b0 / 2 + 2] = q.z;
                    Rn[b0 / 2 + 3] = q.w;
                }
                uint32_t packed = 0;
#pragma unroll
                for (int e = 7; e >= 0; --e) {  // ... before the first LDS add of the batch
                    const uint32_t code = en[e].y + (x[e] > __uint_as_float(en[e].x) ? 1u : 0u);
                    if (QUANT) packed = (packed << 4) + code;
                    if (LLOYD) {
                        const double xd = (double)x[e];
                        const double inc = fma(xd, inc_mul, inc_add);
                        atomicAdd(&acc[code * 64 + lane], (unsigned long long)__double_as_longlong(inc));
                        sxx = fma(xd, xd, sxx);
                    }
                }
                if (QUANT) out[b0 / 8] = packed;
                __builtin_amdgcn_sched_barrier(0);  // batches stay apart: mixing them costs more registers than it gains
            }
        } else {
#pragma unroll
            for (int j = 0; j < C::SEG / 8; ++j) {
                uint32_t packed = 0;
#pragma unroll
                for (int e = 7; e >= 0; --e) {
                    const float f = seg_f32(R, 8 * j + e);
                    const float x = (m_eff == 0.0f) ? 0.0f : f / m_eff;
                    const uint32_t code = (uint32_t)assign_code_generic(x, cb);
                    if (QUANT) packed = (packed << 4) + code;
                    if (LLOYD) {
                        const double xd = (double)x;
                        const double inc = fma(xd, inc_mul, inc_add);
                        atomicAdd(&acc[code * 64 + lane], (unsigned long long)__double_as_longlong(inc));
                        sxx = fma(xd, xd, sxx);
                    }
                }
                if (QUANT) out[j] = packed;
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int k = 0; k < (STAGED ? 0 : C::NV); ++k) {
                const uint4 q = pn[k];
                Rn[4 * k] = q.x;
                Rn[4 * k + 1] = q.y;
                Rn[4 * k + 2] = q.z;
                Rn[4 * k + 3] = q.w;
            }
        }
        if (QUANT && active) {
            uint4* dst = reinterpret_cast<uint4*>(codes + seg * (C::SEG / 8));
#pragma unroll
            for (int q = 0; q < C::SEG / 32; ++q)
                store_stream(&dst[q], make_uint4(out[4 * q], out[4 * q + 1], out[4 * q + 2], out[4 * q + 3]));
            if ((lane & (C::LPB - 1)) == 0) scales[seg / C::LPB] = (uint16_t)s16;
        }
        if (RELOAD && pend_n != 0u) {  // wave-uniform
            const uint32_t pos = pend_first + lane;
            if (lane < pend_n && pos < os.region_cap) {
                const uint64_t at = gw * (uint64_t)os.region_cap + pos;
                os.idx[at] = (int64_t)((t * 64 + (pend_entry >> 6)) * C::SEG + (pend_entry & 63u));
                os.val[at] = (uint16_t)f32_to_f16_bits(bf16_bits_to_f32(pend_raw));
            }
        }
        if (LLOYD) {
            const double gd = active ? (double)g : 0.0;
            sxx_g = fma(gd, sxx, sxx_g);
            if (OPQ) {
                // The zeroed outliers went through the loop as x = 0 and sit in this lane's column of the zero level:
                // take out again exactly what they put there, k_out times the operand of x = 0, as integers - the
                // column then holds the block's other weights only, count and sum, and nothing has to be corrected
                // later in floating point (where a region whose other weights all weigh nothing kept a residue).
                if (k_out != 0u)
                    atomicAdd(&acc[bt.code_of_zero * 64 + lane],
                              0ull - (unsigned long long)k_out * (unsigned long long)__double_as_longlong(inc_add));
                kout += k_out;
            }
            if (t * 64 + 64 > n_seg) {  // wave-uniform: the ragged last tile of the tensor
                wave_lds_fence();
                if (!active) {
#pragma unroll
                    for (int l = 0; l < 16; ++l) acc[l * 64 + lane] = 0ull;
                }
            }
            // fold (all lanes)
            wave_lds_fence();
            const float gq[4] = {g, quad_xor<1>(g), quad_xor<2>(g), quad_xor<3>(g)};
            unsigned long long col[16];
#pragma unroll
            for (int c = 0; c < 4; ++c)
#pragma unroll
                for (int k = 0; k < 4; ++k) col[4 * c + k] = atomicExch(fold_col[c] + k * 64, 0ull);  // read and clear
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const double gc = (double)gq[c];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const unsigned long long v = col[4 * c + k];
                    const uint32_t hi = (uint32_t)(v >> 32), lo = (uint32_t)v;
                    const uint32_t k15 = hi >> 20;
                    // 2^52 + sum: the column's mantissa under the exponent of 2^52 (one bit-field insert)
                    uint32_t dhi;
                    asm("v_bfi_b32 %0, %1, %2, %3" : "=v"(dhi) : "v"(0xFFFFFu), "v"(hi), "v"(0x43300000u));
                    const double D = __hiloint2double((int)dhi, (int)lo) - 0x1p52;  // sum (x+2) 2^40
                    A[k] = fma(gc, D, A[k]);
                    den15[k] = fma(gc, (double)k15, den15[k]);
                    cnt15[k] += k15;
                }
            }
            wave_lds_fence();
        }
        if (!STAGED) {
#pragma unroll
            for (int d = 0; d < C::NR; ++d) R[d] = Rn[d];
        }
    }
    if (EXTRACT && lane == 0) os.wave_count[gw] = wcount;
    if (!LLOYD) return;
    // Lanes with the same p hold partial sums of the same four levels: fixed-order butterfly over the other lane bits,
    // then the four waves of the workgroup in wave order.
    __shared__ double wave_totals[LLOYD ? WAVES_PER_WG * LLOYD_PART : 1];
    double* wtot = wave_totals + wave * LLOYD_PART;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        double a = A[k] * 0x1p-40, d = den15[k];
        unsigned long long c = cnt15[k];
#pragma unroll
        for (int mk = 32; mk >= 4; mk >>= 1) {
            a += __shfl_xor(a, mk, 64);
            d += __shfl_xor(d, mk, 64);
            c += (unsigned long long)__shfl_xor((long long)c, mk, 64);
        }
        if (lane < 4) {
            wtot[p4 + k] = a;
            wtot[16 + p4 + k] = d;
            wtot[32 + p4 + k] = __longlong_as_double((long long)c);
        }
    }
    {
        double a = sxx_g;
        unsigned long long kc = kout;
#pragma unroll
        for (int mk = 32; mk >= 1; mk >>= 1) {
            a += __shfl_xor(a, mk, 64);
            kc += (unsigned long long)__shfl_xor((long long)kc, mk, 64);
        }
        if (lane == 0) {
            wtot[48] = a;
            wtot[49] = 0.0;                                 // (not used)
            wtot[50] = __longlong_as_double((long long)kc); // outlier count
        }
    }
    __syncthreads();
    if (tid < 51) {
        const double* all = wave_totals;
        const bool is_int = (tid >= 32 && tid < 48) || tid == 50;
        double sd = 0.0;
        unsigned long long si = 0;
        for (int k = 0; k < WAVES_PER_WG; ++k) {
            if (is_int) si += (unsigned long long)__double_as_longlong(all[k * LLOYD_PART + tid]);
            else sd += all[k * LLOYD_PART + tid];
        }
        partials[(uint64_t)blockIdx.x * LLOYD_PART + tid] = is_int ? __longlong_as_double((long long)si) : sd;
    }
}

// One workgroup per staging region: it adds up the outlier counts of the regions before its own (that sum is where
// its entries start in the caller's ascending list) and copies its region there.  The workgroup of the last region
// has then seen every count: it publishes *total_out = number of outliers, with bit 63 set if some wave overflowed its
// staging region.
__global__ __launch_bounds__(256) void seg_outlier_gather_kernel(OutlierStage os, uint32_t n_waves,
                                                                  int64_t* __restrict__ out_idx,
                                                                  uint16_t* __restrict__ out_val, uint64_t capacity,
                                                                  uint64_t* __restrict__ total_out) {
    const uint32_t r = blockIdx.x, tid = threadIdx.x;
    uint64_t before = 0;
    uint32_t over = 0;
    for (uint32_t i0 = 0; i0 < r; i0 += 256 * 4) {  // four independent loads in flight per lane
        uint32_t ci[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const uint32_t i = i0 + 256 * t + tid;
            ci[t] = i < r ? os.wave_count[i] : 0u;
        }
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            before += ci[t];
            over |= (ci[t] > os.region_cap) ? 1u : 0u;
        }
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        before += (uint64_t)__shfl_xor((long long)before, d, 64);
        over |= (uint32_t)__shfl_xor((int)over, d, 64);
    }
    __shared__ uint64_t before_w[4];
    __shared__ uint32_t over_w[4];
    if ((tid & 63u) == 0) {
        before_w[tid >> 6] = before;
        over_w[tid >> 6] = over;
    }
    __syncthreads();
    before = (before_w[0] + before_w[1]) + (before_w[2] + before_w[3]);  // integers: any order
    over = over_w[0] | over_w[1] | over_w[2] | over_w[3];
    const uint32_t own = os.wave_count[r];
    if (r == n_waves - 1 && tid == 0)  // one 64-bit store at system scope: a host that watches the word sees it whole
        __hip_atomic_store(reinterpret_cast<unsigned long long*>(total_out),
                           (unsigned long long)((before + own) |
                                                ((uint64_t)((over | (own > os.region_cap ? 1u : 0u)) != 0) << 63)),
                           __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
    const uint32_t c = own > os.region_cap ? os.region_cap : own;
    const uint64_t src = (uint64_t)r * os.region_cap;
    for (uint32_t j = tid; j < c; j += 256) {
        if (before + j < capacity) {
            out_idx[before + j] = os.idx[src + j];
            out_val[before + j] = os.val[src + j];
        }
    }
}

// Reduce the per-wave partials in a fixed order and turn them into the statistics of the C ABI:
//   num = A - 2 den,  sse = sum g x^2 - 2 sum_l c_l num_l + sum_l c_l^2 den_l   (the three sums of the expanded square).
// `out` has the memory layout of bof4_lloyd_stats: [0..15] num, [16..31] den, [32..47] cnt (integers), [48] sse,
// [49] n_used, [50] n_outliers (integers); it may point into the workspace or at device-visible host memory.
__global__ __launch_bounds__(1024) void seg_lloyd_final_kernel(const double* __restrict__ partials, uint32_t n_part,
                                                                CodebookArgs cb, uint32_t code_of_zero,
                                                                double* __restrict__ out) {
    __shared__ double red[16][LLOYD_PART];
    __shared__ double tot[LLOYD_PART];
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    // lane = quantity, wave w takes partials w, w+16, ... in order (each read is one contiguous record); eight
    // independent loads are in flight before they are added, in index order
    if (lane < 51) {
        const bool is_int = (lane >= 32 && lane < 48) || lane == 50;
        double s = 0.0;
        unsigned long long si = 0;
        for (uint32_t p0 = wave; p0 < n_part; p0 += 16 * 8) {
            double v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                uint32_t p = p0 + 16 * u;
                v[u] = p < n_part ? partials[(uint64_t)p * LLOYD_PART + lane] : 0.0;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                if (is_int) si += (unsigned long long)__double_as_longlong(v[u]);
                else s += v[u];
            }
        }
        red[wave][lane] = is_int ? __longlong_as_double((long long)si) : s;
    }
    __syncthreads();
    if (threadIdx.x < 51) {
        const uint32_t q = threadIdx.x;
        const bool is_int = (q >= 32 && q < 48) || q == 50;
        double s = 0.0;
        unsigned long long si = 0;
        for (int k = 0; k < 16; ++k) {
            if (is_int) si += (unsigned long long)__double_as_longlong(red[k][q]);
            else s += red[k][q];
        }
        tot[q] = is_int ? __longlong_as_double((long long)si) : s;
    }
    __syncthreads();
    __shared__ double sse_part[16];
    __shared__ unsigned long long cnt_part[16];
    if (threadIdx.x < 16) {
        const uint32_t l = threadIdx.x;
        const unsigned long long kout = (unsigned long long)__double_as_longlong(tot[50]);
        double den = tot[16 + l] * (1.0 / 15.0);
        double a = tot[l];
        // 15 K is a multiple of 15 below 2^53: the binary64 quotient is the exact integer
        unsigned long long c = (unsigned long long)((double)(unsigned long long)__double_as_longlong(tot[32 + l]) / 15.0);
        double num = a - 2.0 * den;
        if (c == 0ull) den = num = 0.0;  // an empty region has no mass (a - 2 den may leave rounding residue)
        out[l] = num;
        out[16 + l] = den;
        out[32 + l] = __longlong_as_double((long long)c);
        sse_part[l] = cb.cb64[l] * (cb.cb64[l] * den - 2.0 * num);
        cnt_part[l] = c;
        if (l == 0) out[50] = __longlong_as_double((long long)kout);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        double sse = tot[48];
        unsigned long long used = 0;
        for (int l = 0; l < 16; ++l) {
            sse += sse_part[l];
            used += cnt_part[l];
        }
        out[48] = sse;
        // written last, after everything above has reached system memory: a host that watches this word may read
        // the record as soon as it changes
        __hip_atomic_store(reinterpret_cast<unsigned long long*>(&out[49]), used, __ATOMIC_RELEASE,
                           __HIP_MEMORY_SCOPE_SYSTEM);
    }
}

}  // namespace bof4
