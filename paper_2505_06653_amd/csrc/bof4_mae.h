// bof4_mae.h - Lloyd step under the MAE criterion (section 3.2 eq. 7-8, appendix B.4): per region the weighted
// median of the normalised weights, weighted by the absolute block maximum - or, on request, the plain median of
// appendix D (every weight one unit).
//
// A weighted median over 10^8 samples is found without sorting, by a radix search on an order-preserving integer
// key of x.  Region l can only hold keys between klo[l] (its lower threshold) and its upper threshold, so the search
// runs on sub = key - klo[l], which has bits[l] <= 31 significant bits; every pass over the weights fixes the next 8
// of them: a histogram of the weight that falls on each value of those 8 bits (among the elements that agree with
// the bits fixed so far), then the smallest value d for which twice the weight up to and including d reaches the
// region's total.  Three passes settle an ordinary region, four the one that contains zero (its keys span both
// signs).  Weights are exact integers, |block constant| * 2^24 (the constant is a binary16 number), added in 64
// bits; additions of integers commute, so the result does not depend on the order of the atomics.
// The second pass also writes every element that agrees with the first digit of its region (about one in 200) to a
// list - key, region and block constant in 8 bytes - and the passes after it read that list instead of the weights.
// Every wave appends to a region of its own; if one of them runs full (a tensor of equal numbers), the later passes
// scan the weights as before.
// Large tensors get by with ONE pass over all the weights: a first-digit histogram over one tile in 16 (picked by a
// hash of the tile number) says where every region's median will be to within a few digits; the full first pass then
// writes the elements whose first digit lies in that window to the list while it fills the exact histogram.  If the
// exact first digit of every region falls inside its window (it does unless the sampled tiles differ from the rest),
// all later passes read the list; if not, they scan the weights, as they do when the list runs full.
//
// What is computed is "the smallest x_k with 2 * sum_{x_j <= x_k} a_j >= sum_j a_j" - the lower weighted median,
// which minimises sum a_j |x_j - c|.  (The closing formula of appendix B.4 names the element before it; its own
// derivation puts the minimum where this rule does.)
#pragma once
#include "bof4_segment.h"

namespace bof4 {

// Search state of one region, in the workspace.
struct MaeLevelState {
    uint32_t klo;     // key of the region's lower bound
    uint32_t hi;      // bits [hi, 32) of sub are fixed to `prefix`; 0 = finished
    uint32_t prefix;  // their value
    uint32_t pad;     // 1: the caller does not want this region's median (no search after the first pass)
    unsigned long long base;   // weight of the elements whose sub lies below prefix << hi
    unsigned long long total;  // weight of the whole region
    uint32_t win_lo;   // first digits win_lo .. win_lo + win_len - 1: what a capturing first pass writes to the list
    uint32_t win_len;
};
// Per-region constants from the host: key range of the region.
struct MaeLevelConst {
    uint32_t klo[16];
    uint32_t bits[16];  // significant bits of (key of upper bound - klo)
};
constexpr int MAE_REC = 51;  // doubles of the result record (layout of bof4_mae_stats)

// Order-preserving map from binary32 to uint32 (negative numbers reversed below the positive ones).
__device__ __forceinline__ uint32_t order_key(float x) {
    const uint32_t b = __float_as_uint(x);
    return b ^ ((uint32_t)((int)b >> 31) | 0x80000000u);
}
__device__ __forceinline__ float key_to_float(uint32_t k) {
    return __uint_as_float((k & 0x80000000u) ? (k ^ 0x80000000u) : ~k);
}

// Sets up the search (state from the host's constants) and clears the accumulators.
__global__ __launch_bounds__(256) void mae_init_kernel(MaeLevelConst lc, MaeLevelState* __restrict__ state,
                                                       unsigned long long* __restrict__ hist) {
    const uint32_t t = blockIdx.x * 256 + threadIdx.x;
    if (t < 16 * 256) hist[t] = 0ull;
    if (t < 16) {
        MaeLevelState s;
        s.klo = lc.klo[t];
        s.hi = lc.bits[t];
        s.prefix = 0;
        s.pad = 0;
        s.base = 0ull;
        s.total = 0ull;
        s.win_lo = 0;
        s.win_len = 0;
        state[t] = s;
    }
}

// Which tiles the sampling pass looks at: one in (sample_mask + 1), spread by a multiplicative hash so that the choice
// does not follow the rows and columns of the matrices behind the tensor.
__host__ __device__ inline bool mae_tile_sampled(uint64_t t, uint32_t sample_mask) {
    return ((((uint32_t)t * 0x9E3779B1u) >> 16) & sample_mask) == 0u;
}

// One pass over the weights.  FIRST also counts the regions' elements and accumulates the error sum
// sum |block constant| |x - level| at the current codebook; with CAPTURE it writes the elements whose first digit lies
// in the region's window to the list.  sample_mask != 0: only the sampled tiles.
template <int I, bool FAST, bool OPQ, bool FIRST, bool CAPTURE = false>
__global__ __launch_bounds__(256, 2) void mae_pass_kernel(const uint4* __restrict__ w, uint64_t n_seg, CodebookArgs cb,
                                                           BinTable bt, int signed_norm, double T2,
                                                           const MaeLevelState* __restrict__ state,
                                                           unsigned long long* __restrict__ hist_g,
                                                           unsigned long long* __restrict__ cnt_part,
                                                           double* __restrict__ sae_part,
                                                           unsigned long long* __restrict__ cand,
                                                           uint32_t* __restrict__ cand_count, uint32_t cand_cap,
                                                           const uint32_t* __restrict__ gate, int unweighted,
                                                           uint32_t sample_mask) {
    using C = SegCfg<I>;
    static_assert(FIRST || !CAPTURE, "only the first pass captures by window");
    // `gate`: this launch only matters if the word it points to is set (the scan that stands in for a list that ran
    // full).  `cand`: append the elements that still count to this wave's stretch of the list.
    if (gate != nullptr && *gate == 0u) return;
    struct Shared {  // one object, so that the table sits at LDS offset 0 (reachable by an immediate offset)
        uint2 tab[BIN_TABLE_ENTRIES];
        uint4 info[16];    // per region: klo, (lo | hi << 8 | digit mask << 16), then prefix and active flag; in
                           // the first pass (no prefix yet, every region active, its key range has exactly hi bits):
                           // klo, (lo | window start << 8 | window length << 16), the region's level as binary64
        unsigned long long hist[16 * 256];
        uint32_t cntcol[WAVES_PER_WG * 8 * 64];  // per lane, two 16-bit counters per word: regions 2p and 2p + 1
        char stage[WAVES_PER_WG * C::STAGE_BYTES];
        uint16_t tie[WAVES_PER_WG * TIE_BUF_HALFWORDS] __attribute__((aligned(16)));
    };
    __shared__ __attribute__((aligned(16))) Shared sh;
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    bin_table_fill(sh.tab, bt, tid, blockDim.x);
    if (tid < 16) {
        const MaeLevelState s = state[tid];
        const uint32_t hi = s.hi, lo = hi > 8 ? hi - 8 : 0;
        const uint32_t packed = lo | (hi << 8) | (((1u << (hi - lo)) - 1u) << 16);
        if (FIRST) {
            const unsigned long long lv = (unsigned long long)__double_as_longlong(cb.cb64[tid]);
            sh.info[tid] = make_uint4(s.klo, lo | (s.win_lo << 8) | (s.win_len << 16), (uint32_t)lv, (uint32_t)(lv >> 32));
        } else {
            sh.info[tid] = make_uint4(s.klo, packed, s.prefix, (hi != 0 && s.total != 0ull && s.pad == 0u) ? 1u : 0u);
        }
    }
    for (uint32_t i = tid; i < 16 * 256; i += 256) sh.hist[i] = 0ull;
    uint32_t* cntcol = sh.cntcol + wave * 8 * 64;
    if (FIRST) {
#pragma unroll
        for (int p = 0; p < 8; ++p) cntcol[p * 64 + lane] = 0u;
    }
    __syncthreads();
    const uint2* tab = sh.tab;
    const uint32_t lane_off = bin_lane_offset(threadIdx.x & 63u);
    char* stage = sh.stage + wave * C::STAGE_BYTES;
    uint16_t* tie_buf = sh.tie + wave * TIE_BUF_HALFWORDS;
    const uint64_t n_vec = n_seg * C::NV;
    const uint64_t n_tiles = (n_seg + 63) / 64;
    const uint64_t n_waves = (uint64_t)gridDim.x * WAVES_PER_WG;
    const uint64_t gw = (uint64_t)blockIdx.x * WAVES_PER_WG + wave;
    const uint64_t t0 = n_tiles * gw / n_waves, t1 = n_tiles * (gw + 1) / n_waves;

    // outliers were zeroed: they ran through the loop as x = +0 of the zero region and are taken out again
    const uint32_t cz = bt.code_of_zero;
    const uint32_t key0 = order_key(0.0f);
    double sae = 0.0, w_est = 0.0;
    uint32_t kout = 0, tiles_since_flush = 0;
    uint32_t wave_cand = 0;  // entries this wave has appended to the list (wave-uniform; may pass the capacity)
    uint2* my_cand = reinterpret_cast<uint2*>(cand) + gw * cand_cap;  // this wave's stretch of the list
    // The 16-bit lane counters are added up over the wave before they can overflow; lane l < 16 keeps the wave's count
    // of region l.  (Every wave adding its counts to 17 shared words at the end of the kernel cost more than the pass.)
    unsigned long long wave_cnt = 0ull;
    auto flush_counts = [&]() {
#pragma unroll
        for (int p = 0; p < 8; ++p) {
            const uint32_t v = cntcol[p * 64 + lane];
            cntcol[p * 64 + lane] = 0u;
            uint32_t c0 = v & 0xffffu, c1 = v >> 16;  // at most 65535 each: the wave's sum fits 32 bits
#pragma unroll
            for (int mk = 32; mk >= 1; mk >>= 1) {
                c0 += (uint32_t)__shfl_xor((int)c0, mk, 64);
                c1 += (uint32_t)__shfl_xor((int)c1, mk, 64);
            }
            if (lane == 2u * p) wave_cnt += c0;
            if (lane == 2u * p + 1u) wave_cnt += c1;
        }
    };
    uint4 G[C::NV];
    uint32_t R[C::NR];
    // the wave's tiles in turn - all of them, or those the sampling picks (wave-uniform)
    auto next_tile = [&](uint64_t t) {
        while (sample_mask != 0u && t < t1 && !mae_tile_sampled(t, sample_mask)) ++t;
        return t;
    };
    uint64_t t_first = next_tile(t0);
    if (t_first < t1) tile_issue_loads<I>(w, t_first * 64 * C::NV, n_vec, lane, G);
    for (uint64_t t = t_first, t_next; t < t1; t = t_next) {
        t_next = next_tile(t + 1);
        wave_lds_fence();
        tile_stage<I>(stage, lane, G);
        if (t_next < t1) tile_issue_loads<I>(w, t_next * 64 * C::NV, n_vec, lane, G);
        wave_lds_fence();
        tile_fetch<I>(stage, lane, R);
        const uint64_t seg = t * 64 + lane;
        const bool active = seg < n_seg;
        uint32_t k_out = 0;
        if (OPQ) {
            uint32_t omap[2];
            opq_zero_outliers<I>(R, opq_theta<I>(R, T2), omap);
            k_out = opq_count(omap);
        }
        uint32_t maxabs, sign;
        block_constant<I>(R, lane, signed_norm != 0, maxabs, sign, tie_buf);
        const float m = bf16_bits_to_f32(maxabs | (sign << 15));
        const float m_eff = f16_bits_to_f32(f32_to_f16_bits(m));
        const float a = fabsf(m_eff);
        // |block constant| in units of 2^-24; a constant beyond binary16 (infinite) carries no weight
        // (unweighted: the plain median of the normalised weights - every element of such a block weighs one unit)
        const unsigned long long W =
            (a < 65536.0f) ? (unweighted ? 1ull : (unsigned long long)((double)a * 16777216.0)) : 0ull;
        const double a_sum = unweighted ? 1.0 : (double)a;  // what an element's |x - level| counts with in the error sum
        const bool fast = FAST && __builtin_amdgcn_ballot_w64(!maxabs_is_ordinary(maxabs)) == 0;
        const uint32_t m15_shifted = (f32_to_f16_bits(a) & 0x7fffu) << 4;
        if (active) {
            const BlockDiv dv = make_block_div(m_eff);
            double dsum = 0.0;
            // batches of 8: the table reads of a batch are issued together, then the reads of the regions' search
            // state, then the (few) histogram additions - two dependent LDS round trips per batch instead of per weight
#pragma unroll
            for (int b0 = 0; b0 < C::SEG; b0 += 8) {
                float x[8];
                uint32_t code[8];
                if (fast) {
                    uint2 en[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        x[e] = div_fast(seg_f32(R, b0 + e), dv);
                        en[e] = bin_lookup(tab, x[e], lane_off);
                    }
#pragma unroll
                    for (int e = 0; e < 8; ++e) code[e] = en[e].y + (x[e] > __uint_as_float(en[e].x) ? 1u : 0u);
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const float f = seg_f32(R, b0 + e);
                        x[e] = (m_eff == 0.0f) ? 0.0f : f / m_eff;
                        code[e] = (uint32_t)assign_code_generic(x[e], cb);
                    }
                }
                uint4 inf[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) inf[e] = sh.info[code[e]];
                uint32_t bin[8], subk[8];
                bool counts[8], any = false;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const uint32_t sub = order_key(x[e]) - inf[e].x;
                    subk[e] = sub;
                    if (FIRST) {
                        // the region's keys span exactly its hi bits, of which the first pass takes the top 8 (all of
                        // them if there are fewer): sub >> lo is the digit, and every element counts
                        const uint32_t digit = sub >> (inf[e].y & 31u);
                        bin[e] = code[e] * 256 + digit;
                        counts[e] = CAPTURE && (digit - ((inf[e].y >> 8) & 255u)) < (inf[e].y >> 16);
                    } else {
                        const uint32_t lo = inf[e].y & 0xffu, hi = (inf[e].y >> 8) & 0xffu, dmask = inf[e].y >> 16;
                        counts[e] = inf[e].w != 0u && (sub >> hi) == inf[e].z;
                        bin[e] = code[e] * 256 + ((sub >> lo) & dmask);
                    }
                    any = any || counts[e];
                }
                if (FIRST) {  // every weight lands in some bin: no branches
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        atomicAdd(&sh.hist[bin[e]], W);
                        atomicAdd(&cntcol[(code[e] >> 1) * 64 + lane], 1u << ((code[e] & 1u) * 16u));
                        dsum += fabs((double)x[e] - __hiloint2double((int)inf[e].w, (int)inf[e].z));
                        // pin the addition here: left alone, the compiler sinks all of them below the loop and keeps
                        // every x and level alive until then (it spilled 300 registers)
                        asm volatile("" : "+v"(dsum));
                    }
                    if (CAPTURE && __builtin_amdgcn_ballot_w64(any) != 0) {  // about one weight in 100 is captured
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            const unsigned long long who = __builtin_amdgcn_ballot_w64(counts[e]);
                            if (who == 0ull) continue;  // wave-uniform
                            const uint32_t pos = wave_cand + __builtin_amdgcn_mbcnt_hi(
                                (uint32_t)(who >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)who, 0u));
                            if (counts[e] && pos < cand_cap)  // entry: key | region << 32 | constant << 36
                                my_cand[pos] = make_uint2(subk[e], code[e] | m15_shifted);
                            wave_cand += (uint32_t)__builtin_popcountll(who);
                        }
                    }
                } else if (__builtin_amdgcn_ballot_w64(any) != 0) {  // later passes: one weight in 256 still counts
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const unsigned long long who = __builtin_amdgcn_ballot_w64(counts[e]);
                        if (who == 0ull) continue;  // wave-uniform: three times out of four nobody's element e counts
                        if (counts[e]) atomicAdd(&sh.hist[bin[e]], W);
                        if (cand != nullptr) {  // wave-uniform
                            const uint32_t pos = wave_cand + __builtin_amdgcn_mbcnt_hi(
                                (uint32_t)(who >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)who, 0u));
                            if (counts[e] && pos < cand_cap)  // entry: key | region << 32 | constant << 36
                                my_cand[pos] = make_uint2(subk[e], code[e] | m15_shifted);
                            wave_cand += (uint32_t)__builtin_popcountll(who);
                        }
                    }
                }
            }
            if (OPQ && k_out != 0u) {
                const uint4 inf = sh.info[cz];
                const uint32_t sub = key0 - inf.x;
                const uint32_t lo = FIRST ? (inf.y & 31u) : (inf.y & 0xffu), hi = (inf.y >> 8) & 0xffu;
                const uint32_t dmask = FIRST ? 0xffu : (inf.y >> 16);
                const bool counts = FIRST ? true : (inf.w != 0u && (sub >> hi) == inf.z);
                if (counts)
                    atomicAdd(&sh.hist[cz * 256 + ((sub >> lo) & dmask)], 0ull - (unsigned long long)k_out * W);
                if (FIRST) {
                    atomicAdd(&cntcol[(cz >> 1) * 64 + lane], 0u - (k_out << ((cz & 1u) * 16u)));
                    dsum -= (double)k_out * fabs(__hiloint2double((int)inf.w, (int)inf.z));
                    kout += k_out;
                }
            }
            if (FIRST) {
                sae = fma(a_sum, dsum, sae);
                w_est = fma(a_sum, (double)(C::SEG - k_out), w_est);
            }
        }
        if (FIRST && ++tiles_since_flush == 65535u / C::SEG) {
            flush_counts();
            tiles_since_flush = 0;
        }
    }
    if (FIRST) {
        flush_counts();
        // counts leave as per-wave partials [17][waves], the two floating-point sums as per-workgroup partials (added
        // later in a fixed order)
        unsigned long long kc = kout;
        double s = sae, we = w_est;
#pragma unroll
        for (int mk = 32; mk >= 1; mk >>= 1) {
            kc += (unsigned long long)__shfl_xor((long long)kc, mk, 64);
            s += __shfl_xor(s, mk, 64);
            we += __shfl_xor(we, mk, 64);
        }
        if (lane < 17) cnt_part[lane * n_waves + gw] = lane == 16 ? kc : wave_cnt;
        __shared__ double wave_sums[WAVES_PER_WG][2];
        if (lane == 0) {
            wave_sums[wave][0] = s;
            wave_sums[wave][1] = we;
        }
        __syncthreads();
        if (tid == 0) {
            double s0 = 0.0, s1 = 0.0;
            for (int k = 0; k < WAVES_PER_WG; ++k) {
                s0 += wave_sums[k][0];
                s1 += wave_sums[k][1];
            }
            sae_part[2 * blockIdx.x] = s0;
            sae_part[2 * blockIdx.x + 1] = s1;
        }
    }
    if (cand != nullptr && lane == 0) cand_count[gw] = wave_cand;
    __syncthreads();
    // 64-bit integer atomics: exact and order-free (measured: no slower than writing per-workgroup partials)
    for (uint32_t i = tid; i < 16 * 256; i += 256) {
        const unsigned long long v = sh.hist[i];
        if (v != 0ull) atomicAdd(&hist_g[i], v);
    }
}

// A pass over the list instead of the weights: every wave reads the stretch the wave of the same number wrote.  Does
// nothing when the list ran full (*full != 0: the gated scan of the weights runs instead).
__global__ __launch_bounds__(256) void mae_list_kernel(const unsigned long long* __restrict__ cand,
                                                       const uint32_t* __restrict__ cand_count, uint32_t cand_cap,
                                                       const uint32_t* __restrict__ full,
                                                       const MaeLevelState* __restrict__ state,
                                                       unsigned long long* __restrict__ hist_g, int unweighted) {
    if (*full != 0u) return;
    __shared__ uint4 info[16];
    __shared__ unsigned long long hist[16 * 256];
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid < 16) {
        const MaeLevelState s = state[tid];
        const uint32_t hi = s.hi, lo = hi > 8 ? hi - 8 : 0;
        info[tid] = make_uint4(lo, hi, s.prefix, (hi != 0 && s.total != 0ull && s.pad == 0u) ? 1u : 0u);
    }
    for (uint32_t i = tid; i < 16 * 256; i += 256) hist[i] = 0ull;
    __syncthreads();
    const uint64_t gw = (uint64_t)blockIdx.x * WAVES_PER_WG + wave;
    const uint32_t count = cand_count[gw];  // at most cand_cap, or the list would count as full
    const unsigned long long* mine = cand + gw * cand_cap;
    for (uint32_t i = lane; i < count; i += 64) {
        const unsigned long long e = mine[i];
        const uint32_t sub = (uint32_t)e, l = (uint32_t)(e >> 32) & 15u, m15 = (uint32_t)(e >> 36) & 0x7fffu;
        const uint4 inf = info[l];
        if (inf.w != 0u && (sub >> inf.y) == inf.z) {
            const float a = f16_bits_to_f32(m15);
            const unsigned long long W =
                (a < 65536.0f) ? (unweighted ? 1ull : (unsigned long long)((double)a * 16777216.0)) : 0ull;
            atomicAdd(&hist[l * 256 + ((sub >> inf.x) & ((1u << (inf.y - inf.x)) - 1u))], W);
        }
    }
    __syncthreads();
    for (uint32_t i = tid; i < 16 * 256; i += 256) {
        const unsigned long long v = hist[i];
        if (v != 0ull) atomicAdd(&hist_g[i], v);
    }
}

// After the sampling pass: one wave per region reads the sampled first-digit histogram, finds where the sample's
// weighted median lies, and sets the window of first digits that the full first pass will capture: the sampled place
// plus or minus six standard deviations of a sampled quantile (0.5 / sqrt(samples), widened by half for the unequal
// weights), converted to digits by the share of the region's weight that the median's digit holds, at least half a
// digit to either side.  Clears the bins.  The search state proper is left alone.
__global__ __launch_bounds__(1024) void mae_predict_kernel(MaeLevelState* __restrict__ state,
                                                           unsigned long long* __restrict__ hist,
                                                           const unsigned long long* __restrict__ cnt_part,
                                                           uint32_t n_part, uint32_t skip_mask) {
    const uint32_t lane = threadIdx.x & 63, l = threadIdx.x >> 6;  // wave l = region l
    unsigned long long b[4], sum = 0ull;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        b[k] = hist[l * 256 + 4 * lane + k];
        hist[l * 256 + 4 * lane + k] = 0ull;
        sum += b[k];
    }
    unsigned long long incl = sum;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const unsigned long long up = (unsigned long long)__shfl_up((long long)incl, d, 64);
        if (lane >= (uint32_t)d) incl += up;
    }
    const unsigned long long total = (unsigned long long)__shfl((long long)incl, 63, 64);
    const uint32_t n_waves = n_part * WAVES_PER_WG;
    unsigned long long samples = 0ull;
    for (uint32_t i = lane; i < n_waves; i += 64) samples += cnt_part[l * n_waves + i];
#pragma unroll
    for (int mk = 32; mk >= 1; mk >>= 1) samples += (unsigned long long)__shfl_xor((long long)samples, mk, 64);
    uint32_t win_lo = 0, win_len = 0;
    if (total != 0ull && samples != 0ull && ((skip_mask >> l) & 1u) == 0u) {  // wave-uniform
        const unsigned long long ballot = __builtin_amdgcn_ballot_w64(2ull * incl >= total);
        const uint32_t L = ballot ? (uint32_t)__builtin_ctzll(ballot) : 63u;
        unsigned long long c = incl - sum;  // weight below this lane's four bins
        uint32_t k_sel = 3;
        unsigned long long below = c, mass = b[3];
        bool found = false;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (!found && 2ull * (c + b[k]) >= total) {
                found = true;
                k_sel = (uint32_t)k;
                below = c;
                mass = b[k];
            }
            c += b[k];
        }
        const uint32_t digit = (uint32_t)__shfl((int)(4 * lane + k_sel), (int)L, 64);
        const double below_d = (double)(unsigned long long)__shfl((long long)below, (int)L, 64);
        const double mass_d = (double)(unsigned long long)__shfl((long long)mass, (int)L, 64);
        const double tot = (double)total;
        const double place = (double)digit + (mass_d > 0.0 ? (0.5 * tot - below_d) / mass_d : 0.5);
        const double sigma_q = 0.75 / sqrt((double)samples);
        double half = mass_d > 0.0 ? 6.0 * sigma_q * tot / mass_d : 256.0;
        if (half < 0.5) half = 0.5;
        if (half > 256.0) half = 256.0;
        const double lo_d = floor(place - half), hi_d = floor(place + half);
        const int lo_i = lo_d < 0.0 ? 0 : (int)lo_d, hi_i = hi_d > 255.0 ? 255 : (int)hi_d;
        win_lo = (uint32_t)lo_i;
        win_len = hi_i >= lo_i ? (uint32_t)(hi_i - lo_i + 1) : 0u;
    }
    if (lane == 0) {
        state[l].win_lo = win_lo;
        state[l].win_len = win_len;
    }
}

// After a pass: one wave per region reads its 256 bins, fixes the next digit and clears the bins.  FIRST also takes
// the region's total from the bins.  LAST writes the result record (layout of bof4_mae_stats): [0..15] median,
// [16..31] den, [32..47] cnt (integers), [48] sae, [49] n_used, [50] n_outliers (integers); word 49 is stored last, at
// system scope, so that a host watching it may read the record as soon as it changes.
__global__ __launch_bounds__(1024) void mae_select_kernel(MaeLevelState* __restrict__ state,
                                                          unsigned long long* __restrict__ hist,
                                                          const unsigned long long* __restrict__ cnt_part,
                                                          const double* __restrict__ sae_part, uint32_t n_part,
                                                          int first, int last, uint32_t skip_mask,
                                                          const uint32_t* __restrict__ cand_count,
                                                          uint32_t cand_waves, uint32_t cand_cap,
                                                          uint32_t* __restrict__ cand_full, int check_window,
                                                          double* __restrict__ out, int unweighted) {
    const uint32_t lane = threadIdx.x & 63, l = threadIdx.x >> 6;  // wave l = region l
    // after the pass that wrote the list: did every wave's stretch hold its entries?  (and, below, if the list was
    // captured by windows: does every region's digit lie inside its window?)
    uint32_t list_bad = 0;
    if (cand_count != nullptr)
        for (uint32_t i = threadIdx.x; i < cand_waves; i += 1024) list_bad |= cand_count[i] > cand_cap ? 1u : 0u;
    MaeLevelState s = state[l];
    unsigned long long b[4], sum = 0ull;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        b[k] = hist[l * 256 + 4 * lane + k];
        hist[l * 256 + 4 * lane + k] = 0ull;
        sum += b[k];
    }
    unsigned long long incl = sum;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const unsigned long long up = (unsigned long long)__shfl_up((long long)incl, d, 64);
        if (lane >= (uint32_t)d) incl += up;
    }
    if (first) s.total = (unsigned long long)__shfl((long long)incl, 63, 64);
    const bool skipped = ((skip_mask >> l) & 1u) != 0u;  // only the region's mass was wanted: no search
    if (skipped) s.pad = 1u;
    if (!skipped && s.hi != 0u && s.total != 0ull) {  // wave-uniform
        const uint32_t lo = s.hi > 8 ? s.hi - 8 : 0;
        // smallest digit d with 2 (base + weight of digits <= d) >= total; totals stay below 2^62 (checked below)
        const bool reached = 2ull * (s.base + incl) >= s.total;
        const unsigned long long ballot = __builtin_amdgcn_ballot_w64(reached);
        // the bins of this pass hold all the weight between base and the end of the prefix's range, and the prefix
        // was chosen because the total is reached inside it: some lane has reached it
        const uint32_t L = ballot ? (uint32_t)__builtin_ctzll(ballot) : 63u;
        unsigned long long c = s.base + incl - sum;  // weight below this lane's four bins
        uint32_t k_sel = 3;
        unsigned long long below = 0ull;
        bool found = false;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (!found && 2ull * (c + b[k]) >= s.total) {
                found = true;
                k_sel = (uint32_t)k;
                below = c;
            }
            c += b[k];
        }
        if (!found) below = c - b[3];
        const uint32_t digit = (uint32_t)__shfl((int)(4 * lane + k_sel), (int)L, 64);
        const unsigned long long nb = (unsigned long long)__shfl((long long)below, (int)L, 64);
        s.prefix = (s.prefix << (s.hi - lo)) | digit;
        s.base = nb;
        s.hi = lo;
        if (check_window && !((digit - s.win_lo) < s.win_len)) list_bad = 1u;
    }
    if (lane == 0) state[l] = s;
    if (cand_count != nullptr) {  // uniform
        const int any = __syncthreads_or((int)list_bad);
        if (threadIdx.x == 0) *cand_full = any ? 1u : 0u;
    }
    if (!last) return;
    __shared__ double med[16], den[16];
    __shared__ unsigned long long cnt[17];
    const uint32_t n_waves = n_part * WAVES_PER_WG;
    unsigned long long k_l = 0ull, k_out = 0ull;
    for (uint32_t i0 = lane; i0 < n_waves; i0 += 64 * 8) {  // eight independent loads in flight (integers: any order)
        unsigned long long a[8], b[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const uint32_t i = i0 + 64 * u;
            a[u] = i < n_waves ? cnt_part[l * n_waves + i] : 0ull;
            b[u] = (l == 15 && i < n_waves) ? cnt_part[16 * n_waves + i] : 0ull;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            k_l += a[u];
            k_out += b[u];
        }
    }
#pragma unroll
    for (int mk = 32; mk >= 1; mk >>= 1) {
        k_l += (unsigned long long)__shfl_xor((long long)k_l, mk, 64);
        k_out += (unsigned long long)__shfl_xor((long long)k_out, mk, 64);
    }
    if (lane == 0) {
        med[l] = (s.total != 0ull && s.hi == 0u && s.pad == 0u) ? (double)key_to_float(s.klo + s.prefix)
                                                                  : __builtin_nan("");
        den[l] = (double)s.total * (unweighted ? 1.0 : 0x1p-24);  // correctly rounded conversion of the integer
        cnt[l] = k_l;
        if (l == 15) cnt[16] = k_out;
    }
    __syncthreads();
    // the floating-point partials in a fixed order: lane i of wave 0 adds records 8 i .. 8 i + 7, then the 64 sums in order
    __shared__ double part_sum[64][2];
    if (l == 0) {
        double s0 = 0.0, s1 = 0.0;
        for (uint32_t p = 8 * lane; p < min(8 * lane + 8, n_part); ++p) {
            s0 += sae_part[2 * p];
            s1 += sae_part[2 * p + 1];
        }
        part_sum[lane][0] = s0;
        part_sum[lane][1] = s1;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        double sae = 0.0, w_est = 0.0;
        for (int i = 0; i < 64; ++i) {
            sae += part_sum[i][0];
            w_est += part_sum[i][1];
        }
        unsigned long long used = 0ull;
        const bool too_large = !(w_est < 0x1p38);  // 64-bit weight sums need sum |constant| < 2^39 (NaN counts too)
        for (int q = 0; q < 16; ++q) {
            out[q] = too_large ? __builtin_nan("") : med[q];
            out[16 + q] = den[q];
            out[32 + q] = __longlong_as_double((long long)cnt[q]);
            used += cnt[q];
        }
        out[48] = too_large ? __builtin_nan("") : sae;
        out[50] = __longlong_as_double((long long)cnt[16]);
        __hip_atomic_store(reinterpret_cast<unsigned long long*>(&out[49]), used, __ATOMIC_RELEASE,
                           __HIP_MEMORY_SCOPE_SYSTEM);
    }
}

}  // namespace bof4
