// bof4.hip - HIP (gfx950) implementation of the C ABI declared in include/bof4.h.
//
// Hot path of BOF4 / BOF4-S / OPQ (arxiv 2505.06653): block (signed) absmax normalisation (section 2.1 eq. 1-3,
// section 3.1 eq. 4), nearest-of-16 assignment (section 3.2), 4-bit packing, OPQ outlier extraction (section 3.3
// eq. 9, appendix E.1), decoding, and the per-region sums of the data-driven Lloyd step (section 3.2 eq. 6,
// appendix B.3).  Nothing here is a dense contraction, so there is no MFMA: the kernels are streaming scans
// bounded by HBM bandwidth and plain VALU issue.
//
// Rounding contract shared by all kernels (and by the independent CPU oracle used in the tests):
//   * the block constant is stored as binary16 and the quantiser normalises by the stored value;
//   * x = w / m is one correctly rounded binary32 division, denormals kept;
//   * code(x) = #{k : x > thr[k]}, thr[k] = largest binary32 <= mid-point of levels k, k+1;
//   * the lowest index wins when several elements share the largest magnitude;
//   * OPQ: w^2 * I(I-1) > T^2 * V with V = fma(-S, S, I*Q) in binary64, S = sum w, Q = sum w^2 over the block.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>
#include <cstring>

#include "bof4.h"
#include "bof4_device.h"
#include "bof4_segment.h"
#include "bof4_mae.h"
#include "bof4_gemv.h"
#include "bof4_gemm.h"
#include "bof4_error.h"
#include "bof4_theory.h"

namespace {
using namespace bof4;

// ------------------------------------------------------------------------------------------------ host state
thread_local char g_err[256] = "";
thread_local int g_hip_err = 0;
// Caller-owned events to be recorded around the main kernel of the next call (bof4_time_next_call).
thread_local hipEvent_t g_ev_start = nullptr, g_ev_stop = nullptr;
void timing_begin(hipStream_t s) {
    if (g_ev_start) (void)hipEventRecord(g_ev_start, s);
}
void timing_end(hipStream_t s) {
    if (g_ev_stop) (void)hipEventRecord(g_ev_stop, s);
    g_ev_start = nullptr;
    g_ev_stop = nullptr;
}

int fail(int code, const char* msg) {
    snprintf(g_err, sizeof(g_err), "%s", msg);
    return code;
}
int fail_hip(hipError_t e, const char* where) {
    g_hip_err = (int)e;
    snprintf(g_err, sizeof(g_err), "%s: %s", where, hipGetErrorString(e));
    return BOF4_ERR_HIP;
}
#define HIP_TRY(expr)                                  \
    do {                                               \
        hipError_t e_ = (expr);                        \
        if (e_ != hipSuccess) return fail_hip(e_, #expr); \
    } while (0)

// Device address of a host pointer that the GPU can write (pinned / registered memory), or nullptr for ordinary
// pageable memory.
void* device_view_of_host(const void* host_ptr) {
    hipPointerAttribute_t attr;
    if (hipPointerGetAttributes(&attr, host_ptr) != hipSuccess) {
        (void)hipGetLastError();  // pageable memory is reported as an error: not one
        return nullptr;
    }
    if (attr.type != hipMemoryTypeHost) return nullptr;
    return attr.devicePointer;
}

bool valid_block(uint32_t b) { return b == 32 || b == 64 || b == 128 || b == 256; }
bool valid_codebook(const double* cb) {
    if (!cb) return false;
    for (int l = 0; l < 16; ++l)
        if (!std::isfinite(cb[l])) return false;
    for (int l = 1; l < 16; ++l)
        if (!(cb[l] > cb[l - 1])) return false;
    return true;
}
bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

void make_thresholds(const double* cb, float* thr) {
    for (int k = 0; k < 15; ++k) {
        double mid = (cb[k] + cb[k + 1]) * 0.5;
        float f = (float)mid;  // round to nearest
        if ((double)f > mid) f = std::nextafterf(f, -INFINITY);
        thr[k] = f;
    }
}
CodebookArgs make_codebook_args(const double* cb) {
    CodebookArgs a;
    make_thresholds(cb, a.thr);
    a.thr[15] = INFINITY;
    for (int l = 0; l < 16; ++l) {
        a.lv32[l] = (float)cb[l];
        a.cb64[l] = cb[l];
    }
    return a;
}

// Host replica of the kernels' bin index (same fused multiply-add, same mask): monotone in x.
uint32_t host_bin(float x) {
    float t = std::fmaf(x, BIN_SCALE, BIN_MAGIC);
    uint32_t u;
    std::memcpy(&u, &t, 4);
    return (u & BIN_MASK) >> BIN_SHIFT;
}
// Builds the per-bin (threshold, base code) table: for x in bin b, code(x) = base[b] + (x > thr[b]).  A bin that
// two thresholds cut, or a threshold too close to zero, switches the shortcut path off (fast = 0).
struct BinEdges {
    float xlo[33], xhi[33];  // smallest and largest binary32 x in [-1, 1] that falls into each bin
    BinEdges() {
        xlo[0] = -1.0f;
        xhi[32] = 1.0f;
        for (uint32_t b = 1; b <= 32; ++b) {  // smallest x whose bin is >= b, by bisection over binary32 values
            float lo = -1.0f, hi = 1.0f;      // bin(lo) < b <= bin(hi)
            while (std::nextafterf(lo, hi) != hi) {
                float mid = 0.5f * lo + 0.5f * hi;
                if (!(mid > lo && mid < hi)) mid = std::nextafterf(lo, hi);
                if (host_bin(mid) >= b) hi = mid; else lo = mid;
            }
            xlo[b] = hi;
            xhi[b - 1] = lo;
        }
    }
};
BinTable make_bin_table(const CodebookArgs& cb) {
    static const BinEdges edges;  // the same for every codebook: found once
    const float* xlo = edges.xlo;
    const float* xhi = edges.xhi;
    BinTable t;
    t.fast = 1;
    for (uint32_t b = 0; b <= 32; ++b) {
        uint32_t base = 0, inside = 0;
        float thr = INFINITY;
        for (int k = 0; k < 15; ++k) {
            if (cb.thr[k] < xlo[b]) base++;
            else if (cb.thr[k] < xhi[b]) { inside++; thr = cb.thr[k]; }
        }
        if (inside > 1) t.fast = 0;
        t.base[b] = base;
        t.thr[b] = thr;
    }
    t.code_of_zero = 0;
    for (int k = 0; k < 15; ++k) {
        if (0.0f > cb.thr[k]) t.code_of_zero++;
        if (std::fabs(cb.thr[k]) < 0x1p-30f) t.fast = 0;
    }
    return t;
}

// ------------------------------------------------------------------------------------------------ workspace
constexpr uint32_t QTILE = 2048;         // weights per quantise tile (256 threads x 8)
size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct QuantWsLayout {
    size_t header, tile_cnt, tile_base, tile_off, stage_idx, stage_val, total;
};
QuantWsLayout quant_ws_layout(uint64_t n, uint64_t cap) {
    QuantWsLayout L;
    uint64_t nt = (n + QTILE - 1) / QTILE;
    size_t o = 0;
    L.header = o;    o += 256;
    L.tile_cnt = o;  o += align_up(nt * 4, 256);
    L.tile_base = o; o += align_up(nt * 8, 256);
    L.tile_off = o;  o += align_up(nt * 8, 256);
    L.stage_idx = o; o += align_up(cap * 8, 256);
    L.stage_val = o; o += align_up(cap * 2, 256);
    L.total = o;
    return L;
}
constexpr uint32_t SEG_GRID = 512;              // persistent workgroups of the MAE and error kernels (2 per CU)
// persistent workgroups of a pass: as many as the 256 compute units hold at once
constexpr uint32_t pass_grid(bool opq, bool quant, bool lloyd) {
    return 256u * (uint32_t)pass_waves_per_simd(opq, quant, lloyd);
}
constexpr uint32_t PASS_GRID_MAX = 1024;         // what the workspaces are sized for
struct SegWsLayout {
    size_t header, wave_count, idx, val, total;
    uint32_t region_cap;
};
SegWsLayout seg_ws_layout(uint64_t cap) {
    SegWsLayout L;
    const uint64_t nw = (uint64_t)PASS_GRID_MAX * WAVES_PER_WG;  // one staging region per wave of the largest grid
    uint64_t rc = 4 * ((cap + nw - 1) / nw) + 64;  // four times the even share: room for uneven outlier density
    if (rc > 0x7fffffffull) rc = 0x7fffffffull;
    L.region_cap = (uint32_t)rc;
    size_t o = 0;
    L.header = o;     o += 256;
    L.wave_count = o; o += align_up(nw * 4, 256);
    L.idx = o;        o += align_up(nw * rc * 8, 256);
    L.val = o;        o += align_up(nw * rc * 2, 256);
    L.total = o;
    return L;
}
size_t quant_ws_bytes(uint64_t n, uint64_t cap) {
    size_t a = quant_ws_layout(n, cap).total, b = seg_ws_layout(cap).total;
    return a > b ? a : b;
}
// Where the Lloyd records of bof4_quantize_lloyd lie: behind the quantiser's part of the workspace, if it has one.
size_t fused_lloyd_offset(uint64_t n, uint64_t cap, bool opq) { return opq ? align_up(quant_ws_bytes(n, cap), 256) : 0; }
// Wait for the stream to drain.  The calls that hand results to the host are short (a fraction of a millisecond), so
// the host first polls the stream, which notices completion sooner than the blocking wait; work that takes longer
// than the polling budget falls through to the blocking wait.
hipError_t wait_for_stream(hipStream_t s) {
    for (int spin = 0; spin < 4000; ++spin) {
        const hipError_t q = hipStreamQuery(s);
        if (q == hipSuccess) return hipSuccess;
        if (q != hipErrorNotReady) return q;
    }
    return hipStreamSynchronize(s);
}
// Wait for a result that the last kernel of a call stores straight into pinned host memory.  The host puts
// FLAG_PENDING, a value no result can have, into the 64-bit word that the kernel writes last (with release
// semantics at system scope, so the rest of the record is there first) and watches that word; every so often it
// also asks the stream, so that an error, or a store that only becomes visible when the kernel has ended, ends the
// watch.  On return the result is in host memory; the call's device outputs are complete in stream order.
constexpr uint64_t FLAG_PENDING = ~0ull;
hipError_t wait_for_flag(hipStream_t s, const uint64_t* flag_host) {
    const volatile uint64_t* flag = flag_host;
    for (uint32_t spin = 1;; ++spin) {
        if (*flag != FLAG_PENDING) {
            std::atomic_thread_fence(std::memory_order_acquire);
            return hipSuccess;
        }
        if ((spin & 255u) == 0) {
            const hipError_t q = hipStreamQuery(s);
            if (q != hipErrorNotReady) {
                if (q != hipSuccess) return q;
                break;  // drained
            }
        }
    }
    return hipStreamSynchronize(s);
}
size_t lloyd_ws_bytes() { return ((size_t)PASS_GRID_MAX + 1) * LLOYD_PART * 8; }
static_assert(pass_grid(false, true, false) <= PASS_GRID_MAX && pass_grid(false, false, true) <= PASS_GRID_MAX &&
                  SEG_GRID <= PASS_GRID_MAX,
              "workspace sized for fewer workgroups");
// MAE step: histogram, search state, per-wave counts, per-workgroup floating-point partials, result record.
// Entries of the candidate list of the MAE step, dealt out evenly to the waves of the pass kernels: n / 32 (four
// times what the windows of the one-pass search let through on a large tensor, five times what a second pass
// leaves), at most 2^27; below 2^29 weights n / 16, because the windows are wider there (fewer samples to place them:
// 4 to 5 % of the weights at 2^26) and a wave's share of the list is small enough for its fill to vary.
// The MAE step samples one tile in 16 to place its windows, from 16384 wave tiles (2^26 weights at block 64) up: below
// that the second pass over the weights costs less than it would save.
constexpr uint32_t MAE_SAMPLE_MASK = 15;
constexpr uint64_t MAE_SAMPLING_MIN_TILES = 16384;
uint64_t mae_cand_entries(uint64_t n) {
    const uint64_t e = n < (1ull << 29) ? n / 16 : n / 32;
    return e < (1ull << 27) ? e : (1ull << 27);
}
struct MaeWsLayout {
    size_t hist, state, cnt_part, sae_part, record, cand_count, cand_full, cand, total;
};
MaeWsLayout mae_ws_layout(uint64_t n) {
    MaeWsLayout L;
    size_t o = 0;
    L.hist = o;     o += 16 * 256 * 8;
    L.state = o;    o += align_up(16 * sizeof(MaeLevelState), 256);
    L.cnt_part = o; o += align_up((size_t)17 * SEG_GRID * WAVES_PER_WG * 8, 256);
    L.sae_part = o; o += align_up((size_t)SEG_GRID * 2 * 8, 256);
    L.record = o;   o += align_up(MAE_REC * 8, 256);
    L.cand_count = o; o += align_up((size_t)SEG_GRID * WAVES_PER_WG * 4, 256);
    L.cand_full = o;  o += 256;
    L.cand = o;       o += align_up(mae_cand_entries(n) * 8, 256);
    L.total = o;
    return L;
}
// Order-preserving key of a binary32 number (host replica of the kernels' map).
uint32_t host_order_key(float x) {
    uint32_t b;
    std::memcpy(&b, &x, 4);
    return b ^ ((b >> 31) ? 0xFFFFFFFFu : 0x80000000u);
}

// ------------------------------------------------------------------------------------------------ device helpers
__device__ __forceinline__ int assign_code(float x, const CodebookArgs& cb) { return assign_code_generic(x, cb); }
// argmax key: larger magnitude first, then lower index; the sign rides in bit 0 and never decides.
__device__ __forceinline__ uint32_t max_key(uint32_t bits16, uint32_t idx) {
    return ((bits16 & 0x7fffu) << 16) | ((0x7fffu - idx) << 1) | (bits16 >> 15);
}
template <int WIDTH>
__device__ __forceinline__ uint32_t group_max_u32(uint32_t v) {
#pragma unroll
    for (int m = 1; m < WIDTH; m <<= 1) v = max(v, (uint32_t)__shfl_xor((int)v, m, 64));
    return v;
}
template <int WIDTH>
__device__ __forceinline__ double group_sum_f64(double v) {
#pragma unroll
    for (int m = 1; m < WIDTH; m <<= 1) v += __shfl_xor(v, m, 64);
    return v;
}

// ------------------------------------------------------------------------------------------------ quantise
// General path, slower than the segment kernel of bof4_segment.h and taken only when a wave of that kernel found more
// outliers than its staging region holds: tiles append their outliers through one global counter, so any
// distribution of outliers over the tensor fits the caller's capacity.  Plain binary64 OPQ statistics, IEEE
// division, 15 compares.
// One lane owns 8 consecutive weights (one 16-byte load); a block of I weights spans I/8 neighbouring lanes.
template <int I, bool SIGNED, bool OPQ>
__global__ __launch_bounds__(256) void quantize_kernel(const uint4* __restrict__ w, uint64_t n_vec,
                                                        CodebookArgs cb, double T2, uint32_t* __restrict__ codes,
                                                        uint16_t* __restrict__ scales, uint64_t* total_ctr,
                                                        uint32_t* tile_cnt, uint64_t* tile_base,
                                                        int64_t* stage_idx, uint16_t* stage_val, uint64_t capacity) {
    constexpr int G = I / 8;  // lanes per block
    __shared__ uint32_t wave_tot[4];
    __shared__ uint64_t base_sh;
    const uint64_t tile = blockIdx.x;
    const uint64_t v = tile * 256 + threadIdx.x;
    const bool active = v < n_vec;
    uint4 q = active ? w[v] : make_uint4(0, 0, 0, 0);
    uint32_t r[4] = {q.x, q.y, q.z, q.w};
    uint32_t b[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) b[e] = (e & 1) ? (r[e >> 1] >> 16) : (r[e >> 1] & 0xffffu);
    const uint32_t lane_in_group = threadIdx.x & (G - 1);

    uint32_t omask = 0;
    if (OPQ) {
        double S = 0.0, Q = 0.0;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            double d = (double)bf16_bits_to_f32(b[e]);
            S += d;
            Q = fma(d, d, Q);
        }
        S = group_sum_f64<G>(S);
        Q = group_sum_f64<G>(Q);
        double V = fma(-S, S, (double)I * Q);
        double rhs = T2 * V;
        constexpr double II1 = (double)I * (double)(I - 1);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            double d = (double)bf16_bits_to_f32(b[e]);
            if (V > 0.0 && (d * d) * II1 > rhs) omask |= 1u << e;
        }
    }
    uint32_t key = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        uint32_t be = (omask >> e) & 1u ? 0u : b[e];
        key = max(key, max_key(be, lane_in_group * 8 + e));
    }
    key = group_max_u32<G>(key);
    uint32_t mbits = (key >> 16) | (SIGNED ? ((key & 1u) << 15) : 0u);
    float m = bf16_bits_to_f32(mbits);
    uint32_t s16 = f32_to_f16_bits(m);
    float m_eff = f16_bits_to_f32(s16);
    uint32_t packed = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        float f = (omask >> e) & 1u ? 0.0f : bf16_bits_to_f32(b[e]);
        float x = (m_eff == 0.0f) ? 0.0f : f / m_eff;
        packed |= (uint32_t)assign_code(x, cb) << (4 * e);
    }
    if (active) {
        codes[v] = packed;
        if (lane_in_group == 0) scales[v / G] = (uint16_t)s16;
    }
    if (OPQ) {
        // ordered compaction of this tile's outliers into a contiguous run of the staging list
        const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
        uint32_t cntv = active ? __popc(omask) : 0;
        uint32_t incl = cntv;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            uint32_t t = (uint32_t)__shfl_up((int)incl, d, 64);
            if (lane >= (uint32_t)d) incl += t;
        }
        if (lane == 63) wave_tot[wave] = incl;
        __syncthreads();
        uint32_t wbase = 0, tot = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            uint32_t t = wave_tot[k];
            if ((uint32_t)k < wave) wbase += t;
            tot += t;
        }
        if (threadIdx.x == 0) {
            uint64_t base = 0;
            if (tot) base = atomicAdd((unsigned long long*)total_ctr, (unsigned long long)tot);
            base_sh = base;
            tile_cnt[tile] = tot;
            tile_base[tile] = base;
        }
        __syncthreads();
        if (cntv) {
            uint64_t pos = base_sh + wbase + (incl - cntv);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                if ((omask >> e) & 1u) {
                    if (pos < capacity) {
                        stage_idx[pos] = (int64_t)(v * 8 + e);
                        stage_val[pos] = (uint16_t)f32_to_f16_bits(bf16_bits_to_f32(b[e]));
                    }
                    ++pos;
                }
            }
        }
    }
}

// Exclusive prefix sum of the per-tile outlier counts (one workgroup, tiles in index order).
__global__ __launch_bounds__(1024) void tile_scan_kernel(const uint32_t* __restrict__ tile_cnt, uint64_t n_tiles,
                                                          uint64_t* __restrict__ tile_off) {
    __shared__ uint64_t wsum[16];
    __shared__ uint64_t carry_sh;
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (threadIdx.x == 0) carry_sh = 0;
    __syncthreads();
    for (uint64_t t0 = 0; t0 < n_tiles; t0 += 1024) {
        uint64_t t = t0 + threadIdx.x;
        uint64_t c = t < n_tiles ? tile_cnt[t] : 0;
        uint64_t incl = c;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            uint64_t u = (uint64_t)__shfl_up((long long)incl, d, 64);
            if (lane >= (uint32_t)d) incl += u;
        }
        if (lane == 63) wsum[wave] = incl;
        __syncthreads();
        uint64_t wbase = 0, tot = 0;
        for (int k = 0; k < 16; ++k) {
            uint64_t u = wsum[k];
            if ((uint32_t)k < wave) wbase += u;
            tot += u;
        }
        uint64_t carry = carry_sh;
        if (t < n_tiles) tile_off[t] = carry + wbase + incl - c;
        __syncthreads();
        if (threadIdx.x == 0) carry_sh = carry + tot;
        __syncthreads();
    }
}

// Move every tile's run from the staging list to its final, globally ascending position.
__global__ __launch_bounds__(256) void outlier_gather_kernel(const uint32_t* __restrict__ tile_cnt,
                                                              const uint64_t* __restrict__ tile_base,
                                                              const uint64_t* __restrict__ tile_off,
                                                              uint64_t n_tiles, const int64_t* __restrict__ stage_idx,
                                                              const uint16_t* __restrict__ stage_val,
                                                              int64_t* __restrict__ out_idx,
                                                              uint16_t* __restrict__ out_val, uint64_t capacity) {
    uint64_t t = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= n_tiles) return;
    uint32_t c = tile_cnt[t];
    uint64_t src = tile_base[t], dst = tile_off[t];
    for (uint32_t j = 0; j < c; ++j) {
        if (src + j < capacity && dst + j < capacity) {
            out_idx[dst + j] = stage_idx[src + j];
            out_val[dst + j] = stage_val[src + j];
        }
    }
}

__global__ void zero_u64_kernel(uint64_t* p) { *p = 0; }

// ------------------------------------------------------------------------------------------------ dequantise
// One lane decodes 8 codes (one 32-bit load) into 8 bfloat16 (one 16-byte store); a workgroup walks DEQ_VPT chunks of
// 256 such vectors, all loads first.  w~ = constant * level (section 2.1 eq. 3): one binary32 multiply, rounded to
// bfloat16 (nearest even) by the hardware conversion.

constexpr int DEQ_VPT = 4;  // 16-byte vectors per lane and tile
constexpr uint64_t DEQ_RESIDENT_WGS = 2048;  // 256 compute units x 8 workgroups of 256 lanes
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2_rne(float lo, float hi) {
    f32x2_t v = {lo, hi};
    bf16x2_t r = __builtin_convertvector(v, bf16x2_t);
    uint32_t u;
    __builtin_memcpy(&u, &r, 4);
    return u;
}
// With an outlier list (section 3.3: outliers are kept in 16 bit beside the codes and replace their zero placeholders)
// a workgroup takes a contiguous run of tiles (256 * DEQ_VPT * 8 weights each): it finds once where its first weight
// falls in the ascending list - a 256-way search, three rounds for any list a call can carry - and then walks
// the list forward: every tile is decoded into LDS, one lane per listed outlier overwrites its weight there, and the
// tile is stored.  Every output line is written exactly once: patching lines that have left the caches costs a
// partial write each, about as much as writing a third of the tensor again.  Without a list the tile takes the same
// way through LDS: its stores then leave in one burst behind the barrier, which the memory system takes 10 % faster
// than stores that trickle out between the decode arithmetic.
template <int I>
__global__ __launch_bounds__(256) void dequantize_kernel(const uint32_t* __restrict__ codes,
                                                          const uint16_t* __restrict__ scales, uint64_t n_vec,
                                                          uint32_t tiles_per_wg, uint32_t window, CodebookArgs cb,
                                                          const int64_t* __restrict__ out_idx,
                                                          const uint16_t* __restrict__ out_val, uint64_t n_out,
                                                          uint4* __restrict__ out) {
    constexpr int G = I / 8;
    constexpr int TILE_VEC = 256 * DEQ_VPT;
    __shared__ float lv[16];
    __shared__ uint4 stage[TILE_VEC];
    if (threadIdx.x < 16) lv[threadIdx.x] = cb.lv32[threadIdx.x];
    __syncthreads();
    // Workgroups go to the 8 accelerator dies (XCDs, each with an L2 of its own) in turn: die k takes the k-th eighth
    // of the runs, so that the stretch of the list a die's workgroups search and walk is fetched into one L2 only.
    const uint32_t q8 = gridDim.x / 8, r8 = gridDim.x % 8, k8 = blockIdx.x % 8;
    const uint32_t run = k8 * q8 + (k8 < r8 ? k8 : r8) + blockIdx.x / 8;
    const uint64_t first_tile = (uint64_t)run * tiles_per_wg;
    uint64_t lo = 0;
    {
        // first list position whose index is >= the workgroup's first weight; invariant: every entry before lo is
        // smaller, every entry from hi on is not
        const int64_t target = (int64_t)(first_tile * TILE_VEC * 8);
        uint64_t hi = n_out;
        while (lo < hi) {
            const uint64_t step = (hi - lo + 255) / 256;
            const uint64_t p = lo + threadIdx.x * step;
            const int below = (p < hi && out_idx[p] < target) ? 1 : 0;
            const uint64_t cnt = (uint64_t)__syncthreads_count(below);  // the list ascends: the first cnt probes
            const uint64_t new_hi = lo + cnt * step;
            if (cnt > 0) lo = lo + (cnt - 1) * step + 1;
            if (new_hi < hi) hi = new_hi;
        }
    }
    for (uint32_t t = 0; t < tiles_per_wg; ++t) {
        // Without a list the tiles are dealt out in turn (workgroup b takes tiles b, b + gridDim.x, ...): at any moment
        // the chip then writes one compact stretch of the output, which the memory system takes 9 % faster than one
        // far-apart stream per workgroup.  (With a list every tile would have to find its place in it: measured, the
        // probes cost more than the order gains.)
        const uint64_t tile = n_out == 0 ? (uint64_t)blockIdx.x + (uint64_t)t * gridDim.x : first_tile + t;
        const uint64_t base = tile * TILE_VEC + threadIdx.x;
        if (tile * TILE_VEC >= n_vec) break;
        // the next `window` list entries (the host sizes it to what a tile usually holds) travel with the codes
        int64_t pre_i = -1, pre_nxt = -1;
        uint32_t pre_val = 0;
        if (threadIdx.x < window) {
            const uint64_t j = lo + threadIdx.x;
            if (j < n_out) {
                pre_i = out_idx[j];
                pre_val = out_val[j];
            }
            if (j + 1 < n_out) pre_nxt = out_idx[j + 1];
        }
        uint32_t c[DEQ_VPT];
        float s[DEQ_VPT];
#pragma unroll
        for (int k = 0; k < DEQ_VPT; ++k) {
            const uint64_t v = base + 256 * k;
            c[k] = v < n_vec ? __builtin_nontemporal_load(&codes[v]) : 0u;
            s[k] = v < n_vec ? f16_bits_to_f32(scales[v / G]) : 0.0f;
        }
#pragma unroll
        for (int k = 0; k < DEQ_VPT; ++k) {
            uint32_t o[4];
#pragma unroll
            for (int p = 0; p < 4; ++p)
                o[p] = pack_bf16x2_rne(s[k] * lv[(c[k] >> (8 * p)) & 15u], s[k] * lv[(c[k] >> (8 * p + 4)) & 15u]);
            stage[256 * k + threadIdx.x] = make_uint4(o[0], o[1], o[2], o[3]);
        }
        __syncthreads();
        if (n_out != 0) {  // uniform
            const int64_t tile_begin = (int64_t)(tile * TILE_VEC * 8);
            const int64_t tile_end = tile_begin + TILE_VEC * 8;
            uint16_t* stage16 = reinterpret_cast<uint16_t*>(stage);
            for (bool first = true;; first = false) {
                const uint64_t j = lo + threadIdx.x;
                const bool mine = threadIdx.x < window;
                int64_t i = pre_i, nxt = pre_nxt;
                uint32_t val = pre_val;
                if (!first) {
                    i = nxt = -1;
                    if (mine && j < n_out) {
                        i = out_idx[j];
                        val = out_val[j];
                    }
                    if (mine && j + 1 < n_out) nxt = out_idx[j + 1];
                }
                const int inside = (mine && j < n_out && i >= tile_begin && i < tile_end) ? 1 : 0;
                // of several entries with one index the last one counts
                if (inside && nxt != i) stage16[i - tile_begin] = (uint16_t)f32_to_bf16_rne(f16_bits_to_f32(val));
                const uint32_t cnt = (uint32_t)__syncthreads_count(inside);
                lo += cnt;
                if (cnt < window) break;
            }
            // the barrier inside the loop has ordered the patches before these reads
        }
#pragma unroll
        for (int k = 0; k < DEQ_VPT; ++k) {
            const uint64_t v = base + 256 * k;
            if (v < n_vec) store_stream(&out[v], stage[256 * k + threadIdx.x]);
        }
        __syncthreads();  // the next tile overwrites the stage
    }
}

// ------------------------------------------------------------------------------------------------ dispatch
// Arguments of one pass over the weights (seg_pass_kernel) and the launch of the variant that fits them.
struct PassArgs {
    const uint4* w;
    uint64_t n_seg;
    CodebookArgs cb;
    BinTable bt;
    int signed_norm, weight_by_max2;
    double T2;
    uint32_t* codes;
    uint16_t* scales;
    OutlierStage os;
    double* partials;
};
template <int I, bool QUANT, bool LLOYD>
void launch_pass_i(bool opq, uint32_t grid, hipStream_t s, const PassArgs& a) {
#define BOF4_PASS(FAST_, OPQ_)                                                                                       \
    hipLaunchKernelGGL((seg_pass_kernel<I, FAST_, OPQ_, QUANT, LLOYD>), dim3(grid), dim3(256), 0, s, a.w, a.n_seg,   \
                       a.cb, a.bt, a.signed_norm, a.weight_by_max2, a.T2, LLOYD_INC_MUL, LLOYD_INC_ADD, a.codes,    \
                       a.scales, a.os, a.partials)
    if (a.bt.fast && opq) BOF4_PASS(true, true);
    else if (a.bt.fast) BOF4_PASS(true, false);
    else if (opq) BOF4_PASS(false, true);
    else BOF4_PASS(false, false);
#undef BOF4_PASS
}
// Returns the grid it launched (one Lloyd partial record per workgroup, four outlier staging regions).
template <bool QUANT, bool LLOYD>
uint32_t launch_pass(uint32_t block, bool opq, hipStream_t s, const PassArgs& a) {
    const uint64_t tiles = (a.n_seg + 63) / 64;
    const uint64_t want = (tiles + WAVES_PER_WG - 1) / WAVES_PER_WG;
    const uint32_t full = pass_grid(opq, QUANT, LLOYD);
    const uint32_t grid = (uint32_t)(want < full ? want : full);
    switch (block) {
        case 32: launch_pass_i<32, QUANT, LLOYD>(opq, grid, s, a); break;
        case 64: launch_pass_i<64, QUANT, LLOYD>(opq, grid, s, a); break;
        case 128: launch_pass_i<128, QUANT, LLOYD>(opq, grid, s, a); break;
        default: launch_pass_i<256, QUANT, LLOYD>(opq, grid, s, a); break;
    }
    return grid;
}
uint32_t pass_grid_for(uint64_t n_seg, bool opq, bool quant, bool lloyd) {
    const uint64_t tiles = (n_seg + 63) / 64;
    const uint64_t want = (tiles + WAVES_PER_WG - 1) / WAVES_PER_WG;
    const uint32_t full = pass_grid(opq, quant, lloyd);
    return (uint32_t)(want < full ? want : full);
}

template <int I, bool SIGNED, bool OPQ>
void launch_quantize(dim3 grid, hipStream_t s, const uint4* w, uint64_t n_vec, const CodebookArgs& cb, double T2,
                     uint32_t* codes, uint16_t* scales, uint64_t* total, uint32_t* tc, uint64_t* tb, int64_t* si,
                     uint16_t* sv, uint64_t cap) {
    hipLaunchKernelGGL((quantize_kernel<I, SIGNED, OPQ>), grid, dim3(256), 0, s, w, n_vec, cb, T2, codes, scales,
                       total, tc, tb, si, sv, cap);
}
template <int I>
void launch_quantize_i(bool sg, bool opq, dim3 grid, hipStream_t s, const uint4* w, uint64_t n_vec,
                       const CodebookArgs& cb, double T2, uint32_t* codes, uint16_t* scales, uint64_t* total,
                       uint32_t* tc, uint64_t* tb, int64_t* si, uint16_t* sv, uint64_t cap) {
    if (sg && opq) launch_quantize<I, true, true>(grid, s, w, n_vec, cb, T2, codes, scales, total, tc, tb, si, sv, cap);
    else if (sg) launch_quantize<I, true, false>(grid, s, w, n_vec, cb, T2, codes, scales, total, tc, tb, si, sv, cap);
    else if (opq) launch_quantize<I, false, true>(grid, s, w, n_vec, cb, T2, codes, scales, total, tc, tb, si, sv, cap);
    else launch_quantize<I, false, false>(grid, s, w, n_vec, cb, T2, codes, scales, total, tc, tb, si, sv, cap);
}

}  // namespace

// ================================================================================================ C ABI
extern "C" {

const char* bof4_last_error(void) { return g_err; }
int bof4_time_next_call(void* start_event, void* stop_event) {
    g_ev_start = (hipEvent_t)start_event;
    g_ev_stop = (hipEvent_t)stop_event;
    return BOF4_OK;
}
int bof4_last_hip_error(void) { return g_hip_err; }

size_t bof4_workspace_bytes(uint64_t n, uint32_t block, uint64_t out_capacity) {
    if (!valid_block(block) || n == 0 || n % block != 0) return 0;
    // the quantiser's part and, behind it, the Lloyd records (bof4_quantize_lloyd uses both at once)
    size_t q = fused_lloyd_offset(n, out_capacity, true) + lloyd_ws_bytes();
    const size_t m = mae_ws_layout(n).total;
    return m > q ? m : q;
}

double bof4_opq_threshold(double q, uint32_t block) {
    if (!(q > 0.0 && q < 1.0) || block < 2) return NAN;
    // F_M(t) = (2 G(t) - 1)^I = q  <=>  G(t) = (1 + q^(1/I)) / 2; Newton on the normal cdf written with erfc
    const double p = 0.5 * (1.0 + std::exp(std::log(q) / (double)block));
    const double tail = 1.0 - p;  // upper tail probability
    double t = std::sqrt(-2.0 * std::log(tail));
    for (int it = 0; it < 100; ++it) {
        double up = 0.5 * std::erfc(t / std::sqrt(2.0));
        double pdf = std::exp(-0.5 * t * t) / std::sqrt(2.0 * M_PI);
        double step = (up - tail) / pdf;
        t += step;
        if (std::fabs(step) < 1e-15 * std::fabs(t)) break;
    }
    return t;
}

int bof4_thresholds(const double* cb_host, float* thr_host) {
    if (!valid_codebook(cb_host) || !thr_host) return fail(BOF4_ERR_ARG, "bof4_thresholds: bad codebook or null output");
    make_thresholds(cb_host, thr_host);
    return BOF4_OK;
}

int bof4_bin_table(const double* cb_host, float* thr33_host, uint32_t* base33_host, int* fast_host) {
    if (!valid_codebook(cb_host) || !thr33_host || !base33_host || !fast_host)
        return fail(BOF4_ERR_ARG, "bof4_bin_table: bad codebook or null output");
    const BinTable t = make_bin_table(make_codebook_args(cb_host));
    for (int b = 0; b < 33; ++b) {
        thr33_host[b] = t.thr[b];
        base33_host[b] = t.base[b];
    }
    *fast_host = (int)t.fast;
    return BOF4_OK;
}

int bof4_quant_error(const void* w_dev, uint64_t n, uint32_t block, const double* cb_host, int signed_norm,
                     double opq_T, bof4_error_stats* out_host, void* ws_dev, size_t ws_bytes, void* stream) {
    if (!w_dev || !out_host) return fail(BOF4_ERR_ARG, "bof4_quant_error: null pointer");
    if (!valid_block(block) || n == 0 || n % block != 0) return fail(BOF4_ERR_ARG, "bof4_quant_error: bad n or block");
    if (!valid_codebook(cb_host)) return fail(BOF4_ERR_ARG, "bof4_quant_error: codebook must be 16 finite ascending levels");
    if (!(opq_T >= 0.0) || !std::isfinite(opq_T)) return fail(BOF4_ERR_ARG, "bof4_quant_error: opq_T must be finite and >= 0");
    if (!aligned(w_dev, 16)) return fail(BOF4_ERR_ARG, "bof4_quant_error: misaligned weights");
    if (!ws_dev || !aligned(ws_dev, 256)) return fail(BOF4_ERR_ARG, "bof4_quant_error: workspace null or misaligned");
    static_assert((SEG_GRID + 2) * ERR_PART <= (PASS_GRID_MAX + 1) * LLOYD_PART, "the Lloyd workspace holds the error records");
    if (ws_bytes < lloyd_ws_bytes()) return fail(BOF4_ERR_WORKSPACE, "bof4_quant_error: workspace too small");
    static_assert(sizeof(bof4_error_stats) == 5 * 8, "result record and bof4_error_stats must match");
    hipStream_t s = (hipStream_t)stream;
    const uint32_t seg = block < 64 ? block : 64;
    const uint64_t n_seg = n / seg;
    const CodebookArgs cb = make_codebook_args(cb_host);
    const BinTable bt = make_bin_table(cb);
    double* partials = (double*)ws_dev;
    const double T2 = opq_T * opq_T;
    const bool opq = opq_T > 0.0;
    const uint4* w = (const uint4*)w_dev;
    const uint64_t tiles = (n_seg + 63) / 64;
    const uint64_t wantg = (tiles + WAVES_PER_WG - 1) / WAVES_PER_WG;
    const uint32_t sgrid = (uint32_t)(wantg < SEG_GRID ? wantg : SEG_GRID);
    timing_begin(s);
#define BOF4_LAUNCH_ERR(II)                                                                                          \
    if (bt.fast && opq) hipLaunchKernelGGL((seg_error_kernel<II, true, true>), dim3(sgrid), dim3(256), 0, s, w, n_seg, \
                                           cb, bt, signed_norm, T2, partials);                                       \
    else if (bt.fast) hipLaunchKernelGGL((seg_error_kernel<II, true, false>), dim3(sgrid), dim3(256), 0, s, w, n_seg,  \
                                         cb, bt, signed_norm, T2, partials);                                         \
    else if (opq) hipLaunchKernelGGL((seg_error_kernel<II, false, true>), dim3(sgrid), dim3(256), 0, s, w, n_seg, cb,  \
                                     bt, signed_norm, T2, partials);                                                 \
    else hipLaunchKernelGGL((seg_error_kernel<II, false, false>), dim3(sgrid), dim3(256), 0, s, w, n_seg, cb, bt,      \
                            signed_norm, T2, partials);
    switch (block) {
        case 32: BOF4_LAUNCH_ERR(32) break;
        case 64: BOF4_LAUNCH_ERR(64) break;
        case 128: BOF4_LAUNCH_ERR(128) break;
        default: BOF4_LAUNCH_ERR(256) break;
    }
#undef BOF4_LAUNCH_ERR
    timing_end(s);
    double* rec_dev = partials + (uint64_t)sgrid * ERR_PART;
    double* direct = (double*)device_view_of_host(out_host);
    if (direct) out_host->n = FLAG_PENDING;  // the word the final kernel writes last
    hipLaunchKernelGGL(error_final_kernel, dim3(1), dim3(64), 0, s, partials, sgrid, n, direct ? direct : rec_dev);
    HIP_TRY(hipGetLastError());
    if (direct) {
        HIP_TRY(wait_for_flag(s, &out_host->n));
    } else {
        HIP_TRY(hipMemcpyAsync(out_host, rec_dev, sizeof(bof4_error_stats), hipMemcpyDeviceToHost, s));
        HIP_TRY(wait_for_stream(s));
    }
    return BOF4_OK;
}

size_t bof4_theory_workspace_bytes(uint32_t n_grid) { return ((size_t)3 * n_grid + 32) * sizeof(double); }

int bof4_theory_centroids(const double* pdf_host, const double* cdf_host, uint32_t n_grid, double u_max, uint32_t block,
                          const double* cb_host, uint16_t pinned_mask, int signed_norm, double* cb_out_host,
                          void* ws_dev, size_t ws_bytes, void* stream) {
    if (!pdf_host || !cdf_host || !cb_out_host || !ws_dev) return fail(BOF4_ERR_ARG, "bof4_theory_centroids: null pointer");
    if (n_grid < 3 || n_grid % 2 == 0 || n_grid > (1u << 24) || !(u_max > 0.0) || !std::isfinite(u_max))
        return fail(BOF4_ERR_ARG, "bof4_theory_centroids: the grid needs an odd number of points (3 .. 2^24) and u_max > 0");
    if (block < 2) return fail(BOF4_ERR_ARG, "bof4_theory_centroids: block must be at least 2");
    if (!valid_codebook(cb_host)) return fail(BOF4_ERR_ARG, "bof4_theory_centroids: codebook must be 16 finite ascending levels");
    if (!((pinned_mask >> 15) & 1u) || (!signed_norm && !(pinned_mask & 1u)))
        return fail(BOF4_ERR_ARG, "bof4_theory_centroids: a region that holds a point mass of the normalised weights "
                                  "(level 15; level 0 for absolute normalisation) must be pinned");
    if (cb_host[0] < -1.0 || cb_host[15] > 1.0) return fail(BOF4_ERR_ARG, "bof4_theory_centroids: levels outside [-1, 1]");
    if (!aligned(ws_dev, 256)) return fail(BOF4_ERR_ARG, "bof4_theory_centroids: workspace misaligned");
    if (ws_bytes < bof4_theory_workspace_bytes(n_grid)) return fail(BOF4_ERR_WORKSPACE, "bof4_theory_centroids: workspace too small");
    hipStream_t s = (hipStream_t)stream;
    double* pdf = (double*)ws_dev;
    double* cdf = pdf + n_grid;
    double* psi = cdf + n_grid;
    double* sums = psi + n_grid;
    const double h = u_max / (double)(n_grid - 1);
    TheoryRegions rg;
    rg.skip_mask = pinned_mask;
    for (int l = 0; l < 16; ++l) {
        const double a = l > 0 ? 0.5 * (cb_host[l - 1] + cb_host[l]) : -1.0;
        rg.a[l] = a < -1.0 ? -1.0 : a;
        rg.b[l] = l < 15 ? 0.5 * (cb_host[l] + cb_host[l + 1]) : 1.0;
    }
    HIP_TRY(hipMemcpyAsync(pdf, pdf_host, (size_t)n_grid * 8, hipMemcpyHostToDevice, s));
    HIP_TRY(hipMemcpyAsync(cdf, cdf_host, (size_t)n_grid * 8, hipMemcpyHostToDevice, s));
    hipLaunchKernelGGL(theory_psi_kernel, dim3(1), dim3(1024), 0, s, pdf, n_grid, h, psi);
    hipLaunchKernelGGL(theory_centroid_kernel, dim3(16), dim3(256), 0, s, pdf, cdf, psi, n_grid, h, block, rg, sums);
    HIP_TRY(hipGetLastError());
    double host_sums[32];
    HIP_TRY(hipMemcpyAsync(host_sums, sums, sizeof(host_sums), hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    for (int l = 0; l < 16; ++l) {
        cb_out_host[l] = cb_host[l];
        if (!((pinned_mask >> l) & 1u) && host_sums[2 * l + 1] > 0.0) cb_out_host[l] = host_sums[2 * l] / host_sums[2 * l + 1];
    }
    return BOF4_OK;
}

int bof4_codebook_update(const bof4_lloyd_stats* st, uint16_t pinned_mask, double* cb_host) {
    if (!st || !cb_host) return fail(BOF4_ERR_ARG, "bof4_codebook_update: null pointer");
    for (int l = 0; l < 16; ++l) {
        if ((pinned_mask >> l) & 1u) continue;
        if (st->den[l] > 0.0) cb_host[l] = st->num[l] / st->den[l];
    }
    return BOF4_OK;
}

}  // extern "C"

namespace {
// bof4_quantize in two halves.  phase 0: enqueue the kernels and collect the count (the plain call); 1: enqueue only
// (the count has to go to pinned host memory, where phase 2 finds it); 2: collect only, for the same arguments.
enum QuantPhase { QUANT_WHOLE = 0, QUANT_ENQUEUE = 1, QUANT_COLLECT = 2 };
// With stats_host the same pass also takes the Lloyd sums (bof4_quantize_lloyd).
int quantize_impl(int phase, const void* w_dev, uint64_t n, uint32_t block, const double* cb_host, int signed_norm,
                  double opq_T, uint8_t* codes_dev, uint16_t* scales_dev, int64_t* out_idx_dev, uint16_t* out_val_dev,
                  uint64_t out_capacity, uint64_t* n_outliers_host, void* ws_dev, size_t ws_bytes, void* stream,
                  bof4_lloyd_stats* stats_host = nullptr, int weight_by_max2 = 1) {
    if (!w_dev || !codes_dev || !scales_dev || !n_outliers_host) return fail(BOF4_ERR_ARG, "bof4_quantize: null pointer");
    if (!valid_block(block) || n == 0 || n % block != 0) return fail(BOF4_ERR_ARG, "bof4_quantize: bad n or block");
    if (!valid_codebook(cb_host)) return fail(BOF4_ERR_ARG, "bof4_quantize: codebook must be 16 finite ascending levels");
    if (!(opq_T >= 0.0) || !std::isfinite(opq_T)) return fail(BOF4_ERR_ARG, "bof4_quantize: opq_T must be finite and >= 0");
    if (!aligned(w_dev, 16) || !aligned(codes_dev, 4) || !aligned(scales_dev, 2))
        return fail(BOF4_ERR_ARG, "bof4_quantize: misaligned pointer");
    const bool opq = opq_T > 0.0;
    const bool lloyd = stats_host != nullptr;
    hipStream_t s = (hipStream_t)stream;
    const uint64_t n_tiles = (n + QTILE - 1) / QTILE;
    if (n_tiles > 0x7fffffffull) return fail(BOF4_ERR_ARG, "bof4_quantize: n too large for one call");
    const size_t lloyd_off = fused_lloyd_offset(n, out_capacity, opq);
    if (opq) {
        if (out_capacity > 0 && (!out_idx_dev || !out_val_dev)) return fail(BOF4_ERR_ARG, "bof4_quantize: null outlier buffers");
        if (!aligned(out_idx_dev, 8) || !aligned(out_val_dev, 2)) return fail(BOF4_ERR_ARG, "bof4_quantize: misaligned outlier buffers");
    }
    if (opq || lloyd) {
        if (!ws_dev || !aligned(ws_dev, 256)) return fail(BOF4_ERR_ARG, "bof4_quantize: workspace null or misaligned");
        if (ws_bytes < (lloyd ? lloyd_off + lloyd_ws_bytes() : quant_ws_bytes(n, out_capacity)))
            return fail(BOF4_ERR_WORKSPACE, "bof4_quantize: workspace too small");
    }
    const CodebookArgs cb = make_codebook_args(cb_host);
    const BinTable bt = make_bin_table(cb);
    const double T2 = opq_T * opq_T;
    const uint32_t seg = block < 64 ? block : 64;
    const uint64_t n_seg = n / seg;
    const uint32_t sgrid = pass_grid_for(n_seg, opq, true, lloyd);
    const uint32_t n_waves = sgrid * WAVES_PER_WG;
    const uint4* wv = (const uint4*)w_dev;
    uint32_t* cd = (uint32_t*)codes_dev;
    OutlierStage os = {nullptr, nullptr, nullptr, 0};
    SegWsLayout SL = seg_ws_layout(out_capacity);
    uint64_t* total_dev = nullptr;
    if (opq) {
        char* base = (char*)ws_dev;
        total_dev = (uint64_t*)(base + SL.header);
        os.wave_count = (uint32_t*)(base + SL.wave_count);
        os.idx = (int64_t*)(base + SL.idx);
        os.val = (uint16_t*)(base + SL.val);
        os.region_cap = SL.region_cap;
    }
    uint64_t* direct = opq ? (uint64_t*)device_view_of_host(n_outliers_host) : nullptr;
    if (phase != QUANT_WHOLE && opq && !direct)
        return fail(BOF4_ERR_ARG, "bof4_quantize_begin / _finish: the outlier count must go to pinned host memory");
    double* partials = lloyd ? (double*)((char*)ws_dev + lloyd_off) : nullptr;
    double* rec_dev = lloyd ? partials + (uint64_t)sgrid * LLOYD_PART : nullptr;
    double* stats_direct = lloyd ? (double*)device_view_of_host(stats_host) : nullptr;
    if (phase != QUANT_WHOLE && lloyd && !stats_direct)
        return fail(BOF4_ERR_ARG, "bof4_quantize_lloyd_begin: the record must lie in pinned host memory");
    if (phase != QUANT_COLLECT) {
    const PassArgs pa = {wv, n_seg, cb, bt, signed_norm, weight_by_max2, T2, cd, scales_dev, os, partials};
    timing_begin(s);
    if (lloyd) launch_pass<true, true>(block, opq, s, pa);
    else launch_pass<true, false>(block, opq, s, pa);
    timing_end(s);
    HIP_TRY(hipGetLastError());
    if (opq) {
        // total_dev[0] = count, with bit 63 set if a wave overflowed its staging region.  A caller's counter in pinned
        // host memory receives it straight from the gather kernel.
        *n_outliers_host = direct ? FLAG_PENDING : 0;
        hipLaunchKernelGGL(seg_outlier_gather_kernel, dim3(n_waves), dim3(256), 0, s, os, n_waves, out_idx_dev,
                           out_val_dev, out_capacity, direct ? direct : total_dev);
    }
    if (lloyd) {
        if (stats_direct) stats_host->n_used = FLAG_PENDING;  // the word the final kernel writes last
        hipLaunchKernelGGL(seg_lloyd_final_kernel, dim3(1), dim3(1024), 0, s, partials, sgrid, cb, bt.code_of_zero,
                           stats_direct ? stats_direct : rec_dev);
    }
    HIP_TRY(hipGetLastError());
    if (phase == QUANT_ENQUEUE) {
        if (!opq) *n_outliers_host = 0;
        return BOF4_OK;
    }
    if (lloyd) {  // the plain call hands the sums over as well
        if (stats_direct) {
            HIP_TRY(wait_for_flag(s, &stats_host->n_used));
        } else {
            HIP_TRY(hipMemcpyAsync(stats_host, rec_dev, sizeof(bof4_lloyd_stats), hipMemcpyDeviceToHost, s));
            HIP_TRY(wait_for_stream(s));
        }
    }
    }
    if (!opq) {
        *n_outliers_host = 0;
        return BOF4_OK;
    }
    uint64_t head = 0;
    if (direct) {
        HIP_TRY(wait_for_flag(s, n_outliers_host));
        head = *n_outliers_host;
    } else {
        HIP_TRY(hipMemcpyAsync(&head, total_dev, 8, hipMemcpyDeviceToHost, s));
        HIP_TRY(wait_for_stream(s));
    }
    uint64_t tot = head & ~(1ull << 63);
    const bool staged_overflow = (head >> 63) != 0;
    if (staged_overflow && tot <= out_capacity) {
        // Some wave found more outliers than its staging region holds although the caller's buffers are large enough
        // (outliers piled up in one stretch of the tensor): redo the extraction with the general, slower kernel that
        // appends tile by tile through one global counter.
        QuantWsLayout L = quant_ws_layout(n, out_capacity);
        char* base = (char*)ws_dev;
        uint64_t* total = (uint64_t*)(base + L.header);
        uint32_t* tc = (uint32_t*)(base + L.tile_cnt);
        uint64_t* tb = (uint64_t*)(base + L.tile_base);
        uint64_t* to = (uint64_t*)(base + L.tile_off);
        int64_t* si = (int64_t*)(base + L.stage_idx);
        uint16_t* sv = (uint16_t*)(base + L.stage_val);
        hipLaunchKernelGGL(zero_u64_kernel, dim3(1), dim3(1), 0, s, total);
        const uint64_t n_vec = n / 8;
        dim3 grid((uint32_t)n_tiles);
        switch (block) {
            case 32: launch_quantize_i<32>(signed_norm != 0, true, grid, s, wv, n_vec, cb, T2, cd, scales_dev, total, tc, tb, si, sv, out_capacity); break;
            case 64: launch_quantize_i<64>(signed_norm != 0, true, grid, s, wv, n_vec, cb, T2, cd, scales_dev, total, tc, tb, si, sv, out_capacity); break;
            case 128: launch_quantize_i<128>(signed_norm != 0, true, grid, s, wv, n_vec, cb, T2, cd, scales_dev, total, tc, tb, si, sv, out_capacity); break;
            default: launch_quantize_i<256>(signed_norm != 0, true, grid, s, wv, n_vec, cb, T2, cd, scales_dev, total, tc, tb, si, sv, out_capacity); break;
        }
        hipLaunchKernelGGL(tile_scan_kernel, dim3(1), dim3(1024), 0, s, tc, n_tiles, to);
        hipLaunchKernelGGL(outlier_gather_kernel, dim3((uint32_t)((n_tiles + 255) / 256)), dim3(256), 0, s, tc, tb, to,
                           n_tiles, si, sv, out_idx_dev, out_val_dev, out_capacity);
        HIP_TRY(hipGetLastError());
        HIP_TRY(hipMemcpyAsync(&tot, total, 8, hipMemcpyDeviceToHost, s));
        HIP_TRY(wait_for_stream(s));
    }
    *n_outliers_host = tot;
    if (tot > out_capacity) return fail(BOF4_ERR_CAPACITY, "bof4_quantize: outlier buffers too small");
    return BOF4_OK;
}
}  // namespace

extern "C" {

int bof4_quantize(const void* w_dev, uint64_t n, uint32_t block, const double* cb_host, int signed_norm, double opq_T,
                  uint8_t* codes_dev, uint16_t* scales_dev, int64_t* out_idx_dev, uint16_t* out_val_dev,
                  uint64_t out_capacity, uint64_t* n_outliers_host, void* ws_dev, size_t ws_bytes, void* stream) {
    return quantize_impl(QUANT_WHOLE, w_dev, n, block, cb_host, signed_norm, opq_T, codes_dev, scales_dev, out_idx_dev,
                         out_val_dev, out_capacity, n_outliers_host, ws_dev, ws_bytes, stream);
}

int bof4_quantize_begin(const void* w_dev, uint64_t n, uint32_t block, const double* cb_host, int signed_norm,
                        double opq_T, uint8_t* codes_dev, uint16_t* scales_dev, int64_t* out_idx_dev,
                        uint16_t* out_val_dev, uint64_t out_capacity, uint64_t* n_outliers_host, void* ws_dev,
                        size_t ws_bytes, void* stream) {
    return quantize_impl(QUANT_ENQUEUE, w_dev, n, block, cb_host, signed_norm, opq_T, codes_dev, scales_dev,
                         out_idx_dev, out_val_dev, out_capacity, n_outliers_host, ws_dev, ws_bytes, stream);
}

int bof4_quantize_finish(const void* w_dev, uint64_t n, uint32_t block, const double* cb_host, int signed_norm,
                         double opq_T, uint8_t* codes_dev, uint16_t* scales_dev, int64_t* out_idx_dev,
                         uint16_t* out_val_dev, uint64_t out_capacity, uint64_t* n_outliers_host, void* ws_dev,
                         size_t ws_bytes, void* stream) {
    return quantize_impl(QUANT_COLLECT, w_dev, n, block, cb_host, signed_norm, opq_T, codes_dev, scales_dev,
                         out_idx_dev, out_val_dev, out_capacity, n_outliers_host, ws_dev, ws_bytes, stream);
}

int bof4_quantize_lloyd(const void* w_dev, uint64_t n, uint32_t block, const double* cb_host, int signed_norm,
                        double opq_T, int weight_by_max2, uint8_t* codes_dev, uint16_t* scales_dev,
                        int64_t* out_idx_dev, uint16_t* out_val_dev, uint64_t out_capacity, uint64_t* n_outliers_host,
                        bof4_lloyd_stats* stats_host, void* ws_dev, size_t ws_bytes, void* stream) {
    if (!stats_host) return fail(BOF4_ERR_ARG, "bof4_quantize_lloyd: null pointer");
    return quantize_impl(QUANT_WHOLE, w_dev, n, block, cb_host, signed_norm, opq_T, codes_dev, scales_dev, out_idx_dev,
                         out_val_dev, out_capacity, n_outliers_host, ws_dev, ws_bytes, stream, stats_host,
                         weight_by_max2);
}

int bof4_quantize_lloyd_begin(const void* w_dev, uint64_t n, uint32_t block, const double* cb_host, int signed_norm,
                              double opq_T, int weight_by_max2, uint8_t* codes_dev, uint16_t* scales_dev,
                              int64_t* out_idx_dev, uint16_t* out_val_dev, uint64_t out_capacity,
                              uint64_t* n_outliers_host, bof4_lloyd_stats* stats_host, void* ws_dev, size_t ws_bytes,
                              void* stream) {
    if (!stats_host) return fail(BOF4_ERR_ARG, "bof4_quantize_lloyd_begin: null pointer");
    return quantize_impl(QUANT_ENQUEUE, w_dev, n, block, cb_host, signed_norm, opq_T, codes_dev, scales_dev,
                         out_idx_dev, out_val_dev, out_capacity, n_outliers_host, ws_dev, ws_bytes, stream, stats_host,
                         weight_by_max2);
}

int bof4_quantize_lloyd_finish(const void* w_dev, uint64_t n, uint32_t block, const double* cb_host, int signed_norm,
                               double opq_T, int weight_by_max2, uint8_t* codes_dev, uint16_t* scales_dev,
                               int64_t* out_idx_dev, uint16_t* out_val_dev, uint64_t out_capacity,
                               uint64_t* n_outliers_host, bof4_lloyd_stats* stats_host, void* ws_dev, size_t ws_bytes,
                               void* stream) {
    if (!stats_host) return fail(BOF4_ERR_ARG, "bof4_quantize_lloyd_finish: null pointer");
    return quantize_impl(QUANT_COLLECT, w_dev, n, block, cb_host, signed_norm, opq_T, codes_dev, scales_dev,
                         out_idx_dev, out_val_dev, out_capacity, n_outliers_host, ws_dev, ws_bytes, stream, stats_host,
                         weight_by_max2);
}

int bof4_dequantize(const uint8_t* codes_dev, const uint16_t* scales_dev, uint64_t n, uint32_t block,
                    const double* cb_host, const int64_t* out_idx_dev, const uint16_t* out_val_dev,
                    uint64_t n_outliers, void* w_out_dev, void* stream) {
    if (!codes_dev || !scales_dev || !w_out_dev) return fail(BOF4_ERR_ARG, "bof4_dequantize: null pointer");
    if (!valid_block(block) || n == 0 || n % block != 0) return fail(BOF4_ERR_ARG, "bof4_dequantize: bad n or block");
    if (!valid_codebook(cb_host)) return fail(BOF4_ERR_ARG, "bof4_dequantize: codebook must be 16 finite ascending levels");
    if (n_outliers > 0 && (!out_idx_dev || !out_val_dev)) return fail(BOF4_ERR_ARG, "bof4_dequantize: null outlier buffers");
    if (!aligned(w_out_dev, 16) || !aligned(codes_dev, 4) || !aligned(scales_dev, 2) || !aligned(out_idx_dev, 8) ||
        !aligned(out_val_dev, 2))
        return fail(BOF4_ERR_ARG, "bof4_dequantize: misaligned pointer");
    hipStream_t s = (hipStream_t)stream;
    const uint64_t n_vec = n / 8;
    const uint64_t n_tiles = (n_vec + 256 * DEQ_VPT - 1) / (256 * DEQ_VPT);
    // DEQ_RESIDENT_WGS workgroups that each walk a run of tiles (what the chip holds at once: no second round)
    uint64_t tiles_per_wg = (n_tiles + DEQ_RESIDENT_WGS - 1) / DEQ_RESIDENT_WGS;
    const uint64_t nb = (n_tiles + tiles_per_wg - 1) / tiles_per_wg;
    if (nb > 0x7fffffffull || tiles_per_wg > 0xffffffffull)
        return fail(BOF4_ERR_ARG, "bof4_dequantize: n too large for one call");
    CodebookArgs cb = make_codebook_args(cb_host);
    dim3 grid((uint32_t)nb);
    // list entries a workgroup looks at per round: what a tile holds on average, rounded up to whole waves
    uint32_t window = 64;
    while (window < 256 && (double)window * (double)n_tiles < (double)n_outliers) window += 64;
    const uint32_t* codes = (const uint32_t*)codes_dev;
    uint4* out = (uint4*)w_out_dev;
    timing_begin(s);
#define BOF4_LAUNCH_DEQ(I_)                                                                                  \
    hipLaunchKernelGGL((dequantize_kernel<I_>), grid, dim3(256), 0, s, codes, scales_dev, n_vec,             \
                       (uint32_t)tiles_per_wg, window, cb, out_idx_dev, out_val_dev, n_outliers, out);
    switch (block) {
        case 32: BOF4_LAUNCH_DEQ(32) break;
        case 64: BOF4_LAUNCH_DEQ(64) break;
        case 128: BOF4_LAUNCH_DEQ(128) break;
        default: BOF4_LAUNCH_DEQ(256) break;
    }
#undef BOF4_LAUNCH_DEQ
    timing_end(s);
    HIP_TRY(hipGetLastError());
    return BOF4_OK;
}

// Workgroups of one bof4_gemv kernel variant that the current device holds at once (cached per variant, workgroup
// size and dynamic LDS; 0 on failure).
uint64_t gemv_resident_workgroups(int variant, uint32_t threads, size_t lds) {
    struct Key {
        int device, variant;
        uint32_t threads;
        size_t lds;
        uint64_t slots;
    };
    static thread_local Key cache[8] = {};
    static thread_local int next = 0;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    for (const Key& k : cache)
        if (k.slots && k.device == dev && k.variant == variant && k.threads == threads && k.lds == lds) return k.slots;
    int per_cu = 0, cus = 0;
    hipError_t e;
    switch (variant) {
        case 0: e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, gemv_kernel<1, false>, (int)threads, lds); break;
        case 1: e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, gemv_kernel<1, true>, (int)threads, lds); break;
        case 2: e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, gemv_kernel<2, false>, (int)threads, lds); break;
        default: e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, gemv_kernel<2, true>, (int)threads, lds); break;
    }
    if (e != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
        return 0;
    if (per_cu < 1) per_cu = 1;
    Key& slot = cache[next];
    next = (next + 1) % 8;
    slot = Key{dev, variant, threads, lds, (uint64_t)per_cu * (uint64_t)cus};
    return slot.slots;
}

// Outlier table of bof4_gemv: offsets [rows * strips + 1] (padded to 8 bytes), then one {column, delta} pair per entry.
struct GemvTableLayout {
    size_t entries, total;
};
GemvTableLayout gemv_table_layout(uint64_t rows, uint64_t strips, uint64_t n_outliers) {
    GemvTableLayout L;
    L.entries = align_up((rows * strips + 1) * 4, 8);
    L.total = L.entries + n_outliers * 8;
    return L;
}

size_t bof4_gemv_outlier_table_bytes(uint64_t rows, uint64_t cols, uint64_t n_outliers) {
    if (rows == 0 || cols == 0) return 0;
    return gemv_table_layout(rows, (cols + GEMV_STRIP - 1) / GEMV_STRIP, n_outliers).total;
}

}  // extern "C"

namespace {
// rounded = false: the entries of bof4_gemv (value - m * level); true: those of bof4_gemm (both terms in bfloat16).
int outlier_table_impl(bool rounded, const uint8_t* codes_dev, const uint16_t* scales_dev, uint64_t rows,
                       uint64_t cols, uint32_t block, const double* cb_host, const int64_t* out_idx_dev,
                       const uint16_t* out_val_dev, uint64_t n_outliers, void* table_dev, size_t table_bytes,
                       void* stream) {
    if (!codes_dev || !scales_dev || !table_dev || (n_outliers > 0 && (!out_idx_dev || !out_val_dev)))
        return fail(BOF4_ERR_ARG, "outlier table: null pointer");
    if (!valid_block(block) || rows == 0 || cols == 0 || cols % block != 0)
        return fail(BOF4_ERR_ARG, "outlier table: bad rows, cols (a positive multiple of block) or block");
    const uint64_t strips = (cols + GEMV_STRIP - 1) / GEMV_STRIP;
    if (rows > 0xfffffffeull || strips > GEMV_MAX_STRIPS || n_outliers > 0xffffffffull)
        return fail(BOF4_ERR_ARG, "outlier table: rows and the list length must fit 32 bits, cols <= 32768");
    if (!valid_codebook(cb_host))
        return fail(BOF4_ERR_ARG, "outlier table: codebook must be 16 finite ascending levels");
    if (!aligned(out_idx_dev, 8) || !aligned(out_val_dev, 2) || !aligned(scales_dev, 2) || !aligned(table_dev, 8))
        return fail(BOF4_ERR_ARG, "outlier table: misaligned pointer (the table needs 8 bytes)");
    const GemvTableLayout L = gemv_table_layout(rows, strips, n_outliers);
    if (table_bytes < L.total) return fail(BOF4_ERR_WORKSPACE, "outlier table: table buffer too small");
    hipStream_t s = (hipStream_t)stream;
    const CodebookArgs cb = make_codebook_args(cb_host);
    uint32_t log2_block = 5;
    while ((1u << log2_block) < block) ++log2_block;
    const uint64_t count = rows * strips + 1;
    hipLaunchKernelGGL(outlier_strip_offsets_kernel, dim3((uint32_t)((count + 255) / 256)), dim3(256), 0, s,
                       out_idx_dev, (uint32_t)n_outliers, rows, cols, (uint32_t)strips, (uint32_t*)table_dev);
    if (n_outliers > 0)
        hipLaunchKernelGGL(outlier_delta_kernel, dim3((uint32_t)((n_outliers + 255) / 256)), dim3(256), 0, s,
                           codes_dev, scales_dev, rows * cols, cols, log2_block, cb, out_idx_dev, out_val_dev,
                           (uint32_t)n_outliers, rounded ? 1u : 0u, (uint2*)((char*)table_dev + L.entries));
    HIP_TRY(hipGetLastError());
    return BOF4_OK;
}

// Tiles of 32 rows per wave: with two, every word of x read serves 64 rows, at twice the accumulators.  Measured
// better for more than 32 tokens on all but small matrices, and for very large ones at any number of tokens.
uint32_t gemm_row_tiles_per_wg(uint64_t rows, uint64_t cols, uint64_t n_tokens) {
    return ((n_tokens > GEMM_TOKENS && (rows >= 8192 || cols >= 8192)) || rows * cols >= (1ull << 27)) ? 2 : 1;
}
uint64_t gemm_row_tiles(uint64_t rows) {  // in the packed matrix: a multiple of GEMM_MAX_R
    return (rows + GEMM_ROWS * GEMM_MAX_R - 1) / (GEMM_ROWS * GEMM_MAX_R) * GEMM_MAX_R;
}
// How many workgroups share the columns of their rows: the fewest that put GEMM_TARGET_WGS workgroups on the chip,
// each with at least one chunk per wave.
uint32_t gemm_split(uint64_t rows, uint64_t cols, uint64_t n_tokens) {
    const uint64_t groups = gemm_row_tiles(rows) / gemm_row_tiles_per_wg(rows, cols, n_tokens);
    const uint64_t chunks = (cols + GEMM_CHUNK - 1) / GEMM_CHUNK;
    uint64_t split = (GEMM_TARGET_WGS + groups - 1) / groups;
    const uint64_t most = chunks / GEMM_MAX_WAVES;
    if (split > most) split = most;
    return (uint32_t)(split < 1 ? 1 : split);
}

// Workspace of bof4_gemm: x in the order of the products, x transposed (for the list), the partial results.
constexpr uint32_t GEMM_MAX_TOKENS = 65536;
struct GemmWsLayout {
    size_t xp, xt, part, total;
};
GemmWsLayout gemm_ws_layout(uint64_t rows, uint64_t cols, uint64_t n_tokens) {
    const uint64_t n_pad = (n_tokens + GEMM_TOKENS - 1) / GEMM_TOKENS * GEMM_TOKENS;
    const uint64_t chunks = (cols + GEMM_CHUNK - 1) / GEMM_CHUNK, split = gemm_split(rows, cols, n_tokens);
    const uint64_t per_launch = n_pad < GEMM_TOKENS * GEMM_MAX_TILES ? n_pad : GEMM_TOKENS * GEMM_MAX_TILES;
    GemmWsLayout L;
    L.xp = 0;
    L.xt = align_up(L.xp + n_pad * chunks * GEMM_CHUNK * 2, 256);
    L.part = align_up(L.xt + cols * n_pad * 2, 256);
    L.total = L.part + (split > 1 ? split * per_launch * rows * 4 : 0);
    return L;
}
}  // namespace

extern "C" {

int bof4_gemv_outlier_table(const uint8_t* codes_dev, const uint16_t* scales_dev, uint64_t rows, uint64_t cols,
                            uint32_t block, const double* cb_host, const int64_t* out_idx_dev,
                            const uint16_t* out_val_dev, uint64_t n_outliers, void* table_dev, size_t table_bytes,
                            void* stream) {
    return outlier_table_impl(false, codes_dev, scales_dev, rows, cols, block, cb_host, out_idx_dev, out_val_dev,
                              n_outliers, table_dev, table_bytes, stream);
}

int bof4_gemm_outlier_table(const uint8_t* codes_dev, const uint16_t* scales_dev, uint64_t rows, uint64_t cols,
                            uint32_t block, const double* cb_host, const int64_t* out_idx_dev,
                            const uint16_t* out_val_dev, uint64_t n_outliers, void* table_dev, size_t table_bytes,
                            void* stream) {
    return outlier_table_impl(true, codes_dev, scales_dev, rows, cols, block, cb_host, out_idx_dev, out_val_dev,
                              n_outliers, table_dev, table_bytes, stream);
}

size_t bof4_gemm_workspace_bytes(uint64_t rows, uint64_t cols, uint32_t n_tokens) {
    if (rows == 0 || cols == 0 || n_tokens == 0) return 0;
    return gemm_ws_layout(rows, cols, n_tokens).total;
}

size_t bof4_gemm_packed_bytes(uint64_t rows, uint64_t cols) {
    return (size_t)(gemm_row_tiles(rows) * ((cols + GEMM_CHUNK - 1) / GEMM_CHUNK) * GEMM_TILE_BYTES);
}

int bof4_gemm_pack(const uint8_t* codes_dev, const uint16_t* scales_dev, uint64_t rows, uint64_t cols, uint32_t block,
                   void* packed_dev, size_t packed_bytes, void* stream) {
    if (!codes_dev || !scales_dev || !packed_dev) return fail(BOF4_ERR_ARG, "bof4_gemm_pack: null pointer");
    if (!valid_block(block) || rows == 0 || cols == 0 || cols % block != 0)
        return fail(BOF4_ERR_ARG, "bof4_gemm_pack: bad rows, cols (a positive multiple of block) or block");
    if (rows > 0xfffffffeull || cols > GEMV_MAX_STRIPS * GEMV_STRIP)
        return fail(BOF4_ERR_ARG, "bof4_gemm_pack: at most 2^32 - 2 rows and 32768 columns");
    if (!aligned(codes_dev, 16) || !aligned(scales_dev, 2) || !aligned(packed_dev, 16))
        return fail(BOF4_ERR_ARG, "bof4_gemm_pack: misaligned pointer (codes and the packed copy need 16 bytes)");
    if (packed_bytes < bof4_gemm_packed_bytes(rows, cols))
        return fail(BOF4_ERR_WORKSPACE, "bof4_gemm_pack: buffer for the packed copy too small");
    uint32_t log2_block = 5;
    while ((1u << log2_block) < block) ++log2_block;
    const uint32_t chunks = (uint32_t)((cols + GEMM_CHUNK - 1) / GEMM_CHUNK);
    const uint64_t n_tiles = gemm_row_tiles(rows) * chunks;
    hipLaunchKernelGGL(gemm_pack_weights_kernel, dim3((uint32_t)((n_tiles * 64 + 255) / 256)), dim3(256), 0,
                       (hipStream_t)stream, (const uint4*)codes_dev, scales_dev, (uint32_t)rows, (uint32_t)cols,
                       log2_block, chunks, n_tiles, (char*)packed_dev);
    HIP_TRY(hipGetLastError());
    return BOF4_OK;
}

int bof4_gemm(const void* packed_dev, uint64_t rows, uint64_t cols, const double* cb_host, const void* table_dev,
              uint64_t n_outliers, const void* x_dev, uint32_t n_tokens, float* y_dev, void* ws_dev, size_t ws_bytes,
              void* stream) {
    if (!packed_dev || !x_dev || !y_dev || !ws_dev) return fail(BOF4_ERR_ARG, "bof4_gemm: null pointer");
    if (rows == 0 || cols == 0 || cols % 32 != 0 || n_tokens == 0)
        return fail(BOF4_ERR_ARG, "bof4_gemm: bad rows, cols (a positive multiple of 32) or n_tokens");
    const uint64_t strips = (cols + GEMV_STRIP - 1) / GEMV_STRIP;
    if (rows > 0xfffffffeull || strips > GEMV_MAX_STRIPS || n_tokens > GEMM_MAX_TOKENS)
        return fail(BOF4_ERR_ARG, "bof4_gemm: at most 2^32 - 2 rows, 32768 columns and 65536 tokens");
    if (!valid_codebook(cb_host)) return fail(BOF4_ERR_ARG, "bof4_gemm: codebook must be 16 finite ascending levels");
    if (n_outliers > 0 && !table_dev) return fail(BOF4_ERR_ARG, "bof4_gemm: outliers without their table");
    if (n_outliers > 0xffffffffull) return fail(BOF4_ERR_ARG, "bof4_gemm: more than 2^32 - 1 outliers");
    if (!aligned(packed_dev, 16) || !aligned(x_dev, 16) || !aligned(y_dev, 4) || !aligned(table_dev, 8) ||
        !aligned(ws_dev, 256))
        return fail(BOF4_ERR_ARG, "bof4_gemm: misaligned pointer (packed matrix and x need 16 bytes, the table 8, the workspace 256)");
    const GemmWsLayout L = gemm_ws_layout(rows, cols, n_tokens);
    if (ws_bytes < L.total) return fail(BOF4_ERR_WORKSPACE, "bof4_gemm: workspace too small");
    const uint32_t* offsets_dev = (const uint32_t*)table_dev;
    const uint2* entries_dev =
        table_dev ? (const uint2*)((const char*)table_dev + gemv_table_layout(rows, strips, n_outliers).entries) : nullptr;
    hipStream_t s = (hipStream_t)stream;
    const CodebookArgs cb = make_codebook_args(cb_host);
    const uint32_t split = gemm_split(rows, cols, n_tokens);
    const uint32_t chunks = (uint32_t)((cols + GEMM_CHUNK - 1) / GEMM_CHUNK), per_wg = (chunks + split - 1) / split;
    const uint32_t waves = per_wg < GEMM_MAX_WAVES ? per_wg : GEMM_MAX_WAVES;
    const uint32_t per_wg_tiles = gemm_row_tiles_per_wg(rows, cols, n_tokens);
    const uint32_t row_groups = (uint32_t)(gemm_row_tiles(rows) / per_wg_tiles);
    const uint32_t n_pad = (n_tokens + GEMM_TOKENS - 1) / GEMM_TOKENS * GEMM_TOKENS, tok_tiles = n_pad / GEMM_TOKENS;
    const uint4* xp = (const uint4*)((char*)ws_dev + L.xp);
    const uint16_t* xt = (const uint16_t*)((char*)ws_dev + L.xt);
    float* part = (float*)((char*)ws_dev + L.part);
    {
        const uint64_t total = (uint64_t)tok_tiles * chunks * 256;
        hipLaunchKernelGGL(gemm_pack_x_kernel, dim3((uint32_t)((total + 255) / 256)), dim3(256), 0, s,
                           (const uint16_t*)x_dev, n_tokens, (uint32_t)cols, chunks, n_pad, (uint4*)xp,
                           n_outliers > 0 ? (uint16_t*)xt : nullptr);
    }
    timing_begin(s);
    for (uint32_t tile0 = 0; tile0 < tok_tiles;) {
        const uint32_t left = tok_tiles - tile0, nt_tiles = left >= 4 ? 4 : left;
        const uint32_t t0 = tile0 * GEMM_TOKENS;
        const uint32_t nt = n_tokens - t0 < nt_tiles * GEMM_TOKENS ? n_tokens - t0 : nt_tiles * GEMM_TOKENS;
        float* yt = y_dev + (uint64_t)t0 * rows;
        float* dst = split > 1 ? part : yt;
#define BOF4_LAUNCH_GEMM(R_, NT_, OUT_)                                                                           \
    hipLaunchKernelGGL((gemm_kernel<R_, NT_, OUT_>), dim3(row_groups, split), dim3(64 * waves), 0, s,             \
                       (const char*)packed_dev, (uint32_t)rows, (uint32_t)cols, cb, offsets_dev, entries_dev,     \
                       (uint32_t)n_outliers, (uint32_t)strips, xp, xt, n_pad, tile0, nt, dst);
#define BOF4_LAUNCH_GEMM_NT(R_, OUT_)                                                                             \
    if (nt_tiles == 4) { BOF4_LAUNCH_GEMM(R_, 4, OUT_) } else if (nt_tiles == 3) { BOF4_LAUNCH_GEMM(R_, 3, OUT_) } \
    else if (nt_tiles == 2) { BOF4_LAUNCH_GEMM(R_, 2, OUT_) } else { BOF4_LAUNCH_GEMM(R_, 1, OUT_) }
        if (n_outliers > 0) {
            if (per_wg_tiles == 2) { BOF4_LAUNCH_GEMM_NT(2, true) } else { BOF4_LAUNCH_GEMM_NT(1, true) }
        } else {
            if (per_wg_tiles == 2) { BOF4_LAUNCH_GEMM_NT(2, false) } else { BOF4_LAUNCH_GEMM_NT(1, false) }
        }
#undef BOF4_LAUNCH_GEMM_NT
#undef BOF4_LAUNCH_GEMM
        if (split > 1) {
            const uint64_t count = (uint64_t)nt * rows;
            hipLaunchKernelGGL(gemm_sum_kernel, dim3((uint32_t)((count + 255) / 256)), dim3(256), 0, s, part, split,
                               count, yt);
        }
        tile0 += nt_tiles;
    }
    timing_end(s);
    HIP_TRY(hipGetLastError());
    return BOF4_OK;
}

int bof4_gemv(const uint8_t* codes_dev, const uint16_t* scales_dev, uint64_t rows, uint64_t cols, uint32_t block,
              const double* cb_host, const void* table_dev, uint64_t n_outliers, const void* x_dev,
              uint32_t n_tokens, float* y_dev, void* stream) {
    if (!codes_dev || !scales_dev || !x_dev || !y_dev) return fail(BOF4_ERR_ARG, "bof4_gemv: null pointer");
    if (!valid_block(block) || rows == 0 || cols == 0 || cols % block != 0 || n_tokens == 0)
        return fail(BOF4_ERR_ARG, "bof4_gemv: bad rows, cols (a positive multiple of block), block or n_tokens");
    const uint64_t strips = (cols + GEMV_STRIP - 1) / GEMV_STRIP;
    if (rows > 0xfffffffeull || strips > GEMV_MAX_STRIPS)
        return fail(BOF4_ERR_ARG, "bof4_gemv: at most 2^32 - 2 rows and 32768 columns");
    if (!valid_codebook(cb_host)) return fail(BOF4_ERR_ARG, "bof4_gemv: codebook must be 16 finite ascending levels");
    if (n_outliers > 0 && !table_dev) return fail(BOF4_ERR_ARG, "bof4_gemv: outliers without their table");
    if (n_outliers > 0xffffffffull) return fail(BOF4_ERR_ARG, "bof4_gemv: more than 2^32 - 1 outliers");
    if (!aligned(codes_dev, 16) || !aligned(x_dev, 16) || !aligned(scales_dev, 2) || !aligned(y_dev, 4) ||
        !aligned(table_dev, 8))
        return fail(BOF4_ERR_ARG, "bof4_gemv: misaligned pointer (codes and x need 16 bytes, the table 8)");
    const uint32_t* offsets_dev = (const uint32_t*)table_dev;
    const uint2* entries_dev =
        table_dev ? (const uint2*)((const char*)table_dev + gemv_table_layout(rows, strips, n_outliers).entries) : nullptr;
    hipStream_t s = (hipStream_t)stream;
    const CodebookArgs cb = make_codebook_args(cb_host);
    uint32_t log2_block = 5;
    while ((1u << log2_block) < block) ++log2_block;
    const uint4* codes = (const uint4*)codes_dev;
    const uint16_t* x = (const uint16_t*)x_dev;
    timing_begin(s);
    for (uint32_t t0 = 0; t0 < n_tokens; t0 += GEMV_MAX_TOKENS) {
        const uint32_t nt = n_tokens - t0 < GEMV_MAX_TOKENS ? n_tokens - t0 : GEMV_MAX_TOKENS;
        const uint16_t* xt = x + (uint64_t)t0 * cols;
        float* yt = y_dev + (uint64_t)t0 * rows;
        // with a list every wave keeps its slice of x in LDS as well
        const uint32_t waves = (uint32_t)(strips < GEMV_MAX_WAVES ? strips : GEMV_MAX_WAVES);
        const size_t lds = n_outliers > 0 ? (size_t)waves * GEMV_STRIP * 2 * nt : 0;
        // Rows per workgroup: every workgroup pays for its slice of x, the level table and two barriers, so the
        // rows are dealt out evenly over as many workgroups as the chip holds at once - one round, no tail.
        const int variant = (nt == 1 ? 0 : 2) + (n_outliers > 0 ? 1 : 0);
        const uint64_t slots = gemv_resident_workgroups(variant, 64 * waves, lds);
        if (slots == 0) return fail(BOF4_ERR_HIP, "bof4_gemv: occupancy query failed");
        uint64_t rc64 = (rows + slots - 1) / slots;
        const uint32_t rc = (uint32_t)(rc64 < 4 ? 4 : rc64 > GEMV_MAX_RC ? GEMV_MAX_RC : rc64);
        const uint32_t grid = (uint32_t)((rows + rc - 1) / rc);
#define BOF4_LAUNCH_GEMV(T_, OUT_)                                                                                \
    hipLaunchKernelGGL((gemv_kernel<T_, OUT_>), dim3(grid), dim3(64 * waves), lds, s, codes, scales_dev,          \
                       (uint32_t)rows, (uint32_t)cols, log2_block, rc, (uint32_t)strips, cb, offsets_dev,         \
                       entries_dev, (uint32_t)n_outliers, xt, yt);
        if (n_outliers > 0) {
            if (nt == 1) { BOF4_LAUNCH_GEMV(1, true) } else { BOF4_LAUNCH_GEMV(2, true) }
        } else {
            if (nt == 1) { BOF4_LAUNCH_GEMV(1, false) } else { BOF4_LAUNCH_GEMV(2, false) }
        }
#undef BOF4_LAUNCH_GEMV
    }
    timing_end(s);
    HIP_TRY(hipGetLastError());
    return BOF4_OK;
}

}  // extern "C"

// Workspace of bof4_lloyd_step_static: device memory that comes with the library's code object instead of a
// caller's buffer, for callers that cannot allocate.  Every GPU holds its own copy at its own address; host code
// must not use the array's name as an address (it is only a handle for hipGetSymbolAddress).
constexpr size_t STATIC_SCRATCH_BYTES = ((size_t)1024 + 1) * 56 * 8;  // = lloyd_ws_bytes(): one record per workgroup + result
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

namespace {
static_assert(STATIC_SCRATCH_BYTES == ((size_t)PASS_GRID_MAX + 1) * LLOYD_PART * 8, "scratch must hold the Lloyd workspace");
// Address of `scratch` on the current device, looked up once per device with that device current.
constexpr int STATIC_MAX_DEVICES = 64;
std::atomic<void*> g_scratch_ptr[STATIC_MAX_DEVICES];
int static_scratch(void** out) {
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= STATIC_MAX_DEVICES) return fail(BOF4_ERR_ARG, "bof4_lloyd_step_static: device index above 63");
    void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(BOF4_ERR_HIP, "bof4_lloyd_step_static: no address for the scratch array");
        g_scratch_ptr[dev].store(p, std::memory_order_release);  // every thread finds the same address
    }
    *out = p;
    return BOF4_OK;
}

// wait = false: enqueue only; the record must lie in pinned host memory, where bof4_wait_result finds it.
int lloyd_step_impl(bool wait, const void* w_dev, uint64_t n, uint32_t block, const double* cb_host, int signed_norm,
                    double opq_T, int weight_by_max2, bof4_lloyd_stats* out_host, void* ws_dev, size_t ws_bytes,
                    void* stream) {
    if (!w_dev || !out_host) return fail(BOF4_ERR_ARG, "bof4_lloyd_step: null pointer");
    if (!valid_block(block) || n == 0 || n % block != 0) return fail(BOF4_ERR_ARG, "bof4_lloyd_step: bad n or block");
    if (!valid_codebook(cb_host)) return fail(BOF4_ERR_ARG, "bof4_lloyd_step: codebook must be 16 finite ascending levels");
    if (!(opq_T >= 0.0) || !std::isfinite(opq_T)) return fail(BOF4_ERR_ARG, "bof4_lloyd_step: opq_T must be finite and >= 0");
    if (!aligned(w_dev, 16)) return fail(BOF4_ERR_ARG, "bof4_lloyd_step: misaligned weights");
    if (!ws_dev || !aligned(ws_dev, 256)) return fail(BOF4_ERR_ARG, "bof4_lloyd_step: workspace null or misaligned");
    if (ws_bytes < lloyd_ws_bytes()) return fail(BOF4_ERR_WORKSPACE, "bof4_lloyd_step: workspace too small");
    hipStream_t s = (hipStream_t)stream;
    const uint32_t seg = block < 64 ? block : 64;
    const uint64_t n_seg = n / seg;
    CodebookArgs cb = make_codebook_args(cb_host);
    double* partials = (double*)ws_dev;
    const double T2 = opq_T * opq_T;
    const bool opq = opq_T > 0.0;
    const uint4* w = (const uint4*)w_dev;
    // If the caller's struct lies in pinned (device-visible) host memory the final kernel writes it in place;
    // otherwise the record goes through the workspace and one copy.
    double* direct = (double*)device_view_of_host(out_host);
    if (!wait && !direct)
        return fail(BOF4_ERR_ARG, "bof4_lloyd_step_begin: the record must lie in pinned host memory");
    {
        BinTable bt = make_bin_table(cb);
        const OutlierStage no_stage = {nullptr, nullptr, nullptr, 0};
        const PassArgs pa = {w, n_seg, cb, bt, signed_norm, weight_by_max2, T2, nullptr, nullptr, no_stage, partials};
        timing_begin(s);
        const uint32_t n_part = launch_pass<false, true>(block, opq, s, pa);  // one partial record per workgroup
        timing_end(s);
        // The result record has the layout of bof4_lloyd_stats.
        static_assert(sizeof(bof4_lloyd_stats) == 51 * 8, "result record and bof4_lloyd_stats must match");
        double* rec_dev = partials + (uint64_t)n_part * LLOYD_PART;
        if (direct) out_host->n_used = FLAG_PENDING;  // the word the final kernel writes last
        hipLaunchKernelGGL(seg_lloyd_final_kernel, dim3(1), dim3(1024), 0, s, partials, n_part, cb, bt.code_of_zero,
                           direct ? direct : rec_dev);
        HIP_TRY(hipGetLastError());
        if (!wait) return BOF4_OK;
        if (direct) {
            HIP_TRY(wait_for_flag(s, &out_host->n_used));
        } else {
            HIP_TRY(hipMemcpyAsync(out_host, rec_dev, sizeof(bof4_lloyd_stats), hipMemcpyDeviceToHost, s));
            HIP_TRY(wait_for_stream(s));
        }
    }
    return BOF4_OK;
}
}  // namespace

extern "C" {

int bof4_lloyd_step(const void* w_dev, uint64_t n, uint32_t block, const double* cb_host, int signed_norm,
                    double opq_T, int weight_by_max2, bof4_lloyd_stats* out_host, void* ws_dev, size_t ws_bytes,
                    void* stream) {
    return lloyd_step_impl(true, w_dev, n, block, cb_host, signed_norm, opq_T, weight_by_max2, out_host, ws_dev,
                           ws_bytes, stream);
}

int bof4_lloyd_step_begin(const void* w_dev, uint64_t n, uint32_t block, const double* cb_host, int signed_norm,
                          double opq_T, int weight_by_max2, bof4_lloyd_stats* out_host, void* ws_dev, size_t ws_bytes,
                          void* stream) {
    return lloyd_step_impl(false, w_dev, n, block, cb_host, signed_norm, opq_T, weight_by_max2, out_host, ws_dev,
                           ws_bytes, stream);
}

int bof4_lloyd_step_static(const void* w_dev, uint64_t n, uint32_t block, const double* cb_host, int signed_norm,
                           double opq_T, int weight_by_max2, bof4_lloyd_stats* out_host, void* stream) {
    if (n > BOF4_STATIC_MAX_N)
        return fail(BOF4_ERR_ARG, "bof4_lloyd_step_static: n exceeds BOF4_STATIC_MAX_N (2^36 weights)");
    if (!out_host || !device_view_of_host(out_host))
        return fail(BOF4_ERR_ARG, "bof4_lloyd_step_static: the record must lie in pinned host memory");
    void* ws = nullptr;
    const int rc = static_scratch(&ws);
    if (rc != BOF4_OK) return rc;
    return lloyd_step_impl(true, w_dev, n, block, cb_host, signed_norm, opq_T, weight_by_max2, out_host, ws,
                           STATIC_SCRATCH_BYTES, stream);
}

int bof4_wait_result(const uint64_t* word_host, void* stream) {
    if (!word_host) return fail(BOF4_ERR_ARG, "bof4_wait_result: null pointer");
    HIP_TRY(wait_for_flag((hipStream_t)stream, word_host));
    return BOF4_OK;
}

int bof4_codebook_update_mae(const bof4_mae_stats* st, uint16_t pinned_mask, double* cb_host) {
    if (!st || !cb_host) return fail(BOF4_ERR_ARG, "bof4_codebook_update_mae: null pointer");
    for (int l = 0; l < 16; ++l) {
        if ((pinned_mask >> l) & 1u) continue;
        if (st->median[l] == st->median[l]) cb_host[l] = st->median[l];
    }
    return BOF4_OK;
}

int bof4_lloyd_step_mae(const void* w_dev, uint64_t n, uint32_t block, const double* cb_host, int signed_norm,
                        double opq_T, int weight_by_max, uint16_t skip_mask, bof4_mae_stats* out_host, void* ws_dev,
                        size_t ws_bytes, void* stream) {
    if (!w_dev || !out_host) return fail(BOF4_ERR_ARG, "bof4_lloyd_step_mae: null pointer");
    if (!valid_block(block) || n == 0 || n % block != 0) return fail(BOF4_ERR_ARG, "bof4_lloyd_step_mae: bad n or block");
    if (!valid_codebook(cb_host)) return fail(BOF4_ERR_ARG, "bof4_lloyd_step_mae: codebook must be 16 finite ascending levels");
    if (!(opq_T >= 0.0) || !std::isfinite(opq_T)) return fail(BOF4_ERR_ARG, "bof4_lloyd_step_mae: opq_T must be finite and >= 0");
    if (!aligned(w_dev, 16)) return fail(BOF4_ERR_ARG, "bof4_lloyd_step_mae: misaligned pointer");
    if (!ws_dev || !aligned(ws_dev, 256)) return fail(BOF4_ERR_ARG, "bof4_lloyd_step_mae: workspace null or misaligned");
    const MaeWsLayout ML = mae_ws_layout(n);
    if (ws_bytes < ML.total) return fail(BOF4_ERR_WORKSPACE, "bof4_lloyd_step_mae: workspace too small");
    static_assert(sizeof(bof4_mae_stats) == MAE_REC * 8, "result record and bof4_mae_stats must match");
    hipStream_t s = (hipStream_t)stream;
    const CodebookArgs cb = make_codebook_args(cb_host);
    const BinTable bt = make_bin_table(cb);
    // Key range of every region.  A normalised weight lies in [-1, 1], up to 1.5 in magnitude when the block constant
    // is a binary16 subnormal; region l holds thr[l-1] < x <= thr[l].
    MaeLevelConst lc;
    uint32_t passes = 1;
    for (int l = 0; l < 16; ++l) {
        const float lower = l == 0 ? -2.0f : std::nextafterf(cb.thr[l - 1], INFINITY);
        const float upper = l == 15 ? 2.0f : cb.thr[l];
        const uint32_t klo = host_order_key(lower), khi = host_order_key(upper);
        uint32_t bits = 1;
        if (khi > klo)
            while (bits < 32 && ((uint64_t)(khi - klo) >> bits) != 0) ++bits;
        if (bits > 31) return fail(BOF4_ERR_ARG, "bof4_lloyd_step_mae: a region spans more than 2^31 binary32 values");
        lc.klo[l] = klo;
        lc.bits[l] = bits;
        if (!((skip_mask >> l) & 1u) && (bits + 7) / 8 > passes) passes = (bits + 7) / 8;
    }
    char* base = (char*)ws_dev;
    unsigned long long* hist = (unsigned long long*)(base + ML.hist);
    MaeLevelState* state = (MaeLevelState*)(base + ML.state);
    unsigned long long* cnt_part = (unsigned long long*)(base + ML.cnt_part);
    double* sae_part = (double*)(base + ML.sae_part);
    double* rec_dev = (double*)(base + ML.record);
    const bool opq = opq_T > 0.0;
    const int unweighted = weight_by_max ? 0 : 1;
    const double T2 = opq_T * opq_T;
    const uint32_t seg = block < 64 ? block : 64;
    const uint64_t n_seg = n / seg;
    const uint64_t tiles = (n_seg + 63) / 64;
    const uint64_t wantg = (tiles + WAVES_PER_WG - 1) / WAVES_PER_WG;
    const uint32_t sgrid = (uint32_t)(wantg < SEG_GRID ? wantg : SEG_GRID);
    const uint4* w = (const uint4*)w_dev;
    double* direct = (double*)device_view_of_host(out_host);
    if (direct) out_host->n_used = FLAG_PENDING;  // the word the last kernel writes last
    // The candidate list: written by the second pass, read by the passes after it.  Not used when there is no third
    // pass, when a wave's stretch would be tiny, or when zeroed outliers run through the search of the region around
    // zero (they are taken out again by a negative weight, which an entry cannot carry).
    uint32_t* cand_count = (uint32_t*)(base + ML.cand_count);
    uint32_t* cand_full = (uint32_t*)(base + ML.cand_full);
    unsigned long long* cand = (unsigned long long*)(base + ML.cand);
    const uint32_t cand_waves = sgrid * WAVES_PER_WG;
    const uint32_t cand_cap = (uint32_t)(mae_cand_entries(n) / cand_waves);
    const bool zero_region_searched = !((skip_mask >> bt.code_of_zero) & 1u);
    const bool use_list = passes >= 3 && cand_cap >= 8 && !(opq && zero_region_searched);
    // One pass over all the weights instead of two (large tensors): a sampling pass over one tile in 16 tells the full
    // first pass which first digits to write to the list (bof4_mae.h).
    const bool sampling = use_list && tiles >= MAE_SAMPLING_MIN_TILES && std::getenv("BOF4_MAE_NO_SAMPLING") == nullptr;
    hipLaunchKernelGGL(mae_init_kernel, dim3(16), dim3(256), 0, s, lc, state, hist);
#define BOF4_LAUNCH_MAE(II, FIRST_, CAPTURE_, CAND_, GATE_, SAMPLE_)                                                  \
    if (bt.fast && opq) hipLaunchKernelGGL((mae_pass_kernel<II, true, true, FIRST_, CAPTURE_>), dim3(sgrid), dim3(256), \
                                           0, s, w, n_seg, cb, bt, signed_norm, T2, state, hist, cnt_part, sae_part,  \
                                           CAND_, cand_count, cand_cap, GATE_, unweighted, SAMPLE_);                  \
    else if (bt.fast) hipLaunchKernelGGL((mae_pass_kernel<II, true, false, FIRST_, CAPTURE_>), dim3(sgrid), dim3(256),  \
                                         0, s, w, n_seg, cb, bt, signed_norm, T2, state, hist, cnt_part, sae_part,    \
                                         CAND_, cand_count, cand_cap, GATE_, unweighted, SAMPLE_);                    \
    else if (opq) hipLaunchKernelGGL((mae_pass_kernel<II, false, true, FIRST_, CAPTURE_>), dim3(sgrid), dim3(256), 0,   \
                                     s, w, n_seg, cb, bt, signed_norm, T2, state, hist, cnt_part, sae_part, CAND_,    \
                                     cand_count, cand_cap, GATE_, unweighted, SAMPLE_);                               \
    else hipLaunchKernelGGL((mae_pass_kernel<II, false, false, FIRST_, CAPTURE_>), dim3(sgrid), dim3(256), 0, s, w,     \
                            n_seg, cb, bt, signed_norm, T2, state, hist, cnt_part, sae_part, CAND_, cand_count,       \
                            cand_cap, GATE_, unweighted, SAMPLE_);
#define BOF4_LAUNCH_MAE_BLOCK(FIRST_, CAPTURE_, CAND_, GATE_, SAMPLE_)                 \
    switch (block) {                                                                   \
        case 32: BOF4_LAUNCH_MAE(32, FIRST_, CAPTURE_, CAND_, GATE_, SAMPLE_) break;   \
        case 64: BOF4_LAUNCH_MAE(64, FIRST_, CAPTURE_, CAND_, GATE_, SAMPLE_) break;   \
        case 128: BOF4_LAUNCH_MAE(128, FIRST_, CAPTURE_, CAND_, GATE_, SAMPLE_) break; \
        default: BOF4_LAUNCH_MAE(256, FIRST_, CAPTURE_, CAND_, GATE_, SAMPLE_) break;  \
    }
    unsigned long long* const no_cand = nullptr;
    const uint32_t* const no_gate = nullptr;
    if (sampling) {
        BOF4_LAUNCH_MAE_BLOCK(true, false, no_cand, no_gate, MAE_SAMPLE_MASK)
        hipLaunchKernelGGL(mae_predict_kernel, dim3(1), dim3(1024), 0, s, state, hist, cnt_part, sgrid,
                           (uint32_t)skip_mask);
    }
    for (uint32_t p = 0; p < passes; ++p) {
        const bool first = p == 0;
        // the pass that writes the list: the first one if it captures by windows, else the second
        const uint32_t list_pass = sampling ? 0u : 1u;
        const bool writes_list = use_list && p == list_pass, reads_list = use_list && p > list_pass;
        unsigned long long* cand_w = writes_list ? cand : nullptr;
        const uint32_t* gate = reads_list ? cand_full : nullptr;  // the scan only runs if the list cannot be used
        if (first) timing_begin(s);
        if (reads_list)
            hipLaunchKernelGGL(mae_list_kernel, dim3(sgrid), dim3(256), 0, s, cand, cand_count, cand_cap, cand_full,
                               state, hist, unweighted);
        if (first && sampling) {
            BOF4_LAUNCH_MAE_BLOCK(true, true, cand_w, gate, 0u)
        } else if (first) {
            BOF4_LAUNCH_MAE_BLOCK(true, false, cand_w, gate, 0u)
        } else {
            BOF4_LAUNCH_MAE_BLOCK(false, false, cand_w, gate, 0u)
        }
        if (first) timing_end(s);
        hipLaunchKernelGGL(mae_select_kernel, dim3(1), dim3(1024), 0, s, state, hist, cnt_part, sae_part, sgrid,
                           first ? 1 : 0, p + 1 == passes ? 1 : 0, (uint32_t)skip_mask,
                           writes_list ? cand_count : (const uint32_t*)nullptr, cand_waves, cand_cap, cand_full,
                           (writes_list && sampling) ? 1 : 0, direct ? direct : rec_dev, unweighted);
    }
#undef BOF4_LAUNCH_MAE_BLOCK
#undef BOF4_LAUNCH_MAE
    HIP_TRY(hipGetLastError());
    if (direct) {
        HIP_TRY(wait_for_flag(s, &out_host->n_used));
    } else {
        HIP_TRY(hipMemcpyAsync(out_host, rec_dev, sizeof(bof4_mae_stats), hipMemcpyDeviceToHost, s));
        HIP_TRY(wait_for_stream(s));
    }
    if (std::getenv("BOF4_MAE_TRACE") != nullptr) {  // debugging aid: which way the search went
        uint32_t unusable = 0;
        if (use_list) HIP_TRY(hipMemcpy(&unusable, cand_full, 4, hipMemcpyDeviceToHost));
        std::fprintf(stderr, "bof4_lloyd_step_mae: passes %u, list %d, sampling %d, list unusable %u\n", passes,
                     (int)use_list, (int)sampling, unusable);
        if (use_list && std::getenv("BOF4_MAE_TRACE")[0] == '2') {  // the fullest stretch of the list, the windows
            std::vector<uint32_t> counts(cand_waves);
            HIP_TRY(hipMemcpy(counts.data(), cand_count, (size_t)cand_waves * 4, hipMemcpyDeviceToHost));
            uint32_t most = 0;
            for (uint32_t c : counts) most = c > most ? c : most;
            MaeLevelState st[16];
            HIP_TRY(hipMemcpy(st, state, sizeof(st), hipMemcpyDeviceToHost));
            std::fprintf(stderr, "  fullest stretch %u of %u entries;", most, cand_cap);
            for (int l = 0; l < 16; ++l)
                std::fprintf(stderr, " [%d: window %u+%u, key %u of %u bits]", l, st[l].win_lo, st[l].win_len,
                             st[l].prefix, lc.bits[l]);
            std::fprintf(stderr, "\n");
        }
    }
    if (out_host->sae != out_host->sae)
        return fail(BOF4_ERR_ARG, "bof4_lloyd_step_mae: block constants too large for exact weighted medians");
    return BOF4_OK;
}

}  // extern "C"
