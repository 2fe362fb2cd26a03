// bench_ceilings.hip - plain streaming kernels that measure what this GPU's memory system delivers for the traffic
// mixes of the hot path.  Benchmark-only code (loaded by bench.py --ceilings, not part of the library): a kernel of
// the library that moves R bytes in and W bytes out per weight cannot run faster than the plain kernel with the same
// mix, so its distance to that ceiling - not only to the 8 TB/s data-sheet figure - says how much is left in it.
//
// Every kernel moves 16-byte vectors with nontemporal loads / stores (what the library's kernels use).  A workgroup
// of 256 lanes handles "groups": per group it reads R x 256 consecutive vectors and writes W x 256 consecutive
// vectors; the grid walks the groups with a stride of gridDim.x.  Mixes: R:W = 1:0 (read only), 0:1 (write only),
// 1:1 (copy), 4:1 (the quantiser: 2 bytes read, 0.5 written per weight), 1:4 (the decoder).
#include <hip/hip_runtime.h>

#include <cstdint>

namespace {
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int R, int W>
__global__ __launch_bounds__(256) void stream_kernel(const u32x4* __restrict__ in, u32x4* __restrict__ out,
                                                     uint64_t n_groups, uint32_t never) {
    u32x4 acc = {threadIdx.x, 1u, 2u, 3u};
    for (uint64_t g = blockIdx.x; g < n_groups; g += gridDim.x) {
        u32x4 v[R > 0 ? R : 1];
#pragma unroll
        for (int r = 0; r < R; ++r) v[r] = __builtin_nontemporal_load(&in[(g * R + r) * 256 + threadIdx.x]);
#pragma unroll
        for (int r = 0; r < R; ++r) acc ^= v[r];
#pragma unroll
        for (int w = 0; w < W; ++w) {
            u32x4 o = acc;
            o.x += (uint32_t)w;
            __builtin_nontemporal_store(o, &out[(g * W + w) * 256 + threadIdx.x]);
        }
    }
    // keeps the loads of the read-only kernel alive; `never` is 0xFFFFFFFF and no lane ever matches
    if (W == 0 && (acc.x ^ acc.y ^ acc.z ^ acc.w) == never && threadIdx.x == never) out[0] = acc;
}

template <int R, int W>
int run(const void* in, void* out, uint64_t n_groups, uint32_t grid, int reps, hipStream_t s, float* ms_out) {
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return -1;
    hipLaunchKernelGGL((stream_kernel<R, W>), dim3(grid), dim3(256), 0, s, (const u32x4*)in, (u32x4*)out, n_groups,
                       0xFFFFFFFFu);  // warm-up
    (void)hipEventRecord(e0, s);
    for (int i = 0; i < reps; ++i)
        hipLaunchKernelGGL((stream_kernel<R, W>), dim3(grid), dim3(256), 0, s, (const u32x4*)in, (u32x4*)out,
                           n_groups, 0xFFFFFFFFu);
    (void)hipEventRecord(e1, s);
    int rc = hipEventSynchronize(e1) == hipSuccess && hipGetLastError() == hipSuccess ? 0 : -1;
    float ms = 0.0f;
    if (rc == 0 && hipEventElapsedTime(&ms, e0, e1) != hipSuccess) rc = -1;
    *ms_out = ms / (float)reps;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return rc;
}
}  // namespace

extern "C" {
// kind: 0 read only, 1 write only, 2 copy 1:1, 3 read 4 : write 1, 4 read 1 : write 4.
// in_dev must hold R * 4096 * n_groups bytes, out_dev W * 4096 * n_groups bytes (16-byte aligned; out_dev at least 16
// bytes for the read-only kernel).  grid: workgroups launched (1 .. n_groups).  Returns 0 and the average
// milliseconds per launch over `reps` launches (HIP events on `stream`), or -1.
int bench_ceiling(int kind, const void* in_dev, void* out_dev, uint64_t n_groups, uint32_t grid, int reps, void* stream,
                  float* ms_out) {
    if (!in_dev || !out_dev || !ms_out || n_groups == 0 || grid == 0 || reps < 1) return -1;
    if ((uint64_t)grid > n_groups) grid = (uint32_t)n_groups;
    hipStream_t s = (hipStream_t)stream;
    switch (kind) {
        case 0: return run<1, 0>(in_dev, out_dev, n_groups, grid, reps, s, ms_out);
        case 1: return run<0, 1>(in_dev, out_dev, n_groups, grid, reps, s, ms_out);
        case 2: return run<1, 1>(in_dev, out_dev, n_groups, grid, reps, s, ms_out);
        case 3: return run<4, 1>(in_dev, out_dev, n_groups, grid, reps, s, ms_out);
        case 4: return run<1, 4>(in_dev, out_dev, n_groups, grid, reps, s, ms_out);
        default: return -1;
    }
}
}
