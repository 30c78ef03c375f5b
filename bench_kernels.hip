// Measurement aids of bench.py (NOT part of the library, and not linked into it): plain streaming kernels of
// known traffic, used (1) to measure what this GPU's memory system reaches for reads only, writes only, a copy,
// one read fanned out to k writes and k reads summed into one write, with the executor's access pattern (256
// lanes x 8 independent 16-byte vectors per lane and tile, tiles handed out grid-stride), and (2) to calibrate
// the hardware byte counters (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE) against a kernel whose traffic is known.
// Build: hipcc --offload-arch=gfx950 -O3 -shared -fPIC bench_kernels.hip -o libbench_kernels.so
#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>

namespace {

typedef uint32_t u4 __attribute__((ext_vector_type(4)));
constexpr int U = 8;                         // vectors per lane and tile
constexpr size_t TILE = 256 * U;             // vectors per tile

__global__ void __launch_bounds__(256) bench_read_kernel(const u4* __restrict__ src, size_t ntiles, uint32_t* sink) {
    u4 acc = {0, 0, 0, 0};
    for (size_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        const u4* p = src + t * TILE + threadIdx.x;
        u4 x[U];
#pragma unroll
        for (int u = 0; u < U; u++) x[u] = p[u * 256];
#pragma unroll
        for (int u = 0; u < U; u++) acc ^= x[u];
    }
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345678u) sink[0] = 1;      // keeps the loads alive
}

__global__ void __launch_bounds__(256) bench_write_kernel(u4* __restrict__ dst, size_t ntiles) {
    const u4 v = {threadIdx.x, 1, 2, 3};
    for (size_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        u4* p = dst + t * TILE + threadIdx.x;
#pragma unroll
        for (int u = 0; u < U; u++) p[u * 256] = v;
    }
}

// k == 1: a copy; k > 1: one read, k writes `stride` vectors apart
__global__ void __launch_bounds__(256) bench_fanout_kernel(u4* __restrict__ dst, const u4* __restrict__ src, size_t ntiles,
                                                           size_t stride, int k) {
    for (size_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        const size_t o = t * TILE + threadIdx.x;
        u4 x[U];
#pragma unroll
        for (int u = 0; u < U; u++) x[u] = src[o + u * 256];
        for (int d = 0; d < k; d++)
#pragma unroll
            for (int u = 0; u < U; u++) dst[d * stride + o + u * 256] = x[u];
    }
}

// k reads `stride` vectors apart, summed (wrapping 32-bit), one write
__global__ void __launch_bounds__(256) bench_fanin_kernel(u4* __restrict__ dst, const u4* __restrict__ src, size_t ntiles,
                                                          size_t stride, int k) {
    constexpr int V = 4;                     // fewer vectors per lane: k loads per vector are in flight
    for (size_t t = blockIdx.x; t < ntiles * (U / V); t += gridDim.x) {
        const size_t o = t * 256 * V + threadIdx.x;
        u4 acc[V];
#pragma unroll
        for (int u = 0; u < V; u++) acc[u] = src[o + u * 256];
        for (int d = 1; d < k; d++)
#pragma unroll
            for (int u = 0; u < V; u++) acc[u] += src[d * stride + o + u * 256];
#pragma unroll
        for (int u = 0; u < V; u++) dst[o + u * 256] = acc[u];
    }
}

// does nothing: what is measured around it is the launch itself
__global__ void __launch_bounds__(256) bench_empty_kernel(uint32_t* sink) {
    if (sink && threadIdx.x == 1000) sink[0] = 1;
}

}  // namespace

extern "C" {

// `grid` workgroups of `threads` lanes (64 .. 256) that do nothing.  Returns 0, -1 for a bad argument, -2 when the launch failed.
int bench_empty(int grid, int threads, void* sink, void* stream) {
    if (grid < 1 || threads < 64 || threads > 256) return -1;
    hipLaunchKernelGGL(bench_empty_kernel, dim3(grid), dim3(threads), 0, (hipStream_t)stream, (uint32_t*)sink);
    return hipGetLastError() == hipSuccess ? 0 : -2;
}

// mode 0: read `bytes` from src.  1: write `bytes` to dst.  2: copy `bytes`.  3: read `bytes` from src, write them
// to k regions of dst, `bytes` apart.  4: read k regions of src, `bytes` apart, write their sum (`bytes`) to dst.
// bytes must be a multiple of 32 KiB (one tile); pointers 16-byte aligned device memory of the sizes implied;
// `sink` is 4 bytes of device memory (mode 0).  Returns 0, -1 for a bad argument, -2 when the launch failed.
int bench_stream(int mode, void* dst, const void* src, size_t bytes, int k, int grid, void* sink, void* stream) {
    if (mode < 0 || mode > 4 || bytes == 0 || bytes % (TILE * 16) != 0 || grid < 1 || k < 1) return -1;
    const size_t ntiles = bytes / (TILE * 16), stride = bytes / 16;
    hipStream_t s = (hipStream_t)stream;
    switch (mode) {
        case 0: hipLaunchKernelGGL(bench_read_kernel, dim3(grid), dim3(256), 0, s, (const u4*)src, ntiles, (uint32_t*)sink); break;
        case 1: hipLaunchKernelGGL(bench_write_kernel, dim3(grid), dim3(256), 0, s, (u4*)dst, ntiles); break;
        case 2: hipLaunchKernelGGL(bench_fanout_kernel, dim3(grid), dim3(256), 0, s, (u4*)dst, (const u4*)src, ntiles, stride, 1); break;
        case 3: hipLaunchKernelGGL(bench_fanout_kernel, dim3(grid), dim3(256), 0, s, (u4*)dst, (const u4*)src, ntiles, stride, k); break;
        default: hipLaunchKernelGGL(bench_fanin_kernel, dim3(grid), dim3(256), 0, s, (u4*)dst, (const u4*)src, ntiles, stride, k); break;
    }
    return hipGetLastError() == hipSuccess ? 0 : -2;
}

}  // extern "C"
