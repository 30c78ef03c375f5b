// Measurement aid (standalone program, not part of the library): what streaming bandwidth this GPU
// reaches for reads only, writes only, a copy, a 1-read : 7-write fan-out and an 8-read : 1-write
// fan-in, with the access pattern of the executor (256 lanes x U vectors of 16 B per tile,
// grid-stride over tiles, 2 GiB per buffer).  These are the ceilings the executor's traffic is
// compared with.  Build: hipcc --offload-arch=gfx950 -O3 bw_probe.hip -o bw_probe
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
typedef unsigned u4 __attribute__((ext_vector_type(4)));
#define CHECK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); exit(1); } } while (0)

template <int U> __global__ void __launch_bounds__(256) k_read(const u4* __restrict__ src, size_t ntiles, unsigned* out) {
    u4 acc = {0, 0, 0, 0};
    for (size_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        const u4* p = src + t * 256 * U + threadIdx.x;
        u4 x[U];
#pragma unroll
        for (int u = 0; u < U; u++) x[u] = p[u * 256];
#pragma unroll
        for (int u = 0; u < U; u++) acc ^= x[u];
    }
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345678u) out[0] = 1;
}
template <int U> __global__ void __launch_bounds__(256) k_write(u4* __restrict__ dst, size_t ntiles) {
    u4 v = {threadIdx.x, 1, 2, 3};
    for (size_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        u4* p = dst + t * 256 * U + threadIdx.x;
#pragma unroll
        for (int u = 0; u < U; u++) p[u * 256] = v;
    }
}
template <int U> __global__ void __launch_bounds__(256) k_copy(u4* __restrict__ dst, const u4* __restrict__ src, size_t ntiles) {
    for (size_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        const size_t o = t * 256 * U + threadIdx.x;
        u4 x[U];
#pragma unroll
        for (int u = 0; u < U; u++) x[u] = src[o + u * 256];
#pragma unroll
        for (int u = 0; u < U; u++) dst[o + u * 256] = x[u];
    }
}
// 1 read : 7 writes (allgather-like) and 5 reads : 1 write (reduce-like)
template <int U> __global__ void __launch_bounds__(256) k_fanout(u4* __restrict__ dst, const u4* __restrict__ src, size_t ntiles, size_t stride, int k) {
    for (size_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        const size_t o = t * 256 * U + threadIdx.x;
        u4 x[U];
#pragma unroll
        for (int u = 0; u < U; u++) x[u] = src[o + u * 256];
        for (int d = 0; d < k; d++)
#pragma unroll
            for (int u = 0; u < U; u++) dst[d * stride + o + u * 256] = x[u];
    }
}
template <int U> __global__ void __launch_bounds__(256) k_fanin(u4* __restrict__ dst, const u4* __restrict__ src, size_t ntiles, size_t stride, int k) {
    for (size_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        const size_t o = t * 256 * U + threadIdx.x;
        u4 acc[U];
#pragma unroll
        for (int u = 0; u < U; u++) acc[u] = src[o + u * 256];
        for (int d = 1; d < k; d++)
#pragma unroll
            for (int u = 0; u < U; u++) acc[u] += src[d * stride + o + u * 256];
#pragma unroll
        for (int u = 0; u < U; u++) dst[o + u * 256] = acc[u];
    }
}

int main() {
    const size_t bytes = (size_t)1 << 31;     // 2 GiB per buffer
    char *a, *b; unsigned* flag;
    CHECK(hipMalloc(&a, bytes)); CHECK(hipMalloc(&b, bytes)); CHECK(hipMalloc(&flag, 4));
    CHECK(hipMemset(a, 1, bytes)); CHECK(hipMemset(b, 2, bytes));
    hipEvent_t e0, e1; CHECK(hipEventCreate(&e0)); CHECK(hipEventCreate(&e1));
    const int grids[] = {256, 512, 1024, 2048};
    for (int gi = 0; gi < 4; gi++) {
        const int grid = grids[gi];
#define RUN(name, traffic, launch) do { float best = 1e30f; for (int r = 0; r < 6; r++) { CHECK(hipEventRecord(e0)); launch; CHECK(hipEventRecord(e1)); CHECK(hipEventSynchronize(e1)); float ms; CHECK(hipEventElapsedTime(&ms, e0, e1)); if (r > 0 && ms < best) best = ms; } printf("%-22s grid %5d  %8.3f ms  %8.1f GB/s\n", name, grid, best, (double)(traffic) / best / 1e6); fflush(stdout); } while (0)
        RUN("read  U=8", bytes, (k_read<8><<<grid, 256>>>((const u4*)a, bytes / (256 * 8 * 16), flag)));
        RUN("read  U=4", bytes, (k_read<4><<<grid, 256>>>((const u4*)a, bytes / (256 * 4 * 16), flag)));
        RUN("write U=8", bytes, (k_write<8><<<grid, 256>>>((u4*)b, bytes / (256 * 8 * 16))));
        RUN("write U=4", bytes, (k_write<4><<<grid, 256>>>((u4*)b, bytes / (256 * 4 * 16))));
        RUN("copy  U=8", 2 * bytes, (k_copy<8><<<grid, 256>>>((u4*)b, (const u4*)a, bytes / (256 * 8 * 16))));
        RUN("copy  U=4", 2 * bytes, (k_copy<4><<<grid, 256>>>((u4*)b, (const u4*)a, bytes / (256 * 4 * 16))));
        // 1 read of 256 MiB fanned out to 7 x 256 MiB; 8 reads of 256 MiB reduced into 256 MiB
        const size_t part = bytes / 8;
        RUN("fanout 1r:7w U=8", 8 * part, (k_fanout<8><<<grid, 256>>>((u4*)b, (const u4*)a, part / (256 * 8 * 16), part / 16, 7)));
        RUN("fanin  8r:1w U=4", 9 * part, (k_fanin<4><<<grid, 256>>>((u4*)b, (const u4*)a, part / (256 * 4 * 16), part / 16, 8)));
    }
    CHECK(hipDeviceSynchronize());
    return 0;
}
