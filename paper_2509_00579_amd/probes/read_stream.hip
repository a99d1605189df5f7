// Ceiling of a plain streaming read on this GPU: every workgroup sums a contiguous chunk of a large buffer with
// 16-byte loads (UNROLL loads in flight per lane) and writes one word.  Prints GB/s for a few launch shapes.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#define CHECK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("%s: %s\n", #x, hipGetErrorString(e)); exit(1); } } while (0)

template <int UNROLL>
__global__ __launch_bounds__(256) void read_sum(const uint4 *__restrict__ src, size_t n16, unsigned *out) {
    const size_t per_wg = n16 / gridDim.x;  // host makes this a multiple of 256 * UNROLL
    const uint4 *p = src + (size_t)blockIdx.x * per_wg + threadIdx.x;
    unsigned acc = 0;
    for (size_t i = 0; i < per_wg; i += 256 * UNROLL) {
        uint4 v[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; u++) v[u] = p[i + (size_t)u * 256];
#pragma unroll
        for (int u = 0; u < UNROLL; u++) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    if (acc == 0x12345678u) out[blockIdx.x] = acc;  // never true for the fill pattern: keeps the loads alive
}

template <int UNROLL>
static void run(const uint4 *d, size_t bytes, unsigned *d_out, int grid) {
    const size_t chunk = (size_t)grid * 256 * UNROLL * 16;
    const size_t used = bytes / chunk * chunk;
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0)); CHECK(hipEventCreate(&e1));
    for (int i = 0; i < 2; i++) hipLaunchKernelGGL(read_sum<UNROLL>, dim3(grid), dim3(256), 0, 0, d, used / 16, d_out);
    CHECK(hipEventRecord(e0, 0));
    const int reps = 10;
    for (int i = 0; i < reps; i++) hipLaunchKernelGGL(read_sum<UNROLL>, dim3(grid), dim3(256), 0, 0, d, used / 16, d_out);
    CHECK(hipEventRecord(e1, 0));
    CHECK(hipEventSynchronize(e1));
    float ms = 0;
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    printf("%4zu MiB, grid %5d, %d loads in flight per lane: %7.1f us per pass, %6.0f GB/s\n", used >> 20, grid, UNROLL,
           ms * 1e3 / reps, used / (ms * 1e-3 / reps) / 1e9);
}

int main() {
    uint4 *d; unsigned *d_out;
    const size_t big = (size_t)2 << 30;
    CHECK(hipMalloc(&d, big)); CHECK(hipMemset(d, 1, big));
    CHECK(hipMalloc(&d_out, 1 << 20));
    for (size_t bytes : {(size_t)512 << 20, big})   // 512 MiB: the fp16 cache of the long workloads; 2 GiB: beyond the last-level cache
        for (int grid : {1024, 2048, 4096, 8192}) {
            run<4>(d, bytes, d_out, grid);
            run<8>(d, bytes, d_out, grid);
        }
    return 0;
}
