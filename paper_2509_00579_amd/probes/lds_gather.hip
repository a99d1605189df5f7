// LDS gather throughput: 64 lanes read random words of a table of W words; cycles per wave-instruction per CU.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <vector>
#define CHECK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("%s: %s\n", #x, hipGetErrorString(e)); exit(1); } } while (0)

template <int MODE>  // 0: b32 reads, 1: u16 reads, 2: b64 reads
__global__ __launch_bounds__(256) void probe(const uint32_t *addrs, int iters, uint32_t *out, long long *cyc) {
    __shared__ uint32_t tab[8192];
    for (int i = threadIdx.x; i < 8192; i += 256) tab[i] = i * 2654435761u;
    uint32_t a[16];
    for (int k = 0; k < 16; k++) a[k] = addrs[(blockIdx.x * 256 + threadIdx.x) * 16 + k];
    __syncthreads();
    uint32_t s0 = 0, s1 = 0, s2 = 0, s3 = 0;
    const char *base = reinterpret_cast<const char *>(tab);
    long long t0 = clock64();
    for (int it = 0; it < iters; it++) {
#pragma unroll
        for (int k = 0; k < 16; k += 4) {
            if (MODE == 0) {
                s0 += *reinterpret_cast<const uint32_t *>(base + a[k]);
                s1 += *reinterpret_cast<const uint32_t *>(base + a[k + 1]);
                s2 += *reinterpret_cast<const uint32_t *>(base + a[k + 2]);
                s3 += *reinterpret_cast<const uint32_t *>(base + a[k + 3]);
            } else if (MODE == 1) {
                s0 += *reinterpret_cast<const uint16_t *>(base + a[k]);
                s1 += *reinterpret_cast<const uint16_t *>(base + a[k + 1]);
                s2 += *reinterpret_cast<const uint16_t *>(base + a[k + 2]);
                s3 += *reinterpret_cast<const uint16_t *>(base + a[k + 3]);
            } else {
                uint2 v0 = *reinterpret_cast<const uint2 *>(base + a[k]);
                uint2 v1 = *reinterpret_cast<const uint2 *>(base + a[k + 1]);
                uint2 v2 = *reinterpret_cast<const uint2 *>(base + a[k + 2]);
                uint2 v3 = *reinterpret_cast<const uint2 *>(base + a[k + 3]);
                s0 += v0.x ^ v0.y; s1 += v1.x ^ v1.y; s2 += v2.x ^ v2.y; s3 += v3.x ^ v3.y;
            }
        }
        asm volatile("" ::: "memory");
    }
    long long t1 = clock64();
    out[blockIdx.x * 256 + threadIdx.x] = s0 + s1 + s2 + s3;
    if (threadIdx.x == 0) cyc[blockIdx.x] = t1 - t0;
}

int main() {
    const int n_wg = 256 * 4, iters = 2000;  // 4 workgroups of 4 waves per CU
    uint32_t *d_addr, *d_out; long long *d_cyc;
    CHECK(hipMalloc(&d_addr, n_wg * 256 * 16 * 4));
    CHECK(hipMalloc(&d_out, n_wg * 256 * 4));
    CHECK(hipMalloc(&d_cyc, n_wg * 8));
    std::vector<uint32_t> h(n_wg * 256 * 16);
    std::vector<long long> hc(n_wg);
    struct Case { const char *name; int mode; int bytes; int gran; };
    // gran: address granularity in bytes; bytes: table size
    const Case cases[] = {
        {"b32 W=32 words", 0, 128, 4}, {"b32 W=64", 0, 256, 4}, {"b32 W=128", 0, 512, 4}, {"b32 W=256", 0, 1024, 4},
        {"b32 W=1024", 0, 4096, 4}, {"b32 W=4096", 0, 16384, 4},
        {"u16 64 entries (32 words)", 1, 128, 2}, {"u16 128 entries", 1, 256, 2}, {"u16 256 entries", 1, 512, 2},
        {"u16 1024 entries", 1, 2048, 2},
        {"b64 W=64 dwords", 2, 256, 8}, {"b64 W=256 dwords", 2, 1024, 8}, {"b64 4096 dwords", 2, 16384, 8},
        {"b32 same word (broadcast)", 0, 4, 4}, {"b32 lane-linear", 0, -1, 4},
    };
    for (const Case &c : cases) {
        srand(1);
        for (size_t i = 0; i < h.size(); i++) {
            const int lane = (int)((i / 16) % 64);
            if (c.bytes < 0) h[i] = (uint32_t)(lane * 4 + (i % 16) * 256);
            else h[i] = (uint32_t)((rand() % (c.bytes / c.gran)) * c.gran);
        }
        CHECK(hipMemcpy(d_addr, h.data(), h.size() * 4, hipMemcpyHostToDevice));
        for (int rep = 0; rep < 2; rep++) {
            if (c.mode == 0) hipLaunchKernelGGL(probe<0>, dim3(n_wg), dim3(256), 0, 0, d_addr, iters, d_out, d_cyc);
            if (c.mode == 1) hipLaunchKernelGGL(probe<1>, dim3(n_wg), dim3(256), 0, 0, d_addr, iters, d_out, d_cyc);
            if (c.mode == 2) hipLaunchKernelGGL(probe<2>, dim3(n_wg), dim3(256), 0, 0, d_addr, iters, d_out, d_cyc);
            CHECK(hipDeviceSynchronize());
        }
        CHECK(hipMemcpy(hc.data(), d_cyc, n_wg * 8, hipMemcpyDeviceToHost));
        double sum = 0; for (long long v : hc) sum += (double)v;
        const double per_wave_loop = sum / n_wg;                 // cycles for iters*16 reads by one wave
        // 16 waves per CU share the LDS: CU cycles per wave-instruction = loop cycles / (reads per wave * 16 waves)
        printf("%-30s %8.1f cycles/read per wave, %6.2f CU-cycles per wave-instruction\n", c.name,
               per_wave_loop / (iters * 16.0), per_wave_loop / (iters * 16.0) / 16.0);
        fflush(stdout);
    }
    return 0;
}
