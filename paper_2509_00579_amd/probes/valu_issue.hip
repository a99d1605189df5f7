// VALU issue: cycles per instruction per wave and per SIMD for 1..8 waves per SIMD (independent accumulators):
// kind 0 v_fmac_f32, 1 v_and_b32, 2 v_lshrrev_b32, 3 v_fmac_f32 with a DPP quad broadcast, 4 v_cvt_f32_ubyte1,
// 5 v_readlane_b32, 6 v_perm_b32, 7 v_pk_add_f16, 8 v_cvt_f16_u16 with an SDWA byte select, 9 v_pack_b32_f16,
// 10 v_cvt_f32_u32, 11 v_or_b32.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <chrono>
#define CHECK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("%s: %s\n", #x, hipGetErrorString(e)); exit(1); } } while (0)

template <int KIND>
__global__ __launch_bounds__(256) void probe(float *out, long long *cyc, int iters) {
    float a = out[threadIdx.x], b = out[threadIdx.x + 256];
    float x[8] = {a, b, a + 1.f, b + 1.f, a + 2.f, b + 2.f, a + 3.f, b + 3.f};
    unsigned u[8] = {1, 2, 3, 4, 5, 6, 7, 8};
    long long t0 = clock64();
    for (int it = 0; it < iters; it++) {
#pragma unroll
        for (int r = 0; r < 8; r++)
#pragma unroll
            for (int k = 0; k < 8; k++) {
                if (KIND == 0) asm volatile("v_fmac_f32 %0, %1, %2" : "+v"(x[k]) : "v"(a), "v"(b));
                if (KIND == 1) asm volatile("v_and_b32 %0, %1, %0" : "+v"(u[k]) : "v"(a));
                if (KIND == 2) asm volatile("v_lshrrev_b32 %0, %1, %0" : "+v"(u[k]) : "v"(a));
                if (KIND == 3) asm volatile("v_fmac_f32_dpp %0, %1, %2 quad_perm:[1,1,1,1] row_mask:0xf bank_mask:0xf" : "+v"(x[k]) : "v"(a), "v"(b));
                if (KIND == 4) asm volatile("v_cvt_f32_ubyte1 %0, %1" : "=v"(x[k]) : "v"(u[k]));
                if (KIND == 5) asm volatile("v_readlane_b32 %0, %1, 3" : "=s"(u[k]) : "v"(a));
                if (KIND == 6) asm volatile("v_perm_b32 %0, %1, %0, %2" : "+v"(u[k]) : "v"(a), "v"(b));
                if (KIND == 7) asm volatile("v_pk_add_f16 %0, %1, %0" : "+v"(u[k]) : "v"(a));
                if (KIND == 8) asm volatile("v_cvt_f16_u16_sdwa %0, %1 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_1" : "=v"(u[k]) : "v"(a));
                if (KIND == 9) asm volatile("v_pack_b32_f16 %0, %1, %0" : "+v"(u[k]) : "v"(a));
                if (KIND == 10) asm volatile("v_cvt_f32_u32 %0, %1" : "=v"(x[k]) : "v"(u[k]));
                if (KIND == 11) asm volatile("v_or_b32 %0, %1, %0" : "+v"(u[k]) : "v"(a));
            }
    }
    long long t1 = clock64();
    float s = 0; for (int k = 0; k < 8; k++) s += x[k] + (float)u[k];
    out[blockIdx.x * 256 + threadIdx.x] = s;
    if (threadIdx.x == 0) { cyc[blockIdx.x] = t1 - t0; cyc[8192 + blockIdx.x] = wall_clock64(); }
}

int main() {
    float *d_out; long long *d_cyc;
    CHECK(hipMalloc(&d_out, 8192 * 256 * 4)); CHECK(hipMemset(d_out, 0, 8192 * 256 * 4));
    CHECK(hipMalloc(&d_cyc, 2 * 8192 * 8));
    const int iters = 20000;
    for (int kind = 0; kind < 12; kind++)
        for (int wps : {1, 4}) {
            const int n_wg = 256 * wps;
            double us = 0;
            for (int rep = 0; rep < 2; rep++) {
                CHECK(hipDeviceSynchronize());
                auto w0 = std::chrono::steady_clock::now();
                if (kind == 0) hipLaunchKernelGGL(probe<0>, dim3(n_wg), dim3(256), 0, 0, d_out, d_cyc, iters);
                if (kind == 1) hipLaunchKernelGGL(probe<1>, dim3(n_wg), dim3(256), 0, 0, d_out, d_cyc, iters);
                if (kind == 2) hipLaunchKernelGGL(probe<2>, dim3(n_wg), dim3(256), 0, 0, d_out, d_cyc, iters);
                if (kind == 3) hipLaunchKernelGGL(probe<3>, dim3(n_wg), dim3(256), 0, 0, d_out, d_cyc, iters);
                if (kind == 4) hipLaunchKernelGGL(probe<4>, dim3(n_wg), dim3(256), 0, 0, d_out, d_cyc, iters);
                if (kind == 5) hipLaunchKernelGGL(probe<5>, dim3(n_wg), dim3(256), 0, 0, d_out, d_cyc, iters);
                if (kind == 6) hipLaunchKernelGGL(probe<6>, dim3(n_wg), dim3(256), 0, 0, d_out, d_cyc, iters);
                if (kind == 7) hipLaunchKernelGGL(probe<7>, dim3(n_wg), dim3(256), 0, 0, d_out, d_cyc, iters);
                if (kind == 8) hipLaunchKernelGGL(probe<8>, dim3(n_wg), dim3(256), 0, 0, d_out, d_cyc, iters);
                if (kind == 9) hipLaunchKernelGGL(probe<9>, dim3(n_wg), dim3(256), 0, 0, d_out, d_cyc, iters);
                if (kind == 10) hipLaunchKernelGGL(probe<10>, dim3(n_wg), dim3(256), 0, 0, d_out, d_cyc, iters);
                if (kind == 11) hipLaunchKernelGGL(probe<11>, dim3(n_wg), dim3(256), 0, 0, d_out, d_cyc, iters);
                CHECK(hipDeviceSynchronize());
                us = std::chrono::duration<double, std::micro>(std::chrono::steady_clock::now() - w0).count();
            }
            long long c; CHECK(hipMemcpy(&c, d_cyc, 8, hipMemcpyDeviceToHost));
            static long long ends[8192]; CHECK(hipMemcpy(ends, d_cyc + 8192, n_wg * 8, hipMemcpyDeviceToHost));
            long long mn = ends[0], mx = ends[0]; int early = 0;
            for (int i = 0; i < n_wg; i++) { if (ends[i] < mn) mn = ends[i]; if (ends[i] > mx) mx = ends[i]; }
            for (int i = 0; i < n_wg; i++) if (ends[i] - mn < (mx - mn) / 4) early++;
            printf("   end times spread %.0f us, %d of %d workgroups end in the first quarter of the spread\n", (mx - mn) * 0.01, early, n_wg);
            const double n = iters * 64.0;
            printf("kind %d, %d waves/SIMD: %.2f ticks per instr per wave, %.2f ticks per instr per SIMD; wall %.0f us -> %.2f ns per instr per SIMD, tick = %.3f ns\n",
                   kind, wps, c / n, c / n / wps, us, us * 1e3 / n / wps, us * 1e3 / (double)c);
        }
    return 0;
}
