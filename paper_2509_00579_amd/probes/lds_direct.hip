// Checks what the fused kernel's tile path relies on when it stages a record with LDS-direct loads
// (global_load_lds_dwordx4, gfx950): lane l of a load delivers its 16 bytes to LDS byte (M0 base) + 16 l, and lanes
// that are masked out neither load nor write.  Prints, for several record sizes (in 16-byte units), how many staged
// units differ from the source and how many LDS units beyond the record were touched; both must be 0.
//
//   hipcc --offload-arch=gfx950 -O3 -std=c++17 -Xclang -target-feature -Xclang -packed-fp32-ops lds_direct.hip -o lds_direct
#include <hip/hip_runtime.h>
#include <cstdio>
#include <vector>
__global__ void k(const uint4* src, uint4* out, unsigned n16) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int lane = threadIdx.x & 63;
    for (int i = lane; i < 512 + 64; i += 64) reinterpret_cast<uint4*>(smem)[i] = make_uint4(0xdeadbeef, 0, 0, 0);
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 8; i++)
        if (lane + 64 * i < n16)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + lane + 64 * i),
                                             (__attribute__((address_space(3))) void*)(smem + 1024 * i), 16, 0, 0);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    for (int i = lane; i < 512 + 64; i += 64) out[i] = reinterpret_cast<uint4*>(smem)[i];
}
int main() {
    const int N = 512 + 64;
    std::vector<uint4> h(N), o(N);
    for (int i = 0; i < N; i++) h[i] = make_uint4(i, i * 3 + 1, i * 7 + 2, i * 11 + 3);
    uint4 *d, *dout;
    if (hipMalloc(&d, N * 16) != hipSuccess || hipMalloc(&dout, N * 16) != hipSuccess) return 1;
    if (hipMemcpy(d, h.data(), N * 16, hipMemcpyHostToDevice) != hipSuccess) return 1;
    for (unsigned n16 : {512u, 431u, 64u, 1u, 100u}) {
        (void)hipMemset(dout, 0, N * 16);
        hipLaunchKernelGGL(k, dim3(1), dim3(64), (512 + 64) * 16, 0, d, dout, n16);
        if (hipDeviceSynchronize() != hipSuccess) { printf("launch failed\n"); return 1; }
        if (hipMemcpy(o.data(), dout, N * 16, hipMemcpyDeviceToHost) != hipSuccess) return 1;
        int bad = 0, touched_beyond = 0;
        for (unsigned i = 0; i < (unsigned)N; i++) {
            if (i < n16) bad += !(o[i].x == h[i].x && o[i].y == h[i].y && o[i].z == h[i].z && o[i].w == h[i].w);
            else touched_beyond += o[i].x != 0xdeadbeef;
        }
        printf("n16 %u: wrong %d, touched beyond the record %d\n", n16, bad, touched_beyond);
    }
    return 0;
}
