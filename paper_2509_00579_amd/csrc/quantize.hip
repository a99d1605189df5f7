// Store side, first half (Section 3, Store stage; Section 3.1.1): quantize 2D blocks and histogram the codes on the
// device.  The codebook itself is built on the host from this histogram.
#include "tile_quant.cuh"

namespace kvc {

// One workgroup walks over several 2D blocks and keeps the histogram in LDS as [bin][32 copies], copy = lane % 32:
// the lanes of a half-wave always hit 32 different banks and never the same word, so an LDS atomic instruction costs
// its minimum however peaked the code distribution is (with one copy per wave, lanes with the same code serialise
// and the kernel was bound by its LDS atomics).  The copies are summed and added to the global histogram at the end.
// KEEP: the codes ([block][64][128] bytes) and the unit min/max ([block][units] {min,max} fp16 pairs) of every block also
// go to a caller's workspace, from where the encoder takes them instead of quantizing the input again (kvcomp_prefill).
template <int WHICH, bool KEEP>
__global__ __launch_bounds__(256, 4) void histogram_kernel(Geo g, const uint16_t *__restrict__ X, int seq_stride,
                                                         int n_blk_per_bh, int n_blk_total, uint8_t *__restrict__ codes,
                                                         uint32_t *__restrict__ minmax) {
    __shared__ QuantShared sh;
    __shared__ uint32_t hist[256][32];
    const int tid = threadIdx.x, copy = tid & 31;
    for (int i = tid; i < 256 * 32; i += 256) (&hist[0][0])[i] = 0;
    __syncthreads();
    bool bad = false;
    TileRaw raw;
    auto fetch = [&](int blk) {  // clamped to the last block: the loads of the block after the last are harmless
        const int bl = min(blk, n_blk_total - 1);
        const int bh = bl / n_blk_per_bh, j = bl - bh * n_blk_per_bh;
        load_tile_raw(X, seq_stride, g.H, bh / g.H, bh % g.H, j, tid, raw);
    };
    fetch(blockIdx.x);
    for (int blk = blockIdx.x; blk < n_blk_total; blk += gridDim.x) {
        TileRegs r;
        bad |= unpack_tile(raw, r);
        fetch(blk + gridDim.x);  // the next block's loads travel while this one is quantized
        quantize_tile<WHICH>(r, sh, tid, g.two_eb[WHICH], g.n_sym[WHICH], g.k_units);
#pragma unroll
        for (int i = 0; i < 4; i++)
#pragma unroll
            for (int k = 0; k < 8; k++) atomicAdd(&hist[r.code[i][k]][copy], 1u);
        if constexpr (KEEP) {
            const int c0 = tile_chan0(tid);
#pragma unroll
            for (int i = 0; i < 4; i++) {
                uint2 pk;
                pk.x = r.code[i][0] | (r.code[i][1] << 8) | (r.code[i][2] << 16) | (r.code[i][3] << 24);
                pk.y = r.code[i][4] | (r.code[i][5] << 8) | (r.code[i][6] << 16) | (r.code[i][7] << 24);
                *reinterpret_cast<uint2 *>(codes + (size_t)blk * kTile + tile_token(tid, i) * kD + c0) = pk;
            }
            const int units = WHICH == 0 ? g.k_units : kBT;
            if (tid < units)
                minmax[(size_t)blk * units + tid] = float_to_half_bits(sh.unit_mn[tid]) | (float_to_half_bits(sh.unit_mx[tid]) << 16);
        }
        __syncthreads();  // unit_mn/unit_mx are rewritten by the next iteration
    }
    __syncthreads();
    uint32_t total = 0;
#pragma unroll
    for (int c = 0; c < 32; c++) total += hist[tid][(c + tid) & 31];  // rotated: conflict-free across the bins
    if (total) atomicAdd(&g.hist[WHICH * 256 + tid], total);
    if (bad) atomicOr(&g.ctrl->nonfinite, 1u);
}

// Parity export: codes [blocks][64][128] and unit min/max [blocks][units][2] as fp16 bit patterns.
template <int WHICH>
__global__ __launch_bounds__(256) void debug_codes_kernel(Geo g, const uint16_t *__restrict__ X, int seq_stride,
                                                           int n_blk_per_bh, uint8_t *__restrict__ codes,
                                                           uint16_t *__restrict__ minmax) {
    __shared__ QuantShared sh;
    const int tid = threadIdx.x, blk = blockIdx.x;
    const int bh = blk / n_blk_per_bh, j = blk - bh * n_blk_per_bh;
    TileRegs r;
    const bool bad = load_tile(X, seq_stride, g.H, bh / g.H, bh % g.H, j, tid, r);
    quantize_tile<WHICH>(r, sh, tid, g.two_eb[WHICH], g.n_sym[WHICH], g.k_units);
    const int c0 = tile_chan0(tid);
#pragma unroll
    for (int i = 0; i < 4; i++) {
        const int t = tile_token(tid, i);
        uint2 pk;
        pk.x = r.code[i][0] | (r.code[i][1] << 8) | (r.code[i][2] << 16) | (r.code[i][3] << 24);
        pk.y = r.code[i][4] | (r.code[i][5] << 8) | (r.code[i][6] << 16) | (r.code[i][7] << 24);
        *reinterpret_cast<uint2 *>(codes + (size_t)blk * kTile + t * kD + c0) = pk;
    }
    const int units = WHICH == 0 ? g.k_units : kBT;
    if (tid < units) {
        minmax[((size_t)blk * units + tid) * 2 + 0] = (uint16_t)float_to_half_bits(sh.unit_mn[tid]);
        minmax[((size_t)blk * units + tid) * 2 + 1] = (uint16_t)float_to_half_bits(sh.unit_mx[tid]);
    }
    if (bad) atomicOr(&g.ctrl->nonfinite, 1u);
}

// codes / minmax != NULL: also keep the codes and the unit min/max of every block there
hipError_t launch_histogram(const Geo &g, int which, const uint16_t *X, int seq_stride, int n_blk_per_bh,
                            uint8_t *codes, uint32_t *minmax, hipStream_t s) {
    const int total = g.B * g.H * n_blk_per_bh;
    if (total <= 0) return hipSuccess;
    const int grid = total < 1024 ? total : 1024;  // four workgroups per CU (32 KiB of LDS each), several blocks each
    const bool keep = codes != nullptr;
    if (which == 0 && !keep)
        hipLaunchKernelGGL((histogram_kernel<0, false>), dim3(grid), dim3(256), 0, s, g, X, seq_stride, n_blk_per_bh, total, codes, minmax);
    else if (which == 0)
        hipLaunchKernelGGL((histogram_kernel<0, true>), dim3(grid), dim3(256), 0, s, g, X, seq_stride, n_blk_per_bh, total, codes, minmax);
    else if (!keep)
        hipLaunchKernelGGL((histogram_kernel<1, false>), dim3(grid), dim3(256), 0, s, g, X, seq_stride, n_blk_per_bh, total, codes, minmax);
    else
        hipLaunchKernelGGL((histogram_kernel<1, true>), dim3(grid), dim3(256), 0, s, g, X, seq_stride, n_blk_per_bh, total, codes, minmax);
    return hipGetLastError();
}

hipError_t launch_debug_codes(const Geo &g, int which, const uint16_t *X, int seq_stride, int n_blk_per_bh,
                              uint8_t *d_codes, uint16_t *d_minmax, hipStream_t s) {
    const int total = g.B * g.H * n_blk_per_bh;
    if (total <= 0) return hipSuccess;
    if (which == 0)
        hipLaunchKernelGGL(debug_codes_kernel<0>, dim3(total), dim3(256), 0, s, g, X, seq_stride, n_blk_per_bh, d_codes,
                           d_minmax);
    else
        hipLaunchKernelGGL(debug_codes_kernel<1>, dim3(total), dim3(256), 0, s, g, X, seq_stride, n_blk_per_bh, d_codes,
                           d_minmax);
    return hipGetLastError();
}

__global__ void fill_zero_kernel(uint4 *p, size_t n16) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n16; i += stride) p[i] = make_uint4(0, 0, 0, 0);
}

// Clears a 16-byte aligned region with a kernel (safe inside a captured graph, unlike a memset node).
hipError_t launch_fill_zero(void *p, size_t bytes, hipStream_t s) {
    const size_t n16 = bytes / 16;
    if (n16 == 0) return hipSuccess;
    size_t grid = (n16 + 255) / 256;
    if (grid > 4096) grid = 4096;
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)grid), dim3(256), 0, s, reinterpret_cast<uint4 *>(p), n16);
    return hipGetLastError();
}

}  // namespace kvc
