// Store side, first half (Section 3, Store stage; Section 3.1.1): quantize 2D blocks and histogram the codes on the
// device.  The codebook itself is built on the host from this histogram.
#include "tile_quant.cuh"

namespace kvc {

// One workgroup walks over several 2D blocks and keeps the histogram in LDS as [bin][32 copies], copy = lane % 32:
// the lanes of a half-wave always hit 32 different banks and never the same word, so an LDS atomic instruction costs
// its minimum however peaked the code distribution is (with one copy per wave, lanes with the same code serialise
// and the kernel was bound by its LDS atomics).  The copies are summed and added to the global histogram at the end.
// KEEP: the codes ([block][64][128] bytes), the unit min/max ([block][units] {min,max} fp16 pairs) and the histogram
// ([block][256] u16) of every block also go to a caller's workspace, from where the encoder takes them instead of
// quantizing the input again (kvcomp_prefill): the record sizes then come from the block histograms and the code
// lengths alone.  The LDS histogram is then that of one block: after a block's atomics thread b sums and clears the
// copies of bin b.
// byte 0 of four words as one word, a's in the lowest byte
__device__ __forceinline__ uint32_t pack_low_bytes(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
    const uint32_t lo = __builtin_amdgcn_perm(b, a, 0x0c0c0400u), hi = __builtin_amdgcn_perm(d, c, 0x0c0c0400u);
    return __builtin_amdgcn_perm(hi, lo, 0x05040100u);
}

template <int WHICH, bool KEEP>
__global__ __launch_bounds__(256, 4) void histogram_kernel(Geo g, const uint16_t *__restrict__ X, int seq_stride,
                                                         int n_blk_per_bh, int n_blk_total, uint8_t *__restrict__ codes,
                                                         uint32_t *__restrict__ minmax,
                                                         uint16_t *__restrict__ block_hist) {
    __shared__ QuantShared sh;
    __shared__ __attribute__((aligned(16))) uint32_t hist[256][32];
    const int tid = threadIdx.x, copy = tid & 31;
    for (int i = tid; i < 256 * 32; i += 256) (&hist[0][0])[i] = 0;
    __syncthreads();
    bool bad = false;
    uint32_t total = 0;  // of bin `tid`, over this workgroup's blocks
    TileRaw raw;
    // Work items are numbered (batch, block, head), head fastest: a token's row holds all heads (H x 256 bytes), so
    // workgroups that run side by side read neighbouring pieces of the same rows and DRAM pages are used whole.  With
    // the blocks of one head side by side every 256-byte piece would open a page of its own.
    auto block_of = [&](int item, int &b, int &h, int &j) {
        const int per_b = g.H * n_blk_per_bh;
        b = item / per_b;
        const int rest = item - b * per_b;
        j = rest / g.H;
        h = rest - j * g.H;
    };
    TileOffsets off;
    off.set(g.H, tid);
    auto fetch = [&](int item) {  // clamped to the last item: the loads of the item after the last are harmless
        int b, h, j;
        block_of(min(item, n_blk_total - 1), b, h, j);
        load_tile_raw(tile_base(X, seq_stride, g.H, b, h, j), off, raw);
    };
    fetch(blockIdx.x);
    // this thread's place in a block's kept codes: rows of 128 bytes, token-major
    uint32_t keep_at[4];
#pragma unroll
    for (int i = 0; i < 4; i++) keep_at[i] = (uint32_t)(tile_token(tid, i) * kD + tile_chan0(tid));
    for (int item = blockIdx.x; item < n_blk_total; item += gridDim.x) {
        int b_, h_, j_;
        block_of(item, b_, h_, j_);
        const int blk = (b_ * g.H + h_) * n_blk_per_bh + j_;  // where the block's codes and min/max are kept
        TileRegs r;
        unpack_tile(raw, r);
        fetch(item + gridDim.x);  // the next block's loads travel while this one is quantized
        bad |= quantize_tile<WHICH, true>(r, sh, tid, g.two_eb[WHICH], g.n_sym[WHICH], g.k_units);
        // the codes carry kRoundMagicBits (zero in its low 24 bits): the subtraction folds into the address constant,
        // the packing takes the low bytes
#pragma unroll
        for (int i = 0; i < 4; i++)
#pragma unroll
            for (int k = 0; k < 8; k++) atomicAdd(&hist[r.code[i][k] - kRoundMagicBits][copy], 1u);
        if constexpr (KEEP) {
            uint8_t *dst = codes + (size_t)blk * kTile;
#pragma unroll
            for (int i = 0; i < 4; i++) {
                uint2 pk;
                pk.x = pack_low_bytes(r.code[i][0], r.code[i][1], r.code[i][2], r.code[i][3]);
                pk.y = pack_low_bytes(r.code[i][4], r.code[i][5], r.code[i][6], r.code[i][7]);
                *reinterpret_cast<uint2 *>(dst + keep_at[i]) = pk;
            }
            const int units = WHICH == 0 ? g.k_units : kBT;
            if (tid < units)
                minmax[(size_t)blk * units + tid] = float_to_half_bits(sh.unit_mn[tid]) | (float_to_half_bits(sh.unit_mx[tid]) << 16);
            __syncthreads();  // the block's atomics are done
            uint32_t cnt = 0;
            if (tid < g.n_sym[WHICH]) {  // codes stay below the number of levels: the other bins are never touched
                uint4 *mine = reinterpret_cast<uint4 *>(&hist[tid][0]);
#pragma unroll
                for (int c = 0; c < 8; c++) {  // rotated: neighbouring bins start at different banks
                    const uint4 v = mine[(c + tid) & 7];
                    cnt += (v.x + v.y) + (v.z + v.w);
                    mine[(c + tid) & 7] = make_uint4(0, 0, 0, 0);
                }
            }
            total += cnt;
            block_hist[(size_t)blk * 256 + tid] = (uint16_t)cnt;  // at most 8192
        }
        __syncthreads();  // unit_mn/unit_mx are rewritten by the next iteration; KEEP: the histogram is clear again
    }
    if constexpr (!KEEP) {
        __syncthreads();
#pragma unroll
        for (int c = 0; c < 32; c++) total += hist[tid][(c + tid) & 31];  // rotated: conflict-free across the bins
    }
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
    load_tile(X, seq_stride, g.H, bh / g.H, bh % g.H, j, tid, r);
    const bool bad = quantize_tile<WHICH>(r, sh, tid, g.two_eb[WHICH], g.n_sym[WHICH], g.k_units);
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

// codes / minmax / block_hist != NULL: also keep the codes, the unit min/max and the histogram of every block there
hipError_t launch_histogram(const Geo &g, int which, const uint16_t *X, int seq_stride, int n_blk_per_bh,
                            uint8_t *codes, uint32_t *minmax, uint16_t *block_hist, hipStream_t s) {
    const int total = g.B * g.H * n_blk_per_bh;
    if (total <= 0) return hipSuccess;
    const int grid = total < 1024 ? total : 1024;  // four workgroups per CU (32 KiB of LDS each), several blocks each
    const bool keep = codes != nullptr;
    if (which == 0 && !keep)
        hipLaunchKernelGGL((histogram_kernel<0, false>), dim3(grid), dim3(256), 0, s, g, X, seq_stride, n_blk_per_bh, total, codes, minmax, block_hist);
    else if (which == 0)
        hipLaunchKernelGGL((histogram_kernel<0, true>), dim3(grid), dim3(256), 0, s, g, X, seq_stride, n_blk_per_bh, total, codes, minmax, block_hist);
    else if (!keep)
        hipLaunchKernelGGL((histogram_kernel<1, false>), dim3(grid), dim3(256), 0, s, g, X, seq_stride, n_blk_per_bh, total, codes, minmax, block_hist);
    else
        hipLaunchKernelGGL((histogram_kernel<1, true>), dim3(grid), dim3(256), 0, s, g, X, seq_stride, n_blk_per_bh, total, codes, minmax, block_hist);
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

// Copies n16 16-byte units and clears zero16 more at `zero`; src may be pinned host memory (the codebook tables: a copy
// engine transfer of this size was measured at 17 us on the stream, this launch at 4).
__global__ void copy16_kernel(uint4 *__restrict__ dst, const uint4 *__restrict__ src, size_t n16, uint4 *__restrict__ zero,
                              size_t zero16) {
    const size_t stride = (size_t)gridDim.x * blockDim.x, first = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (size_t i = first; i < n16; i += stride) dst[i] = src[i];
    for (size_t i = first; i < zero16; i += stride) zero[i] = make_uint4(0, 0, 0, 0);
}
hipError_t launch_copy16(void *dst, const void *src, size_t bytes, void *zero, size_t zero_bytes, hipStream_t s) {
    const size_t n16 = bytes / 16;
    if (n16 == 0) return hipSuccess;
    size_t grid = (n16 + 255) / 256;
    if (grid > 1024) grid = 1024;
    hipLaunchKernelGGL(copy16_kernel, dim3((unsigned)grid), dim3(256), 0, s, reinterpret_cast<uint4 *>(dst),
                       reinterpret_cast<const uint4 *>(src), n16, reinterpret_cast<uint4 *>(zero), zero_bytes / 16);
    return hipGetLastError();
}

}  // namespace kvc
