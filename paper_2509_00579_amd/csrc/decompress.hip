// Stand-alone decompression: the first stage of the multi-kernel pipeline that Section 4.3 compares the fused kernel
// with (decode -> dequantize -> write the cache back in its own precision; a separate matrix-vector kernel then reads
// it).  One wave per 2D block: the record is staged in LDS, decoded with the same table decoder as the fused kernel
// (four chains per lane) into a code tile in LDS, and written out as fp16 rows with 16-byte stores,
//     x' = fp16( min + float(code) * width ),   binary32 multiply, binary32 add, one rounding.
#include "huff_decode.cuh"
#include "kvcomp_internal.h"

namespace kvc {

constexpr int kDecWaves = 4;
constexpr int kTileRow = kD + 8;  // padded row of the code tile (bytes; keeps 8-byte reads aligned)

struct DecompArgs {
    Geo g;
    uint16_t *out;
    int which, n_blocks, seq_stride, stage_bytes;
    uint32_t mask2;
};

// One chain of the bit-serial decoder of Section 3.3.1: one stream bit per step, node = tree[node][bit], a symbol
// is emitted and the walk restarts at the root when a leaf is reached; no branch depends on the data.
struct TreeWalk {
    int node, count;  // current inner node, symbols emitted so far
    __device__ __forceinline__ void init() { node = 0; count = 0; }
    // returns the symbol (>= 0) if this bit completed a code word of a chain that still has symbols to give, else -1
    __device__ __forceinline__ int step(const int16_t *tree, uint32_t bit) {
        const int next = tree[node * 2 + (int)bit];
        const bool leaf = next < 0, live = count < kHalf;
        node = leaf ? 0 : next;
        const int sym = (leaf && live) ? ~next : -1;
        count += (leaf && live) ? 1 : 0;
        return sym;
    }
};

// LB > 0: table decoder compiled for code words of up to LB bits.  LB == 0: the paper's bit-serial tree walk, kept for
// an A/B on this hardware.
template <int LB>
__global__ __launch_bounds__(64 * kDecWaves) void decompress_kernel(DecompArgs a) {
    constexpr bool kTree = LB == 0;
    constexpr int kWindowBits = 31;  // stream bits per window of 16-bit table entries
    constexpr int NS = kTree ? 1 : kWindowBits / (kTree ? 1 : LB);
    __shared__ __attribute__((aligned(16))) uint16_t lut_s[kTree ? 512 : (1 << LB)];
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];  // per wave: record staging, then the code tile
    const Geo &g = a.g;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int which = a.which;
    if constexpr (kTree) {  // the tree of this tensor: 256 nodes x 2 children, 16 bits each
        const uint4 *src = reinterpret_cast<const uint4 *>(tree_of(g, which));
        for (int i = tid; i < 64; i += 64 * kDecWaves) reinterpret_cast<uint4 *>(lut_s)[i] = src[i];
    } else {
        const uint4 *src = reinterpret_cast<const uint4 *>(lut_of(g, which));
        uint4 *dst = reinterpret_cast<uint4 *>(lut_s);
        const int n16 = max(1, (2 << g.lut_bits[which]) / 16);
        for (int i = tid; i < n16; i += 64 * kDecWaves) dst[i] = src[i];
    }
    __syncthreads();
    const long long item = (long long)blockIdx.x * kDecWaves + wave;  // (b*H + h) * n_blocks + j
    if (item >= (long long)g.B * g.H * a.n_blocks) return;
    const int bh = (int)(item / a.n_blocks), j = (int)(item - (long long)bh * a.n_blocks);
    const int b = bh / g.H, h = bh - b * g.H;
    uint8_t *stage = smem + (size_t)wave * (a.stage_bytes + kBT * kTileRow);
    uint8_t *tile = stage + a.stage_bytes;
    const BlockEntry e = g.table[((size_t)which * g.B * g.H + bh) * g.max_blocks + j];
    const uint32_t size16 = __builtin_amdgcn_readfirstlane(e.size16), off16 = __builtin_amdgcn_readfirstlane(e.off16);
    const uint4 *src = reinterpret_cast<const uint4 *>(g.payload + (size_t)off16 * 16);
    // a record larger than the staging area (the host sizes it from the largest record, so only a corrupted table gets
    // here) is not decoded: the fault bit makes the next synchronising call fail
    if (size16 * 16u + 16u > (uint32_t)a.stage_bytes) {
        if (lane == 0) atomicOr(&g.ctrl->fault, kFaultStageSmall);
        return;
    }
    for (uint32_t i = lane; i < size16; i += 64) reinterpret_cast<uint4 *>(stage)[i] = src[i];
    wave_sync();
    const uint32_t *hdr32 = reinterpret_cast<const uint32_t *>(stage);
    const int mmb = which == 0 ? g.k_minmax_bytes : kMinMaxBytesV;
    const uint32_t sb = hdr32[mmb / 4 + lane];
    const uint32_t start = wave_excl_scan((sb & 0xffffu) + (sb >> 16), lane);
    const uint32_t *wm1 = hdr32 + (mmb + 2 * kSlices) / 4 - 1;
    const char *lut = reinterpret_cast<const char *>(lut_s);
    Quad<1> qd;
    qd.open(wm1, start, sb & 0xffffu, sb >> 16);
    constexpr int kRounds = kHalf / NS, kTail = kHalf - kRounds * NS;
    // K: lane = token, chains au/ad = channels 0..63 (up / down), bu/bd = channels 64..127
    // V: lane = channels 2*lane (au/ad) and 2*lane+1 (bu/bd), symbol index = token
    auto put = [&](int idx, uint32_t eu, uint32_t ed, uint32_t fu, uint32_t fd) {
        const int up = idx, dn = kSliceLen - 1 - idx;
        if (which == 0) {
            tile[lane * kTileRow + up] = (uint8_t)(eu >> 8);
            tile[lane * kTileRow + dn] = (uint8_t)(ed >> 8);
            tile[lane * kTileRow + kSliceLen + up] = (uint8_t)(fu >> 8);
            tile[lane * kTileRow + kSliceLen + dn] = (uint8_t)(fd >> 8);
        } else {
            tile[up * kTileRow + 2 * lane] = (uint8_t)(eu >> 8);
            tile[dn * kTileRow + 2 * lane] = (uint8_t)(ed >> 8);
            tile[up * kTileRow + 2 * lane + 1] = (uint8_t)(fu >> 8);
            tile[dn * kTileRow + 2 * lane + 1] = (uint8_t)(fd >> 8);
        }
    };
    if constexpr (kTree) {
        // All four chains of the lane walk one bit per step; a window gives 31 bits, then every reader moves on by
        // 31.  A chain stops emitting after its 32 symbols; the wave runs until every chain of every lane is done.
        const int16_t *tree = reinterpret_cast<const int16_t *>(lut_s);
        TreeWalk tw[4];
#pragma unroll
        for (int c = 0; c < 4; c++) tw[c].init();
        auto emit = [&](int c, int sym, int idx) {  // chain c emitted its idx-th symbol
            if (sym < 0) return;
            const int pos = (c & 1) ? kSliceLen - 1 - idx : idx;  // chains 1 and 3 read downwards
            if (which == 0) tile[lane * kTileRow + (c >> 1) * kSliceLen + pos] = (uint8_t)sym;
            else tile[pos * kTileRow + 2 * lane + (c >> 1)] = (uint8_t)sym;
        };
        // 32 symbols of at most 12 bits need at most 13 windows of 31 bits: the bound also ends the loop on a
        // damaged table
        bool busy = true;
        for (int round = 0; round < 16 && busy; round++) {
            uint32_t w0 = qd.au.window(wm1) >> 1, w1 = qd.ad.window(wm1) >> 1;
            uint32_t w2 = qd.bu.window(wm1) >> 1, w3 = qd.bd.window(wm1) >> 1;
#pragma unroll 1
            for (int k = 0; k < kWindowBits; k++) {
                const int i0 = tw[0].count, i1 = tw[1].count, i2 = tw[2].count, i3 = tw[3].count;
                emit(0, tw[0].step(tree, w0 & 1u), i0);
                emit(1, tw[1].step(tree, w1 & 1u), i1);
                emit(2, tw[2].step(tree, w2 & 1u), i2);
                emit(3, tw[3].step(tree, w3 & 1u), i3);
                w0 >>= 1; w1 >>= 1; w2 >>= 1; w3 >>= 1;
            }
            qd.au.advance(wm1, kWindowBits);
            qd.ad.advance(wm1, kWindowBits);
            qd.bu.advance(wm1, kWindowBits);
            qd.bd.advance(wm1, kWindowBits);
            const bool mine = tw[0].count < kHalf || tw[1].count < kHalf || tw[2].count < kHalf || tw[3].count < kHalf;
            busy = __any(mine);
        }
    } else {
#pragma unroll 2
        for (int r = 0; r < kRounds; r++) {
            uint32_t fau[NS], fad[NS], fbu[NS], fbd[NS];
            qd.template step<NS>(wm1, lut, a.mask2, fau, fad, fbu, fbd);
#pragma unroll
            for (int k = 0; k < NS; k++) put(r * NS + k, fau[k], fad[k], fbu[k], fbd[k]);
        }
        if constexpr (kTail > 0) {
            uint32_t fau[kTail], fad[kTail], fbu[kTail], fbd[kTail];
            qd.template step<kTail>(wm1, lut, a.mask2, fau, fad, fbu, fbd);
#pragma unroll
            for (int k = 0; k < kTail; k++) put(kRounds * NS + k, fau[k], fad[k], fbu[k], fbd[k]);
        }
    }
    wave_sync();
    // dequantize and write: instruction i covers tokens 4 i + lane / 16, channels 8 (lane % 16) .. + 7 (four rows)
    const int c0 = (lane & 15) * 8, sub = lane >> 4;
    const float two_eb = g.two_eb[which];
    float mn[8], st[8];
    if (which == 0) {
#pragma unroll
        for (int k = 0; k < 8; k++) {
            const uint32_t mm = hdr32[g.k_units == 1 ? 0 : c0 + k];
            mn[k] = h2f(mm & 0xffffu);
            st[k] = two_eb * (h2f(mm >> 16) - mn[k]);
        }
    }
    uint16_t *dst = a.out + (((size_t)b * a.seq_stride + (size_t)j * kBT) * g.H + h) * kD + c0;
#pragma unroll 4
    for (int i = 0; i < 16; i++) {
        const int t = 4 * i + sub;
        if (which == 1) {
            const uint32_t mm = hdr32[t];
            const float m1 = h2f(mm & 0xffffu), s1 = two_eb * (h2f(mm >> 16) - m1);
#pragma unroll
            for (int k = 0; k < 8; k++) { mn[k] = m1; st[k] = s1; }
        }
        const uint2 cb = *reinterpret_cast<const uint2 *>(tile + t * kTileRow + c0);
        const uint32_t w[2] = {cb.x, cb.y};
        uint32_t hv[8];
#pragma unroll
        for (int k = 0; k < 8; k++) {
            const float code = (float)((w[k >> 2] >> (8 * (k & 3))) & 0xffu);
            const float prod = code * st[k];
            const float v = mn[k] + prod;
            hv[k] = (uint32_t)__half_as_ushort(__float2half_rn(v));
        }
        uint4 o;
        o.x = hv[0] | (hv[1] << 16); o.y = hv[2] | (hv[3] << 16); o.z = hv[4] | (hv[5] << 16); o.w = hv[6] | (hv[7] << 16);
        *reinterpret_cast<uint4 *>(dst + (size_t)t * g.H * kD) = o;
    }
}

// the buffered fp16 tokens follow the blocks: token r of the buffer (oldest first) sits in slot
// (res_head + r) mod res_tokens of the ring
__global__ void decompress_tail_kernel(Geo g, int which, uint16_t *out, int n_blocks, int res_head, int n_res,
                                       int seq_stride) {
    const size_t res_tensor = (size_t)g.B * g.res_tokens * g.H * kD;
    const size_t per_tok = (size_t)g.H * kD / 8;  // 16-byte units
    const size_t per_b = (size_t)n_res * per_tok;
    const size_t n16 = (size_t)g.B * per_b;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x) {
        const size_t b = i / per_b, rem = i - b * per_b;  // rem indexes [r][h][c/8]
        const size_t r = rem / per_tok, in_tok = rem - r * per_tok;
        size_t slot = (size_t)res_head + r;
        if (slot >= (size_t)g.res_tokens) slot -= (size_t)g.res_tokens;
        const uint4 v = reinterpret_cast<const uint4 *>(g.res + which * res_tensor +
                                                        (b * g.res_tokens + slot) * g.H * kD)[in_tok];
        reinterpret_cast<uint4 *>(out + ((size_t)b * seq_stride + (size_t)n_blocks * kBT) * g.H * kD)[rem] = v;
    }
}

template <int LB>
static hipError_t launch_dec(const DecompArgs &a, size_t lds, int grid, hipStream_t s) {
    static size_t attr_set = 0;
    if (lds > attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&decompress_kernel<LB>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set = lds;
    }
    hipLaunchKernelGGL((decompress_kernel<LB>), dim3(grid), dim3(64 * kDecWaves), lds, s, a);
    return hipGetLastError();
}

hipError_t launch_decompress(const Geo &g, int which, uint16_t *out, int n_blocks, int res_head, int n_res, int seq_stride,
                             int stage_bytes, int tree_walk, hipStream_t s) {
    if (n_blocks > 0) {
        DecompArgs a;
        a.g = g;
        a.out = out;
        a.which = which;
        a.n_blocks = n_blocks;
        a.seq_stride = seq_stride;
        a.stage_bytes = stage_bytes;
        const int bits = g.lut_bits[which];
        if (bits < 1 || bits > kLutBits) return hipErrorInvalidValue;
        a.mask2 = ((1u << bits) - 1u) << 1;
        const size_t lds = (size_t)kDecWaves * ((size_t)stage_bytes + kBT * kTileRow);
        const long long items = (long long)g.B * g.H * n_blocks;
        const int grid = (int)((items + kDecWaves - 1) / kDecWaves);
        hipError_t e;
        if (tree_walk) {
            e = launch_dec<0>(a, lds, grid, s);
        } else
        switch (fused_table_bits(bits)) {
            case 6:
            case 7: e = launch_dec<7>(a, lds, grid, s); break;
            case 8: e = launch_dec<8>(a, lds, grid, s); break;
            case 10: e = launch_dec<10>(a, lds, grid, s); break;
            default: e = launch_dec<12>(a, lds, grid, s); break;
        }
        if (e != hipSuccess) return e;
    }
    if (n_res > 0) {
        hipLaunchKernelGGL(decompress_tail_kernel, dim3(64), dim3(256), 0, s, g, which, out, n_blocks, res_head, n_res,
                           seq_stride);
        return hipGetLastError();
    }
    return hipSuccess;
}

}  // namespace kvc
