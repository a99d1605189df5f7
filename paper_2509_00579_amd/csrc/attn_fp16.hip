// The uncompressed comparison kernel (Section 4.3 compares the fused kernel with a plain fp16 matrix-vector
// product): decode attention on the fp16 cache [B, S, H, 128], sequence split over workgroups with an online
// softmax, merged inside the kernel like the fused path.  HBM-bound: every K and V byte is read once with 16-byte
// loads.  Groups of 1 and 2 query heads form the scores on the vector ALU; groups of 4 and 8 (one K row serves
// several heads, a small matrix product) on the matrix cores.
#include <hip/hip_fp16.h>

#include <mutex>

#include "huff_decode.cuh"
#include "kvcomp_internal.h"
#include "split_combine.cuh"

namespace kvc {

__device__ __forceinline__ float bh2f(uint32_t bits) { return __half2float(__ushort_as_half((unsigned short)bits)); }

__device__ __forceinline__ void unpack8(const uint4 &v, float (&x)[8]) {
    x[0] = bh2f(v.x & 0xffffu); x[1] = bh2f(v.x >> 16);
    x[2] = bh2f(v.y & 0xffffu); x[3] = bh2f(v.y >> 16);
    x[4] = bh2f(v.z & 0xffffu); x[5] = bh2f(v.z >> 16);
    x[6] = bh2f(v.w & 0xffffu); x[7] = bh2f(v.w >> 16);
}

constexpr int kBWaves = 4;

// The waves of a workgroup have left (o[128], m, l) per query head in comb: merge them into the workgroup's partial
// and, in the last workgroup of the (batch, kv head), the splits into the output.
template <int G>
__device__ __forceinline__ void merge_waves_and_splits(const float (&comb)[kBWaves][G][kPartialStride],
                                                       float *__restrict__ partials, uint32_t *__restrict__ counters,
                                                       float *__restrict__ out, int b, int h, int Hq, int split, int bh,
                                                       int tid, int split_stride) {
    for (int i = tid; i < G * kD; i += 64 * kBWaves) {
        const int g = i / kD, c = i - g * kD;
        float M = -INFINITY;
        for (int w = 0; w < kBWaves; w++) M = fmaxf(M, comb[w][g][kD]);
        float L = 0.f, O = 0.f;
        for (int w = 0; w < kBWaves; w++) {
            const float mw = comb[w][g][kD];
            const float f = mw == -INFINITY ? 0.f : __expf(mw - M);
            L += comb[w][g][kD + 1] * f;
            O += comb[w][g][c] * f;
        }
        if (gridDim.x == 1) {
            out[((size_t)b * Hq + (size_t)h * G + g) * kD + c] = O / L;
        } else {
            float *dst = partials + (((size_t)b * Hq + (size_t)h * G + g) * split_stride + split) * kPartialStride;
            store_agent(dst + c, O);
            if (c == 0) { store_agent(dst + kD, M); store_agent(dst + kD + 1, L); }
        }
    }
    if (gridDim.x > 1)
        finish_splits<G>(partials, counters + bh, b * Hq + h * G, (int)gridDim.x, out, tid, 64 * kBWaves, split_stride);
}


// Lane l of a wave owns channels 8*(l%16)..+7 and the tokens 4*i + l/16 (i = 0..15) of a 64-token tile: one load
// instruction of the wave reads four whole 256-byte rows.  The loop is software-pipelined: the K rows of the next
// tile are requested as soon as the scores of the current one are formed, behind the current tile's V rows, so that
// a wave always has 16 KiB (and most of the time 32 KiB) on its way from memory; the 16-lane dot-product sums run on
// DPP row operations, not on LDS permutes.
template <int G>
__global__ __launch_bounds__(64 * kBWaves, 2) void baseline_attn_kernel(int B, int H, int Hq, const uint16_t *__restrict__ K,
                                                                         const uint16_t *__restrict__ V, int seq,
                                                                         const uint16_t *__restrict__ q, float scale,
                                                                         float *__restrict__ partials,
                                                                         uint32_t *__restrict__ counters,
                                                                         float *__restrict__ out, int tokens_per_split, int split_stride) {
    __shared__ float comb[kBWaves][G][kPartialStride];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int split = blockIdx.x, bh = blockIdx.y, b = bh / H, h = bh - b * H;
    const int cc = (lane & 15) * 8, sub = lane >> 4;
    float qr[G][8];
#pragma unroll
    for (int g = 0; g < G; g++) {
        const uint4 v = *reinterpret_cast<const uint4 *>(q + ((size_t)b * Hq + (size_t)h * G + g) * kD + cc);
        unpack8(v, qr[g]);
    }
    float m[G], lsum[G], acc[G][8];
#pragma unroll
    for (int g = 0; g < G; g++) {
        m[g] = -INFINITY;
        lsum[g] = 0.f;
#pragma unroll
        for (int k = 0; k < 8; k++) acc[g][k] = 0.f;
    }
    const int t_begin = split * tokens_per_split;
    const int t_end = min(t_begin + tokens_per_split, seq);
    const size_t row = (size_t)H * kD;  // elements between consecutive tokens
    const uint16_t *Kb = K + ((size_t)b * seq * H + h) * kD + cc;
    const uint16_t *Vb = V + ((size_t)b * seq * H + h) * kD + cc;

    uint4 kv[16];
    auto load_k = [&](int t0) {
#pragma unroll
        for (int i = 0; i < 16; i++) {
            const int t = t0 + 4 * i + sub;
            kv[i] = t < t_end ? *reinterpret_cast<const uint4 *>(Kb + (size_t)t * row) : make_uint4(0, 0, 0, 0);
        }
    };
    int t0 = t_begin + wave * 64;
    if (t0 < t_end) load_k(t0);
    for (; t0 < t_end; t0 += 64 * kBWaves) {
        float s[G][16];
#pragma unroll
        for (int i = 0; i < 16; i++) {
            float x[8];
            unpack8(kv[i], x);
            const bool valid = t0 + 4 * i + sub < t_end;
#pragma unroll
            for (int g = 0; g < G; g++) {
                float d = 0.f;
#pragma unroll
                for (int k = 0; k < 8; k++) d = fmaf(qr[g][k], x[k], d);
                d += dpp_f<kDppXor1>(d);
                d += dpp_f<kDppXor2>(d);
                d += dpp_f<kDppHalfMirror>(d);
                d += dpp_f<kDppMirror>(d);  // the row's 16 lanes all hold its dot product
                s[g][i] = valid ? scale * d : -INFINITY;
            }
        }
        uint4 vv[16];
#pragma unroll
        for (int i = 0; i < 16; i++) {
            const int t = t0 + 4 * i + sub;
            vv[i] = t < t_end ? *reinterpret_cast<const uint4 *>(Vb + (size_t)t * row) : make_uint4(0, 0, 0, 0);
        }
        if (t0 + 64 * kBWaves < t_end) load_k(t0 + 64 * kBWaves);  // behind the V rows: they are waited for first
        float p[G][16];
#pragma unroll
        for (int g = 0; g < G; g++) {
            float ml = s[g][0];
#pragma unroll
            for (int i = 1; i < 16; i++) ml = fmaxf(ml, s[g][i]);
            ml = fmaxf(ml, __shfl_xor(ml, 16));
            ml = fmaxf(ml, __shfl_xor(ml, 32));
            const float mnew = fmaxf(m[g], ml);
            const float alpha = __expf(m[g] - mnew);
            m[g] = mnew;
            float ps = 0.f;
#pragma unroll
            for (int i = 0; i < 16; i++) {
                p[g][i] = __expf(s[g][i] - mnew);
                ps += p[g][i];
            }
            lsum[g] = lsum[g] * alpha + ps;
#pragma unroll
            for (int k = 0; k < 8; k++) acc[g][k] *= alpha;
        }
#pragma unroll
        for (int i = 0; i < 16; i++) {
            float x[8];
            unpack8(vv[i], x);
#pragma unroll
            for (int g = 0; g < G; g++)
#pragma unroll
                for (int k = 0; k < 8; k++) acc[g][k] = fmaf(p[g][i], x[k], acc[g][k]);
        }
    }
    // reduce the four token sub-groups of the wave, then the waves of the workgroup
#pragma unroll
    for (int g = 0; g < G; g++) {
        lsum[g] += __shfl_xor(lsum[g], 16);
        lsum[g] += __shfl_xor(lsum[g], 32);
#pragma unroll
        for (int k = 0; k < 8; k++) {
            acc[g][k] += __shfl_xor(acc[g][k], 16);
            acc[g][k] += __shfl_xor(acc[g][k], 32);
        }
        if (sub == 0) {
#pragma unroll
            for (int k = 0; k < 8; k++) comb[wave][g][cc + k] = acc[g][k];
        }
        if (lane == 0) {
            comb[wave][g][kD] = m[g];
            comb[wave][g][kD + 1] = lsum[g];
        }
    }
    __syncthreads();
    merge_waves_and_splits<G>(comb, partials, counters, out, b, h, Hq, split, bh, tid, split_stride);
}

// ---- groups of 4 and 8 query heads --------------------------------------------------------------------------------
// Scores of 16 tokens x (up to 16) heads per v_mfma_f32_16x16x16_f16: S^T = K Q^T, A = K tile, B = Q^T.
//   A: lane l holds row (token) l % 16, reduction slots 4 * (l / 16) .. + 3
//   B: lane l holds column (head) l % 16, the same slots;  D: lane l holds column l % 16, rows 4 * (l / 16) .. + 3
// Which channel a reduction slot stands for is free as long as A and B agree: step (i, hh) maps slot (l / 16, r) to
// channel 8 * (l / 16 + 4 i) + 4 hh + r, so that a lane's A operands for two steps are one 16-byte load of its K row.
// The P V product stays on the vector ALU (lane = 8 channels x one token in four, as in the kernel above); the
// softmax numerators reach it through LDS.
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef float float4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ half4_t as_half4(uint32_t lo, uint32_t hi) {
    const uint2 v = make_uint2(lo, hi);
    return __builtin_bit_cast(half4_t, v);
}
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int G>
__global__ __launch_bounds__(64 * kBWaves, G == 8 ? 2 : 3) void baseline_attn_gqa_kernel(
    int B, int H, int Hq, const uint16_t *__restrict__ K, const uint16_t *__restrict__ V, int seq,
    const uint16_t *__restrict__ q, float scale, float *__restrict__ partials, uint32_t *__restrict__ counters,
    float *__restrict__ out, int tokens_per_split, int split_stride) {
    static_assert(G == 4 || G == 8, "group size");
    __shared__ float comb[kBWaves][G][kPartialStride];
    __shared__ __attribute__((aligned(16))) float p_s[kBWaves][64][G];  // numerators of the wave's current tokens
    __shared__ float alpha_s[kBWaves][G];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int split = blockIdx.x, bh = blockIdx.y, b = bh / H, h = bh - b * H;
    const int j = lane & 15, gq = lane >> 4;  // matrix column / row group;  V phase: channels 8 j .. + 7, tokens 4 i + gq
    const int cc = j * 8;
    half4_t qb[4][2];
#pragma unroll
    for (int i = 0; i < 4; i++) {
        uint4 v = make_uint4(0, 0, 0, 0);
        if (j < G) v = *reinterpret_cast<const uint4 *>(q + ((size_t)b * Hq + (size_t)h * G + j) * kD + 8 * (gq + 4 * i));
        qb[i][0] = as_half4(v.x, v.y);
        qb[i][1] = as_half4(v.z, v.w);
    }
    float m = -INFINITY, lsum = 0.f;  // running maximum and sum of head j (lanes with j >= G idle along)
    float acc[G][8];
#pragma unroll
    for (int g = 0; g < G; g++)
#pragma unroll
        for (int k = 0; k < 8; k++) acc[g][k] = 0.f;
    const int t_begin = split * tokens_per_split;
    const int t_end = min(t_begin + tokens_per_split, seq);
    const size_t row = (size_t)H * kD;
    const uint16_t *Kb = K + ((size_t)b * seq * H + h) * kD + 8 * gq;
    const uint16_t *Vb = V + ((size_t)b * seq * H + h) * kD + cc;

    uint4 kv[16];
    auto load_k = [&](int t0) {
#pragma unroll
        for (int tt = 0; tt < 4; tt++) {
            const int t = t0 + 16 * tt + j;
#pragma unroll
            for (int i = 0; i < 4; i++)
                kv[tt * 4 + i] = t < t_end ? *reinterpret_cast<const uint4 *>(Kb + (size_t)t * row + 32 * i)
                                           : make_uint4(0, 0, 0, 0);
        }
    };
    // Groups of 8 run two waves per SIMD anyway (their accumulators) and have the registers to request the next
    // tile's K rows early; groups of 4 are better off with three waves per SIMD and no look-ahead (measured).
    constexpr bool kAhead = G == 8;
    int t0 = t_begin + wave * 64;
    if (kAhead && t0 < t_end) load_k(t0);
    for (; t0 < t_end; t0 += 64 * kBWaves) {
        if (!kAhead) load_k(t0);
        float s[16];
        float ml = -INFINITY;
#pragma unroll
        for (int tt = 0; tt < 4; tt++) {
            float4_t d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int i = 0; i < 4; i++) {
                const uint4 &v = kv[tt * 4 + i];
                d = __builtin_amdgcn_mfma_f32_16x16x16f16(as_half4(v.x, v.y), qb[i][0], d, 0, 0, 0);
                d = __builtin_amdgcn_mfma_f32_16x16x16f16(as_half4(v.z, v.w), qb[i][1], d, 0, 0, 0);
            }
            const float dd[4] = {d.x, d.y, d.z, d.w};
#pragma unroll
            for (int r = 0; r < 4; r++) {  // token t0 + 16 tt + 4 gq + r, head j
                s[tt * 4 + r] = t0 + 16 * tt + 4 * gq + r < t_end ? scale * dd[r] : -INFINITY;
                ml = fmaxf(ml, s[tt * 4 + r]);
            }
        }
        ml = fmaxf(ml, __shfl_xor(ml, 16));
        ml = fmaxf(ml, __shfl_xor(ml, 32));
        const float mnew = fmaxf(m, ml);  // finite: the tile holds at least one token
        const float alpha = __expf(m - mnew);
        m = mnew;
        float ps = 0.f;
#pragma unroll
        for (int tt = 0; tt < 4; tt++)
#pragma unroll
            for (int r = 0; r < 4; r++) {
                const float pv = __expf(s[tt * 4 + r] - mnew);
                ps += pv;
                if (j < G) p_s[wave][16 * tt + 4 * gq + r][j] = pv;
            }
        lsum = lsum * alpha + ps;
        if (gq == 0 && j < G) alpha_s[wave][j] = alpha;
        wave_lds_sync();
#pragma unroll
        for (int g = 0; g < G; g++) {
            const float al = alpha_s[wave][g];
#pragma unroll
            for (int k = 0; k < 8; k++) acc[g][k] *= al;
        }
        // the K rows of the next tile travel with the V rows of this one (the scores above were their last use)
        if (kAhead && t0 + 64 * kBWaves < t_end) load_k(t0 + 64 * kBWaves);
        constexpr int kChunk = G == 8 ? 8 : 16;  // V rows in flight per lane (register budget)
#pragma unroll 1
        for (int i0 = 0; i0 < 16; i0 += kChunk) {
            uint4 vv[kChunk];
#pragma unroll
            for (int i = 0; i < kChunk; i++) {
                const int t = t0 + 4 * (i0 + i) + gq;
                vv[i] = t < t_end ? *reinterpret_cast<const uint4 *>(Vb + (size_t)t * row) : make_uint4(0, 0, 0, 0);
            }
#pragma unroll
            for (int i = 0; i < kChunk; i++) {
                float x[8];
                unpack8(vv[i], x);
                float pg[G];
#pragma unroll
                for (int g4 = 0; g4 < G; g4 += 4) {
                    const float4 t4 = *reinterpret_cast<const float4 *>(&p_s[wave][4 * (i0 + i) + gq][g4]);
                    pg[g4] = t4.x; pg[g4 + 1] = t4.y; pg[g4 + 2] = t4.z; pg[g4 + 3] = t4.w;
                }
#pragma unroll
                for (int g = 0; g < G; g++)
#pragma unroll
                    for (int k = 0; k < 8; k++) acc[g][k] = fmaf(pg[g], x[k], acc[g][k]);
            }
        }
        wave_lds_sync();  // the next tile overwrites p_s
    }
    lsum += __shfl_xor(lsum, 16);
    lsum += __shfl_xor(lsum, 32);
    if (gq == 0 && j < G) {
        comb[wave][j][kD] = m;
        comb[wave][j][kD + 1] = lsum;
    }
#pragma unroll
    for (int g = 0; g < G; g++) {
#pragma unroll
        for (int k = 0; k < 8; k++) {
            acc[g][k] += __shfl_xor(acc[g][k], 16);
            acc[g][k] += __shfl_xor(acc[g][k], 32);
        }
        if (gq == 0) {
#pragma unroll
            for (int k = 0; k < 8; k++) comb[wave][g][cc + k] = acc[g][k];
        }
    }
    __syncthreads();
    merge_waves_and_splits<G>(comb, partials, counters, out, b, h, Hq, split, bh, tid, split_stride);
}

// ---- a plain streaming read: the bound for any kernel that has to read the fp16 cache ---------------------------------
// Every workgroup reads one contiguous chunk with 16-byte loads, eight in flight per lane, and folds the words;
// the fold is stored only if it equals a value the caller's data does not produce (the loads must not be optimised
// away), so normally nothing is written.
constexpr int kStreamLoads = 8;
__global__ __launch_bounds__(256) void read_stream_kernel(const uint4 *__restrict__ src, size_t per_wg16,
                                                          uint32_t *__restrict__ sink) {
    const uint4 *p = src + (size_t)blockIdx.x * per_wg16 + threadIdx.x;
    uint32_t acc = 0;
    for (size_t i = 0; i < per_wg16; i += 256 * kStreamLoads) {
        uint4 v[kStreamLoads];
#pragma unroll
        for (int u = 0; u < kStreamLoads; u++) v[u] = p[i + (size_t)u * 256];
#pragma unroll
        for (int u = 0; u < kStreamLoads; u++) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    if (acc == 0x9e3779b9u && threadIdx.x == 1023) sink[0] = acc;  // never: blockDim.x is 256
}

// Up to 2048 workgroups, each reading a whole number of 32 KiB pieces (256 lanes x 8 loads x 16 bytes); *bytes_read
// receives what is read in total (the largest such amount that fits into `bytes`).
hipError_t launch_read_stream(const void *src, size_t bytes, uint32_t *sink, size_t *bytes_read, hipStream_t s) {
    const size_t piece = (size_t)256 * kStreamLoads * 16;
    const size_t grid = bytes / piece < 2048 ? bytes / piece : 2048;
    *bytes_read = 0;
    if (grid == 0) return hipSuccess;
    const size_t per_wg = bytes / grid / piece * piece;
    *bytes_read = per_wg * grid;
    hipLaunchKernelGGL(read_stream_kernel, dim3((unsigned)grid), dim3(256), 0, s, static_cast<const uint4 *>(src),
                       per_wg / 16, sink);
    return hipGetLastError();
}

// ---- scratch of the entry point that allocates nothing ---------------------------------------------------------
// kvcomp_baseline_fp16_attn_noalloc keeps the split tickets and the split partials in this array instead of a
// caller's workspace.  Every GPU holds its own copy at its own address until the process ends.  Layout: tickets (one
// per (batch, kv head), zero between launches: the merging workgroup resets its ticket) in the first
// kStaticTicketBytes, the partials [batch * q heads][splits used][130] fp32 behind them.
constexpr size_t kStaticTicketBytes = 64 * 1024;    // 16384 (batch, kv head) pairs
constexpr size_t kStaticScratchBytes = 4u << 20;    // tickets + partials
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// Device address of `scratch` on the current device (the array's name is a host-side stand-in, not an address that a
// kernel may be given), looked up once per device.
hipError_t baseline_static_scratch(uint32_t **tickets, float **partials, size_t *max_tickets, size_t *partial_bytes) {
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static unsigned char *per_device[kMaxDevices] = {};
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    unsigned char *ptr;
    {
        std::lock_guard<std::mutex> lock(mu);
        if (!per_device[dev]) {
            void *p = nullptr;
            e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
            if (e != hipSuccess) return e;
            if (!p) return hipErrorInvalidSymbol;
            per_device[dev] = static_cast<unsigned char *>(p);
        }
        ptr = per_device[dev];
    }
    *tickets = reinterpret_cast<uint32_t *>(ptr);
    *partials = reinterpret_cast<float *>(ptr + kStaticTicketBytes);
    *max_tickets = kStaticTicketBytes / sizeof(uint32_t);
    *partial_bytes = kStaticScratchBytes - kStaticTicketBytes;
    return hipSuccess;
}

// Sequence splits that a launch really uses for `seq` tokens when n_splits are asked for (whole 64-token tiles).
int baseline_splits(int seq, int n_splits) {
    int tps = (seq + n_splits - 1) / n_splits;
    tps = (tps + 63) / 64 * 64;
    return (seq + tps - 1) / tps;
}

// split_stride: splits per query head that the layout of `partials` has room for (>= the splits used)
hipError_t launch_baseline_attn(int B, int H, int Hq, const uint16_t *K, const uint16_t *V, int seq, const uint16_t *q,
                                float scale, float *out, float *partials, uint32_t *counters, int n_splits,
                                int split_stride, hipStream_t s) {
    const int G = Hq / H;
    int tps = (seq + n_splits - 1) / n_splits;
    tps = (tps + 63) / 64 * 64;
    n_splits = (seq + tps - 1) / tps;
    if (n_splits > split_stride) return hipErrorInvalidValue;
    const dim3 grid(n_splits, B * H), block(64 * kBWaves);
    switch (G) {
        case 1: hipLaunchKernelGGL(baseline_attn_kernel<1>, grid, block, 0, s, B, H, Hq, K, V, seq, q, scale, partials, counters, out, tps, split_stride); break;
        case 2: hipLaunchKernelGGL(baseline_attn_kernel<2>, grid, block, 0, s, B, H, Hq, K, V, seq, q, scale, partials, counters, out, tps, split_stride); break;
        case 4: hipLaunchKernelGGL(baseline_attn_gqa_kernel<4>, grid, block, 0, s, B, H, Hq, K, V, seq, q, scale, partials, counters, out, tps, split_stride); break;
        case 8: hipLaunchKernelGGL(baseline_attn_gqa_kernel<8>, grid, block, 0, s, B, H, Hq, K, V, seq, q, scale, partials, counters, out, tps, split_stride); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace kvc
