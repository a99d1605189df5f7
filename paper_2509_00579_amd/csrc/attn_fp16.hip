// The uncompressed comparison kernel (Section 4.3 compares the fused kernel with a plain fp16 matrix-vector
// product): decode attention on the fp16 cache [B, S, H, 128], sequence split over workgroups with an online
// softmax, merged by the same combine kernel as the fused path.  HBM-bound: every K and V byte is read once with
// 16-byte loads, four 256-byte rows per wave instruction.
#include <hip/hip_fp16.h>

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

// Lane l of a wave owns channels 8*(l%16)..+7 and the tokens 4*i + l/16 (i = 0..15) of a 64-token tile.
template <int G>
__global__ __launch_bounds__(64 * kBWaves) void baseline_attn_kernel(int B, int H, int Hq, const uint16_t *__restrict__ K,
                                                                      const uint16_t *__restrict__ V, int seq,
                                                                      const uint16_t *__restrict__ q, float scale,
                                                                      float *__restrict__ partials,
                                                                      uint32_t *__restrict__ counters,
                                                                      float *__restrict__ out, int tokens_per_split) {
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

    for (int t0 = t_begin + wave * 64; t0 < t_end; t0 += 64 * kBWaves) {
        float s[G][16];
        uint4 kv[16];
#pragma unroll
        for (int i = 0; i < 16; i++) {
            const int t = t0 + 4 * i + sub;
            kv[i] = t < t_end ? *reinterpret_cast<const uint4 *>(Kb + (size_t)t * row) : make_uint4(0, 0, 0, 0);
        }
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
#pragma unroll
                for (int msk = 1; msk < 16; msk <<= 1) d += __shfl_xor(d, msk);
                s[g][i] = valid ? scale * d : -INFINITY;
            }
        }
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
            const int t = t0 + 4 * i + sub;
            const uint4 v = t < t_end ? *reinterpret_cast<const uint4 *>(Vb + (size_t)t * row) : make_uint4(0, 0, 0, 0);
            float x[8];
            unpack8(v, x);
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
            float *dst = partials + (((size_t)b * Hq + (size_t)h * G + g) * kMaxSplits + split) * kPartialStride;
            store_agent(dst + c, O);
            if (c == 0) { store_agent(dst + kD, M); store_agent(dst + kD + 1, L); }
        }
    }
    if (gridDim.x > 1)
        finish_splits<G, 64 * kBWaves>(partials, counters + bh, b * Hq + h * G, (int)gridDim.x, out, tid);
}

hipError_t launch_baseline_attn(int B, int H, int Hq, const uint16_t *K, const uint16_t *V, int seq, const uint16_t *q,
                                float scale, float *out, float *partials, uint32_t *counters, int n_splits,
                                hipStream_t s) {
    const int G = Hq / H;
    int tps = (seq + n_splits - 1) / n_splits;
    tps = (tps + 63) / 64 * 64;
    n_splits = (seq + tps - 1) / tps;
    const dim3 grid(n_splits, B * H), block(64 * kBWaves);
    switch (G) {
        case 1: hipLaunchKernelGGL(baseline_attn_kernel<1>, grid, block, 0, s, B, H, Hq, K, V, seq, q, scale, partials, counters, out, tps); break;
        case 2: hipLaunchKernelGGL(baseline_attn_kernel<2>, grid, block, 0, s, B, H, Hq, K, V, seq, q, scale, partials, counters, out, tps); break;
        case 4: hipLaunchKernelGGL(baseline_attn_kernel<4>, grid, block, 0, s, B, H, Hq, K, V, seq, q, scale, partials, counters, out, tps); break;
        case 8: hipLaunchKernelGGL(baseline_attn_kernel<8>, grid, block, 0, s, B, H, Hq, K, V, seq, q, scale, partials, counters, out, tps); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace kvc
