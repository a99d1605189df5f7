// Fetch side (Section 3.3, Figure 1): one decode-attention step straight from the compressed cache.
//
// Per 2D block a single wavefront (64 lanes) stages the K record in LDS, every lane Huffman-decodes the slice of
// one token (128 symbols) with a 12-bit lookup table and accumulates q.k in registers; the wave then updates a
// running softmax and decodes the V record of the same block, every lane owning two channels (two slices of 64
// symbols) and accumulating p.v in registers.  No decompressed value ever leaves the registers (Section 3.3.2).
//
// What differs from the paper's kernel, and why (gfx950):
//  * lookup-table decode instead of the bit-serial tree walk of Section 3.3.1: all 64 lanes of a wave advance in
//    symbol lock-step (same trip count for every lane, no divergence), so the dequantization weight of the current
//    symbol is the same for the whole wave and is read from LDS as a broadcast;
//  * the dequantization is folded into the weights: q.k' = sum_c q_c min_c + sum_c (q_c step_c) code_tc, and
//    p.v'  = sum_t p_t min_t + sum_t (p_t step_t) code_tc: one convert and one FMA per decoded symbol;
//  * K and V of a block are handled by the same wave back to back with an online softmax, so scores never go to
//    memory and the sequence is split over workgroups; a small second kernel merges the splits (the "sum
//    reduction" of Section 3.3.2).
#include <hip/hip_fp16.h>

#include "kvcomp_internal.h"

namespace kvc {

__device__ __forceinline__ void wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ __forceinline__ float h2f(uint32_t bits) { return __half2float(__ushort_as_half((unsigned short)bits)); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v = fmaxf(v, __shfl_xor(v, m));
    return v;
}
// exclusive prefix sum over the 64 lanes; *total receives the sum
__device__ __forceinline__ uint32_t wave_excl_scan(uint32_t v, int lane, uint32_t *total) {
    uint32_t inc = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t o = __shfl_up(inc, d);
        if (lane >= d) inc += o;
    }
    *total = __shfl(inc, 63);
    return inc - v;
}

// One lane's view of a bit stream: a 64-bit window {hi,lo} over consecutive 32-bit words, `s` = position of the
// next unread bit inside lo.  Bit i of the stream is bit (i % 32) of word (i / 32).
struct BitReader {
    uint32_t lo, hi, s, next;
    template <class Src>
    __device__ __forceinline__ void open(const Src &src, uint32_t bitpos) {
        const uint32_t w = bitpos >> 5;
        s = bitpos & 31u;
        lo = src.word(w);
        hi = src.word(w + 1);
        next = w + 2;
    }
    // returns the table entry of the next symbol and consumes its bits
    template <class Src>
    __device__ __forceinline__ uint32_t get(const Src &src, const uint16_t *lut) {
        const uint32_t win = __builtin_amdgcn_alignbit(hi, lo, s);
        const uint32_t e = lut[win & (kLutSize - 1)];
        s += e & 0xffu;
        if (s >= 32u) {
            lo = hi;
            hi = src.word(next++);
            s -= 32u;
        }
        return e;
    }
};

struct WordSrc {  // payload words, either staged in LDS or in global memory
    const uint32_t *base;
    __device__ __forceinline__ uint32_t word(uint32_t i) const { return base[i]; }
};

struct FusedArgs {
    Geo g;
    const uint16_t *q;
    float scale;
    int n_blocks, n_res, blocks_per_split, n_splits, stage_bytes;
};

// softmax state of one wave for G query heads
template <int G>
struct Soft {
    float m[G], l[G], bv[G], acc[G][2];
    __device__ __forceinline__ void init() {
#pragma unroll
        for (int g = 0; g < G; g++) { m[g] = -INFINITY; l[g] = 0.f; bv[g] = 0.f; acc[g][0] = 0.f; acc[g][1] = 0.f; }
    }
    // s: this lane's score (-inf for an invalid lane).  Returns p and rescales the running sums.
    __device__ __forceinline__ float update(int g, float s) {
        const float mloc = wave_max(s);
        const float mnew = fmaxf(m[g], mloc);
        const float alpha = __expf(m[g] - mnew);
        const float p = __expf(s - mnew);
        l[g] = l[g] * alpha + p;
        bv[g] *= alpha;
        acc[g][0] *= alpha;
        acc[g][1] *= alpha;
        m[g] = mnew;
        return p;
    }
};

// ---- K block: lane = token --------------------------------------------------------------------------------------
template <int G>
__device__ __forceinline__ void k_block(const uint32_t *hdr32, const WordSrc &pay, const uint16_t *lut, float *wts,
                                        const float (&qreg)[G][2], float two_eb, float scale, int lane,
                                        float (&score)[G]) {
    const uint32_t mm0 = hdr32[lane], mm1 = hdr32[lane + 64];
    const float mn0 = h2f(mm0 & 0xffffu), mn1 = h2f(mm1 & 0xffffu);
    const float st0 = two_eb * (h2f(mm0 >> 16) - mn0), st1 = two_eb * (h2f(mm1 >> 16) - mn1);
    float bias[G];
#pragma unroll
    for (int g = 0; g < G; g++) {
        wts[g * kD + lane] = qreg[g][0] * st0;
        wts[g * kD + lane + 64] = qreg[g][1] * st1;
        bias[g] = wave_sum(qreg[g][0] * mn0 + qreg[g][1] * mn1);
    }
    const uint32_t sb = reinterpret_cast<const uint16_t *>(hdr32)[kMinMaxBytesK / 2 + lane];
    uint32_t total;
    const uint32_t start = wave_excl_scan(sb, lane, &total);
    wave_sync();
    BitReader br;
    br.open(pay, start);
    float acc[G];
#pragma unroll
    for (int g = 0; g < G; g++) acc[g] = 0.f;
#pragma unroll 1
    for (int c = 0; c < kD; c += 4) {
        float4 w[G];
#pragma unroll
        for (int g = 0; g < G; g++) w[g] = *reinterpret_cast<const float4 *>(wts + g * kD + c);
#pragma unroll
        for (int u = 0; u < 4; u++) {
            const float f = (float)(br.get(pay, lut) >> 8);
#pragma unroll
            for (int g = 0; g < G; g++) acc[g] = fmaf(u == 0 ? w[g].x : u == 1 ? w[g].y : u == 2 ? w[g].z : w[g].w, f, acc[g]);
        }
    }
#pragma unroll
    for (int g = 0; g < G; g++) score[g] = scale * (acc[g] + bias[g]);
}

// ---- V block: lane = channels lane and lane+64 -------------------------------------------------------------------
template <int G>
__device__ __forceinline__ void v_block(const uint32_t *hdr32, const WordSrc &pay, const uint16_t *lut, float *wts,
                                        const float (&p)[G], float two_eb, int lane, Soft<G> &st) {
    const uint32_t mm = hdr32[lane];
    const float mn = h2f(mm & 0xffffu);
    const float step = two_eb * (h2f(mm >> 16) - mn);
#pragma unroll
    for (int g = 0; g < G; g++) {
        wts[g * kBT + lane] = p[g] * step;
        st.bv[g] += p[g] * mn;
    }
    const uint16_t *sb16 = reinterpret_cast<const uint16_t *>(hdr32) + kMinMaxBytesV / 2;
    uint32_t tot0, tot1;
    const uint32_t s0 = wave_excl_scan(sb16[lane], lane, &tot0);
    const uint32_t s1 = tot0 + wave_excl_scan(sb16[lane + 64], lane, &tot1);
    wave_sync();
    BitReader b0, b1;
    b0.open(pay, s0);
    b1.open(pay, s1);
#pragma unroll 1
    for (int t = 0; t < kBT; t += 4) {
        float4 w[G];
#pragma unroll
        for (int g = 0; g < G; g++) w[g] = *reinterpret_cast<const float4 *>(wts + g * kBT + t);
#pragma unroll
        for (int u = 0; u < 4; u++) {
            const float f0 = (float)(b0.get(pay, lut) >> 8);
            const float f1 = (float)(b1.get(pay, lut) >> 8);
#pragma unroll
            for (int g = 0; g < G; g++) {
                const float wv = u == 0 ? w[g].x : u == 1 ? w[g].y : u == 2 ? w[g].z : w[g].w;
                st.acc[g][0] = fmaf(wv, f0, st.acc[g][0]);
                st.acc[g][1] = fmaf(wv, f1, st.acc[g][1]);
            }
        }
    }
}

// copy a record (n16 units of 16 bytes) from global memory into this wave's LDS staging area
__device__ __forceinline__ void stage_record(uint4 *stage, const uint4 *rec, uint32_t n16, int lane) {
    for (uint32_t i = lane; i < n16; i += 64) stage[i] = rec[i];
}

constexpr int kWaves = 4;

template <int G>
__global__ __launch_bounds__(64 * kWaves, 4) void fused_attn_kernel(FusedArgs a) {
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    // LDS map: [lut K 8K][lut V 8K][q as float G*128][per wave: stage][per wave: wts G*128 floats]
    uint16_t *lutK = reinterpret_cast<uint16_t *>(smem);
    uint16_t *lutV = lutK + kLutSize;
    float *qf = reinterpret_cast<float *>(smem + 2 * kLutSize * 2);
    uint8_t *stage_base = reinterpret_cast<uint8_t *>(qf + G * kD);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint8_t *stage = stage_base + (size_t)wave * a.stage_bytes;
    float *wts = reinterpret_cast<float *>(stage_base + (size_t)kWaves * a.stage_bytes) + wave * G * kD;

    const Geo &g = a.g;
    const int split = blockIdx.x, bh = blockIdx.y;
    const int b = bh / g.H, h = bh - b * g.H;

    // workgroup prologue: lookup tables and the G query vectors of this KV head
    {
        const uint4 *src = reinterpret_cast<const uint4 *>(g.lut);
        uint4 *dst = reinterpret_cast<uint4 *>(smem);
        for (int i = tid; i < 2 * kLutSize * 2 / 16; i += 64 * kWaves) dst[i] = src[i];
        for (int i = tid; i < G * kD; i += 64 * kWaves)
            qf[i] = h2f(a.q[((size_t)b * g.Hq + (size_t)h * G) * kD + i]);
    }
    __syncthreads();
    float qreg[G][2];
#pragma unroll
    for (int gg = 0; gg < G; gg++) { qreg[gg][0] = qf[gg * kD + lane]; qreg[gg][1] = qf[gg * kD + lane + 64]; }

    Soft<G> st;
    st.init();

    const int j0 = split * a.blocks_per_split;
    const int j1 = min(j0 + a.blocks_per_split, a.n_blocks);
    const BlockEntry *tabK = g.table + ((size_t)0 * g.B * g.H + bh) * g.max_blocks;
    const BlockEntry *tabV = g.table + ((size_t)1 * g.B * g.H + bh) * g.max_blocks;
    const uint32_t stage16 = (uint32_t)a.stage_bytes / 16 - 1;  // one unit of slack for the reader's look-ahead

    for (int j = j0 + wave; j < j1; j += kWaves) {
        float score[G], p[G];
        {
            const BlockEntry e = tabK[j];
            const uint8_t *rec = g.payload + (size_t)e.off16 * 16;
            if (e.size16 <= stage16) {
                stage_record(reinterpret_cast<uint4 *>(stage), reinterpret_cast<const uint4 *>(rec), e.size16, lane);
                wave_sync();
                WordSrc pay{reinterpret_cast<const uint32_t *>(stage + kHdrBytesK)};
                k_block<G>(reinterpret_cast<const uint32_t *>(stage), pay, lutK, wts, qreg, g.two_eb[0], a.scale, lane, score);
            } else {  // record larger than the staging area: decode from global memory
                WordSrc pay{reinterpret_cast<const uint32_t *>(rec + kHdrBytesK)};
                k_block<G>(reinterpret_cast<const uint32_t *>(rec), pay, lutK, wts, qreg, g.two_eb[0], a.scale, lane, score);
            }
        }
#pragma unroll
        for (int gg = 0; gg < G; gg++) p[gg] = st.update(gg, score[gg]);
        wave_sync();  // all lanes are done with the K stage and weights before they are overwritten
        {
            const BlockEntry e = tabV[j];
            const uint8_t *rec = g.payload + (size_t)e.off16 * 16;
            if (e.size16 <= stage16) {
                stage_record(reinterpret_cast<uint4 *>(stage), reinterpret_cast<const uint4 *>(rec), e.size16, lane);
                wave_sync();
                WordSrc pay{reinterpret_cast<const uint32_t *>(stage + kHdrBytesV)};
                v_block<G>(reinterpret_cast<const uint32_t *>(stage), pay, lutV, wts, p, g.two_eb[1], lane, st);
            } else {
                WordSrc pay{reinterpret_cast<const uint32_t *>(rec + kHdrBytesV)};
                v_block<G>(reinterpret_cast<const uint32_t *>(rec), pay, lutV, wts, p, g.two_eb[1], lane, st);
            }
        }
        wave_sync();
    }

    // The buffered fp16 tokens (Section 3.2.3: the newest vectors take part too): last split, wave 0.
    if (split == a.n_splits - 1 && wave == 0 && a.n_res > 0) {
        const size_t res_tensor = (size_t)g.B * kBT * g.H * kD;
        float acc[G];
#pragma unroll
        for (int gg = 0; gg < G; gg++) acc[gg] = 0.f;
        if (lane < a.n_res) {
            const uint16_t *kr = g.res + (((size_t)b * kBT + lane) * g.H + h) * kD;
            for (int c = 0; c < kD; c += 8) {
                const uint4 v = *reinterpret_cast<const uint4 *>(kr + c);
                const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int k = 0; k < 4; k++) {
                    const float x0 = h2f(w[k] & 0xffffu), x1 = h2f(w[k] >> 16);
#pragma unroll
                    for (int gg = 0; gg < G; gg++) {
                        acc[gg] = fmaf(qf[gg * kD + c + 2 * k], x0, acc[gg]);
                        acc[gg] = fmaf(qf[gg * kD + c + 2 * k + 1], x1, acc[gg]);
                    }
                }
            }
        }
#pragma unroll
        for (int gg = 0; gg < G; gg++) {
            const float s = lane < a.n_res ? a.scale * acc[gg] : -INFINITY;
            wts[gg * kBT + lane] = st.update(gg, s);
        }
        wave_sync();
        const uint16_t *vr = g.res + res_tensor + (((size_t)b * kBT) * g.H + h) * kD;
        for (int t = 0; t < a.n_res; t++) {
            const float v0 = h2f(vr[(size_t)t * g.H * kD + lane]);
            const float v1 = h2f(vr[(size_t)t * g.H * kD + lane + 64]);
#pragma unroll
            for (int gg = 0; gg < G; gg++) {
                const float pw = wts[gg * kBT + t];
                st.acc[gg][0] = fmaf(pw, v0, st.acc[gg][0]);
                st.acc[gg][1] = fmaf(pw, v1, st.acc[gg][1]);
            }
        }
        wave_sync();
    }

    // merge the waves of this workgroup, then write one partial (o[128], m, l) per query head and split
    float *comb = reinterpret_cast<float *>(stage);  // this wave's own staging area: G * 130 floats
#pragma unroll
    for (int gg = 0; gg < G; gg++) {
        const float l = wave_sum(st.l[gg]);
        const float bv = wave_sum(st.bv[gg]);
        comb[gg * kPartialStride + lane] = st.acc[gg][0] + bv;
        comb[gg * kPartialStride + lane + 64] = st.acc[gg][1] + bv;
        if (lane == 0) {
            comb[gg * kPartialStride + kD] = st.m[gg];
            comb[gg * kPartialStride + kD + 1] = l;
        }
    }
    __syncthreads();
    for (int i = tid; i < G * kD; i += 64 * kWaves) {
        const int gg = i / kD, c = i - gg * kD;
        float M = -INFINITY;
        for (int w = 0; w < kWaves; w++)
            M = fmaxf(M, reinterpret_cast<const float *>(stage_base + (size_t)w * a.stage_bytes)[gg * kPartialStride + kD]);
        float L = 0.f, O = 0.f;
        for (int w = 0; w < kWaves; w++) {
            const float *cw = reinterpret_cast<const float *>(stage_base + (size_t)w * a.stage_bytes) + gg * kPartialStride;
            const float mw = cw[kD];
            const float f = mw == -INFINITY ? 0.f : __expf(mw - M);
            L += cw[kD + 1] * f;
            O += cw[c] * f;
        }
        float *dst = g.partials + (((size_t)b * g.Hq + (size_t)h * G + gg) * kMaxSplits + split) * kPartialStride;
        dst[c] = O;
        if (c == 0) { dst[kD] = M; dst[kD + 1] = L; }
    }
}

// Merge the sequence splits: out = sum_s o_s e^{m_s - M} / sum_s l_s e^{m_s - M}.
__global__ __launch_bounds__(kD) void combine_kernel(const float *__restrict__ partials, int n_splits,
                                                      float *__restrict__ out) {
    const int row = blockIdx.x, c = threadIdx.x;
    const float *p = partials + (size_t)row * kMaxSplits * kPartialStride;
    float M = -INFINITY;
    for (int s = 0; s < n_splits; s++) M = fmaxf(M, p[s * kPartialStride + kD]);
    float L = 0.f, O = 0.f;
    for (int s = 0; s < n_splits; s++) {
        const float ms = p[s * kPartialStride + kD];
        const float f = ms == -INFINITY ? 0.f : __expf(ms - M);
        L += p[s * kPartialStride + kD + 1] * f;
        O += p[s * kPartialStride + c] * f;
    }
    out[(size_t)row * kD + c] = O / L;
}

hipError_t launch_combine(const float *partials, int rows, int n_splits, float *out, hipStream_t s) {
    hipLaunchKernelGGL(combine_kernel, dim3(rows), dim3(kD), 0, s, partials, n_splits, out);
    return hipGetLastError();
}

template <int G>
static hipError_t launch_fused_g(const FusedArgs &a, size_t lds, hipEvent_t ev0, hipEvent_t ev1, hipStream_t s) {
    static size_t attr_set = 0;
    if (lds > attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&fused_attn_kernel<G>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set = lds;
    }
    if (ev0) (void)hipEventRecord(ev0, s);
    hipLaunchKernelGGL(fused_attn_kernel<G>, dim3(a.n_splits, a.g.B * a.g.H), dim3(64 * kWaves), lds, s, a);
    if (ev1) (void)hipEventRecord(ev1, s);
    return hipGetLastError();
}

size_t fused_lds_bytes(int G, int stage_bytes) {
    return (size_t)2 * kLutSize * 2 + (size_t)G * kD * 4 + (size_t)kWaves * stage_bytes + (size_t)kWaves * G * kD * 4;
}

hipError_t launch_fused_attn(const Geo &g, const uint16_t *q, float scale, float *out, int n_blocks, int n_res,
                             int n_splits, int stage_bytes, hipEvent_t ev0, hipEvent_t ev1, hipStream_t s) {
    FusedArgs a;
    a.g = g;
    a.q = q;
    a.scale = scale;
    a.n_blocks = n_blocks;
    a.n_res = n_res;
    a.blocks_per_split = n_blocks > 0 ? (n_blocks + n_splits - 1) / n_splits : 0;
    a.n_splits = n_blocks > 0 ? (n_blocks + a.blocks_per_split - 1) / a.blocks_per_split : 1;
    a.stage_bytes = stage_bytes;
    const size_t lds = fused_lds_bytes(g.G, stage_bytes);
    hipError_t e;
    switch (g.G) {
        case 1: e = launch_fused_g<1>(a, lds, ev0, ev1, s); break;
        case 2: e = launch_fused_g<2>(a, lds, ev0, ev1, s); break;
        case 4: e = launch_fused_g<4>(a, lds, ev0, ev1, s); break;
        case 8: e = launch_fused_g<8>(a, lds, ev0, ev1, s); break;
        default: return hipErrorInvalidValue;
    }
    if (e != hipSuccess) return e;
    return launch_combine(g.partials, g.B * g.Hq, a.n_splits, out, s);
}

}  // namespace kvc
