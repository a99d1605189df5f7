// Device code shared by the store-side kernels: load one 2D block (64 tokens x 128 channels, fp16) with a
// 256-thread workgroup, reduce the min/max of every quantization unit and produce the 8-bit codes in registers.
//
// Quantization follows Section 3.1.1 (K: channel-wise inside the block, V: token-wise) with the relative scale of
// Section 4.2 read as bin width = 2 * rel_eb * (max - min):
//     code = round_half_even((x - min) / width), clamped to [0, n_sym - 1];  range 0 -> code 0.
// The codes are those of IEEE binary32 arithmetic taken one operation at a time (this file is compiled with
// -ffp-contract=off and correctly rounded division), so that an independent implementation of the same operation
// sequence agrees bit for bit; quant_codes reaches them by a cheaper route wherever that provably gives the same
// integer.
//
// Thread map (tid = 64*w + l): load i in 0..3 covers token 16*w + 4*i + l/16, channels 8*(l%16) .. +7, i.e. one wave
// load instruction reads four contiguous 256-byte rows.
#pragma once

#include <hip/hip_fp16.h>

#include "kvcomp_internal.h"

namespace kvc {

struct TileRegs {
    float x[4][8];       // values
    uint32_t code[4][8];  // after quantize_tile
};

__device__ __forceinline__ int tile_token(int tid, int i) { return 16 * (tid >> 6) + 4 * i + ((tid & 63) >> 4); }
__device__ __forceinline__ int tile_chan0(int tid) { return (tid & 15) * 8; }

__device__ __forceinline__ float half_bits_to_float(uint32_t h) {
    return __half2float(__ushort_as_half((unsigned short)h));
}
__device__ __forceinline__ uint32_t float_to_half_bits(float f) {  // f is exactly representable
    return (uint32_t)__half_as_ushort(__float2half_rn(f));
}

// The four 16-byte pieces of a thread, still packed: issued early (for the block after the current one) so that the
// loads travel while the current block is quantized.
struct TileRaw {
    uint4 v[4];
};
// Byte offsets of a thread's four pieces from the first element of a block: they depend on the thread and on H only,
// so a kernel that walks over blocks computes them once and adds the (wave-uniform) address of each block.
struct TileOffsets {
    uint32_t at[4];
    __device__ __forceinline__ void set(int H, int tid) {
#pragma unroll
        for (int i = 0; i < 4; i++) at[i] = ((uint32_t)tile_token(tid, i) * (uint32_t)H * kD + (uint32_t)tile_chan0(tid)) * 2u;
    }
};
// first element of block blk of (b, h) in X [B][seq_stride][H][128]
__device__ __forceinline__ const uint16_t *tile_base(const uint16_t *X, int seq_stride, int H, int b, int h, int blk) {
    return X + (((size_t)b * (size_t)seq_stride + (size_t)blk * kBT) * (size_t)H + (size_t)h) * kD;
}
__device__ __forceinline__ void load_tile_raw(const uint16_t *base, const TileOffsets &off, TileRaw &raw) {
#pragma unroll
    for (int i = 0; i < 4; i++)
        raw.v[i] = *reinterpret_cast<const uint4 *>(reinterpret_cast<const char *>(base) + off.at[i]);
}
__device__ __forceinline__ void unpack_tile(const TileRaw &raw, TileRegs &r) {
#pragma unroll
    for (int i = 0; i < 4; i++) {
        const uint32_t w[4] = {raw.v[i].x, raw.v[i].y, raw.v[i].z, raw.v[i].w};
#pragma unroll
        for (int k = 0; k < 4; k++) {
            r.x[i][2 * k] = half_bits_to_float(w[k] & 0xffffu);
            r.x[i][2 * k + 1] = half_bits_to_float(w[k] >> 16);
        }
    }
}
__device__ __forceinline__ void load_tile(const uint16_t *X, int seq_stride, int H, int b, int h, int blk, int tid,
                                          TileRegs &r) {
    TileOffsets off;
    off.set(H, tid);
    TileRaw raw;
    load_tile_raw(tile_base(X, seq_stride, H, b, h, blk), off, raw);
    unpack_tile(raw, r);
}

// Codes of N values of one quantization unit: code = clamp(rint((x - mn) / step), 0, top) with the correctly rounded
// binary32 division, 0 if the unit's range is 0.  Returns true if a value is Inf or NaN.
// BIASED: the codes come with kRoundMagicBits added (the histogram kernel uses them as they fall out of the rounding).
// The quantizer is most of the store kernels' instructions, so the common case takes a cheaper route to the same
// integers:
//   * the quotient is formed as q = d * rcp(step): v_rcp_f32 is accurate to 1 ulp and the product adds half an ulp,
//     so q is within 2^-22 relative (below 2^-14 absolute for quotients under 256) of the correctly rounded
//     quotient, and rounds to the same integer unless it lies within that distance of k + 1/2;
//   * q is rounded by adding 2^23 (round to nearest even at unit spacing, like rint): the bit pattern of the sum is
//     that of 2^23 plus the integer, which also makes the conversion; q >= 0 (mn is the minimum of the same values),
//     so only the upper clamp is left;
//   * a value within 2^-13 of a boundary k + 1/2 in any lane sends the wave to the division for that value (one
//     wave in 60 per value).  Inf and NaN inputs take that path by themselves: they make q a NaN in their own lane
//     (x - mn, or (x - mn) * 0 when the range is infinite), and the test is written so that a NaN fails it; the
//     common path needs no test for them.
constexpr float kRoundMagic = 8388608.0f;          // 2^23
constexpr uint32_t kRoundMagicBits = 0x4B000000u;  // its bit pattern
constexpr float kNearBoundary = 0x1p-13f;
template <int N, bool BIASED>
__device__ __forceinline__ bool quant_codes(const float (&x)[N], float mn, float step, float range, float top,
                                            uint32_t (&code)[N]) {
    const float inv = range == 0.0f ? 0.0f : __builtin_amdgcn_rcpf(step);  // range 0: every code 0
    const uint32_t top_bits = kRoundMagicBits + (uint32_t)top;
    constexpr uint32_t kBias = BIASED ? kRoundMagicBits : 0u;
    bool bad = false;
#pragma unroll
    for (int n = 0; n < N; n++) {
        const float q = (x[n] - mn) * inv;
        code[n] = min(__float_as_uint(q + kRoundMagic), top_bits) - (kRoundMagicBits - kBias);
        const bool far = fabsf(__builtin_amdgcn_fractf(q) - 0.5f) >= kNearBoundary;  // false for a NaN
        if (__builtin_amdgcn_ballot_w64(!far) != 0) {
            bad |= !(fabsf(x[n]) < INFINITY);
            const float k = fminf(fmaxf(rintf((x[n] - mn) / step), 0.0f), top);
            code[n] = (range == 0.0f ? 0u : (uint32_t)k) + kBias;
        }
    }
    return bad;
}

__device__ __forceinline__ float canon_zero(float v) { return v == 0.0f ? 0.0f : v; }

// LDS scratch needed by quantize_tile.
struct __attribute__((aligned(16))) QuantShared {
    float part_mn[4][kD];
    float part_mx[4][kD];
    float unit_mn[kD];  // K: per channel;  V: per token (first 64 entries)
    float unit_mx[kD];
};

// Computes r.code and leaves the unit minima / maxima in sh.unit_mn / sh.unit_mx.  Returns true if one of this
// thread's values is Inf or NaN.
// Contains __syncthreads(): must be called by all 256 threads of the workgroup.
// k_units: 128 = K channel-wise inside the block (Section 3.1.1), 1 = one unit per K block (BlockQuant, Section 4.2);
// ignored for V.
// v_min_f32 / v_max_f32 on values that came through a lane exchange: the compiler would first pass them through a
// canonicalising instruction each, which changes nothing here (the values are conversions from fp16).
__device__ __forceinline__ float min_raw(float a, float b) {
    float o;
    asm("v_min_f32 %0, %1, %2" : "=v"(o) : "v"(a), "v"(b));
    return o;
}
__device__ __forceinline__ float max_raw(float a, float b) {
    float o;
    asm("v_max_f32 %0, %1, %2" : "=v"(o) : "v"(a), "v"(b));
    return o;
}
// Minimum / maximum over the 16 lanes of a DPP row, result in every lane: the exchange rides on the min/max
// instruction itself.  The s_nop in front of each step covers the wait states that a DPP operand needs after the
// vector instruction that wrote it (two), and in front of the first step those after a vector write of EXEC (five).
#define KVC_ROW_REDUCE(OP, v)                                                                              \
    asm volatile("s_nop 4\n\t" OP " %0, %0, %0 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"                \
        "s_nop 1\n\t" OP " %0, %0, %0 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"                \
        "s_nop 1\n\t" OP " %0, %0, %0 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"                    \
        "s_nop 1\n\t" OP " %0, %0, %0 row_mirror row_mask:0xf bank_mask:0xf"                              \
        : "+v"(v))
__device__ __forceinline__ float row_min(float v) {
    KVC_ROW_REDUCE("v_min_f32_dpp", v);
    return v;
}
__device__ __forceinline__ float row_max(float v) {
    KVC_ROW_REDUCE("v_max_f32_dpp", v);
    return v;
}
#undef KVC_ROW_REDUCE

template <int WHICH, bool BIASED = false>
__device__ __forceinline__ bool quantize_tile(TileRegs &r, QuantShared &sh, int tid, float two_eb, int n_sym,
                                              int k_units) {
    const float top = (float)(n_sym - 1);
    bool bad = false;
    if (WHICH == 0 && k_units == 1) {
        float a = r.x[0][0], z = r.x[0][0];
#pragma unroll
        for (int i = 0; i < 4; i++)
#pragma unroll
            for (int k = 0; k < 8; k++) {
                a = fminf(a, r.x[i][k]);
                z = fmaxf(z, r.x[i][k]);
            }
#pragma unroll
        for (int m = 1; m < 64; m <<= 1) {
            a = fminf(a, __shfl_xor(a, m));
            z = fmaxf(z, __shfl_xor(z, m));
        }
        if ((tid & 63) == 0) {
            sh.part_mn[tid >> 6][0] = a;
            sh.part_mx[tid >> 6][0] = z;
        }
        __syncthreads();
        if (tid == 0) {
            sh.unit_mn[0] = canon_zero(fminf(fminf(sh.part_mn[0][0], sh.part_mn[1][0]),
                                             fminf(sh.part_mn[2][0], sh.part_mn[3][0])));
            sh.unit_mx[0] = canon_zero(fmaxf(fmaxf(sh.part_mx[0][0], sh.part_mx[1][0]),
                                             fmaxf(sh.part_mx[2][0], sh.part_mx[3][0])));
        }
        __syncthreads();
        a = sh.unit_mn[0];
        z = sh.unit_mx[0];
        const float range = z - a;
        const float step = two_eb * range;
#pragma unroll
        for (int i = 0; i < 4; i++) bad |= quant_codes<8, BIASED>(r.x[i], a, step, range, top, r.code[i]);
    } else if (WHICH == 0) {
        float mn[8], mx[8];
#pragma unroll
        for (int k = 0; k < 8; k++) {
            mn[k] = fminf(fminf(r.x[0][k], r.x[1][k]), fminf(r.x[2][k], r.x[3][k]));
            mx[k] = fmaxf(fmaxf(r.x[0][k], r.x[1][k]), fmaxf(r.x[2][k], r.x[3][k]));
            mn[k] = min_raw(mn[k], __shfl_xor(mn[k], 16));
            mx[k] = max_raw(mx[k], __shfl_xor(mx[k], 16));
            mn[k] = min_raw(mn[k], __shfl_xor(mn[k], 32));
            mx[k] = max_raw(mx[k], __shfl_xor(mx[k], 32));
        }
        const int w = tid >> 6, c0 = tile_chan0(tid);
        if (((tid & 63) >> 4) == 0) {  // 16-byte accesses: a thread's eight channels are neighbours, lanes follow each other
            float4 *pmn = reinterpret_cast<float4 *>(&sh.part_mn[w][c0]), *pmx = reinterpret_cast<float4 *>(&sh.part_mx[w][c0]);
            pmn[0] = make_float4(mn[0], mn[1], mn[2], mn[3]);
            pmn[1] = make_float4(mn[4], mn[5], mn[6], mn[7]);
            pmx[0] = make_float4(mx[0], mx[1], mx[2], mx[3]);
            pmx[1] = make_float4(mx[4], mx[5], mx[6], mx[7]);
        }
        __syncthreads();
        if (tid < kD) {
            const float a = fminf(fminf(sh.part_mn[0][tid], sh.part_mn[1][tid]),
                                  fminf(sh.part_mn[2][tid], sh.part_mn[3][tid]));
            const float z = fmaxf(fmaxf(sh.part_mx[0][tid], sh.part_mx[1][tid]),
                                  fmaxf(sh.part_mx[2][tid], sh.part_mx[3][tid]));
            sh.unit_mn[tid] = canon_zero(a);
            sh.unit_mx[tid] = canon_zero(z);
        }
        __syncthreads();
        float umn[8], umx[8];
        {
            const float4 *pmn = reinterpret_cast<const float4 *>(&sh.unit_mn[c0]), *pmx = reinterpret_cast<const float4 *>(&sh.unit_mx[c0]);
            const float4 a0 = pmn[0], a1 = pmn[1], z0 = pmx[0], z1 = pmx[1];
            umn[0] = a0.x; umn[1] = a0.y; umn[2] = a0.z; umn[3] = a0.w; umn[4] = a1.x; umn[5] = a1.y; umn[6] = a1.z; umn[7] = a1.w;
            umx[0] = z0.x; umx[1] = z0.y; umx[2] = z0.z; umx[3] = z0.w; umx[4] = z1.x; umx[5] = z1.y; umx[6] = z1.z; umx[7] = z1.w;
        }
#pragma unroll
        for (int k = 0; k < 8; k++) {
            const float a = umn[k], z = umx[k];
            const float range = z - a;
            const float step = two_eb * range;
            const float xs[4] = {r.x[0][k], r.x[1][k], r.x[2][k], r.x[3][k]};
            uint32_t cs[4];
            bad |= quant_codes<4, BIASED>(xs, a, step, range, top, cs);
#pragma unroll
            for (int i = 0; i < 4; i++) r.code[i][k] = cs[i];
        }
    } else {
#pragma unroll
        for (int i = 0; i < 4; i++) {
            float a = r.x[i][0], z = r.x[i][0];
#pragma unroll
            for (int k = 1; k < 8; k++) {
                a = fminf(a, r.x[i][k]);
                z = fmaxf(z, r.x[i][k]);
            }
            a = row_min(a);  // the 16 lanes of a DPP row hold one token's row
            z = row_max(z);
            a = canon_zero(a);
            z = canon_zero(z);
            if ((tid & 15) == 0) {
                sh.unit_mn[tile_token(tid, i)] = a;
                sh.unit_mx[tile_token(tid, i)] = z;
            }
            const float range = z - a;
            const float step = two_eb * range;
            bad |= quant_codes<8, BIASED>(r.x[i], a, step, range, top, r.code[i]);
        }
        __syncthreads();
    }
    return bad;
}

}  // namespace kvc
