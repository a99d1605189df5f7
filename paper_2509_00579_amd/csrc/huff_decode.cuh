// Wave-level Huffman decode machinery shared by the fused decode-attention kernel and the stand-alone decompressor:
// wave reductions on DPP, the stream readers of a slice (two chains per slice, read from both ends), and the
// lookup-table decode of several symbols per 32-bit window (Section 3.3.1 replaced by a table decode, see
// attn_fused.hip for the reasons).
#pragma once

#include <hip/hip_fp16.h>

#include "kvcomp_internal.h"

namespace kvc {

__device__ __forceinline__ void wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ __forceinline__ float h2f(uint32_t bits) { return __half2float(__ushort_as_half((unsigned short)bits)); }

// value of `v` in lane `lane_idx` (wave-uniform index), delivered in a scalar register
__device__ __forceinline__ float bcast(float v, int lane_idx) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane_idx));
}

// Wave-wide reductions and the prefix sum run on DPP row operations and v_readlane, not on ds_bpermute: the LDS pipe
// is the busiest unit of this kernel and a butterfly of six dependent LDS round trips costs far more latency.
template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {  // lanes without a source read 0
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, true);
}
constexpr int kDppXor1 = 0xB1, kDppXor2 = 0x4E;              // quad_perm [1,0,3,2] and [2,3,0,1]
constexpr int kDppHalfMirror = 0x141, kDppMirror = 0x140;    // lane i <-> 7 - i (within 8) and i <-> 15 - i (within 16)
constexpr int kDppRowShr = 0x110;                            // + n: lane i reads lane i - n of its row of 16

// the same value in every lane
__device__ __forceinline__ float wave_sum(float v) {
    v += dpp_f<kDppXor1>(v);
    v += dpp_f<kDppXor2>(v);
    v += dpp_f<kDppHalfMirror>(v);
    v += dpp_f<kDppMirror>(v);  // every lane: sum of its row of 16
    return (bcast(v, 0) + bcast(v, 16)) + (bcast(v, 32) + bcast(v, 48));
}
__device__ __forceinline__ float wave_max(float v) {
    v = fmaxf(v, dpp_f<kDppXor1>(v));
    v = fmaxf(v, dpp_f<kDppXor2>(v));
    v = fmaxf(v, dpp_f<kDppHalfMirror>(v));
    v = fmaxf(v, dpp_f<kDppMirror>(v));
    return fmaxf(fmaxf(bcast(v, 0), bcast(v, 16)), fmaxf(bcast(v, 32), bcast(v, 48)));
}
// exclusive prefix sum over the 64 lanes
__device__ __forceinline__ uint32_t wave_excl_scan(uint32_t v, int lane) {
    uint32_t inc = v;
    inc += dpp_u<kDppRowShr + 1>(inc);
    inc += dpp_u<kDppRowShr + 2>(inc);
    inc += dpp_u<kDppRowShr + 4>(inc);
    inc += dpp_u<kDppRowShr + 8>(inc);  // inclusive within each row of 16
    const uint32_t t0 = __builtin_amdgcn_readlane(inc, 15), t1 = __builtin_amdgcn_readlane(inc, 31),
                   t2 = __builtin_amdgcn_readlane(inc, 47);
    const int row = lane >> 4;
    const uint32_t before = row == 0 ? 0u : row == 1 ? t0 : row == 2 ? t0 + t1 : t0 + t1 + t2;
    return inc + before - v;
}

// A slice holds two decode chains (see the record layout): symbols 0..31 are read upwards from the slice start,
// symbols 63..32 downwards from the slice end.
//   wm1   payload words, pointer moved back by one word: payload bit x is bit x + 32 of wm1
// A window is 32 bits whose lowest J bits are don't-cares and whose bits J.. are the next unread stream bits in
// reading order, i.e. the stream already scaled to the byte offset of a table entry of 2^J bytes (J = 1: 16-bit
// entries, one symbol each; J = 2: 32-bit entries that deliver two symbols).
// (Unaligned 4-byte LDS reads at byte granularity, and re-reading both words of every window, were tried: slower.)
//
// Readers keep a 64-bit piece {hi,lo} of the stream in registers plus the next word in reading direction, fetched
// one window ahead: one 4-byte LDS read per window, off the critical path (only table lookups depend on each other).
template <int J>
struct UpReader {
    uint32_t P, idx, lo, hi, nx;  // P = (next unread payload bit) + 32 - J = window start in wm1 bit coordinates
    __device__ __forceinline__ void open(const uint32_t *wm1, uint32_t first_bit) {
        P = first_bit + (uint32_t)(32 - J);
        idx = P >> 5;
        lo = wm1[idx];
        hi = wm1[idx + 1];
        nx = wm1[idx + 2];
    }
    __device__ __forceinline__ uint32_t window(const uint32_t *) const { return __builtin_amdgcn_alignbit(hi, lo, P); }
    __device__ __forceinline__ void advance(const uint32_t *wm1, uint32_t used) {  // used <= 32 - J
        P += used;
        const uint32_t nidx = P >> 5;
        const bool adv = nidx != idx;
        lo = adv ? hi : lo;
        hi = adv ? nx : hi;
        idx = nidx;
        nx = wm1[nidx + 2];
    }
};
template <int J>
struct DownReader {
    uint32_t P, idx, lo, hi, pv;  // P = (one past the next unread payload bit) + J: the window [P, P+32) of wm1 ends J
                                  // bits above the next unread bit; bit-reversed it reads downwards
    __device__ __forceinline__ void open(const uint32_t *wm1, uint32_t end_bit) {
        P = end_bit + (uint32_t)J;
        idx = P >> 5;
        lo = wm1[idx];
        hi = wm1[idx + 1];
        pv = wm1[(int)idx - 1];
    }
    __device__ __forceinline__ uint32_t window(const uint32_t *) const {
        return __builtin_bitreverse32(__builtin_amdgcn_alignbit(hi, lo, P));
    }
    __device__ __forceinline__ void advance(const uint32_t *wm1, uint32_t used) {  // used <= 32 - J
        P -= used;
        const uint32_t nidx = P >> 5;
        const bool adv = nidx != idx;
        hi = adv ? lo : hi;
        lo = adv ? pv : lo;
        idx = nidx;
        pv = wm1[(int)nidx - 1];
    }
};

// CNT table lookups in a window.  J = 1: 16-bit entries (symbol << 8) | code length, indexed by the next `bits` stream
// bits, mask = ((1 << bits) - 1) << 1.  J = 2: 32-bit entries of the pair table, indexed by the next 12 stream bits
// (mask = 0xfff << 2): byte 0 = length of two consecutive code words together, byte 1 = first symbol, byte 2 = second
// symbol.  CNT * (index width) <= 32 - J is the caller's promise.  e[] receives the entries; returns the number of
// bits used.
template <int J, int CNT>
__device__ __forceinline__ uint32_t lookup(uint32_t win, const char *lut, uint32_t mask, uint32_t (&e)[CNT]) {
    uint32_t tot = 0;
#pragma unroll
    for (int k = 0; k < CNT; k++) {
        if constexpr (J == 1) e[k] = *reinterpret_cast<const uint16_t *>(lut + (win & mask));
        else e[k] = *reinterpret_cast<const uint32_t *>(lut + (win & mask));
        win >>= (e[k] & 31u);
        tot += e[k];  // low byte: running sum of code lengths (at most 31, never carries)
    }
    return tot & 0xffu;
}

// the symbols of a table entry as fp32 (one v_cvt_f32_ubyte1 / v_cvt_f32_ubyte2)
__device__ __forceinline__ float sym_f32(uint32_t e) { return (float)((e >> 8) & 0xffu); }
__device__ __forceinline__ float sym2_f32(uint32_t e) { return (float)((e >> 16) & 0xffu); }

// The four chains of one lane (two slices x two directions) advance together, CNT lookups each.
template <int J>
struct Quad {
    UpReader<J> au, bu;
    DownReader<J> ad, bd;
    // a = [a0, a0 + abits), b follows it
    __device__ __forceinline__ void open(const uint32_t *wm1, uint32_t a0, uint32_t abits, uint32_t bbits) {
        au.open(wm1, a0);
        ad.open(wm1, a0 + abits);
        bu.open(wm1, a0 + abits);
        bd.open(wm1, a0 + abits + bbits);
    }
    // the same for two slices that do not follow each other in the record
    __device__ __forceinline__ void open2(const uint32_t *wm1, uint32_t a0, uint32_t abits, uint32_t b0, uint32_t bbits) {
        au.open(wm1, a0);
        ad.open(wm1, a0 + abits);
        bu.open(wm1, b0);
        bd.open(wm1, b0 + bbits);
    }
    template <int CNT>
    __device__ __forceinline__ void step(const uint32_t *wm1, const char *lut, uint32_t mask, uint32_t (&fau)[CNT],
                                         uint32_t (&fad)[CNT], uint32_t (&fbu)[CNT], uint32_t (&fbd)[CNT]) {
        const uint32_t u0 = lookup<J, CNT>(au.window(wm1), lut, mask, fau);
        const uint32_t u1 = lookup<J, CNT>(ad.window(wm1), lut, mask, fad);
        const uint32_t u2 = lookup<J, CNT>(bu.window(wm1), lut, mask, fbu);
        const uint32_t u3 = lookup<J, CNT>(bd.window(wm1), lut, mask, fbd);
        au.advance(wm1, u0);
        ad.advance(wm1, u1);
        bu.advance(wm1, u2);
        bd.advance(wm1, u3);
    }
};

constexpr int kHalf = kSliceLen / 2;  // symbols per chain
constexpr int kPairIndexBits = 12;    // index width of the pair table: two code words of up to 6 bits
constexpr int kPairLongest = kPairIndexBits / 2;

// How a kernel compiled for code words of up to LB bits decodes.  LB <= 6: the pair table (every lookup delivers two
// symbols, so a chain of 32 symbols is 16 dependent lookups).  Otherwise the single-symbol table of 2^LB 16-bit
// entries.
template <int LB>
struct DecodeMode {
    static constexpr bool kPair = LB <= kPairLongest;
    static constexpr int J = kPair ? 2 : 1;                               // log2 of the entry size in bytes
    static constexpr int kIndexBits = kPair ? kPairIndexBits : LB;
    static constexpr int kSymsPerLookup = kPair ? 2 : 1;
    static constexpr int kLookupsPerWindow = (32 - J) / kIndexBits;       // pair table: 2; 7, 8, 10, 12 bits: 4, 3, 3, 2
    static constexpr int kSymsPerWindow = kSymsPerLookup * kLookupsPerWindow;
    static constexpr int kLookupsPerChain = kHalf / kSymsPerLookup;
    static constexpr int kTableBytes = (kPair ? 4 : 2) << kIndexBits;     // per tensor
};

}  // namespace kvc
