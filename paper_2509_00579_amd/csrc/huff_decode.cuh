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
// A window is 32 stream bits whose bit 0 is a don't-care and whose bits 1.. are the next unread bits in reading
// order, i.e. the stream already scaled to the byte offset of a 16-bit table entry.
// (Unaligned 4-byte LDS reads at byte granularity, and re-reading both words of every window, were tried: slower.)
constexpr int kJunkBits = 1;                  // low window bits that are not stream bits
constexpr int kWindowBits = 32 - kJunkBits;  // stream bits per window
// Readers keep a 64-bit piece {hi,lo} of the stream in registers plus the next word in reading direction, fetched
// one window ahead: one 4-byte LDS read per window, off the critical path (only table lookups depend on each other).
struct UpReader {
    uint32_t P, idx, lo, hi, nx;  // P = (next unread payload bit) + 32 - kJunkBits = window start in wm1 bit coordinates
    __device__ __forceinline__ void open(const uint32_t *wm1, uint32_t first_bit) {
        P = first_bit + (uint32_t)(32 - kJunkBits);
        idx = P >> 5;
        lo = wm1[idx];
        hi = wm1[idx + 1];
        nx = wm1[idx + 2];
    }
    __device__ __forceinline__ uint32_t window(const uint32_t *) const { return __builtin_amdgcn_alignbit(hi, lo, P); }
    __device__ __forceinline__ void advance(const uint32_t *wm1, uint32_t used) {  // used <= 31
        P += used;
        const uint32_t nidx = P >> 5;
        const bool adv = nidx != idx;
        lo = adv ? hi : lo;
        hi = adv ? nx : hi;
        idx = nidx;
        nx = wm1[nidx + 2];
    }
};
struct DownReader {
    uint32_t P, idx, lo, hi, pv;  // P = (one past the next unread payload bit) + kJunkBits: the window [P, P+32) of wm1 ends
                                  // kJunkBits bits above the next unread bit; bit-reversed it reads downwards
    __device__ __forceinline__ void open(const uint32_t *wm1, uint32_t end_bit) {
        P = end_bit + (uint32_t)kJunkBits;
        idx = P >> 5;
        lo = wm1[idx];
        hi = wm1[idx + 1];
        pv = wm1[(int)idx - 1];
    }
    __device__ __forceinline__ uint32_t window(const uint32_t *) const {
        return __builtin_bitreverse32(__builtin_amdgcn_alignbit(hi, lo, P));
    }
    __device__ __forceinline__ void advance(const uint32_t *wm1, uint32_t used) {  // used <= 31
        P -= used;
        const uint32_t nidx = P >> 5;
        const bool adv = nidx != idx;
        hi = adv ? lo : hi;
        lo = adv ? pv : lo;
        idx = nidx;
        pv = wm1[(int)nidx - 1];
    }
};

// Decode CNT symbols from a window.  lut: 16-bit entries (symbol << 8) | code length, indexed by the next `bits`
// stream bits; mask2 = ((1 << bits) - 1) << 1.  CNT * (longest code word) <= kWindowBits is the caller's promise.
// e[] receives the entries; returns the number of bits used.
// `win` is left at the first bit that was not used, so that a further call continues in the same window.
template <int CNT>
__device__ __forceinline__ uint32_t lookup_more(uint32_t &win, const char *lut, uint32_t mask2, uint32_t (&e)[CNT]) {
    uint32_t tot = 0;
#pragma unroll
    for (int k = 0; k < CNT; k++) {
        e[k] = *reinterpret_cast<const uint16_t *>(lut + (win & mask2));
        win >>= (e[k] & 31u);
        tot += e[k];  // low byte: running sum of code lengths (at most 31, never carries)
    }
    return tot & 0xffu;
}
template <int CNT>
__device__ __forceinline__ uint32_t lookup(uint32_t win, const char *lut, uint32_t mask2, uint32_t (&e)[CNT]) {
    return lookup_more<CNT>(win, lut, mask2, e);
}

// the symbol of a table entry as fp32 (one v_cvt_f32_ubyte1)
__device__ __forceinline__ float sym_f32(uint32_t e) { return (float)(e >> 8); }

// The four chains of one lane (two slices x two directions) advance together, CNT symbols each.
struct Quad {
    UpReader au, bu;
    DownReader ad, bd;
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
    __device__ __forceinline__ void step(const uint32_t *wm1, const char *lut, uint32_t mask2, uint32_t (&fau)[CNT],
                                         uint32_t (&fad)[CNT], uint32_t (&fbu)[CNT], uint32_t (&fbd)[CNT]) {
        const uint32_t u0 = lookup<CNT>(au.window(wm1), lut, mask2, fau);
        const uint32_t u1 = lookup<CNT>(ad.window(wm1), lut, mask2, fad);
        const uint32_t u2 = lookup<CNT>(bu.window(wm1), lut, mask2, fbu);
        const uint32_t u3 = lookup<CNT>(bd.window(wm1), lut, mask2, fbd);
        au.advance(wm1, u0);
        ad.advance(wm1, u1);
        bu.advance(wm1, u2);
        bd.advance(wm1, u3);
    }
    // The same in pieces, for windows that hold more symbols than the caller wants table entries in flight:
    // begin(), then part<CNT>() once per piece (the pieces' CNT add up to what fits a window), then end().
    uint32_t w0, w1, w2, w3, u0, u1, u2, u3;  // the four windows and the bits used so far; live from begin() to end()
    __device__ __forceinline__ void begin(const uint32_t *wm1) {
        w0 = au.window(wm1);
        w1 = ad.window(wm1);
        w2 = bu.window(wm1);
        w3 = bd.window(wm1);
        u0 = u1 = u2 = u3 = 0;
    }
    template <int CNT>
    __device__ __forceinline__ void part(const char *lut, uint32_t mask2, uint32_t (&fau)[CNT], uint32_t (&fad)[CNT],
                                         uint32_t (&fbu)[CNT], uint32_t (&fbd)[CNT]) {
        u0 += lookup_more<CNT>(w0, lut, mask2, fau);
        u1 += lookup_more<CNT>(w1, lut, mask2, fad);
        u2 += lookup_more<CNT>(w2, lut, mask2, fbu);
        u3 += lookup_more<CNT>(w3, lut, mask2, fbd);
    }
    __device__ __forceinline__ void end(const uint32_t *wm1) {
        au.advance(wm1, u0);
        ad.advance(wm1, u1);
        bu.advance(wm1, u2);
        bd.advance(wm1, u3);
    }
};

constexpr int kHalf = kSliceLen / 2;  // symbols per chain

}  // namespace kvc
