// Fetch side (Section 3.3, Figure 1): one decode-attention step straight from the compressed cache.
//
// Per 2D block a single wavefront (64 lanes) stages the K record in LDS, every lane Huffman-decodes the two slices
// of one token with a lookup table -- each slice from both ends, four independent decode chains of 32 symbols per
// lane -- and accumulates q.k in registers; the wave then updates a running softmax and decodes the V record of the
// same block, every lane owning two channels (two slices, again four chains) and accumulating p.v in registers.  No
// decompressed value ever leaves the registers (Section 3.3.2): groups of 4 and 8 query heads keep the decoded
// quantization codes packed four to a register and hand them to the matrix cores from there.
//
// What differs from the paper's kernel, and why (gfx950):
//  * lookup-table decode instead of the bit-serial tree walk of Section 3.3.1: all 64 lanes of a wave advance in
//    symbol lock-step (same trip count for every lane, no divergence), so the dequantization weight of the current
//    symbol is the same for the whole wave.  For groups of 1 and 2 query heads it reaches the FMA through a DPP quad
//    broadcast of values fetched from LDS once per four steps, which keeps it off the VALU and nearly off the LDS pipe
//    that the table lookups load; for groups of 4 and 8 the wave packs the decoded bytes into registers and multiplies
//    them with the weights of all heads on int8 MFMA (see "tile path" below).  The table is
//    indexed by as many stream bits as the longest code word of the codebook, and one 32-bit window serves several
//    symbols (floor(31 / table width)) with no refill test in between;
//  * the dequantization is folded into the weights: q.k' = sum_c q_c min_c + sum_c (q_c step_c) code_tc, and
//    p.v'  = sum_t p_t min_t + sum_t (p_t step_t) code_tc: one convert and one FMA per decoded symbol;
//  * K and V of a block are handled by the same wave back to back with an online softmax, so scores never go to
//    memory; while one record is decoded the next one is already on its way from HBM into registers (tile path:
//    straight into LDS while the products of the previous record run);
//  * the sequence is split over workgroups; the workgroup that finishes last merges the splits (the "sum
//    reduction" of Section 3.3.2) inside the same launch.
#include <hip/hip_fp16.h>

#include "huff_decode.cuh"
#include "kvcomp_internal.h"
#include "split_combine.cuh"

namespace kvc {

struct FusedArgs {
    Geo g;
    const uint16_t *q;
    float *out;
    float scale;
    int n_blocks, res_head, n_res, blocks_per_split, n_splits, stage_bytes;
    uint32_t mask[2];   // table index mask of each tensor, already scaled to the byte offset of an entry
    // append fused into this launch: the newest buffered token (number new_row of the buffer, oldest = 0) is not in the
    // buffer yet but in k_new / v_new [B][H][128]; the wave that reads it also stores it there.  new_row < 0: none.
    const uint16_t *k_new, *v_new;
    int new_row;
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

// ---- accumulation of one round of decoded symbols -----------------------------------------------------------------
// The folded weight of the current symbol is wave-uniform.
//
// Query-head groups of 1 and 2: every fourth step, lane i of each quad of lanes fetches the weight of step s + i from
// LDS (four addresses, no bank conflict); the FMA of step s + i then takes it through a quad broadcast.  No
// instruction is spent on the broadcast itself.  (Groups of 4 and 8: the tile path further down.)
constexpr int kTileMinG = 4;  // smallest query-head group on the tile path

// acc + (w of lane Q of this lane's quad) * symbol: the quad broadcast is a DPP modifier of the FMA's first operand,
// no instruction of its own.  w must not have been written by a VALU instruction in the two instructions before
// (it comes from an LDS read).
template <int Q>
__device__ __forceinline__ float fma_quad_c(float w, float sym, float acc) {
    static_assert(Q >= 0 && Q < 4, "quad lane");
    if constexpr (Q == 0) asm("v_fmac_f32_dpp %0, %1, %2 quad_perm:[0,0,0,0] row_mask:0xf bank_mask:0xf" : "+v"(acc) : "v"(w), "v"(sym));
    if constexpr (Q == 1) asm("v_fmac_f32_dpp %0, %1, %2 quad_perm:[1,1,1,1] row_mask:0xf bank_mask:0xf" : "+v"(acc) : "v"(w), "v"(sym));
    if constexpr (Q == 2) asm("v_fmac_f32_dpp %0, %1, %2 quad_perm:[2,2,2,2] row_mask:0xf bank_mask:0xf" : "+v"(acc) : "v"(w), "v"(sym));
    if constexpr (Q == 3) asm("v_fmac_f32_dpp %0, %1, %2 quad_perm:[3,3,3,3] row_mask:0xf bank_mask:0xf" : "+v"(acc) : "v"(w), "v"(sym));
    return acc;
}
__device__ __forceinline__ float fma_quad(float w, int q, float sym, float acc) {
    switch (q & 3) {
        case 0: return fma_quad_c<0>(w, sym, acc);
        case 1: return fma_quad_c<1>(w, sym, acc);
        case 2: return fma_quad_c<2>(w, sym, acc);
        default: return fma_quad_c<3>(w, sym, acc);
    }
}

// K, groups of 1 and 2: symbol index `up` of chain au/bu is channel up / 64+up, index `dn` of chain ad/bd is channel
// dn / 64+dn.  wl = weights + (lane & 3) * G, wdn = weights - (lane & 3) * G, weights laid out [channel][head].
// CNT table entries of SP symbols each, the first of them symbol `first` of its chain.
template <int G, int CNT, int SP>
__device__ __forceinline__ void k_accum(const float *wl, const float *wdn, float (&wq)[4][G], int first,
                                        const uint32_t (&fau)[CNT], const uint32_t (&fad)[CNT],
                                        const uint32_t (&fbu)[CNT], const uint32_t (&fbd)[CNT], float (&acc)[G]) {
#pragma unroll
    for (int k = 0; k < CNT * SP; k++) {
        const int up = first + k, dn = kSliceLen - 1 - up;  // symbol index inside the slice
        const int q = up & 3;
        if (q == 0) {
#pragma unroll
            for (int g = 0; g < G; g++) {
                wq[0][g] = wl[up * G + g];
                wq[1][g] = wdn[dn * G + g];
                wq[2][g] = wl[(kSliceLen + up) * G + g];
                wq[3][g] = wdn[(kSliceLen + dn) * G + g];
            }
        }
        const bool second = SP == 2 && (k & 1);
        const float s0 = second ? sym2_f32(fau[k / SP]) : sym_f32(fau[k / SP]);
        const float s1 = second ? sym2_f32(fad[k / SP]) : sym_f32(fad[k / SP]);
        const float s2 = second ? sym2_f32(fbu[k / SP]) : sym_f32(fbu[k / SP]);
        const float s3 = second ? sym2_f32(fbd[k / SP]) : sym_f32(fbd[k / SP]);
#pragma unroll
        for (int g = 0; g < G; g++) {
            acc[g] = fma_quad(wq[0][g], q, s0, acc[g]);
            acc[g] = fma_quad(wq[1][g], q, s1, acc[g]);
            acc[g] = fma_quad(wq[2][g], q, s2, acc[g]);
            acc[g] = fma_quad(wq[3][g], q, s3, acc[g]);
        }
    }
}

// V, groups of 1 and 2: symbol index = token; chains au/ad belong to channel 2*lane, bu/bd to channel 2*lane+1.
template <int G, int CNT, int SP>
__device__ __forceinline__ void v_accum(const float *wl, const float *wdn, float (&wq)[2][G], int first,
                                        const uint32_t (&fau)[CNT], const uint32_t (&fad)[CNT],
                                        const uint32_t (&fbu)[CNT], const uint32_t (&fbd)[CNT], float (&acc)[G][2]) {
#pragma unroll
    for (int k = 0; k < CNT * SP; k++) {
        const int up = first + k, dn = kSliceLen - 1 - up;  // token index inside the block
        const int q = up & 3;
        if (q == 0) {
#pragma unroll
            for (int g = 0; g < G; g++) {
                wq[0][g] = wl[up * G + g];
                wq[1][g] = wdn[dn * G + g];
            }
        }
        const bool second = SP == 2 && (k & 1);
        const float s0 = second ? sym2_f32(fau[k / SP]) : sym_f32(fau[k / SP]);
        const float s1 = second ? sym2_f32(fad[k / SP]) : sym_f32(fad[k / SP]);
        const float s2 = second ? sym2_f32(fbu[k / SP]) : sym_f32(fbu[k / SP]);
        const float s3 = second ? sym2_f32(fbd[k / SP]) : sym_f32(fbd[k / SP]);
#pragma unroll
        for (int g = 0; g < G; g++) {
            acc[g][0] = fma_quad(wq[0][g], q, s0, acc[g][0]);
            acc[g][0] = fma_quad(wq[1][g], q, s1, acc[g][0]);
            acc[g][1] = fma_quad(wq[0][g], q, s2, acc[g][1]);
            acc[g][1] = fma_quad(wq[1][g], q, s3, acc[g][1]);
        }
    }
}

// ---- K block: lane = token; its two slices are channels 0..63 and 64..127 ------------------------------------------
// hdr32: the record (LDS or global); wts: this wave's LDS weight area.  Leaves scale * q.k' of this lane's token in
// score[].  LB: the table width the kernel is compiled for (see DecodeMode).
template <int G, int LB>
__device__ __forceinline__ void k_block(const uint32_t *hdr32, const char *lut, uint32_t mask, float *wts,
                                        const float (&qreg)[G][2], float two_eb, float scale, int lane, int kmm,
                                        float (&score)[G]) {
    using M = DecodeMode<LB>;
    constexpr int SP = M::kSymsPerLookup, NL = M::kLookupsPerWindow;
    // lane c holds the folded weights q_c * step_c of channels c and c + 64.  kmm = bytes of the {min,max} pairs in
    // the header: 512 (one pair per channel) or 16 (BlockQuant: one pair for the whole block)
    const bool per_channel = kmm == kMinMaxBytesK;
    const uint32_t mm0 = hdr32[per_channel ? lane : 0], mm1 = hdr32[per_channel ? lane + 64 : 0];
    const float mn0 = h2f(mm0 & 0xffffu), mn1 = h2f(mm1 & 0xffffu);
    const float st0 = two_eb * (h2f(mm0 >> 16) - mn0), st1 = two_eb * (h2f(mm1 >> 16) - mn1);
    float w0[G], w1[G], acc[G];
#pragma unroll
    for (int g = 0; g < G; g++) {
        w0[g] = qreg[g][0] * st0;
        w1[g] = qreg[g][1] * st1;
        acc[g] = 0.f;
    }
    const uint32_t sb = hdr32[kmm / 4 + lane];  // bit counts of slices 2*lane and 2*lane+1
    const uint32_t start = wave_excl_scan((sb & 0xffffu) + (sb >> 16), lane);
    const uint32_t *wm1 = hdr32 + (kmm + 2 * kSlices) / 4 - 1;
    constexpr int kRounds = M::kLookupsPerChain / NL, kTail = M::kLookupsPerChain - kRounds * NL;
    static_assert(G < kTileMinG, "groups of 4 and 8 take the tile path");
    Quad<M::J> qd;
    {
#pragma unroll
        for (int g = 0; g < G; g++) {  // LDS layout [channel][head]
            wts[lane * G + g] = w0[g];
            wts[(kSliceLen + lane) * G + g] = w1[g];
        }
        const float *wl = wts + (lane & 3) * G, *wdn = wts - (lane & 3) * G;
        float wq[4][G];
        wave_sync();
        qd.open(wm1, start, sb & 0xffffu, sb >> 16);
        // fully unrolled: the step number decides at compile time which quad lane holds the weight, and the
        // scheduler may overlap the table lookups of one round with the accumulation of the previous one
#pragma unroll
        for (int r = 0; r < kRounds; r++) {
            uint32_t fau[NL], fad[NL], fbu[NL], fbd[NL];
            qd.template step<NL>(wm1, lut, mask, fau, fad, fbu, fbd);
            k_accum<G, NL, SP>(wl, wdn, wq, r * NL * SP, fau, fad, fbu, fbd, acc);
        }
        if constexpr (kTail > 0) {
            uint32_t fau[kTail ? kTail : 1], fad[kTail ? kTail : 1], fbu[kTail ? kTail : 1], fbd[kTail ? kTail : 1];
            qd.template step<(kTail ? kTail : 1)>(wm1, lut, mask, fau, fad, fbu, fbd);
            k_accum<G, (kTail ? kTail : 1), SP>(wl, wdn, wq, kRounds * NL * SP, fau, fad, fbu, fbd, acc);
        }
    }
    // the constant part of the dot product, sum_c q_c min_c, is shared by all tokens of the block
#pragma unroll
    for (int g = 0; g < G; g++) score[g] = scale * (acc[g] + wave_sum(qreg[g][0] * mn0 + qreg[g][1] * mn1));
}

// ---- V block: lane = channels 2*lane and 2*lane+1 (its two slices) -------------------------------------------------
// p[g] = softmax numerator of token `lane`.
template <int G, int LB>
__device__ __forceinline__ void v_block(const uint32_t *hdr32, const char *lut, uint32_t mask, float *wts,
                                        const float (&p)[G], float two_eb, int lane, Soft<G> &st) {
    using M = DecodeMode<LB>;
    constexpr int SP = M::kSymsPerLookup, NL = M::kLookupsPerWindow;
    // lane t holds the folded weight p_t * step_t of token t
    const uint32_t mm = hdr32[lane];
    const float mn = h2f(mm & 0xffffu);
    const float step = two_eb * (h2f(mm >> 16) - mn);
    float w[G];
#pragma unroll
    for (int g = 0; g < G; g++) {
        w[g] = p[g] * step;
        st.bv[g] += p[g] * mn;
    }
    const uint32_t sb = hdr32[kMinMaxBytesV / 4 + lane];
    const uint32_t start = wave_excl_scan((sb & 0xffffu) + (sb >> 16), lane);
    const uint32_t *wm1 = hdr32 + kHdrBytesV / 4 - 1;
    constexpr int kRounds = M::kLookupsPerChain / NL, kTail = M::kLookupsPerChain - kRounds * NL;
    static_assert(G < kTileMinG, "groups of 4 and 8 take the tile path");
    Quad<M::J> qd;
    {
#pragma unroll
        for (int g = 0; g < G; g++) wts[lane * G + g] = w[g];  // LDS layout [token][head]
        const float *wl = wts + (lane & 3) * G, *wdn = wts - (lane & 3) * G;
        float wq[2][G];
        wave_sync();
        qd.open(wm1, start, sb & 0xffffu, sb >> 16);
#pragma unroll
        for (int r = 0; r < kRounds; r++) {
            uint32_t fau[NL], fad[NL], fbu[NL], fbd[NL];
            qd.template step<NL>(wm1, lut, mask, fau, fad, fbu, fbd);
            v_accum<G, NL, SP>(wl, wdn, wq, r * NL * SP, fau, fad, fbu, fbd, st.acc);
        }
        if constexpr (kTail > 0) {
            uint32_t fau[kTail ? kTail : 1], fad[kTail ? kTail : 1], fbu[kTail ? kTail : 1], fbd[kTail ? kTail : 1];
            qd.template step<(kTail ? kTail : 1)>(wm1, lut, mask, fau, fad, fbu, fbd);
            v_accum<G, (kTail ? kTail : 1), SP>(wl, wdn, wq, kRounds * NL * SP, fau, fad, fbu, fbd, st.acc);
        }
    }
}

// Rare path: a record larger than the LDS staging area is decoded straight from global memory.  Kept out of line so
// that it costs the common path no registers.
template <int G, int LB>
__device__ __noinline__ void k_block_global(const uint32_t *rec, const char *lut, uint32_t mask, float *wts,
                                            const float (&qreg)[G][2], float two_eb, float scale, int lane, int kmm,
                                            float (&score)[G]) {
    k_block<G, LB>(rec, lut, mask, wts, qreg, two_eb, scale, lane, kmm, score);
}
template <int G, int LB>
__device__ __noinline__ void v_block_global(const uint32_t *rec, const char *lut, uint32_t mask, float *wts,
                                            const float (&p)[G], float two_eb, int lane, Soft<G> &st) {
    v_block<G, LB>(rec, lut, mask, wts, p, two_eb, lane, st);
}

// ---- groups of 4 and 8 query heads, tile path ---------------------------------------------------------------------
// With several query heads per KV head the update of the accumulators is a matrix product, (heads x symbols) weights
// times the decoded block, and the decode itself is the same for all heads.  The wave therefore only packs the
// decoded symbols, four table entries to a register -- less work than one conversion and one FMA per symbol and
// head -- and multiplies them with the folded weights on v_mfma_i32_32x32x16_i8, whose result tiles (32 rows of
// weights x 32 columns) give the path its name:
//   * the table holds the symbols biased by -128 (symbol ^ 0x80 read as int8), so a register of packed symbols is an
//     MFMA operand as it is, with no conversion; the operand wants 32 columns x 16 positions from 64 lanes that hold
//     one slice each, which one v_permlane32_swap_b32 per register arranges (step_operands);
//   * a weight w is scaled by a per-block power of two to an integer W below 2^22 and split into three signed bytes,
//     W = sum_j d_j 256^j; row 4 * head + j of the A operand holds digit j, the products are exact in int32, and the
//     digit rows of a head land in the same lane of the result, where they are recombined in fp32;
//   * sum_c W_c (s_c - 128) misses 128 * sum_c W_c, which joins the constant term of the block.
// Lane l of the result tiles holds column l % 32 (token of a K block, channel of a V block) for the heads
// l / 32 + 2 i: the running softmax state lives in that layout and is converted to the per-channel layout of the
// other paths once, after the last block.
typedef int v16i __attribute__((ext_vector_type(16)));

template <int G>
struct TileSoft {
    static constexpr int HL = G / 2;  // heads per lane: l / 32 + 2 i
    float m[HL], l[HL], bv[HL], acc[HL][4];  // l, bv: this lane's share; acc[i][ct]: channel 32 ct + l % 32
    __device__ __forceinline__ void init() {
#pragma unroll
        for (int i = 0; i < HL; i++) {
            m[i] = -INFINITY; l[i] = 0.f; bv[i] = 0.f;
#pragma unroll
            for (int c = 0; c < 4; c++) acc[i][c] = 0.f;
        }
    }
};

// maximum / sum over the 32 lanes of this lane's half of the wave
__device__ __forceinline__ float half_max(float v, bool upper) {
    v = fmaxf(v, dpp_f<kDppXor1>(v));
    v = fmaxf(v, dpp_f<kDppXor2>(v));
    v = fmaxf(v, dpp_f<kDppHalfMirror>(v));
    v = fmaxf(v, dpp_f<kDppMirror>(v));
    const float lo = fmaxf(bcast(v, 0), bcast(v, 16)), hi = fmaxf(bcast(v, 32), bcast(v, 48));
    return upper ? hi : lo;
}
__device__ __forceinline__ float half_sum(float v, bool upper) {
    v += dpp_f<kDppXor1>(v);
    v += dpp_f<kDppXor2>(v);
    v += dpp_f<kDppHalfMirror>(v);
    v += dpp_f<kDppMirror>(v);
    const float lo = bcast(v, 0) + bcast(v, 16), hi = bcast(v, 32) + bcast(v, 48);
    return upper ? hi : lo;
}

// bytes 1 of four table entries (the biased symbols) as one word, first entry in the lowest byte
__device__ __forceinline__ uint32_t pack_syms(uint32_t e0, uint32_t e1, uint32_t e2, uint32_t e3) {
    const uint32_t lo = __builtin_amdgcn_perm(e1, e0, 0x0c0c0501u), hi = __builtin_amdgcn_perm(e3, e2, 0x0c0c0501u);
    return __builtin_amdgcn_perm(hi, lo, 0x05040100u);
}
// the same from two entries of the pair table (bytes 1 and 2 of each are two consecutive symbols): e0's symbols in
// the two lowest bytes; and with the four symbols in the opposite order (a chain that was read downwards)
__device__ __forceinline__ uint32_t pack_pairs(uint32_t e0, uint32_t e1) { return __builtin_amdgcn_perm(e1, e0, 0x06050201u); }
__device__ __forceinline__ uint32_t pack_pairs_rev(uint32_t e0, uint32_t e1) { return __builtin_amdgcn_perm(e1, e0, 0x01020506u); }

// The table entries of a lane's four chains while they wait to be packed (fully unrolled code: an entry lives in a
// register from its lookup to the packing of its word).  NE entries per chain: 32 one-symbol or 16 two-symbol ones.
template <int NE>
struct ChainSyms {
    uint32_t au[NE], ad[NE], bu[NE], bd[NE];
};
// The decoded symbols (biased bytes) of the lane's two slices, four per word, in ascending position inside the slice:
// word j of a slice holds positions 4j .. 4j+3.  The up chain delivers words 0, 1, .. and the down chain 15, 14, ..
struct SliceWords {
    uint32_t a[16], b[16];
};
// Decodes symbols S0 .. S1-1 of this lane's four chains (whole windows from S0 on; the last window of a chain may be
// short) and packs every word whose four symbols are there.
template <int LB, int S0, int S1>
__device__ __forceinline__ void decode_span(Quad<DecodeMode<LB>::J> &qd, const uint32_t *wm1, const char *lut, uint32_t mask,
                                            ChainSyms<DecodeMode<LB>::kLookupsPerChain> &e, SliceWords &p) {
    using M = DecodeMode<LB>;
    constexpr int SP = M::kSymsPerLookup, NL = M::kLookupsPerWindow, NS = M::kSymsPerWindow;
    static_assert(S0 % NS == 0 && S0 < S1 && S1 <= kHalf && (S1 % NS == 0 || S1 == kHalf), "whole windows");
    auto pack_words = [&](int w0, int w1) {
#pragma unroll
        for (int w = w0; w < w1; w++) {
            if constexpr (SP == 1) {
                p.a[w] = pack_syms(e.au[4 * w], e.au[4 * w + 1], e.au[4 * w + 2], e.au[4 * w + 3]);
                p.a[15 - w] = pack_syms(e.ad[4 * w + 3], e.ad[4 * w + 2], e.ad[4 * w + 1], e.ad[4 * w]);
                p.b[w] = pack_syms(e.bu[4 * w], e.bu[4 * w + 1], e.bu[4 * w + 2], e.bu[4 * w + 3]);
                p.b[15 - w] = pack_syms(e.bd[4 * w + 3], e.bd[4 * w + 2], e.bd[4 * w + 1], e.bd[4 * w]);
            } else {
                p.a[w] = pack_pairs(e.au[2 * w], e.au[2 * w + 1]);
                p.a[15 - w] = pack_pairs_rev(e.ad[2 * w], e.ad[2 * w + 1]);
                p.b[w] = pack_pairs(e.bu[2 * w], e.bu[2 * w + 1]);
                p.b[15 - w] = pack_pairs_rev(e.bd[2 * w], e.bd[2 * w + 1]);
            }
        }
    };
    constexpr int kFull = (S1 - S0) / NS, kTailSyms = (S1 - S0) - kFull * NS, kTail = kTailSyms / SP;
    static_assert(kTailSyms % SP == 0, "a span ends on a whole table entry");
#pragma unroll
    for (int r = 0; r < kFull; r++) {
        uint32_t fau[NL], fad[NL], fbu[NL], fbd[NL];
        qd.template step<NL>(wm1, lut, mask, fau, fad, fbu, fbd);
        const int s = S0 + r * NS;
#pragma unroll
        for (int k = 0; k < NL; k++) {
            e.au[s / SP + k] = fau[k]; e.ad[s / SP + k] = fad[k]; e.bu[s / SP + k] = fbu[k]; e.bd[s / SP + k] = fbd[k];
        }
        pack_words(s / 4, (s + NS) / 4);
    }
    if constexpr (kTail > 0) {
        uint32_t fau[kTail ? kTail : 1], fad[kTail ? kTail : 1], fbu[kTail ? kTail : 1], fbd[kTail ? kTail : 1];
        qd.template step<(kTail ? kTail : 1)>(wm1, lut, mask, fau, fad, fbu, fbd);
        constexpr int s = S0 + kFull * NS;
#pragma unroll
        for (int k = 0; k < kTail; k++) {
            e.au[s / SP + k] = fau[k]; e.ad[s / SP + k] = fad[k]; e.bu[s / SP + k] = fbu[k]; e.bd[s / SP + k] = fbd[k];
        }
        pack_words(s / 4, (s + kTailSyms) / 4);
    }
}
// first symbol that the second span of a block decodes when the products run after each half: the first half's
// windows are whole, so they may reach into the second half
constexpr int tile_first_span(int NS) { return (16 + NS - 1) / NS * NS; }

// The B operands of v_mfma_i32_32x32x16_i8 for one step of 16 positions (words w[0..3] of a slice) straight from
// registers.  Lane l of the operand supplies column l % 32 and positions 8 (l / 32) .. +7.  With one slice per lane and
// 64 lanes there are two column tiles: tile 0 wants words 0, 1 of lanes 0..31 in its lower half and words 2, 3 of the
// same lanes in its upper half, tile 1 words 0, 1 of lanes 32..63 in its lower half and their words 2, 3 in its upper
// half -- which is what v_permlane32_swap_b32 makes of (word 0, word 2) and of (word 1, word 3).
typedef unsigned int v2u __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void step_operands(uint32_t w0, uint32_t w1, uint32_t w2, uint32_t w3, long &tile0, long &tile1) {
    const v2u r0 = __builtin_amdgcn_permlane32_swap(w0, w2, false, false);
    const v2u r1 = __builtin_amdgcn_permlane32_swap(w1, w3, false, false);
    tile0 = (long)(((unsigned long long)r1.x << 32) | r0.x);
    tile1 = (long)(((unsigned long long)r1.y << 32) | r0.y);
}

// power-of-two factor that brings the largest weight of the wave into [2^21, 2^22) (1 if all are zero); *inv = 1/f
__device__ __forceinline__ float int_scale(float amax, float *inv) {
    const float m = wave_max(amax);
    int e = 0;
    if (m > 0.f) (void)frexpf(m, &e);  // m = f * 2^e, f in [0.5, 1)
    const int up = min(22 - e, 120);
    *inv = ldexpf(1.f, -up);
    return m > 0.f ? ldexpf(1.f, up) : 1.f;
}
// |W| <= 2^22 as d2 2^16 + d1 2^8 + d0 with signed bytes d_j: bytes 0..2 of the result
__device__ __forceinline__ uint32_t signed_digits(int W) { return ((uint32_t)W + 0x00008080u) ^ 0x00008080u; }
// Rounding to an integer inside the multiplication: for |a * b| <= 2^22, fma(a, b, 1.5 * 2^23) is rounded (to nearest,
// ties to even) at unit spacing, and its bit pattern is kMagicBits + W with W = rint(a * b), also across the binade
// boundary at W = 2^22.  One instruction instead of a product, a rounding and a conversion; W stays implicit:
//   magic_digits(bits) = signed_digits(W), and sums of W are sums of bit patterns minus n * kMagicBits.
constexpr float kMagic = 12582912.f;          // 1.5 * 2^23
constexpr uint32_t kMagicBits = 0x4B400000u;  // its bit pattern
__device__ __forceinline__ uint32_t magic_round(float a, float b) { return __float_as_uint(fmaf(a, b, kMagic)); }
__device__ __forceinline__ uint32_t magic_digits(uint32_t bits) { return (bits + (0x00008080u - kMagicBits)) ^ 0x00008080u; }
// words a..d (byte j = digit j of four consecutive columns) -> o[j] = digit j of the four columns, j < 3
__device__ __forceinline__ void transpose_digits(uint32_t a, uint32_t b, uint32_t c, uint32_t d, uint32_t (&o)[3]) {
    const uint32_t t0 = __builtin_amdgcn_perm(b, a, 0x05010400u), t1 = __builtin_amdgcn_perm(b, a, 0x07030602u);
    const uint32_t t2 = __builtin_amdgcn_perm(d, c, 0x05010400u), t3 = __builtin_amdgcn_perm(d, c, 0x07030602u);
    o[0] = __builtin_amdgcn_perm(t2, t0, 0x05040100u);
    o[1] = __builtin_amdgcn_perm(t2, t0, 0x07060302u);
    o[2] = __builtin_amdgcn_perm(t3, t1, 0x05040100u);
}
__device__ __forceinline__ long lds_pair(const uint8_t *p) {
    const uint32_t *w = reinterpret_cast<const uint32_t *>(p);
    return (long)(((unsigned long long)w[1] << 32) | w[0]);
}
// the digit sums of one head, rows 4 i .. 4 i + 2 of a result tile, as one number
template <int I>
__device__ __forceinline__ float join_digits(const v16i &d) {
    return fmaf(fmaf((float)d[4 * I + 2], 256.f, (float)d[4 * I + 1]), 256.f, (float)d[4 * I]);
}
template <int HL>
__device__ __forceinline__ void join_all(const v16i &d, float (&out)[HL]) {
    out[0] = join_digits<0>(d);
    out[1] = join_digits<1>(d);
    if constexpr (HL > 2) {
        out[HL > 2 ? 2 : 0] = join_digits<2>(d);
        out[HL > 2 ? 3 : 0] = join_digits<3>(d);
    }
}
// Bytes per row of the A operand while it is laid out in the tile area.  Only the three digit rows of every head are
// stored: row 4 * head + digit of the operand sits at row a_row() of the area; the operand's remaining rows are zero.
constexpr int kARowK = kARowBytes, kARowV = kBT + 4;
// x = row of the A operand that a lane supplies -> its row in the area (rows without a digit read a neighbour's and
// are cleared afterwards)
template <int G>
__device__ __forceinline__ int a_row(int x) {
    const int xr = min(x, 4 * G - 1);
    return 3 * (xr >> 2) + min(xr & 3, 2);
}

// How far a score may exceed the softmax reference before the state is rescaled.  The numerators of a block then
// reach e^kLazyMax, and because the integer weights of all heads share one power-of-two scale per block, a head
// whose reference is behind costs the other heads that factor in weight resolution: 2 keeps the attention error
// within a factor 8 of rescaling always (measured at the 70B shape: 1e-5 instead of 4e-6; with 8 it reached 1e-3).
constexpr float kLazyMax = 2.f;

// K block.  hdr32: the record (LDS or global); tile: this wave's LDS area for laying out the A operand; qf: the query
// rows in LDS.
// Updates the softmax state and leaves the softmax numerators of tokens l%32 and 32 + l%32 in p.
// record_done() is called once the record has been read for the last time, before the last products: the place to
// request the next record, whose loads then travel while few registers are live.
template <int G, int LB, class F>
__device__ __forceinline__ void k_tile_block(const uint32_t *hdr32, const char *lut, uint32_t mask2, uint8_t *tile,
                                             const float *qf, float two_eb, float scale, int lane, int kmm,
                                             TileSoft<G> &ts, float (&p)[G / 2][2], F &&record_done) {
    constexpr int HL = G / 2;
    // everything derived from the lane number is recomputed per block (a few instructions) instead of being kept in
    // registers, or spilled, across the whole decode loop
    asm volatile("" : "+v"(lane));
    const int x = lane & 31, hv = lane >> 5;
    const bool upper = hv != 0;
    const bool per_channel = kmm == kMinMaxBytesK;
    // the A operand: folded weights q_c * step_c as integers, heads l/32 + 2i, channels 4 (l%32) .. +3
    float cst[HL], inv;
    long a[8];
    {
        float mn[4], stp[4];
#pragma unroll
        for (int c = 0; c < 4; c++) {
            const uint32_t mm = hdr32[per_channel ? 4 * x + c : 0];
            mn[c] = h2f(mm & 0xffffu);
            stp[c] = two_eb * (h2f(mm >> 16) - mn[c]);
        }
        float qa[HL][4], amax = 0.f;
#pragma unroll
        for (int c = 0; c < 4; c++) {   // the largest |q_c step_c| of this lane: steps are not negative
            float qmax = 0.f;
#pragma unroll
            for (int i = 0; i < HL; i++) {
                qa[i][c] = qf[(hv + 2 * i) * kD + 4 * x + c];
                qmax = fmaxf(qmax, fabsf(qa[i][c]));
            }
            amax = fmaxf(amax, qmax * stp[c]);
        }
        const float f = int_scale(amax, &inv);
#pragma unroll
        for (int c = 0; c < 4; c++) stp[c] *= f;   // exact: f is a power of two
#pragma unroll
        for (int i = 0; i < HL; i++) {
            uint32_t dg[4], wbits = 0;
            float qm = 0.f;
#pragma unroll
            for (int c = 0; c < 4; c++) {
                const uint32_t bits = magic_round(qa[i][c], stp[c]);  // W = rint(q_c step_c f), |W| <= 2^22
                wbits += bits;
                qm = fmaf(qa[i][c], mn[c], qm);
                dg[c] = magic_digits(bits);
            }
            const float wsum = (float)(int)(wbits - 4u * kMagicBits);
            uint32_t rows[3];
            transpose_digits(dg[0], dg[1], dg[2], dg[3], rows);
            const int head = hv + 2 * i;
#pragma unroll
            for (int j = 0; j < 3; j++) *reinterpret_cast<uint32_t *>(tile + (3 * head + j) * kARowK + 4 * x) = rows[j];
            cst[i] = half_sum(fmaf(128.f * inv, wsum, qm), upper);
        }
        wave_sync();
#pragma unroll
        for (int ks = 0; ks < 8; ks++) {
            a[ks] = lds_pair(tile + a_row<G>(x) * kARowK + 16 * ks + 8 * hv);
            if ((x & 3) == 3 || x >= 4 * G) a[ks] = 0;  // rows that hold no digit
        }
        wave_sync();
    }
    const uint32_t sb = hdr32[kmm / 4 + lane];  // bit counts of slices 2*lane and 2*lane+1
    const uint32_t start = wave_excl_scan((sb & 0xffffu) + (sb >> 16), lane);
    const uint32_t *wm1 = hdr32 + (kmm + 2 * kSlices) / 4 - 1;
    Quad<DecodeMode<LB>::J> qd;
    qd.open(wm1, start, sb & 0xffffu, sb >> 16);
    constexpr bool kBoth = tile_halves_at_once(G, LB) == 2;  // one recombination per block instead of one per half
    float sc[HL][2];
    v16i d[2];  // result tiles: tokens 0..31 and 32..63
    ChainSyms<DecodeMode<LB>::kLookupsPerChain> syms;
    SliceWords pw;  // lane = token: slice a = its channels 0..63, slice b = its channels 64..127
    // one step of 16 channels of either slice: steps 0..3 are channels 0..63, steps 4..7 channels 64..127
    // fresh: the result tiles start at zero (the matrix instruction takes the constant as its addend: no register
    // is cleared)
    auto products = [&](int ks, bool fresh) {
        const v16i zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
        long t0, t1;
        step_operands(pw.a[4 * ks], pw.a[4 * ks + 1], pw.a[4 * ks + 2], pw.a[4 * ks + 3], t0, t1);
        d[0] = __builtin_amdgcn_mfma_i32_32x32x16_i8(a[ks], t0, fresh ? zero : d[0], 0, 0, 0);
        d[1] = __builtin_amdgcn_mfma_i32_32x32x16_i8(a[ks], t1, fresh ? zero : d[1], 0, 0, 0);
        step_operands(pw.b[4 * ks], pw.b[4 * ks + 1], pw.b[4 * ks + 2], pw.b[4 * ks + 3], t0, t1);
        d[0] = __builtin_amdgcn_mfma_i32_32x32x16_i8(a[4 + ks], t0, d[0], 0, 0, 0);
        d[1] = __builtin_amdgcn_mfma_i32_32x32x16_i8(a[4 + ks], t1, d[1], 0, 0, 0);
    };
    auto join = [&](bool first) {
#pragma unroll
        for (int t = 0; t < 2; t++) {
            float v[HL];
            join_all<HL>(d[t], v);
#pragma unroll
            for (int i = 0; i < HL; i++) sc[i][t] = first ? v[i] : sc[i][t] + v[i];
        }
    };
    constexpr int kP = tile_first_span(DecodeMode<LB>::kSymsPerWindow);
    // a half of a block is 16 symbols of every chain: the up chains deliver step h, the down chains step 3 - h
    // The products of the first half run while the second half is decoded (no fence in between: everything is in
    // registers).
    decode_span<LB, 0, kP>(qd, wm1, lut, mask2, syms, pw);
    products(0, true);
    products(3, false);
    if constexpr (!kBoth) join(true);
    decode_span<LB, kP, kHalf>(qd, wm1, lut, mask2, syms, pw);
    wave_sync();
    record_done();
    products(1, !kBoth);
    products(2, false);
    join(kBoth);
    // Online softmax with a reference value m that only moves when it has to: the state is rescaled (a maximum over
    // the tokens of every head, six multiplications per head) only when some score of the block exceeds its head's m
    // by more than kLazyMax, which after the first blocks of a sequence split is rare.  Until then the numerators are
    // at most e^kLazyMax instead of 1; the merges divide by the same m.
    const float si = scale * inv;
    float over = -INFINITY;
#pragma unroll
    for (int i = 0; i < HL; i++) {
        const float sk = scale * cst[i];
        sc[i][0] = fmaf(si, sc[i][0], sk);
        sc[i][1] = fmaf(si, sc[i][1], sk);
        over = fmaxf(over, fmaxf(sc[i][0], sc[i][1]) - ts.m[i]);   // m = -inf before the first block: +inf
    }
    if (__builtin_amdgcn_ballot_w64(over > kLazyMax) != 0) {
#pragma unroll
        for (int i = 0; i < HL; i++) {
            const float mnew = fmaxf(ts.m[i], half_max(fmaxf(sc[i][0], sc[i][1]), upper));
            const float alpha = __expf(ts.m[i] - mnew);
            ts.l[i] *= alpha;
            ts.bv[i] *= alpha;
#pragma unroll
            for (int c = 0; c < 4; c++) ts.acc[i][c] *= alpha;
            ts.m[i] = mnew;
        }
    }
#pragma unroll
    for (int i = 0; i < HL; i++) {
        p[i][0] = __expf(sc[i][0] - ts.m[i]);
        p[i][1] = __expf(sc[i][1] - ts.m[i]);
        ts.l[i] += p[i][0] + p[i][1];
    }
}

// V block.  p: softmax numerators of tokens l%32 and 32 + l%32 for this lane's heads.
template <int G, int LB, class F>
__device__ __forceinline__ void v_tile_block(const uint32_t *hdr32, const char *lut, uint32_t mask2, uint8_t *tile,
                                             const float (&p)[G / 2][2], float two_eb, int lane, TileSoft<G> &ts,
                                             F &&record_done) {
    constexpr int HL = G / 2;
    asm volatile("" : "+v"(lane));
    const int x = lane & 31, hv = lane >> 5;
    float inv;
    long a[4];
    {
        float mn[2], stp[2];
#pragma unroll
        for (int t = 0; t < 2; t++) {
            const uint32_t mm = hdr32[32 * t + x];
            mn[t] = h2f(mm & 0xffffu);
            stp[t] = two_eb * (h2f(mm >> 16) - mn[t]);
        }
        float pmax[2] = {0.f, 0.f};
#pragma unroll
        for (int i = 0; i < HL; i++) {
            pmax[0] = fmaxf(pmax[0], p[i][0]);
            pmax[1] = fmaxf(pmax[1], p[i][1]);
        }
        const float f = int_scale(fmaxf(pmax[0] * stp[0], pmax[1] * stp[1]), &inv);
        stp[0] *= f;   // exact: f is a power of two
        stp[1] *= f;
#pragma unroll
        for (int i = 0; i < HL; i++) {
            const int head = hv + 2 * i;
            uint32_t wbits = 0;
#pragma unroll
            for (int t = 0; t < 2; t++) {
                const uint32_t bits = magic_round(p[i][t], stp[t]);  // W = rint(p_t step_t f), |W| <= 2^22
                wbits += bits;
                const uint32_t dg = magic_digits(bits);
#pragma unroll
                for (int j = 0; j < 3; j++) tile[(3 * head + j) * kARowV + 32 * t + x] = (uint8_t)(dg >> (8 * j));
            }
            const float wsum = (float)(int)(wbits - 2u * kMagicBits);
            ts.bv[i] += fmaf(128.f * inv, wsum, fmaf(p[i][0], mn[0], p[i][1] * mn[1]));
        }
        wave_sync();
#pragma unroll
        for (int ks = 0; ks < 4; ks++) {
            a[ks] = lds_pair(tile + a_row<G>(x) * kARowV + 16 * ks + 8 * hv);
            if ((x & 3) == 3 || x >= 4 * G) a[ks] = 0;
        }
        wave_sync();
    }
    // lane = channels lane (slice a) and 64 + lane (slice b), so that a result tile of 32 channels is one slice of 32
    // neighbouring lanes; slice s starts where the bits of slices 0 .. s-1 end
    const uint16_t *bits16 = reinterpret_cast<const uint16_t *>(hdr32 + kMinMaxBytesV / 4);
    const uint32_t abits = bits16[lane], bbits = bits16[kSliceLen + lane];
    const uint32_t start_a = wave_excl_scan(abits, lane);
    const uint32_t start_b = (uint32_t)__builtin_amdgcn_readlane((int)(start_a + abits), 63) + wave_excl_scan(bbits, lane);
    const uint32_t *wm1 = hdr32 + kHdrBytesV / 4 - 1;
    Quad<DecodeMode<LB>::J> qd;
    qd.open2(wm1, start_a, abits, start_b, bbits);
    constexpr bool kBoth = tile_halves_at_once(G, LB) == 2;
    v16i d[4];  // result tiles: channels 0..31, 32..63 (slice a), 64..95, 96..127 (slice b)
    ChainSyms<DecodeMode<LB>::kLookupsPerChain> syms;
    SliceWords pw;
    // one step of 16 tokens of both slices
    auto products = [&](int ks, bool fresh) {   // fresh: the result tiles start at zero
        const v16i zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
        long t0, t1;
        step_operands(pw.a[4 * ks], pw.a[4 * ks + 1], pw.a[4 * ks + 2], pw.a[4 * ks + 3], t0, t1);
        d[0] = __builtin_amdgcn_mfma_i32_32x32x16_i8(a[ks], t0, fresh ? zero : d[0], 0, 0, 0);
        d[1] = __builtin_amdgcn_mfma_i32_32x32x16_i8(a[ks], t1, fresh ? zero : d[1], 0, 0, 0);
        step_operands(pw.b[4 * ks], pw.b[4 * ks + 1], pw.b[4 * ks + 2], pw.b[4 * ks + 3], t0, t1);
        d[2] = __builtin_amdgcn_mfma_i32_32x32x16_i8(a[ks], t0, fresh ? zero : d[2], 0, 0, 0);
        d[3] = __builtin_amdgcn_mfma_i32_32x32x16_i8(a[ks], t1, fresh ? zero : d[3], 0, 0, 0);
    };
    auto join = [&] {
#pragma unroll
        for (int ct = 0; ct < 4; ct++) {
            float v[HL];
            join_all<HL>(d[ct], v);
#pragma unroll
            for (int i = 0; i < HL; i++) ts.acc[i][ct] = fmaf(inv, v[i], ts.acc[i][ct]);
        }
    };
    constexpr int kP = tile_first_span(DecodeMode<LB>::kSymsPerWindow);
    decode_span<LB, 0, kP>(qd, wm1, lut, mask2, syms, pw);
    products(0, true);
    products(3, false);
    if constexpr (!kBoth) join();
    decode_span<LB, kP, kHalf>(qd, wm1, lut, mask2, syms, pw);
    wave_sync();
    record_done();
    products(1, !kBoth);
    products(2, false);
    join();
}

// Rare path: a record larger than the LDS staging area (one that an append flushed after the host last looked at the
// record sizes) is decoded straight from global memory, out of line.
template <int G, int LB>
__device__ __noinline__ void k_tile_block_global(const uint32_t *rec, const char *lut, uint32_t mask2, uint8_t *tile,
                                                 const float *qf, float two_eb, float scale, int lane, int kmm,
                                                 TileSoft<G> &ts, float (&p)[G / 2][2]) {
    k_tile_block<G, LB>(rec, lut, mask2, tile, qf, two_eb, scale, lane, kmm, ts, p, [] {});
}
template <int G, int LB>
__device__ __noinline__ void v_tile_block_global(const uint32_t *rec, const char *lut, uint32_t mask2, uint8_t *tile,
                                                 const float (&p)[G / 2][2], float two_eb, int lane, TileSoft<G> &ts) {
    v_tile_block<G, LB>(rec, lut, mask2, tile, p, two_eb, lane, ts, [] {});
}

// A wave's softmax state parked in LDS, G * 128 + 3 * G floats: o[g][channel] then {m, l, bv} per head with l and bv
// already summed over the lanes.  The state crosses the call of the out-of-line buffered-token code this way (through
// a reference it would cross in scratch memory, i.e. through the memory system: microseconds on the critical path of
// the wave that finishes last), and the tile path changes its layout this way.
template <int G>
__device__ __forceinline__ void soft_to_area(const Soft<G> &st, float *area, int lane) {
    wave_sync();
#pragma unroll
    for (int g = 0; g < G; g++) {
        area[g * kD + 2 * lane] = st.acc[g][0];
        area[g * kD + 2 * lane + 1] = st.acc[g][1];
        const float l = wave_sum(st.l[g]), bv = wave_sum(st.bv[g]);
        if (lane == 0) {
            area[G * kD + 3 * g] = st.m[g];
            area[G * kD + 3 * g + 1] = l;
            area[G * kD + 3 * g + 2] = bv;
        }
    }
    wave_sync();
}
// lane = channels 2*lane, 2*lane+1 of every head; l and bv in lane 0 only
template <int G>
__device__ __forceinline__ void area_to_soft(const float *area, int lane, Soft<G> &st) {
    wave_sync();
#pragma unroll
    for (int g = 0; g < G; g++) {
        st.acc[g][0] = area[g * kD + 2 * lane];
        st.acc[g][1] = area[g * kD + 2 * lane + 1];
        st.m[g] = area[G * kD + 3 * g];
        st.l[g] = lane == 0 ? area[G * kD + 3 * g + 1] : 0.f;
        st.bv[g] = lane == 0 ? area[G * kD + 3 * g + 2] : 0.f;
    }
    wave_sync();
}
// the tile path's state (lane l: column l % 32, heads l / 32 + 2 i) into the area
template <int G>
__device__ __forceinline__ void tile_state_to_area(const TileSoft<G> &ts, float *area, int lane) {
    constexpr int HL = G / 2;
    const int x = lane & 31, hv = lane >> 5;
    wave_sync();
#pragma unroll
    for (int i = 0; i < HL; i++) {
        const int head = hv + 2 * i;
#pragma unroll
        for (int ct = 0; ct < 4; ct++) area[head * kD + 32 * ct + x] = ts.acc[i][ct];
        const float l = half_sum(ts.l[i], hv != 0), bv = half_sum(ts.bv[i], hv != 0);
        if (x == 0) {
            area[G * kD + 3 * head] = ts.m[i];
            area[G * kD + 3 * head + 1] = l;
            area[G * kD + 3 * head + 2] = bv;
        }
    }
    wave_sync();
}


// The buffered fp16 tokens (Section 3.2.3: the newest vectors take part too), in units of 16 tokens; this wave takes
// units first_unit, first_unit + unit_step, ...  Token r of the buffer sits in slot (res_head + r) mod res_tokens;
// res_head is a multiple of 64, so a unit never wraps.
// A unit is read with 4 coalesced loads per tensor (one instruction = 4 rows of 256 bytes: lane = row l/16, 16-byte
// piece l%16), K and V together and all in flight at once: a single wave has nothing else to hide the memory
// latency with, and small units spread the buffer over many waves.  Scores of row 4i + l/16 are formed by a sum over
// the row's 16 lanes, which is also the layout the V rows arrive in; the channel sums are then folded over the four
// row groups and handed to the lanes that own them (lane l: channels 2l, 2l+1).
// When the append of the newest token is fused into the launch (new_row >= 0), its row comes from k_new / v_new
// instead of the buffer, and the 16 lanes that read it store it into its buffer slot for the launches to come: one
// wave of the grid per (batch, head) owns that row, so there is one writer and no reader of the slot in this launch.
// Out of line: it runs once, after the decode loop, and must not weigh on that loop's registers.
constexpr int kUnitTokens = 16;
template <int G>
__device__ __noinline__ void buffered_tokens(const uint16_t *res, int res_tokens, int B, int H, int b, int h,
                                             int res_head, int n_res, int first_unit, int unit_step,
                                             const float *qf, float scale, int lane, const uint16_t *k_new,
                                             const uint16_t *v_new, int new_row, float *area) {
    Soft<G> st;
    area_to_soft<G>(area, lane, st);
    const size_t res_tensor = (size_t)B * res_tokens * H * kD;
    const size_t row4 = (size_t)4 * H * kD;  // elements from one load to the next
    const int n_units = (n_res + kUnitTokens - 1) / kUnitTokens;
    const int grp = lane >> 4, sub = lane & 15;
    const bool hi2 = (grp & 2) != 0, hi1 = (grp & 1) != 0;
    const int owner = 16 * (lane & 3) + (lane >> 2);  // after the fold: the lane that holds channels 2*lane, 2*lane+1
    for (int u = first_unit; u < n_units; u += unit_step) {
        const int n_tok = min(kUnitTokens, n_res - u * kUnitTokens);
        int slot0 = res_head + u * kUnitTokens;
        if (slot0 >= res_tokens) slot0 -= res_tokens;
        const size_t buf_off = (((size_t)b * res_tokens + slot0 + grp) * H + h) * kD + 8 * sub;
        const size_t new_off = ((size_t)b * H + h) * kD + 8 * sub;
        const int row0 = u * kUnitTokens + grp;  // number of this lane's first row in the buffer, oldest token = 0
        uint4 rk[4], rv[4];
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const uint16_t *src = row0 + 4 * i == new_row ? k_new + new_off : res + buf_off + i * row4;
            rk[i] = 4 * i + grp < n_tok ? *reinterpret_cast<const uint4 *>(src) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const uint16_t *src = row0 + 4 * i == new_row ? v_new + new_off : res + res_tensor + buf_off + i * row4;
            rv[i] = 4 * i + grp < n_tok ? *reinterpret_cast<const uint4 *>(src) : make_uint4(0, 0, 0, 0);
        }
        if (new_row >= 0) {
            uint16_t *wr = const_cast<uint16_t *>(res) + buf_off;
#pragma unroll
            for (int i = 0; i < 4; i++)
                if (row0 + 4 * i == new_row) {
                    *reinterpret_cast<uint4 *>(wr + i * row4) = rk[i];
                    *reinterpret_cast<uint4 *>(wr + res_tensor + i * row4) = rv[i];
                }
        }
#pragma unroll 1
        for (int gg = 0; gg < G; gg++) {
            float qv[8];
#pragma unroll
            for (int k = 0; k < 8; k++) qv[k] = qf[gg * kD + 8 * sub + k];
            float sc[4], mloc = -INFINITY;
#pragma unroll
            for (int i = 0; i < 4; i++) {
                const uint32_t w[4] = {rk[i].x, rk[i].y, rk[i].z, rk[i].w};
                float d = 0.f;
#pragma unroll
                for (int k = 0; k < 4; k++) {
                    d = fmaf(qv[2 * k], h2f(w[k] & 0xffffu), d);
                    d = fmaf(qv[2 * k + 1], h2f(w[k] >> 16), d);
                }
                d += dpp_f<kDppXor1>(d);
                d += dpp_f<kDppXor2>(d);
                d += dpp_f<kDppHalfMirror>(d);
                d += dpp_f<kDppMirror>(d);  // the row's 16 lanes all hold its dot product
                sc[i] = 4 * i + grp < n_tok ? scale * d : -INFINITY;
                mloc = fmaxf(mloc, sc[i]);
            }
            mloc = wave_max(mloc);
            const float mnew = fmaxf(st.m[gg], mloc);
            const float alpha = __expf(st.m[gg] - mnew);
            float psum = 0.f;
#pragma unroll
            for (int i = 0; i < 4; i++) {
                sc[i] = __expf(sc[i] - mnew);
                psum += sc[i];
            }
            st.l[gg] = st.l[gg] * alpha + (sub == 0 ? psum : 0.f);  // each row counted once
            st.bv[gg] *= alpha;
            st.m[gg] = mnew;
            float av[8];
#pragma unroll
            for (int k = 0; k < 8; k++) av[k] = 0.f;
#pragma unroll
            for (int i = 0; i < 4; i++) {
                const uint32_t w[4] = {rv[i].x, rv[i].y, rv[i].z, rv[i].w};
#pragma unroll
                for (int k = 0; k < 4; k++) {
                    av[2 * k] = fmaf(sc[i], h2f(w[k] & 0xffffu), av[2 * k]);
                    av[2 * k + 1] = fmaf(sc[i], h2f(w[k] >> 16), av[2 * k + 1]);
                }
            }
            // fold the four row groups: groups 0,1 keep elements 0..3 and groups 2,3 elements 4..7, then each group r
            // keeps elements 2r, 2r+1 -- the channels 8*sub + 2r, +1 summed over all 16 rows
            float w4[4], w2[2];
#pragma unroll
            for (int k = 0; k < 4; k++) w4[k] = (hi2 ? av[4 + k] : av[k]) + __shfl_xor(hi2 ? av[k] : av[4 + k], 32);
#pragma unroll
            for (int k = 0; k < 2; k++) w2[k] = (hi1 ? w4[2 + k] : w4[k]) + __shfl_xor(hi1 ? w4[k] : w4[2 + k], 16);
            st.acc[gg][0] = st.acc[gg][0] * alpha + __shfl(w2[0], owner);
            st.acc[gg][1] = st.acc[gg][1] * alpha + __shfl(w2[1], owner);
        }
    }
    soft_to_area<G>(st, area, lane);
}

// A record on its way from global memory to the wave's LDS staging area: the first 8 KiB travel through
// registers (loads issued early, stored to LDS later), the rest is copied at commit time.
constexpr int kPrefetchRegs = 8;
// The part of a record beyond what travels through registers (records above 8 KiB: only with code words near the
// 12-bit limit).  Out of line so that its address arithmetic is not hoisted into the kernel's register budget.
__device__ __noinline__ void copy_rest(uint4 *stage, const uint4 *src, uint32_t n16, int lane) {
    for (uint32_t i = lane + 64 * kPrefetchRegs; i < n16; i += 64) stage[i] = src[i];
}

struct Prefetch {
    uint4 r[kPrefetchRegs];
    const uint4 *src;
    uint32_t n16;
    __device__ __forceinline__ void issue(const uint8_t *rec, uint32_t size16, int lane) {
        src = reinterpret_cast<const uint4 *>(rec);
        n16 = size16;
#pragma unroll
        for (int i = 0; i < kPrefetchRegs; i++) {
            const uint32_t at = min((uint32_t)(lane + 64 * i), size16 - 1u);  // clamped: every load is in bounds
            r[i] = src[at];
        }
    }
    __device__ __forceinline__ void commit(uint4 *stage, int lane) const {
#pragma unroll
        for (int i = 0; i < kPrefetchRegs; i++)
            if (lane + 64 * i < n16) stage[lane + 64 * i] = r[i];
        if (n16 > 64u * kPrefetchRegs) copy_rest(stage, src, n16, lane);
    }
};

// The tile path's variant: the record goes from global memory straight into the staging area with LDS-direct loads
// (lane l of load i delivers its 16 bytes to byte 1024 i + 16 l; lanes beyond the record are masked out), issued when
// the previous record has been decoded -- no register holds it on the way.  The rest of a record above 8 KiB is copied
// at wait time.
struct DirectStage {
    const uint4 *src;
    uint32_t n16;
    __device__ __forceinline__ void issue(const uint8_t *rec, uint32_t size16, uint8_t *stage, int lane) {
        src = reinterpret_cast<const uint4 *>(rec);
        n16 = size16;
#pragma unroll
        for (int i = 0; i < kPrefetchRegs; i++)
            if (lane + 64 * i < size16)
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(src + lane + 64 * i),
                                                 (__attribute__((address_space(3))) void *)(stage + 1024 * i), 16, 0, 0);
    }
    __device__ __forceinline__ void wait(uint4 *stage4, int lane) const {
        __builtin_amdgcn_s_waitcnt(0);  // vmcnt(0): the loads have written the LDS
        if (n16 > 64u * kPrefetchRegs) copy_rest(stage4, src, n16, lane);
    }
};

// One workgroup per CU, as many waves as the registers allow per SIMD (fused_waves_per_simd): 4 (128 VGPRs), 3 (168)
// or 2 (256).  The host may launch fewer waves per workgroup (short sequences,
// large staging areas).
template <int G, int LB> struct MaxWaves { static constexpr int value = 4 * fused_waves_per_simd(G, LB); };

// LB = the table width the kernel is compiled for (>= longest code word of both codebooks), see DecodeMode.
template <int G, int LB>
__global__ __launch_bounds__((64 * MaxWaves<G, LB>::value), 1) void fused_attn_kernel(FusedArgs a) {
    using M = DecodeMode<LB>;
    constexpr bool kTile = G >= kTileMinG;  // packed symbols in registers, int8 MFMA
    __shared__ __attribute__((aligned(16))) uint8_t lut_s[2][M::kTableBytes];
    __shared__ __attribute__((aligned(16))) float qf[G * kD];
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];  // per wave: staging area + weights
    const int tid = threadIdx.x, lane = tid & 63, n_threads = blockDim.x;
    // the wave number and everything derived from it (block numbers, table entries, record addresses) are scalars
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n_waves = __builtin_amdgcn_readfirstlane(n_threads >> 6);
    uint8_t *stage = smem + (size_t)wave * a.stage_bytes;
    constexpr int kWeightBytes = (int)fused_weight_bytes(G);
    float *wts = reinterpret_cast<float *>(smem + (size_t)n_waves * a.stage_bytes + (size_t)wave * kWeightBytes);
    const char *lutK = reinterpret_cast<const char *>(&lut_s[0][0]);
    const char *lutV = reinterpret_cast<const char *>(&lut_s[1][0]);

    const Geo &g = a.g;
    // Workgroups go to the eight XCDs round-robin by their linear number, and each XCD has its own L2.  Numbering the
    // (batch-head, split) pairs so that an XCD gets a contiguous range of them keeps the splits of one head -- whose
    // records are neighbours in memory and share cache lines at their ends, and whose partials the last of them
    // merges -- behind one L2.
    int item = blockIdx.x;
    if ((gridDim.x & (kXCDs - 1)) == 0) item = (item & (kXCDs - 1)) * (gridDim.x / kXCDs) + item / kXCDs;
    const int bh = item / a.n_splits, split = item - bh * a.n_splits;
    const int b = bh / g.H, h = bh - b * g.H;

    const int j0 = split * a.blocks_per_split;
    const int j1 = min(j0 + a.blocks_per_split, a.n_blocks);
    const BlockEntry *tabK = g.table + ((size_t)0 * g.B * g.H + bh) * g.max_blocks;
    const BlockEntry *tabV = g.table + ((size_t)1 * g.B * g.H + bh) * g.max_blocks;
    const uint32_t stage16 = (uint32_t)a.stage_bytes / 16 - 1;  // one unit of slack for the streams' look-ahead
    uint4 *stage4 = reinterpret_cast<uint4 *>(stage);
    const uint32_t *stage32 = reinterpret_cast<const uint32_t *>(stage);

    // Prologue.  The first Block Offsets Array entries are requested before the decode tables and the query so that
    // their round trip overlaps; the first K record is requested before the workgroup barrier.
    int j = j0 + wave;
    BlockEntry eK = {0, 0}, eV = {0, 0};
    if (j < j1) {
        eK = tabK[j];
        eV = tabV[j];
    }
    for (int t = 0; t < 2; t++) {
        // pair table: 4096 entries of 4 bytes; otherwise 2^(longest code word of this tensor) entries of 2 bytes
        const uint4 *src = M::kPair ? reinterpret_cast<const uint4 *>(pair_of(g, t))
                                    : reinterpret_cast<const uint4 *>(lut_of(g, t));
        uint4 *dst = reinterpret_cast<uint4 *>(&lut_s[t][0]);
        const int n16 = M::kPair ? M::kTableBytes / 16 : max(1, (2 << g.lut_bits[t]) / 16);
        const uint32_t flip = !kTile ? 0u : M::kPair ? 0x00808000u : 0x80008000u;  // the MFMA operands hold symbol - 128 as int8
        for (int i = tid; i < n16; i += n_threads) {
            uint4 v = src[i];
            v.x ^= flip; v.y ^= flip; v.z ^= flip; v.w ^= flip;
            dst[i] = v;
        }
    }
    const uint32_t maskK = a.mask[0], maskV = a.mask[1];
    for (int i = tid; i < G * kD; i += n_threads) qf[i] = h2f(a.q[((size_t)b * g.Hq + (size_t)h * G) * kD + i]);
    Prefetch pf;
#pragma unroll
    for (int i = 0; i < kPrefetchRegs; i++) pf.r[i] = make_uint4(0, 0, 0, 0);
    pf.src = nullptr;
    pf.n16 = 0;
    DirectStage ds;
    ds.src = nullptr;
    ds.n16 = 0;
    if (j < j1 && eK.size16 <= stage16) {
        if constexpr (kTile) ds.issue(g.payload + (size_t)eK.off16 * 16, eK.size16, stage, lane);
        else pf.issue(g.payload + (size_t)eK.off16 * 16, eK.size16, lane);
    }
    __syncthreads();
    // q in registers: channels lane and lane + 64 (the tile path reads its q from LDS once per block)
    constexpr int kQ0 = kTile ? G / 2 : G;
    float qreg[kTile ? 1 : G][2];
    if constexpr (!kTile) {
#pragma unroll
        for (int gg = 0; gg < G; gg++) { qreg[gg][0] = qf[gg * kD + lane]; qreg[gg][1] = qf[gg * kD + lane + 64]; }
    }

    Soft<G> st;
    st.init();
    TileSoft<kTile ? G : 2> ts;
    ts.init();
    uint8_t *tile = reinterpret_cast<uint8_t *>(wts);

    if (j < j1) {
        if (eK.size16 <= stage16) {
            if constexpr (kTile) ds.wait(stage4, lane);
            else pf.commit(stage4, lane);
        }
        wave_sync();
    }
    __builtin_amdgcn_s_setprio(3);
    while (j < j1) {
        float score[G], p[G];
        const bool k_staged = eK.size16 <= stage16, v_staged = eV.size16 <= stage16;
        const uint8_t *recK = g.payload + (size_t)eK.off16 * 16, *recV = g.payload + (size_t)eV.off16 * 16;
        if (!kTile && v_staged) pf.issue(recV, eV.size16, lane);  // V record travels while K is decoded
        const int jn = j + n_waves;  // the next pair's Block Offsets Array entries travel with it
        BlockEntry eKn = {0, 0}, eVn = {0, 0};
        if (jn < j1) {
            eKn = tabK[jn];
            eVn = tabV[jn];
        }
        float pt[kQ0][2];  // tile path: softmax numerators in the layout of the result tiles
        if constexpr (kTile) {
            // The next record is requested when the current one has been decoded: its registers are then live across
            // the products and the softmax only, not across a decode.
            if (k_staged) {
                k_tile_block<G, LB>(stage32, lutK, maskK, tile, qf, g.two_eb[0], a.scale, lane, g.k_minmax_bytes, ts, pt,
                                    [&] { if (v_staged) ds.issue(recV, eV.size16, stage, lane); });
            } else {
                TileSoft<G> ts_tmp = ts;
                float p_tmp[kQ0][2];
                k_tile_block_global<G, LB>(reinterpret_cast<const uint32_t *>(recK), lutK, maskK, tile, qf, g.two_eb[0],
                                           a.scale, lane, g.k_minmax_bytes, ts_tmp, p_tmp);
                ts = ts_tmp;
#pragma unroll
                for (int i = 0; i < kQ0; i++) { pt[i][0] = p_tmp[i][0]; pt[i][1] = p_tmp[i][1]; }
                if (v_staged) ds.issue(recV, eV.size16, stage, lane);
            }
        } else {
        if (k_staged) {
            k_block<G, LB>(stage32, lutK, maskK, wts, qreg, g.two_eb[0], a.scale, lane, g.k_minmax_bytes, score);
        } else {  // larger than the staging area: decode from global memory (copies keep the hot state in registers)
            float q_tmp[G][2], s_tmp[G];
#pragma unroll
            for (int gg = 0; gg < G; gg++) { q_tmp[gg][0] = qreg[gg][0]; q_tmp[gg][1] = qreg[gg][1]; }
            k_block_global<G, LB>(reinterpret_cast<const uint32_t *>(recK), lutK, maskK, wts, q_tmp, g.two_eb[0], a.scale,
                                  lane, g.k_minmax_bytes, s_tmp);
#pragma unroll
            for (int gg = 0; gg < G; gg++) score[gg] = s_tmp[gg];
        }
        }
        if constexpr (!kTile) {
#pragma unroll
            for (int gg = 0; gg < G; gg++) p[gg] = st.update(gg, score[gg]);
        }
        wave_sync();  // every lane is done with the K record
        if (v_staged) {
            if constexpr (kTile) ds.wait(stage4, lane);
            else pf.commit(stage4, lane);
        }
        wave_sync();
        eKn.off16 = __builtin_amdgcn_readfirstlane(eKn.off16);
        eKn.size16 = __builtin_amdgcn_readfirstlane(eKn.size16);
        eVn.off16 = __builtin_amdgcn_readfirstlane(eVn.off16);
        eVn.size16 = __builtin_amdgcn_readfirstlane(eVn.size16);
        const bool next_staged = jn < j1 && eKn.size16 <= stage16;
        if (!kTile && next_staged) pf.issue(g.payload + (size_t)eKn.off16 * 16, eKn.size16, lane);
        if constexpr (kTile) {
            if (v_staged) {
                v_tile_block<G, LB>(stage32, lutV, maskV, tile, pt, g.two_eb[1], lane, ts,
                                    [&] { if (next_staged) ds.issue(g.payload + (size_t)eKn.off16 * 16, eKn.size16, stage, lane); });
            } else {
                TileSoft<G> ts_tmp = ts;
                float p_tmp[kQ0][2];
#pragma unroll
                for (int i = 0; i < kQ0; i++) { p_tmp[i][0] = pt[i][0]; p_tmp[i][1] = pt[i][1]; }
                v_tile_block_global<G, LB>(reinterpret_cast<const uint32_t *>(recV), lutV, maskV, tile, p_tmp, g.two_eb[1],
                                           lane, ts_tmp);
                ts = ts_tmp;
                if (next_staged) ds.issue(g.payload + (size_t)eKn.off16 * 16, eKn.size16, stage, lane);
            }
        } else {
        if (v_staged) {
            v_block<G, LB>(stage32, lutV, maskV, wts, p, g.two_eb[1], lane, st);
        } else {
            Soft<G> st_tmp = st;
            float p_tmp[G];
#pragma unroll
            for (int gg = 0; gg < G; gg++) p_tmp[gg] = p[gg];
            v_block_global<G, LB>(reinterpret_cast<const uint32_t *>(recV), lutV, maskV, wts, p_tmp, g.two_eb[1], lane,
                                  st_tmp);
            st = st_tmp;
        }
        }
        wave_sync();
        if (jn < j1 && eKn.size16 <= stage16) {
            if constexpr (kTile) ds.wait(stage4, lane);
            else pf.commit(stage4, lane);
        }
        wave_sync();
        eK = eKn;
        eV = eVn;
        j = jn;
        {   // The SIMD issues from its oldest wave first, so its resident waves finish one after the other and the
            // last one runs alone, unable to fill the VALU.  Waves that are behind get the issue slots instead:
            // the priority falls with the share of the work that is done, and the waves finish together.
            const int total = (j1 - j0 - wave + n_waves - 1) / n_waves, left = (j1 - j + n_waves - 1) / n_waves;
            const int q4 = total > 0 ? (4 * left + total - 1) / total : 0;  // 4 .. 0
            if (q4 >= 4) __builtin_amdgcn_s_setprio(3);
            else if (q4 == 3) __builtin_amdgcn_s_setprio(2);
            else if (q4 == 2) __builtin_amdgcn_s_setprio(1);
            else __builtin_amdgcn_s_setprio(0);
        }
    }

    // The record area is free now: the tile path changes the layout of its state through it, and a wave with buffered
    // tokens parks its state there across the out-of-line call.
    float *area = reinterpret_cast<float *>(stage);
    bool parked = false;
    if constexpr (kTile) {
        tile_state_to_area<G>(ts, area, lane);
        parked = true;
    }
    // the buffered fp16 tokens in units of 16: unit u goes to split n_splits-1 - u % n_splits (the last split is the
    // short one), there to the waves in turn, starting after the wave that took the split's last block
    if (a.n_res > 0) {
        int turn = (wave - (j1 - j0)) % n_waves;
        if (turn < 0) turn += n_waves;
        const int first = a.n_splits - 1 - split + a.n_splits * turn;
        if (first * kUnitTokens < a.n_res) {
            if (!parked) soft_to_area<G>(st, area, lane);
            parked = true;
            buffered_tokens<G>(g.res, g.res_tokens, g.B, g.H, b, h, a.res_head, a.n_res, first, n_waves * a.n_splits, qf,
                               a.scale, lane, a.k_new, a.v_new, a.new_row, area);
        }
    }
    if (parked) area_to_soft<G>(area, lane, st);
    wave_sync();

    // merge the waves of this workgroup into one partial (o[128], m, l) per query head
    float *comb = reinterpret_cast<float *>(stage);  // this wave's own staging area: G * 130 floats
#pragma unroll
    for (int gg = 0; gg < G; gg++) {
        const float l = wave_sum(st.l[gg]);
        const float bv = wave_sum(st.bv[gg]);
        comb[gg * kPartialStride + 2 * lane] = st.acc[gg][0] + bv;
        comb[gg * kPartialStride + 2 * lane + 1] = st.acc[gg][1] + bv;
        if (lane == 0) {
            comb[gg * kPartialStride + kD] = st.m[gg];
            comb[gg * kPartialStride + kD + 1] = l;
        }
    }
    __syncthreads();
    const int row0 = b * g.Hq + h * G;
    // the thread number is rebuilt from the lane and the (scalar) wave number: nothing of the prologue has to stay
    // in a register, or be spilled, across the decode loop for the sake of the merge
    const int tid_m = lane + 64 * wave, nt_m = 64 * n_waves;
    for (int i = tid_m; i < G * kD; i += nt_m) {
        const int gg = i / kD, c = i - gg * kD;
        float M_ = -INFINITY;
        for (int w = 0; w < n_waves; w++)
            M_ = fmaxf(M_, reinterpret_cast<const float *>(smem + (size_t)w * a.stage_bytes)[gg * kPartialStride + kD]);
        float L = 0.f, O = 0.f;
        for (int w = 0; w < n_waves; w++) {
            const float *cw = reinterpret_cast<const float *>(smem + (size_t)w * a.stage_bytes) + gg * kPartialStride;
            const float mw = cw[kD];
            const float f = mw == -INFINITY ? 0.f : __expf(mw - M_);
            L += cw[kD + 1] * f;
            O += cw[c] * f;
        }
        if (a.n_splits == 1) {
            a.out[(size_t)(row0 + gg) * kD + c] = O / L;
        } else {
            float *dst = g.partials + ((size_t)(row0 + gg) * kMaxSplits + split) * kPartialStride;
            store_agent(dst + c, O);
            if (c == 0) { store_agent(dst + kD, M_); store_agent(dst + kD + 1, L); }
        }
    }
    if (a.n_splits > 1) finish_splits<G>(g.partials, g.counters + bh, row0, a.n_splits, a.out, tid_m, nt_m);
}

template <int G, int LB>
static hipError_t launch_fused_gn(const FusedArgs &a, int n_waves, size_t lds, hipEvent_t ev0, hipEvent_t ev1,
                                  hipStream_t s) {
    static size_t attr_set = 0;
    if (lds > attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&fused_attn_kernel<G, LB>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set = lds;
    }
    if (n_waves < 1 || n_waves > MaxWaves<G, LB>::value) return hipErrorInvalidValue;
    if (ev0) (void)hipEventRecord(ev0, s);
    hipLaunchKernelGGL((fused_attn_kernel<G, LB>), dim3(a.n_splits * a.g.B * a.g.H), dim3(64 * n_waves), lds, s, a);
    if (ev1) (void)hipEventRecord(ev1, s);
    return hipGetLastError();
}

template <int G>
static hipError_t launch_fused_g(const FusedArgs &a, int longest, int n_waves, size_t lds, hipEvent_t ev0, hipEvent_t ev1,
                                 hipStream_t s) {
    switch (fused_table_bits(longest)) {
        case 6: return launch_fused_gn<G, 6>(a, n_waves, lds, ev0, ev1, s);
        case 7: return launch_fused_gn<G, 7>(a, n_waves, lds, ev0, ev1, s);
        case 8: return launch_fused_gn<G, 8>(a, n_waves, lds, ev0, ev1, s);
        case 10: return launch_fused_gn<G, 10>(a, n_waves, lds, ev0, ev1, s);
        default: return launch_fused_gn<G, 12>(a, n_waves, lds, ev0, ev1, s);
    }
}

hipError_t launch_fused_attn(const Geo &g, const uint16_t *q, float scale, float *out, int n_blocks, int res_head,
                             int n_res, const uint16_t *k_new, const uint16_t *v_new, int n_splits, int n_waves,
                             int stage_bytes, hipEvent_t ev0, hipEvent_t ev1, hipStream_t s) {
    FusedArgs a;
    a.k_new = k_new;
    a.v_new = v_new;
    a.new_row = k_new ? n_res - 1 : -1;  // n_res counts the token being appended
    a.g = g;
    a.q = q;
    a.out = out;
    a.scale = scale;
    a.n_blocks = n_blocks;
    a.res_head = res_head;
    a.n_res = n_res;
    a.blocks_per_split = n_blocks > 0 ? (n_blocks + n_splits - 1) / n_splits : 0;
    a.n_splits = n_blocks > 0 ? (n_blocks + a.blocks_per_split - 1) / a.blocks_per_split : 1;
    a.stage_bytes = stage_bytes;
    const int bits_k = g.lut_bits[0], bits_v = g.lut_bits[1];
    const int longest = bits_k > bits_v ? bits_k : bits_v;
    if (longest < 1 || longest > kLutBits) return hipErrorInvalidValue;
    if (fused_table_bits(longest) == 6) {  // pair tables: 12 index bits, entries of 4 bytes
        a.mask[0] = a.mask[1] = ((1u << kPairIndexBits) - 1u) << 2;
    } else {
        a.mask[0] = ((1u << bits_k) - 1u) << 1;
        a.mask[1] = ((1u << bits_v) - 1u) << 1;
    }
    const size_t lds = (size_t)n_waves * ((size_t)stage_bytes + fused_weight_bytes(g.G));
    switch (g.G) {
        case 1: return launch_fused_g<1>(a, longest, n_waves, lds, ev0, ev1, s);
        case 2: return launch_fused_g<2>(a, longest, n_waves, lds, ev0, ev1, s);
        case 4: return launch_fused_g<4>(a, longest, n_waves, lds, ev0, ev1, s);
        case 8: return launch_fused_g<8>(a, longest, n_waves, lds, ev0, ev1, s);
        default: return hipErrorInvalidValue;
    }
}

// ---- statistics (metrics path, not part of the hot loop) --------------------------------------------------------
// Sums record sizes and code-word bits over all blocks in use by walking the Block Offsets Array and the slice bit
// counts in the record headers.
__global__ __launch_bounds__(256) void stats_kernel(Geo g, int n_blocks) {
    const int BH = g.B * g.H;
    const long long n_items = 2ll * BH * n_blocks;
    unsigned long long bits[2] = {0, 0}, rec16[2] = {0, 0};
    const int lane = threadIdx.x & 63;
    const long long wave_id = ((long long)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const long long n_waves = ((long long)gridDim.x * blockDim.x) >> 6;
    for (long long i = wave_id; i < n_items; i += n_waves) {
        const int which = (int)(i / ((long long)BH * n_blocks));
        const long long rem = i - (long long)which * BH * n_blocks;
        const int bh = (int)(rem / n_blocks), j = (int)(rem - (long long)bh * n_blocks);
        const BlockEntry e = g.table[((size_t)which * BH + bh) * g.max_blocks + j];
        const uint16_t *sb = reinterpret_cast<const uint16_t *>(g.payload + (size_t)e.off16 * 16 +
                                                                (which ? kMinMaxBytesV : g.k_minmax_bytes));
        const uint32_t v = (uint32_t)sb[lane] + sb[lane + 64];
        bits[which] += v;
        if (lane == 0) rec16[which] += e.size16;
    }
    for (int w = 0; w < 2; w++) {
        unsigned long long bsum = bits[w], rsum = rec16[w];
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) {
            bsum += __shfl_xor(bsum, m);
            rsum += __shfl_xor(rsum, m);
        }
        if (lane == 0 && (bsum | rsum)) {
            atomicAdd(&g.ctrl->payload_bits[w], bsum);
            atomicAdd(&g.ctrl->record16[w], rsum);
        }
    }
}

hipError_t launch_stats(const Geo &g, int n_blocks, hipStream_t s) {
    if (n_blocks <= 0) return hipSuccess;
    hipLaunchKernelGGL(stats_kernel, dim3(128), dim3(256), 0, s, g, n_blocks);
    return hipGetLastError();
}

}  // namespace kvc
