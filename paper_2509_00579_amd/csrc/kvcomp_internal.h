// Internal declarations shared by the host side of libkvcomp and its HIP kernels (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kvcomp_consts.h"

namespace kvc {

// Device-side control words, first bytes of the arena.
struct Ctrl {
    uint32_t tail16;        // first free 16-byte unit of the payload arena
    uint32_t max_size16;    // largest record so far
    uint32_t nonfinite;     // set when an input value was Inf/NaN
    uint32_t fault;         // kFault* bits set by kernels that refused work; read and cleared at the synchronising calls
    uint32_t tail_base;     // the arena tail that the running placement starts from (tail16 moves at its end)
    // filled by the statistics kernel only (kvcomp_get_stats)
    unsigned long long payload_bits[2];
    unsigned long long record16[2];  // sum of record sizes per tensor, 16-byte units
};

// Ctrl::fault bits
constexpr uint32_t kFaultArenaFull = 1u;    // a placement would have run past the record arena: nothing was written
constexpr uint32_t kFaultStageSmall = 2u;   // the stand-alone decompressor met a record larger than its staging area

// Geometry + device pointers, passed by value to kernels.
struct Geo {
    int B, H, Hq, G;
    int max_blocks;
    int k_units;             // quantization units of a K block: 128 (one per channel) or 1 (BlockQuant, Section 4.2)
    int k_minmax_bytes;      // their {min,max} fp16 pairs in the record header, padded to 16 bytes: 512 or 16
    float two_eb[2];   // bin width factor 2*rel_eb
    int n_sym[2];
    Ctrl *ctrl;
    uint32_t *hist;          // [2][256]
    uint8_t *tables;         // [2 tensors][kTensorTablesBytes], see enc_of / lut_of / tree_of / pair_of below
    int lut_bits[2];         // index width of each decode table = longest code word of that codebook
    uint32_t *counters;      // [B*H] split tickets of the fused kernel, zero between launches
    uint32_t *place_sums;    // record sizes summed per chunk of kPlaceChunk Block Offsets Array entries (placement)
    BlockEntry *table;       // [2][B*H][max_blocks]
    uint16_t *res;           // [2][B][res_tokens][H][128] fp16 buffer of the newest tokens
    int res_tokens;          // its capacity per sequence = maximum buffer size (Section 4.2), a multiple of 64
    float *partials;         // [B*Hq][max_splits][kPartialStride]
    uint8_t *payload;        // record arena
    uint32_t payload_cap16;  // its capacity in 16-byte units
};

// The tables of tensor t (0 = K, 1 = V):
//   enc  [2][256] (len << 16) | code word as it goes into the LSB-first stream: [0] first-bit-first (symbols 0..31 of
//        a slice), [1] last-bit-first (32..63)
//   lut  [4096] (symbol << 8) | len, indexed by the next lut_bits[t] stream bits
//   tree [256][2] array-based Huffman tree (Section 3.3.1): child of node n for stream bit b; >= 0: inner node,
//        < 0: leaf holding symbol ~child; the root is node 0
//   pair [4096] valid when the codebook has code words of at most 6 bits: indexed by the next 12 stream bits;
//        byte 0 = length of two code words together, byte 1 = first symbol, byte 2 = second symbol
__host__ __device__ inline const uint32_t *enc_of(const Geo &g, int t) {
    return reinterpret_cast<const uint32_t *>(g.tables + (size_t)t * kTensorTablesBytes + kTabEncOff);
}
__host__ __device__ inline const uint16_t *lut_of(const Geo &g, int t) {
    return reinterpret_cast<const uint16_t *>(g.tables + (size_t)t * kTensorTablesBytes + kTabLutOff);
}
__host__ __device__ inline const int16_t *tree_of(const Geo &g, int t) {
    return reinterpret_cast<const int16_t *>(g.tables + (size_t)t * kTensorTablesBytes + kTabTreeOff);
}
__host__ __device__ inline const uint32_t *pair_of(const Geo &g, int t) {
    return reinterpret_cast<const uint32_t *>(g.tables + (size_t)t * kTensorTablesBytes + kTabPairOff);
}

constexpr int kCUs = 256;  // compute units of the MI355X
constexpr int kXCDs = 8;   // accelerator dies, each with its own L2; workgroups are dealt to them round-robin
// Groups of 4 and 8 query heads: a wave packs the decoded symbols of a block into registers and multiplies them with the
// weights of all heads on int8 MFMA.  A wave's LDS area next to its staging area holds the A operand while it is laid
// out: three digit rows per head, 128 + 4 bytes each.
constexpr int kARowBytes = kD + 4;
constexpr int tile_bytes(int G) { return 3 * G * kARowBytes; }
// Both groups multiply after every half of a block (16 symbols of every decode chain), so that the products of the
// first half run while the second half is decoded, and recombine the result tiles after each half.  Groups of 8 on the
// kernels with two waves per SIMD (single-symbol tables), where registers are plentiful, keep the integer accumulators
// across both halves and recombine once.  2 = recombine once.
constexpr int tile_halves_at_once(int G, int table_bits) { return G >= 8 && table_bits > 6 ? 2 : 1; }
// Waves of the fused kernel per SIMD, as the registers allow: groups of 4 and 8 query heads trade occupancy for
// registers.  One workgroup per CU holds them all (4 SIMDs: up to 16 waves).
// The pair-table kernels (longest code word <= 6 bits) keep fewer table entries in flight and fit one wave more.
constexpr int fused_waves_per_simd(int G, int table_bits) {
    return table_bits <= 6 ? (G >= 4 ? 3 : 4) : (G >= 8 ? 2 : G >= 4 ? 3 : 4);
}
// Table width a decode kernel is compiled for, given the longest code word in use.  6: code words of up to 6 bits,
// decoded two at a time with the pair table (the fused kernel only; the stand-alone decompressor uses its 7-bit build).
constexpr int fused_table_bits(int longest) {
    return longest <= 6 ? 6 : longest <= 7 ? 7 : longest <= 8 ? 8 : longest <= 10 ? 10 : 12;
}
constexpr int kLdsBytesPerCU = 160 * 1024;
// Bytes of one wave's LDS area next to its staging area.  Groups of 1 and 2 heads: fp32 weights [128][G].  Groups of
// 4 and 8: the area in which the A operand is laid out.
constexpr size_t fused_weight_bytes(int G) { return G >= 4 ? (size_t)tile_bytes(G) : (size_t)G * kD * 4; }
// LDS of one fused-kernel workgroup apart from the per-wave areas: the two decode tables, the query rows, the merge flag.
constexpr size_t fused_lds_fixed(int G, int longest) {
    return (fused_table_bits(longest) == 6 ? (size_t)2 * kPairTableEntries * 4 : (size_t)4 << fused_table_bits(longest)) +
           (size_t)G * kD * 4 + 512;
}

// ---- launches implemented in the .hip files ----
hipError_t launch_decompress(const Geo &g, int which, uint16_t *out, int n_blocks, int res_head, int n_res, int seq_stride,
                             int stage_bytes, int tree_walk, hipStream_t s);
hipError_t launch_histogram(const Geo &g, int which, const uint16_t *X, int seq_stride, int n_blk_per_bh,
                            uint8_t *codes, uint32_t *minmax, uint16_t *block_hist, hipStream_t s);
hipError_t launch_encode_kept(const Geo &g, int which, const uint8_t *codes, const uint32_t *mm, const uint16_t *block_hist,
                              int kept_blk_per_bh, int n_blk_per_bh, hipStream_t s);
hipError_t launch_debug_codes(const Geo &g, int which, const uint16_t *X, int seq_stride, int n_blk_per_bh,
                              uint8_t *d_codes, uint16_t *d_minmax, hipStream_t s);
// size pass -> table[...].size16 ; place -> off16 + ctrl ; write pass -> records
hipError_t launch_encode(const Geo &g, const uint16_t *XK, const uint16_t *XV, int seq_stride, int n_blk_per_bh,
                         int dst_blk0, hipStream_t s);
hipError_t launch_copy_tail(const Geo &g, const uint16_t *XK, const uint16_t *XV, int seq, int first_tok, int n_tok,
                            hipStream_t s);
hipError_t launch_append(const Geo &g, const uint16_t *k_new, const uint16_t *v_new, int slot, hipStream_t s);
// k_new / v_new != NULL: the newest of the n_res buffered tokens is still in k_new / v_new [B][H][128]; the kernel
// reads it from there and stores it into its buffer slot (append fused into the launch)
hipError_t launch_fused_attn(const Geo &g, const uint16_t *q, float scale, float *out, int n_blocks, int res_head,
                             int n_res, const uint16_t *k_new, const uint16_t *v_new, int n_splits, int n_waves,
                             int stage_bytes, hipEvent_t ev0, hipEvent_t ev1, hipStream_t s);
hipError_t launch_baseline_attn(int B, int H, int Hq, const uint16_t *K, const uint16_t *V, int seq, const uint16_t *q,
                                float scale, float *out, float *partials, uint32_t *counters, int n_splits,
                                int split_stride, hipStream_t s);
int baseline_splits(int seq, int n_splits);
// the static device array behind kvcomp_baseline_fp16_attn_noalloc, on the current device
hipError_t baseline_static_scratch(uint32_t **tickets, float **partials, size_t *max_tickets, size_t *partial_bytes);
hipError_t launch_read_stream(const void *src, size_t bytes, uint32_t *sink, size_t *bytes_read, hipStream_t s);
hipError_t launch_stats(const Geo &g, int n_blocks, hipStream_t s);
hipError_t launch_fill_zero(void *p, size_t bytes, hipStream_t s);
// device copy of a multiple of 16 bytes, 16-byte aligned; src may be pinned host memory (its device-side pointer);
// the same launch clears zero_bytes at `zero` (may be 0)
hipError_t launch_copy16(void *dst, const void *src, size_t bytes, void *zero, size_t zero_bytes, hipStream_t s);

}  // namespace kvc
