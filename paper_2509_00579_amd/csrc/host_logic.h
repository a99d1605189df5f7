// Host-only logic of libkvcomp, free of HIP types so that it also compiles with a plain C++ compiler (the CPU
// sanitizer test builds it that way): configuration checks, the arena layout, the canonical length-limited Huffman
// codebook that the paper builds on the CPU from the GPU histogram (Section 3, Section 3.1.2), and the encode /
// decode tables derived from it.
#pragma once

#include <algorithm>
#include <cstring>
#include <numeric>
#include <vector>

#include "../../include/kvcomp.h"
#include "kvcomp_consts.h"

namespace kvc {
namespace host {

constexpr int kPairEntries = kPairTableEntries;  // entries of a pair table (12 index bits)

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

inline int n_sym_for(float rel_eb) {
    if (!(rel_eb > 0.0f) || rel_eb > 0.5f) return -1;
    const float two_eb = 2.0f * rel_eb;
    const int n = (int)__builtin_rintf(1.0f / two_eb) + 1;
    return (n < 2 || n > 256) ? -1 : n;
}

inline bool valid_cfg(const kvcomp_config *c) {
    if (!c) return false;
    if (c->batch < 1 || c->n_kv_heads < 1 || c->n_q_heads < c->n_kv_heads) return false;
    if (c->n_q_heads % c->n_kv_heads) return false;
    const int G = c->n_q_heads / c->n_kv_heads;
    if (G != 1 && G != 2 && G != 4 && G != 8) return false;
    if (c->head_dim != kD || c->block_tokens != kBT) return false;
    if (c->max_seq < 1) return false;
    if (n_sym_for(c->rel_eb_k) < 0 || n_sym_for(c->rel_eb_v) < 0) return false;
    if (c->k_mode != 0 && c->k_mode != 1) return false;
    if (c->max_code_len != 0) {  // every level needs a code word: 2^max_code_len >= number of levels
        const int levels = std::max(n_sym_for(c->rel_eb_k), n_sym_for(c->rel_eb_v));
        if (c->max_code_len > kLutBits || (1 << c->max_code_len) < levels) return false;
    }
    if ((long long)c->batch * c->n_kv_heads * ((long long)c->max_seq / kBT + 1) > (1ll << 28)) return false;
    if (c->buffer_tokens != 0 && (c->buffer_tokens < kBT || c->buffer_tokens % kBT || c->buffer_tokens > kMaxBufferTokens))
        return false;
    return true;
}

// capacity of the fp16 buffer of new tokens (Section 3.2.1; the maximum buffer size of Section 4.2)
inline int buffer_tokens(const kvcomp_config &c) { return c.buffer_tokens ? c.buffer_tokens : kBT; }

// header of a K record: {min,max} pairs (one per channel, or one for the block padded to 16 bytes) + slice bit counts
inline int k_minmax_bytes(const kvcomp_config &c) { return c.k_mode == 1 ? 16 : kMinMaxBytesK; }
inline int k_header_bytes(const kvcomp_config &c) { return k_minmax_bytes(c) + 2 * kSlices; }

inline int code_len_limit(const kvcomp_config &c) { return c.max_code_len ? c.max_code_len : kLutBits; }

struct Layout {
    size_t ctrl, hist, tables, counters, place_sums, table, res, partials, payload, total;
    size_t payload_cap16;
    int max_blocks;
};

inline Layout make_layout(const kvcomp_config &c) {
    Layout L;
    const size_t BH = (size_t)c.batch * c.n_kv_heads;
    L.max_blocks = c.max_seq / kBT;
    const int lim = code_len_limit(c);
    const size_t worst_k = align_up((size_t)k_header_bytes(c) + (size_t)kTile * lim / 8, 16);
    const size_t worst_v = align_up(kHdrBytesV + (size_t)kTile * lim / 8, 16);
    size_t at = 0;
    L.ctrl = at; at += 256;
    L.hist = at; at += 2 * 256 * 4;
    L.tables = at; at += 2 * (size_t)kTensorTablesBytes;
    L.counters = at; at += align_up(BH * 4, 256);
    L.place_sums = at; at += align_up((2 * BH * (size_t)std::max(L.max_blocks, 1) / kPlaceChunk + 1) * 4, 256);
    L.table = at; at += align_up(2 * BH * (size_t)std::max(L.max_blocks, 1) * sizeof(BlockEntry), 256);
    L.res = at; at += align_up(2 * (size_t)c.batch * buffer_tokens(c) * c.n_kv_heads * kD * 2, 256);
    L.partials = at; at += align_up((size_t)c.batch * c.n_q_heads * kMaxSplits * kPartialStride * 4, 256);
    L.payload = at;
    const size_t pay = BH * (size_t)L.max_blocks * (worst_k + worst_v) + 256;
    L.payload_cap16 = pay / 16;
    at += align_up(pay, 256);
    L.total = at;
    return L;
}

// ---- Huffman codebook (Section 3.1.2), canonical and length-limited --------------------------------------------
// Two-queue construction over leaves sorted by (count, symbol); on equal weight a leaf is taken before a merged
// node and merged nodes leave in creation order, which fixes the code lengths uniquely.
// This runs between two device passes of a prompt compression, with the GPU idle: fixed arrays, no allocation.
// key: the n <= 256 leaves as (weight << 8) | symbol, weights below 2^40, sorted ascending (which is the stable sort
// by weight); len: code length per symbol.
inline void huffman_lengths(const uint64_t *key, int n, int *len) {
    uint64_t w[512];
    int kid[512][2], depth[512];
    for (int i = 0; i < n; i++) w[i] = key[i] >> 8;
    int leaf = 0, ihead = n, n_nodes = n;
    auto take = [&]() {
        const bool has_leaf = leaf < n, has_int = ihead < n_nodes;
        if (has_leaf && (!has_int || w[leaf] <= w[ihead])) return leaf++;
        return ihead++;
    };
    for (int k = 0; k < n - 1; k++) {
        const int a = take(), b = take();
        w[n_nodes] = w[a] + w[b];
        kid[n_nodes][0] = a;
        kid[n_nodes][1] = b;
        n_nodes++;
    }
    for (int i = 0; i < n_nodes; i++) depth[i] = 0;
    for (int i = n_nodes - 1; i >= n; i--) {
        depth[kid[i][0]] = depth[i] + 1;
        depth[kid[i][1]] = depth[i] + 1;
    }
    for (int i = 0; i < n; i++) len[(int)(key[i] & 0xffu)] = depth[i];
}

inline void build_codebook_host(const uint32_t *hist, int n_sym, int max_len, uint8_t *len_out, uint32_t *code_out) {
    uint64_t key[256];
    int len[256];
    // later blocks reuse the codebook: no level may be unencodable
    for (int s = 0; s < n_sym; s++) key[s] = ((uint64_t)(hist[s] ? hist[s] : 1) << 8) | (uint64_t)s;
    std::sort(key, key + n_sym);
    for (;;) {
        huffman_lengths(key, n_sym, len);
        if (*std::max_element(len, len + n_sym) <= max_len) break;
        // too deep: halve every weight (rounding up, at least 1) and try again.  Halving keeps the order of the
        // weights; only leaves that became equal may have to swap into symbol order: an insertion sort over an
        // almost sorted array
        for (int i = 0; i < n_sym; i++) {
            const uint64_t wgt = std::max<uint64_t>(1, ((key[i] >> 8) + 1) >> 1);
            uint64_t k = (wgt << 8) | (key[i] & 0xffu);
            int j = i;
            for (; j > 0 && key[j - 1] > k; j--) key[j] = key[j - 1];
            key[j] = k;
        }
    }
    std::memset(len_out, 0, 256);
    std::memset(code_out, 0, 256 * sizeof(uint32_t));
    // canonical code words: symbols by (length, symbol)
    uint32_t by[256];
    for (int s = 0; s < n_sym; s++) by[s] = ((uint32_t)len[s] << 8) | (uint32_t)s;
    std::sort(by, by + n_sym);
    uint32_t code = 0;
    for (int i = 0; i < n_sym; i++) {
        const int s = (int)(by[i] & 0xffu), L = (int)(by[i] >> 8);
        if (i) code = (code + 1) << (L - (int)(by[i - 1] >> 8));
        len_out[s] = (uint8_t)L;
        code_out[s] = code;
    }
}

inline uint32_t reverse_bits(uint32_t v, int n) {
    uint32_t r = 0;
    for (int i = 0; i < n; i++) r |= ((v >> i) & 1u) << (n - 1 - i);
    return r;
}


// Tables of one codebook.  enc: [2][256] (length << 16) | code word as it enters the stream, [0]: first bit first (the
// code word bit-reversed, since the stream fills words from bit 0), [1]: last bit first.  lut: 2^bits entries
// (symbol << 8) | length indexed by the next `bits` stream bits, bits = longest code word (returned).  tree: the same
// codebook as an array-based tree (Section 3.3.1): tree[2 n + b] = child of node n for stream bit b, >= 0 inner node,
// < 0 leaf holding symbol ~child; root = node 0.
inline int build_tables(const uint8_t *len, const uint32_t *code, uint32_t *enc, uint16_t *lut, int16_t *tree) {
    std::memset(enc, 0, 512 * 4);
    std::memset(lut, 0, kLutSize * 2);
    const int bits = *std::max_element(len, len + 256);
    for (int sy = 0; sy < 256; sy++) {
        const int L = len[sy];
        if (!L) continue;
        const uint32_t rev = reverse_bits(code[sy], L);  // first stream bit = bit 0 of the index
        enc[sy] = ((uint32_t)L << 16) | rev;
        enc[256 + sy] = ((uint32_t)L << 16) | code[sy];
        for (uint32_t k = 0; k < (1u << (bits - L)); k++) lut[rev | (k << L)] = (uint16_t)((sy << 8) | L);
    }
    std::memset(tree, 0, 512 * 2);
    int n_nodes = 1;
    for (int sy = 0; sy < 256; sy++) {
        const int L = len[sy];
        if (!L) continue;
        int node = 0;
        for (int i = 0; i < L; i++) {
            const int bit = (code[sy] >> (L - 1 - i)) & 1;  // code words enter the stream first bit first
            int16_t &child = tree[node * 2 + bit];
            if (i == L - 1) {
                child = (int16_t)~sy;
            } else {
                if (child == 0) child = (int16_t)n_nodes++;
                node = child;
            }
        }
    }
    return bits;
}

// Pair table of a codebook whose code words have at most 6 bits (`bits` = its longest, lut = its decode table from
// build_tables): entry i, for the next 12 stream bits i, = (length of the first two code words together) | first
// symbol << 8 | second symbol << 16.  The code is complete (Kraft sum 1), so every bit pattern starts with a code word.
inline void build_pair_table(const uint16_t *lut, int bits, uint32_t *lut2) {
    const uint32_t m = (1u << bits) - 1u;
    for (uint32_t i = 0; i < (uint32_t)kPairEntries; i++) {
        const uint32_t e1 = lut[i & m], l1 = e1 & 0xffu;
        const uint32_t e2 = lut[(i >> l1) & m], l2 = e2 & 0xffu;
        lut2[i] = (l1 + l2) | ((e1 >> 8) << 8) | ((e2 >> 8) << 16);
    }
}

}  // namespace host
}  // namespace kvc
