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

constexpr int kPairEntries = 1 << 12;  // entries of a pair table (12 index bits)

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
    size_t ctrl, hist, enc, lut, tree, lut2, counters, table, res, partials, payload, total;
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
    L.enc = at; at += 4 * 256 * 4;
    L.lut = at; at += 2 * kLutSize * 2;
    L.tree = at; at += 2 * 256 * 2 * 2;
    L.lut2 = at; at += 2 * kPairEntries * 4;
    L.counters = at; at += align_up(BH * 4, 256);
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
inline void huffman_lengths(const std::vector<uint64_t> &f, std::vector<int> &len) {
    const int n = (int)f.size();
    std::vector<int> order(n);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return f[a] < f[b]; });
    struct Node { uint64_t w; int kid[2]; };
    std::vector<Node> nodes;
    nodes.reserve(2 * n);
    for (int i = 0; i < n; i++) nodes.push_back({f[order[i]], {-1, -1}});
    int leaf = 0, ihead = n;
    auto take = [&]() {
        const bool has_leaf = leaf < n, has_int = ihead < (int)nodes.size();
        if (has_leaf && (!has_int || nodes[leaf].w <= nodes[ihead].w)) return leaf++;
        return ihead++;
    };
    for (int k = 0; k < n - 1; k++) {
        const int a = take(), b = take();
        nodes.push_back({nodes[a].w + nodes[b].w, {a, b}});
    }
    std::vector<int> depth(nodes.size(), 0);
    for (int i = (int)nodes.size() - 1; i >= n; i--) {
        depth[nodes[i].kid[0]] = depth[i] + 1;
        depth[nodes[i].kid[1]] = depth[i] + 1;
    }
    len.assign(n, 0);
    for (int i = 0; i < n; i++) len[order[i]] = depth[i];
}

inline void build_codebook_host(const uint32_t *hist, int n_sym, int max_len, uint8_t *len_out, uint32_t *code_out) {
    std::vector<uint64_t> f(n_sym);
    for (int s = 0; s < n_sym; s++) f[s] = hist[s] ? hist[s] : 1;  // later blocks reuse the codebook: no level unencodable
    std::vector<int> len;
    for (;;) {
        huffman_lengths(f, len);
        if (*std::max_element(len.begin(), len.end()) <= max_len) break;
        for (auto &v : f) v = std::max<uint64_t>(1, (v + 1) >> 1);
    }
    std::memset(len_out, 0, 256);
    std::memset(code_out, 0, 256 * sizeof(uint32_t));
    std::vector<int> by(n_sym);
    std::iota(by.begin(), by.end(), 0);
    std::stable_sort(by.begin(), by.end(), [&](int a, int b) { return len[a] < len[b]; });
    uint32_t code = 0;
    for (int i = 0; i < n_sym; i++) {
        const int s = by[i];
        if (i) code = (code + 1) << (len[s] - len[by[i - 1]]);
        len_out[s] = (uint8_t)len[s];
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
