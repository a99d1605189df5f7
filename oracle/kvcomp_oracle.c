/*
 * kvcomp_oracle.c -- CPU ORACLE for the KVComp hot path.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, step-by-step implementation of what the compressed KV-cache path computes, written from the
 * paper's description: block-wise quantization with a fixed relative error bound (Section 3.1.1, Section 4.2
 * "relative quantization scale"), a histogram of the codes and one shared Huffman codebook per tensor
 * (Section 3, Store stage; Section 3.2), per-slice Huffman encoding aggregated into one contiguous chunk per
 * 2D block (Section 3.2.2, Figure 4), bit-serial decoding -- both a canonical-code decoder and the branch-free
 * array-tree walk of Section 3.3.1 -- and decode attention on the dequantized cache (Figure 1, Section 3.3.2).
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may use this file.  It shares no code,
 * header, table or constant generator with the HIP library; the product path never calls it.
 *
 * Precision: the bit-exact parts (min/max, codes) use IEEE binary32 operations one at a time (build with
 * -ffp-contract=off, no fast-math); dequantization and attention use binary64.
 *
 * Conventions fixed where the paper is silent (all listed in the design notes of the repository):
 *   - a 2D block is 64 tokens x 128 channels of one (batch, head); tile arrays are [64][128], token-major;
 *   - quantization units: K (mode 0) = one channel of the block (64 values); K (mode 1, "BlockQuant") = the
 *     whole block; V = one token of the block (128 values);
 *   - bin width = 2 * rel_eb * (max - min), codes = round-half-even((x - min) / width), reconstruction
 *     min + code * width, so |x - x'| <= rel_eb * (max - min);
 *   - slices (the vector one GPU thread encodes, Section 3.2.2): 128 slices of 64 symbols in every block.
 *     K slice s = token s/2, channels 64*(s%2) .. +63 in channel order (half a token row: the dot product of
 *     Section 3.3.2 runs along head_dim); V slice s = channel s, tokens 0..63 in token order (the dot product runs
 *     along the context);
 *   - bit stream: bit i of a payload is bit (i mod 32) of little-endian 32-bit word (i div 32);
 *   - a slice is written from both ends: the code words of its symbols 0..31 follow each other first-bit-first
 *     (most significant bit of the canonical code first) from the slice start upwards, and the code words of
 *     symbols 32..63 come after them, each written last-bit-first.  Read DOWNWARDS from the slice end, the bits are
 *     therefore the code words of symbols 63, 62, .., 32, first-bit-first: a slice holds two independently decodable
 *     chains and needs no second offset, because its end is the next slice's start.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define D 128            /* head_dim */
#define BT 64            /* tokens per block */
#define NSYM_MAX 256

/* ---------------------------------------------------------------- fp16 -> real ---------------------------- */

/* Exact value of an IEEE binary16 bit pattern.  Returns 0 in *finite for Inf/NaN. */
static double half_value(uint16_t h, int *finite) {
    int sign = (h >> 15) & 1, e = (h >> 10) & 0x1f, m = h & 0x3ff;
    double v;
    *finite = 1;
    if (e == 31) { *finite = 0; return 0.0; }
    if (e == 0) v = ldexp((double)m, -24);
    else v = ldexp((double)(m + 1024), e - 25);
    return sign ? -v : v;
}

static float half_to_float(uint16_t h) { int f; return (float)half_value(h, &f); }

/* ---------------------------------------------------------------- geometry -------------------------------- */

/* which: 0 = K, 1 = V.  k_mode: 0 = channel-wise inside the block, 1 = one unit per block (K only). */
int orc_n_units(int which, int k_mode) {
    if (which == 1) return BT;
    return k_mode == 1 ? 1 : D;
}
static int unit_of(int which, int k_mode, int t, int c) {
    if (which == 1) return t;
    return k_mode == 1 ? 0 : c;
}
#define NSLICE 128       /* slices per block */
#define SLICE 64         /* symbols per slice */
#define HALF 32          /* symbols 0..31 are read upwards from the slice start, 63..32 downwards from its end */
int orc_n_slices(int which) { (void)which; return NSLICE; }
static int slice_len(int which) { (void)which; return SLICE; }
/* symbol k of slice s sits at tile position (t, c) */
static void slice_pos(int which, int s, int k, int *t, int *c) {
    if (which == 0) { *t = s / 2; *c = SLICE * (s % 2) + k; } else { *t = k; *c = s; }
}
/* record header: [min/max pairs, padded to 16 bytes][u16 bit count per slice] */
int orc_minmax_bytes(int which, int k_mode) {
    int b = 4 * orc_n_units(which, k_mode);
    return (b + 15) / 16 * 16;
}
int orc_header_bytes(int which, int k_mode) { return orc_minmax_bytes(which, k_mode) + 2 * orc_n_slices(which); }

/* ---------------------------------------------------------------- quantization ---------------------------- */

/* number of code levels for a relative error bound: bins of width 2*rel_eb*range cover [min, max]  */
int orc_n_sym(float rel_eb) {
    float two_eb, inv;
    int n;
    if (!(rel_eb > 0.0f) || rel_eb > 0.5f) return -1;
    two_eb = 2.0f * rel_eb;
    inv = 1.0f / two_eb;
    n = (int)rintf(inv) + 1;
    if (n < 2 || n > NSYM_MAX) return -1;
    return n;
}

/*
 * Quantize one 2D block (Section 3.1.1; scale definition of Section 4.2 read as bin width = 2 * error bound).
 * tile:   [64][128] binary16 bit patterns.  codes: [64][128].  minmax: [n_units][2] binary16 bit patterns.
 * Returns 0, or -5 if an input is not finite, -1 on a bad argument.
 */
int orc_quantize_block(int which, int k_mode, const uint16_t *tile, float rel_eb, uint8_t *codes, uint16_t *minmax) {
    int n_sym = orc_n_sym(rel_eb), nu = orc_n_units(which, k_mode);
    float two_eb = 2.0f * rel_eb;
    int u, t, c;
    if (n_sym < 0) return -1;
    for (u = 0; u < nu; u++) {
        /* unit minimum and maximum over the binary16 values (exact comparisons) */
        int first = 1;
        uint16_t mn = 0, mx = 0;
        double vmn = 0, vmx = 0;
        float fmn, fmx, range, step;
        for (t = 0; t < BT; t++)
            for (c = 0; c < D; c++) {
                int fin;
                double v;
                if (unit_of(which, k_mode, t, c) != u) continue;
                v = half_value(tile[t * D + c], &fin);
                if (!fin) return -5;
                if (first || v < vmn) { vmn = v; mn = tile[t * D + c]; }
                if (first || v > vmx) { vmx = v; mx = tile[t * D + c]; }
                first = 0;
            }
        if (vmn == 0.0) mn = 0; /* -0 and +0 compare equal: store +0 */
        if (vmx == 0.0) mx = 0;
        minmax[2 * u] = mn;
        minmax[2 * u + 1] = mx;
        fmn = half_to_float(mn);
        fmx = half_to_float(mx);
        range = fmx - fmn;        /* one binary32 subtraction */
        step = two_eb * range;    /* one binary32 multiplication: the bin width */
        for (t = 0; t < BT; t++)
            for (c = 0; c < D; c++) {
                float x, d, r, k;
                if (unit_of(which, k_mode, t, c) != u) continue;
                if (range == 0.0f) { codes[t * D + c] = 0; continue; }
                x = half_to_float(tile[t * D + c]);
                d = x - fmn;      /* binary32 subtraction */
                r = d / step;     /* correctly rounded binary32 division */
                k = rintf(r);     /* round half to even */
                if (k < 0.0f) k = 0.0f;
                if (k > (float)(n_sym - 1)) k = (float)(n_sym - 1);
                codes[t * D + c] = (uint8_t)k;
            }
    }
    return 0;
}

/* The bin width the decoder recomputes from the stored min/max (same binary32 operations as above). */
static float unit_step(uint16_t mn, uint16_t mx, float rel_eb) {
    float two_eb = 2.0f * rel_eb;
    float range = half_to_float(mx) - half_to_float(mn);
    return two_eb * range;
}

/* x' = min + code * width, evaluated in binary64.  out: [64][128]. */
void orc_dequantize_block(int which, int k_mode, const uint8_t *codes, const uint16_t *minmax, float rel_eb, double *out) {
    int t, c;
    for (t = 0; t < BT; t++)
        for (c = 0; c < D; c++) {
            int u = unit_of(which, k_mode, t, c);
            double mn = (double)half_to_float(minmax[2 * u]);
            double st = (double)unit_step(minmax[2 * u], minmax[2 * u + 1], rel_eb);
            out[t * D + c] = mn + (double)codes[t * D + c] * st;
        }
}

/* binary32 -> binary16, round to nearest even (overflow to infinity, gradual underflow). */
static uint16_t float_to_half(float f) {
    uint32_t x, sign, mant;
    int32_t e;
    memcpy(&x, &f, 4);
    sign = (x >> 16) & 0x8000u;
    e = (int32_t)((x >> 23) & 0xffu);
    mant = x & 0x7fffffu;
    if (e == 0xff) return (uint16_t)(sign | 0x7c00u | (mant ? 0x200u : 0u));
    e -= 127;
    if (e > 15) return (uint16_t)(sign | 0x7c00u);
    if (e >= -14) {                       /* normal half: keep 10 mantissa bits, round on the 13 dropped ones */
        uint32_t h = ((uint32_t)(e + 15) << 10) | (mant >> 13);
        uint32_t rest = mant & 0x1fffu;
        if (rest > 0x1000u || (rest == 0x1000u && (h & 1u))) h++;   /* a carry runs into the exponent: correct */
        return (uint16_t)(sign | h);
    }
    if (e < -25) return (uint16_t)sign;    /* below half of the smallest subnormal */
    {                                      /* subnormal half: value = m * 2^-24 */
        uint32_t full = mant | 0x800000u;  /* 1.m as a 24-bit integer, value = full * 2^(e-23) */
        int shift = -e - 1;                /* m = full >> shift, shift in 14..24 */
        uint32_t h = full >> shift;
        uint32_t rest = full & ((1u << shift) - 1u), halfway = 1u << (shift - 1);
        if (rest > halfway || (rest == halfway && (h & 1u))) h++;
        return (uint16_t)(sign | h);
    }
}
uint16_t orc_float_to_half(float f) { return float_to_half(f); }

/* Reconstruction as binary16, for the stand-alone decompression of the multi-kernel pipeline (Section 4.3 writes
 * the decompressed cache back to memory in the cache's own precision): binary32 product code * width, binary32 sum
 * with the minimum, one rounding to binary16.  out: [64][128] bit patterns. */
void orc_reconstruct_block_fp16(int which, int k_mode, const uint8_t *codes, const uint16_t *minmax, float rel_eb,
                                uint16_t *out) {
    int t, c;
    for (t = 0; t < BT; t++)
        for (c = 0; c < D; c++) {
            int u = unit_of(which, k_mode, t, c);
            float mn = half_to_float(minmax[2 * u]);
            float st = unit_step(minmax[2 * u], minmax[2 * u + 1], rel_eb);
            float prod = (float)codes[t * D + c] * st;
            float v = mn + prod;
            out[t * D + c] = float_to_half(v);
        }
}

/* ---------------------------------------------------------------- histogram ------------------------------- */

void orc_histogram(const uint8_t *codes, size_t n, uint64_t *hist) {
    size_t i;
    for (i = 0; i < n; i++) hist[codes[i]]++;
}

/* ---------------------------------------------------------------- Huffman codebook ------------------------ */

/*
 * Code lengths of a Huffman tree over weights f[0..n-1] (all >= 1, n >= 2): repeatedly merge the two lightest
 * live nodes.  Ties are resolved by a total order so that any implementation of the same rule agrees:
 * lighter first; at equal weight a leaf before a merged node; among leaves the smaller symbol; among merged
 * nodes the one created earlier.
 */
static void huffman_lengths(const uint64_t *f, int n, int *len) {
    uint64_t w[2 * NSYM_MAX];
    int kind[2 * NSYM_MAX], ord[2 * NSYM_MAX], parent[2 * NSYM_MAX], live[2 * NSYM_MAX];
    int total = n, merges, i;
    for (i = 0; i < n; i++) { w[i] = f[i]; kind[i] = 0; ord[i] = i; parent[i] = -1; live[i] = 1; }
    for (merges = 0; merges < n - 1; merges++) {
        int pick[2], p;
        for (p = 0; p < 2; p++) {
            int best = -1;
            for (i = 0; i < total; i++) {
                if (!live[i]) continue;
                if (best < 0 || w[i] < w[best] || (w[i] == w[best] && (kind[i] < kind[best] ||
                    (kind[i] == kind[best] && ord[i] < ord[best]))))
                    best = i;
            }
            pick[p] = best;
            live[best] = 0;
        }
        w[total] = w[pick[0]] + w[pick[1]];
        kind[total] = 1;
        ord[total] = merges;
        parent[total] = -1;
        live[total] = 1;
        parent[pick[0]] = total;
        parent[pick[1]] = total;
        total++;
    }
    for (i = 0; i < n; i++) {
        int d = 0, p = i;
        while (parent[p] >= 0) { p = parent[p]; d++; }
        len[i] = d;
    }
}

/*
 * Shared codebook for one tensor (Section 3, Store stage: histogram on the GPU, codebook once at prefill,
 * reused afterwards).  Every representable level s < n_sym gets a code (count floored to 1) because blocks
 * compressed later reuse the codebook.  If the longest code exceeds max_len the counts are halved (rounding
 * up, floor 1) and the tree rebuilt.  Codes are canonical: ordered by (length, symbol), the first is 0, each
 * next one is (previous + 1) shifted left by the growth in length.
 * Returns the number of halvings performed (>= 0), or -1 on a bad argument.
 */
int orc_build_codebook(const uint64_t *hist, int n_sym, int max_len, uint8_t *len_out, uint32_t *code_out) {
    uint64_t f[NSYM_MAX];
    int len[NSYM_MAX], s, halvings = 0, L;
    uint32_t next = 0;
    int prev_len = 0, started = 0;
    if (n_sym < 2 || n_sym > NSYM_MAX || max_len < 1 || max_len > 16 || (1 << max_len) < n_sym) return -1;
    for (s = 0; s < n_sym; s++) f[s] = hist[s] > 0 ? hist[s] : 1;
    for (;;) {
        int longest = 0;
        huffman_lengths(f, n_sym, len);
        for (s = 0; s < n_sym; s++) if (len[s] > longest) longest = len[s];
        if (longest <= max_len) break;
        for (s = 0; s < n_sym; s++) { f[s] = (f[s] + 1) >> 1; if (f[s] < 1) f[s] = 1; }
        halvings++;
    }
    for (s = 0; s < NSYM_MAX; s++) { len_out[s] = 0; code_out[s] = 0; }
    for (L = 1; L <= max_len; L++)
        for (s = 0; s < n_sym; s++) {
            if (len[s] != L) continue;
            if (started) next = (next + 1) << (L - prev_len);
            started = 1;
            prev_len = L;
            len_out[s] = (uint8_t)L;
            code_out[s] = next;
        }
    return halvings;
}

/* ---------------------------------------------------------------- encoding -------------------------------- */

static void put_bit(uint8_t *payload, size_t i, int bit) {
    /* bit i lives in 32-bit little-endian word i/32 at bit position i%32, i.e. byte (i/8), bit (i%8) */
    if (bit) payload[i >> 3] |= (uint8_t)(1u << (i & 7));
}
static int get_bit(const uint8_t *payload, size_t i) { return (payload[i >> 3] >> (i & 7)) & 1; }

/*
 * Encode one quantized 2D block into its record (Section 3.2.2 stages 2-4, Figure 4):
 *   [min/max pairs (padded to 16 B)] [u16 bit count of each slice] [all slices' code words, concatenated at bit
 *   granularity in slice order, in whole 32-bit words] [zero padding to a multiple of 16 bytes].
 * Inside a slice the first 32 code words go out first-bit-first and the last 32 last-bit-first (see the header).
 * Returns the record size in bytes, or 0 if cap is too small / a code has no code word.
 */
size_t orc_encode_block(int which, int k_mode, const uint8_t *codes, const uint16_t *minmax, const uint8_t *len,
                        const uint32_t *code, uint8_t *rec, size_t cap) {
    int ns = orc_n_slices(which), sl = slice_len(which), mmb = orc_minmax_bytes(which, k_mode);
    int hdr = orc_header_bytes(which, k_mode), nu = orc_n_units(which, k_mode);
    size_t total_bits = 0, pos = 0, bytes;
    int s, k, b;
    for (s = 0; s < ns; s++)
        for (k = 0; k < sl; k++) {
            int t, c;
            slice_pos(which, s, k, &t, &c);
            if (len[codes[t * D + c]] == 0) return 0;
            total_bits += len[codes[t * D + c]];
        }
    bytes = (size_t)hdr + (total_bits + 31) / 32 * 4;
    bytes = (bytes + 15) / 16 * 16;
    if (bytes > cap) return 0;
    memset(rec, 0, bytes);
    for (s = 0; s < nu; s++) {
        rec[4 * s + 0] = (uint8_t)(minmax[2 * s] & 0xff);
        rec[4 * s + 1] = (uint8_t)(minmax[2 * s] >> 8);
        rec[4 * s + 2] = (uint8_t)(minmax[2 * s + 1] & 0xff);
        rec[4 * s + 3] = (uint8_t)(minmax[2 * s + 1] >> 8);
    }
    for (s = 0; s < ns; s++) {
        size_t start = pos;
        for (k = 0; k < sl; k++) {
            int t, c, sym, L;
            slice_pos(which, s, k, &t, &c);
            sym = codes[t * D + c];
            L = len[sym];
            if (k < HALF)
                for (b = L - 1; b >= 0; b--) put_bit(rec + hdr, pos++, (code[sym] >> b) & 1);
            else
                for (b = 0; b < L; b++) put_bit(rec + hdr, pos++, (code[sym] >> b) & 1);
        }
        rec[mmb + 2 * s + 0] = (uint8_t)((pos - start) & 0xff);
        rec[mmb + 2 * s + 1] = (uint8_t)((pos - start) >> 8);
    }
    return bytes;
}

static void read_minmax(int which, int k_mode, const uint8_t *rec, uint16_t *minmax) {
    int u, nu = orc_n_units(which, k_mode);
    for (u = 0; u < nu; u++) {
        minmax[2 * u] = (uint16_t)(rec[4 * u] | (rec[4 * u + 1] << 8));
        minmax[2 * u + 1] = (uint16_t)(rec[4 * u + 2] | (rec[4 * u + 3] << 8));
    }
}

/* ---------------------------------------------------------------- decoder A: canonical, bit-serial -------- */

/*
 * Canonical-code decoder: read one bit at a time, extend the candidate code word, and stop as soon as the
 * candidate falls inside the range of code words of its length.  Uses only the code lengths.
 * Returns 0 on success, -1 on a malformed stream.
 */
int orc_decode_block_serial(int which, int k_mode, const uint8_t *rec, const uint8_t *len, uint8_t *codes, uint16_t *minmax) {
    int ns = orc_n_slices(which), sl = slice_len(which), mmb = orc_minmax_bytes(which, k_mode);
    int hdr = orc_header_bytes(which, k_mode);
    int count[33] = {0}, first_index[33], sorted[NSYM_MAX];
    uint32_t first_code[33];
    int L, s, k, n = 0;
    uint32_t next = 0;
    size_t pos = 0;
    for (s = 0; s < NSYM_MAX; s++) if (len[s]) count[len[s]]++;
    for (L = 1; L <= 32; L++) {
        next <<= 1;
        first_code[L] = next;
        first_index[L] = n;
        for (s = 0; s < NSYM_MAX; s++) if (len[s] == L) sorted[n++] = s;
        next += (uint32_t)count[L];
    }
    read_minmax(which, k_mode, rec, minmax);
    for (s = 0; s < ns; s++) {
        size_t start = pos;
        size_t want = (size_t)(rec[mmb + 2 * s] | (rec[mmb + 2 * s + 1] << 8));
        size_t up = start, down = start + want; /* next bit going up; one past the next bit going down */
        for (k = 0; k < sl; k++) {
            /* symbols 0..31 in order from the start; then 63, 62, .., 32 from the end */
            int sym_index = k < HALF ? k : sl - 1 - (k - HALF);
            uint32_t cand = 0;
            int t, c, found = 0;
            for (L = 1; L <= 32 && !found; L++) {
                int bit;
                if (k < HALF) bit = get_bit(rec + hdr, up++);
                else { if (down == 0) return -1; bit = get_bit(rec + hdr, --down); }
                cand = (cand << 1) | (uint32_t)bit;
                if (count[L] && cand >= first_code[L] && cand - first_code[L] < (uint32_t)count[L]) {
                    slice_pos(which, s, sym_index, &t, &c);
                    codes[t * D + c] = (uint8_t)sorted[first_index[L] + (int)(cand - first_code[L])];
                    found = 1;
                }
            }
            if (!found) return -1;
        }
        if (up != down) return -1; /* the two chains must meet exactly */
        pos = start + want;
    }
    return 0;
}

/* ---------------------------------------------------------------- decoder B: array tree walk -------------- */

/*
 * The decoder of Section 3.3.1: the Huffman tree is an array of nodes {is_symbol, symbol, indexes[2]}; each
 * stream bit selects the next node through indexes[bit]; the current node's symbol is always stored but the
 * write position only advances on symbol nodes; the position in the tree is reset to the root with a mask
 * computed from is_symbol instead of a branch.  Each slice is walked twice: upwards from its start for symbols
 * 0..31 and downwards from its end for symbols 63..32; the walk stops when 32 symbols have been written.
 */
typedef struct { int is_symbol; int symbol; int indexes[2]; } tree_node;

int orc_decode_block_tree(int which, int k_mode, const uint8_t *rec, const uint8_t *len, const uint32_t *code,
                          uint8_t *codes, uint16_t *minmax) {
    int ns = orc_n_slices(which), sl = slice_len(which), mmb = orc_minmax_bytes(which, k_mode);
    int hdr = orc_header_bytes(which, k_mode);
    tree_node nodes[2 * NSYM_MAX];
    int n_nodes = 1, s, b;
    size_t pos = 0;
    nodes[0].is_symbol = 0; nodes[0].symbol = 0; nodes[0].indexes[0] = nodes[0].indexes[1] = 0;
    for (s = 0; s < NSYM_MAX; s++) {
        int at = 0;
        if (!len[s]) continue;
        for (b = len[s] - 1; b >= 0; b--) {
            int bit = (code[s] >> b) & 1;
            if (nodes[at].indexes[bit] == 0) {
                if (n_nodes >= 2 * NSYM_MAX) return -1;
                nodes[n_nodes].is_symbol = 0; nodes[n_nodes].symbol = 0;
                nodes[n_nodes].indexes[0] = nodes[n_nodes].indexes[1] = 0;
                nodes[at].indexes[bit] = n_nodes++;
            }
            at = nodes[at].indexes[bit];
        }
        nodes[at].is_symbol = 1;
        nodes[at].symbol = s;
    }
    read_minmax(which, k_mode, rec, minmax);
    for (s = 0; s < ns; s++) {
        size_t nbits = (size_t)(rec[mmb + 2 * s] | (rec[mmb + 2 * s + 1] << 8));
        size_t up = pos, down = pos + nbits;
        uint8_t buf[HALF + 1];
        int dir, k;
        for (dir = 0; dir < 2; dir++) { /* 0: upwards from the start; 1: downwards from the end */
            int write_idx = 0, index = 0;
            while (write_idx < HALF) {
                int bit;
                if (up >= down) return -1;
                bit = dir == 0 ? get_bit(rec + hdr, up++) : get_bit(rec + hdr, --down);
                index = nodes[index].indexes[bit];
                buf[write_idx] = (uint8_t)nodes[index].symbol;
                write_idx += nodes[index].is_symbol;
                index &= ~(-nodes[index].is_symbol);
            }
            for (k = 0; k < HALF; k++) {
                int t, c;
                slice_pos(which, s, dir == 0 ? k : sl - 1 - k, &t, &c);
                codes[t * D + c] = buf[k];
            }
        }
        if (up != down) return -1;
        pos += nbits;
    }
    return 0;
}

/* ---------------------------------------------------------------- attention ------------------------------- */

/*
 * Decode attention for one query head over S tokens (Figure 1): scores = scale * K q, weights = softmax(scores),
 * out = weights^T V.  Kd, Vd: [S][128] binary64; q: 128 binary16 bit patterns; out: 128 binary64.
 */
void orc_attention_head(const double *Kd, const double *Vd, long S, const uint16_t *q, double scale, double *out) {
    double *sc = (double *)malloc(sizeof(double) * (size_t)(S > 0 ? S : 1));
    double mx = -INFINITY, sum = 0.0;
    long t;
    int c;
    for (c = 0; c < D; c++) out[c] = 0.0;
    for (t = 0; t < S; t++) {
        double a = 0.0;
        for (c = 0; c < D; c++) a += (double)half_to_float(q[c]) * Kd[t * D + c];
        sc[t] = scale * a;
        if (sc[t] > mx) mx = sc[t];
    }
    for (t = 0; t < S; t++) { sc[t] = exp(sc[t] - mx); sum += sc[t]; }
    for (t = 0; t < S; t++) {
        double p = sc[t] / sum;
        for (c = 0; c < D; c++) out[c] += p * Vd[t * D + c];
    }
    free(sc);
}

/* ---------------------------------------------------------------- whole-tensor drivers -------------------- */

/* Copy block j of (b, h) out of X [B][S][H][128] into a [64][128] tile. */
static void gather_tile(const uint16_t *X, long S, int H, int b, int h, long j, uint16_t *tile) {
    int t;
    for (t = 0; t < BT; t++)
        memcpy(tile + t * D, X + (((size_t)b * (size_t)S + (size_t)(j * BT + t)) * (size_t)H + (size_t)h) * D,
               D * sizeof(uint16_t));
}

/*
 * Quantize every full block of X.  codes: [B*H*NB][64*128]; minmax: [B*H*NB][n_units*2], blocks in (b, h, j)
 * order, NB = S / 64.
 */
int orc_tensor_quantize(int which, int k_mode, const uint16_t *X, int B, long S, int H, float rel_eb, uint8_t *codes,
                        uint16_t *minmax) {
    long NB = S / BT, nblk = (long)B * H * NB, i;
    int nu = orc_n_units(which, k_mode), err = 0;
#pragma omp parallel for schedule(static)
    for (i = 0; i < nblk; i++) {
        uint16_t tile[BT * D];
        int b = (int)(i / (H * NB)), h = (int)((i / NB) % H);
        long j = i % NB;
        int r;
        gather_tile(X, S, H, b, h, j, tile);
        r = orc_quantize_block(which, k_mode, tile, rel_eb, codes + (size_t)i * BT * D, minmax + (size_t)i * nu * 2);
        if (r) {
#pragma omp critical
            err = r;
        }
    }
    return err;
}

/*
 * Encode blocks one after the other into out (compact placement in block order).  sizes16[i] receives the record
 * size of block i in 16-byte units.  Returns the total bytes written, or 0 on overflow.
 */
size_t orc_tensor_encode(int which, int k_mode, const uint8_t *codes, const uint16_t *minmax, long nblk,
                         const uint8_t *len, const uint32_t *code, uint8_t *out, size_t cap, uint32_t *sizes16) {
    int nu = orc_n_units(which, k_mode);
    size_t at = 0;
    long i;
    for (i = 0; i < nblk; i++) {
        size_t n = orc_encode_block(which, k_mode, codes + (size_t)i * BT * D, minmax + (size_t)i * nu * 2, len, code,
                                    out + at, cap - at);
        if (n == 0) return 0;
        sizes16[i] = (uint32_t)(n / 16);
        at += n;
    }
    return at;
}

/*
 * One decode-attention step over the compressed cache plus the uncompressed residual tokens
 * (Section 3.3.2; Section 3.2.3: the whole cache, including the newest vectors, takes part).
 *   arena                 compressed records; k_off16 / v_off16 [B*H][max_blocks] give each block's record offset
 *                         in 16-byte units (the Block Offsets Array of Section 3)
 *   resK / resV           [B][res_tokens][H][128] binary16, the buffer of uncompressed tokens (Section 3.2.1:
 *                         up to buffer_size of them), oldest first, the first n_res token slots valid
 *   q                     [B][Hq][128] binary16; query head g reads kv head g / (Hq / H)
 *   out                   [B][Hq][128] binary64
 * Returns 0 or a negative error.
 */
int orc_attn_decode(int B, int H, int Hq, int k_mode, float rel_eb_k, float rel_eb_v, long n_blocks, long max_blocks,
                    const uint8_t *arena, const uint32_t *k_off16, const uint32_t *v_off16, const uint8_t *lenK,
                    const uint8_t *lenV, const uint16_t *resK, const uint16_t *resV, int res_tokens, int n_res,
                    const uint16_t *q, double scale, double *out) {
    int G = Hq / H, err = 0;
    long S = n_blocks * BT + n_res, bh;
    if (G < 1 || G * H != Hq || n_res > res_tokens) return -1;
#pragma omp parallel for schedule(dynamic, 1)
    for (bh = 0; bh < (long)B * H; bh++) {
        int b = (int)(bh / H), h = (int)(bh % H), g, t, c, fin;
        long j;
        double *Kd = (double *)malloc(sizeof(double) * (size_t)(S > 0 ? S : 1) * D);
        double *Vd = (double *)malloc(sizeof(double) * (size_t)(S > 0 ? S : 1) * D);
        uint8_t codes[BT * D];
        uint16_t mm[2 * D];
        for (j = 0; j < n_blocks; j++) {
            const uint8_t *rk = arena + (size_t)k_off16[bh * max_blocks + j] * 16;
            const uint8_t *rv = arena + (size_t)v_off16[bh * max_blocks + j] * 16;
            if (orc_decode_block_serial(0, k_mode, rk, lenK, codes, mm)) err = -2;
            orc_dequantize_block(0, k_mode, codes, mm, rel_eb_k, Kd + (size_t)j * BT * D);
            if (orc_decode_block_serial(1, 0, rv, lenV, codes, mm)) err = -2;
            orc_dequantize_block(1, 0, codes, mm, rel_eb_v, Vd + (size_t)j * BT * D);
        }
        for (t = 0; t < n_res; t++)
            for (c = 0; c < D; c++) {
                size_t src = (((size_t)b * (size_t)res_tokens + (size_t)t) * (size_t)H + (size_t)h) * D + (size_t)c;
                Kd[((size_t)n_blocks * BT + (size_t)t) * D + c] = half_value(resK[src], &fin);
                Vd[((size_t)n_blocks * BT + (size_t)t) * D + c] = half_value(resV[src], &fin);
            }
        for (g = 0; g < G; g++) {
            int hq = h * G + g;
            orc_attention_head(Kd, Vd, S, q + ((size_t)b * Hq + hq) * D, scale, out + ((size_t)b * Hq + hq) * D);
        }
        free(Kd);
        free(Vd);
    }
    return err;
}

int orc_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* n >= 1: number of threads for the following calls (timing with one core); no effect without OpenMP */
void orc_set_num_threads(int n) {
#ifdef _OPENMP
    if (n >= 1) omp_set_num_threads(n);
#else
    (void)n;
#endif
}
