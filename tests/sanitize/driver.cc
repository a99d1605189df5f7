// CPU-only check program, built by tests/test_sanitizers.py with -fsanitize=address,undefined (never on a GPU machine's
// device code): the oracle's C functions and the library's host-only logic run under the sanitizers on seeded
// random inputs, and the pins that need no device are repeated here:
//   * the library's host codebook (two-queue Huffman, count halving, canonical codes) equals the oracle's for
//     random histograms and every admissible length limit; the decode table and the array tree built from it
//     send every code word back to its symbol;
//   * quantize -> encode -> both oracle decoders round-trips, records stay inside the worst-case size;
//   * configuration checks and the arena layout over a sweep of valid and invalid configurations.
// Exit status 0 = all checks passed (a sanitizer report aborts the program).
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <vector>

#include "../../paper_2509_00579_amd/csrc/host_logic.h"

extern "C" {
int orc_n_sym(float rel_eb);
int orc_n_units(int which, int k_mode);
int orc_header_bytes(int which, int k_mode);
int orc_quantize_block(int which, int k_mode, const uint16_t *tile, float rel_eb, uint8_t *codes, uint16_t *minmax);
int orc_build_codebook(const uint64_t *hist, int n_sym, int max_len, uint8_t *len_out, uint32_t *code_out);
size_t orc_encode_block(int which, int k_mode, const uint8_t *codes, const uint16_t *minmax, const uint8_t *len,
                        const uint32_t *code, uint8_t *rec, size_t cap);
int orc_decode_block_serial(int which, int k_mode, const uint8_t *rec, const uint8_t *len, uint8_t *codes, uint16_t *minmax);
int orc_decode_block_tree(int which, int k_mode, const uint8_t *rec, const uint8_t *len, const uint32_t *code,
                          uint8_t *codes, uint16_t *minmax);
void orc_histogram(const uint8_t *codes, size_t n, uint64_t *hist);
uint16_t orc_float_to_half(float f);
}

#define CHECK(cond)                                                                 \
    do {                                                                            \
        if (!(cond)) {                                                              \
            std::fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #cond); \
            std::exit(1);                                                           \
        }                                                                           \
    } while (0)

using namespace kvc;
using namespace kvc::host;

static void codebooks(std::mt19937_64 &rng) {
    int cases = 0;
    for (int round = 0; round < 300; round++) {
        const int n_sym = 2 + (int)(rng() % 255);  // 2..256
        uint64_t hist64[256] = {0};
        uint32_t hist32[256] = {0};
        const int shape = (int)(rng() % 4);
        for (int s = 0; s < n_sym; s++) {
            uint32_t v;
            if (shape == 0) v = (uint32_t)(rng() % 1000);
            else if (shape == 1) v = (uint32_t)(1u << (rng() % 24));         // wide dynamic range: long code words
            else if (shape == 2) v = s < 3 ? (uint32_t)(rng() % 100000) : 0;  // most levels unseen
            else v = (uint32_t)(0xffffffffu >> (s % 32));                     // geometric, forces count halving
            hist32[s] = v;
            hist64[s] = v;
        }
        int min_limit = 1;
        while ((1 << min_limit) < n_sym) min_limit++;
        for (int limit = min_limit; limit <= kLutBits; limit++) {
            uint8_t len_o[256], len_h[256];
            uint32_t code_o[256], code_h[256];
            CHECK(orc_build_codebook(hist64, n_sym, limit, len_o, code_o) >= 0);
            build_codebook_host(hist32, n_sym, limit, len_h, code_h);
            CHECK(std::memcmp(len_o, len_h, 256) == 0);
            CHECK(std::memcmp(code_o, code_h, sizeof(code_o)) == 0);
            std::vector<uint32_t> enc(512);
            std::vector<uint16_t> lut(kLutSize);
            std::vector<int16_t> tree(512);
            const int bits = build_tables(len_h, code_h, enc.data(), lut.data(), tree.data());
            CHECK(bits >= 1 && bits <= limit);
            for (int s = 0; s < n_sym; s++) {
                const int L = len_h[s];
                CHECK(L >= 1 && L <= bits);
                const uint32_t rev = reverse_bits(code_h[s], L);
                CHECK((enc[s] >> 16) == (uint32_t)L && (enc[s] & 0xffffu) == rev && (enc[256 + s] & 0xffffu) == code_h[s]);
                for (uint32_t k = 0; k < (1u << (bits - L)); k++)      // whatever bits follow the code word
                    CHECK(lut[rev | (k << L)] == (uint16_t)((s << 8) | L));
                int node = 0;                                          // the tree walk reaches the same symbol
                for (int i = 0; i < L; i++) {
                    const int child = tree[2 * node + ((code_h[s] >> (L - 1 - i)) & 1)];
                    if (i == L - 1) CHECK(child == (int16_t)~s);
                    else { CHECK(child > 0 && child < 256); node = child; }
                }
            }
            cases++;
        }
    }
    std::printf("codebooks: %d cases, library host code == oracle\n", cases);
}

static void codec(std::mt19937_64 &rng) {
    std::normal_distribution<float> normal(0.f, 1.f);
    int cases = 0;
    for (int round = 0; round < 24; round++) {
        const int which = round & 1, k_mode = which == 0 ? (round >> 1) & 1 : 0;
        const float rel_eb = (round % 3 == 0) ? 5e-3f : (round % 3 == 1) ? 1e-2f : 5e-2f;
        const int n_sym = orc_n_sym(rel_eb);
        std::vector<uint16_t> tile(kTile), minmax(2 * 128), minmax2(2 * 128);
        for (int i = 0; i < kTile; i++) tile[i] = orc_float_to_half(normal(rng) * (1.f + (float)(i % 128 % 7)));
        if (round % 5 == 0)
            for (int t = 0; t < 64; t++) tile[t * 128 + 9] = orc_float_to_half(0.25f);  // a constant K unit
        std::vector<uint8_t> codes(kTile), back(kTile);
        CHECK(orc_quantize_block(which, k_mode, tile.data(), rel_eb, codes.data(), minmax.data()) == 0);
        uint64_t hist[256];
        orc_histogram(codes.data(), codes.size(), hist);
        int min_limit = 1;
        while ((1 << min_limit) < n_sym) min_limit++;
        const int limit = min_limit + (int)(rng() % (kLutBits - min_limit + 1));
        uint8_t len[256];
        uint32_t code[256];
        CHECK(orc_build_codebook(hist, n_sym, limit, len, code) >= 0);
        const size_t cap = (size_t)orc_header_bytes(which, k_mode) + (size_t)kTile * limit / 8 + 16;
        std::vector<uint8_t> rec(cap);   // exactly the worst case: an overrun is an address-sanitizer report
        const size_t bytes = orc_encode_block(which, k_mode, codes.data(), minmax.data(), len, code, rec.data(), cap);
        CHECK(bytes > 0 && bytes <= cap);
        std::vector<uint8_t> exact(rec.begin(), rec.begin() + (long)((bytes + 15) / 16 * 16 <= cap ? (bytes + 15) / 16 * 16 : cap));
        CHECK(orc_decode_block_serial(which, k_mode, exact.data(), len, back.data(), minmax2.data()) == 0);
        CHECK(back == codes);
        std::fill(back.begin(), back.end(), 0);
        CHECK(orc_decode_block_tree(which, k_mode, exact.data(), len, code, back.data(), minmax2.data()) == 0);
        CHECK(back == codes);
        const int nu = orc_n_units(which, k_mode);
        CHECK(std::memcmp(minmax.data(), minmax2.data(), (size_t)nu * 4) == 0);
        cases++;
    }
    std::printf("codec: %d blocks, encode -> both decoders round-trip\n", cases);
}

static void layouts() {
    int valid = 0, invalid = 0;
    const float ebs[] = {0.f, 1e-3f, 2e-3f, 1e-2f, 0.1f, 0.5f, 0.6f};
    for (int B : {0, 1, 3})
        for (int H : {0, 1, 8})
            for (int G : {1, 2, 3, 4, 8, 16})
                for (int seq : {0, 1, 63, 64, 4096, 100000})
                    for (float eb : ebs)
                        for (int k_mode : {0, 1, 2})
                            for (int lim : {0, 3, 6, 7, 12, 13})
                                for (int buf : {0, 32, 64, 100, 4096, 8192}) {
                                    kvcomp_config c = {B, H, H * G, 128, 64, seq, eb, eb, k_mode, lim, buf};
                                    if (!valid_cfg(&c)) { invalid++; continue; }
                                    valid++;
                                    const Layout L = make_layout(c);
                                    CHECK(L.ctrl == 0 && L.hist >= 256 && L.payload % 256 == 0 && L.total % 256 == 0);
                                    CHECK(L.hist < L.tables && L.tables + 2 * (size_t)kvc::kTensorTablesBytes <= L.counters);
                                    CHECK(L.counters < L.table && L.table < L.res && L.res < L.partials && L.partials < L.payload);
                                    CHECK(L.payload + L.payload_cap16 * 16 <= L.total);
                                    // room for every block of every (batch, head) at the worst case
                                    const size_t worst = ((size_t)k_header_bytes(c) + kHdrBytesV + 2 * (size_t)kTile * code_len_limit(c) / 8 + 30);
                                    CHECK(L.payload_cap16 * 16 + 512 >= (size_t)B * H * (size_t)(seq / 64) * (worst - 30));
                                    CHECK(buffer_tokens(c) >= 64 && buffer_tokens(c) % 64 == 0);
                                }
    CHECK(valid > 0 && invalid > 0);
    kvcomp_config ok = {1, 1, 1, 128, 64, 128, 1e-2f, 1e-2f, 0, 0, 0};
    CHECK(valid_cfg(&ok) && !valid_cfg(nullptr));
    std::printf("layouts: %d valid and %d invalid configurations\n", valid, invalid);
}

int main() {
    std::mt19937_64 rng(20250907);
    codebooks(rng);
    codec(rng);
    layouts();
    std::printf("sanitizer driver: ok\n");
    return 0;
}
