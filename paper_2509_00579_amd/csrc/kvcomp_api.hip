// Host side of libkvcomp: the C ABI declared in include/kvcomp.h, arena bookkeeping, and the host-built
// Huffman codebook (the paper builds the codebooks on the CPU from a GPU histogram, Section 3).
#include <algorithm>
#include <cstdarg>
#include <cstddef>
#include <cstdio>
#include <cstring>
#include <new>
#include <numeric>
#include <vector>

#include "../../include/kvcomp.h"
#include "host_logic.h"
#include "kvcomp_internal.h"

using namespace kvc;
using namespace kvc::host;

namespace {

thread_local char g_err[512] = "";

kvcomp_status fail(kvcomp_status st, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return st;
}

#define HIP_TRY(expr)                                                                              \
    do {                                                                                           \
        hipError_t e_ = (expr);                                                                    \
        if (e_ != hipSuccess) return fail(KVCOMP_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

}  // namespace

struct kvcomp_ctx {
    kvcomp_config cfg;
    Layout lay;
    Geo geo;
    uint8_t *arena;
    bool have_codebook;
    int n_blocks, n_res;
    int res_head;  // ring slot of the oldest buffered token, a multiple of 64
    uint8_t len[2][256];
    uint32_t code[2][256];
    uint32_t max_size16;
    int tune_splits, tune_stage, tune_waves;
    bool profiling;
    std::vector<hipEvent_t> events;  // pairs
    size_t events_used;
    int prof_launches;
    double prof_ms;
    // pinned host staging
    Ctrl *h_ctrl;
    uint32_t *h_hist;  // [2][256]
    uint8_t *h_tables; // [2 tensors][kTensorTablesBytes], laid out like Geo::tables
    uint8_t *h_tables_dev;  // the same memory as kernels address it
    hipEvent_t ev_hist[2];  // the histogram of K, of V has reached the host
};

namespace {

kvcomp_status read_ctrl(kvcomp_ctx *ctx, hipStream_t s) {
    HIP_TRY(hipMemcpyAsync(ctx->h_ctrl, ctx->geo.ctrl, sizeof(Ctrl), hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    return KVCOMP_OK;
}

kvcomp_status fold_profile(kvcomp_ctx *ctx) {
    for (size_t i = 0; i + 1 < ctx->events_used; i += 2) {
        HIP_TRY(hipEventSynchronize(ctx->events[i + 1]));
        float ms = 0.f;
        HIP_TRY(hipEventElapsedTime(&ms, ctx->events[i], ctx->events[i + 1]));
        ctx->prof_ms += ms;
        ctx->prof_launches++;
    }
    ctx->events_used = 0;
    return KVCOMP_OK;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// After read_ctrl: what the kernels flagged since the last synchronising call (a non-finite input value, e.g. in a
// token that an append flushed; a kernel that refused work).  Clears the flags on the device.
kvcomp_status check_flags(kvcomp_ctx *ctx, hipStream_t s) {
    const uint32_t nonfinite = ctx->h_ctrl->nonfinite, fault = ctx->h_ctrl->fault;
    if (!nonfinite && !fault) return KVCOMP_OK;
    static_assert(offsetof(Ctrl, nonfinite) == 8 && offsetof(Ctrl, fault) == 12, "the two flags are neighbours");
    HIP_TRY(hipMemsetAsync(&ctx->geo.ctrl->nonfinite, 0, 2 * sizeof(uint32_t), s));
    HIP_TRY(hipStreamSynchronize(s));
    if (nonfinite) return fail(KVCOMP_ERR_NONFINITE, "an input held Inf or NaN");
    if (fault & kFaultArenaFull)
        return fail(KVCOMP_ERR_CAPACITY, "a flush found the record arena full (a captured flush replayed without the "
                                         "eager calls in between?): its blocks were not written");
    return fail(KVCOMP_ERR_STATE, "the decompressor met a record larger than its staging area: that block was skipped");
}

}  // namespace

extern "C" {

const char *kvcomp_last_error(void) { return g_err; }

size_t kvcomp_arena_bytes(const kvcomp_config *cfg) {
    if (!valid_cfg(cfg)) return 0;
    return make_layout(*cfg).total;
}

kvcomp_status kvcomp_create(const kvcomp_config *cfg, void *d_arena, size_t arena_bytes, void *stream,
                            kvcomp_ctx **out) {
    if (!out) return fail(KVCOMP_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    if (!valid_cfg(cfg)) return fail(KVCOMP_ERR_INVALID_ARG, "invalid configuration");
    if (!d_arena || (reinterpret_cast<uintptr_t>(d_arena) & 255u))
        return fail(KVCOMP_ERR_INVALID_ARG, "arena must be a 256-byte aligned device pointer");
    const Layout L = make_layout(*cfg);
    if (arena_bytes < L.total) return fail(KVCOMP_ERR_CAPACITY, "arena has %zu bytes, %zu needed", arena_bytes, L.total);
    if (L.payload_cap16 >= (1ull << 32)) return fail(KVCOMP_ERR_CAPACITY, "payload arena exceeds 64 GiB");
    kvcomp_ctx *c = new (std::nothrow) kvcomp_ctx();
    if (!c) return fail(KVCOMP_ERR_INVALID_ARG, "out of host memory");
    c->cfg = *cfg;
    c->lay = L;
    c->arena = static_cast<uint8_t *>(d_arena);
    c->have_codebook = false;
    c->n_blocks = c->n_res = c->res_head = 0;
    c->max_size16 = 0;
    c->tune_splits = c->tune_stage = c->tune_waves = 0;
    c->profiling = false;
    c->events_used = 0;
    c->prof_launches = 0;
    c->prof_ms = 0.0;
    Geo &g = c->geo;
    g.B = cfg->batch;
    g.H = cfg->n_kv_heads;
    g.Hq = cfg->n_q_heads;
    g.G = g.Hq / g.H;
    g.max_blocks = std::max(L.max_blocks, 1);
    g.k_units = cfg->k_mode == 1 ? 1 : kD;
    g.k_minmax_bytes = k_minmax_bytes(*cfg);
    g.two_eb[0] = 2.0f * cfg->rel_eb_k;
    g.two_eb[1] = 2.0f * cfg->rel_eb_v;
    g.n_sym[0] = n_sym_for(cfg->rel_eb_k);
    g.n_sym[1] = n_sym_for(cfg->rel_eb_v);
    g.ctrl = reinterpret_cast<Ctrl *>(c->arena + L.ctrl);
    g.hist = reinterpret_cast<uint32_t *>(c->arena + L.hist);
    g.tables = c->arena + L.tables;
    g.lut_bits[0] = g.lut_bits[1] = kLutBits;
    g.counters = reinterpret_cast<uint32_t *>(c->arena + L.counters);
    g.place_sums = reinterpret_cast<uint32_t *>(c->arena + L.place_sums);
    g.table = reinterpret_cast<BlockEntry *>(c->arena + L.table);
    g.res = reinterpret_cast<uint16_t *>(c->arena + L.res);
    g.res_tokens = buffer_tokens(*cfg);
    g.partials = reinterpret_cast<float *>(c->arena + L.partials);
    g.payload = c->arena + L.payload;
    g.payload_cap16 = (uint32_t)L.payload_cap16;
    void *pinned = nullptr;
    const size_t pin_bytes = 256 + 2 * 256 * 4 + 2 * (size_t)kTensorTablesBytes;
    hipError_t e = hipHostMalloc(&pinned, pin_bytes, hipHostMallocDefault);
    if (e != hipSuccess) {
        delete c;
        return fail(KVCOMP_ERR_HIP, "hipHostMalloc: %s", hipGetErrorString(e));
    }
    uint8_t *pb = static_cast<uint8_t *>(pinned);
    c->h_ctrl = reinterpret_cast<Ctrl *>(pb);
    c->h_hist = reinterpret_cast<uint32_t *>(pb + 256);
    c->h_tables = pb + 256 + 2048;
    {
        void *dev = nullptr;
        e = hipHostGetDevicePointer(&dev, pinned, 0);
        if (e != hipSuccess) {
            (void)hipHostFree(pinned);
            delete c;
            return fail(KVCOMP_ERR_HIP, "hipHostGetDevicePointer: %s", hipGetErrorString(e));
        }
        c->h_tables_dev = static_cast<uint8_t *>(dev) + 256 + 2048;
    }
    c->ev_hist[0] = c->ev_hist[1] = nullptr;
    for (int w = 0; w < 2 && e == hipSuccess; w++) e = hipEventCreateWithFlags(&c->ev_hist[w], hipEventDisableTiming);
    if (e != hipSuccess) {
        for (int w = 0; w < 2; w++)
            if (c->ev_hist[w]) (void)hipEventDestroy(c->ev_hist[w]);
        (void)hipHostFree(pinned);
        delete c;
        return fail(KVCOMP_ERR_HIP, "hipEventCreate: %s", hipGetErrorString(e));
    }
    // control words, histogram, tables and the Block Offsets Array start at zero
    e = launch_fill_zero(c->arena, L.res, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) {
        for (int w = 0; w < 2; w++) (void)hipEventDestroy(c->ev_hist[w]);
        (void)hipHostFree(pinned);
        delete c;
        return fail(KVCOMP_ERR_HIP, "arena init: %s", hipGetErrorString(e));
    }
    *out = c;
    return KVCOMP_OK;
}

kvcomp_status kvcomp_destroy(kvcomp_ctx *ctx) {
    if (!ctx) return KVCOMP_OK;
    for (hipEvent_t ev : ctx->events) (void)hipEventDestroy(ev);
    for (int w = 0; w < 2; w++) (void)hipEventDestroy(ctx->ev_hist[w]);
    (void)hipHostFree(ctx->h_ctrl);
    delete ctx;
    return KVCOMP_OK;
}

kvcomp_status kvcomp_reset(kvcomp_ctx *ctx, int keep_codebook, void *stream) {
    if (!ctx) return fail(KVCOMP_ERR_INVALID_ARG, "ctx is NULL");
    hipStream_t s = static_cast<hipStream_t>(stream);
    HIP_TRY(launch_fill_zero(ctx->geo.ctrl, 256, s));
    ctx->n_blocks = ctx->n_res = ctx->res_head = 0;
    ctx->max_size16 = 0;
    if (!keep_codebook) ctx->have_codebook = false;
    return KVCOMP_OK;
}

// Where kvcomp_prefill keeps the quantization codes and unit min/max between its histogram pass and its encode pass.
struct PrefillWs {
    uint8_t *codes[2];
    uint32_t *minmax[2];
    uint16_t *block_hist[2];  // [block][256]
    size_t total;
};
static PrefillWs prefill_layout(const kvcomp_config &c, int seq, void *base) {
    const size_t nblk = (size_t)c.batch * c.n_kv_heads * (seq / kBT);
    const size_t k_units = c.k_mode == 1 ? 1 : kD;
    uint8_t *p = static_cast<uint8_t *>(base);
    PrefillWs w;
    size_t at = 0;
    w.codes[0] = p + at; at += nblk * kTile;
    w.codes[1] = p + at; at += nblk * kTile;
    w.minmax[0] = reinterpret_cast<uint32_t *>(p + at); at += align_up(nblk * k_units * 4, 16);
    w.minmax[1] = reinterpret_cast<uint32_t *>(p + at); at += align_up(nblk * kBT * 4, 16);
    w.block_hist[0] = reinterpret_cast<uint16_t *>(p + at); at += nblk * 512;
    w.block_hist[1] = reinterpret_cast<uint16_t *>(p + at); at += nblk * 512;
    w.total = at;
    return w;
}

// The codebook of tensor w from its histogram on the host, its tables, and their upload by a kernel that reads the
// pinned staging block (stream-ordered: whatever uses the tables comes after it on the same stream, and this tensor's
// part of the staging block is not rewritten before the next codebook).
static kvcomp_status codebook_of(kvcomp_ctx *ctx, int w, const uint32_t *hist, hipStream_t s) {
    Geo &g = ctx->geo;
    uint8_t *tab = ctx->h_tables + (size_t)w * kTensorTablesBytes;
    uint16_t *lut = reinterpret_cast<uint16_t *>(tab + kTabLutOff);
    uint32_t *pair = reinterpret_cast<uint32_t *>(tab + kTabPairOff);
    build_codebook_host(hist, g.n_sym[w], code_len_limit(ctx->cfg), ctx->len[w], ctx->code[w]);
    g.lut_bits[w] = build_tables(ctx->len[w], ctx->code[w], reinterpret_cast<uint32_t *>(tab + kTabEncOff), lut,
                                 reinterpret_cast<int16_t *>(tab + kTabTreeOff));
    if (g.lut_bits[w] <= 6) build_pair_table(lut, g.lut_bits[w], pair);
    else std::memset(pair, 0, kPairEntries * 4);
    static_assert(kTensorTablesBytes % 16 == 0, "whole 16-byte units");
    // V's upload (the last thing that runs after both histograms have been read) also clears the device histogram
    // for the next call
    HIP_TRY(launch_copy16(g.tables + (size_t)w * kTensorTablesBytes, ctx->h_tables_dev + (size_t)w * kTensorTablesBytes,
                          kTensorTablesBytes, g.hist, w == 1 ? 2 * 256 * 4 : 0, s));
    return KVCOMP_OK;
}

// Histogram on the device, codebooks on the host, tables to the device (Section 3).  ws != NULL: the histogram pass
// also keeps the codes, min/max and histogram of every block there, and the encoding of the first n_blk blocks per
// (batch, head) is queued for each tensor as soon as its tables are.
// The host's part for K runs while the device histograms V, and K's records are written while the host does V's.
static kvcomp_status codebook_impl(kvcomp_ctx *ctx, const void *d_K, const void *d_V, int seq, const PrefillWs *ws,
                                   int n_blk, hipStream_t s) {
    if (!aligned16(d_K) || !aligned16(d_V)) return fail(KVCOMP_ERR_INVALID_ARG, "K/V must be 16-byte aligned");
    if (seq < kBT || seq > ctx->cfg.max_seq)
        return fail(KVCOMP_ERR_INVALID_ARG, "seq %d outside [64, max_seq=%d]", seq, ctx->cfg.max_seq);
    // the codebooks are built once, at prefill, and reused (Section 3): new tables under existing records would make
    // every one of them decode to garbage
    if (ctx->n_blocks || ctx->n_res) return fail(KVCOMP_ERR_STATE, "cache is not empty: kvcomp_reset first");
    const long long symbols = (long long)ctx->geo.B * ctx->geo.H * (seq / kBT) * kTile;
    if (symbols >= (1ll << 32)) return fail(KVCOMP_ERR_INVALID_ARG, "more than 2^32 symbols per tensor");
    Geo &g = ctx->geo;
    static_assert(sizeof(Ctrl) <= 256, "control words fill the first 256 bytes");
    // the device histogram is zero here: the arena starts that way, and every call that got as far as reading it
    // back leaves it so (codebook_of for V, or the failure path below)
    HIP_TRY(launch_histogram(g, 0, static_cast<const uint16_t *>(d_K), seq, seq / kBT, ws ? ws->codes[0] : nullptr,
                             ws ? ws->minmax[0] : nullptr, ws ? ws->block_hist[0] : nullptr, s));
    HIP_TRY(hipMemcpyAsync(ctx->h_hist, g.hist, 256 * 4, hipMemcpyDeviceToHost, s));
    HIP_TRY(hipEventRecord(ctx->ev_hist[0], s));
    HIP_TRY(launch_histogram(g, 1, static_cast<const uint16_t *>(d_V), seq, seq / kBT, ws ? ws->codes[1] : nullptr,
                             ws ? ws->minmax[1] : nullptr, ws ? ws->block_hist[1] : nullptr, s));
    // control words and the histogram of V (neighbours of K's histogram in the arena and in the staging block, which
    // therefore travels again: the same values over the same bytes)
    HIP_TRY(hipMemcpyAsync(ctx->h_ctrl, g.ctrl, 256 + 2 * 256 * 4, hipMemcpyDeviceToHost, s));
    HIP_TRY(hipEventRecord(ctx->ev_hist[1], s));
    HIP_TRY(hipEventSynchronize(ctx->ev_hist[0]));
    {
        uint32_t hist_k[256];
        std::memcpy(hist_k, ctx->h_hist, sizeof(hist_k));
        kvcomp_status st = codebook_of(ctx, 0, hist_k, s);
        if (st) return st;
    }
    if (ws) HIP_TRY(launch_encode_kept(g, 0, ws->codes[0], ws->minmax[0], ws->block_hist[0], seq / kBT, n_blk, s));
    HIP_TRY(hipEventSynchronize(ctx->ev_hist[1]));
    {
        kvcomp_status st = check_flags(ctx, s);
        if (st) {
            // K's records may be on their way already: the cache was empty at entry, so it is again with the control
            // words back at zero (arena tail, largest record)
            if (ws) (void)launch_fill_zero(g.ctrl, 256, s);
            (void)launch_fill_zero(g.hist, 2 * 256 * 4, s);
            return st;
        }
        st = codebook_of(ctx, 1, ctx->h_hist + 256, s);
        if (st) return st;
    }
    if (ws) HIP_TRY(launch_encode_kept(g, 1, ws->codes[1], ws->minmax[1], ws->block_hist[1], seq / kBT, n_blk, s));
    ctx->have_codebook = true;
    return KVCOMP_OK;
}

// After the encode launches of a prompt: the newest tokens to the fp16 buffer, then the one synchronisation that
// brings the arena tail, the largest record and the flags to the host.
static kvcomp_status finish_prompt(kvcomp_ctx *ctx, const uint16_t *K, const uint16_t *V, int seq, int nb, hipStream_t s) {
    const Geo &g = ctx->geo;
    HIP_TRY(launch_copy_tail(g, K, V, seq, nb * kBT, seq - nb * kBT, s));
    kvcomp_status st = read_ctrl(ctx, s);
    if (st) return st;
    if (ctx->h_ctrl->nonfinite || ctx->h_ctrl->fault) {
        st = check_flags(ctx, s);
        (void)launch_fill_zero(g.ctrl, 256, s);  // nothing of this call stays in the cache
        return st;
    }
    ctx->n_blocks = nb;
    ctx->n_res = seq - nb * kBT;
    ctx->res_head = 0;
    ctx->max_size16 = ctx->h_ctrl->max_size16;
    return KVCOMP_OK;
}

// blocks that seq appended tokens leave compressed: the buffer keeps the newest tokens, its oldest block is cut off
// whenever it holds res_tokens of them
static int prompt_blocks(const Geo &g, int seq) { return seq < g.res_tokens ? 0 : (seq - g.res_tokens) / kBT + 1; }

kvcomp_status kvcomp_build_codebook(kvcomp_ctx *ctx, const void *d_K, const void *d_V, int seq, void *stream) {
    if (!ctx || !d_K || !d_V) return fail(KVCOMP_ERR_INVALID_ARG, "NULL argument");
    hipStream_t s = static_cast<hipStream_t>(stream);
    kvcomp_status st = codebook_impl(ctx, d_K, d_V, seq, nullptr, 0, s);
    if (st) return st;
    HIP_TRY(hipStreamSynchronize(s));
    return KVCOMP_OK;
}

kvcomp_status kvcomp_compress_blocks(kvcomp_ctx *ctx, const void *d_K, const void *d_V, int seq, void *stream) {
    if (!ctx || !d_K || !d_V) return fail(KVCOMP_ERR_INVALID_ARG, "NULL argument");
    if (!aligned16(d_K) || !aligned16(d_V)) return fail(KVCOMP_ERR_INVALID_ARG, "K/V must be 16-byte aligned");
    if (!ctx->have_codebook) return fail(KVCOMP_ERR_STATE, "no codebook: call kvcomp_build_codebook first");
    if (ctx->n_blocks || ctx->n_res) return fail(KVCOMP_ERR_STATE, "cache is not empty");
    if (seq < 1) return fail(KVCOMP_ERR_INVALID_ARG, "seq must be positive");
    if (seq > ctx->cfg.max_seq) return fail(KVCOMP_ERR_CAPACITY, "seq %d exceeds max_seq %d", seq, ctx->cfg.max_seq);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const Geo &g = ctx->geo;
    const int nb = prompt_blocks(g, seq);
    const uint16_t *K = static_cast<const uint16_t *>(d_K), *V = static_cast<const uint16_t *>(d_V);
    HIP_TRY(launch_encode(g, K, V, seq, nb, 0, s));
    return finish_prompt(ctx, K, V, seq, nb, s);
}

size_t kvcomp_prefill_workspace_bytes(const kvcomp_config *cfg, int seq) {
    if (!valid_cfg(cfg) || seq < kBT) return 0;
    return prefill_layout(*cfg, seq, nullptr).total;
}

kvcomp_status kvcomp_prefill(kvcomp_ctx *ctx, const void *d_K, const void *d_V, int seq, void *d_workspace,
                             size_t workspace_bytes, void *stream) {
    if (!ctx || !d_K || !d_V || !d_workspace) return fail(KVCOMP_ERR_INVALID_ARG, "NULL argument");
    if (!aligned16(d_workspace)) return fail(KVCOMP_ERR_INVALID_ARG, "workspace must be 16-byte aligned");
    if (seq < kBT || seq > ctx->cfg.max_seq)
        return fail(KVCOMP_ERR_INVALID_ARG, "seq %d outside [64, max_seq=%d]", seq, ctx->cfg.max_seq);
    const PrefillWs ws = prefill_layout(ctx->cfg, seq, d_workspace);
    if (workspace_bytes < ws.total)
        return fail(KVCOMP_ERR_CAPACITY, "workspace has %zu bytes, %zu needed", workspace_bytes, ws.total);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const Geo &g = ctx->geo;
    const int nb = prompt_blocks(g, seq);
    kvcomp_status st = codebook_impl(ctx, d_K, d_V, seq, &ws, nb, s);
    if (st) return st;
    return finish_prompt(ctx, static_cast<const uint16_t *>(d_K), static_cast<const uint16_t *>(d_V), seq, nb, s);
}

kvcomp_status kvcomp_append_token(kvcomp_ctx *ctx, const void *d_k_new, const void *d_v_new, void *stream) {
    if (!ctx || !d_k_new || !d_v_new) return fail(KVCOMP_ERR_INVALID_ARG, "NULL argument");
    if (!aligned16(d_k_new) || !aligned16(d_v_new)) return fail(KVCOMP_ERR_INVALID_ARG, "k/v must be 16-byte aligned");
    if (!ctx->have_codebook) return fail(KVCOMP_ERR_STATE, "no codebook: call kvcomp_build_codebook first");
    if (ctx->n_blocks * kBT + ctx->n_res + 1 > ctx->cfg.max_seq)
        return fail(KVCOMP_ERR_CAPACITY, "max_seq %d reached", ctx->cfg.max_seq);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const Geo &g = ctx->geo;
    const int slot = (ctx->res_head + ctx->n_res) % g.res_tokens;
    HIP_TRY(launch_append(g, static_cast<const uint16_t *>(d_k_new), static_cast<const uint16_t *>(d_v_new), slot, s));
    ctx->n_res++;
    if (ctx->n_res == g.res_tokens) {
        // the buffer is full: cut its oldest block off, compress it as one block per (batch, head), append the records
        const uint16_t *rk = g.res + (size_t)ctx->res_head * g.H * kD;
        const uint16_t *rv = rk + (size_t)g.B * g.res_tokens * g.H * kD;
        HIP_TRY(launch_encode(g, rk, rv, g.res_tokens, 1, ctx->n_blocks, s));
        ctx->n_blocks++;
        ctx->n_res -= kBT;
        ctx->res_head = (ctx->res_head + kBT) % g.res_tokens;
    }
    return KVCOMP_OK;
}

// One launch of the fused kernel over the cache as the host counts it (n_blocks, n_res).  k_new / v_new != NULL: the
// newest buffered token is still there and not in the buffer.
static kvcomp_status attn_impl(kvcomp_ctx *ctx, const void *d_q, float scale, float *d_out, const uint16_t *k_new,
                               const uint16_t *v_new, hipStream_t s) {
    const Geo &g = ctx->geo;
    // Work split: one workgroup per CU, holding as many waves as the registers allow per SIMD (16, 12 or 8 for groups
    // of 1-2, 4, 8 query heads) and the LDS has room for (decode tables + a staging area per wave); the grid is one
    // round of workgroups, every wave owning whole block pairs.  Per-workgroup costs (tables, split merge) are then
    // paid once per CU, and the waves of a head's split merge through LDS.
    const int longest = std::max(g.lut_bits[0], g.lut_bits[1]);
    const size_t lds_fixed = fused_lds_fixed(g.G, longest);
    int stage = ctx->tune_stage;
    if (stage <= 0) stage = (int)align_up((size_t)ctx->max_size16 * 16 + 16, 256);
    stage = std::max(stage, 4608);
    stage = (int)align_up(stage, 16);
    const size_t per_wave_rest = fused_weight_bytes(g.G);
    const int reg_waves = 4 * fused_waves_per_simd(g.G, fused_table_bits(longest));
    int max_waves = reg_waves;
    if (ctx->tune_waves > 0) max_waves = std::min(max_waves, ctx->tune_waves);
    max_waves = std::max(1, std::min(max_waves, (int)((kLdsBytesPerCU - lds_fixed) / ((size_t)stage + per_wave_rest))));
    if (lds_fixed + (size_t)stage + per_wave_rest > (size_t)kLdsBytesPerCU)
        stage = (int)((kLdsBytesPerCU - lds_fixed - per_wave_rest) / 16 * 16);  // one wave, records above it from global memory
    const int wgs_per_cu = std::max(1, std::min(reg_waves / max_waves,
                                                (int)(kLdsBytesPerCU / (lds_fixed + max_waves * ((size_t)stage + per_wave_rest)))));
    int n_splits = ctx->tune_splits;
    if (n_splits <= 0) {
        const int bh = g.B * g.H;
        const int by_chip = std::max(1, kCUs * wgs_per_cu / bh);
        const int by_work = std::max(1, (ctx->n_blocks + 3) / 4);  // at least one block pair per SIMD of the CU
        n_splits = std::min(by_chip, by_work);
    }
    n_splits = std::max(1, std::min({n_splits, (int)kMaxSplits, std::max(ctx->n_blocks, 1)}));
    // waves of a workgroup: no more than its split has block pairs (a short sequence leaves wave slots empty rather
    // than CUs), at least enough for the buffered tokens' units to spread
    const int bps = ctx->n_blocks > 0 ? (ctx->n_blocks + n_splits - 1) / n_splits : 0;
    int n_waves = std::max(1, std::min(max_waves, std::max(bps, std::min(4, (ctx->n_res + 15) / 16))));
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    if (ctx->profiling) {
        if (ctx->events_used + 2 > ctx->events.size()) {
            if (ctx->events.size() >= 8192) {
                kvcomp_status st = fold_profile(ctx);
                if (st) return st;
            } else {
                for (int i = 0; i < 2; i++) {
                    hipEvent_t ev;
                    HIP_TRY(hipEventCreate(&ev));
                    ctx->events.push_back(ev);
                }
            }
        }
        ev0 = ctx->events[ctx->events_used];
        ev1 = ctx->events[ctx->events_used + 1];
        ctx->events_used += 2;
    }
    HIP_TRY(launch_fused_attn(g, static_cast<const uint16_t *>(d_q), scale, d_out, ctx->n_blocks, ctx->res_head, ctx->n_res,
                              k_new, v_new, n_splits, n_waves, stage, ev0, ev1, s));
    return KVCOMP_OK;
}

kvcomp_status kvcomp_attn_decode(kvcomp_ctx *ctx, const void *d_q, float scale, float *d_out, void *stream) {
    if (!ctx || !d_q || !d_out) return fail(KVCOMP_ERR_INVALID_ARG, "NULL argument");
    if (ctx->n_blocks == 0 && ctx->n_res == 0) return fail(KVCOMP_ERR_STATE, "cache is empty");
    if (ctx->n_blocks && !ctx->have_codebook) return fail(KVCOMP_ERR_STATE, "no codebook");
    return attn_impl(ctx, d_q, scale, d_out, nullptr, nullptr, static_cast<hipStream_t>(stream));
}

kvcomp_status kvcomp_append_attn_decode(kvcomp_ctx *ctx, const void *d_k_new, const void *d_v_new, const void *d_q,
                                        float scale, float *d_out, void *stream) {
    if (!ctx || !d_k_new || !d_v_new || !d_q || !d_out) return fail(KVCOMP_ERR_INVALID_ARG, "NULL argument");
    if (ctx->n_res + 1 == ctx->geo.res_tokens) {  // this token fills the buffer: the block is cut off first
        kvcomp_status st = kvcomp_append_token(ctx, d_k_new, d_v_new, stream);
        if (st) return st;
        return kvcomp_attn_decode(ctx, d_q, scale, d_out, stream);
    }
    if (!aligned16(d_k_new) || !aligned16(d_v_new)) return fail(KVCOMP_ERR_INVALID_ARG, "k/v must be 16-byte aligned");
    if (!ctx->have_codebook) return fail(KVCOMP_ERR_STATE, "no codebook: call kvcomp_build_codebook first");
    if (ctx->n_blocks * kBT + ctx->n_res + 1 > ctx->cfg.max_seq)
        return fail(KVCOMP_ERR_CAPACITY, "max_seq %d reached", ctx->cfg.max_seq);
    ctx->n_res++;  // the kernel reads the token from d_k_new / d_v_new and stores it into its buffer slot
    kvcomp_status st = attn_impl(ctx, d_q, scale, d_out, static_cast<const uint16_t *>(d_k_new),
                                 static_cast<const uint16_t *>(d_v_new), static_cast<hipStream_t>(stream));
    if (st) ctx->n_res--;
    return st;
}

kvcomp_status kvcomp_get_stats(kvcomp_ctx *ctx, kvcomp_stats *o, void *stream) {
    if (!ctx || !o) return fail(KVCOMP_ERR_INVALID_ARG, "NULL argument");
    hipStream_t s = static_cast<hipStream_t>(stream);
    HIP_TRY(hipMemsetAsync(ctx->geo.ctrl->payload_bits, 0, 4 * sizeof(unsigned long long), s));
    HIP_TRY(launch_stats(ctx->geo, ctx->n_blocks, s));
    kvcomp_status st = read_ctrl(ctx, s);
    if (st) return st;
    st = check_flags(ctx, s);
    if (st) return st;
    const Ctrl &c = *ctx->h_ctrl;
    const long long BH = (long long)ctx->geo.B * ctx->geo.H;
    const long long nblk = BH * ctx->n_blocks;
    const long long tokens = (long long)ctx->n_blocks * kBT + ctx->n_res;
    o->n_blocks = ctx->n_blocks;
    o->n_res = ctx->n_res;
    o->raw_bytes = 2 * BH * tokens * kD * 2;
    o->record_bytes_k = (int64_t)c.record16[0] * 16;
    o->record_bytes_v = (int64_t)c.record16[1] * 16;
    o->header_bytes = nblk * (k_header_bytes(ctx->cfg) + kHdrBytesV);
    o->offsets_bytes = 2 * nblk * (long long)sizeof(BlockEntry);
    o->residual_bytes = 2 * BH * ctx->n_res * kD * 2;
    o->payload_bits_k = (int64_t)c.payload_bits[0];
    o->payload_bits_v = (int64_t)c.payload_bits[1];
    o->stored_bytes = o->record_bytes_k + o->record_bytes_v + o->offsets_bytes + o->residual_bytes;
    o->max_record_bytes = (int64_t)c.max_size16 * 16;
    o->compression_ratio = o->stored_bytes ? (double)o->raw_bytes / (double)o->stored_bytes : 0.0;
    return KVCOMP_OK;
}

kvcomp_status kvcomp_debug_codes(kvcomp_ctx *ctx, int which, const void *d_in, int seq, void *d_scratch,
                                 size_t scratch_bytes, uint8_t *h_codes, uint16_t *h_minmax, void *stream) {
    if (!ctx || !d_in || !d_scratch || !h_codes || !h_minmax) return fail(KVCOMP_ERR_INVALID_ARG, "NULL argument");
    if (which != 0 && which != 1) return fail(KVCOMP_ERR_INVALID_ARG, "which must be 0 (K) or 1 (V)");
    if (!aligned16(d_in) || !aligned16(d_scratch)) return fail(KVCOMP_ERR_INVALID_ARG, "pointers must be 16-byte aligned");
    if (seq < kBT) return fail(KVCOMP_ERR_INVALID_ARG, "seq must hold a full block");
    const Geo &g = ctx->geo;
    const size_t nblk = (size_t)g.B * g.H * (seq / kBT);
    const size_t units = which == 0 ? (size_t)g.k_units : kBT;
    const size_t codes_bytes = nblk * kTile, mm_bytes = nblk * units * 4;
    if (scratch_bytes < codes_bytes + mm_bytes) return fail(KVCOMP_ERR_CAPACITY, "scratch too small");
    hipStream_t s = static_cast<hipStream_t>(stream);
    uint8_t *dc = static_cast<uint8_t *>(d_scratch);
    uint16_t *dm = reinterpret_cast<uint16_t *>(dc + codes_bytes);
    HIP_TRY(launch_debug_codes(g, which, static_cast<const uint16_t *>(d_in), seq, seq / kBT, dc, dm, s));
    HIP_TRY(hipMemcpyAsync(h_codes, dc, codes_bytes, hipMemcpyDeviceToHost, s));
    HIP_TRY(hipMemcpyAsync(h_minmax, dm, mm_bytes, hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    return KVCOMP_OK;
}

kvcomp_status kvcomp_get_histogram(kvcomp_ctx *ctx, int which, uint32_t *h_hist256, void *stream) {
    if (!ctx || !h_hist256 || (which != 0 && which != 1)) return fail(KVCOMP_ERR_INVALID_ARG, "bad argument");
    if (!ctx->have_codebook) return fail(KVCOMP_ERR_STATE, "no codebook");
    (void)stream;
    // the host's copy from the last codebook build (the device histogram is cleared for the next one right after it
    // has been read)
    std::memcpy(h_hist256, ctx->h_hist + 256 * which, 256 * 4);
    return KVCOMP_OK;
}

kvcomp_status kvcomp_get_codebook(kvcomp_ctx *ctx, int which, uint8_t *h_len256, uint32_t *h_code256) {
    if (!ctx || !h_len256 || !h_code256 || (which != 0 && which != 1)) return fail(KVCOMP_ERR_INVALID_ARG, "bad argument");
    if (!ctx->have_codebook) return fail(KVCOMP_ERR_STATE, "no codebook");
    std::memcpy(h_len256, ctx->len[which], 256);
    std::memcpy(h_code256, ctx->code[which], 256 * sizeof(uint32_t));
    return KVCOMP_OK;
}

kvcomp_status kvcomp_get_block_entry(kvcomp_ctx *ctx, int which, int b, int h, int blk, uint32_t *h_off16,
                                     uint32_t *h_size16, void *stream) {
    if (!ctx || !h_off16 || !h_size16 || (which != 0 && which != 1)) return fail(KVCOMP_ERR_INVALID_ARG, "bad argument");
    const Geo &g = ctx->geo;
    if (b < 0 || b >= g.B || h < 0 || h >= g.H || blk < 0 || blk >= ctx->n_blocks)
        return fail(KVCOMP_ERR_INVALID_ARG, "block index out of range");
    BlockEntry e;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const BlockEntry *src = g.table + ((size_t)which * g.B * g.H + (size_t)b * g.H + h) * g.max_blocks + blk;
    HIP_TRY(hipMemcpyAsync(&e, src, sizeof(e), hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    *h_off16 = e.off16;
    *h_size16 = e.size16;
    return KVCOMP_OK;
}

kvcomp_status kvcomp_get_block(kvcomp_ctx *ctx, int which, int b, int h, int blk, void *h_buf, size_t cap,
                               size_t *h_bytes, void *stream) {
    if (!h_buf || !h_bytes) return fail(KVCOMP_ERR_INVALID_ARG, "NULL argument");
    uint32_t off16, size16;
    kvcomp_status st = kvcomp_get_block_entry(ctx, which, b, h, blk, &off16, &size16, stream);
    if (st) return st;
    const size_t bytes = (size_t)size16 * 16;
    *h_bytes = bytes;
    if (bytes > cap) return fail(KVCOMP_ERR_CAPACITY, "record has %zu bytes, buffer %zu", bytes, cap);
    if ((size_t)off16 + size16 > ctx->lay.payload_cap16) return fail(KVCOMP_ERR_STATE, "corrupt block entry");
    hipStream_t s = static_cast<hipStream_t>(stream);
    HIP_TRY(hipMemcpyAsync(h_buf, ctx->geo.payload + (size_t)off16 * 16, bytes, hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    return KVCOMP_OK;
}

kvcomp_status kvcomp_get_residual(kvcomp_ctx *ctx, int which, uint16_t *h_buf, int *h_n_res, void *stream) {
    if (!ctx || !h_buf || !h_n_res || (which != 0 && which != 1)) return fail(KVCOMP_ERR_INVALID_ARG, "bad argument");
    const Geo &g = ctx->geo;
    const size_t per_tok = (size_t)g.H * kD, per_b = (size_t)g.res_tokens * per_tok;
    const uint16_t *src = g.res + (size_t)g.B * per_b * which;
    const size_t first = (size_t)(g.res_tokens - ctx->res_head);  // slots res_head .. end of the ring come first
    hipStream_t s = static_cast<hipStream_t>(stream);
    for (int b = 0; b < g.B; b++) {
        HIP_TRY(hipMemcpyAsync(h_buf + b * per_b, src + b * per_b + ctx->res_head * per_tok, first * per_tok * 2,
                               hipMemcpyDeviceToHost, s));
        if (ctx->res_head)
            HIP_TRY(hipMemcpyAsync(h_buf + b * per_b + first * per_tok, src + b * per_b, ctx->res_head * per_tok * 2,
                                   hipMemcpyDeviceToHost, s));
    }
    HIP_TRY(hipStreamSynchronize(s));
    *h_n_res = ctx->n_res;
    return KVCOMP_OK;
}

static kvcomp_status decompress_impl(kvcomp_ctx *ctx, int which, void *d_out, int seq_stride, int tree_walk,
                                     void *stream) {
    if (!ctx || !d_out) return fail(KVCOMP_ERR_INVALID_ARG, "NULL argument");
    if (which != 0 && which != 1) return fail(KVCOMP_ERR_INVALID_ARG, "which must be 0 (K) or 1 (V)");
    if (!aligned16(d_out)) return fail(KVCOMP_ERR_INVALID_ARG, "d_out must be 16-byte aligned");
    const int tokens = ctx->n_blocks * kBT + ctx->n_res;
    if (seq_stride < tokens) return fail(KVCOMP_ERR_CAPACITY, "seq_stride %d below the %d tokens in the cache", seq_stride, tokens);
    if (ctx->n_blocks && !ctx->have_codebook) return fail(KVCOMP_ERR_STATE, "no codebook");
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (ctx->n_blocks) {  // the largest record may have grown through flushes since the last synchronising call
        kvcomp_status st = read_ctrl(ctx, s);
        if (st) return st;
        st = check_flags(ctx, s);
        if (st) return st;
        ctx->max_size16 = std::max(ctx->max_size16, ctx->h_ctrl->max_size16);
    }
    const int stage = (int)align_up((size_t)ctx->max_size16 * 16 + 16, 256);
    HIP_TRY(launch_decompress(ctx->geo, which, static_cast<uint16_t *>(d_out), ctx->n_blocks, ctx->res_head, ctx->n_res,
                              seq_stride, stage, tree_walk, s));
    return KVCOMP_OK;
}

kvcomp_status kvcomp_decompress(kvcomp_ctx *ctx, int which, void *d_out, int seq_stride, void *stream) {
    return decompress_impl(ctx, which, d_out, seq_stride, 0, stream);
}

kvcomp_status kvcomp_decompress_tree_walk(kvcomp_ctx *ctx, int which, void *d_out, int seq_stride, void *stream) {
    return decompress_impl(ctx, which, d_out, seq_stride, 1, stream);
}

kvcomp_status kvcomp_set_tuning(kvcomp_ctx *ctx, int n_splits, int stage_bytes, int waves_per_workgroup) {
    if (!ctx || n_splits < 0 || stage_bytes < 0 || waves_per_workgroup < 0) return fail(KVCOMP_ERR_INVALID_ARG, "bad argument");
    ctx->tune_splits = n_splits;
    ctx->tune_stage = stage_bytes;
    ctx->tune_waves = waves_per_workgroup;
    return KVCOMP_OK;
}

kvcomp_status kvcomp_set_profiling(kvcomp_ctx *ctx, int enable) {
    if (!ctx) return fail(KVCOMP_ERR_INVALID_ARG, "ctx is NULL");
    ctx->profiling = enable != 0;
    return KVCOMP_OK;
}

kvcomp_status kvcomp_get_profile(kvcomp_ctx *ctx, int *h_launches, double *h_total_ms) {
    if (!ctx || !h_launches || !h_total_ms) return fail(KVCOMP_ERR_INVALID_ARG, "NULL argument");
    kvcomp_status st = fold_profile(ctx);
    if (st) return st;
    *h_launches = ctx->prof_launches;
    *h_total_ms = ctx->prof_ms;
    ctx->prof_launches = 0;
    ctx->prof_ms = 0.0;
    return KVCOMP_OK;
}

size_t kvcomp_baseline_workspace_bytes(const kvcomp_config *cfg) {
    if (!cfg || cfg->batch < 1 || cfg->n_q_heads < 1) return 0;
    return (size_t)cfg->batch * cfg->n_q_heads * kMaxSplits * kPartialStride * 4 + (size_t)cfg->batch * cfg->n_kv_heads * 4;
}

kvcomp_status kvcomp_probe_read_stream(const void *d_buf, size_t bytes, void *d_sink, size_t *h_bytes_read, void *stream) {
    if (!d_buf || !d_sink || !h_bytes_read) return fail(KVCOMP_ERR_INVALID_ARG, "NULL argument");
    if (!aligned16(d_buf)) return fail(KVCOMP_ERR_INVALID_ARG, "d_buf must be 16-byte aligned");
    HIP_TRY(launch_read_stream(d_buf, bytes, static_cast<uint32_t *>(d_sink), h_bytes_read, static_cast<hipStream_t>(stream)));
    return KVCOMP_OK;
}

// arguments of the two comparison-kernel entry points; *n_splits receives the library's choice if it was 0
static kvcomp_status baseline_check(const kvcomp_config *cfg, const void *d_K, const void *d_V, int seq, const void *d_q,
                                    const float *d_out, int *n_splits) {
    if (!cfg || !d_K || !d_V || !d_q || !d_out) return fail(KVCOMP_ERR_INVALID_ARG, "NULL argument");
    if (!aligned16(d_K) || !aligned16(d_V) || !aligned16(d_q)) return fail(KVCOMP_ERR_INVALID_ARG, "pointers must be 16-byte aligned");
    if (cfg->batch < 1 || cfg->n_kv_heads < 1 || cfg->n_q_heads % cfg->n_kv_heads || cfg->head_dim != kD)
        return fail(KVCOMP_ERR_INVALID_ARG, "invalid configuration");
    const int G = cfg->n_q_heads / cfg->n_kv_heads;
    if (G != 1 && G != 2 && G != 4 && G != 8) return fail(KVCOMP_ERR_INVALID_ARG, "group size must be 1, 2, 4 or 8");
    if (seq < 1) return fail(KVCOMP_ERR_INVALID_ARG, "seq must be positive");
    if (*n_splits <= 0) {
        // measured best with one workgroup per CU (two for groups of 8 heads): every wave keeps 16 to 32 KiB in flight,
        // and more concurrent streams only cost locality in the memory system
        const int bh = cfg->batch * cfg->n_kv_heads;
        const int target = (G == 8 ? 2 : 1) * kCUs;
        *n_splits = std::min({(int)kMaxSplits, std::max(1, seq / 256), std::max(1, (target + bh - 1) / bh)});
    }
    *n_splits = std::max(1, std::min(*n_splits, (int)kMaxSplits));
    return KVCOMP_OK;
}

kvcomp_status kvcomp_baseline_fp16_attn(const kvcomp_config *cfg, const void *d_K, const void *d_V, int seq,
                                        const void *d_q, float scale, float *d_out, void *d_workspace,
                                        size_t workspace_bytes, int n_splits, void *stream) {
    if (!d_workspace) return fail(KVCOMP_ERR_INVALID_ARG, "NULL argument");
    kvcomp_status st = baseline_check(cfg, d_K, d_V, seq, d_q, d_out, &n_splits);
    if (st) return st;
    if (workspace_bytes < kvcomp_baseline_workspace_bytes(cfg)) return fail(KVCOMP_ERR_CAPACITY, "workspace too small");
    HIP_TRY(launch_baseline_attn(cfg->batch, cfg->n_kv_heads, cfg->n_q_heads, static_cast<const uint16_t *>(d_K),
                                 static_cast<const uint16_t *>(d_V), seq, static_cast<const uint16_t *>(d_q), scale, d_out,
                                 static_cast<float *>(d_workspace),
                                 reinterpret_cast<uint32_t *>(static_cast<float *>(d_workspace) +
                                                              (size_t)cfg->batch * cfg->n_q_heads * kMaxSplits * kPartialStride),
                                 n_splits, kMaxSplits, static_cast<hipStream_t>(stream)));
    return KVCOMP_OK;
}

kvcomp_status kvcomp_baseline_fp16_attn_noalloc(const kvcomp_config *cfg, const void *d_K, const void *d_V, int seq,
                                                const void *d_q, float scale, float *d_out, int n_splits, void *stream) {
    kvcomp_status st = baseline_check(cfg, d_K, d_V, seq, d_q, d_out, &n_splits);
    if (st) return st;
    uint32_t *tickets = nullptr;
    float *partials = nullptr;
    size_t max_tickets = 0, partial_bytes = 0;
    HIP_TRY(baseline_static_scratch(&tickets, &partials, &max_tickets, &partial_bytes));
    // the partials are laid out for the splits this launch really uses, not for the maximum
    const int used = baseline_splits(seq, n_splits);
    const size_t bh = (size_t)cfg->batch * cfg->n_kv_heads;
    const size_t need = (size_t)cfg->batch * cfg->n_q_heads * used * kPartialStride * sizeof(float);
    if (bh > max_tickets || need > partial_bytes)
        return fail(KVCOMP_ERR_CAPACITY,
                    "%zu (batch, kv head) pairs and %zu bytes of split partials (%d splits) exceed the static scratch "
                    "(%zu pairs, %zu bytes): use kvcomp_baseline_fp16_attn with a workspace, or fewer splits",
                    bh, need, used, max_tickets, partial_bytes);
    HIP_TRY(launch_baseline_attn(cfg->batch, cfg->n_kv_heads, cfg->n_q_heads, static_cast<const uint16_t *>(d_K),
                                 static_cast<const uint16_t *>(d_V), seq, static_cast<const uint16_t *>(d_q), scale, d_out,
                                 partials, tickets, n_splits, used, static_cast<hipStream_t>(stream)));
    return KVCOMP_OK;
}

}  // extern "C"
