/*
 * kvcomp.h -- C ABI of libkvcomp, a gfx950 (MI355X) implementation of the KVComp hot path:
 * block-wise error-bounded quantization + Huffman coding of a growing fp16 KV cache, and decode attention that
 * consumes the compressed cache directly (Huffman decode + dequantize + matrix-vector product fused in one kernel).
 *
 * General conventions
 *   - Plain C; every function returns a kvcomp_status (0 = OK, negative = error) unless stated otherwise;
 *     kvcomp_last_error() returns a thread-local, human readable description of the last failure.
 *   - Pointers named d_* are DEVICE pointers (HIP global memory), pointers named h_* are HOST pointers.
 *   - The caller owns all device memory, including the arena handed to kvcomp_create; the library allocates no
 *     device memory.  `stream` arguments are a hipStream_t passed as void* (NULL = the default stream).
 *   - The stream-ordered calls may be captured into a HIP graph (they launch kernels only).  A replay repeats the
 *     device work, not the host-side bookkeeping of the context (block and buffer counts): replay a captured sequence
 *     only from the cache state its capture started from, and bring the context back to a known state with eager
 *     calls (kvcomp_reset + kvcomp_compress_blocks) before using it eagerly again.
 *   - One context holds the cache of one transformer layer (Section 3: buffers and codebooks are per layer).
 *     A context must be used by one host thread at a time.
 *   - KV tensors are fp16, shape [batch, seq, n_kv_heads, 128] (the paper's [context_len, head_num, head_dim]
 *     of Section 2.1 with a batch dimension outermost), contiguous: element (b, t, h, c) at
 *     ((b*seq + t)*n_kv_heads + h)*128 + c.
 *   - A 2D block is 64 consecutive tokens x 128 channels of one (batch, head) (Section 3.2.1).
 */
#ifndef KVCOMP_H
#define KVCOMP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct kvcomp_ctx kvcomp_ctx; /* opaque, host object owned by the library */

typedef enum {
    KVCOMP_OK = 0,
    KVCOMP_ERR_INVALID_ARG = -1,
    KVCOMP_ERR_STATE = -2,     /* call order: e.g. compress before the codebook exists, cache not empty      */
    KVCOMP_ERR_CAPACITY = -3,  /* arena too small, or max_seq exceeded                                        */
    KVCOMP_ERR_HIP = -4,       /* a HIP runtime call failed                                                   */
    KVCOMP_ERR_NONFINITE = -5  /* an input held Inf or NaN (detected at the synchronising calls)              */
} kvcomp_status;

enum { KVCOMP_K = 0, KVCOMP_V = 1 };

typedef struct {
    int32_t batch;        /* sequences in the batch                                                           */
    int32_t n_kv_heads;   /* KV heads                                                                         */
    int32_t n_q_heads;    /* query heads; n_q_heads / n_kv_heads must be 1, 2, 4 or 8                         */
    int32_t head_dim;     /* must be 128                                                                      */
    int32_t block_tokens; /* must be 64                                                                       */
    int32_t max_seq;      /* capacity in tokens per sequence (prefill + appended)                             */
    float rel_eb_k;       /* relative error bound for K: |x - x'| <= rel_eb * (max - min) of the unit; the    */
    float rel_eb_v;       /*   paper's "relative quantization scale" (Section 4.2) is the bin width = 2*rel_eb */
    int32_t k_mode;       /* 0: K units are channels inside a block (Section 3.1.1); 1: one unit per K block
                             (BlockQuant, Section 4.2): the K record header then holds one {min,max} pair padded
                             to 16 bytes instead of 128 pairs */
    int32_t max_code_len; /* longest Huffman code word allowed, <= 12 and 2^max_code_len >= number of levels  */
                          /*   (0 = default 12); shorter words cost compression but decode faster            */
    int32_t buffer_tokens; /* capacity of the fp16 buffer of new tokens per sequence (Section 3.2.1; the "maximum
                             buffer size" of Section 4.2): a multiple of 64 in 64..4096, 0 = 64.  The newest tokens
                             stay uncompressed; the append that brings the buffer to buffer_tokens tokens cuts its
                             oldest 64 off as one block and compresses it, so a warm cache holds the newest
                             buffer_tokens-64 .. buffer_tokens-1 tokens as fp16 */
} kvcomp_config;

typedef struct {
    int64_t n_blocks;         /* compressed 2D blocks per (batch, head), same for K and V                     */
    int64_t n_res;            /* tokens in the fp16 buffer (0 .. buffer_tokens-1)                             */
    int64_t raw_bytes;        /* fp16 bytes of K and V for all tokens held                                    */
    int64_t record_bytes_k;   /* compressed records of K: headers + code words + padding                      */
    int64_t record_bytes_v;
    int64_t header_bytes;     /* part of the records: min/max pairs and per-slice bit counts                  */
    int64_t offsets_bytes;    /* Block Offsets Array entries in use (8 bytes per block)                       */
    int64_t residual_bytes;   /* fp16 bytes of the buffered tokens                                            */
    int64_t payload_bits_k;   /* sum of code-word bits                                                        */
    int64_t payload_bits_v;
    int64_t stored_bytes;     /* record_bytes_k + record_bytes_v + offsets_bytes + residual_bytes             */
    int64_t max_record_bytes; /* largest record so far                                                        */
    double compression_ratio; /* raw_bytes / stored_bytes                                                     */
} kvcomp_stats;

/* ---- life cycle ------------------------------------------------------------------------------------------ */

/* Device bytes the caller must provide for `cfg` (worst case over all inputs: every code word max_code_len bits).
 * Returns 0 if cfg is invalid. */
size_t kvcomp_arena_bytes(const kvcomp_config *cfg);

/* Create a context over a caller-owned device arena (256-byte aligned, >= kvcomp_arena_bytes(cfg), must outlive the
 * context and must not be touched by the caller while the context lives).  The arena is initialised on `stream`.
 * Errors: INVALID_ARG (bad cfg / alignment), CAPACITY (arena_bytes too small), HIP. */
kvcomp_status kvcomp_create(const kvcomp_config *cfg, void *d_arena, size_t arena_bytes, void *stream, kvcomp_ctx **out);
kvcomp_status kvcomp_destroy(kvcomp_ctx *ctx);

/* Drop all cached tokens (compressed blocks and buffered tokens).  keep_codebook != 0 keeps the Huffman codebooks
 * (they are built once at prefill and reused, Section 3).  Stream-ordered, does not synchronise. */
kvcomp_status kvcomp_reset(kvcomp_ctx *ctx, int keep_codebook, void *stream);

/* ---- the four calls of the hot path ---------------------------------------------------------------------- */

/* Store stage, step "histogram on the GPU, codebook once at prefill" (Section 3; Section 3.2): quantize the
 * floor(seq/64) full blocks of d_K and d_V (K: per channel inside each block, or per block with k_mode 1; V: per
 * token; Section 3.1.1, Section 4.2),
 * histogram the codes on the device, build one canonical Huffman codebook for K and one for V on the host and
 * upload the encode table and the decode lookup table.  d_K, d_V: device fp16 [batch, seq, n_kv_heads, 128],
 * read-only.  The cache must be empty (the codebooks are built once per prefill and reused, Section 3; new tables
 * would invalidate existing records): kvcomp_reset first.  SYNCHRONISES `stream` (the histogram crosses to the host,
 * as in the paper).
 * Errors: INVALID_ARG (seq < 64 or > max_seq), STATE (cache not empty), NONFINITE, HIP. */
kvcomp_status kvcomp_build_codebook(kvcomp_ctx *ctx, const void *d_K, const void *d_V, int seq, void *stream);

/* Store stage for the prompt (Section 3.2.2, Figure 4): quantize and Huffman-encode the oldest blocks of every
 * (batch, head), one record per 2D block placed compactly in the arena (K records in (b,h,block) order, then V
 * records), fill the Block Offsets Array; the newest tokens go to the fp16 buffer.  The split is the one that seq
 * calls of kvcomp_append_token would leave: floor(seq/64) blocks and seq%64 buffered tokens with the default
 * buffer, in general n = 0 if seq < buffer_tokens, else floor((seq - buffer_tokens)/64) + 1 blocks and seq - 64 n
 * buffered tokens.  The cache must be empty.  Inputs as for kvcomp_build_codebook.  SYNCHRONISES `stream` once at
 * the end (reads back the arena tail and the largest record size, and the non-finite flag).
 * Errors: STATE (no codebook / cache not empty), CAPACITY (seq > max_seq), NONFINITE, HIP. */
kvcomp_status kvcomp_compress_blocks(kvcomp_ctx *ctx, const void *d_K, const void *d_V, int seq, void *stream);

/* kvcomp_build_codebook followed by kvcomp_compress_blocks on the same tensors as one call (Section 3: the Store stage
 * at prefill), with ONE quantization pass instead of three: the histogram pass keeps the quantization codes (one byte
 * per value), the unit min/max and a histogram per block in d_workspace; the record sizes then come from the block
 * histograms and the write pass of the encoder reads the codes instead of loading and quantizing the fp16 input
 * again.  Same cache contents, byte for byte, as the two calls.  d_workspace: DEVICE, caller-owned, 16-byte aligned,
 * at least kvcomp_prefill_workspace_bytes(cfg, seq) bytes (about half the size of K and V together); it is scratch
 * and may be freed or reused once the call has returned.  The cache must be empty.
 * The host waits for the device three times (histogram of K, histogram of V; arena tail, largest record and flags at
 * the end); its codebook work for K runs while the device histograms V.
 * Errors: INVALID_ARG (seq < 64 or > max_seq, alignment), STATE (cache not empty), CAPACITY (workspace too small),
 * NONFINITE, HIP. */
size_t kvcomp_prefill_workspace_bytes(const kvcomp_config *cfg, int seq);
kvcomp_status kvcomp_prefill(kvcomp_ctx *ctx, const void *d_K, const void *d_V, int seq, void *d_workspace,
                             size_t workspace_bytes, void *stream);

/* Decode-phase store (Section 3.2.1, Section 3.2.3): append one token per sequence.  d_k_new, d_v_new: device fp16
 * [batch, n_kv_heads, 128].  The token is copied into the fp16 buffer; the call that fills the buffer's last slot
 * compresses the buffer's oldest 64 tokens as one block for every (batch, head) with the existing codebooks and
 * appends the records at the arena tail.
 * Stream-ordered, never synchronises.  Errors: STATE (no codebook), CAPACITY (max_seq reached), HIP.  An Inf or NaN
 * in an appended token is noticed when its block is compressed and reported (NONFINITE) by the next call that
 * synchronises: kvcomp_get_stats, kvcomp_decompress, kvcomp_compress_blocks, kvcomp_build_codebook. */
kvcomp_status kvcomp_append_token(kvcomp_ctx *ctx, const void *d_k_new, const void *d_v_new, void *stream);

/* Fetch stage (Section 3.3.2, Figure 1): one decode-attention step over the whole cache.  For every query head:
 * scores = scale * q.K'^T over all compressed blocks (Huffman decode + dequantize fused into the dot product) and
 * the buffered fp16 tokens, softmax over all of them, out = weights . V'.  Query head g reads KV head
 * g / (n_q_heads / n_kv_heads).  d_q: device fp16 [batch, n_q_heads, 128]; d_out: device fp32
 * [batch, n_q_heads, 128], caller-owned.  Stream-ordered, never synchronises.
 * Errors: STATE (empty cache), HIP. */
kvcomp_status kvcomp_attn_decode(kvcomp_ctx *ctx, const void *d_q, float scale, float *d_out, void *stream);

/* kvcomp_append_token followed by kvcomp_attn_decode (Section 3.2.3 then Section 3.3.2: the step of the decode
 * phase) in one call and, except for the token that fills the buffer and triggers the compression of a block, in
 * one kernel launch: the wave that owns the newest token's row reads it from d_k_new / d_v_new and stores it into
 * the fp16 buffer on the way.  Same arguments, same result definition, same errors as the two calls; d_k_new and
 * d_v_new must stay unchanged until the launch has run.  Stream-ordered, never synchronises. */
kvcomp_status kvcomp_append_attn_decode(kvcomp_ctx *ctx, const void *d_k_new, const void *d_v_new, const void *d_q,
                                        float scale, float *d_out, void *stream);

/* ---- metrics, parity and debug exports (these SYNCHRONISE `stream` and copy to HOST buffers) ------------- */

/* Also reports, once, what kernels flagged since the last synchronising call: NONFINITE (an appended token held Inf
 * or NaN), CAPACITY (a flush found the record arena full and wrote nothing: only a captured flush replayed without
 * the eager calls in between gets there). */
kvcomp_status kvcomp_get_stats(kvcomp_ctx *ctx, kvcomp_stats *h_out, void *stream);

/* Quantization codes and unit min/max of the full blocks of d_in (which = KVCOMP_K or KVCOMP_V) without touching the
 * cache.  h_codes: [batch*n_kv_heads*floor(seq/64)][64][128] bytes, blocks in (b,h,block) order, token-major tiles;
 * h_minmax_fp16: [blocks][units][2] fp16 bit patterns (units: 128 channels for K, or 1 with k_mode 1; 64 tokens for V).
 * d_scratch: device scratch of at least blocks*(8192 + 4*units) bytes. */
kvcomp_status kvcomp_debug_codes(kvcomp_ctx *ctx, int which, const void *d_in, int seq, void *d_scratch,
                                 size_t scratch_bytes, uint8_t *h_codes, uint16_t *h_minmax_fp16, void *stream);
/* The code histogram of tensor `which` that the last codebook was built from (256 counts, host memory).
 * Errors: STATE before the first codebook. */
kvcomp_status kvcomp_get_histogram(kvcomp_ctx *ctx, int which, uint32_t *h_hist256, void *stream);
kvcomp_status kvcomp_get_codebook(kvcomp_ctx *ctx, int which, uint8_t *h_len256, uint32_t *h_code256);
/* Block Offsets Array entry of block (b, h, blk): record offset and size in 16-byte units. */
kvcomp_status kvcomp_get_block_entry(kvcomp_ctx *ctx, int which, int b, int h, int blk, uint32_t *h_off16,
                                     uint32_t *h_size16, void *stream);
/* Copy the record of block (b, h, blk) to h_buf (capacity cap); *h_bytes receives its size. */
kvcomp_status kvcomp_get_block(kvcomp_ctx *ctx, int which, int b, int h, int blk, void *h_buf, size_t cap,
                               size_t *h_bytes, void *stream);
/* Copy the fp16 buffer to h_buf, layout [batch][buffer_tokens][n_kv_heads][128] with the oldest buffered token
 * first; *h_n_res receives the valid token count. */
kvcomp_status kvcomp_get_residual(kvcomp_ctx *ctx, int which, uint16_t *h_buf, int *h_n_res, void *stream);

/* Stand-alone decompression, the first stage of the multi-kernel pipeline that Section 4.3 compares the fused
 * kernel with: writes the whole cache of one tensor (which: 0 = K, 1 = V) as fp16, element (b, t, h, c) at
 * ((b*seq_stride + t)*n_kv_heads + h)*128 + c, for t < tokens in the cache: blocks reconstructed as
 * fp16(min + float(code)*width) (binary32 multiply and add, one rounding), then the buffered tokens unchanged.
 * d_out: DEVICE, caller-owned, 16-byte aligned, batch*seq_stride*n_kv_heads*128 fp16; seq_stride >= tokens
 * (KVCOMP_ERR_CAPACITY otherwise).  Synchronises the stream once (it reads the largest record size, and reports
 * the flags described at kvcomp_get_stats). */
kvcomp_status kvcomp_decompress(kvcomp_ctx *ctx, int which, void *d_out, int seq_stride, void *stream);

/* The same call with the decoder of Section 3.3.1 instead of the table decoder: a branch-free walk of the
 * array-based Huffman tree, one stream bit per step.  Same arguments, same output bit for bit; kept to compare the
 * two decoders on this hardware. */
kvcomp_status kvcomp_decompress_tree_walk(kvcomp_ctx *ctx, int which, void *d_out, int seq_stride, void *stream);

/* Tuning knobs for measurements (0 = library default): number of sequence splits of the fused kernel, LDS staging
 * bytes per wave (records larger than this are decoded straight from global memory), waves per workgroup of the
 * fused kernel (at most 16, 12, 8 for groups of 1-2, 4, 8 query heads). */
kvcomp_status kvcomp_set_tuning(kvcomp_ctx *ctx, int n_splits, int stage_bytes, int waves_per_workgroup);

/* Kernel timing with HIP events on the launch stream: when enabled, every kvcomp_attn_decode records an event pair
 * around its fused decode kernel.  kvcomp_get_profile synchronises, returns the number of timed launches and their
 * total duration in milliseconds since the last call, and resets the counters. */
kvcomp_status kvcomp_set_profiling(kvcomp_ctx *ctx, int enable);
kvcomp_status kvcomp_get_profile(kvcomp_ctx *ctx, int *h_launches, double *h_total_ms);

/* ---- the uncompressed comparison kernel (Section 4.3 compares against a plain fp16 matrix-vector product) - */

/* Decode attention on the uncompressed fp16 cache: same result definition as kvcomp_attn_decode with K' = K and
 * V' = V.  d_K, d_V: device fp16 [batch, seq, n_kv_heads, 128]; d_workspace: device scratch of at least
 * kvcomp_baseline_workspace_bytes(cfg) bytes that the caller ZERO-FILLS ONCE before the first call (it holds the
 * split tickets, which every launch leaves at zero again); two launches must not share it concurrently.
 * Stream-ordered.  n_splits 0 = default. */
size_t kvcomp_baseline_workspace_bytes(const kvcomp_config *cfg);
kvcomp_status kvcomp_baseline_fp16_attn(const kvcomp_config *cfg, const void *d_K, const void *d_V, int seq,
                                        const void *d_q, float scale, float *d_out, void *d_workspace,
                                        size_t workspace_bytes, int n_splits, void *stream);

/* kvcomp_baseline_fp16_attn for callers that cannot allocate or hand over a workspace (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): same arguments without the workspace, same result.  The split
 * tickets and split partials live in a static device array of the library, 4 MiB per GPU that the library runs on,
 * held until the process ends (64 KiB of tickets, the rest partials laid out for the splits the call really uses).
 * The call allocates nothing and launches one kernel.  Limits: batch * n_kv_heads <= 16384 and
 * batch * n_q_heads * splits * 520 bytes <= 4 MiB - 64 KiB, where splits = n_splits (0 = the library's choice)
 * after rounding the split length up to whole 64-token tiles; beyond that: KVCOMP_ERR_CAPACITY and nothing is
 * launched.  All calls on one GPU share the array: two of them must not overlap in time (on different streams, or
 * from two threads), or they race on the tickets and partials; calls on one stream are safe back to back.
 * Stream-ordered. */
kvcomp_status kvcomp_baseline_fp16_attn_noalloc(const kvcomp_config *cfg, const void *d_K, const void *d_V, int seq,
                                                const void *d_q, float scale, float *d_out, int n_splits, void *stream);

/* Measurement aid: one plain streaming read of d_buf (DEVICE, 16-byte aligned) with 16-byte loads, the bound for any
 * kernel that has to read an uncompressed cache of that size.  Up to 2048 workgroups read a whole number of 32 KiB pieces each,
 * as much as fits into `bytes` (*h_bytes_read receives the total; 0 = nothing launched) and writes nothing; d_sink: DEVICE, 4 bytes, needed only so
 * that the loads cannot be optimised away.  Stream-ordered; the caller times it. */
kvcomp_status kvcomp_probe_read_stream(const void *d_buf, size_t bytes, void *d_sink, size_t *h_bytes_read, void *stream);

const char *kvcomp_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* KVCOMP_H */
