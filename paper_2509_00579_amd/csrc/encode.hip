// Store side, second half (Section 3.2.2, Figure 4; Section 3.2.3): Huffman-encode quantized 2D blocks into
// one contiguous record each, place the records compactly and deterministically, and keep the fp16 buffer of
// the newest tokens.
//
// The paper reserves space with a global atomic offset, which makes the layout depend on execution order.  Here
// the same contiguous layout is produced in a fixed order by three steps:
//   1. size pass   : sum the code lengths of the block -> record size into the Block Offsets Array
//   2. place       : the sizes are scanned in (tensor, batch, head, block) order starting at the arena tail
//   3. write pass  : encode, write the record at its offset
// Blocks that the fp16 buffer sheds during decoding are quantized by both passes from the buffer (the store side runs
// once per token block while the fetch side runs every decode step, Section 3.3: the second read of 64 tokens is the
// cheaper trade against a staging copy of the records).  A prompt goes through the histogram pass first, which keeps
// the codes, the unit min/max and a histogram per block: its sizes come from the block histograms and its write pass
// reads the kept codes.
#include <algorithm>

#include "tile_quant.cuh"

namespace kvc {

constexpr int kCodeRow = kD + 4;  // padded row of the LDS code tile (bytes)
// Byte offset of token row t in the tile.  The second 32 rows start 64 bytes later: the two threads of a V slice read
// rows t and t + 32 of one column in the same instruction, and 32 rows of 33 words are a whole number of LDS bank
// rounds apart.
constexpr int kCodeTileBytes = kBT * kCodeRow + 64;
__device__ __forceinline__ int code_row(int t) { return t * kCodeRow + ((t >> 5) << 6); }

template <int WHICH>
struct Rec {
    static constexpr int n_slices = kSlices;
    static constexpr int parts = 2;  // threads per slice, 32 symbols each
    __device__ static int n_units(const Geo &g) { return WHICH == 0 ? g.k_units : kBT; }
    __device__ static int minmax_bytes(const Geo &g) { return WHICH == 0 ? g.k_minmax_bytes : kMinMaxBytesV; }
    __device__ static int hdr_bytes(const Geo &g) { return minmax_bytes(g) + 2 * kSlices; }
};

__device__ __forceinline__ uint32_t record_size16(int hdr_bytes, uint32_t total_bits) {
    const uint32_t bytes = (uint32_t)hdr_bytes + ((total_bits + 31u) >> 5) * 4u;
    return (bytes + 15u) >> 4;
}

// Sum over the workgroup (256 threads); result valid in every thread.  scratch: 4 words of LDS.
__device__ __forceinline__ uint32_t block_sum(uint32_t v, uint32_t *scratch, int tid) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m);
    __syncthreads();
    if ((tid & 63) == 0) scratch[tid >> 6] = v;
    __syncthreads();
    return scratch[0] + scratch[1] + scratch[2] + scratch[3];
}

// Codes and unit min/max that an earlier pass kept (launch_histogram with a workspace): where the write pass finds
// them instead of quantizing the input.  Blocks are numbered bh * blk_per_bh + j there.
struct Kept {
    const uint8_t *codes;    // [block][64][128]
    const uint32_t *minmax;  // [block][units] {min,max} fp16 pairs
    int blk_per_bh;
};
// ---- 1. size pass ------------------------------------------------------------------------------------------
template <int WHICH>
__global__ __launch_bounds__(256) void size_kernel(Geo g, const uint16_t *__restrict__ X, int seq_stride,
                                                    int n_blk_per_bh, int dst_blk0) {
    __shared__ QuantShared sh;
    __shared__ uint32_t enc[256];
    __shared__ uint32_t scratch[4];
    const int tid = threadIdx.x, blk = blockIdx.x;
    const int bh = blk / n_blk_per_bh, j = blk - bh * n_blk_per_bh;
    enc[tid] = enc_of(g, WHICH)[tid];
    TileRegs r;
    load_tile(X, seq_stride, g.H, bh / g.H, bh % g.H, j, tid, r);
    const bool bad = quantize_tile<WHICH>(r, sh, tid, g.two_eb[WHICH], g.n_sym[WHICH], g.k_units);  // has barriers: enc[] is visible after it
    uint32_t bits = 0;
#pragma unroll
    for (int i = 0; i < 4; i++)
#pragma unroll
        for (int k = 0; k < 8; k++) bits += enc[r.code[i][k]] >> 16;
    const uint32_t total = block_sum(bits, scratch, tid);
    if (tid == 0) {
        const uint32_t s16 = record_size16(Rec<WHICH>::hdr_bytes(g), total);
        g.table[((size_t)WHICH * g.B * g.H + bh) * g.max_blocks + dst_blk0 + j].size16 = s16;
    }
    if (bad) atomicOr(&g.ctrl->nonfinite, 1u);
}

// The size pass from the block histograms that the histogram pass kept ([block][256] u16, blocks numbered
// bh * kept_blk_per_bh + j): a record's payload is sum over the symbols of count x code length.  One wave per block,
// lane l takes symbols 4l .. 4l+3.
constexpr int kSizeBlocksPerWave = 4;
template <int WHICH>
__global__ __launch_bounds__(256) void size_from_hist_kernel(Geo g, const uint16_t *__restrict__ block_hist,
                                                              int kept_blk_per_bh, int n_blk_per_bh) {
    const int lane = threadIdx.x & 63;
    const int total = g.B * g.H * n_blk_per_bh;
    uint32_t len[4];
#pragma unroll
    for (int k = 0; k < 4; k++) len[k] = enc_of(g, WHICH)[4 * lane + k] >> 16;
    const int n_waves = gridDim.x * 4;
    for (int item = blockIdx.x * 4 + (threadIdx.x >> 6); item < total; item += n_waves) {
        const int bh = item / n_blk_per_bh, j = item - bh * n_blk_per_bh;
        const uint2 c = *reinterpret_cast<const uint2 *>(block_hist + ((size_t)bh * kept_blk_per_bh + j) * 256 + 4 * lane);
        uint32_t bits = (c.x & 0xffffu) * len[0] + (c.x >> 16) * len[1] + (c.y & 0xffffu) * len[2] + (c.y >> 16) * len[3];
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) bits += __shfl_xor(bits, m);
        if (lane == 0)
            g.table[((size_t)WHICH * g.B * g.H + bh) * g.max_blocks + j].size16 = record_size16(Rec<WHICH>::hdr_bytes(g), bits);
    }
}

// ---- 2. placement ------------------------------------------------------------------------------------------
// Items in order: tensor K then V (or one of them: the other's records are then placed by a launch of their own,
// K's first); inside a tensor (b,h) major, block minor.  Two launches over chunks of kPlaceChunk
// items, one workgroup of 256 threads per chunk (eight consecutive items per thread):
//   place_sum_kernel  : the sizes of a chunk summed -> place_sums[chunk]; the arena tail is copied to tail_base
//   place_scan_kernel : every workgroup adds up the chunk sums before its own (and all of them: what the placement
//                       needs in total), scans its own items from there and writes their offsets; the first
//                       workgroup moves the tail.
// Loads and stores of the table are coalesced through an LDS copy of the chunk.
constexpr int kPlaceThreads = 256, kPlacePerThread = kPlaceChunk / kPlaceThreads;
__device__ __forceinline__ int place_pad(int i) { return i + (i >> 5); }  // one spare word per 32: no bank conflicts

// tensors: 0 = K only, 1 = V only, 2 = K then V
struct PlaceItems {
    BlockEntry *table;
    int max_blocks, n_blk_per_bh, dst_blk0, n_items, row0;
    __device__ PlaceItems(const Geo &g, int n_blk_per_bh_, int dst_blk0_, int tensors)
        : table(g.table), max_blocks(g.max_blocks), n_blk_per_bh(n_blk_per_bh_), dst_blk0(dst_blk0_),
          n_items((tensors == 2 ? 2 : 1) * g.B * g.H * n_blk_per_bh_), row0(tensors == 1 ? g.B * g.H : 0) {}
    __device__ BlockEntry *entry(int i) const {  // row = tensor * B*H + (b*H + h)
        const int row = i / n_blk_per_bh, j = i - row * n_blk_per_bh;
        return &table[(size_t)(row0 + row) * max_blocks + dst_blk0 + j];
    }
};

__global__ __launch_bounds__(kPlaceThreads) void place_sum_kernel(Geo g, int n_blk_per_bh, int dst_blk0, int tensors) {
    __shared__ uint32_t wave_tot[kPlaceThreads / 64];
    const PlaceItems it(g, n_blk_per_bh, dst_blk0, tensors);
    const int tid = threadIdx.x, c0 = blockIdx.x * kPlaceChunk;
    uint32_t sum = 0;
#pragma unroll
    for (int k = 0; k < kPlacePerThread; k++) {
        const int i = c0 + k * kPlaceThreads + tid;
        if (i < it.n_items) sum += it.entry(i)->size16;
    }
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) sum += __shfl_xor(sum, m);
    if ((tid & 63) == 0) wave_tot[tid >> 6] = sum;
    __syncthreads();
    if (tid == 0) {
        uint32_t all = 0;
        for (int w = 0; w < kPlaceThreads / 64; w++) all += wave_tot[w];
        g.place_sums[blockIdx.x] = all;   // a chunk of 2048 records of at most 13 KiB: far below 2^32 units
        if (blockIdx.x == 0) g.ctrl->tail_base = g.ctrl->tail16;
    }
}

__global__ __launch_bounds__(kPlaceThreads) void place_scan_kernel(Geo g, int n_blk_per_bh, int dst_blk0, int tensors) {
    __shared__ uint32_t val[kPlaceChunk + kPlaceChunk / 32];
    __shared__ uint32_t wave_tot[kPlaceThreads / 64];
    __shared__ unsigned long long sums_s[2][kPlaceThreads / 64];
    const PlaceItems it(g, n_blk_per_bh, dst_blk0, tensors);
    const int tid = threadIdx.x, c0 = blockIdx.x * kPlaceChunk;
    // what the chunks before this one need, and what all chunks need
    unsigned long long before_me = 0, need = 0;
    for (int c = tid; c < (int)gridDim.x; c += kPlaceThreads) {
        const uint32_t v = g.place_sums[c];
        need += v;
        if (c < (int)blockIdx.x) before_me += v;
    }
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) {
        need += __shfl_xor(need, m);
        before_me += __shfl_xor(before_me, m);
    }
    if ((tid & 63) == 0) {
        sums_s[0][tid >> 6] = need;
        sums_s[1][tid >> 6] = before_me;
    }
    __syncthreads();
    need = 0;
    before_me = 0;
    for (int w = 0; w < kPlaceThreads / 64; w++) {
        need += sums_s[0][w];
        before_me += sums_s[1][w];
    }
    // The host only starts a placement that fits the arena.  A replay of a captured flush without the eager calls in
    // between (which the interface forbids) would advance the tail on every replay: a placement that would run past
    // the arena sets a fault bit, points its entries at the arena start (so that later readers stay in bounds) and
    // leaves the tail where it is; the write pass then writes nothing.
    const uint32_t tail0 = g.ctrl->tail_base;
    if ((unsigned long long)tail0 + need > (unsigned long long)g.payload_cap16) {
#pragma unroll
        for (int k = 0; k < kPlacePerThread; k++) {
            const int i = c0 + k * kPlaceThreads + tid;
            if (i < it.n_items) it.entry(i)->off16 = 0;
        }
        if (blockIdx.x == 0 && tid == 0) atomicOr(&g.ctrl->fault, kFaultArenaFull);
        return;
    }
    uint32_t biggest = 0;
#pragma unroll
    for (int k = 0; k < kPlacePerThread; k++) {
        const int i = c0 + k * kPlaceThreads + tid;
        const uint32_t s16 = i < it.n_items ? it.entry(i)->size16 : 0u;
        biggest = max(biggest, s16);
        val[place_pad(k * kPlaceThreads + tid)] = s16;
    }
    __syncthreads();
    uint32_t mine[kPlacePerThread], sum = 0;
#pragma unroll
    for (int k = 0; k < kPlacePerThread; k++) {
        mine[k] = val[place_pad(tid * kPlacePerThread + k)];
        sum += mine[k];
    }
    uint32_t inc = sum;  // inclusive scan of `sum` over the workgroup
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t o = __shfl_up(inc, d);
        if ((tid & 63) >= d) inc += o;
    }
    if ((tid & 63) == 63) wave_tot[tid >> 6] = inc;
    __syncthreads();
    uint32_t before = 0;
    for (int w = 0; w < (tid >> 6); w++) before += wave_tot[w];
    uint32_t at = tail0 + (uint32_t)before_me + before + inc - sum;
#pragma unroll
    for (int k = 0; k < kPlacePerThread; k++) {
        val[place_pad(tid * kPlacePerThread + k)] = at;
        at += mine[k];
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < kPlacePerThread; k++) {
        const int i = c0 + k * kPlaceThreads + tid;
        if (i < it.n_items) it.entry(i)->off16 = val[place_pad(k * kPlaceThreads + tid)];
    }
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) biggest = max(biggest, (uint32_t)__shfl_xor(biggest, m));
    if ((tid & 63) == 0 && biggest) atomicMax(&g.ctrl->max_size16, biggest);
    if (blockIdx.x == 0 && tid == 0) g.ctrl->tail16 = tail0 + (uint32_t)need;
}

static void launch_place(const Geo &g, int n_blk_per_bh, int dst_blk0, int tensors, hipStream_t s) {
    const int n_items = (tensors == 2 ? 2 : 1) * g.B * g.H * n_blk_per_bh;
    const int chunks = (n_items + kPlaceChunk - 1) / kPlaceChunk;
    hipLaunchKernelGGL(place_sum_kernel, dim3(chunks), dim3(kPlaceThreads), 0, s, g, n_blk_per_bh, dst_blk0, tensors);
    hipLaunchKernelGGL(place_scan_kernel, dim3(chunks), dim3(kPlaceThreads), 0, s, g, n_blk_per_bh, dst_blk0, tensors);
}

// ---- 3. write pass -----------------------------------------------------------------------------------------
template <int WHICH, bool KEPT>
__global__ __launch_bounds__(256) void write_kernel(Geo g, const uint16_t *__restrict__ X, int seq_stride,
                                                     int n_blk_per_bh, int dst_blk0, Kept kept) {
    using R = Rec<WHICH>;
    __shared__ QuantShared sh;
    __shared__ uint32_t enc[512];  // [0..256) first-bit-first, [256..512) last-bit-first
    __shared__ uint32_t wave_tot[4];
    __shared__ __attribute__((aligned(16))) uint8_t code_tile[kCodeTileBytes];
    __shared__ __attribute__((aligned(16))) uint32_t rec[(kMaxRecordBytes + 15) / 16 * 4];
    const int tid = threadIdx.x, blk = blockIdx.x;
    const int bh = blk / n_blk_per_bh, j = blk - bh * n_blk_per_bh;
    if (g.ctrl->fault & kFaultArenaFull) return;  // the placement found no room (uniform over the workgroup)
    enc[tid] = enc_of(g, WHICH)[tid];
    enc[256 + tid] = enc_of(g, WHICH)[256 + tid];
    static_assert(sizeof(rec) % 16 == 0, "whole 16-byte units");
    for (int i = tid; i < (int)(sizeof(rec) / 16); i += 256) reinterpret_cast<uint4 *>(rec)[i] = make_uint4(0, 0, 0, 0);
    // codes -> LDS tile (token-major rows, padded), header -> record
    const int c0 = tile_chan0(tid);
    if constexpr (KEPT) {  // the kept codes are already packed the way the tile wants them
        const uint8_t *src = kept.codes + ((size_t)bh * kept.blk_per_bh + j) * kTile;
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const int t = tile_token(tid, i);
            const uint2 pk = *reinterpret_cast<const uint2 *>(src + t * kD + c0);
            uint32_t *dst = reinterpret_cast<uint32_t *>(code_tile + code_row(t) + c0);
            dst[0] = pk.x;
            dst[1] = pk.y;
        }
    } else {
        TileRegs r;
        load_tile(X, seq_stride, g.H, bh / g.H, bh % g.H, j, tid, r);
        quantize_tile<WHICH>(r, sh, tid, g.two_eb[WHICH], g.n_sym[WHICH], g.k_units);
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const int t = tile_token(tid, i);
            uint32_t *dst = reinterpret_cast<uint32_t *>(code_tile + code_row(t) + c0);
            dst[0] = r.code[i][0] | (r.code[i][1] << 8) | (r.code[i][2] << 16) | (r.code[i][3] << 24);
            dst[1] = r.code[i][4] | (r.code[i][5] << 8) | (r.code[i][6] << 16) | (r.code[i][7] << 24);
        }
    }
    if (tid < R::n_units(g)) {
        if constexpr (KEPT) rec[tid] = kept.minmax[((size_t)bh * kept.blk_per_bh + j) * R::n_units(g) + tid];
        else rec[tid] = float_to_half_bits(sh.unit_mn[tid]) | (float_to_half_bits(sh.unit_mx[tid]) << 16);
    }
    __syncthreads();
    // Each thread encodes 32 symbols, half of one slice (Section 3.2.2 stage 2).  K: slice s = token s/2, channels
    // 64*(s%2)..+63 in channel order; V: slice s = channel s, tokens in order.  The first half of a slice is written
    // first-bit-first, the second half last-bit-first (it is decoded downwards from the slice end).
    const int slice = tid / R::parts, part = tid % R::parts;
    uint32_t sym[32];
    uint32_t bits = 0;
#pragma unroll
    for (int k = 0; k < 32; k++) {
        const int t = WHICH == 0 ? (slice >> 1) : 32 * part + k;
        const int c = WHICH == 0 ? kSliceLen * (slice & 1) + 32 * part + k : slice;
        sym[k] = enc[256 * part + code_tile[code_row(t) + c]];
        bits += sym[k] >> 16;
    }
    // stage 3: inclusive scan of the bit counts over the workgroup -> bit offset of every thread
    uint32_t inc = bits;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t o = __shfl_up(inc, d);
        if ((tid & 63) >= d) inc += o;
    }
    if ((tid & 63) == 63) wave_tot[tid >> 6] = inc;
    uint32_t slice_bits = bits;
#pragma unroll
    for (int m = 1; m < R::parts; m <<= 1) slice_bits += __shfl_xor(slice_bits, m);
    if (part == 0) reinterpret_cast<uint16_t *>(rec)[R::minmax_bytes(g) / 2 + slice] = (uint16_t)slice_bits;
    __syncthreads();
    uint32_t before = 0, total = 0;
#pragma unroll
    for (int w = 0; w < 4; w++) {
        if (w < (tid >> 6)) before += wave_tot[w];
        total += wave_tot[w];
    }
    // stage 4: aggregate all code words into one contiguous chunk in LDS.  Bit i of the chunk is bit (i % 32) of
    // word (i / 32); the table holds every code word in the bit order in which it enters the chunk.
    uint32_t *pay = rec + R::hdr_bytes(g) / 4;
    uint32_t pos = before + inc - bits;
    // Several code words at a time go into a 64-bit accumulator that starts at bit `fill` < 32 of word `word`: four
    // when the codebook's longest code word has at most 8 bits (4 x 8 + 31 pending bits fit), else two (2 x 12 + 31).
    // When the accumulator's low word is full it is ORed into the chunk.  No branch per group: a group that fills
    // nothing ORs a zero.  Neighbouring threads share the words at their borders, hence the atomic OR.
    static_assert(2 * kLutBits + 31 < 64, "a pair of code words behind 31 pending bits fits the accumulator");
    uint32_t word = pos >> 5, fill = pos & 31;
    uint32_t lo = 0, hi = 0;
    auto push = [&](uint32_t group, uint32_t len) {  // len <= 32
        const unsigned long long at = (unsigned long long)group << fill;
        lo |= (uint32_t)at;
        hi |= (uint32_t)(at >> 32);
        fill += len;
        const bool full = fill >= 32;
        atomicOr(&pay[word], full ? lo : 0u);
        lo = full ? hi : lo;
        hi = full ? 0u : hi;
        word += full ? 1u : 0u;
        fill &= 31u;
    };
    if (g.lut_bits[WHICH] <= 8) {  // uniform over the launch
#pragma unroll
        for (int k = 0; k < 32; k += 4) {
            const uint32_t l0 = sym[k] >> 16, l1 = l0 + (sym[k + 1] >> 16), l2 = l1 + (sym[k + 2] >> 16);
            const uint32_t four = (sym[k] & 0xffffu) | ((sym[k + 1] & 0xffffu) << l0) | ((sym[k + 2] & 0xffffu) << l1) |
                                  ((sym[k + 3] & 0xffffu) << l2);
            push(four, l2 + (sym[k + 3] >> 16));
        }
    } else {
#pragma unroll
        for (int k = 0; k < 32; k += 2) {
            const uint32_t l0 = sym[k] >> 16;
            push((sym[k] & 0xffffu) | ((sym[k + 1] & 0xffffu) << l0), l0 + (sym[k + 1] >> 16));
        }
    }
    if (fill) atomicOr(&pay[word], lo);
    __syncthreads();
    // stages 5-6: the offset was fixed by the placement; coalesced 16-byte stores of header + chunk + padding
    const BlockEntry e = g.table[((size_t)WHICH * g.B * g.H + bh) * g.max_blocks + dst_blk0 + j];
    const uint32_t n16 = record_size16(R::hdr_bytes(g), total);  // equals e.size16 by construction
    uint4 *dst = reinterpret_cast<uint4 *>(g.payload + (size_t)e.off16 * 16);
    const uint4 *src = reinterpret_cast<const uint4 *>(rec);
    if ((unsigned long long)e.off16 + e.size16 > (unsigned long long)g.payload_cap16) return;
    for (uint32_t i = tid; i < n16 && i < e.size16; i += 256) dst[i] = src[i];
}

hipError_t launch_encode(const Geo &g, const uint16_t *XK, const uint16_t *XV, int seq_stride, int n_blk_per_bh,
                         int dst_blk0, hipStream_t s) {
    const int total = g.B * g.H * n_blk_per_bh;
    if (total <= 0) return hipSuccess;
    const Kept none = {nullptr, nullptr, 0};
    hipLaunchKernelGGL(size_kernel<0>, dim3(total), dim3(256), 0, s, g, XK, seq_stride, n_blk_per_bh, dst_blk0);
    hipLaunchKernelGGL(size_kernel<1>, dim3(total), dim3(256), 0, s, g, XV, seq_stride, n_blk_per_bh, dst_blk0);
    launch_place(g, n_blk_per_bh, dst_blk0, 2, s);
    hipLaunchKernelGGL((write_kernel<0, false>), dim3(total), dim3(256), 0, s, g, XK, seq_stride, n_blk_per_bh, dst_blk0, none);
    hipLaunchKernelGGL((write_kernel<1, false>), dim3(total), dim3(256), 0, s, g, XV, seq_stride, n_blk_per_bh, dst_blk0, none);
    return hipGetLastError();
}

// The same for one tensor from what launch_histogram kept (kept_blk_per_bh blocks per (batch, head) there, of which the
// first n_blk_per_bh are encoded): sizes from the block histograms, placement of this tensor's records behind the
// arena tail, write pass from the kept codes.  K's records come before V's in the arena, so K can be placed and
// written as soon as its codebook is on the device, before V's sizes exist.
hipError_t launch_encode_kept(const Geo &g, int which, const uint8_t *codes, const uint32_t *mm, const uint16_t *block_hist,
                              int kept_blk_per_bh, int n_blk_per_bh, hipStream_t s) {
    const int total = g.B * g.H * n_blk_per_bh;
    if (total <= 0) return hipSuccess;
    const int grid = std::min((total + 4 * kSizeBlocksPerWave - 1) / (4 * kSizeBlocksPerWave), 2048);
    const Kept k = {codes, mm, kept_blk_per_bh};
    if (which == 0) {
        hipLaunchKernelGGL(size_from_hist_kernel<0>, dim3(grid), dim3(256), 0, s, g, block_hist, kept_blk_per_bh, n_blk_per_bh);
        launch_place(g, n_blk_per_bh, 0, 0, s);
        hipLaunchKernelGGL((write_kernel<0, true>), dim3(total), dim3(256), 0, s, g, nullptr, 0, n_blk_per_bh, 0, k);
    } else {
        hipLaunchKernelGGL(size_from_hist_kernel<1>, dim3(grid), dim3(256), 0, s, g, block_hist, kept_blk_per_bh, n_blk_per_bh);
        launch_place(g, n_blk_per_bh, 0, 1, s);
        hipLaunchKernelGGL((write_kernel<1, true>), dim3(total), dim3(256), 0, s, g, nullptr, 0, n_blk_per_bh, 0, k);
    }
    return hipGetLastError();
}

// ---- fp16 buffer of the newest tokens (Section 3.2.1) ------------------------------------------------------
// Buffer layout [tensor][B][res_tokens][H][128]: the same as an input tensor of res_tokens tokens, so a block of the
// buffer (64 consecutive slots) is compressed by the kernels above without a gather.  res_tokens is the maximum
// buffer size (a multiple of 64); the host uses the slots as a ring of 64-token blocks.
__global__ void copy_tail_kernel(Geo g, const uint16_t *__restrict__ XK, const uint16_t *__restrict__ XV, int seq,
                                 int first_tok, int n_tok) {
    const size_t per_tensor = (size_t)g.B * n_tok * g.H * 16;  // 16-byte chunks
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < 2 * per_tensor; i += stride) {
        const int which = i >= per_tensor;
        size_t r = i - which * per_tensor;
        const int ch = (int)(r % 16); r /= 16;
        const int h = (int)(r % g.H); r /= g.H;
        const int t = (int)(r % n_tok);
        const int b = (int)(r / n_tok);
        const uint16_t *X = which ? XV : XK;
        const uint4 v = *reinterpret_cast<const uint4 *>(X + (((size_t)b * seq + first_tok + t) * g.H + h) * kD + ch * 8);
        uint16_t *dst = g.res + (size_t)which * g.B * g.res_tokens * g.H * kD +
                        (((size_t)b * g.res_tokens + t) * g.H + h) * kD + ch * 8;
        *reinterpret_cast<uint4 *>(dst) = v;
    }
}

hipError_t launch_copy_tail(const Geo &g, const uint16_t *XK, const uint16_t *XV, int seq, int first_tok, int n_tok,
                            hipStream_t s) {
    if (n_tok <= 0) return hipSuccess;
    const size_t n = 2 * (size_t)g.B * n_tok * g.H * 16;
    const unsigned grid = (unsigned)((n + 255) / 256 > 2048 ? 2048 : (n + 255) / 256);
    hipLaunchKernelGGL(copy_tail_kernel, dim3(grid), dim3(256), 0, s, g, XK, XV, seq, first_tok, n_tok);
    return hipGetLastError();
}

// One new token per sequence: k_new, v_new [B][H][128] -> buffer slot `slot`.
__global__ void append_kernel(Geo g, const uint16_t *__restrict__ k_new, const uint16_t *__restrict__ v_new, int slot) {
    const int per_tensor = g.B * g.H * 16;
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= 2 * per_tensor) return;
    const int which = i >= per_tensor;
    int r = i - which * per_tensor;
    const int ch = r % 16; r /= 16;
    const int h = r % g.H;
    const int b = r / g.H;
    const uint16_t *src = (which ? v_new : k_new) + ((size_t)b * g.H + h) * kD + ch * 8;
    uint16_t *dst = g.res + (size_t)which * g.B * g.res_tokens * g.H * kD +
                    (((size_t)b * g.res_tokens + slot) * g.H + h) * kD + ch * 8;
    *reinterpret_cast<uint4 *>(dst) = *reinterpret_cast<const uint4 *>(src);
}

hipError_t launch_append(const Geo &g, const uint16_t *k_new, const uint16_t *v_new, int slot, hipStream_t s) {
    const int n = 2 * g.B * g.H * 16;
    hipLaunchKernelGGL(append_kernel, dim3((n + 255) / 256), dim3(256), 0, s, g, k_new, v_new, slot);
    return hipGetLastError();
}

}  // namespace kvc
