// Sizes of the record format and of the decode tables: plain constants, no HIP types, so that the host-only logic
// (host_logic.h) compiles with any C++ compiler.
#pragma once

#include <stdint.h>

namespace kvc {

constexpr int kD = 128;        // head_dim
constexpr int kBT = 64;        // tokens per 2D block
constexpr int kTile = kD * kBT;  // symbols per block
constexpr int kLutBits = 12;   // decode table index width = longest code word allowed
constexpr int kLutSize = 1 << kLutBits;
constexpr int kMaxBufferTokens = 4096;  // largest fp16 buffer of new tokens per sequence

// Record layout (Section 3.2.2: per-thread bit counts + one contiguous chunk per 2D block):
//   K: [128 x {min,max} fp16][128 x u16 slice bits][payload words][pad to 16 B]
//   V: [ 64 x {min,max} fp16][128 x u16 slice bits][payload words][pad to 16 B]
// Every block has 128 slices of 64 symbols: K slice s = token s/2, channels 64*(s%2)..+63; V slice s = channel s,
// tokens 0..63.  A decoding lane owns two consecutive slices (K: one token; V: channels 2*lane, 2*lane+1).
// A slice is written from both ends: symbols 0..31 first-bit-first upwards from its start, symbols 32..63
// last-bit-first after them, so that reading downwards from the slice end yields symbols 63..32 first-bit-first.
// Each slice is thus two independent decode chains; its end needs no extra offset (it is the next slice's start).
constexpr int kSlices = 128;
constexpr int kSliceLen = 64;
constexpr int kMinMaxBytesK = 4 * kD;
constexpr int kMinMaxBytesV = 4 * kBT;
constexpr int kHdrBytesK = kMinMaxBytesK + 2 * kSlices;   // 768 (channel-wise units; BlockQuant: 16 + 256)
constexpr int kHdrBytesV = kMinMaxBytesV + 2 * kSlices;   // 512
constexpr int kMaxPayloadBytes = kTile * kLutBits / 8;  // 12288
constexpr int kMaxRecordBytes = kHdrBytesK + kMaxPayloadBytes + 16;

// Block Offsets Array entry (Section 3): where the record of a 2D block lives, in 16-byte units from the start of
// the payload arena, and how long it is.
struct BlockEntry {
    uint32_t off16;
    uint32_t size16;
};

// The tables of one tensor's codebook sit together, in the arena and in the host's staging block, so that one copy
// uploads them: [encode table 2 x 256 u32][decode table 4096 u16][tree 256 x 2 i16][pair table 4096 u32]
constexpr int kPairTableEntries = 1 << 12;
constexpr int kTabEncOff = 0;
constexpr int kTabLutOff = kTabEncOff + 2 * 256 * 4;
constexpr int kTabTreeOff = kTabLutOff + kLutSize * 2;
constexpr int kTabPairOff = kTabTreeOff + 256 * 2 * 2;
constexpr int kTensorTablesBytes = kTabPairOff + kPairTableEntries * 4;

// The placement of records walks the Block Offsets Array in chunks of this many entries, one workgroup per chunk.
constexpr int kPlaceChunk = 2048;

constexpr int kPartialStride = kD + 2;  // o[128], m, l
constexpr int kMaxSplits = 128;

}  // namespace kvc
