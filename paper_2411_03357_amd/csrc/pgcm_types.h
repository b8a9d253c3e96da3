// Structures shared by the host side of the library and its kernels.
#pragma once
#include <stdint.h>

namespace pgcm {

// A wavefront handles 64 consecutive 16-byte blocks (one 1 KiB "row") per step, one block per
// lane.  A segment is the unit of scheduling: one wavefront walks it row by row.
constexpr uint32_t kRowBlocks = 64;
constexpr uint32_t kSegBlocks = 4096;  // 64 KiB
constexpr uint32_t kSegBytes = kSegBlocks * 16;
constexpr uint32_t kWavesPerGroup = 16;
constexpr uint32_t kGroupThreads = kWavesPerGroup * 64;

// GHASH tables hold, for one constant C = H^(2^k), the products of C with every value of every
// nibble position of a block: entry [2 * byte + (0: high nibble, 1: low nibble)][value], 16 bytes
// each, 8 KiB per constant.
constexpr uint32_t kNibbleTableEntries = 32 * 16;
constexpr uint32_t kNumPowers = 19;   // H^(2^0) .. H^(2^18)
constexpr uint32_t kRowPower = 6;     // H^64: one row further along a lane's stripe
constexpr uint32_t kSegPower = 12;    // H^4096: one full segment further along a chunk
static_assert((1u << kRowPower) == kRowBlocks, "row power");
static_assert((1u << kSegPower) == kSegBlocks, "segment power");

struct alignas(16) Block {
    uint32_t w[4];  // bytes 4i..4i+3 of the block, loaded little-endian into w[i]
};

struct alignas(16) KeyTables {
    uint32_t rk[60];       // AES-256 round key words, little-endian loads of the FIPS-197 bytes
    uint32_t pad_[4];
    uint32_t te[4][256];   // round tables: te[r][x] = MixColumns contribution of S(x) in row r
    Block h;               // GHASH key H = E_K(0^128)
    Block ghash[kNumPowers][kNibbleTableEntries];
};

struct ChunkDesc {
    const uint8_t* src;
    uint8_t* dst;
    const uint8_t* aad;
    uint64_t len;
    uint32_t aad_len;
    uint32_t part_base;     // index of this chunk's first segment among all work items
    uint32_t nseg;          // number of segments (0 for an empty chunk)
    uint32_t first_blocks;  // blocks in segment 0; every later segment has kSegBlocks
};

}  // namespace pgcm
