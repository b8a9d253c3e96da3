// Structures shared by the host side of the library and its kernels.
#pragma once
#include <stddef.h>
#include <stdint.h>

namespace pgcm {

// A wavefront handles 64 consecutive 16-byte blocks (one 1 KiB "row") per step, one block per
// lane.  A unit is the piece of a chunk one wavefront walks in one go, and the granule of the
// dynamic schedule; units are counted back from the chunk's end, so only a chunk's first unit
// can be short.  A unit is 2^unit_power blocks.  Batches that do not fill the chip get the
// smallest size, from one row up, that still gives every unit a wavefront of its own, so that the
// batch spreads over as many wavefronts as there are and no unit waits.  Batches that do fill it
// get sixteen rows, handed out dynamically.  Larger units (up to 2^kMaxUnitPower blocks) can be
// forced for measurements.
constexpr uint32_t kRowBlocks = 64;
constexpr uint32_t kRowPower = 6;      // H^64: one row further along a lane's stripe
constexpr uint32_t kUnitPower = 10;    // the unit of the dynamic schedule: 1024 blocks = 16 KiB
constexpr uint32_t kMaxUnitPower = 20; // the largest unit that can be forced: 2^20 blocks = 16 MiB
constexpr uint32_t kMinUnitPower = kRowPower;
constexpr uint32_t kUnitBlocks = 1u << kUnitPower;
constexpr uint32_t kUnitBytes = kUnitBlocks * 16;
// wavefront slots of a 256-CU chip at sixteen per compute unit: a batch gets the smallest unit
// with which it has at most this many units (the full unit if none has)
constexpr uint32_t kWaveSlots = 4096;
constexpr uint32_t kWavesPerGroup = 16;
constexpr uint32_t kGroupThreads = kWavesPerGroup * 64;
static_assert((1u << kRowPower) == kRowBlocks, "row power");

// Every unit leaves a "partial set": the 64 per-lane GHASH sums of its rows (1 KiB).  Sets of one
// chunk are folded 32 at a time (again counted back from the end), level by level, until at most
// 32 remain; the per-chunk final step folds those and the 64 lanes.
constexpr uint32_t kFanPower = 5;
constexpr uint32_t kFan = 1u << kFanPower;
constexpr uint32_t kMaxLevels = 4;     // 2^22 units (the GCM length limit) / 32^4 <= 32
// The sets a fold level or the final step works on lie 2^(unit_power + 5 * level) blocks apart;
// that exponent must name one of the tables below.

// GHASH tables hold, for one constant C = H^(2^k), the products of C with every value of every
// nibble position of a block: entry [2 * byte + (0: high nibble, 1: low nibble)][value], 16 bytes
// each, 8 KiB per constant.
constexpr uint32_t kNibbleTableEntries = 32 * 16;
constexpr uint32_t kNumPowers = kUnitPower + kFanPower * kMaxLevels + 1;  // H^(2^0) .. H^(2^30)

// Multiplication by H^64 is linear over GF(2): a 128 x 128 bit matrix.  As operands of the 4-bit
// floating-point matrix instruction (an entry per nibble) it takes as much room as a nibble table.
constexpr uint32_t kRowMatrixWords = 128 * 128 / 8;
static_assert(kRowMatrixWords * 4 == kNibbleTableEntries * 16, "same room as a nibble table");

// The lane tree of the kernels that finish large chunks folds the 64 lanes in groups of four,
// three multiplications deep; beside H^(2^k) it needs the nibble tables of H^3, H^12 and H^48.
constexpr uint32_t kNumLanePowers = 3;

struct alignas(16) Block {
    uint32_t w[4];  // bytes 4i..4i+3 of the block, loaded little-endian into w[i]
};

struct alignas(16) KeyTables {
    uint32_t rk[60];       // round key words 0 .. 4 (rounds + 1) - 1, little-endian loads of the
                           // FIPS-197 bytes; the rest zero
    uint32_t rounds;       // Nr: 10, 12 or 14 for 128-, 192-, 256-bit keys (the paper's: 14)
    uint32_t pad_[3];
    uint32_t te[4][256];   // round tables: te[r][x] = MixColumns contribution of S(x) in row r
    Block h;               // GHASH key H = E_K(0^128)
    Block ghash[kNumPowers][kNibbleTableEntries];
    uint32_t row_matrix[kRowMatrixWords];  // multiplication by H^64 as matrix-core operands
    Block ghash_lane[kNumLanePowers][kNibbleTableEntries];  // nibble tables of H^3, H^12, H^48
};

struct alignas(16) ChunkDesc {
    const uint8_t* src;
    uint8_t* dst;
    const uint8_t* aad;
    uint64_t len;
    uint32_t aad_len;
    uint32_t unit_base;     // index of this chunk's first unit among all units = its set slot
    uint32_t nunits;        // 0 for an empty chunk
    uint32_t first_blocks;  // blocks in unit 0; every later unit has 2^unit_power
    uint32_t final_base;    // first set slot the final step folds
    uint32_t final_count;   // number of sets it folds: 1..32, or 0 for an empty chunk
    uint32_t final_power;   // log2 of the distance, in blocks, between consecutive such sets
    uint32_t index;         // the chunk's place in the caller's ivs, tags and ok arrays
};
static_assert(sizeof(ChunkDesc) == 64, "descriptor layout");

// One fold of up to 32 consecutive sets of a chunk into one set of the next level.
struct alignas(16) FoldItem {
    uint32_t in_base;   // first input slot
    uint32_t in_count;  // 1..32
    uint32_t out_slot;
    uint32_t pad_;
};

// A batch of few chunks that does not fill the chip (every unit gets a wavefront of its own) is
// done by ONE kernel, its descriptors travelling as kernel arguments: the paper's swaps arrive a
// few chunks at a time between synchronisations (section 5.1), and for them the time of a call
// counts, not the rate.  Every chunk gets workgroups of its own, sixteen units each, counted back
// from the chunk's end so that only its first workgroup can be short.
constexpr uint32_t kArgChunks = 24;
struct alignas(16) ArgChunk {
    const uint8_t* src;
    uint8_t* dst;
    const uint8_t* aad;
    uint64_t len;
    uint32_t aad_len;
    uint32_t nunits;        // 0 for an empty chunk
    uint32_t first_blocks;  // blocks in unit 0; every later unit has 2^unit_power
    uint32_t index;         // the chunk's place in the caller's ivs, tags and ok arrays
    uint32_t group_base;    // first workgroup of the chunk = its first set slot
    uint32_t ngroups;       // max(1, ceil(nunits / 16))
    uint32_t pad_[2];
};
static_assert(sizeof(ArgChunk) == 64, "argument layout");
struct alignas(16) ArgBatch {
    uint32_t nchunks;
    uint32_t unit_power;
    uint32_t pad_[2];
    ArgChunk c[kArgChunks];
};

// A batch whose chunks are all at most this long takes the small-transfer path: one kernel (the
// paper's non-swap transfers are usually < 8 KB, section 4.2): eight rows of 64 blocks.
constexpr uint64_t kSmallChunkBytes = 8192;
// ... and when they are all at most this long (63 blocks: one row together with "block -1") the
// kernel is the one with a wavefront per chunk
constexpr uint64_t kSmallRowBytes = 1008;
// The kernel with a workgroup per chunk is there for the latency of a few transfers; a batch of
// more chunks than this (two rounds of resident workgroups; measured crossover) longer than one
// row goes through the unit schedule instead, which gets more chunks per second out of the chip.
constexpr size_t kSmallWideMaxChunks = 512;

// Items of the dynamic schedule are grabbed from a counter; to find an item's chunk a wavefront
// starts at coarse_map[item >> kCoarseShift] and walks unit_base[] forward.
constexpr uint32_t kCoarseShift = 4;

}  // namespace pgcm
