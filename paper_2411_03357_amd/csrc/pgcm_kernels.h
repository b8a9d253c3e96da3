// Kernel declarations shared by the kernel file and the host side of the library.
#pragma once
#include <hip/hip_runtime.h>

#include "pgcm_types.h"

namespace pgcm {

__global__ void expand_key_kernel(KeyTables* kt, const uint32_t* key_words, uint32_t nk);

__global__ void j0_kernel(const KeyTables* kt, const ChunkDesc* chunks, const uint8_t* ivs,
                          uint32_t iv_len, uint32_t nchunks, Block* j0);

// kRounds: 10, 12 or 14; kMatrixHash: the GHASH multiplication of every row runs on the matrix
// cores (from KeyTables::row_matrix) instead of table lookups in LDS
template <bool kDecrypt, int kRounds, bool kMatrixHash>
__global__ void bulk_kernel(const KeyTables* kt, const ChunkDesc* chunks,
                            const uint32_t* unit_base, const uint32_t* coarse_map,
                            uint32_t nunits_total, uint32_t unit_power, uint32_t* counter,
                            const uint8_t* ivs, const Block* j0, Block* ekj0, Block* sets);

// The whole invocation of a few chunks in one launch: gridDim.x = sum of the chunks' ngroups.
// ekj0: one block per chunk; sets: one set (64 blocks) per workgroup; arrive: one word per
// chunk, zero on entry and left zero.
template <bool kDecrypt, int kRounds>
__global__ void swap_kernel(const KeyTables* kt, ArgBatch batch, const uint8_t* ivs, Block* ekj0,
                            Block* sets, uint32_t* arrive, uint8_t* tags, uint8_t* ok);

__global__ void clear_words_kernel(uint32_t* words, uint32_t n);

__global__ void fold_kernel(const KeyTables* kt, const FoldItem* items, uint32_t power,
                            Block* sets);

constexpr uint32_t kFoldTreeWaves = 16;
__global__ void fold_tree_kernel(const KeyTables* kt, const FoldItem* items, uint32_t power,
                                 Block* sets);

template <bool kDecrypt>
__global__ void final_kernel(const KeyTables* kt, const ChunkDesc* chunks, uint32_t nchunks,
                             const uint8_t* ivs, const Block* j0, const Block* ekj0,
                             const Block* sets, uint8_t* tags, uint8_t* ok, uint32_t unit_power,
                             uint32_t* counter, uint32_t chunks_per_group);
constexpr uint32_t kFinalWaves = 16;  // wavefronts of a final_kernel workgroup

constexpr uint32_t kSmallChunksPerGroup = 4;

// chunks of at most kSmallRowBytes each
template <bool kDecrypt, int kRounds>
__global__ void small_kernel(const KeyTables* kt, const ChunkDesc* chunks_host, uint32_t nchunks,
                             const uint8_t* ivs, uint32_t iv_len, uint8_t* tags, uint8_t* ok);

// chunks of at most kSmallChunkBytes each, one workgroup per chunk
constexpr uint32_t kSmallWideWaves = 8;
template <bool kDecrypt, int kRounds>
__global__ void small_wide_kernel(const KeyTables* kt, const ChunkDesc* chunks_host,
                                  uint32_t nchunks, const uint8_t* ivs, uint32_t iv_len,
                                  uint8_t* tags, uint8_t* ok);

__global__ void upload_kernel(uint4* dst, const uint4* src_host, uint32_t n16, uint32_t* clear);

}  // namespace pgcm

namespace pgcm_bitsliced {
// pgcm_bitsliced.hip: keystream of counter blocks by a bitsliced round function (measurement)
constexpr uint32_t kLaneBlocks = 32;   // counter blocks per lane: one per bit of a register
constexpr uint32_t kGroupLanes = 64;
template <int kRounds>
__global__ void keystream_kernel(const pgcm::KeyTables* kt, uint32_t iv0, uint32_t iv1,
                                 uint32_t iv2, uint32_t ctr_base, uint32_t* out);
}  // namespace pgcm_bitsliced
