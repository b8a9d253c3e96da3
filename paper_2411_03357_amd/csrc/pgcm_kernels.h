// Kernel declarations shared by the kernel file and the host side of the library.
#pragma once
#include <hip/hip_runtime.h>

#include "pgcm_types.h"

namespace pgcm {

__global__ void expand_key_kernel(KeyTables* kt, const uint32_t* key_words);

__global__ void aad_state_kernel(const KeyTables* kt, const ChunkDesc* chunks, uint32_t n,
                                 Block* aad_state);

template <bool kDecrypt>
__global__ void bulk_kernel(const KeyTables* kt, const ChunkDesc* chunks,
                            const uint32_t* item_chunk, uint32_t nitems, const uint8_t* ivs,
                            const Block* aad_state, Block* partials);

template <bool kDecrypt>
__global__ void finalize_kernel(const KeyTables* kt, const ChunkDesc* chunks, uint32_t n,
                                const uint8_t* ivs, const Block* aad_state, const Block* partials,
                                uint8_t* tags, uint8_t* ok);

__global__ void wipe_rejected_kernel(const ChunkDesc* chunks, uint32_t n, const uint8_t* ok);

}  // namespace pgcm
