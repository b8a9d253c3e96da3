// A bitsliced AES counter-mode keystream kernel for gfx950: no table lookups, no LDS.
//
// It exists to MEASURE the one alternative to the table-driven round function of the batch
// kernels (AES rounds as lookups in LDS, pgcm_kernels.hip): the paper's transport needs nothing
// but throughput from its cipher (section 2.2: every transfer is an AES-GCM invocation; section
// 3: the cipher is the bottleneck), so the question is which formulation of FIPS-197's round
// this chip runs fastest.  Here a 32-bit register holds ONE bit position of ONE state byte for
// 32 counter blocks of a lane, so a wavefront instruction advances 2048 blocks at once; SubBytes
// is a Boolean circuit of three-input instructions (pgcm_bitsliced_gen.h, generated from the
// S-box's definition), ShiftRows is a renaming, MixColumns and AddRoundKey are XORs of planes.
// The batch calls do not use this kernel; pgcm_bitsliced_keystream runs it for tests (bit-exact
// against the oracle's block cipher) and for the benchmark that reports its cost.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pgcm_bitsliced_gen.h"
#include "pgcm_kernels.h"

namespace pgcm_bitsliced {

// mask (0 or ~0) of bit `bit` of byte `byte` (FIPS-197 order) of a round-key word loaded
// little-endian: uniform over the wavefront, so it lives in scalar registers
__device__ __forceinline__ uint32_t key_mask(uint32_t word, int byte, int bit) {
    return 0u - ((word >> (8 * byte + bit)) & 1u);
}

// 32 x 32 bit transpose of w[0..31] in place: afterwards bit i of w[j] is what bit j of w[i] was
template <int S, uint32_t M>
__device__ __forceinline__ void transpose_stage(uint32_t w[32]) {
#pragma unroll
    for (int i = 0; i < 32; ++i) {
        if ((i & S) == 0) {
            const uint32_t t = ((w[i] >> S) ^ w[i + S]) & M;
            w[i + S] ^= t;
            w[i] ^= t << S;
        }
    }
}
__device__ __forceinline__ void transpose32(uint32_t w[32]) {
    transpose_stage<16, 0x0000FFFFu>(w);
    transpose_stage<8, 0x00FF00FFu>(w);
    transpose_stage<4, 0x0F0F0F0Fu>(w);
    transpose_stage<2, 0x33333333u>(w);
    transpose_stage<1, 0x55555555u>(w);
}

// Lane L of the launch produces the keystream of counter blocks ctr_base + 32 L .. + 31 (counter
// field modulo 2^32; ctr_base must be a multiple of 32 so that the low five bits of a block's
// counter are its place in the lane's register).  out: 16 bytes per block, block order.
// Every lane of every workgroup must have all of its 32 blocks inside nblocks (host: nblocks is a
// multiple of 32 * blockDim.x and the grid covers it exactly).
template <int kRounds>
__global__ __launch_bounds__(64) void keystream_kernel(const pgcm::KeyTables* __restrict__ kt,
                                                       uint32_t iv0, uint32_t iv1, uint32_t iv2,
                                                       uint32_t ctr_base,
                                                       uint32_t* __restrict__ out) {
    const uint32_t lane_global = blockIdx.x * blockDim.x + threadIdx.x;
    const uint32_t hi = (ctr_base >> 5) + lane_global;     // counter bits 5 .. 31 of this lane
    uint32_t s[16][8];
    // round 0: the counter block (IV || be32(counter)) ^ round key 0, as planes
    {
        const uint32_t ivw[3] = {iv0, iv1, iv2};
#pragma unroll
        for (int b = 0; b < 12; ++b)
#pragma unroll
            for (int i = 0; i < 8; ++i)
                s[b][i] = key_mask(ivw[b / 4], b % 4, i) ^ key_mask(kt->rk[b / 4], b % 4, i);
        const uint32_t low[5] = {0xAAAAAAAAu, 0xCCCCCCCCu, 0xF0F0F0F0u, 0xFF00FF00u, 0xFFFF0000u};
#pragma unroll
        for (int k = 0; k < 32; ++k) {
            // counter bit k sits in byte 15 - k / 8 (big endian), bit k % 8
            const uint32_t plane = k < 5 ? low[k] : 0u - ((hi >> (k - 5)) & 1u);
            const int b = 15 - k / 8, i = k % 8;
            s[b][i] = plane ^ key_mask(kt->rk[3], b % 4, i);
        }
    }
#pragma unroll 1
    for (int r = 1; r < kRounds; ++r) {
#pragma unroll
        for (int b = 0; b < 16; ++b) sbox_planes(s[b]);
        uint32_t n[16][8];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            uint32_t a[64], o[32];
            const uint32_t kw = kt->rk[4 * r + c];
#pragma unroll
            for (int row = 0; row < 4; ++row)
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    a[8 * row + i] = s[row + 4 * ((c + row) % 4)][i];   // ShiftRows
                    a[32 + 8 * row + i] = key_mask(kw, row, i);
                }
            mixcolumn_addkey_planes(a, o);
#pragma unroll
            for (int row = 0; row < 4; ++row)
#pragma unroll
                for (int i = 0; i < 8; ++i) n[4 * c + row][i] = o[8 * row + i];
        }
#pragma unroll
        for (int b = 0; b < 16; ++b)
#pragma unroll
            for (int i = 0; i < 8; ++i) s[b][i] = n[b][i];
    }
    // last round: SubBytes, ShiftRows, AddRoundKey; then back from planes to blocks: word j of
    // the block (bytes 4j .. 4j + 3, little-endian load) has bit 8 k + i = plane [4j + k][i]
#pragma unroll
    for (int b = 0; b < 16; ++b) sbox_planes(s[b]);
    uint32_t* dst = out + (uint64_t)lane_global * 32 * 4;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        uint32_t w[32];
        const uint32_t kw = kt->rk[4 * kRounds + c];
#pragma unroll
        for (int row = 0; row < 4; ++row)
#pragma unroll
            for (int i = 0; i < 8; ++i)
                w[8 * row + i] = s[row + 4 * ((c + row) % 4)][i] ^ key_mask(kw, row, i);
        transpose32(w);   // now w[j] is word c of the lane's block j
#pragma unroll
        for (int j = 0; j < 32; ++j) dst[4 * j + c] = w[j];
    }
}

template __global__ void keystream_kernel<10>(const pgcm::KeyTables*, uint32_t, uint32_t, uint32_t,
                                              uint32_t, uint32_t*);
template __global__ void keystream_kernel<12>(const pgcm::KeyTables*, uint32_t, uint32_t, uint32_t,
                                              uint32_t, uint32_t*);
template __global__ void keystream_kernel<14>(const pgcm::KeyTables*, uint32_t, uint32_t, uint32_t,
                                              uint32_t, uint32_t*);

}  // namespace pgcm_bitsliced
