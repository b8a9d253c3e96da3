// HIP kernels for batched AES-GCM on gfx950 (MI355X).
//
// What is computed is the AES-GCM transform the paper's transport applies to every transfer
// (paper sections 2.2 and 4.1), i.e. FIPS-197 AES-256 in the GCM mode of NIST SP 800-38D with a
// 96-bit IV; the other two key lengths and other IV lengths are served by the same kernels
// (round count as a template parameter, pre-counter blocks hashed beforehand).  How:
//   * AES rounds read four 1 KiB round tables, each replicated 32 times in LDS so that lane l
//     always reads bank l % 32: table lookups never collide, whatever the data.  AddRoundKey is
//     folded into forming the next round's lookup addresses (one SDWA XOR per state byte).
//   * GHASH multiplies by fixed powers of H with 4-bit tables (Shoup).  In the bulk kernel the
//     row power H^64 sits in LDS and its thirty-two lookups are spread over the AES rounds;
//     as an alternative the same multiplication runs on the matrix cores, as a product with a
//     128 x 128 matrix over GF(2) (GhashRowMatrix).
//   * One wavefront walks one unit (1 to 16 KiB of one chunk, the size chosen per batch) in rows
//     of 64 blocks, one block per lane, 16-byte coalesced loads and stores, ciphertext hashed
//     from registers.  Wavefront w starts with unit w; what is left is handed out by a
//     device-side counter.  Each unit leaves 64 per-lane hash sums; fold kernels (a chain per
//     wavefront, or a tree per workgroup when there are few) and the final kernel combine them
//     per chunk (powers of H from tables; the 64 lanes are folded in groups of four).
//   * A batch of short chunks only is done by one kernel, a wavefront per chunk.
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <type_traits>

#include "pgcm_kernels.h"

namespace pgcm {

// ------------------------------------------------------------------------------------------
// S-box, generated at compile time from its definition (FIPS-197 5.1.1): inverse in
// GF(2^8) mod x^8+x^4+x^3+x+1, then the affine map.
namespace {

constexpr uint8_t xtime(uint8_t a) { return (uint8_t)((a << 1) ^ ((a & 0x80) ? 0x1B : 0)); }

constexpr uint8_t mul8(uint8_t a, uint8_t b) {
    uint8_t p = 0;
    for (int i = 0; i < 8; ++i) {
        if (b & (1 << i)) p ^= a;
        a = xtime(a);
    }
    return p;
}

constexpr uint8_t inv8(uint8_t a) {
    // a^254: the inverse of every non-zero element, and 0 for 0
    uint8_t r = 1, s = a;
    for (int bit = 1; bit < 8; ++bit) {
        s = mul8(s, s);    // a^(2^bit)
        r = mul8(r, s);
    }
    return r;              // a^(2+4+...+128) = a^254
}

constexpr uint8_t rotl8(uint8_t v, int k) { return (uint8_t)((v << k) | (v >> (8 - k))); }

struct SboxTable {
    uint8_t v[256];
};

constexpr SboxTable make_sbox() {
    SboxTable t{};
    for (int x = 0; x < 256; ++x) {
        uint8_t b = inv8((uint8_t)x);
        t.v[x] = (uint8_t)(b ^ rotl8(b, 1) ^ rotl8(b, 2) ^ rotl8(b, 3) ^ rotl8(b, 4) ^ 0x63);
    }
    return t;
}

__device__ const SboxTable kSbox = make_sbox();
static_assert(make_sbox().v[0x00] == 0x63 && make_sbox().v[0x53] == 0xED, "S-box");

// ------------------------------------------------------------------------------------------
// GF(2^128) in GCM's bit order (SP 800-38D 6.3): bit 0 of a block is the top bit of byte 0.
// For shifting, a block is held as two big-endian 64-bit halves.
struct Gf {
    uint64_t hi, lo;
};

__device__ __forceinline__ uint32_t bswap32(uint32_t v) { return __builtin_bswap32(v); }

__device__ __forceinline__ Gf gf_from_block(const Block& b) {
    Gf g;
    g.hi = ((uint64_t)bswap32(b.w[0]) << 32) | bswap32(b.w[1]);
    g.lo = ((uint64_t)bswap32(b.w[2]) << 32) | bswap32(b.w[3]);
    return g;
}

__device__ __forceinline__ Block gf_to_block(const Gf& g) {
    Block b;
    b.w[0] = bswap32((uint32_t)(g.hi >> 32));
    b.w[1] = bswap32((uint32_t)g.hi);
    b.w[2] = bswap32((uint32_t)(g.lo >> 32));
    b.w[3] = bswap32((uint32_t)g.lo);
    return b;
}

// bit-serial product (SP 800-38D algorithm 1); used for set-up only
__device__ Gf gf_mul_bits(const Gf& x, const Gf& y) {
    Gf z{0, 0}, v = y;
    for (int i = 0; i < 128; ++i) {
        uint64_t bit = (i < 64) ? (x.hi >> (63 - i)) & 1 : (x.lo >> (127 - i)) & 1;
        uint64_t m = 0 - bit;
        z.hi ^= v.hi & m;
        z.lo ^= v.lo & m;
        uint64_t carry = 0 - (v.lo & 1);
        v.lo = (v.lo >> 1) | (v.hi << 63);
        v.hi = (v.hi >> 1) ^ (carry & 0xE100000000000000ull);
    }
    return z;
}

// a ^ b ^ c in one instruction (gfx950's three-input bitwise op, truth table 0x96)
__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c) {
    return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);
}

__device__ __forceinline__ void block_xor(Block& a, const Block& b) {
    a.w[0] ^= b.w[0];
    a.w[1] ^= b.w[1];
    a.w[2] ^= b.w[2];
    a.w[3] ^= b.w[3];
}

// X * C from C's nibble table in global memory: 32 lookups of 16 bytes
__device__ Block gf_mul_table(const Block* __restrict__ tbl, const Block& x) {
    Block z{{0, 0, 0, 0}};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            uint32_t byte = (x.w[i] >> (8 * k)) & 0xFF;
            uint32_t pos = 2 * (4 * i + k);
            block_xor(z, tbl[pos * 16 + (byte >> 4)]);
            block_xor(z, tbl[(pos + 1) * 16 + (byte & 15)]);
        }
    }
    return z;
}

// ------------------------------------------------------------------------------------------
// AES block encryption from tables in global memory (set-up, J0, not the bulk path)
__device__ __forceinline__ uint32_t byte_of(uint32_t w, int k) { return (w >> (8 * k)) & 0xFF; }

__device__ void aes_block_global(const KeyTables* __restrict__ kt, uint32_t s[4]) {
    const uint32_t* rk = kt->rk;
    const int nr = (int)kt->rounds;
    uint32_t a0 = s[0] ^ rk[0], a1 = s[1] ^ rk[1], a2 = s[2] ^ rk[2], a3 = s[3] ^ rk[3];
    for (int r = 1; r < nr; ++r) {
        uint32_t t0 = kt->te[0][byte_of(a0, 0)] ^ kt->te[1][byte_of(a1, 1)] ^
                      kt->te[2][byte_of(a2, 2)] ^ kt->te[3][byte_of(a3, 3)] ^ rk[4 * r + 0];
        uint32_t t1 = kt->te[0][byte_of(a1, 0)] ^ kt->te[1][byte_of(a2, 1)] ^
                      kt->te[2][byte_of(a3, 2)] ^ kt->te[3][byte_of(a0, 3)] ^ rk[4 * r + 1];
        uint32_t t2 = kt->te[0][byte_of(a2, 0)] ^ kt->te[1][byte_of(a3, 1)] ^
                      kt->te[2][byte_of(a0, 2)] ^ kt->te[3][byte_of(a1, 3)] ^ rk[4 * r + 2];
        uint32_t t3 = kt->te[0][byte_of(a3, 0)] ^ kt->te[1][byte_of(a0, 1)] ^
                      kt->te[2][byte_of(a1, 2)] ^ kt->te[3][byte_of(a2, 3)] ^ rk[4 * r + 3];
        a0 = t0, a1 = t1, a2 = t2, a3 = t3;
    }
    const uint8_t* S = kSbox.v;
    auto last = [&](uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3) {
        return (uint32_t)S[byte_of(c0, 0)] | ((uint32_t)S[byte_of(c1, 1)] << 8) |
               ((uint32_t)S[byte_of(c2, 2)] << 16) | ((uint32_t)S[byte_of(c3, 3)] << 24);
    };
    s[0] = last(a0, a1, a2, a3) ^ rk[4 * nr + 0];
    s[1] = last(a1, a2, a3, a0) ^ rk[4 * nr + 1];
    s[2] = last(a2, a3, a0, a1) ^ rk[4 * nr + 2];
    s[3] = last(a3, a0, a1, a2) ^ rk[4 * nr + 3];
}

__device__ __forceinline__ uint32_t sub_word(uint32_t w) {
    const uint8_t* S = kSbox.v;
    return (uint32_t)S[w & 0xFF] | ((uint32_t)S[(w >> 8) & 0xFF] << 8) |
           ((uint32_t)S[(w >> 16) & 0xFF] << 16) | ((uint32_t)S[w >> 24] << 24);
}

}  // namespace

// ------------------------------------------------------------------------------------------
// Key set-up: key schedule (FIPS-197 5.2), round tables, H and the nibble tables of H^(2^k).
// One workgroup; `key_words` are the key bytes as nk = 4, 6 or 8 little-endian words.
__global__ __launch_bounds__(1024) void expand_key_kernel(KeyTables* __restrict__ kt,
                                                          const uint32_t* __restrict__ key_words,
                                                          uint32_t nk) {
    __shared__ Gf powers[kNumPowers];
    __shared__ Gf lane_powers[kNumLanePowers];
    const uint32_t tid = threadIdx.x;

    // round tables: te[0][x] = (2s, s, s, 3s) in bytes 0..3, te[r] = te[0] rotated left by 8r bits
    for (uint32_t x = tid; x < 256; x += blockDim.x) {
        uint32_t s = kSbox.v[x];
        uint32_t s2 = xtime((uint8_t)s), s3 = s2 ^ s;
        uint32_t t0 = s2 | (s << 8) | (s << 16) | (s3 << 24);
        kt->te[0][x] = t0;
        kt->te[1][x] = (t0 << 8) | (t0 >> 24);
        kt->te[2][x] = (t0 << 16) | (t0 >> 16);
        kt->te[3][x] = (t0 << 24) | (t0 >> 8);
    }
    if (tid == 0) {
        const uint32_t nr = nk + 6, nwords = 4 * (nr + 1);
        uint32_t w[60];
        for (uint32_t i = 0; i < 60; ++i) w[i] = 0;
        for (uint32_t i = 0; i < nk; ++i) w[i] = key_words[i];
        uint32_t rcon = 1;
        for (uint32_t i = nk; i < nwords; ++i) {
            uint32_t t = w[i - 1];
            if (i % nk == 0) {
                t = sub_word((t >> 8) | (t << 24)) ^ rcon;  // RotWord on little-endian bytes
                rcon = xtime((uint8_t)rcon);
            } else if (nk > 6 && i % nk == 4) {
                t = sub_word(t);
            }
            w[i] = w[i - nk] ^ t;
        }
        for (uint32_t i = 0; i < 60; ++i) kt->rk[i] = w[i];
        kt->rounds = nr;
        for (int i = 0; i < 3; ++i) kt->pad_[i] = 0;
    }
    __threadfence();
    __syncthreads();
    if (tid == 0) {
        uint32_t z[4] = {0, 0, 0, 0};
        aes_block_global(kt, z);
        Block h{{z[0], z[1], z[2], z[3]}};
        kt->h = h;
        Gf p = gf_from_block(h);
        powers[0] = p;
        for (uint32_t k = 1; k < kNumPowers; ++k) {
            p = gf_mul_bits(p, p);
            powers[k] = p;
        }
        lane_powers[0] = gf_mul_bits(powers[1], powers[0]);  // H^3
        lane_powers[1] = gf_mul_bits(powers[3], powers[2]);  // H^12
        lane_powers[2] = gf_mul_bits(powers[5], powers[4]);  // H^48
    }
    __syncthreads();
    for (uint32_t e = tid; e < kNumPowers * kNibbleTableEntries; e += blockDim.x) {
        uint32_t k = e / kNibbleTableEntries, idx = e % kNibbleTableEntries;
        uint32_t pos = idx / 16, val = idx % 16;
        uint32_t byte = pos / 2;
        uint32_t bits = (pos & 1) ? val : (val << 4);
        Block x{{0, 0, 0, 0}};
        x.w[byte / 4] = bits << (8 * (byte % 4));
        kt->ghash[k][idx] = gf_to_block(gf_mul_bits(gf_from_block(x), powers[k]));
    }
    for (uint32_t e = tid; e < kNumLanePowers * kNibbleTableEntries; e += blockDim.x) {
        uint32_t k = e / kNibbleTableEntries, idx = e % kNibbleTableEntries;
        uint32_t pos = idx / 16, val = idx % 16;
        uint32_t byte = pos / 2;
        uint32_t bits = (pos & 1) ? val : (val << 4);
        Block x{{0, 0, 0, 0}};
        x.w[byte / 4] = bits << (8 * (byte % 4));
        kt->ghash_lane[k][idx] = gf_to_block(gf_mul_bits(gf_from_block(x), lane_powers[k]));
    }

    // Multiplication by H^64 as a 128 x 128 matrix over GF(2), laid out as operands of the
    // 4-bit floating-point matrix instruction (see GhashRowMatrix): cols[b] = x^b * H^64 for the
    // block whose only set bit is bit b % 32 of word b / 32.
    __shared__ Block cols[128];
    if (tid < 128) {
        Block x{{0, 0, 0, 0}};
        x.w[tid / 32] = 1u << (tid % 32);
        cols[tid] = gf_to_block(gf_mul_bits(gf_from_block(x), powers[kRowPower]));
    }
    __syncthreads();
    for (uint32_t e = tid; e < kRowMatrixWords; e += blockDim.x) {
        const uint32_t r = e % 4, lane = (e / 4) % 64, ks = (e / 256) % 2, mt = e / 512;
        // the operand row this lane holds, the product bit it makes, the operand quarter
        const uint32_t ml = lane % 32, h = lane / 32, reg = 4 * (ml / 8) + ml % 4;
        const uint32_t word = 2 * ((ml / 4) % 2) + mt / 2, bit = 16 * (reg / 8) + 8 * (mt % 2) + reg % 8;
        uint32_t v = 0;
        for (uint32_t j = 0; j < 8; ++j) {
            const uint32_t in = 32 * r + 4 * j + 2 * ks + h;
            if ((cols[in].w[word] >> bit) & 1u) v |= 0x2u << (4 * j);  // 1.0 in e2m1
        }
        kt->row_matrix[e] = v;
    }
}

// ------------------------------------------------------------------------------------------
// GHASH state after the AAD of a chunk (SP 800-38D 6.4 over A || 0-pad), hashed serially with the
// table of H in global memory: meant for the short headers AAD is used for.  All lanes that call
// it with the same arguments compute the same value.
namespace {
__device__ Block aad_hash(const KeyTables* __restrict__ kt, const uint8_t* __restrict__ aad,
                          uint32_t aad_len) {
    Block y{{0, 0, 0, 0}};
    for (uint32_t off = 0; off < aad_len; off += 16) {
        uint32_t m = aad_len - off < 16 ? aad_len - off : 16;
        uint32_t x[4] = {0, 0, 0, 0};
#pragma unroll
        for (uint32_t b = 0; b < 16; ++b) {
            if (b < m) x[b / 4] |= (uint32_t)aad[off + b] << (8 * (b % 4));
        }
        y.w[0] ^= x[0], y.w[1] ^= x[1], y.w[2] ^= x[2], y.w[3] ^= x[3];
        y = gf_mul_table(kt->ghash[0], y);
    }
    return y;
}

// Pre-counter block of a chunk (SP 800-38D 7.1 step 2): IV || 0^31 1 for a 96-bit IV, else
// GHASH_H(IV || 0-pad || 0^64 || [8 |IV|]_64).  Same remark on lanes as above.
__device__ Block j0_from_iv(const KeyTables* __restrict__ kt, const uint8_t* __restrict__ iv,
                            uint32_t iv_len) {
    if (iv_len == 12) {
        Block j;
        for (int w = 0; w < 3; ++w)
            j.w[w] = (uint32_t)iv[4 * w] | ((uint32_t)iv[4 * w + 1] << 8) |
                     ((uint32_t)iv[4 * w + 2] << 16) | ((uint32_t)iv[4 * w + 3] << 24);
        j.w[3] = 0x01000000u;  // be32(1)
        return j;
    }
    Block y = aad_hash(kt, iv, iv_len);
    const uint64_t bits = (uint64_t)iv_len * 8;
    y.w[2] ^= bswap32((uint32_t)(bits >> 32));
    y.w[3] ^= bswap32((uint32_t)bits);
    return gf_mul_table(kt->ghash[0], y);
}

// J0 of the batch's chunk number `chunk`: read from `j0` when the host had it hashed beforehand
// (IVs that are not 96 bits long), otherwise formed from the IV bytes, which sit at the chunk's
// place `index` in the caller's array.
__device__ __forceinline__ Block chunk_j0(const KeyTables* __restrict__ kt,
                                          const uint8_t* __restrict__ ivs,
                                          const Block* __restrict__ j0, uint32_t chunk,
                                          uint32_t index) {
    if (j0 != nullptr) return j0[chunk];
    return j0_from_iv(kt, ivs + (uint64_t)index * 12, 12);
}
}  // namespace

// One thread per chunk: J0 of IVs whose length is not 96 bits, for the kernels that follow.
__global__ __launch_bounds__(64) void j0_kernel(const KeyTables* __restrict__ kt,
                                                const ChunkDesc* __restrict__ chunks,
                                                const uint8_t* __restrict__ ivs, uint32_t iv_len,
                                                uint32_t nchunks, Block* __restrict__ j0) {
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < nchunks) j0[i] = j0_from_iv(kt, ivs + (uint64_t)chunks[i].index * iv_len, iv_len);
}

// ------------------------------------------------------------------------------------------
// The bulk kernel.  LDS map (byte addresses; the object below is the kernel's only LDS):
//   [0, 8 KiB)           nibble table of H^64 (entry offsets fit the 16-bit DS offset field)
//   [8 KiB, 72 KiB)      row x (256 B): te[0][x] in dwords 0..31, te[1][x] in dwords 32..63
//   [72 KiB, 136 KiB)    the same for te[2], te[3]
// A round-table lookup address is  pair << 16 | x << 8 | 4 * (lane % 32)  plus a constant DS
// offset, so lane l always reads bank l % 32: lookups never collide, whatever the data.
namespace {

constexpr uint32_t kLdsGhBytes = kNibbleTableEntries * 16;
constexpr uint32_t kLdsTeBase = kLdsGhBytes;
constexpr uint32_t kLdsTeBytes = 4 * 256 * 32 * 4;
constexpr uint32_t kLdsBytes = kLdsGhBytes + kLdsTeBytes;

struct alignas(16) BulkLds {
    Block gh[kNibbleTableEntries];
    uint32_t te[kLdsTeBytes / 4];
};
static_assert(sizeof(BulkLds) == kLdsBytes && offsetof(BulkLds, gh) == 0 &&
                  offsetof(BulkLds, te) == kLdsTeBase,
              "LDS map");

typedef __attribute__((address_space(3))) const uint32_t* lds_u32_ptr;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) const u32x4* lds_u128_ptr;
typedef __attribute__((address_space(1))) const u32x4* global_u128_cptr;
typedef __attribute__((address_space(1))) u32x4* global_u128_ptr;

// payload accesses go through global (not flat) instructions, so that waiting for LDS results
// never waits for them
__device__ __forceinline__ u32x4 global_read128(const uint8_t* p) {
    return *reinterpret_cast<global_u128_cptr>(reinterpret_cast<uintptr_t>(p));
}
__device__ __forceinline__ void global_write128(uint8_t* p, u32x4 v) {
    *reinterpret_cast<global_u128_ptr>(reinterpret_cast<uintptr_t>(p)) = v;
}
// ... and so do the single bytes of a ragged last block: one flat access anywhere in the row loop
// would make every wait in it a wait for everything
typedef __attribute__((address_space(1))) const uint8_t* global_u8_cptr;
typedef __attribute__((address_space(1))) uint8_t* global_u8_ptr;
__device__ __forceinline__ uint8_t global_read8(const uint8_t* p) {
    return *reinterpret_cast<global_u8_cptr>(reinterpret_cast<uintptr_t>(p));
}
__device__ __forceinline__ void global_write8(uint8_t* p, uint8_t v) {
    *reinterpret_cast<global_u8_ptr>(reinterpret_cast<uintptr_t>(p)) = v;
}

// A block written so that a wavefront on another XCD can read it while this kernel still runs:
// the XCDs' L2 caches are not coherent with each other for ordinary accesses, and a release or
// acquire fence at device scope writes back or invalidates the whole L2 (tens of microseconds
// when megabytes of fresh ciphertext sit there).  Relaxed atomic accesses at device scope go
// through to memory instead, for these few bytes only.
__device__ __forceinline__ void store_block_device_scope(Block* p, uint32_t w0, uint32_t w1,
                                                         uint32_t w2, uint32_t w3) {
    uint64_t* q = reinterpret_cast<uint64_t*>(p);
    __hip_atomic_store(q, (uint64_t)w0 | ((uint64_t)w1 << 32), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(q + 1, (uint64_t)w2 | ((uint64_t)w3 << 32), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ Block load_block_device_scope(const Block* p) {
    uint64_t* q = reinterpret_cast<uint64_t*>(const_cast<Block*>(p));
    const uint64_t a = __hip_atomic_load(q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const uint64_t b = __hip_atomic_load(q + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return Block{{(uint32_t)a, (uint32_t)(a >> 32), (uint32_t)b, (uint32_t)(b >> 32)}};
}

// Payload stores that go through to memory at once instead of staying dirty in this XCD's L2:
// for output that a wavefront on another XCD may overwrite later in the same kernel (the wipe of
// a rejected chunk), where two L2s holding different dirty versions of a line would leave it to
// chance which one memory keeps.
__device__ __forceinline__ void global_write128_through(uint8_t* p, u32x4 v) {
    asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1" : : "v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ void global_write8_through(uint8_t* p, uint8_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}

// waits until every global load and store this wavefront has issued is complete (for a
// device-scope store: has reached memory)
__device__ __forceinline__ void wait_for_own_global_accesses() {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

// LDS byte address of a __shared__ object
__device__ __forceinline__ uint32_t lds_offset(const void* p) {
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}

__device__ __forceinline__ uint32_t lds_read32(uint32_t addr) {
    return *reinterpret_cast<lds_u32_ptr>(addr);
}
__device__ __forceinline__ u32x4 lds_read128(uint32_t addr) {
    return *reinterpret_cast<lds_u128_ptr>(addr);
}

// Round-table reads.  `a` already is pair << 16 | x << 8 | lane byte; T selects the table of the
// pair through the constant part of the address, which also carries `base`, the LDS address of
// the kernel's BulkLds object (a link-time constant, 0 when it is the kernel's only LDS object,
// so the sum lands in the instruction's offset field; a[] itself must stay free of it because
// byte 1 of a[] is rewritten every round).
template <int T>
__device__ __forceinline__ uint32_t te_read(uint32_t a, uint32_t base) {
    return lds_read32(a + (base + kLdsTeBase + 128u * (T & 1)));
}

// a.byte1 = rk.byte[KS] ^ v.byte[KV], every other byte of a kept: one SDWA instruction folds the
// AddRoundKey of a state byte into forming its next lookup address.
template <int KS, int KV>
__device__ __forceinline__ void key_xor_into_addr(uint32_t& a, uint32_t rk, uint32_t v) {
    static_assert(KS >= 0 && KS < 4 && KV >= 0 && KV < 4, "byte index");
    if constexpr (KS == 0 && KV == 0)
        asm("v_xor_b32_sdwa %0, %1, %2 dst_sel:BYTE_1 dst_unused:UNUSED_PRESERVE src0_sel:BYTE_0 src1_sel:BYTE_0" : "+v"(a) : "s"(rk), "v"(v));
    else if constexpr (KS == 1 && KV == 1)
        asm("v_xor_b32_sdwa %0, %1, %2 dst_sel:BYTE_1 dst_unused:UNUSED_PRESERVE src0_sel:BYTE_1 src1_sel:BYTE_1" : "+v"(a) : "s"(rk), "v"(v));
    else if constexpr (KS == 2 && KV == 2)
        asm("v_xor_b32_sdwa %0, %1, %2 dst_sel:BYTE_1 dst_unused:UNUSED_PRESERVE src0_sel:BYTE_2 src1_sel:BYTE_2" : "+v"(a) : "s"(rk), "v"(v));
    else if constexpr (KS == 3 && KV == 3)
        asm("v_xor_b32_sdwa %0, %1, %2 dst_sel:BYTE_1 dst_unused:UNUSED_PRESERVE src0_sel:BYTE_3 src1_sel:BYTE_3" : "+v"(a) : "s"(rk), "v"(v));
    else if constexpr (KS == 3 && KV == 0)
        asm("v_xor_b32_sdwa %0, %1, %2 dst_sel:BYTE_1 dst_unused:UNUSED_PRESERVE src0_sel:BYTE_3 src1_sel:BYTE_0" : "+v"(a) : "s"(rk), "v"(v));
    else if constexpr (KS == 2 && KV == 1)
        asm("v_xor_b32_sdwa %0, %1, %2 dst_sel:BYTE_1 dst_unused:UNUSED_PRESERVE src0_sel:BYTE_2 src1_sel:BYTE_1" : "+v"(a) : "s"(rk), "v"(v));
    else if constexpr (KS == 1 && KV == 2)
        asm("v_xor_b32_sdwa %0, %1, %2 dst_sel:BYTE_1 dst_unused:UNUSED_PRESERVE src0_sel:BYTE_1 src1_sel:BYTE_2" : "+v"(a) : "s"(rk), "v"(v));
    else if constexpr (KS == 0 && KV == 3)
        asm("v_xor_b32_sdwa %0, %1, %2 dst_sel:BYTE_1 dst_unused:UNUSED_PRESERVE src0_sel:BYTE_0 src1_sel:BYTE_3" : "+v"(a) : "s"(rk), "v"(v));
    else
        static_assert(KS == KV, "unsupported byte pairing");
}

// Sixteen lookup-address registers, one per state byte: a[j][k] serves byte k (row k) of column
// j and always reads table k.  Bytes 0 and 2 hold the lane's constants for the whole kernel;
// byte 1 is rewritten every round.
struct AesAddr {
    uint32_t a[4][4];
    // the last round key, in vector registers: the sixty key words and everything else a kernel
    // keeps in scalar registers do not fit them all, and one that is spilled costs a vector
    // instruction per use
    uint32_t last_key[4];
};

// last_round_key: the four words of round key Nr
__device__ __forceinline__ void aes_addr_init(AesAddr& A, uint32_t lane,
                                              const uint32_t* __restrict__ last_round_key) {
    const uint32_t lo = (lane & 31) * 4, hi = lo | 0x10000u;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        A.a[j][0] = lo;
        A.a[j][1] = lo;
        A.a[j][2] = hi;
        A.a[j][3] = hi;
        A.last_key[j] = last_round_key[j];
        asm volatile("" : "+v"(A.last_key[j]));  // a vector register, and kept there
    }
}

// The first three words of every counter block of a chunk are its IV, so in round 1 three of the
// four lookups of each column do not depend on the block: their sums are formed once per unit.
struct CtrConsts {
    uint32_t k[4];
};

__device__ __forceinline__ CtrConsts ctr_consts(const uint32_t* __restrict__ rk, uint32_t lane,
                                                uint32_t iv0, uint32_t iv1, uint32_t iv2,
                                                uint32_t base) {
    const uint32_t lo = (lane & 31) * 4, hi = lo | 0x10000u;
    const uint32_t s0 = iv0 ^ rk[0], s1 = iv1 ^ rk[1], s2 = iv2 ^ rk[2];
    auto at = [&](uint32_t w, int k, uint32_t lane_bytes) {
        return (((w >> (8 * k)) & 0xFFu) << 8) | lane_bytes;
    };
    CtrConsts c;
    c.k[0] = te_read<0>(at(s0, 0, lo), base) ^ te_read<1>(at(s1, 1, lo), base) ^ te_read<2>(at(s2, 2, hi), base);
    c.k[1] = te_read<0>(at(s1, 0, lo), base) ^ te_read<1>(at(s2, 1, lo), base) ^ te_read<3>(at(s0, 3, hi), base);
    c.k[2] = te_read<0>(at(s2, 0, lo), base) ^ te_read<2>(at(s0, 2, hi), base) ^ te_read<3>(at(s1, 3, hi), base);
    c.k[3] = te_read<1>(at(s0, 1, lo), base) ^ te_read<2>(at(s1, 2, hi), base) ^ te_read<3>(at(s2, 3, hi), base);
    return c;
}

template <int B, int E, class F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (B < E) {
        f(std::integral_constant<int, B>{});
        static_for<B + 1, E>(f);
    }
}

// (v.byte[K]) & 0xF0: the table offset of a high nibble, in one instruction
template <int K>
__device__ __forceinline__ uint32_t nibble_offset(uint32_t v, uint32_t mask_f0) {
    uint32_t r;
    if constexpr (K == 0)
        asm("v_and_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_0" : "=v"(r) : "s"(mask_f0), "v"(v));
    else if constexpr (K == 1)
        asm("v_and_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_1" : "=v"(r) : "s"(mask_f0), "v"(v));
    else if constexpr (K == 2)
        asm("v_and_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_2" : "=v"(r) : "s"(mask_f0), "v"(v));
    else
        asm("v_and_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_3" : "=v"(r) : "s"(mask_f0), "v"(v));
    return r;
}

// Y * H^64 from the nibble table in LDS, cut into sixteen byte steps (two 16-byte lookups and
// eight XORs each) so that the steps can be spread over the AES rounds of the same row: the
// hash arithmetic then fills the time the wavefront would wait for round-table lookups.
struct GhashRowMul {
    static constexpr bool kMatrix = false;
    uint32_t table; // LDS address of the nibble table of H^64
    uint32_t w[4];  // the multiplicand
    uint32_t t;     // current word << 4: its byte k carries the low nibble of byte k
    uint32_t z0 = 0, z1 = 0, z2 = 0, z3 = 0;
    u32x4 ra, rb;

    template <int S>
    __device__ __forceinline__ void issue() {
        constexpr int i = S / 4, k = S % 4;
        constexpr uint32_t pos = 2 * S;
        const uint32_t f0 = 0xF0u;
        if constexpr (k == 0) t = w[i] << 4;
        ra = lds_read128(nibble_offset<k>(w[i], f0) + (table + pos * 256));
        rb = lds_read128(nibble_offset<k>(t, f0) + (table + (pos + 1) * 256));
    }
    __device__ __forceinline__ void consume() {
        z0 = xor3(z0, ra.x, rb.x);
        z1 = xor3(z1, ra.y, rb.y);
        z2 = xor3(z2, ra.z, rb.z);
        z3 = xor3(z3, ra.w, rb.w);
        // pin the running sums here: otherwise the optimizer moves the whole XOR chain to where
        // its result is used and keeps all thirty-two table entries alive until then
        asm volatile("" : "+v"(z0), "+v"(z1), "+v"(z2), "+v"(z3));
    }
    template <int S>
    __device__ __forceinline__ void step() {
        issue<S>();
        consume();
    }
};

// Y * H^64 on the matrix cores.  Multiplication by a constant is linear over GF(2): product bit
// m is the parity of the number of bits k with M[m][k] = Y[k] = 1, and the matrix instruction
// counts those for 32 product bits of 32 lanes at once when every bit is spread out to a 4-bit
// floating-point number (0 or 1.0).  Per row of 64 lanes: 4 product tiles x 2 column groups (lanes
// 0..31, lanes 32..63) x 2 instructions of depth 64.  Products are scaled down into the denormal
// range, where a float's pattern is the integer it counts in units of 2^-149 (the matrix
// pipeline keeps denormals, in its results and in the sum it continues from), and rows are
// scaled apart: result register i of a lane counts in units of 2^(i % 8), and the second tile of
// a pair shares the first one's registers, another 2^8 up.  So one register holds two counts
// (each at most 128) whose lowest bits, the parities, sit at bits i % 8 and 8 + i % 8: one
// masked OR per register collects them, eight registers to a half word.
// No table lookups: the 8 KiB matrix image is read from LDS, 16 bytes per lane and instruction.
//
// Operand layout of v_mfma_scale_f32_32x32x64_f8f6f4 with 4-bit operands: lane l holds row (or
// column) l % 32, depth elements 32 (l / 32) .. + 31, eight to a register, lowest nibble first;
// one scale (a power of two, biased by 127, in byte 0) per lane.  Result register i of lane l is
// row 8 (i / 4) + 4 (l / 32) + i % 4 of column l % 32.
// Depth element <-> bit of Y: quarter c = 0..3 of the depth holds bits 4 j + c of the four words,
// left where they are inside their nibble (worth 0.5, 1.0, 2.0; bit 3 would be the sign and is
// moved down one place), the lane's scale making up for it.  A column's quarters 0, 2 belong in
// lanes 0..31 and 1, 3 in lanes 32..63: one swap of lane halves per register serves both groups.
// Product bit <-> row: lanes 0..31 make words 0 and 1 of both groups' columns, lanes 32..63
// words 2 and 3; tile pair p makes word 2 (l / 32) + p, register i of tile 2 p + f its bit
// 16 (i / 8) + 8 f + i % 8 (KeyTables::row_matrix is laid out to match).
typedef int v8i32 __attribute__((ext_vector_type(8)));
typedef float v16f32 __attribute__((ext_vector_type(16)));

struct GhashRowMatrix {
    static constexpr bool kMatrix = true;
    uint32_t image;    // LDS address of this lane's first piece of the matrix image
    uint32_t scale_b;  // scale of this lane's quarter of the first depth slice
    uint32_t scale_a;  // scale of this lane's matrix row in the first tile of a pair
    uint32_t scale_a2; // ... in the second
    uint32_t q[4][4];  // operand quarters; after begin(): q[g], q[2 + g] are group g's operands
    uint32_t out[2][2];
    u32x4 a0, a1;
    v16f32 acc;
    uint32_t z0, z1, z2, z3;

    // matrix entries (1.0) are scaled to 2^-127 and up, the other operand's to 2^-22
    static constexpr int kScaleHalf = 127 - 23;  // quarters 2 and 3 hold 2.0

    __device__ __forceinline__ void init(uint32_t lds_table, uint32_t lane) {
        image = lds_table + lane * 16;
        scale_b = lane < 32 ? 127u - 21u : 127u - 22u;  // quarter 0 holds 0.5, quarter 1 1.0
        const uint32_t row = lane & 31, reg = 4 * (row / 8) + row % 4;
        scale_a = reg % 8;  // 2^(reg % 8 - 127)
        scale_a2 = scale_a + 8;
    }
    __device__ __forceinline__ void begin(const uint32_t w[4]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            q[0][i] = w[i] & 0x11111111u;
            q[1][i] = w[i] & 0x22222222u;
            q[2][i] = w[i] & 0x44444444u;
            q[3][i] = (w[i] >> 1) & 0x44444444u;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            // lanes 32..63 of the first operand change places with lanes 0..31 of the second
            auto a = __builtin_amdgcn_permlane32_swap(q[0][i], q[1][i], false, false);
            q[0][i] = a[0], q[1][i] = a[1];
            auto b = __builtin_amdgcn_permlane32_swap(q[2][i], q[3][i], false, false);
            q[2][i] = b[0], q[3][i] = b[1];
        }
    }
    // Chain C = 2 * pair + group is four instructions into one set of sums, in two halves F
    // (the pair's tiles), each in three steps that the caller spreads over an AES round: the
    // tile's two matrix pieces are fetched, the first instruction starts or continues the sums,
    // the second (which has to wait for the first) follows.
    template <int C, int F>
    __device__ __forceinline__ void load() {
        constexpr int mt = 2 * (C / 2) + F;
        a0 = lds_read128(image + (mt * 2 + 0) * 1024);
        a1 = lds_read128(image + (mt * 2 + 1) * 1024);
    }
    template <int C, int F>
    __device__ __forceinline__ void first() {
        constexpr int g = C % 2;
        const v8i32 A0 = {(int)a0.x, (int)a0.y, (int)a0.z, (int)a0.w, 0, 0, 0, 0};
        const v8i32 B0 = {(int)q[g][0], (int)q[g][1], (int)q[g][2], (int)q[g][3], 0, 0, 0, 0};
        if constexpr (F == 0) {
            const v16f32 zero = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f,
                                 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
            acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(A0, B0, zero, 4, 4, 0,
                                                                   (int)scale_a, 0, (int)scale_b);
        } else {
            acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(A0, B0, acc, 4, 4, 0,
                                                                   (int)scale_a2, 0, (int)scale_b);
        }
    }
    template <int C, int F>
    __device__ __forceinline__ void second() {
        constexpr int g = C % 2;
        const v8i32 A1 = {(int)a1.x, (int)a1.y, (int)a1.z, (int)a1.w, 0, 0, 0, 0};
        const v8i32 B1 = {(int)q[2 + g][0], (int)q[2 + g][1], (int)q[2 + g][2], (int)q[2 + g][3],
                          0, 0, 0, 0};
        acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
            A1, B1, acc, 4, 4, 0, (int)(F == 0 ? scale_a : scale_a2), 0, kScaleHalf);
    }
    // the chain's thirty-two parities: registers 0..7 give the low half word, 8..15 the high
    template <int C>
    __device__ __forceinline__ void consume() {
        uint32_t lo = __float_as_uint(acc[0]) & 0x0101u, hi = __float_as_uint(acc[8]) & 0x0101u;
#pragma unroll
        for (int i = 1; i < 8; ++i) {
            // (sum & mask) | collected, in one instruction (truth table 0xEA)
            const uint32_t mask = 0x0101u << i;
            lo = __builtin_amdgcn_bitop3_b32(__float_as_uint(acc[i]), mask, lo, 0xEA);
            hi = __builtin_amdgcn_bitop3_b32(__float_as_uint(acc[8 + i]), mask, hi, 0xEA);
        }
        out[C % 2][C / 2] = (hi << 16) | lo;
    }
    // lanes 0..31 made words 0, 1 of both groups' columns, lanes 32..63 words 2, 3: the halves
    // of every column come home
    __device__ __forceinline__ void finish() {
        auto r0 = __builtin_amdgcn_permlane32_swap(out[0][0], out[1][0], false, false);
        auto r1 = __builtin_amdgcn_permlane32_swap(out[0][1], out[1][1], false, false);
        z0 = r0[0], z1 = r1[0], z2 = r0[1], z3 = r1[1];
    }
};

// E_K(J0[0..95] || be32(ctr)) for this lane's counter, with the row's GHASH multiplication G
// riding along; rk is wave-uniform (scalar registers).  Between rounds the state is carried
// without its round key: the key bytes are added while the next round's addresses are formed.
// The sixteen byte steps of G: three in round 1, the other thirteen spread evenly over rounds
// 2 .. kRounds (one each for AES-256, one or two each for the shorter keys).
// On the matrix cores the multiplication is four chains of four instructions instead: chain c is
// issued in rounds 2 c + 2 and 2 c + 3 (two matrix pieces fetched ahead of each round's lookups,
// two instructions, one before and one after the round's sums) and its result packed in the
// middle of round 2 c + 4, so that neither the fetch nor the matrix pipeline is waited for.
template <int kRounds, class Hash>
__device__ __forceinline__ void aes_ctr_lds(const uint32_t* __restrict__ rk, AesAddr& A,
                                               const CtrConsts& C, uint32_t ctr, Hash& G,
                                               uint32_t base, uint32_t& o0, uint32_t& o1,
                                               uint32_t& o2, uint32_t& o3) {
    static_assert(kRounds >= 10, "eight chains and their packing need rounds 2 .. 10");
    // round 1: the counter is the last word, big endian: state byte k is counter byte 3 - k
    key_xor_into_addr<3, 0>(A.a[3][3], rk[3], ctr);
    key_xor_into_addr<2, 1>(A.a[3][2], rk[3], ctr);
    key_xor_into_addr<1, 2>(A.a[3][1], rk[3], ctr);
    key_xor_into_addr<0, 3>(A.a[3][0], rk[3], ctr);
    uint32_t l0 = te_read<3>(A.a[3][3], base), l1 = te_read<2>(A.a[3][2], base), l2 = te_read<1>(A.a[3][1], base),
             l3 = te_read<0>(A.a[3][0], base);
    if constexpr (!Hash::kMatrix) G.template issue<0>();
    uint32_t u0 = C.k[0] ^ l0, u1 = C.k[1] ^ l1, u2 = C.k[2] ^ l2, u3 = C.k[3] ^ l3;
    if constexpr (!Hash::kMatrix) {
        G.consume();
        G.template step<1>();
        G.template step<2>();
    }
    __builtin_amdgcn_sched_barrier(0);
    static_for<2, kRounds + 1>([&](auto round) __attribute__((always_inline)) {
        constexpr int r = decltype(round)::value;
        constexpr int step_begin = 3 + (13 * (r - 2)) / (kRounds - 1),
                      step_end = 3 + (13 * (r - 1)) / (kRounds - 1);
        static_assert(step_end - step_begin == 1 || step_end - step_begin == 2, "hash steps");
        const uint32_t* k = rk + 4 * (r - 1);
        if constexpr (Hash::kMatrix) {
            if constexpr (r <= 9) G.template load<(r - 2) / 2, (r - 2) % 2>();
            __builtin_amdgcn_sched_barrier(0);
        }
        key_xor_into_addr<0, 0>(A.a[0][0], k[0], u0);
        key_xor_into_addr<1, 1>(A.a[0][1], k[0], u0);
        key_xor_into_addr<2, 2>(A.a[0][2], k[0], u0);
        key_xor_into_addr<3, 3>(A.a[0][3], k[0], u0);
        key_xor_into_addr<0, 0>(A.a[1][0], k[1], u1);
        key_xor_into_addr<1, 1>(A.a[1][1], k[1], u1);
        key_xor_into_addr<2, 2>(A.a[1][2], k[1], u1);
        key_xor_into_addr<3, 3>(A.a[1][3], k[1], u1);
        key_xor_into_addr<0, 0>(A.a[2][0], k[2], u2);
        key_xor_into_addr<1, 1>(A.a[2][1], k[2], u2);
        key_xor_into_addr<2, 2>(A.a[2][2], k[2], u2);
        key_xor_into_addr<3, 3>(A.a[2][3], k[2], u2);
        key_xor_into_addr<0, 0>(A.a[3][0], k[3], u3);
        key_xor_into_addr<1, 1>(A.a[3][1], k[3], u3);
        key_xor_into_addr<2, 2>(A.a[3][2], k[3], u3);
        key_xor_into_addr<3, 3>(A.a[3][3], k[3], u3);
        uint32_t t00 = te_read<0>(A.a[0][0], base), t11 = te_read<1>(A.a[1][1], base),
                 t22 = te_read<2>(A.a[2][2], base), t33 = te_read<3>(A.a[3][3], base);
        uint32_t t10 = te_read<0>(A.a[1][0], base), t21 = te_read<1>(A.a[2][1], base),
                 t32 = te_read<2>(A.a[3][2], base), t03 = te_read<3>(A.a[0][3], base);
        uint32_t t20 = te_read<0>(A.a[2][0], base), t31 = te_read<1>(A.a[3][1], base),
                 t02 = te_read<2>(A.a[0][2], base), t13 = te_read<3>(A.a[1][3], base);
        uint32_t t30 = te_read<0>(A.a[3][0], base), t01 = te_read<1>(A.a[0][1], base),
                 t12 = te_read<2>(A.a[1][2], base), t23 = te_read<3>(A.a[2][3], base);
        if constexpr (Hash::kMatrix) {
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (r >= 4 && r <= 10 && r % 2 == 0) G.template consume<(r - 4) / 2>();
            if constexpr (r <= 9) G.template first<(r - 2) / 2, (r - 2) % 2>();
            __builtin_amdgcn_sched_barrier(0);
        } else {
            G.template issue<step_begin>();
        }
        if constexpr (r < kRounds) {
            u0 = xor3(t00, t11, t22) ^ t33;
            u1 = xor3(t10, t21, t32) ^ t03;
            u2 = xor3(t20, t31, t02) ^ t13;
            u3 = xor3(t30, t01, t12) ^ t23;
        } else {
            // last round, no MixColumns: S(x) is byte 1 of te[0], byte 2 of te[1], byte 0 of
            // te[2] and te[3]
            auto last = [&](uint32_t v0, uint32_t v1, uint32_t v2, uint32_t v3, uint32_t key) {
                uint32_t lo = __builtin_amdgcn_perm(v0, v1, 0x0c0c0205u);  // [v0.b1, v1.b2, 0, 0]
                uint32_t hi = __builtin_amdgcn_perm(v2, v3, 0x00040c0cu);  // [0, 0, v2.b0, v3.b0]
                return xor3(lo, hi, key);
            };
            o0 = last(t00, t11, t22, t33, A.last_key[0]);
            o1 = last(t10, t21, t32, t03, A.last_key[1]);
            o2 = last(t20, t31, t02, t13, A.last_key[2]);
            o3 = last(t30, t01, t12, t23, A.last_key[3]);
        }
        if constexpr (Hash::kMatrix) {
            if constexpr (r <= 9) {
                __builtin_amdgcn_sched_barrier(0);  // after the round's sums, not before
                G.template second<(r - 2) / 2, (r - 2) % 2>();
            }
        } else {
            G.consume();
            if constexpr (step_end - step_begin == 2) G.template step<step_begin + 1>();
        }
        // keep every round's hash step with its round: without this the compiler sinks the
        // hash XORs to the end of the block and spills the table entries they wait for
        __builtin_amdgcn_sched_barrier(0);
    });
}

// Y * C from C's nibble table at LDS address `base`, on its own (not riding along with AES):
// the eight lookups of each word are issued together.
__device__ __forceinline__ void ghash_mul_lds(uint32_t base, uint32_t y[4]) {
    uint32_t z0 = 0, z1 = 0, z2 = 0, z3 = 0;
    const uint32_t f0 = 0xF0u;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t w = y[i], t = y[i] << 4;
        u32x4 e[8];
        e[0] = lds_read128(base + nibble_offset<0>(w, f0) + (8 * i + 0) * 256);
        e[1] = lds_read128(base + nibble_offset<0>(t, f0) + (8 * i + 1) * 256);
        e[2] = lds_read128(base + nibble_offset<1>(w, f0) + (8 * i + 2) * 256);
        e[3] = lds_read128(base + nibble_offset<1>(t, f0) + (8 * i + 3) * 256);
        e[4] = lds_read128(base + nibble_offset<2>(w, f0) + (8 * i + 4) * 256);
        e[5] = lds_read128(base + nibble_offset<2>(t, f0) + (8 * i + 5) * 256);
        e[6] = lds_read128(base + nibble_offset<3>(w, f0) + (8 * i + 6) * 256);
        e[7] = lds_read128(base + nibble_offset<3>(t, f0) + (8 * i + 7) * 256);
#pragma unroll
        for (int k = 0; k < 8; k += 2) {
            z0 = xor3(z0, e[k].x, e[k + 1].x);
            z1 = xor3(z1, e[k].y, e[k + 1].y);
            z2 = xor3(z2, e[k].z, e[k + 1].z);
            z3 = xor3(z3, e[k].w, e[k + 1].w);
        }
    }
    y[0] = z0, y[1] = z1, y[2] = z2, y[3] = z3;
}

// One row of a unit: block `blk` of the chunk in this lane.  On `edge` rows (the first and the
// last row of a chunk; a wave-uniform flag) some lanes may lie before the chunk's start and stay
// idle, the last lane may hold the chunk's ragged last block, and the lane of block 0 folds in
// the AAD state; idle lanes run the cipher on a dummy counter, touch no payload and keep a zero
// hash state.
// kThrough: the payload is written through to memory (see global_write128_through).
// kMatrixHash: the hash multiplication runs on the matrix cores; the first 8 KiB of the LDS
// object then hold the matrix image instead of the nibble table.
// `edge` is the same in every lane and held in a scalar register (walk_unit sees to that), so
// the rows that are no edge rows branch past all of the checks.
template <bool kDecrypt, int kRounds, bool kThrough = false, bool kMatrixHash = false>
__device__ __forceinline__ void bulk_row(const uint32_t* __restrict__ rk, AesAddr& A,
                                         const CtrConsts& C, uint32_t ctr1, const uint8_t* src,
                                         uint8_t* dst, uint64_t len, int64_t blk, bool edge,
                                         const Block& aad_y, Block* __restrict__ ekj0_out,
                                         uint32_t lds_base, uint32_t y[4]) {
    bool active = true;
    uint32_t tail = 0;  // bytes in a ragged block, 0 = whole block
    bool whole = true;
    uint32_t x0, x1, x2, x3;
    const uint8_t* sp = src + blk * 16;
    uint8_t* dp = dst + blk * 16;
    if (!edge) {
        const u32x4 v = global_read128(sp);
        x0 = v.x, x1 = v.y, x2 = v.z, x3 = v.w;
    } else {
        active = blk >= 0;
        if (active && (uint64_t)blk * 16 + 16 > len) tail = (uint32_t)(len & 15);
        whole = active && tail == 0;
        x0 = x1 = x2 = x3 = 0;
        if (whole) {
            const u32x4 v = global_read128(sp);
            x0 = v.x, x1 = v.y, x2 = v.z, x3 = v.w;
        }
        if (tail) {
#pragma unroll
            for (uint32_t b = 0; b < 15; ++b) {
                if (b < tail) {
                    const uint32_t v = (uint32_t)global_read8(sp + b) << (8 * (b % 4));
                    if (b / 4 == 0) x0 |= v;
                    if (b / 4 == 1) x1 |= v;
                    if (b / 4 == 2) x2 |= v;
                    if (b / 4 == 3) x3 |= v;
                }
            }
        }
    }

    // counter block inc32^(blk + 1)(J0): the first 96 bits of J0, then its counter field plus
    // blk + 1 modulo 2^32 (SP 800-38D 6.2, 7.1 step 3; ctr1 is that field plus 1, 2 for a 96-bit
    // IV) ... while the hash state moves one row along: Y <- Y * H^64
    std::conditional_t<kMatrixHash, GhashRowMatrix, GhashRowMul> G;
    if constexpr (kMatrixHash) {
        G.init(lds_base, __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u)));
        G.begin(y);
    } else {
        G.table = lds_base;  // the nibble table is the first member of BulkLds
        G.w[0] = y[0], G.w[1] = y[1], G.w[2] = y[2], G.w[3] = y[3];
    }
    uint32_t s0, s1, s2, s3;
    aes_ctr_lds<kRounds>(rk, A, C, (uint32_t)blk + ctr1, G, lds_base, s0, s1, s2, s3);
    if constexpr (kMatrixHash) G.finish();
    uint32_t o0 = x0 ^ s0, o1 = x1 ^ s1, o2 = x2 ^ s2, o3 = x3 ^ s3;

    auto store_block = [&]() __attribute__((always_inline)) {
        u32x4 o = {o0, o1, o2, o3};
        if constexpr (kThrough)
            global_write128_through(dp, o);
        else
            global_write128(dp, o);
    };
    if (!edge) {
        store_block();
    } else if (whole) {
        store_block();
    }
    if (edge && tail) {
#pragma unroll
        for (uint32_t b = 0; b < 15; ++b) {
            if (b < tail) {
                const uint32_t w = b / 4 == 0 ? o0 : b / 4 == 1 ? o1 : b / 4 == 2 ? o2 : o3;
                if constexpr (kThrough)
                    global_write8_through(dp + b, (uint8_t)(w >> (8 * (b % 4))));
                else
                    global_write8(dp + b, (uint8_t)(w >> (8 * (b % 4))));
            }
        }
        // bytes past the end count as zero in the hash
        const uint32_t keep = tail % 4 ? (1u << (8 * (tail % 4))) - 1u : 0u;  // in the partial word
        const uint32_t q = tail / 4;
        o0 = q > 0 ? o0 : (q == 0 ? o0 & keep : 0u);
        o1 = q > 1 ? o1 : (q == 1 ? o1 & keep : 0u);
        o2 = q > 2 ? o2 : (q == 2 ? o2 & keep : 0u);
        o3 = q == 3 ? o3 & keep : 0u;
    }

    // the ciphertext is what gets hashed: the output when encrypting, the input when decrypting
    uint32_t c0 = kDecrypt ? x0 : o0, c1 = kDecrypt ? x1 : o1, c2 = kDecrypt ? x2 : o2,
             c3 = kDecrypt ? x3 : o3;
    if (edge) {
        if (blk == 0) {
            // GHASH continues from the state the AAD left: same as adding it to the first block
            c0 ^= aad_y.w[0], c1 ^= aad_y.w[1], c2 ^= aad_y.w[2], c3 ^= aad_y.w[3];
        }
        if (blk == -1) {
            // the counter block of "block -1" is J0 itself: this idle lane has just computed
            // E_K(J0), the mask of the chunk's tag (SP 800-38D 7.1 steps 2 and 6)
            // (read by another kernel, or by another workgroup of this one: device scope)
            store_block_device_scope(ekj0_out, s0, s1, s2, s3);
        }
        if (!active) c0 = c1 = c2 = c3 = 0;  // idle lanes only occur before a chunk's start: Y = 0
    }
    y[0] = G.z0 ^ c0, y[1] = G.z1 ^ c1, y[2] = G.z2 ^ c2, y[3] = G.z3 ^ c3;
}

}  // namespace

namespace {

// Brings the bulk kernels' tables into LDS; every thread of the 1024 calls it, and a barrier
// must follow.  Round tables: 32 copies of every entry, lane-interleaved.  A row of the map is
// sixteen 16-byte pieces, eight per table of its pair; every thread fetches the eight entries
// its pieces need at once (independent loads) and writes each four times over in one store, and
// a wavefront's store covers four whole rows, so the stores run at the full LDS width.
template <bool kMatrixHash = false>
__device__ __forceinline__ void fill_bulk_lds(BulkLds& lds, const KeyTables* __restrict__ kt,
                                              uint32_t tid) {
    constexpr uint32_t kPieces = kLdsTeBytes / 16;
    static_assert(kPieces % kGroupThreads == 0, "pieces per thread");
    constexpr uint32_t kPerThread = kPieces / kGroupThreads;
    uint32_t v[kPerThread];
#pragma unroll
    for (uint32_t k = 0; k < kPerThread; ++k) {
        const uint32_t g = k * kGroupThreads + tid;  // piece number
        const uint32_t pair = g >> 12, row = (g >> 4) & 255, t = 2 * pair + ((g >> 3) & 1);
        v[k] = kt->te[t][row];
    }
    u32x4* te4 = reinterpret_cast<u32x4*>(lds.te);
#pragma unroll
    for (uint32_t k = 0; k < kPerThread; ++k) {
        const u32x4 q = {v[k], v[k], v[k], v[k]};
        te4[k * kGroupThreads + tid] = q;
    }
    for (uint32_t i = tid; i < kNibbleTableEntries; i += kGroupThreads) {
        if constexpr (kMatrixHash)
            lds.gh[i] = reinterpret_cast<const Block*>(kt->row_matrix)[i];
        else
            lds.gh[i] = kt->ghash[kRowPower][i];
    }
}

// One unit of one chunk, walked by one wavefront in rows of 64 blocks: keystream, XOR, and the
// lane's GHASH sum over the unit's rows, sum over rows r of C(r, lane) * (H^64)^(rows after r),
// left in y.  unit 0 also takes "block -1", whose counter block is J0, and stores E_K(J0).
template <bool kDecrypt, int kRounds, bool kThrough = false, bool kMatrixHash = false>
__device__ __forceinline__ void walk_unit(const KeyTables* __restrict__ kt,
                                          const uint32_t* __restrict__ rk, AesAddr& A,
                                          uint32_t lane, uint32_t lds_base, const uint8_t* src,
                                          uint8_t* dst, uint64_t len, const uint8_t* aad,
                                          uint32_t aad_len, uint32_t unit, uint32_t nunits,
                                          uint32_t first_blocks, uint32_t unit_power,
                                          const Block& j, Block* __restrict__ ekj0_out,
                                          uint32_t y[4]) {
    // What describes the unit is the same in every lane, and was fetched from memory just now:
    // moved to scalar registers here, (1) the wait for it comes before the row loop (placed at
    // the first use inside the loop, that wait would make every row wait for the previous row's
    // store as well), (2) which rows are edge rows is decided by a scalar branch, and (3) the
    // payload addresses are a scalar base plus the lane's offset.  (The length, which only edge
    // rows look at, stays where it is: scalar registers are short, and one that is spilled
    // costs a vector instruction per use.)
    // (the builtin returns a signed int: without the casts to uint32_t a low half with its top
    // bit set would be sign-extended over the high half)
    auto same_in_all_lanes = [](uint64_t v) __attribute__((always_inline)) {
        const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)v);
        const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
        return (uint64_t)lo | ((uint64_t)hi << 32);
    };
    src = reinterpret_cast<const uint8_t*>(same_in_all_lanes(reinterpret_cast<uint64_t>(src)));
    dst = reinterpret_cast<uint8_t*>(same_in_all_lanes(reinterpret_cast<uint64_t>(dst)));
    unit = __builtin_amdgcn_readfirstlane(unit);
    nunits = __builtin_amdgcn_readfirstlane(nunits);
    first_blocks = __builtin_amdgcn_readfirstlane(first_blocks);
    unit_power = __builtin_amdgcn_readfirstlane(unit_power);

    // the unit's blocks [b0, b1) of the chunk
    const int64_t b0 =
        unit == 0 ? -1 : (int64_t)first_blocks + ((int64_t)(unit - 1) << unit_power);
    const int64_t b1 = unit == 0 ? (int64_t)first_blocks : b0 + ((int64_t)1 << unit_power);
    const uint32_t nrows = (uint32_t)((b1 - b0 + kRowBlocks - 1) / kRowBlocks);

    const CtrConsts C = ctr_consts(rk, lane, j.w[0], j.w[1], j.w[2], lds_base);
    const uint32_t ctr1 = bswap32(j.w[3]) + 1u;

    Block aad_y{{0, 0, 0, 0}};
    if (unit == 0 && aad_len != 0) aad_y = aad_hash(kt, aad, aad_len);

    y[0] = y[1] = y[2] = y[3] = 0;
    // rows are aligned to the unit's end; only rows at the chunk's start can have idle lanes
    // (block index below 0) or block 0, only its very last row can hold a ragged block
    int64_t row_blk = b1 - (int64_t)nrows * kRowBlocks;
    for (uint32_t r = 0; r < nrows; ++r, row_blk += kRowBlocks) {
        const bool edge = row_blk <= 0 || (unit + 1 == nunits && r + 1 == nrows);
        bulk_row<kDecrypt, kRounds, kThrough, kMatrixHash>(rk, A, C, ctr1, src, dst, len,
                                                           row_blk + lane, edge, aad_y, ekj0_out,
                                                           lds_base, y);
    }
}

}  // namespace

// The schedule: wavefront w of the launch starts with unit w; when the launch has a wavefront for
// every unit that is all.  Otherwise the remaining units are handed out through `counter` until
// none is left (the counter serves about one request per 11 ns: a launch whose wavefronts all
// began by asking it would spend its first 50 us queueing, and a batch of many small units would
// be bound by it).  Unit i belongs to the
// chunk c with unit_base[c] <= i < unit_base[c + 1] (unit_base has one entry more than there are
// chunks); coarse_map[i >> kCoarseShift] is a chunk at or before the right one.
// sets[i * 64 + lane] receives lane's GHASH sum over the unit's rows.
// ivs: 96-bit IVs (a chunk's at its `index`), read when j0 is null; otherwise j0[c] is chunk c's J0.
// kMatrixHash: see bulk_row.
template <bool kDecrypt, int kRounds, bool kMatrixHash>
__global__ __launch_bounds__(kGroupThreads) void bulk_kernel(
    const KeyTables* __restrict__ kt, const ChunkDesc* __restrict__ chunks,
    const uint32_t* __restrict__ unit_base, const uint32_t* __restrict__ coarse_map,
    uint32_t nunits_total, uint32_t unit_power, uint32_t* __restrict__ counter,
    const uint8_t* __restrict__ ivs, const Block* __restrict__ j0, Block* __restrict__ ekj0,
    Block* __restrict__ sets) {
    __shared__ BulkLds lds;
    // lookups use raw LDS addresses relative to this object; its own address (0 as long as it
    // is the kernel's only LDS object) rides in the constant part of every lookup address
    const uint32_t lds_base = lds_offset(&lds);

    const uint32_t tid = threadIdx.x;
    fill_bulk_lds<kMatrixHash>(lds, kt, tid);
    __syncthreads();

    const uint32_t lane = tid & 63;
    // the round keys stay in scalar registers for the whole kernel (the last one in vector
    // registers, see AesAddr)
    uint32_t rk[4 * (kRounds + 1)];
#pragma unroll
    for (int i = 0; i < 4 * (kRounds + 1); ++i) rk[i] = kt->rk[i];
    AesAddr A;
    aes_addr_init(A, lane, rk + 4 * kRounds);

    const uint32_t nwaves = gridDim.x * kWavesPerGroup;
    const bool one_each = nunits_total <= nwaves;
    uint32_t item = blockIdx.x * kWavesPerGroup + (tid >> 6);
    for (;;) {
        if (item >= nunits_total) break;  // every wavefront gets here: the counter only grows

        uint32_t chunk = coarse_map[item >> kCoarseShift];
        while (unit_base[chunk + 1] <= item) ++chunk;  // ends: unit_base[nchunks] > item
        const ChunkDesc* __restrict__ cd = chunks + chunk;
        const Block j = chunk_j0(kt, ivs, j0, chunk, cd->index);
        uint32_t y[4];
        walk_unit<kDecrypt, kRounds, false, kMatrixHash>(
            kt, rk, A, lane, lds_base, cd->src, cd->dst, cd->len, cd->aad, cd->aad_len,
            item - cd->unit_base, cd->nunits, cd->first_blocks, unit_power, j, ekj0 + chunk, y);
        sets[(uint64_t)item * 64 + lane] = Block{{y[0], y[1], y[2], y[3]}};
        if (one_each) break;
        if (lane == 0)
            item = nwaves + __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED,
                                                   __HIP_MEMORY_SCOPE_AGENT);
        item = __builtin_amdgcn_readfirstlane(item);
    }
}

#define PGCM_INSTANTIATE_BULK(D, R, M)                                                       \
    template __global__ void bulk_kernel<D, R, M>(                                              \
        const KeyTables*, const ChunkDesc*, const uint32_t*, const uint32_t*, uint32_t, uint32_t, \
        uint32_t*, const uint8_t*, const Block*, Block*, Block*)
PGCM_INSTANTIATE_BULK(false, 10, false);
PGCM_INSTANTIATE_BULK(false, 12, false);
PGCM_INSTANTIATE_BULK(false, 14, false);
PGCM_INSTANTIATE_BULK(true, 10, false);
PGCM_INSTANTIATE_BULK(true, 12, false);
PGCM_INSTANTIATE_BULK(true, 14, false);
PGCM_INSTANTIATE_BULK(false, 10, true);
PGCM_INSTANTIATE_BULK(false, 12, true);
PGCM_INSTANTIATE_BULK(false, 14, true);
PGCM_INSTANTIATE_BULK(true, 10, true);
PGCM_INSTANTIATE_BULK(true, 12, true);
PGCM_INSTANTIATE_BULK(true, 14, true);
#undef PGCM_INSTANTIATE_BULK

// ------------------------------------------------------------------------------------------
// Folding partial sets.  Consecutive sets of a chunk lie 2^power blocks apart, so, lane by lane,
//   folded = (..(set_0 * G + set_1) * G + ..) + set_last   with G = H^(2^power).
namespace {

__device__ __forceinline__ void copy_power_table(Block* lds_table, const KeyTables* __restrict__ kt,
                                                 uint32_t power, uint32_t tid, uint32_t nthreads) {
    for (uint32_t i = tid; i < kNibbleTableEntries; i += nthreads) lds_table[i] = kt->ghash[power][i];
}

// table_addr: LDS address of G's nibble table, or 0xFFFFFFFF to read it from global memory.
// Sets are fetched eight at a time so that their load latencies overlap.
__device__ __forceinline__ void fold_sets(const KeyTables* __restrict__ kt,
                                          const Block* __restrict__ sets, uint32_t base,
                                          uint32_t count, uint32_t power, uint32_t lane,
                                          uint32_t table_addr, uint32_t y[4]) {
    const Block* __restrict__ p = sets + (uint64_t)base * 64 + lane;
    auto absorb = [&](const Block& next) {
        if (table_addr != 0xFFFFFFFFu) {
            ghash_mul_lds(table_addr, y);
        } else {
            Block m = gf_mul_table(kt->ghash[power], Block{{y[0], y[1], y[2], y[3]}});
            y[0] = m.w[0], y[1] = m.w[1], y[2] = m.w[2], y[3] = m.w[3];
        }
        y[0] ^= next.w[0], y[1] ^= next.w[1], y[2] ^= next.w[2], y[3] ^= next.w[3];
    };
    const Block first = p[0];
    y[0] = first.w[0], y[1] = first.w[1], y[2] = first.w[2], y[3] = first.w[3];
    uint32_t s = 1;
    for (; s + 8 <= count; s += 8) {
        Block n[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) n[k] = p[(uint64_t)(s + k) * 64];
#pragma unroll
        for (int k = 0; k < 8; ++k) absorb(n[k]);
    }
    for (; s < count; ++s) absorb(p[(uint64_t)s * 64]);
}

// value of lane (l + S) for S = 1, 2, 4, 8 inside each row of 16 lanes, by DPP
template <int S>
__device__ __forceinline__ uint32_t row_shift_down(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x100 + S, 0xF, 0xF, true);
}

// The 64 lane sums of a chunk -> its GHASH state, in every lane.  Lane j's sum still lacks
// H^(64 - j).  Tree: with s = 32, 16, .., 1 lane j takes Y_j * H^s + Y_(j+s) (DPP inside rows of
// 16 lanes, LDS permutes across them); lane 0 ends with sum_j Y_j * H^(63 - j); then one more H.
// When only the last 2^levels lanes hold anything (a chunk of at most 2^levels blocks; levels is
// wave-uniform) the steps with s >= 2^levels are skipped and lane 64 - 2^levels has the sum.
// tree_tables: LDS address of the nibble tables of H^(2^k), k = 0 .. 5, 8 KiB apart.
__device__ __forceinline__ void fold_lanes(uint32_t tree_tables, uint32_t y[4],
                                           uint32_t levels = 6) {
    auto tree_step = [&](uint32_t k, uint32_t n0, uint32_t n1, uint32_t n2, uint32_t n3) {
        ghash_mul_lds(tree_tables + k * kLdsGhBytes, y);
        y[0] ^= n0, y[1] ^= n1, y[2] ^= n2, y[3] ^= n3;
    };
    if (levels > 5)
        tree_step(5, __shfl_down(y[0], 32, 64), __shfl_down(y[1], 32, 64),
                  __shfl_down(y[2], 32, 64), __shfl_down(y[3], 32, 64));
    if (levels > 4)
        tree_step(4, __shfl_down(y[0], 16, 64), __shfl_down(y[1], 16, 64),
                  __shfl_down(y[2], 16, 64), __shfl_down(y[3], 16, 64));
    if (levels > 3)
        tree_step(3, row_shift_down<8>(y[0]), row_shift_down<8>(y[1]), row_shift_down<8>(y[2]),
                  row_shift_down<8>(y[3]));
    if (levels > 2)
        tree_step(2, row_shift_down<4>(y[0]), row_shift_down<4>(y[1]), row_shift_down<4>(y[2]),
                  row_shift_down<4>(y[3]));
    if (levels > 1)
        tree_step(1, row_shift_down<2>(y[0]), row_shift_down<2>(y[1]), row_shift_down<2>(y[2]),
                  row_shift_down<2>(y[3]));
    if (levels > 0)
        tree_step(0, row_shift_down<1>(y[0]), row_shift_down<1>(y[1]), row_shift_down<1>(y[2]),
                  row_shift_down<1>(y[3]));
    ghash_mul_lds(tree_tables, y);
    // only one lane holds the chunk's sum: hand it to every lane
    const uint32_t holder = 64u - (1u << levels);
    for (int k = 0; k < 4; ++k) y[k] = __builtin_amdgcn_readlane(y[k], holder);
}

// The same fold for whole rows (every lane may hold a sum), in groups of four: three
// multiplications deep instead of seven.  With l = 16 b + 4 c + j, H^(64 - l) =
// H^(16 (3 - b)) * H^(4 - j) * H^(4 (3 - c)).  In every step the four rows of sixteen lanes take
// one power each (a wavefront's table lookups collide in the LDS banks unless the lanes that are
// served together, sixteen neighbours, read one and the same table), and the four rows' products
// are then added up, every row keeping the sum:
//   1. row b multiplies its own sums by H^(16 (3 - b)); after the addition every row holds, at
//      place q = 4 c + j, the value V_q of the sixteen columns;
//   2. row r takes element j = r of every quad and multiplies by H^(4 - r); after the addition
//      every row holds W_c in all of quad c;
//   3. row r takes W_r and multiplies by H^(4 (3 - r)); the addition leaves the chunk's GHASH
//      state in every lane.
// Tables, 8 KiB apart from lane_tables: H^1, H^2, H^3, H^4, H^8, H^12, H^16, H^32, H^48.
constexpr uint32_t kLaneTables = 9;

__device__ __forceinline__ void copy_lane_tables(Block (*tables)[kNibbleTableEntries],
                                                 const KeyTables* __restrict__ kt, uint32_t tid,
                                                 uint32_t nthreads) {
    for (uint32_t i = tid; i < kNibbleTableEntries; i += nthreads) {
        tables[0][i] = kt->ghash[0][i];
        tables[1][i] = kt->ghash[1][i];
        tables[2][i] = kt->ghash_lane[0][i];
        tables[3][i] = kt->ghash[2][i];
        tables[4][i] = kt->ghash[3][i];
        tables[5][i] = kt->ghash_lane[1][i];
        tables[6][i] = kt->ghash[4][i];
        tables[7][i] = kt->ghash[5][i];
        tables[8][i] = kt->ghash_lane[2][i];
    }
}

// the XOR of the four rows' values, lane by lane, left in every row: rows 1, 3 change places with
// rows 0, 2 of a copy, then lanes 32..63 with lanes 0..31
__device__ __forceinline__ uint32_t rows_summed(uint32_t v) {
    const auto a = __builtin_amdgcn_permlane16_swap(v, v, false, false);
    v = a[0] ^ a[1];
    const auto b = __builtin_amdgcn_permlane32_swap(v, v, false, false);
    return b[0] ^ b[1];
}

// element kElement of every quad in all four lanes of the quad, in the rows of kRowMask only
template <int kElement, int kRowMask>
__device__ __forceinline__ uint32_t quad_element(uint32_t keep, uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp((int)keep, (int)v, kElement * 0x55, kRowMask, 0xF,
                                                 false);
}

__device__ __forceinline__ void fold_lanes_by_four(uint32_t lane_tables, uint32_t y[4],
                                                   uint32_t lane) {
    const uint32_t row = lane >> 4;
    const bool last_row = row == 3;
    {
        uint32_t m[4] = {y[0], y[1], y[2], y[3]};
        ghash_mul_lds(lane_tables + (8 - (last_row ? 2 : row)) * kLdsGhBytes, m);  // H^48, 32, 16
#pragma unroll
        for (int k = 0; k < 4; ++k) y[k] = rows_summed(last_row ? y[k] : m[k]);
    }
    {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            uint32_t t = quad_element<0, 1>(y[k], y[k]);
            t = quad_element<1, 2>(t, y[k]);
            t = quad_element<2, 4>(t, y[k]);
            y[k] = quad_element<3, 8>(t, y[k]);
        }
        ghash_mul_lds(lane_tables + (3 - row) * kLdsGhBytes, y);  // H^4, H^3, H^2, H^1
#pragma unroll
        for (int k = 0; k < 4; ++k) y[k] = rows_summed(y[k]);
    }
    {
        uint32_t m[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const uint32_t w0 = __builtin_amdgcn_readlane(y[k], 0), w1 = __builtin_amdgcn_readlane(y[k], 4),
                           w2 = __builtin_amdgcn_readlane(y[k], 8), w3 = __builtin_amdgcn_readlane(y[k], 12);
            y[k] = row == 0 ? w0 : row == 1 ? w1 : row == 2 ? w2 : w3;
            m[k] = y[k];
        }
        ghash_mul_lds(lane_tables + (5 - (last_row ? 2 : row)) * kLdsGhBytes, m);  // H^12, 8, 4
#pragma unroll
        for (int k = 0; k < 4; ++k) y[k] = rows_summed(last_row ? y[k] : m[k]);
    }
}

// From the GHASH state over A and C (the same in every lane) to the end of the invocation:
// length block, one more H, mask with E_K(J0) (SP 800-38D 7.1 steps 5-6); then write the tag, or
// compare it and write the verdict (7.2), wiping the output of a rejected chunk.
// h_table: LDS address of the nibble table of H.
template <bool kDecrypt>
__device__ __forceinline__ void finish_chunk(uint32_t h_table, uint32_t y[4],
                                             const uint32_t mask[4], const ChunkDesc& cd,
                                             uint8_t* __restrict__ tags, uint8_t* __restrict__ ok,
                                             uint32_t lane) {
    // [8 |A|]_64 || [8 |C|]_64, big endian
    const uint64_t abits = (uint64_t)cd.aad_len * 8, cbits = cd.len * 8;
    y[0] ^= bswap32((uint32_t)(abits >> 32));
    y[1] ^= bswap32((uint32_t)abits);
    y[2] ^= bswap32((uint32_t)(cbits >> 32));
    y[3] ^= bswap32((uint32_t)cbits);
    ghash_mul_lds(h_table, y);
    const uint32_t t[4] = {y[0] ^ mask[0], y[1] ^ mask[1], y[2] ^ mask[2], y[3] ^ mask[3]};

    uint8_t* tp = tags + (uint64_t)cd.index * 16;
    if (!kDecrypt) {
        if (lane == 0)
            for (int b = 0; b < 16; ++b) tp[b] = (uint8_t)(t[b / 4] >> (8 * (b % 4)));
    } else {
        // all 16 bytes, no data-dependent exit (every lane holds the same values)
        uint32_t diff = 0;
        for (int b = 0; b < 16; ++b) diff |= (uint32_t)tp[b] ^ ((t[b / 4] >> (8 * (b % 4))) & 0xFF);
        diff = __builtin_amdgcn_readfirstlane(diff);
        if (lane == 0) ok[cd.index] = diff == 0 ? 1 : 0;
        if (diff != 0) {
            // rejected: unauthenticated plaintext must not stay behind; the wavefront zero-fills
            // exactly len bytes
            const uint64_t whole = cd.len / 16;
            uint4* d = reinterpret_cast<uint4*>(cd.dst);
            for (uint64_t b = lane; b < whole; b += 64) d[b] = make_uint4(0, 0, 0, 0);
            for (uint64_t b = whole * 16 + lane; b < cd.len; b += 64) cd.dst[b] = 0;
        }
    }
}

}  // namespace

// One wavefront (= one workgroup) per fold item of one level.
__global__ __launch_bounds__(64) void fold_kernel(const KeyTables* __restrict__ kt,
                                                  const FoldItem* __restrict__ items,
                                                  uint32_t power, Block* __restrict__ sets) {
    __shared__ Block table[kNibbleTableEntries];
    const uint32_t lane = threadIdx.x;
    const FoldItem it = items[blockIdx.x];
    copy_power_table(table, kt, power, lane, 64);
    __syncthreads();
    uint32_t y[4];
    fold_sets(kt, sets, it.in_base, it.in_count, power, lane, lds_offset(table), y);
    sets[(uint64_t)it.out_slot * 64 + lane] = Block{{y[0], y[1], y[2], y[3]}};
}

// The same fold as a tree, for batches with few fold items, where the time of one item counts and
// not the number of items the chip gets through: one workgroup of sixteen wavefronts per item.
// The item's sets, counted back from its last, are the leaves; wavefront w first folds leaves
// 2w and 2w + 1 (missing leaves at the front count as zero, which changes nothing), then four
// rounds through LDS halve the number of partial results, round j with H^(2^(power + j)): five
// multiplications deep instead of thirty-one.
__global__ __launch_bounds__(kFoldTreeWaves * 64) void fold_tree_kernel(
    const KeyTables* __restrict__ kt, const FoldItem* __restrict__ items, uint32_t power,
    Block* __restrict__ sets) {
    constexpr uint32_t kLevels = kFanPower;  // 2^5 leaves
    static_assert(kFoldTreeWaves * 2 == kFan, "two leaves per wavefront");
    __shared__ Block tables[kLevels][kNibbleTableEntries];
    __shared__ Block partial[kFoldTreeWaves][64];
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const FoldItem it = items[blockIdx.x];
    for (uint32_t j = 0; j < kLevels; ++j) copy_power_table(tables[j], kt, power + j, tid, blockDim.x);

    // leaves 2w and 2w + 1 of 32, the item's sets being leaves 32 - in_count .. 31
    const uint32_t pad = kFan - it.in_count;
    const Block* __restrict__ in = sets + (uint64_t)it.in_base * 64 + lane;
    uint32_t y[4] = {0, 0, 0, 0};
    Block second{{0, 0, 0, 0}};
    if (2 * wave >= pad) {
        const Block first = in[(uint64_t)(2 * wave - pad) * 64];
        y[0] = first.w[0], y[1] = first.w[1], y[2] = first.w[2], y[3] = first.w[3];
    }
    if (2 * wave + 1 >= pad) second = in[(uint64_t)(2 * wave + 1 - pad) * 64];
    __syncthreads();  // tables are in place
    ghash_mul_lds(lds_offset(tables[0]), y);
    y[0] ^= second.w[0], y[1] ^= second.w[1], y[2] ^= second.w[2], y[3] ^= second.w[3];
    // every wavefront passes every barrier; only the shrinking front half has work to do
    for (uint32_t j = 1; j < kLevels; ++j) {
        partial[wave][lane] = Block{{y[0], y[1], y[2], y[3]}};
        __syncthreads();
        if (wave < (kFoldTreeWaves >> j)) {
            const Block a = partial[2 * wave][lane], b = partial[2 * wave + 1][lane];
            y[0] = a.w[0], y[1] = a.w[1], y[2] = a.w[2], y[3] = a.w[3];
            ghash_mul_lds(lds_offset(tables[j]), y);
            y[0] ^= b.w[0], y[1] ^= b.w[1], y[2] ^= b.w[2], y[3] ^= b.w[3];
        }
        __syncthreads();
    }
    if (wave == 0) sets[(uint64_t)it.out_slot * 64 + lane] = Block{{y[0], y[1], y[2], y[3]}};
}

// Per chunk (one wavefront each): fold the remaining sets, fold the 64 lanes, finish the tag.
// A workgroup is sixteen wavefronts; all of them bring the tables in, the first chunks_per_group
// of them then take a chunk each (the host spreads a batch of few chunks over the compute units:
// the wavefronts of one unit share its LDS pipe, and every chunk is a chain of dependent
// multiplications).  Workgroup 0 also clears `counter` for the next batch.
// LDS: the nine nibble tables of the lane tree, and those of the two most common fold distances.
// unit_power: log2 of the blocks per unit the batch was cut into.
constexpr uint32_t kFinalTables = kLaneTables + 2;

template <bool kDecrypt>
__global__ __launch_bounds__(kFinalWaves * 64) void final_kernel(
    const KeyTables* __restrict__ kt, const ChunkDesc* __restrict__ chunks, uint32_t nchunks,
    const uint8_t* __restrict__ ivs, const Block* __restrict__ j0, const Block* __restrict__ ekj0,
    const Block* __restrict__ sets, uint8_t* __restrict__ tags, uint8_t* __restrict__ ok,
    uint32_t unit_power, uint32_t* __restrict__ counter, uint32_t chunks_per_group) {
    __shared__ Block tables[kFinalTables][kNibbleTableEntries];
    const uint32_t tid = threadIdx.x, lane = tid & 63;
    if (blockIdx.x == 0 && tid == 0) *counter = 0;
    // tables 0..8: the lane tree's (the first is H's); then the fold distances of chunks with no
    // and with one fold level behind them
    copy_lane_tables(tables, kt, tid, blockDim.x);
    copy_power_table(tables[kLaneTables], kt, unit_power, tid, blockDim.x);
    copy_power_table(tables[kLaneTables + 1], kt, unit_power + kFanPower, tid, blockDim.x);
    __syncthreads();

    if ((tid >> 6) >= chunks_per_group) return;
    const uint32_t i = blockIdx.x * chunks_per_group + (tid >> 6);
    if (i >= nchunks) return;
    const ChunkDesc cd = chunks[i];

    uint32_t y[4] = {0, 0, 0, 0};
    Block mask;
    if (cd.final_count == 0) {
        // no ciphertext, so no unit ran for this chunk: the hash state is what the AAD leaves,
        // and E_K(J0) is still to be computed
        const Block a = aad_hash(kt, cd.aad, cd.aad_len);
        y[0] = a.w[0], y[1] = a.w[1], y[2] = a.w[2], y[3] = a.w[3];
        const Block j = chunk_j0(kt, ivs, j0, i, cd.index);
        uint32_t e[4] = {j.w[0], j.w[1], j.w[2], j.w[3]};
        aes_block_global(kt, e);
        mask = Block{{e[0], e[1], e[2], e[3]}};
    } else {
        uint32_t fold_table = 0xFFFFFFFFu;
        if (cd.final_power == unit_power) fold_table = lds_offset(tables[kLaneTables]);
        if (cd.final_power == unit_power + kFanPower) fold_table = lds_offset(tables[kLaneTables + 1]);
        fold_sets(kt, sets, cd.final_base, cd.final_count, cd.final_power, lane, fold_table, y);
        fold_lanes_by_four(lds_offset(tables[0]), y, lane);
        mask = ekj0[i];
    }
    finish_chunk<kDecrypt>(lds_offset(tables[0]), y, mask.w, cd, tags, ok, lane);
}

template __global__ void final_kernel<false>(const KeyTables*, const ChunkDesc*, uint32_t,
                                             const uint8_t*, const Block*, const Block*,
                                             const Block*, uint8_t*, uint8_t*, uint32_t,
                                             uint32_t*, uint32_t);
template __global__ void final_kernel<true>(const KeyTables*, const ChunkDesc*, uint32_t,
                                            const uint8_t*, const Block*, const Block*,
                                            const Block*, uint8_t*, uint8_t*, uint32_t,
                                            uint32_t*, uint32_t);

// ------------------------------------------------------------------------------------------
// A few chunks in ONE launch (the paper's swaps come a few chunks at a time, section 5.1).
// Descriptors are kernel arguments.  Every wavefront walks one unit as in bulk_kernel; then the
// workgroup, whose sixteen units belong to one chunk, folds their sets as a tree in LDS (the round
// tables are no longer needed: their space takes the GHASH tables of the fold).  A chunk of one
// workgroup is finished there and then.  Otherwise the workgroup writes its set through to memory
// (device-scope stores, no cache-wide fence), waits for the stores to complete and counts itself
// in on the chunk's arrival word; the workgroup that arrives last reads the workgroups' sets
// (device-scope loads) and folds them, each wavefront a run of them and then a tree across the
// wavefronts, folds the lanes and writes the tag or the verdict.  Nobody waits for anybody: every
// workgroup runs to its end whatever the others do.
//
// LDS after the round tables are done with, in tables of 8 KiB:
//   0..8   lane tree (see fold_lanes_by_four); the first is H's, for the length block
//   9..12  H^(2^(p + j)), j = 0 .. 3: tree over the workgroup's sixteen units (p = unit_power);
//          later, in the workgroup that arrives last,
//          H^(2^(p + 4 + l + j)), j = 0 .. 3: tree over the sixteen wavefronts' runs of 2^l sets
//   13     H^(2^(p + 4)): from one workgroup's set to the next
//   15..16 sixteen sets, one per wavefront
namespace {

constexpr uint32_t kSwapLaneTables = 0, kSwapUnitTables = kLaneTables, kSwapRunTable = 13,
                   kSwapWaveTables = kLaneTables, kSwapPartial = 15;
static_assert(kSwapUnitTables + 4 <= kSwapRunTable && kSwapRunTable < kSwapPartial, "table slots");
static_assert((kSwapPartial + 2) * kLdsGhBytes <= kLdsBytes, "tables and sets fit the LDS object");

// sixteen sets (one per wavefront, in y) -> one in wavefront 0, leaves counted back from the
// last: rounds j = 0 .. 3 with H^(2^(first_power + j)) at tables[first_table + j]
__device__ __forceinline__ void fold_waves(Block (*tables)[kNibbleTableEntries], Block (*partial)[64],
                                           uint32_t first_table, uint32_t wave, uint32_t lane,
                                           uint32_t y[4]) {
    // every wavefront passes every barrier; only the shrinking front half has work to do
    for (uint32_t j = 0; j < 4; ++j) {
        partial[wave][lane] = Block{{y[0], y[1], y[2], y[3]}};
        __syncthreads();
        if (wave < (kWavesPerGroup >> (j + 1))) {
            const Block a = partial[2 * wave][lane], b = partial[2 * wave + 1][lane];
            y[0] = a.w[0], y[1] = a.w[1], y[2] = a.w[2], y[3] = a.w[3];
            ghash_mul_lds(lds_offset(tables[first_table + j]), y);
            y[0] ^= b.w[0], y[1] ^= b.w[1], y[2] ^= b.w[2], y[3] ^= b.w[3];
        }
        __syncthreads();
    }
}

}  // namespace

template <bool kDecrypt, int kRounds>
__global__ __launch_bounds__(kGroupThreads) void swap_kernel(
    const KeyTables* __restrict__ kt, const ArgBatch batch, const uint8_t* __restrict__ ivs,
    Block* __restrict__ ekj0, Block* __restrict__ sets, uint32_t* __restrict__ arrive,
    uint8_t* __restrict__ tags, uint8_t* __restrict__ ok) {
    __shared__ BulkLds lds;
    __shared__ uint32_t last_flag;
    const uint32_t lds_base = lds_offset(&lds);
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    fill_bulk_lds(lds, kt, tid);

    // this workgroup's chunk: the one whose workgroups include blockIdx.x (host: the grid is the
    // sum of the chunks' ngroups, so the scan ends inside the array)
    uint32_t chunk = 0;
    while (chunk + 1 < batch.nchunks && batch.c[chunk + 1].group_base <= blockIdx.x) ++chunk;
    const ArgChunk cd = batch.c[chunk];
    const uint32_t unit_power = batch.unit_power;
    // units are dealt to the chunk's workgroups counted back from its end: workgroup g of G takes
    // units nunits - 16 (G - g) + wave; a negative number is a wavefront without a unit
    const uint32_t g = blockIdx.x - cd.group_base;
    const int32_t unit = (int32_t)cd.nunits - (int32_t)(kWavesPerGroup * (cd.ngroups - g)) + (int32_t)wave;
    __syncthreads();

    uint32_t y[4] = {0, 0, 0, 0};
    if (unit >= 0) {
        uint32_t rk[4 * (kRounds + 1)];
#pragma unroll
        for (int i = 0; i < 4 * (kRounds + 1); ++i) rk[i] = kt->rk[i];
        AesAddr A;
        aes_addr_init(A, lane, rk + 4 * kRounds);
        const Block j = j0_from_iv(kt, ivs + (uint64_t)cd.index * 12, 12);
        // When decrypting, the workgroup that finishes the chunk may have to wipe plaintext that
        // other workgroups (on other XCDs) wrote: their stores go through to memory, and must be
        // there before the arrival is counted.  So must E_K(J0), which unit 0's wavefront stores.
        walk_unit<kDecrypt, kRounds, kDecrypt>(kt, rk, A, lane, lds_base, cd.src, cd.dst, cd.len,
                                               cd.aad, cd.aad_len, (uint32_t)unit, cd.nunits,
                                               cd.first_blocks, unit_power, j, ekj0 + chunk, y);
        if (kDecrypt || unit == 0) wait_for_own_global_accesses();
    }
    __syncthreads();  // the round tables are done with: their LDS now takes GHASH tables

    Block(*tables)[kNibbleTableEntries] = reinterpret_cast<Block(*)[kNibbleTableEntries]>(&lds);
    Block(*partial)[64] = reinterpret_cast<Block(*)[64]>(tables[kSwapPartial]);
    const bool alone = cd.ngroups == 1;
    if (cd.nunits > 1)
        for (uint32_t j = 0; j < 4; ++j)
            copy_power_table(tables[kSwapUnitTables + j], kt, unit_power + j, tid, kGroupThreads);
    if (alone) copy_lane_tables(tables + kSwapLaneTables, kt, tid, kGroupThreads);
    __syncthreads();
    if (cd.nunits > 1) fold_waves(tables, partial, kSwapUnitTables, wave, lane, y);
    else if (wave == kWavesPerGroup - 1) {
        // a single unit sits in the last wavefront: hand its set to wavefront 0
        partial[0][lane] = Block{{y[0], y[1], y[2], y[3]}};
    }
    if (cd.nunits <= 1) {
        __syncthreads();
        if (wave == 0) {
            const Block a = partial[0][lane];
            y[0] = a.w[0], y[1] = a.w[1], y[2] = a.w[2], y[3] = a.w[3];
        }
    }

    if (!alone) {
        // hand this workgroup's set over and count it in; the last one to arrive goes on
        if (wave == 0) {
            store_block_device_scope(sets + (uint64_t)blockIdx.x * 64 + lane, y[0], y[1], y[2], y[3]);
            // the set (and E_K(J0), waited for before the last barrier) must have reached memory
            // before the arrival is counted: both are device-scope stores, so waiting for them
            // to complete is enough, and no cache needs writing back
            wait_for_own_global_accesses();
            if (lane == 0) {
                const uint32_t before = __hip_atomic_fetch_add(arrive + chunk, 1u, __ATOMIC_RELAXED,
                                                               __HIP_MEMORY_SCOPE_AGENT);
                last_flag = before + 1 == cd.ngroups;
                if (before + 1 == cd.ngroups)
                    __hip_atomic_store(arrive + chunk, 0u, __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);  // left zero for the next batch
            }
        }
        __syncthreads();
        if (!last_flag) return;  // uniform over the workgroup
        // the others' sets are read with device-scope loads, issued after the arrival count
        // was seen: they come from memory, not from this XCD's caches

        // runs of 2^l sets per wavefront, the smallest l with 16 * 2^l >= ngroups; leaves are
        // counted back from the last set, missing ones at the front count as zero
        uint32_t l = 0;
        while ((kWavesPerGroup << l) < cd.ngroups) ++l;
        copy_lane_tables(tables + kSwapLaneTables, kt, tid, kGroupThreads);
        copy_power_table(tables[kSwapRunTable], kt, unit_power + 4, tid, kGroupThreads);
        for (uint32_t j = 0; j < 4; ++j)
            copy_power_table(tables[kSwapWaveTables + j], kt, unit_power + 4 + l + j, tid,
                             kGroupThreads);
        const uint32_t run = 1u << l, pad = (kWavesPerGroup << l) - cd.ngroups;
        const Block* __restrict__ in = sets + (uint64_t)cd.group_base * 64 + lane;
        y[0] = y[1] = y[2] = y[3] = 0;
        const uint32_t first_leaf = wave * run;
        __syncthreads();
        bool started = false;  // uniform over the wavefront, like everything in this loop
        for (uint32_t k = 0; k < run; ++k) {
            const uint32_t leaf = first_leaf + k;
            if (leaf < pad) continue;
            if (started) ghash_mul_lds(lds_offset(tables[kSwapRunTable]), y);
            started = true;
            const Block b = load_block_device_scope(in + (uint64_t)(leaf - pad) * 64);
            y[0] ^= b.w[0], y[1] ^= b.w[1], y[2] ^= b.w[2], y[3] ^= b.w[3];
        }
        fold_waves(tables, partial, kSwapWaveTables, wave, lane, y);
    }
    if (wave != 0) return;

    // wavefront 0 holds the chunk's 64 lane sums (nothing at all for an empty chunk)
    Block mask;
    if (cd.nunits == 0) {
        const Block a = aad_hash(kt, cd.aad, cd.aad_len);
        y[0] = a.w[0], y[1] = a.w[1], y[2] = a.w[2], y[3] = a.w[3];
        const Block j = j0_from_iv(kt, ivs + (uint64_t)cd.index * 12, 12);
        uint32_t e[4] = {j.w[0], j.w[1], j.w[2], j.w[3]};
        aes_block_global(kt, e);
        mask = Block{{e[0], e[1], e[2], e[3]}};
    } else {
        fold_lanes_by_four(lds_offset(tables[kSwapLaneTables]), y, lane);
        mask = load_block_device_scope(ekj0 + chunk);
    }
    ChunkDesc d{};
    d.dst = cd.dst;
    d.len = cd.len;
    d.aad_len = cd.aad_len;
    d.index = cd.index;
    finish_chunk<kDecrypt>(lds_offset(tables[kSwapLaneTables]), y, mask.w, d, tags, ok, lane);
}

#define PGCM_INSTANTIATE_SWAP(D, R)                                                          \
    template __global__ void swap_kernel<D, R>(const KeyTables*, ArgBatch, const uint8_t*, Block*, \
                                               Block*, uint32_t*, uint8_t*, uint8_t*)
PGCM_INSTANTIATE_SWAP(false, 10);
PGCM_INSTANTIATE_SWAP(false, 12);
PGCM_INSTANTIATE_SWAP(false, 14);
PGCM_INSTANTIATE_SWAP(true, 10);
PGCM_INSTANTIATE_SWAP(true, 12);
PGCM_INSTANTIATE_SWAP(true, 14);
#undef PGCM_INSTANTIATE_SWAP

__global__ __launch_bounds__(64) void clear_words_kernel(uint32_t* __restrict__ words, uint32_t n) {
    for (uint32_t i = threadIdx.x; i < n; i += blockDim.x) words[i] = 0;
}

// ------------------------------------------------------------------------------------------
// The small-transfer path: a batch whose chunks are all at most kSmallChunkBytes long (the
// paper's "other I/O", usually < 8 KB, and the 1-byte NOPs of its error handler, sections 4.2 and
// 5.3) is done by ONE kernel from the first block to the tag, reading its descriptors straight
// from pinned host memory: what matters here is the latency of the call, not bandwidth.  Two
// shapes: a wavefront per chunk when every chunk fits one row, a workgroup of eight wavefronts
// per chunk otherwise.  LDS: the four round tables once (lookups may collide; there are few)
// and the nibble tables the chunks at hand need.
namespace {

template <int kRounds>
__device__ __forceinline__ void aes_block_lds_plain(const uint32_t* __restrict__ rk,
                                                    const uint32_t (*te)[256], uint32_t s[4]) {
    uint32_t a0 = s[0] ^ rk[0], a1 = s[1] ^ rk[1], a2 = s[2] ^ rk[2], a3 = s[3] ^ rk[3];
#pragma unroll
    for (int r = 1; r < kRounds; ++r) {
        uint32_t t0 = xor3(te[0][byte_of(a0, 0)], te[1][byte_of(a1, 1)], te[2][byte_of(a2, 2)]) ^
                      te[3][byte_of(a3, 3)] ^ rk[4 * r + 0];
        uint32_t t1 = xor3(te[0][byte_of(a1, 0)], te[1][byte_of(a2, 1)], te[2][byte_of(a3, 2)]) ^
                      te[3][byte_of(a0, 3)] ^ rk[4 * r + 1];
        uint32_t t2 = xor3(te[0][byte_of(a2, 0)], te[1][byte_of(a3, 1)], te[2][byte_of(a0, 2)]) ^
                      te[3][byte_of(a1, 3)] ^ rk[4 * r + 2];
        uint32_t t3 = xor3(te[0][byte_of(a3, 0)], te[1][byte_of(a0, 1)], te[2][byte_of(a1, 2)]) ^
                      te[3][byte_of(a2, 3)] ^ rk[4 * r + 3];
        a0 = t0, a1 = t1, a2 = t2, a3 = t3;
    }
    // last round: S(x) is byte 1 of te[0], byte 2 of te[1], byte 0 of te[2] and te[3]
    auto last = [&](uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3) {
        uint32_t lo = __builtin_amdgcn_perm(te[0][byte_of(c0, 0)], te[1][byte_of(c1, 1)], 0x0c0c0205u);
        uint32_t hi = __builtin_amdgcn_perm(te[2][byte_of(c2, 2)], te[3][byte_of(c3, 3)], 0x00040c0cu);
        return lo | hi;
    };
    s[0] = last(a0, a1, a2, a3) ^ rk[4 * kRounds + 0];
    s[1] = last(a1, a2, a3, a0) ^ rk[4 * kRounds + 1];
    s[2] = last(a2, a3, a0, a1) ^ rk[4 * kRounds + 2];
    s[3] = last(a3, a0, a1, a2) ^ rk[4 * kRounds + 3];
}

// One row of a short chunk: block `blk` (may be -1 or lower: idle) in this lane.  Reads and writes
// the payload, returns the lane's keystream block in s and what it contributes to the hash in c
// (the ciphertext block, zero-padded; for block 0 with the AAD state folded in; zero when idle).
template <bool kDecrypt, int kRounds>
__device__ __forceinline__ void small_row(const uint32_t* __restrict__ rk,
                                          const uint32_t (*te)[256], const ChunkDesc& cd,
                                          const Block& j, uint32_t ctr1, int64_t blk,
                                          const Block& aad_y, uint32_t s[4], uint32_t c[4]) {
    const bool active = blk >= 0;
    uint32_t tail = 0;
    if (active && (uint64_t)blk * 16 + 16 > cd.len) tail = (uint32_t)(cd.len & 15);
    const bool whole = active && tail == 0;
    uint32_t x[4] = {0, 0, 0, 0};
    const uint8_t* sp = cd.src + blk * 16;
    uint8_t* dp = cd.dst + blk * 16;
    if (whole) {
        u32x4 v = global_read128(sp);
        x[0] = v.x, x[1] = v.y, x[2] = v.z, x[3] = v.w;
    }
    if (tail) {
#pragma unroll
        for (uint32_t b = 0; b < 15; ++b)
            if (b < tail) x[b / 4] |= (uint32_t)sp[b] << (8 * (b % 4));
    }
    s[0] = j.w[0], s[1] = j.w[1], s[2] = j.w[2], s[3] = bswap32((uint32_t)blk + ctr1);
    aes_block_lds_plain<kRounds>(rk, te, s);
    uint32_t o[4] = {x[0] ^ s[0], x[1] ^ s[1], x[2] ^ s[2], x[3] ^ s[3]};
    if (whole) {
        u32x4 v = {o[0], o[1], o[2], o[3]};
        global_write128(dp, v);
    }
    if (tail) {
#pragma unroll
        for (uint32_t b = 0; b < 15; ++b)
            if (b < tail) dp[b] = (uint8_t)(o[b / 4] >> (8 * (b % 4)));
        // bytes past the end count as zero in the hash
#pragma unroll
        for (uint32_t b = 1; b < 16; ++b)
            if (b >= tail) o[b / 4] &= ~(0xFFu << (8 * (b % 4)));
    }
    for (int w = 0; w < 4; ++w) c[w] = kDecrypt ? x[w] : o[w];
    if (blk == 0)
        for (int w = 0; w < 4; ++w) c[w] ^= aad_y.w[w];
    if (!active)
        for (int w = 0; w < 4; ++w) c[w] = 0;
}

// levels of the lane tree a chunk of nblk <= 64 blocks in one row needs
__device__ __forceinline__ uint32_t lane_tree_levels(uint32_t nblk) {
    uint32_t levels = 0;
    while ((1u << levels) < nblk) ++levels;
    return levels;
}

// brings the round tables and the nibble tables named in `needed` (bit k: H^(2^k)) into LDS;
// every thread of the workgroup calls it
template <int kTables>
__device__ __forceinline__ void load_small_tables(uint32_t (*te)[256],
                                                  Block (*tables)[kNibbleTableEntries],
                                                  const KeyTables* __restrict__ kt,
                                                  uint32_t needed, uint32_t tid) {
    for (uint32_t t = tid; t < 4 * 256; t += blockDim.x) te[t >> 8][t & 255] = kt->te[t >> 8][t & 255];
    for (uint32_t k = 0; k < (uint32_t)kTables; ++k)
        if (needed & (1u << k)) copy_power_table(tables[k], kt, k, tid, blockDim.x);
}

}  // namespace

// Chunks of at most one row including "block -1" (63 blocks, 1008 bytes: the NOPs and most of the
// small traffic): one wavefront per chunk, several chunks a workgroup.
// ivs: IVs of iv_len bytes each, a chunk's at its `index`; J0 of an IV that is not 96 bits long is
// hashed here.
template <bool kDecrypt, int kRounds>
__global__ __launch_bounds__(kSmallChunksPerGroup * 64) void small_kernel(
    const KeyTables* __restrict__ kt, const ChunkDesc* __restrict__ chunks_host, uint32_t nchunks,
    const uint8_t* __restrict__ ivs, uint32_t iv_len, uint8_t* __restrict__ tags,
    uint8_t* __restrict__ ok) {
    __shared__ uint32_t te[4][256];
    __shared__ Block tables[6][kNibbleTableEntries];  // H^(2^k), k = 0 .. 5
    __shared__ uint32_t tables_needed;                // bit k: some chunk here uses tables[k]
    const uint32_t tid = threadIdx.x, lane = tid & 63;
    const uint32_t i = blockIdx.x * kSmallChunksPerGroup + (tid >> 6);
    const bool have_chunk = i < nchunks;
    ChunkDesc cd{};
    if (have_chunk) cd = chunks_host[i];
    const uint32_t nblk = (uint32_t)((cd.len + 15) / 16);  // <= 63, the host saw to that
    // the chunk fills only the last nblk lanes of its row: the lane tree starts lower down
    const uint32_t levels = lane_tree_levels(nblk);

    // only the tables this workgroup's chunks use are brought into LDS: H always, H^(2^k) for
    // the lane tree's levels (a 1-byte transfer needs H only)
    if (tid == 0) tables_needed = 0;
    __syncthreads();
    if (lane == 0 && have_chunk) atomicOr(&tables_needed, 1u | ((1u << levels) - 1u));
    __syncthreads();
    load_small_tables<6>(te, tables, kt, tables_needed, tid);
    __syncthreads();
    if (!have_chunk) return;
    const uint32_t* __restrict__ rk = kt->rk;

    Block aad_y{{0, 0, 0, 0}};
    if (cd.aad_len != 0) aad_y = aad_hash(kt, cd.aad, cd.aad_len);
    const Block j = j0_from_iv(kt, ivs + (uint64_t)cd.index * iv_len, iv_len);
    const uint32_t ctr1 = bswap32(j.w[3]) + 1u;

    // the row is aligned to the chunk's end; "block -1" (counter block J0) rides along in the
    // lane before block 0, and its keystream is E_K(J0)
    const int64_t blk = (int64_t)nblk - kRowBlocks + lane;
    uint32_t s[4], y[4], mask[4];
    small_row<kDecrypt, kRounds>(rk, te, cd, j, ctr1, blk, aad_y, s, y);
    for (int w = 0; w < 4; ++w) mask[w] = __shfl(s[w], (int)(kRowBlocks - nblk - 1), 64);

    if (nblk == 0) {
        // nothing was hashed yet: the state is what the AAD left
        for (int w = 0; w < 4; ++w) y[w] = aad_y.w[w];
    } else {
        fold_lanes(lds_offset(tables[0]), y, levels);
    }
    finish_chunk<kDecrypt>(lds_offset(tables[0]), y, mask, cd, tags, ok, lane);
}

#define PGCM_INSTANTIATE_SMALL(D, R)                                                      \
    template __global__ void small_kernel<D, R>(const KeyTables*, const ChunkDesc*, uint32_t, \
                                                const uint8_t*, uint32_t, uint8_t*, uint8_t*)
PGCM_INSTANTIATE_SMALL(false, 10);
PGCM_INSTANTIATE_SMALL(false, 12);
PGCM_INSTANTIATE_SMALL(false, 14);
PGCM_INSTANTIATE_SMALL(true, 10);
PGCM_INSTANTIATE_SMALL(true, 12);
PGCM_INSTANTIATE_SMALL(true, 14);
#undef PGCM_INSTANTIATE_SMALL

// Chunks of up to eight rows (8 KiB): one workgroup of eight wavefronts per chunk, a row each, so
// that the rows' cipher passes run side by side; the rows' lane sums are then folded across the
// wavefronts as a tree through LDS (H^64, H^128, H^256), and wavefront 0 finishes the chunk.
// Rows are aligned to the chunk's end and sit in the last wavefronts of the smallest power of two
// that holds them; E_K(J0) is one more cipher pass in wavefront 0.
template <bool kDecrypt, int kRounds>
__global__ __launch_bounds__(kSmallWideWaves * 64) void small_wide_kernel(
    const KeyTables* __restrict__ kt, const ChunkDesc* __restrict__ chunks_host, uint32_t nchunks,
    const uint8_t* __restrict__ ivs, uint32_t iv_len, uint8_t* __restrict__ tags,
    uint8_t* __restrict__ ok) {
    constexpr uint32_t kTables = kRowPower + 3;  // H^(2^k), k = 0 .. 8
    static_assert(kSmallWideWaves == 8, "three tree levels over the wavefronts");
    __shared__ uint32_t te[4][256];
    __shared__ Block tables[kTables][kNibbleTableEntries];
    __shared__ Block partial[kSmallWideWaves][64];
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (blockIdx.x >= nchunks) return;  // uniform over the workgroup
    const ChunkDesc cd = chunks_host[blockIdx.x];
    const uint32_t nblk = (uint32_t)((cd.len + 15) / 16);          // <= 512
    const uint32_t nrows = (nblk + kRowBlocks - 1) / kRowBlocks;   // 0 .. 8, without block -1
    uint32_t wave_levels = 0;                                      // tree levels over wavefronts
    while ((1u << wave_levels) < nrows) ++wave_levels;
    const uint32_t lane_levels = nrows > 1 ? 6u : lane_tree_levels(nblk);

    uint32_t needed = 1u | ((1u << lane_levels) - 1u);
    needed |= ((1u << wave_levels) - 1u) << kRowPower;
    load_small_tables<kTables>(te, tables, kt, needed, tid);
    __syncthreads();
    const uint32_t* __restrict__ rk = kt->rk;
    const Block j = j0_from_iv(kt, ivs + (uint64_t)cd.index * iv_len, iv_len);
    const uint32_t ctr1 = bswap32(j.w[3]) + 1u;

    // wavefront w of the first 2^wave_levels takes row w - (2^wave_levels - nrows), if there is one
    uint32_t y[4] = {0, 0, 0, 0};
    const int row = (int)wave - (int)((1u << wave_levels) - nrows);
    if (wave < (1u << wave_levels) && row >= 0) {
        Block aad_y{{0, 0, 0, 0}};
        if (row == 0 && cd.aad_len != 0) aad_y = aad_hash(kt, cd.aad, cd.aad_len);
        const int64_t blk = (int64_t)nblk - (int64_t)(nrows - (uint32_t)row) * kRowBlocks + lane;
        uint32_t s[4];
        small_row<kDecrypt, kRounds>(rk, te, cd, j, ctr1, blk, aad_y, s, y);
    }
    uint32_t mask[4] = {j.w[0], j.w[1], j.w[2], j.w[3]};
    if (wave == 0) aes_block_lds_plain<kRounds>(rk, te, mask);  // E_K(J0)

    // every wavefront passes every barrier; only the shrinking front has work to do
    for (uint32_t l = 0; l < wave_levels; ++l) {
        partial[wave][lane] = Block{{y[0], y[1], y[2], y[3]}};
        __syncthreads();
        if (wave < ((1u << wave_levels) >> (l + 1))) {
            const Block a = partial[2 * wave][lane], b = partial[2 * wave + 1][lane];
            y[0] = a.w[0], y[1] = a.w[1], y[2] = a.w[2], y[3] = a.w[3];
            ghash_mul_lds(lds_offset(tables[kRowPower + l]), y);
            y[0] ^= b.w[0], y[1] ^= b.w[1], y[2] ^= b.w[2], y[3] ^= b.w[3];
        }
        __syncthreads();
    }
    if (wave != 0) return;

    if (nblk == 0) {
        // nothing was hashed: the state is what the AAD left
        const Block a = aad_hash(kt, cd.aad, cd.aad_len);
        y[0] = a.w[0], y[1] = a.w[1], y[2] = a.w[2], y[3] = a.w[3];
    } else {
        fold_lanes(lds_offset(tables[0]), y, lane_levels);
    }
    finish_chunk<kDecrypt>(lds_offset(tables[0]), y, mask, cd, tags, ok, lane);
}

#define PGCM_INSTANTIATE_SMALL_WIDE(D, R)                                                   \
    template __global__ void small_wide_kernel<D, R>(const KeyTables*, const ChunkDesc*,       \
                                                     uint32_t, const uint8_t*, uint32_t,       \
                                                     uint8_t*, uint8_t*)
PGCM_INSTANTIATE_SMALL_WIDE(false, 10);
PGCM_INSTANTIATE_SMALL_WIDE(false, 12);
PGCM_INSTANTIATE_SMALL_WIDE(false, 14);
PGCM_INSTANTIATE_SMALL_WIDE(true, 10);
PGCM_INSTANTIATE_SMALL_WIDE(true, 12);
PGCM_INSTANTIATE_SMALL_WIDE(true, 14);
#undef PGCM_INSTANTIATE_SMALL_WIDE

// Brings a batch's descriptors from pinned host memory into the device workspace.  Done by a
// kernel so that the batch stays on one hardware queue: a DMA copy between kernels costs two
// cross-queue hand-overs.  `clear`, when not null, is a word to set to zero as well (the unit
// counter of a new workspace: a fill by a kernel, not a memset node, so that the stream's work
// stays of one kind).
__global__ __launch_bounds__(256) void upload_kernel(uint4* __restrict__ dst,
                                                     const uint4* __restrict__ src_host,
                                                     uint32_t n16, uint32_t* __restrict__ clear) {
    if (clear != nullptr && blockIdx.x == 0 && threadIdx.x == 0) *clear = 0;
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += gridDim.x * blockDim.x)
        dst[i] = src_host[i];
}

}  // namespace pgcm
