/*
 * pgcm: batched AES-GCM (AES-256 first of all) on one AMD MI355X (gfx950).
 *
 * The operation is the one the paper's confidential-computing transport performs for every
 * host<->GPU transfer: an AES-GCM invocation over the transfer's bytes with a shared key and a
 * unique IV, whose receiver decrypts and rejects anything that fails the integrity check
 * (paper section 2.2, "A closer look at NVIDIA CC"; section 4.1, "Swapping sequence and IVs";
 * section 8.3 on why stale ciphertext must be rejected).  A batch is a list of such transfers
 * ("chunks": KV-cache blocks, weight chunks, adapters), each with its own 96-bit IV and 128-bit
 * tag, as issued between two synchronisation points (section 5.1, predictor input).
 * The cipher is AES-256 (FIPS-197) in GCM (NIST SP 800-38D) with 96-bit IVs and full 16-byte tags;
 * the entry points ending in _bytes and _iv open the cipher's other key lengths (128, 192 bits)
 * and IV lengths (SP 800-38D 5.2.1.1, 7.1 step 2) to users of the same transport other than the
 * paper's, those ending in _keys take a key per chunk.
 *
 * Conventions for every call
 *   - "DEVICE" pointers address memory the current HIP device can access: its own memory, or
 *     pinned host memory mapped for it (hipHostMalloc), e.g. a bounce buffer that receives the
 *     ciphertext directly.  "HOST" pointers address ordinary process memory; host arrays are
 *     consumed before the call returns.
 *   - Work is enqueued on `hip_stream` (a hipStream_t cast to void*, NULL = the null stream) and
 *     the call returns without synchronising.  Device outputs are valid once the stream has
 *     reached the end of the batch; device inputs must stay alive and unchanged until then.
 *   - One key object serves any number of streams and host threads at once (the paper's
 *     transport uses one session key for both directions, section 2.2): every batch call takes a
 *     context of the key (descriptor staging and device workspace), bound to the call's stream,
 *     and batches that share a stream are ordered by it.  Not thread-safe: pgcm_free_key and the
 *     test and measurement aids (pgcm_set_unit_bytes, pgcm_set_timing and its readers).
 *   - Errors are return codes.  A call that fails its argument checks (every status but
 *     PGCM_ERR_NOMEM and PGCM_ERR_HIP) has enqueued nothing; after PGCM_ERR_NOMEM or PGCM_ERR_HIP
 *     part of the batch may be on the stream, and its outputs are undefined.  Authentication
 *     failure of a chunk is not an error (see pgcm_decrypt_verify_batch).
 *   - IV uniqueness per key is the caller's duty (the paper's transport uses a counter); it is
 *     not checked.
 *   - The batch calls plan on the host, and they allocate (and wait for the stream) whenever a
 *     batch needs more descriptor or workspace memory than its context has: the first batches on
 *     a stream, and any batch larger than those before it.  pgcm_reserve does that work ahead of
 *     time; pgcm_encrypt_batch_static never allocates at all.
 */
#ifndef PGCM_H
#define PGCM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pgcm_key pgcm_key_t; /* opaque: device round keys, GHASH tables, workspace */

typedef enum {
    PGCM_OK = 0,
    PGCM_ERR_ARG = -1,   /* a required pointer is NULL, n is too large, a key or IV length is
                            not allowed, or the key lives on another GPU */
    PGCM_ERR_ALIGN = -2, /* a src or dst pointer is not 16-byte aligned */
    PGCM_ERR_LEN = -3,   /* a chunk is longer than 2^36 - 32 bytes (the GCM limit), or than a
                            forced unit size allows (pgcm_set_unit_bytes) */
    PGCM_ERR_NOMEM = -4, /* host or device allocation failed */
    PGCM_ERR_HIP = -5,   /* a HIP call failed; see pgcm_last_hip_error */
    PGCM_ERR_BUSY = -6,  /* pgcm_bounce.h: every buffer of a pool is held */
    PGCM_ERR_CAPACITY = -7 /* pgcm_encrypt_batch_static: the batch needs more than the fixed
                              buffers of that call hold */
} pgcm_status;

#define PGCM_MAX_CHUNK_BYTES ((((uint64_t)1) << 36) - 32)

/*
 * Key set-up (once per key, not per batch): the AES-256 key schedule, the GHASH key
 * H = E_K(0^128) and the tables of powers of H the batch kernels use, all computed on the GPU.
 *   key        HOST, 32 bytes.
 *   hip_stream stream the set-up kernel runs on; the call synchronises it before returning.
 *   out        HOST, receives the new object; release it with pgcm_free_key.
 */
int pgcm_expand_key(const uint8_t key[32], void *hip_stream, pgcm_key_t **out);

/*
 * The same for any AES key length (FIPS-197 5.2): key is HOST, key_bytes bytes, key_bytes one of
 * 16, 24, 32; anything else is PGCM_ERR_ARG.  pgcm_expand_key(k, ..) is this call with 32.
 */
int pgcm_expand_key_bytes(const uint8_t *key, uint32_t key_bytes, void *hip_stream,
                          pgcm_key_t **out);

/* Wipes the device and host copies of the key material and frees them.  NULL is allowed.
 * The caller must have synchronised every stream that still uses the key. */
void pgcm_free_key(pgcm_key_t *key);

/*
 * Authenticated encryption of n independent chunks (SP 800-38D section 7.1, once per chunk):
 *   dst[i] = src[i] xor keystream(key, IV_i),  tags[i] = GHASH_H(aad_i, dst[i]) xor E_K(IV_i || 1).
 *   ivs      DEVICE, n * 12 bytes; chunk i uses ivs[12 i .. 12 i + 11].
 *   aad      HOST array of n DEVICE pointers (any alignment); entries with aad_len[i] == 0 are
 *            not read.  Must be NULL exactly when aad_len is NULL.
 *   aad_len  HOST array of n byte counts, or NULL for "no chunk has AAD".  A chunk's AAD is
 *            hashed block after block by one wavefront: meant for headers of tens of bytes
 *            (any length is correct; a megabyte of AAD takes milliseconds).
 *   src      HOST array of n DEVICE pointers, each 16-byte aligned (unused when len[i] == 0).
 *   len      HOST array of n byte counts, 0 <= len[i] <= PGCM_MAX_CHUNK_BYTES; need not be a
 *            multiple of 16.  Exactly len[i] bytes are read and written, never more.
 *   dst      HOST array of n DEVICE pointers, 16-byte aligned.  dst[i] == src[i] (in place) is
 *            allowed; any other overlap between buffers of the batch is undefined.
 *   tags     DEVICE, n * 16 bytes, written.
 * n == 0 succeeds and does nothing.
 */
int pgcm_encrypt_batch(pgcm_key_t *key, size_t n, const uint8_t *ivs, const void *const *aad,
                       const uint32_t *aad_len, const void *const *src, const uint64_t *len,
                       void *const *dst, uint8_t *tags, void *hip_stream);

/*
 * Authenticated decryption of n independent chunks (SP 800-38D section 7.2, once per chunk).
 * Arguments as for pgcm_encrypt_batch, except:
 *   tags     DEVICE, n * 16 bytes, read: the tag received with each chunk.
 *   ok       DEVICE, n bytes, written: 1 when chunk i is authentic, 0 when it is rejected.
 * The tag comparison looks at all 16 bytes with no data-dependent exit.  For a rejected chunk
 * the len[i] bytes at dst[i] are overwritten with zeros before the batch ends on the stream
 * (unauthenticated plaintext is never left behind); the call itself still returns PGCM_OK.
 */
int pgcm_decrypt_verify_batch(pgcm_key_t *key, size_t n, const uint8_t *ivs,
                              const void *const *aad, const uint32_t *aad_len,
                              const void *const *src, const uint64_t *len, void *const *dst,
                              const uint8_t *tags, uint8_t *ok, void *hip_stream);

/*
 * For callers that cannot allocate: code between hipStreamBeginCapture and hipStreamEndCapture,
 * serving loops with a latency budget, harnesses that forbid hipMalloc.  pgcm_encrypt_batch with
 * the same arguments and the same results, except that it never allocates, frees or waits for an
 * allocation, in host or device memory: descriptors are staged in pinned buffers the key object
 * got at pgcm_expand_key, and the kernels' workspace (descriptors, unit maps, per-chunk tag
 * masks, partial hash sums) is one static device array of PGCM_STATIC_WORKSPACE_BYTES per GPU,
 * which the GPU holds from the moment the library is loaded until the process ends.
 * Limits: n <= PGCM_STATIC_MAX_CHUNKS, and descriptors and partial hash sums (1 KiB for every
 * 16 KiB of payload, never fewer than the batch needs to spread over the whole chip: up to 4 MiB
 * for a batch of a few megabytes) that fit the array: roughly 100 MB of payload per call.
 * A batch beyond them is refused with PGCM_ERR_CAPACITY and nothing is enqueued.  (The call
 * still waits on the host, without allocating, when it is more than four batches ahead of the
 * GPU.)
 * Every such call on one GPU, under any key and on any stream, uses the same array: calls whose
 * GPU work can overlap (different streams without ordering between them) race and give wrong
 * results; calls on one stream are safe.  The array keeps the last call's contents; what a call
 * needs at zero it clears itself.  pgcm_free_key wipes the array if the key used it.
 */
#define PGCM_STATIC_WORKSPACE_BYTES ((size_t)8 << 20)
#define PGCM_STATIC_MAX_CHUNKS ((size_t)1024)
int pgcm_encrypt_batch_static(pgcm_key_t *key, size_t n, const uint8_t *ivs,
                              const void *const *aad, const uint32_t *aad_len,
                              const void *const *src, const uint64_t *len, void *const *dst,
                              uint8_t *tags, void *hip_stream);

/*
 * Prepares the key's context for `hip_stream` (section 5.1: the transport knows the sizes of the
 * swaps it will be asked for) so that batch calls on that stream with at most n_max chunks and at
 * most payload_bytes_max bytes in all neither allocate nor wait for the stream: pinned staging
 * for the descriptors and device workspace for the schedule and the partial hash sums (about
 * 1/16 of the payload).  May allocate and synchronise the stream itself.  Call it again after
 * pgcm_set_unit_bytes.  PGCM_ERR_ARG when the numbers are beyond what a batch can be.
 */
int pgcm_reserve(pgcm_key_t *key, void *hip_stream, size_t n_max, uint64_t payload_bytes_max);

/*
 * The two batch calls for IVs of any one length (SP 800-38D 7.1 step 2: an IV that is not 96 bits
 * long is hashed into the pre-counter block J0 = GHASH_H(IV || 0-pad || 0^64 || [8 |IV|]_64), and
 * the 32-bit counter, the last word of J0, wraps modulo 2^32, section 6.2).
 *   ivs       DEVICE, n * iv_bytes bytes; chunk i uses ivs[iv_bytes i .. iv_bytes (i + 1) - 1].
 *   iv_bytes  length of every IV of the batch, >= 1; 0 is PGCM_ERR_ARG.  With 12 these calls are
 *             pgcm_encrypt_batch / pgcm_decrypt_verify_batch.
 * Everything else as above.  Long IVs are hashed by one GPU thread per chunk.
 */
int pgcm_encrypt_batch_iv(pgcm_key_t *key, size_t n, const uint8_t *ivs, uint32_t iv_bytes,
                          const void *const *aad, const uint32_t *aad_len,
                          const void *const *src, const uint64_t *len, void *const *dst,
                          uint8_t *tags, void *hip_stream);
int pgcm_decrypt_verify_batch_iv(pgcm_key_t *key, size_t n, const uint8_t *ivs, uint32_t iv_bytes,
                                 const void *const *aad, const uint32_t *aad_len,
                                 const void *const *src, const uint64_t *len, void *const *dst,
                                 const uint8_t *tags, uint8_t *ok, void *hip_stream);

/*
 * The two batch calls for chunks that do not all share one key (tenants, sessions or directions
 * with keys of their own; the paper's transport has a single session key, section 2.2).
 *   keys       HOST array of nkeys key objects, all created on the current device, any mix of key
 *              lengths; nkeys >= 1.
 *   key_index  HOST array of n entries: chunk i is processed under keys[key_index[i]];
 *              an entry >= nkeys is PGCM_ERR_ARG.
 *   ivs, iv_bytes, tags, ok and the other arrays: as for the _iv calls, indexed by chunk.
 * The chunks are grouped by key, keeping their order, and each group runs as one batch of its key
 * (so each key object's one-stream rule applies), the groups one after the other on hip_stream.
 * All arguments are checked before anything is enqueued; if an allocation or a HIP call fails in
 * a later group, the groups before it stay enqueued.
 */
int pgcm_encrypt_batch_keys(pgcm_key_t *const *keys, size_t nkeys, const uint32_t *key_index,
                            size_t n, const uint8_t *ivs, uint32_t iv_bytes,
                            const void *const *aad, const uint32_t *aad_len,
                            const void *const *src, const uint64_t *len, void *const *dst,
                            uint8_t *tags, void *hip_stream);
int pgcm_decrypt_verify_batch_keys(pgcm_key_t *const *keys, size_t nkeys,
                                   const uint32_t *key_index, size_t n, const uint8_t *ivs,
                                   uint32_t iv_bytes, const void *const *aad,
                                   const uint32_t *aad_len, const void *const *src,
                                   const uint64_t *len, void *const *dst, const uint8_t *tags,
                                   uint8_t *ok, void *hip_stream);

/* Static text for a pgcm_status value. */
const char *pgcm_strerror(int status);

/* The hipError_t (as int) behind the calling thread's most recent PGCM_ERR_HIP, else 0. */
int pgcm_last_hip_error(void);

/*
 * Host-only view of the chunk-to-wavefront schedule (section 5.1: requests arrive as batches of
 * copies of differing sizes).  Every chunk is cut into units of pgcm_batch_unit_bytes(n, len)
 * bytes counted back from its end, so only a chunk's first unit can be short; every wavefront
 * starts with a unit of its own and, when there are more units than wavefronts, takes further
 * ones from a shared counter.  Every unit leaves 64 partial hash sums; a chunk's sums are folded
 * 32 units at a time, level by level, until at most 32 remain for the chunk's final step.
 * Fills, for chunk i: nunits[i] (0 for an empty chunk), first_blocks[i] (16-byte blocks in its
 * first unit), unit_base[i] (index of its first unit among all units of the batch),
 * final_count[i] (partial sets left for the final step, 0..32) and final_power[i] (log2 of the
 * distance in blocks between them).  Any output pointer may be NULL.  Returns the total number
 * of units, or a negative pgcm_status.  Touches no GPU state.
 */
int64_t pgcm_plan_units(size_t n, const uint64_t *len, uint32_t *nunits, uint32_t *first_blocks,
                        uint32_t *unit_base, uint32_t *final_count, uint32_t *final_power);

/* Bytes per unit of the dynamic schedule (a multiple of the 1 KiB a wavefront handles per step). */
uint32_t pgcm_unit_bytes(void);

/*
 * Bytes per unit for a batch with these chunk lengths (len: HOST array of n byte counts): the
 * smallest power of two from 1 KiB to pgcm_unit_bytes() with which the batch has at most 4096
 * units (the wavefront slots of an MI355X, sixteen on each of 256 compute units: every unit then
 * has a wavefront of its own at once, so a batch of a few swap-sized chunks spreads over the
 * whole chip), and pgcm_unit_bytes() when none has (wavefronts then take further units in turn).
 * The batch calls count sixteen slots per compute unit of the key's device, so on a partition of
 * the chip they choose accordingly; this function and pgcm_plan_units describe the whole chip.
 * 0 when len is NULL and n is not 0.  Batches that take the small-transfer path (every chunk at
 * most 8 KiB) are not cut into units at all.
 */
uint32_t pgcm_batch_unit_bytes(size_t n, const uint64_t *len);

/*
 * Test aid, host only: the complete schedule the batch calls would upload for chunks of these
 * lengths (section 5.1: batches of copies of differing sizes), so that its invariants can be
 * checked without a GPU.
 *   unit_bytes   0 = chosen for the batch, else a forced unit size as for pgcm_set_unit_bytes.
 *   wave_slots   wavefront slots of the device (16 per compute unit); 0 = 4096, an MI355X.
 *   info         HOST, filled: offsets of the four arrays inside the image, the image's size, the
 *                device workspace the batch would need, the unit size as log2 of its 16-byte
 *                blocks, the numbers of units, partial-set slots (units + fold outputs), coarse
 *                map entries and fold items, per fold level the count of items and the index of
 *                the first, and the path the batch would take (0: the unit schedule, 1: the
 *                one-kernel path with a wavefront per chunk, 2: with a workgroup per chunk).
 *   image        HOST or NULL; when given it receives, at the offsets in info:
 *                descriptors, 64 bytes per chunk: src, dst, aad (pointers, here dummies), len
 *                  (u64), then u32 aad_len, unit_base, nunits, first_blocks, final_base,
 *                  final_count, final_power, index;
 *                unit_base, u32[n + 1]: index of each chunk's first unit, then the total;
 *                coarse map, u32[ncoarse]: for units 0, 16, 32, ..: a chunk at or before the one
 *                  that holds the unit;
 *                fold items, 16 bytes each: u32 in_base, in_count, out_slot, pad; level l's items
 *                  are fold_first[l] .. fold_first[l] + fold_count[l] - 1.
 *   image_capacity  bytes at image; PGCM_ERR_CAPACITY when smaller than info->image_bytes.
 * Returns PGCM_OK or the status the batch calls would give for these lengths.
 */
typedef struct pgcm_schedule_info {
    uint64_t desc_offset, unit_base_offset, coarse_map_offset, fold_items_offset;
    uint64_t image_bytes, workspace_bytes;
    uint32_t unit_power, nunits, nslots, ncoarse, nfold;
    uint32_t fold_count[4], fold_first[4];
    uint32_t path;
} pgcm_schedule_info;
int pgcm_describe_schedule(size_t n, const uint64_t *len, uint32_t unit_bytes,
                           uint32_t wave_slots, pgcm_schedule_info *info, void *image,
                           size_t image_capacity);

/*
 * Test aid: copies the key object's device tables to out (HOST), synchronising the device: 60
 * round-key words (little-endian loads of the FIPS-197 bytes; unused ones zero), the round count
 * and three zero words, the four round tables te[r][x] (256 words each), H (16 bytes), then for
 * k = 0 .. 30 the nibble table of H^(2^k): entry [2 * byte + (0: high, 1: low nibble)][value] =
 * (that nibble at that byte of an otherwise zero block) * H^(2^k), 16 bytes each.
 * pgcm_key_tables_bytes() is the size of it all; a smaller `bytes` copies a prefix.
 * The copy holds key material: wipe it after use.
 */
size_t pgcm_key_tables_bytes(void);
int pgcm_copy_key_tables(pgcm_key_t *key, void *out, size_t bytes);

/*
 * Tuning and test aid: fixes the unit size of every later batch under this key to unit_bytes
 * (a power of two from 1 KiB to 16 MiB), or returns to the per-batch choice with 0.
 * Anything else is PGCM_ERR_ARG.  A chunk that a forced unit cannot serve (more than 32^5 units
 * of it; or more than 32 GiB with units of 32 KiB or 1 MiB, where the last fold would need a
 * power of H the key object has no table for) is refused with PGCM_ERR_LEN by the batch calls.
 */
int pgcm_set_unit_bytes(pgcm_key_t *key, uint32_t unit_bytes);

/*
 * Tuning and test aid.  A batch of at most 24 chunks with 96-bit IVs that does not fill the chip
 * (every unit gets a wavefront of its own: up to a few megabytes on an MI355X) is done by one
 * kernel launch, the whole invocation from the first block to the tag, its descriptors passed as
 * kernel arguments (section 5.1: swaps come a few chunks at a time, and what counts for them is
 * the time of the call).  enable = 0 sends such batches through the same sequence of kernels as
 * larger ones instead (descriptor upload, unit kernel, fold, final step); results are identical.
 */
int pgcm_set_one_launch(pgcm_key_t *key, int enable);

/*
 * Tuning and test aid.  The kernel that does batches which fill the chip multiplies every
 * lane's running GHASH sum by H^64 once per 1 KiB row: thirty-two lookups in a table in LDS.
 * enable = 1 makes it a product with a fixed 128 x 128 matrix over GF(2) on the matrix cores
 * instead (SP 800-38D 6.3: multiplication by a constant is linear), which takes a fifth of the
 * LDS lookups' time off the LDS pipe and puts more work on the vector ALUs; measured 8 % slower
 * on an MI355X, hence off by default.  Results are identical.
 */
int pgcm_set_matrix_hash(pgcm_key_t *key, int enable);

/*
 * Measurement aid.  With timing enabled, every batch call also records a pair of HIP events on
 * its stream around the bulk kernel (the one launch that touches the payload: keystream, XOR
 * and GHASH of every unit; for the small-transfer path, its one kernel).  The library keeps the
 * pairs of the 256 most recent timed launches, so a run of batches can be enqueued back to back
 * and read afterwards.  Switching timing on (again) forgets earlier launches.
 * pgcm_last_bulk_kernel_ms waits for the most recent timed launch and returns its duration in
 * milliseconds; PGCM_ERR_ARG when nothing was timed.
 * pgcm_bulk_kernel_ms_history waits for and returns the durations of the most recent
 * min(max, 256, launches timed) launches, oldest first, in ms[] (HOST), and returns how many it
 * wrote, or a negative pgcm_status.
 */
int pgcm_set_timing(pgcm_key_t *key, int enable);

/*
 * Measurement aid: the keystream of nblocks consecutive counter blocks, E_K(iv || be32(ctr_base)),
 * E_K(iv || be32(ctr_base + 1)), .. (the blocks the cipher XORs onto a transfer's payload,
 * SP 800-38D 6.5), computed by a BITSLICED round function: no table lookups, the S-box as a
 * Boolean circuit over registers that each hold one bit of 32 blocks.  The batch calls do not use
 * it; it is here so that the cost of the one alternative to their table-driven rounds can be
 * measured on the chip and checked for correctness.
 *   iv         HOST, 12 bytes.
 *   ctr_base   first counter value; a multiple of 32 (a lane's 32 blocks differ in the low five
 *              bits of the counter); the counter wraps modulo 2^32.
 *   nblocks    a multiple of 2048 (32 blocks in each of a wavefront's 64 lanes), at most 2^31.
 *   out        DEVICE, 16 * nblocks bytes, 16-byte aligned, written.
 * PGCM_ERR_ARG when a constraint is not met.
 */
int pgcm_bitsliced_keystream(pgcm_key_t *key, const uint8_t iv[12], uint32_t ctr_base,
                             uint64_t nblocks, void *out, void *hip_stream);

/*
 * Measurement aid: `steps` passes of the path over one batch, enqueued back to back by a loop
 * inside the library, so that what is timed is the library and the GPU and not the caller's
 * language.  A pass is pgcm_encrypt_batch_iv (src -> cipher, tags written) followed by
 * pgcm_decrypt_verify_batch_iv (cipher -> back, tags read, ok written) when direction is 0, the
 * first alone when it is 1, the second alone when it is 2 (cipher and tags must then hold a
 * batch encrypted earlier).  The stream is synchronised before the first pass and after the
 * last; *host_ms receives the host's wall-clock time between the two.  Arrays as for the _iv
 * batch calls.  Stops at the first call that fails and returns its status.
 */
int pgcm_measure_passes(pgcm_key_t *key, size_t n, const uint8_t *ivs, uint32_t iv_bytes,
                        const void *const *aad,
                        const uint32_t *aad_len, const void *const *src, const uint64_t *len,
                        void *const *cipher, void *const *back, uint8_t *tags, uint8_t *ok,
                        void *hip_stream, uint32_t steps, int direction, double *host_ms);
int pgcm_last_bulk_kernel_ms(pgcm_key_t *key, float *ms);
int64_t pgcm_bulk_kernel_ms_history(pgcm_key_t *key, float *ms, size_t max);

#ifdef __cplusplus
}
#endif
#endif /* PGCM_H */
