/*
 * pgcm_pipe: the speculative pipeline put to work on the GPU.
 *
 * pgcm_seq.h decides; this object carries the decisions out with the batch calls of pgcm.h, the
 * way the paper's runtime sits between the application's transfer requests and the encryption
 * (paper section 5, figure "architecture"; section 4.3): chunks the predictor expects are
 * encrypted AHEAD of demand into ciphertext slots the pipe owns, a request that the validator
 * matches is served from its slot without any encryption on the critical path, everything else
 * is encrypted on the spot, and NOPs (1-byte transfers) are issued where the error handler pads
 * the IV sequence (sections 5.1-5.3).  The sender here is the GPU: plaintext chunks are DEVICE
 * memory, e.g. KV-cache blocks about to be swapped out to the host.
 *
 * Every transfer that goes on the wire is handed to the caller's `deliver` function, in IV order
 * without gaps: transfer number iv must be received under IV_0 + iv, which is what a peer that
 * only counts transfers does (section 4.1).
 *
 * One pipe is used by one thread with one stream.  Status codes are those of pgcm.h.
 * A call that is refused for its arguments changes nothing.  A call that fails later, while the
 * pipe is carrying out what the state machine decided (an allocation or a HIP call inside the
 * batch calls), leaves the pipe FAILED: the state machine has counted transfers that never went
 * on the wire, so every later call returns that same status and does nothing; destroy the pipe,
 * and re-establish the IV with the peer (as after any lost transfer) before creating another.
 */
#ifndef PGCM_PIPE_H
#define PGCM_PIPE_H

#include <stddef.h>
#include <stdint.h>

#include "pgcm.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pgcm_pipe pgcm_pipe_t;

typedef struct {
    uint8_t iv0[12];          /* IV of transfer number 0 (big-endian 96-bit counter base) */
    uint32_t depth;           /* predicted swaps kept pre-encrypted, >= 1 */
    uint64_t iv_start;        /* number of the next transfer the peer expects */
    uint32_t leeway;          /* IVs left free before each predicted swap (section 5.1) */
    uint32_t history_limit;   /* past swap-ins the predictor looks back over, >= 1 */
    uint64_t swap_threshold;  /* shorter transfers are never pipelined (section 4.2) */
    uint64_t max_chunk_bytes; /* longest transfer the pipe accepts = size of a ciphertext slot */
} pgcm_pipe_config;

/*
 * Called once per transfer, in wire order.  kind is PGCM_SEQ_SEND (ciphertext made ahead of
 * demand), PGCM_SEQ_NOW (made just now) or PGCM_SEQ_NOP (1-byte dummy; addr is 0, len is 1).
 * ciphertext (len bytes, 16-byte aligned) and tag (16 bytes) are DEVICE memory owned by the pipe:
 * they are complete once hip_stream has run what is enqueued on it so far, and stay untouched by
 * the pipe only for work that this function enqueues on hip_stream (a copy into a bounce buffer,
 * a decrypt by a peer on the same device) or finishes before it returns.
 */
typedef void (*pgcm_pipe_deliver_fn)(void *user, uint32_t kind, uint64_t addr, uint64_t len,
                                     uint64_t iv, const void *ciphertext, const uint8_t *tag,
                                     void *hip_stream);

typedef struct {
    uint64_t transfers;      /* deliveries, NOPs included */
    uint64_t nops;
    uint64_t ahead_bytes;    /* delivered from a slot filled ahead of demand */
    uint64_t critical_bytes; /* encrypted on the critical path */
    uint64_t pre_bytes;      /* encrypted ahead of demand, used or not */
    uint64_t dropped_bytes;  /* encrypted ahead of demand and discarded */
} pgcm_pipe_stats;

/*
 * key: an expanded key on the current device; it must outlive the pipe and is used by it on the
 * pipe's stream only.  Allocates 2 * depth + 1 ciphertext slots of max_chunk_bytes each in device
 * memory.  PGCM_ERR_ARG for NULL pointers, depth or history_limit of 0, max_chunk_bytes of 0 or
 * above PGCM_MAX_CHUNK_BYTES.
 */
int pgcm_pipe_create(pgcm_key_t *key, const pgcm_pipe_config *config, pgcm_pipe_deliver_fn deliver,
                     void *user, pgcm_pipe_t **out);

/* Synchronises the device, wipes and frees the slots.  NULL is allowed. */
void pgcm_pipe_destroy(pgcm_pipe_t *pipe);

/*
 * The events of pgcm_seq.h, each followed at once by carrying out the actions it caused (batch
 * calls enqueued on hip_stream, `deliver` called for every transfer that goes out).
 *   addr  DEVICE, 16-byte aligned: the plaintext chunk; len <= max_chunk_bytes, else PGCM_ERR_LEN.
 * The plaintext of a chunk that was announced by swap_out or asked for before may be read by the
 * pipe at any later time, until notify_write says that it changed.
 */
int pgcm_pipe_swap_out(pgcm_pipe_t *pipe, const void *addr, uint64_t len, void *hip_stream);
int pgcm_pipe_notify_write(pgcm_pipe_t *pipe, const void *addr, uint64_t len, void *hip_stream);
int pgcm_pipe_request(pgcm_pipe_t *pipe, const void *addr, uint64_t len, void *hip_stream);
int pgcm_pipe_sync(pgcm_pipe_t *pipe, void *hip_stream);

/* Counters since creation.  out: HOST. */
int pgcm_pipe_get_stats(const pgcm_pipe_t *pipe, pgcm_pipe_stats *out);

/*
 * The other end: a peer that only counts.  It accepts transfer k under IV_0 + k and nothing else
 * (paper section 4.1), so a replayed, dropped or re-ordered delivery fails authentication.
 * Used with one thread and one stream, like the pipe.
 */
typedef struct pgcm_recv pgcm_recv_t;

/* key as for the pipe; iv0: 12 bytes, HOST; iv_start: number of the first transfer expected. */
int pgcm_recv_create(pgcm_key_t *key, const uint8_t iv0[12], uint64_t iv_start, pgcm_recv_t **out);
void pgcm_recv_destroy(pgcm_recv_t *recv);

/*
 * Decrypts and verifies the next transfer (pgcm_decrypt_verify_batch with n = 1 under the next
 * IV) and counts it, whatever the verdict turns out to be.
 *   ciphertext DEVICE, 16-byte aligned, len bytes (may be pinned host memory: a bounce buffer);
 *   tag        DEVICE, 16 bytes;   dst  DEVICE, 16-byte aligned, receives len bytes;
 *   ok         DEVICE, 1 byte: 1 authentic, 0 rejected (dst then holds zeros).
 * A NOP is accepted like any transfer (len 1); the caller discards its byte.
 */
int pgcm_recv_accept(pgcm_recv_t *recv, const void *ciphertext, uint64_t len, const uint8_t *tag,
                     void *dst, uint8_t *ok, void *hip_stream);

/* Number of the next transfer expected. */
uint64_t pgcm_recv_next_iv(const pgcm_recv_t *recv);

#ifdef __cplusplus
}
#endif
#endif /* PGCM_PIPE_H */
