/*
 * pgcm_seq: the IV-sequenced speculative pipeline of the paper as a host-side state machine.
 *
 * A sender whose peer accepts transfer k only under IV_0 + k (the paper's transport: both ends
 * count transfers, section 4.1) can take encryption off the critical path only by encrypting
 * chunks BEFORE they are asked for, with the IVs they will meet (section 4.3).  This object
 * decides which chunk to pre-encrypt with which IV (predictor, section 5.1), whether a request
 * may use a pre-encrypted ciphertext (validator, section 5.2), and how to recover when the
 * guess was wrong: hold a request whose IV lies ahead until the synchronisation and pad NOPs,
 * re-order inside a batch, or discard and encrypt on the spot (error handler, section 5.3).
 *
 * It touches no GPU state and encrypts nothing.  It turns events into ACTIONS that the caller
 * carries out, for instance with pgcm_encrypt_batch (IV bytes from pgcm_seq_iv_bytes):
 *   PRE   encrypt (addr, len) ahead of demand under iv and keep the ciphertext
 *   SEND  deliver the kept ciphertext of (addr, len); it was made under iv, the current IV
 *   NOW   encrypt (addr, len) under iv on the critical path and deliver it
 *   NOP   deliver a 1-byte dummy under iv (only advances the peer's IV)
 *   DROP  forget the kept ciphertext of (addr, len) made under iv
 * SEND, NOW and NOP appear in strictly increasing, gap-free IV order.
 * All calls are host-only, not thread-safe per object, and return PGCM_OK / PGCM_ERR_ARG /
 * PGCM_ERR_NOMEM as in pgcm.h.
 */
#ifndef PGCM_SEQ_H
#define PGCM_SEQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pgcm_seq pgcm_seq_t;

enum { PGCM_SEQ_PRE = 1, PGCM_SEQ_SEND = 2, PGCM_SEQ_NOW = 3, PGCM_SEQ_NOP = 4, PGCM_SEQ_DROP = 5 };

typedef struct {
    uint32_t kind; /* PGCM_SEQ_* */
    uint32_t reserved;
    uint64_t addr; /* 0 for NOP */
    uint64_t len;  /* 1 for NOP */
    uint64_t iv;   /* transfer number: the IV is IV_0 + iv */
} pgcm_seq_action;

/*
 * iv_start       number of the next transfer the peer expects
 * depth          how many predicted swaps are kept pre-encrypted (>= 1)
 * leeway         IVs left free before each predicted swap for small transfers in between
 * swap_threshold transfers shorter than this many bytes are "small": never pipelined (the paper
 *                separates swaps, usually > 128 KB, from other I/O, usually < 8 KB; section 4.2)
 * history_limit  how many past swap-ins the predictor looks back over (>= 1)
 */
int pgcm_seq_create(uint64_t iv_start, uint32_t depth, uint32_t leeway, uint64_t swap_threshold,
                    uint32_t history_limit, pgcm_seq_t **out);
void pgcm_seq_destroy(pgcm_seq_t *seq);

/* (addr, len) left the device and may be asked for again later. */
int pgcm_seq_swap_out(pgcm_seq_t *seq, uint64_t addr, uint64_t len);
/* Bytes [addr, addr + len) of plaintext changed: kept ciphertexts overlapping them are stale. */
int pgcm_seq_notify_write(pgcm_seq_t *seq, uint64_t addr, uint64_t len);
/* The application asks for (addr, len) to be transferred now. */
int pgcm_seq_request(pgcm_seq_t *seq, uint64_t addr, uint64_t len);
/* The application synchronises: the batch of requests ends. */
int pgcm_seq_sync(pgcm_seq_t *seq);

/* Moves up to cap queued actions, oldest first, into out; returns how many. */
size_t pgcm_seq_take_actions(pgcm_seq_t *seq, pgcm_seq_action *out, size_t cap);
/* Number of the next transfer the peer expects. */
uint64_t pgcm_seq_current_iv(const pgcm_seq_t *seq);

/* out = iv0 + n as a 96-bit big-endian integer (wraps modulo 2^96). */
void pgcm_seq_iv_bytes(const uint8_t iv0[12], uint64_t n, uint8_t out[12]);

#ifdef __cplusplus
}
#endif
#endif /* PGCM_SEQ_H */
