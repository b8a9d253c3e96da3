/*
 * pgcm_bounce: a pool of fixed-size pinned host buffers for ciphertext on its way over PCIe.
 *
 * The paper's transport keeps speculative ciphertext in private memory and moves it to the
 * device through a small number of fixed-size bounce buffers in shared memory, reused in turn so
 * that encryption and the copy overlap (paper section 6, "Ciphertext placement").  Here the
 * cipher runs on the GPU, so the analogue is: pgcm_encrypt_batch writes ciphertext straight into
 * a pool buffer (its dst pointers may be pinned host memory, see pgcm.h) and
 * pgcm_decrypt_verify_batch reads it straight out of one; the pool only hands the buffers out in
 * turn and knows when each is free again.
 *
 * A buffer is HELD from pgcm_bounce_acquire until pgcm_bounce_release, and BUSY from release until
 * the stream named there has passed the point of the release; acquire waits for a busy buffer on
 * the host.  One thread uses a pool at a time.  Status codes are those of pgcm.h.
 */
#ifndef PGCM_BOUNCE_H
#define PGCM_BOUNCE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pgcm_bounce pgcm_bounce_t;

/*
 * count >= 1 pinned buffers of buffer_bytes >= 1 bytes each (rounded up to a multiple of 256),
 * mapped for the current HIP device, 256-byte aligned.  PGCM_ERR_ARG for zero sizes or count
 * above 65536, PGCM_ERR_NOMEM when pinned memory cannot be had.  out: HOST.
 */
int pgcm_bounce_create(size_t buffer_bytes, uint32_t count, pgcm_bounce_t **out);

/* Waits for every busy buffer, wipes and frees the pool.  NULL is allowed. */
void pgcm_bounce_destroy(pgcm_bounce_t *pool);

/*
 * The next buffer in turn (round robin).  If it is still busy the call waits on the host until the
 * stream of its last release has got there; if it is still held, PGCM_ERR_BUSY (every buffer is
 * out: release one first).  *buffer receives the address, valid on host and device; *slot the
 * number to name it by in pgcm_bounce_release.  Both HOST, both required.
 */
int pgcm_bounce_acquire(pgcm_bounce_t *pool, void **buffer, uint32_t *slot);

/*
 * Gives a held buffer back: it may be handed out again once everything enqueued on hip_stream
 * so far (the kernel that reads or writes it, a copy out of it) has finished.  PGCM_ERR_ARG for a
 * slot that is not held.
 */
int pgcm_bounce_release(pgcm_bounce_t *pool, uint32_t slot, void *hip_stream);

/* Bytes per buffer after rounding, and number of buffers; 0 for NULL. */
size_t pgcm_bounce_buffer_bytes(const pgcm_bounce_t *pool);
uint32_t pgcm_bounce_count(const pgcm_bounce_t *pool);

#ifdef __cplusplus
}
#endif
#endif /* PGCM_BOUNCE_H */
