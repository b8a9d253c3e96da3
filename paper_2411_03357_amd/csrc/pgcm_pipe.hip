// Carries out the decisions of the sequencer (pgcm_seq.h) with the batch calls (pgcm.h):
// C ABI of include/pgcm_pipe.h.  Host code only; the cipher runs in the library's kernels.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include <new>
#include <vector>

#include "../../include/pgcm_pipe.h"
#include "../../include/pgcm_seq.h"

namespace {

// IVs travel to the kernels through a ring in pinned memory, 16 bytes apart; when the ring
// wraps the pipe waits for the stream, so that no entry is overwritten before its kernel ran
constexpr uint32_t kIvRing = 1024;

struct Slot {
    bool used = false;
    uint64_t addr = 0, len = 0, iv = 0;
};

}  // namespace

struct pgcm_pipe {
    pgcm_key_t* key = nullptr;
    pgcm_seq_t* seq = nullptr;
    pgcm_pipe_config cfg{};
    pgcm_pipe_deliver_fn deliver = nullptr;
    void* user = nullptr;
    pgcm_pipe_stats stats{};
    // device memory: slots for kept ciphertexts, then one scratch slot for transfers made on
    // the spot, then 256 bytes for the NOP (plaintext byte at +0, ciphertext at +16)
    size_t slot_bytes = 0;
    uint8_t* cipher_mem = nullptr;
    uint8_t* tag_mem = nullptr;  // one tag per slot, then the scratch slot's, then the NOP's
    std::vector<Slot> slots;
    uint8_t* iv_ring = nullptr;  // pinned host memory
    uint32_t iv_pos = 0;
    // PRE actions wait here until something else has to happen, so that they go out as one batch
    std::vector<uint32_t> pending_pre;
    // Set when carrying out the state machine's actions failed half way: the state machine has
    // then moved on (its IV, what it believes is kept) while the slots and the wire have not, so
    // nothing it says afterwards can be trusted.  Every later call returns this status.
    int failed = PGCM_OK;

    uint8_t* slot_cipher(size_t i) const { return cipher_mem + i * slot_bytes; }
    uint8_t* slot_tag(size_t i) const { return tag_mem + 16 * i; }
    size_t scratch() const { return slots.size(); }
    uint8_t* nop_plain() const { return cipher_mem + (slots.size() + 1) * slot_bytes; }
    uint8_t* nop_cipher() const { return nop_plain() + 16; }
    uint8_t* nop_tag() const { return tag_mem + 16 * (slots.size() + 1); }
};

struct pgcm_recv {
    pgcm_key_t* key = nullptr;
    uint8_t iv0[12] = {};
    uint64_t next_iv = 0;
    uint8_t* iv_ring = nullptr;  // pinned host memory, as in the pipe
    uint32_t iv_pos = 0;
};

namespace {

// n consecutive ring entries holding IV_0 + iv[k]; returns the device-visible address of the first
int stage_ivs(pgcm_pipe* p, const uint64_t* iv, uint32_t n, hipStream_t stream, uint8_t** out) {
    if (n > kIvRing) return PGCM_ERR_ARG;
    if (p->iv_pos + n > kIvRing) {
        if (hipStreamSynchronize(stream) != hipSuccess) return PGCM_ERR_HIP;
        p->iv_pos = 0;
    }
    uint8_t* first = p->iv_ring + 16 * (size_t)p->iv_pos;
    // the batch calls read IVs 12 bytes apart: lay them out packed inside the 16-byte entries'
    // span (n * 12 <= n * 16)
    for (uint32_t k = 0; k < n; ++k) pgcm_seq_iv_bytes(p->cfg.iv0, iv[k], first + 12 * (size_t)k);
    p->iv_pos += n;
    *out = first;
    return PGCM_OK;
}

int encrypt_one(pgcm_pipe* p, const void* src, uint64_t len, uint64_t iv, uint8_t* dst,
                uint8_t* tag, hipStream_t stream) {
    uint8_t* ivs = nullptr;
    int rc = stage_ivs(p, &iv, 1, stream, &ivs);
    if (rc != PGCM_OK) return rc;
    const void* srcs[1] = {src};
    void* dsts[1] = {dst};
    const uint64_t lens[1] = {len};
    return pgcm_encrypt_batch(p->key, 1, ivs, nullptr, nullptr, srcs, lens, dsts, tag, stream);
}

// the PRE actions gathered so far, as few batch calls as their slots allow (tags of one call must
// be adjacent, so a call covers a run of consecutive slots)
int flush_pre(pgcm_pipe* p, hipStream_t stream) {
    size_t at = 0;
    const size_t total = p->pending_pre.size();
    while (at < total) {
        size_t run = 1;
        while (at + run < total && p->pending_pre[at + run] == p->pending_pre[at] + run) ++run;
        const void* srcs[64];
        void* dsts[64];
        uint64_t lens[64], ivn[64];
        if (run > 64) run = 64;
        for (size_t k = 0; k < run; ++k) {
            const uint32_t s = p->pending_pre[at + k];
            srcs[k] = (const void*)(uintptr_t)p->slots[s].addr;
            dsts[k] = p->slot_cipher(s);
            lens[k] = p->slots[s].len;
            ivn[k] = p->slots[s].iv;
        }
        uint8_t* ivs = nullptr;
        int rc = stage_ivs(p, ivn, (uint32_t)run, stream, &ivs);
        if (rc != PGCM_OK) return rc;
        rc = pgcm_encrypt_batch(p->key, run, ivs, nullptr, nullptr, srcs, lens, dsts,
                                p->slot_tag(p->pending_pre[at]), stream);
        if (rc != PGCM_OK) return rc;
        at += run;
    }
    p->pending_pre.clear();
    return PGCM_OK;
}

int find_slot(const pgcm_pipe* p, const pgcm_seq_action& a) {
    for (size_t i = 0; i < p->slots.size(); ++i)
        if (p->slots[i].used && p->slots[i].addr == a.addr && p->slots[i].len == a.len &&
            p->slots[i].iv == a.iv)
            return (int)i;
    return -1;
}

int carry_out_actions(pgcm_pipe* p, hipStream_t stream);

// Carries out every action the state machine has queued.  A failure in the middle leaves the
// pipe unusable (see pgcm_pipe::failed).
int carry_out(pgcm_pipe* p, hipStream_t stream) {
    const int rc = carry_out_actions(p, stream);
    if (rc != PGCM_OK) p->failed = rc;
    return rc;
}

int carry_out_actions(pgcm_pipe* p, hipStream_t stream) {
    pgcm_seq_action acts[64];
    for (;;) {
        const size_t n = pgcm_seq_take_actions(p->seq, acts, 64);
        if (n == 0) break;
        for (size_t k = 0; k < n; ++k) {
            const pgcm_seq_action& a = acts[k];
            int rc = PGCM_OK;
            if (a.kind == PGCM_SEQ_PRE) {
                int s = -1;
                for (size_t i = 0; i < p->slots.size() && s < 0; ++i)
                    if (!p->slots[i].used) s = (int)i;
                if (s < 0) return PGCM_ERR_NOMEM;  // more kept ciphertexts than 2 * depth
                p->slots[s].used = true;
                p->slots[s].addr = a.addr, p->slots[s].len = a.len, p->slots[s].iv = a.iv;
                p->pending_pre.push_back((uint32_t)s);
                p->stats.pre_bytes += a.len;
                continue;
            }
            // anything else may depend on the ciphertexts asked for so far
            rc = flush_pre(p, stream);
            if (rc != PGCM_OK) return rc;
            if (a.kind == PGCM_SEQ_SEND) {
                const int s = find_slot(p, a);
                if (s < 0) return PGCM_ERR_ARG;  // the state machine and the slots disagree
                p->deliver(p->user, a.kind, a.addr, a.len, a.iv, p->slot_cipher(s), p->slot_tag(s),
                           stream);
                p->slots[s].used = false;
                p->stats.ahead_bytes += a.len;
                ++p->stats.transfers;
            } else if (a.kind == PGCM_SEQ_NOW) {
                const size_t s = p->scratch();
                rc = encrypt_one(p, (const void*)(uintptr_t)a.addr, a.len, a.iv, p->slot_cipher(s),
                                 p->slot_tag(s), stream);
                if (rc != PGCM_OK) return rc;
                p->deliver(p->user, a.kind, a.addr, a.len, a.iv, p->slot_cipher(s), p->slot_tag(s),
                           stream);
                p->stats.critical_bytes += a.len;
                ++p->stats.transfers;
            } else if (a.kind == PGCM_SEQ_NOP) {
                rc = encrypt_one(p, p->nop_plain(), 1, a.iv, p->nop_cipher(), p->nop_tag(), stream);
                if (rc != PGCM_OK) return rc;
                p->deliver(p->user, a.kind, 0, 1, a.iv, p->nop_cipher(), p->nop_tag(), stream);
                ++p->stats.nops;
                ++p->stats.transfers;
            } else if (a.kind == PGCM_SEQ_DROP) {
                const int s = find_slot(p, a);
                if (s >= 0) {
                    p->slots[s].used = false;
                    p->stats.dropped_bytes += a.len;
                }
            }
        }
    }
    return flush_pre(p, stream);
}

int check_chunk_arg(const pgcm_pipe* p, const void* addr, uint64_t len) {
    if (p == nullptr) return PGCM_ERR_ARG;
    if (p->failed != PGCM_OK) return p->failed;
    if (len > p->cfg.max_chunk_bytes) return PGCM_ERR_LEN;
    if (len != 0 && addr == nullptr) return PGCM_ERR_ARG;
    if ((uintptr_t)addr & 15) return PGCM_ERR_ALIGN;
    return PGCM_OK;
}

}  // namespace

extern "C" {
#pragma GCC visibility push(default)

int pgcm_pipe_create(pgcm_key_t* key, const pgcm_pipe_config* cfg, pgcm_pipe_deliver_fn deliver,
                     void* user, pgcm_pipe_t** out) {
    if (out == nullptr) return PGCM_ERR_ARG;
    *out = nullptr;
    if (key == nullptr || cfg == nullptr || deliver == nullptr) return PGCM_ERR_ARG;
    if (cfg->depth == 0 || cfg->depth > 4096 || cfg->history_limit == 0 ||
        cfg->max_chunk_bytes == 0 || cfg->max_chunk_bytes > PGCM_MAX_CHUNK_BYTES)
        return PGCM_ERR_ARG;
    pgcm_pipe* p = new (std::nothrow) pgcm_pipe();
    if (p == nullptr) return PGCM_ERR_NOMEM;
    p->key = key, p->cfg = *cfg, p->deliver = deliver, p->user = user;
    p->slot_bytes = (size_t)((cfg->max_chunk_bytes + 255) / 256 * 256);
    int rc = PGCM_OK;
    do {
        try {
            p->slots.resize(2 * (size_t)cfg->depth);
            p->pending_pre.reserve(p->slots.size());
        } catch (const std::bad_alloc&) {
            rc = PGCM_ERR_NOMEM;
            break;
        }
        rc = pgcm_seq_create(cfg->iv_start, cfg->depth, cfg->leeway, cfg->swap_threshold,
                             cfg->history_limit, &p->seq);
        if (rc != PGCM_OK) break;
        const size_t cipher_bytes = (p->slots.size() + 1) * p->slot_bytes + 256;
        const size_t tag_bytes = 16 * (p->slots.size() + 2);
        if (hipMalloc((void**)&p->cipher_mem, cipher_bytes) != hipSuccess ||
            hipMalloc((void**)&p->tag_mem, tag_bytes) != hipSuccess ||
            hipHostMalloc((void**)&p->iv_ring, 16 * (size_t)kIvRing, hipHostMallocDefault) !=
                hipSuccess) {
            (void)hipGetLastError();
            rc = PGCM_ERR_NOMEM;
            break;
        }
        if (hipMemset(p->nop_plain(), 0, 256) != hipSuccess) rc = PGCM_ERR_HIP;
    } while (0);
    if (rc != PGCM_OK) {
        pgcm_pipe_destroy(p);
        return rc;
    }
    *out = p;
    return PGCM_OK;
}

void pgcm_pipe_destroy(pgcm_pipe_t* p) {
    if (p == nullptr) return;
    (void)hipDeviceSynchronize();
    if (p->cipher_mem) {
        (void)hipMemset(p->cipher_mem, 0, (p->slots.size() + 1) * p->slot_bytes + 256);
        (void)hipFree(p->cipher_mem);
    }
    if (p->tag_mem) (void)hipFree(p->tag_mem);
    if (p->iv_ring) (void)hipHostFree(p->iv_ring);
    if (p->seq) pgcm_seq_destroy(p->seq);
    delete p;
}

int pgcm_pipe_swap_out(pgcm_pipe_t* p, const void* addr, uint64_t len, void* hip_stream) {
    int rc = check_chunk_arg(p, addr, len);
    if (rc != PGCM_OK) return rc;
    rc = pgcm_seq_swap_out(p->seq, (uint64_t)(uintptr_t)addr, len);
    if (rc != PGCM_OK) return rc;
    return carry_out(p, (hipStream_t)hip_stream);
}

int pgcm_pipe_notify_write(pgcm_pipe_t* p, const void* addr, uint64_t len, void* hip_stream) {
    if (p == nullptr) return PGCM_ERR_ARG;
    if (p->failed != PGCM_OK) return p->failed;
    int rc = pgcm_seq_notify_write(p->seq, (uint64_t)(uintptr_t)addr, len);
    if (rc != PGCM_OK) return rc;
    return carry_out(p, (hipStream_t)hip_stream);
}

int pgcm_pipe_request(pgcm_pipe_t* p, const void* addr, uint64_t len, void* hip_stream) {
    int rc = check_chunk_arg(p, addr, len);
    if (rc != PGCM_OK) return rc;
    rc = pgcm_seq_request(p->seq, (uint64_t)(uintptr_t)addr, len);
    if (rc != PGCM_OK) return rc;
    return carry_out(p, (hipStream_t)hip_stream);
}

int pgcm_pipe_sync(pgcm_pipe_t* p, void* hip_stream) {
    if (p == nullptr) return PGCM_ERR_ARG;
    if (p->failed != PGCM_OK) return p->failed;
    int rc = pgcm_seq_sync(p->seq);
    if (rc != PGCM_OK) return rc;
    return carry_out(p, (hipStream_t)hip_stream);
}

int pgcm_pipe_get_stats(const pgcm_pipe_t* p, pgcm_pipe_stats* out) {
    if (p == nullptr || out == nullptr) return PGCM_ERR_ARG;
    *out = p->stats;
    return PGCM_OK;
}

int pgcm_recv_create(pgcm_key_t* key, const uint8_t iv0[12], uint64_t iv_start,
                     pgcm_recv_t** out) {
    if (out == nullptr) return PGCM_ERR_ARG;
    *out = nullptr;
    if (key == nullptr || iv0 == nullptr) return PGCM_ERR_ARG;
    pgcm_recv* r = new (std::nothrow) pgcm_recv();
    if (r == nullptr) return PGCM_ERR_NOMEM;
    r->key = key;
    memcpy(r->iv0, iv0, 12);
    r->next_iv = iv_start;
    if (hipHostMalloc((void**)&r->iv_ring, 16 * (size_t)kIvRing, hipHostMallocDefault) !=
        hipSuccess) {
        (void)hipGetLastError();
        delete r;
        return PGCM_ERR_NOMEM;
    }
    *out = r;
    return PGCM_OK;
}

void pgcm_recv_destroy(pgcm_recv_t* r) {
    if (r == nullptr) return;
    (void)hipDeviceSynchronize();
    if (r->iv_ring) (void)hipHostFree(r->iv_ring);
    delete r;
}

int pgcm_recv_accept(pgcm_recv_t* r, const void* ciphertext, uint64_t len, const uint8_t* tag,
                     void* dst, uint8_t* ok, void* hip_stream) {
    if (r == nullptr) return PGCM_ERR_ARG;
    hipStream_t stream = (hipStream_t)hip_stream;
    if (r->iv_pos == kIvRing) {
        if (hipStreamSynchronize(stream) != hipSuccess) return PGCM_ERR_HIP;
        r->iv_pos = 0;
    }
    uint8_t* iv = r->iv_ring + 16 * (size_t)r->iv_pos;
    pgcm_seq_iv_bytes(r->iv0, r->next_iv, iv);
    const void* srcs[1] = {ciphertext};
    void* dsts[1] = {dst};
    const uint64_t lens[1] = {len};
    const int rc = pgcm_decrypt_verify_batch(r->key, 1, iv, nullptr, nullptr, srcs, lens, dsts,
                                             tag, ok, stream);
    if (rc != PGCM_OK) return rc;  // nothing was enqueued: the transfer does not count
    ++r->iv_pos;
    ++r->next_iv;
    return PGCM_OK;
}

uint64_t pgcm_recv_next_iv(const pgcm_recv_t* r) { return r ? r->next_iv : 0; }

#pragma GCC visibility pop
}  // extern "C"
