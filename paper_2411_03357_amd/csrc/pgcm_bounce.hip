// Pool of fixed-size pinned host buffers handed out in turn (C ABI of include/pgcm_bounce.h).
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include <new>
#include <vector>

#include "../../include/pgcm.h"
#include "../../include/pgcm_bounce.h"

namespace {

enum class SlotState : uint8_t { kFree, kHeld, kBusy };

struct Slot {
    uint8_t* buffer = nullptr;
    hipEvent_t released = nullptr;  // recorded by release on the caller's stream
    SlotState state = SlotState::kFree;
};

}  // namespace

struct pgcm_bounce {
    size_t buffer_bytes = 0;
    uint8_t* memory = nullptr;  // one pinned allocation cut into the buffers
    std::vector<Slot> slots;
    uint32_t next = 0;
};

extern "C" {
#pragma GCC visibility push(default)

int pgcm_bounce_create(size_t buffer_bytes, uint32_t count, pgcm_bounce_t** out) {
    if (out == nullptr) return PGCM_ERR_ARG;
    *out = nullptr;
    if (buffer_bytes == 0 || count == 0 || count > 65536) return PGCM_ERR_ARG;
    if (buffer_bytes > (SIZE_MAX - 255) / count) return PGCM_ERR_ARG;
    pgcm_bounce* p = new (std::nothrow) pgcm_bounce();
    if (p == nullptr) return PGCM_ERR_NOMEM;
    p->buffer_bytes = (buffer_bytes + 255) / 256 * 256;
    try {
        p->slots.resize(count);
    } catch (const std::bad_alloc&) {
        delete p;
        return PGCM_ERR_NOMEM;
    }
    void* mem = nullptr;
    if (hipHostMalloc(&mem, p->buffer_bytes * count, hipHostMallocDefault) != hipSuccess) {
        (void)hipGetLastError();
        delete p;
        return PGCM_ERR_NOMEM;
    }
    p->memory = (uint8_t*)mem;
    for (uint32_t i = 0; i < count; ++i) {
        p->slots[i].buffer = p->memory + (size_t)i * p->buffer_bytes;
        if (hipEventCreateWithFlags(&p->slots[i].released, hipEventDisableTiming) != hipSuccess) {
            pgcm_bounce_destroy(p);
            return PGCM_ERR_HIP;
        }
    }
    *out = p;
    return PGCM_OK;
}

void pgcm_bounce_destroy(pgcm_bounce_t* p) {
    if (p == nullptr) return;
    for (Slot& s : p->slots) {
        if (s.state == SlotState::kBusy) (void)hipEventSynchronize(s.released);
        if (s.released) (void)hipEventDestroy(s.released);
    }
    if (p->memory) {
        memset(p->memory, 0, p->buffer_bytes * p->slots.size());
        (void)hipHostFree(p->memory);
    }
    delete p;
}

int pgcm_bounce_acquire(pgcm_bounce_t* p, void** buffer, uint32_t* slot) {
    if (p == nullptr || buffer == nullptr || slot == nullptr) return PGCM_ERR_ARG;
    Slot& s = p->slots[p->next];
    if (s.state == SlotState::kHeld) return PGCM_ERR_BUSY;
    if (s.state == SlotState::kBusy) {
        if (hipEventSynchronize(s.released) != hipSuccess) return PGCM_ERR_HIP;
    }
    s.state = SlotState::kHeld;
    *buffer = s.buffer;
    *slot = p->next;
    p->next = (p->next + 1) % (uint32_t)p->slots.size();
    return PGCM_OK;
}

int pgcm_bounce_release(pgcm_bounce_t* p, uint32_t slot, void* hip_stream) {
    if (p == nullptr || slot >= p->slots.size()) return PGCM_ERR_ARG;
    Slot& s = p->slots[slot];
    if (s.state != SlotState::kHeld) return PGCM_ERR_ARG;
    if (hipEventRecord(s.released, (hipStream_t)hip_stream) != hipSuccess) return PGCM_ERR_HIP;
    s.state = SlotState::kBusy;
    return PGCM_OK;
}

size_t pgcm_bounce_buffer_bytes(const pgcm_bounce_t* p) { return p ? p->buffer_bytes : 0; }

uint32_t pgcm_bounce_count(const pgcm_bounce_t* p) { return p ? (uint32_t)p->slots.size() : 0; }

#pragma GCC visibility pop
}  // extern "C"
