// Host side of libpgcm: the C ABI of include/pgcm.h — argument checks, the chunk-to-wavefront
// schedule, descriptor upload and kernel launches.  No cipher arithmetic happens on the host.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#include <new>

#include "../../include/pgcm.h"
#include "pgcm_kernels.h"

using namespace pgcm;

namespace {

thread_local int g_last_hip_error = 0;

inline bool hip_failed(hipError_t e) {
    if (e == hipSuccess) return false;
    g_last_hip_error = (int)e;
    return true;
}

#define PGCM_HIP(call)                             \
    do {                                           \
        if (hip_failed(call)) return PGCM_ERR_HIP; \
    } while (0)

constexpr int kStages = 2;

// Per-chunk schedule: segments are counted back from the chunk's end, so that every segment but
// the first is full and all row boundaries line up with the end of the chunk.
struct SegPlan {
    uint32_t nseg, first_blocks;
};

inline SegPlan plan_chunk(uint64_t len) {
    uint64_t nblk = (len + 15) / 16;
    SegPlan p{0, 0};
    if (nblk == 0) return p;
    uint64_t nseg = (nblk + kSegBlocks - 1) / kSegBlocks;
    p.nseg = (uint32_t)nseg;
    p.first_blocks = (uint32_t)(nblk - (nseg - 1) * kSegBlocks);
    return p;
}

}  // namespace

struct pgcm_key {
    int device = -1;
    int num_cu = 0;
    KeyTables* tables = nullptr;  // device
    // descriptor staging: pinned host buffers used in turn, each guarded by an event that marks
    // the end of its last upload
    uint8_t* stage[kStages] = {nullptr, nullptr};
    size_t stage_cap[kStages] = {0, 0};
    hipEvent_t stage_done[kStages] = {nullptr, nullptr};
    bool stage_used[kStages] = {false, false};
    int next_stage = 0;
    // device workspace: descriptors, item map, per-segment partial hashes, per-chunk AAD states
    uint8_t* work = nullptr;
    size_t work_cap = 0;
    // optional timing of the bulk kernel alone (pgcm_set_timing)
    bool timing = false;
    bool timed = false;
    hipEvent_t bulk_start = nullptr, bulk_stop = nullptr;
};

namespace {

int ensure_stage(pgcm_key* k, int s, size_t bytes) {
    if (k->stage_used[s]) {
        PGCM_HIP(hipEventSynchronize(k->stage_done[s]));
        k->stage_used[s] = false;
    }
    if (k->stage_cap[s] >= bytes) return PGCM_OK;
    if (k->stage[s]) {
        PGCM_HIP(hipHostFree(k->stage[s]));
        k->stage[s] = nullptr;
        k->stage_cap[s] = 0;
    }
    size_t cap = bytes + bytes / 2 + 4096;
    void* p = nullptr;
    if (hip_failed(hipHostMalloc(&p, cap, hipHostMallocDefault))) return PGCM_ERR_NOMEM;
    k->stage[s] = (uint8_t*)p;
    k->stage_cap[s] = cap;
    return PGCM_OK;
}

int ensure_work(pgcm_key* k, size_t bytes, hipStream_t stream) {
    if (k->work_cap >= bytes) return PGCM_OK;
    if (k->work) {
        // earlier batches on this stream may still read the old workspace
        PGCM_HIP(hipStreamSynchronize(stream));
        PGCM_HIP(hipFree(k->work));
        k->work = nullptr;
        k->work_cap = 0;
    }
    size_t cap = bytes + bytes / 2 + 65536;
    void* p = nullptr;
    if (hip_failed(hipMalloc(&p, cap))) return PGCM_ERR_NOMEM;
    k->work = (uint8_t*)p;
    k->work_cap = cap;
    return PGCM_OK;
}

inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

int run_batch(bool decrypt, pgcm_key* key, size_t n, const uint8_t* ivs, const void* const* aad,
              const uint32_t* aad_len, const void* const* src, const uint64_t* len,
              void* const* dst, uint8_t* tags, uint8_t* ok, void* hip_stream) {
    if (key == nullptr || key->tables == nullptr) return PGCM_ERR_ARG;
    if (n == 0) return PGCM_OK;
    if (ivs == nullptr || src == nullptr || len == nullptr || dst == nullptr || tags == nullptr)
        return PGCM_ERR_ARG;
    if ((aad == nullptr) != (aad_len == nullptr)) return PGCM_ERR_ARG;
    if (decrypt && ok == nullptr) return PGCM_ERR_ARG;
    if (n > 0x7FFFFFFFull) return PGCM_ERR_ARG;

    // validate everything before touching any state
    uint64_t nitems64 = 0;
    bool any_aad = false;
    for (size_t i = 0; i < n; ++i) {
        if (len[i] > PGCM_MAX_CHUNK_BYTES) return PGCM_ERR_LEN;
        if (len[i] != 0) {
            if (src[i] == nullptr || dst[i] == nullptr) return PGCM_ERR_ARG;
            if (((uintptr_t)src[i] | (uintptr_t)dst[i]) & 15) return PGCM_ERR_ALIGN;
        }
        if (aad_len != nullptr && aad_len[i] != 0) {
            if (aad[i] == nullptr) return PGCM_ERR_ARG;
            any_aad = true;
        }
        nitems64 += plan_chunk(len[i]).nseg;
    }
    if (nitems64 > 0xFFFFFFF0ull) return PGCM_ERR_ARG;
    const uint32_t nitems = (uint32_t)nitems64;
    const uint32_t nchunks = (uint32_t)n;

    hipStream_t stream = (hipStream_t)hip_stream;
    int prev_device = -1;
    PGCM_HIP(hipGetDevice(&prev_device));
    if (prev_device != key->device) return PGCM_ERR_ARG;  // the key lives on another GPU

    // workspace layout (device and staging share the first two regions)
    const size_t off_desc = 0;
    const size_t off_items = round_up(off_desc + sizeof(ChunkDesc) * n, 256);
    const size_t upload_bytes = round_up(off_items + sizeof(uint32_t) * (size_t)nitems, 256);
    const size_t off_partials = upload_bytes;
    const size_t off_aad = round_up(off_partials + sizeof(Block) * (size_t)nitems, 256);
    const size_t work_bytes = off_aad + sizeof(Block) * n;

    const int s = key->next_stage;
    int rc = ensure_stage(key, s, upload_bytes);
    if (rc != PGCM_OK) return rc;
    rc = ensure_work(key, work_bytes, stream);
    if (rc != PGCM_OK) return rc;

    ChunkDesc* h_desc = reinterpret_cast<ChunkDesc*>(key->stage[s] + off_desc);
    uint32_t* h_items = reinterpret_cast<uint32_t*>(key->stage[s] + off_items);
    uint32_t item = 0;
    for (size_t i = 0; i < n; ++i) {
        SegPlan p = plan_chunk(len[i]);
        ChunkDesc& d = h_desc[i];
        d.src = (const uint8_t*)src[i];
        d.dst = (uint8_t*)dst[i];
        d.len = len[i];
        d.aad_len = aad_len ? aad_len[i] : 0;
        d.aad = d.aad_len ? (const uint8_t*)aad[i] : nullptr;
        d.part_base = item;
        d.nseg = p.nseg;
        d.first_blocks = p.first_blocks;
        for (uint32_t k = 0; k < p.nseg; ++k) h_items[item++] = (uint32_t)i;
    }

    PGCM_HIP(hipMemcpyAsync(key->work, key->stage[s], upload_bytes, hipMemcpyHostToDevice, stream));
    PGCM_HIP(hipEventRecord(key->stage_done[s], stream));
    key->stage_used[s] = true;
    key->next_stage = (s + 1) % kStages;

    const ChunkDesc* d_desc = reinterpret_cast<const ChunkDesc*>(key->work + off_desc);
    const uint32_t* d_items = reinterpret_cast<const uint32_t*>(key->work + off_items);
    Block* d_partials = reinterpret_cast<Block*>(key->work + off_partials);
    Block* d_aad = any_aad ? reinterpret_cast<Block*>(key->work + off_aad) : nullptr;

    if (any_aad) {
        hipLaunchKernelGGL(aad_state_kernel, dim3((nchunks + 63) / 64), dim3(64), 0, stream,
                           key->tables, d_desc, nchunks, d_aad);
    }
    if (nitems > 0) {
        uint32_t groups = (nitems + kWavesPerGroup - 1) / kWavesPerGroup;
        if (groups > (uint32_t)key->num_cu) groups = (uint32_t)key->num_cu;
        if (key->timing) PGCM_HIP(hipEventRecord(key->bulk_start, stream));
        if (decrypt)
            hipLaunchKernelGGL(bulk_kernel<true>, dim3(groups), dim3(kGroupThreads), 0, stream,
                               key->tables, d_desc, d_items, nitems, ivs, d_aad, d_partials);
        else
            hipLaunchKernelGGL(bulk_kernel<false>, dim3(groups), dim3(kGroupThreads), 0, stream,
                               key->tables, d_desc, d_items, nitems, ivs, d_aad, d_partials);
        if (key->timing) {
            PGCM_HIP(hipEventRecord(key->bulk_stop, stream));
            key->timed = true;
        }
    }
    if (decrypt) {
        hipLaunchKernelGGL(finalize_kernel<true>, dim3((nchunks + 63) / 64), dim3(64), 0, stream,
                           key->tables, d_desc, nchunks, ivs, d_aad, d_partials, tags, ok);
        uint32_t wipers = nchunks < 1024 ? nchunks : 1024;
        hipLaunchKernelGGL(wipe_rejected_kernel, dim3(wipers), dim3(256), 0, stream, d_desc,
                           nchunks, ok);
    } else {
        hipLaunchKernelGGL(finalize_kernel<false>, dim3((nchunks + 63) / 64), dim3(64), 0, stream,
                           key->tables, d_desc, nchunks, ivs, d_aad, d_partials, tags, nullptr);
    }
    PGCM_HIP(hipGetLastError());
    return PGCM_OK;
}

}  // namespace

extern "C" {
#pragma GCC visibility push(default)

int pgcm_expand_key(const uint8_t key[32], void* hip_stream, pgcm_key_t** out) {
    if (key == nullptr || out == nullptr) return PGCM_ERR_ARG;
    *out = nullptr;
    pgcm_key* k = new (std::nothrow) pgcm_key();
    if (k == nullptr) return PGCM_ERR_NOMEM;
    hipStream_t stream = (hipStream_t)hip_stream;
    int rc = PGCM_OK;
    uint32_t* d_key = nullptr;
    do {
        if (hip_failed(hipGetDevice(&k->device))) { rc = PGCM_ERR_HIP; break; }
        if (hip_failed(hipDeviceGetAttribute(&k->num_cu, hipDeviceAttributeMultiprocessorCount,
                                             k->device))) { rc = PGCM_ERR_HIP; break; }
        if (k->num_cu < 1) k->num_cu = 1;
        if (hip_failed(hipMalloc((void**)&k->tables, sizeof(KeyTables)))) { rc = PGCM_ERR_NOMEM; break; }
        if (hip_failed(hipMalloc((void**)&d_key, 32))) { rc = PGCM_ERR_NOMEM; break; }
        for (int s = 0; s < kStages; ++s)
            if (hip_failed(hipEventCreateWithFlags(&k->stage_done[s], hipEventDisableTiming))) {
                rc = PGCM_ERR_HIP;
                break;
            }
        if (rc != PGCM_OK) break;
        // a 32-byte pageable copy: staged by the runtime, complete on return for this size
        if (hip_failed(hipMemcpyAsync(d_key, key, 32, hipMemcpyHostToDevice, stream))) { rc = PGCM_ERR_HIP; break; }
        hipLaunchKernelGGL(expand_key_kernel, dim3(1), dim3(1024), 0, stream, k->tables, d_key);
        if (hip_failed(hipGetLastError())) { rc = PGCM_ERR_HIP; break; }
        if (hip_failed(hipMemsetAsync(d_key, 0, 32, stream))) { rc = PGCM_ERR_HIP; break; }
        if (hip_failed(hipStreamSynchronize(stream))) { rc = PGCM_ERR_HIP; break; }
    } while (0);
    if (d_key) (void)hipFree(d_key);
    if (rc != PGCM_OK) {
        pgcm_free_key(k);
        return rc;
    }
    *out = k;
    return PGCM_OK;
}

void pgcm_free_key(pgcm_key_t* k) {
    if (k == nullptr) return;
    if (k->tables) {
        (void)hipMemset(k->tables, 0, sizeof(KeyTables));
        (void)hipFree(k->tables);
    }
    if (k->work) (void)hipFree(k->work);
    for (int s = 0; s < kStages; ++s) {
        if (k->stage[s]) (void)hipHostFree(k->stage[s]);
        if (k->stage_done[s]) (void)hipEventDestroy(k->stage_done[s]);
    }
    if (k->bulk_start) (void)hipEventDestroy(k->bulk_start);
    if (k->bulk_stop) (void)hipEventDestroy(k->bulk_stop);
    delete k;
}

int pgcm_encrypt_batch(pgcm_key_t* key, size_t n, const uint8_t* ivs, const void* const* aad,
                       const uint32_t* aad_len, const void* const* src, const uint64_t* len,
                       void* const* dst, uint8_t* tags, void* hip_stream) {
    return run_batch(false, key, n, ivs, aad, aad_len, src, len, dst, tags, nullptr, hip_stream);
}

int pgcm_decrypt_verify_batch(pgcm_key_t* key, size_t n, const uint8_t* ivs,
                              const void* const* aad, const uint32_t* aad_len,
                              const void* const* src, const uint64_t* len, void* const* dst,
                              const uint8_t* tags, uint8_t* ok, void* hip_stream) {
    return run_batch(true, key, n, ivs, aad, aad_len, src, len, dst, const_cast<uint8_t*>(tags), ok,
                     hip_stream);
}

const char* pgcm_strerror(int status) {
    switch (status) {
        case PGCM_OK: return "success";
        case PGCM_ERR_ARG: return "invalid argument";
        case PGCM_ERR_ALIGN: return "src or dst pointer not 16-byte aligned";
        case PGCM_ERR_LEN: return "chunk longer than the GCM limit of 2^36 - 32 bytes";
        case PGCM_ERR_NOMEM: return "out of host or device memory";
        case PGCM_ERR_HIP: return "a HIP runtime call failed";
        default: return "unknown status";
    }
}

int pgcm_last_hip_error(void) { return g_last_hip_error; }

int64_t pgcm_plan_segments(size_t n, const uint64_t* len, uint32_t* nseg, uint32_t* first_blocks,
                           uint32_t* part_base) {
    if (n != 0 && len == nullptr) return PGCM_ERR_ARG;
    uint64_t total = 0;
    for (size_t i = 0; i < n; ++i) {
        if (len[i] > PGCM_MAX_CHUNK_BYTES) return PGCM_ERR_LEN;
        SegPlan p = plan_chunk(len[i]);
        if (nseg) nseg[i] = p.nseg;
        if (first_blocks) first_blocks[i] = p.first_blocks;
        if (part_base) part_base[i] = (uint32_t)total;
        total += p.nseg;
        if (total > 0xFFFFFFF0ull) return PGCM_ERR_ARG;
    }
    return (int64_t)total;
}

uint32_t pgcm_segment_bytes(void) { return kSegBytes; }

int pgcm_set_timing(pgcm_key_t* key, int enable) {
    if (key == nullptr) return PGCM_ERR_ARG;
    if (enable && key->bulk_start == nullptr) {
        PGCM_HIP(hipEventCreate(&key->bulk_start));
        PGCM_HIP(hipEventCreate(&key->bulk_stop));
    }
    key->timing = enable != 0;
    key->timed = false;
    return PGCM_OK;
}

int pgcm_last_bulk_kernel_ms(pgcm_key_t* key, float* ms) {
    if (key == nullptr || ms == nullptr || !key->timed) return PGCM_ERR_ARG;
    PGCM_HIP(hipEventSynchronize(key->bulk_stop));
    PGCM_HIP(hipEventElapsedTime(ms, key->bulk_start, key->bulk_stop));
    return PGCM_OK;
}

#pragma GCC visibility pop
}  // extern "C"
