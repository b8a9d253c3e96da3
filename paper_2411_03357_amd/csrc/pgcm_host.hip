// Host side of libpgcm: the C ABI of include/pgcm.h — argument checks, the chunk-to-wavefront
// schedule, descriptor upload and kernel launches.  No cipher arithmetic happens on the host.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#include <chrono>
#include <mutex>
#include <new>
#include <vector>

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

// descriptor staging buffers a context uses in turn; a buffer is free again once the batch that
// used it has ended on its stream, so this is how many batches the host may run ahead of the GPU
constexpr int kStages = 4;
constexpr uint32_t kTimingRing = 256;
// contexts a key keeps before it starts re-binding the least recently used one to a new stream
constexpr size_t kMaxContexts = 16;
// limits of the entry point that allocates nothing (pgcm_encrypt_batch_static)
constexpr size_t kScratchBytes = PGCM_STATIC_WORKSPACE_BYTES;
constexpr size_t kFixedMaxChunks = PGCM_STATIC_MAX_CHUNKS;
constexpr int kMaxDevices = 64;
// a fold level with at most this many items (one workgroup each fits the chip at once) is folded
// by the tree kernel
constexpr uint32_t kFoldTreeMaxItems = 256;

// Per-chunk schedule: units are counted back from the chunk's end, so that every unit but the
// first is full and all row boundaries line up with the end of the chunk.
struct UnitPlan {
    uint32_t nunits, first_blocks;
};

inline UnitPlan plan_chunk(uint64_t len, uint32_t unit_power) {
    uint64_t nblk = (len + 15) / 16;
    UnitPlan p{0, 0};
    if (nblk == 0) return p;
    uint64_t nunits = (nblk + ((uint64_t)1 << unit_power) - 1) >> unit_power;
    p.nunits = (uint32_t)nunits;
    p.first_blocks = (uint32_t)(nblk - ((nunits - 1) << unit_power));
    return p;
}

// Partial sets of a chunk are folded kFan at a time until at most kFan remain for the final
// step.  Returns the number of fold levels and, per level, the number of sets it produces.
// More than kMaxLevels levels (only possible when a small unit is forced on a huge chunk) is
// reported as kMaxLevels + 1 with nothing written past the array.
inline uint32_t fold_levels(uint32_t nunits, uint32_t out_counts[kMaxLevels]) {
    uint32_t levels = 0, c = nunits;
    while (c > kFan) {
        if (levels == kMaxLevels) return kMaxLevels + 1;
        c = (c + kFan - 1) / kFan;
        out_counts[levels++] = c;
    }
    return levels;
}

// Unit size of a batch: the smallest, from one row up, with which the batch has at most
// wave_slots units (the wavefronts the device holds at once: sixteen per compute unit), so that
// every unit gets a wavefront of its own at once; kUnitPower and the dynamic schedule when even
// that leaves more.  (Larger units that would again give every
// wavefront exactly one unit, e.g. a whole 320 KiB block each for 4096 of them, can be forced but
// are never chosen: wavefronts do not all run at the same speed, and a launch that cannot hand
// the slow ones less work ends when its slowest wavefront does.)  `order` as for run_batch.
inline uint32_t choose_unit_power(size_t n, const uint32_t* order, const uint64_t* len,
                                  uint32_t wave_slots) {
    constexpr uint32_t kChoices = kUnitPower - kMinUnitPower + 1;
    uint64_t units[kChoices] = {};
    for (size_t k = 0; k < n; ++k) {
        const uint64_t l = len[order ? order[k] : k];
        if (l > PGCM_MAX_CHUNK_BYTES) return kUnitPower;  // rejected later
        const uint64_t nblk = (l + 15) / 16;
        for (uint32_t c = 0; c < kChoices; ++c) {
            const uint32_t u = kMinUnitPower + c;
            units[c] += (nblk + ((uint64_t)1 << u) - 1) >> u;
        }
        if (units[kChoices - 1] > wave_slots) return kUnitPower;
    }
    for (uint32_t c = 0; c < kChoices; ++c)
        if (units[c] <= wave_slots) return kMinUnitPower + c;
    return kUnitPower;
}

}  // namespace

namespace {

// What one batch in flight needs besides the key's tables: pinned staging buffers for the
// descriptors the host writes, and the device workspace the kernels of the batch share.  Batches
// that use one context are ordered by the stream the context is bound to, which is what makes
// reusing its buffers from batch to batch safe; batches on different streams (or from different
// host threads) take different contexts.
struct Context {
    bool growable = true;   // false: the buffers are fixed and a batch that needs more is refused
    uint8_t* stage[kStages] = {};
    size_t stage_cap[kStages] = {};
    hipEvent_t stage_done[kStages] = {};  // end of the batch that last used the buffer
    bool stage_used[kStages] = {};
    int next_stage = 0;
    // device workspace: descriptors, unit maps, fold lists, unit counter, per-chunk E_K(J0),
    // partial sets
    uint8_t* work = nullptr;
    size_t work_cap = 0;
    uint32_t* counter_at = nullptr;  // where the unit counter was last known to be zero
    bool counter_dirty = true;
    bool arrive_clean = false;  // the one-launch path's arrival words (start of `work`) are zero
    // binding
    hipStream_t stream = nullptr;
    bool bound = false;        // has run a batch on `stream`
    bool in_call = false;      // a host thread is inside a batch call with it
    int last_stage = -1;       // stage whose event marks the end of its most recent batch
    uint64_t last_use = 0;
};

}  // namespace

struct pgcm_key {
    int device = -1;
    int num_cu = 0;
    uint32_t wave_slots = kWaveSlots;  // wavefronts the device holds at once: 16 per CU
    int rounds = 0;  // 10, 12 or 14
    uint32_t forced_unit_power = 0;  // 0: chosen per batch
    bool one_launch = true;          // batches of few chunks that do not fill the chip: one kernel
    bool matrix_hash = false;        // unit kernel: GHASH row multiplication on the matrix cores
    KeyTables* tables = nullptr;  // device
    std::mutex mu;                 // guards `contexts` and the binding fields of each context
    std::vector<Context*> contexts;
    uint64_t use_tick = 0;
    // the context of the entry point that allocates nothing: fixed staging buffers, and the
    // device's static scratch array as workspace
    Context fixed;
    bool fixed_used = false;
    // optional timing of the bulk kernel alone (pgcm_set_timing)
    // a ring of event pairs, one pair per timed launch, so that a run of batches can be timed
    // without a host wait in between
    bool timing = false;
    uint64_t timed = 0;  // launches timed since timing was switched on
    hipEvent_t bulk_start[kTimingRing] = {}, bulk_stop[kTimingRing] = {};
};

// Device workspace of the entry point that allocates nothing: one array per GPU, held from the
// moment the library is loaded until the process ends, shared by every such call on that GPU.
// Host code must never pass this name to a kernel: the address the device sees comes from
// hipGetSymbolAddress (scratch_of_device) and is what the kernels get.
static __device__ __align__(256) uint8_t scratch[kScratchBytes];

namespace {

std::mutex g_scratch_mu;
uint8_t* g_scratch_ptr[kMaxDevices] = {};

// Address of `scratch` on `device`, which must be the current device; looked up once per device.
int scratch_of_device(int device, uint8_t** out) {
    if (device < 0 || device >= kMaxDevices) return PGCM_ERR_ARG;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (g_scratch_ptr[device] == nullptr) {
        void* p = nullptr;
        PGCM_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (p == nullptr) return PGCM_ERR_HIP;
        g_scratch_ptr[device] = static_cast<uint8_t*>(p);
    }
    *out = g_scratch_ptr[device];
    return PGCM_OK;
}

int create_stage_events(Context* c) {
    for (int s = 0; s < kStages; ++s)
        PGCM_HIP(hipEventCreateWithFlags(&c->stage_done[s], hipEventDisableTiming));
    return PGCM_OK;
}

void destroy_context(Context* c, bool wipe_work) {
    if (c->work && c->growable) {
        // the workspace holds key-dependent values (tag masks, partial hashes)
        if (wipe_work) (void)hipMemset(c->work, 0, c->work_cap);
        (void)hipFree(c->work);
    }
    for (int s = 0; s < kStages; ++s) {
        if (c->stage[s]) {
            memset(c->stage[s], 0, c->stage_cap[s]);
            (void)hipHostFree(c->stage[s]);
        }
        if (c->stage_done[s]) (void)hipEventDestroy(c->stage_done[s]);
    }
}

// Makes stage s of the context free (waits for the batch that last used it) and at least `bytes`
// large.
int ensure_stage(Context* c, int s, size_t bytes) {
    if (c->stage_used[s]) {
        PGCM_HIP(hipEventSynchronize(c->stage_done[s]));
        c->stage_used[s] = false;
    }
    if (c->stage_cap[s] >= bytes) return PGCM_OK;
    if (!c->growable) return PGCM_ERR_CAPACITY;
    if (c->stage[s]) {
        PGCM_HIP(hipHostFree(c->stage[s]));
        c->stage[s] = nullptr;
        c->stage_cap[s] = 0;
    }
    size_t cap = bytes + bytes / 2 + 4096;
    void* p = nullptr;
    if (hip_failed(hipHostMalloc(&p, cap, hipHostMallocDefault))) return PGCM_ERR_NOMEM;
    c->stage[s] = (uint8_t*)p;
    c->stage_cap[s] = cap;
    return PGCM_OK;
}

int ensure_work(Context* c, size_t bytes, hipStream_t stream) {
    if (c->work_cap >= bytes) return PGCM_OK;
    if (!c->growable) return PGCM_ERR_CAPACITY;
    if (c->work) {
        // earlier batches on this stream may still read the old workspace
        PGCM_HIP(hipStreamSynchronize(stream));
        PGCM_HIP(hipFree(c->work));
        c->work = nullptr;
        c->work_cap = 0;
    }
    c->counter_at = nullptr;  // new memory holds anything, even if it lands at the old address
    c->arrive_clean = false;
    size_t cap = bytes + bytes / 2 + 65536;
    void* p = nullptr;
    if (hip_failed(hipMalloc(&p, cap))) return PGCM_ERR_NOMEM;
    c->work = (uint8_t*)p;
    c->work_cap = cap;
    return PGCM_OK;
}

// The context a batch on `stream` runs with.  In order of preference: a context already bound to
// the stream; one whose last batch has ended (it is re-bound); a new one; and, once the key has
// kMaxContexts of them, the least recently used one, after waiting for its last batch.  Contexts
// that another host thread is using at this moment are never taken.
int acquire_context(pgcm_key* key, hipStream_t stream, Context** out) {
    std::unique_lock<std::mutex> lock(key->mu);
    Context* pick = nullptr;
    for (Context* c : key->contexts)
        if (!c->in_call && c->bound && c->stream == stream) { pick = c; break; }
    bool must_wait = false;
    if (pick == nullptr) {
        Context* lru = nullptr;
        for (Context* c : key->contexts) {
            if (c->in_call) continue;
            // free for re-binding: never bound, or its last batch has ended.  (A context that
            // pgcm_reserve has bound and no batch has used yet is left for its stream.)
            if (!c->bound || (c->last_stage >= 0 &&
                              hipEventQuery(c->stage_done[c->last_stage]) == hipSuccess)) {
                pick = c;
                break;
            }
            if (lru == nullptr || c->last_use < lru->last_use) lru = c;
        }
        (void)hipGetLastError();  // a query that said "not ready" is not an error of this call
        if (pick == nullptr && lru != nullptr && key->contexts.size() >= kMaxContexts) {
            pick = lru;
            must_wait = pick->last_stage >= 0;
        }
    }
    if (pick == nullptr) {
        Context* c = new (std::nothrow) Context();
        if (c == nullptr) return PGCM_ERR_NOMEM;
        int rc = create_stage_events(c);
        if (rc == PGCM_OK) {
            try {
                key->contexts.push_back(c);
            } catch (const std::bad_alloc&) {
                rc = PGCM_ERR_NOMEM;
            }
        }
        if (rc != PGCM_OK) {
            destroy_context(c, false);
            delete c;
            return rc;
        }
        pick = c;
    }
    pick->in_call = true;
    pick->last_use = ++key->use_tick;
    lock.unlock();
    if (pick->bound && pick->stream != stream) {
        // re-binding: everything it enqueued on its old stream must have ended
        if (must_wait && hip_failed(hipEventSynchronize(pick->stage_done[pick->last_stage]))) {
            std::lock_guard<std::mutex> relock(key->mu);
            pick->in_call = false;
            return PGCM_ERR_HIP;
        }
        for (int s = 0; s < kStages; ++s) pick->stage_used[s] = false;
    }
    pick->stream = stream;
    *out = pick;
    return PGCM_OK;
}

void release_context(pgcm_key* key, Context* c) {
    if (c == &key->fixed) return;
    std::lock_guard<std::mutex> lock(key->mu);
    c->in_call = false;
}

// marks the end of a batch that used stage s of the context
int end_of_batch(Context* c, int s, hipStream_t stream) {
    PGCM_HIP(hipEventRecord(c->stage_done[s], stream));
    c->stage_used[s] = true;
    c->last_stage = s;
    c->bound = true;
    c->next_stage = (s + 1) % kStages;
    return PGCM_OK;
}

constexpr size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// the kernels that run the cipher are compiled once per round count
template <bool kDecrypt, bool kMatrixHash, class... Args>
void launch_bulk_rounds(int rounds, dim3 grid, hipStream_t stream, Args... args) {
    if (rounds == 10)
        hipLaunchKernelGGL((bulk_kernel<kDecrypt, 10, kMatrixHash>), grid, dim3(kGroupThreads), 0,
                           stream, args...);
    else if (rounds == 12)
        hipLaunchKernelGGL((bulk_kernel<kDecrypt, 12, kMatrixHash>), grid, dim3(kGroupThreads), 0,
                           stream, args...);
    else
        hipLaunchKernelGGL((bulk_kernel<kDecrypt, 14, kMatrixHash>), grid, dim3(kGroupThreads), 0,
                           stream, args...);
}

// ... and once per engine of the row hash (matrix cores or LDS tables)
template <bool kDecrypt, class... Args>
void launch_bulk(int rounds, bool matrix_hash, dim3 grid, hipStream_t stream, Args... args) {
    if (matrix_hash)
        launch_bulk_rounds<kDecrypt, true>(rounds, grid, stream, args...);
    else
        launch_bulk_rounds<kDecrypt, false>(rounds, grid, stream, args...);
}

template <bool kDecrypt, class... Args>
void launch_swap(int rounds, dim3 grid, hipStream_t stream, Args... args) {
    if (rounds == 10)
        hipLaunchKernelGGL((swap_kernel<kDecrypt, 10>), grid, dim3(kGroupThreads), 0, stream, args...);
    else if (rounds == 12)
        hipLaunchKernelGGL((swap_kernel<kDecrypt, 12>), grid, dim3(kGroupThreads), 0, stream, args...);
    else
        hipLaunchKernelGGL((swap_kernel<kDecrypt, 14>), grid, dim3(kGroupThreads), 0, stream, args...);
}

// wide: a workgroup of eight wavefronts per chunk; otherwise a wavefront per chunk
template <bool kDecrypt, class... Args>
void launch_small(int rounds, bool wide, uint32_t nchunks, hipStream_t stream, Args... args) {
    if (wide) {
        const dim3 grid(nchunks), block(kSmallWideWaves * 64);
        if (rounds == 10)
            hipLaunchKernelGGL((small_wide_kernel<kDecrypt, 10>), grid, block, 0, stream, args...);
        else if (rounds == 12)
            hipLaunchKernelGGL((small_wide_kernel<kDecrypt, 12>), grid, block, 0, stream, args...);
        else
            hipLaunchKernelGGL((small_wide_kernel<kDecrypt, 14>), grid, block, 0, stream, args...);
        return;
    }
    const dim3 grid((nchunks + kSmallChunksPerGroup - 1) / kSmallChunksPerGroup);
    const dim3 block(kSmallChunksPerGroup * 64);
    if (rounds == 10)
        hipLaunchKernelGGL((small_kernel<kDecrypt, 10>), grid, block, 0, stream, args...);
    else if (rounds == 12)
        hipLaunchKernelGGL((small_kernel<kDecrypt, 12>), grid, block, 0, stream, args...);
    else
        hipLaunchKernelGGL((small_kernel<kDecrypt, 14>), grid, block, 0, stream, args...);
}

// The caller's arrays of one batch call.  `order` (may be null) picks the batch's chunks out of
// them: chunk k of the batch is the caller's chunk order[k]; null means 0, 1, .., n - 1.
struct BatchArgs {
    bool decrypt;
    size_t n;
    const uint32_t* order;
    const uint8_t* ivs;
    uint32_t iv_len;
    const void* const* aad;
    const uint32_t* aad_len;
    const void* const* src;
    const uint64_t* len;
    void* const* dst;
    uint8_t* tags;
    uint8_t* ok;
    hipStream_t stream;
    bool fixed = false;  // run in the key's fixed context: allocate nothing, refuse what does not fit

    size_t at(size_t k) const { return order ? order[k] : k; }
};

// what must hold for the arrays of a batch as a whole
int check_batch(const BatchArgs& a) {
    if (a.iv_len == 0) return PGCM_ERR_ARG;  // GCM takes no empty IV
    if (a.n == 0) return PGCM_OK;
    if (a.ivs == nullptr || a.src == nullptr || a.len == nullptr || a.dst == nullptr ||
        a.tags == nullptr)
        return PGCM_ERR_ARG;
    if ((a.aad == nullptr) != (a.aad_len == nullptr)) return PGCM_ERR_ARG;
    if (a.decrypt && a.ok == nullptr) return PGCM_ERR_ARG;
    if (a.n > 0x7FFFFFFFull) return PGCM_ERR_ARG;
    return PGCM_OK;
}

// ... and for the caller's chunk i
inline int check_chunk(const BatchArgs& a, size_t i) {
    if (a.len[i] > PGCM_MAX_CHUNK_BYTES) return PGCM_ERR_LEN;
    if (a.len[i] != 0) {
        if (a.src[i] == nullptr || a.dst[i] == nullptr) return PGCM_ERR_ARG;
        if (((uintptr_t)a.src[i] | (uintptr_t)a.dst[i]) & 15) return PGCM_ERR_ALIGN;
    }
    if (a.aad_len != nullptr && a.aad_len[i] != 0 && a.aad[i] == nullptr) return PGCM_ERR_ARG;
    return PGCM_OK;
}

inline void describe_chunk(const BatchArgs& a, size_t i, ChunkDesc& d) {
    memset(&d, 0, sizeof(d));
    d.src = (const uint8_t*)a.src[i];
    d.dst = (uint8_t*)a.dst[i];
    d.len = a.len[i];
    d.aad_len = a.aad_len ? a.aad_len[i] : 0;
    d.aad = d.aad_len ? (const uint8_t*)a.aad[i] : nullptr;
    d.index = (uint32_t)i;
}

// Sizes of a batch's schedule; filled by plan_batch, which also validates every chunk.
struct BatchPlan {
    bool all_small;       // every chunk fits the small-transfer path
    bool all_one_row;     // ... and its one-wavefront-per-chunk kernel
    uint32_t unit_power;  // log2 of the blocks per unit
    uint32_t nunits;
    uint32_t max_units;   // the most units any one chunk has
    uint32_t nslots;      // partial sets: one per unit and one per fold output
    uint32_t fold_count[kMaxLevels], fold_first[kMaxLevels], nfold;
    uint32_t ncoarse;
};

// forced_unit_power: 0 = chosen for the batch; wave_slots: see choose_unit_power
int plan_batch(uint32_t forced_unit_power, uint32_t wave_slots, const BatchArgs& a,
               BatchPlan* plan) {
    plan->unit_power = forced_unit_power ? forced_unit_power
                                         : choose_unit_power(a.n, a.order, a.len, wave_slots);
    plan->all_small = plan->all_one_row = true;
    uint64_t nunits = 0, nslots = 0;
    plan->max_units = 0;
    uint64_t fold_items[kMaxLevels] = {0, 0, 0, 0};
    for (size_t k = 0; k < a.n; ++k) {
        const size_t i = a.at(k);
        const int rc = check_chunk(a, i);
        if (rc != PGCM_OK) return rc;
        if (a.len[i] > kSmallChunkBytes) plan->all_small = false;
        if (a.len[i] > kSmallRowBytes) plan->all_one_row = false;
        const uint32_t nu = plan_chunk(a.len[i], plan->unit_power).nunits;
        uint32_t outs[kMaxLevels];
        const uint32_t levels = fold_levels(nu, outs);
        // a forced unit the chunk cannot be cut into: too many fold levels, or sets of the last
        // step further apart than the largest power of H with a table
        if (levels > kMaxLevels || plan->unit_power + kFanPower * levels >= kNumPowers)
            return PGCM_ERR_LEN;
        nunits += nu;
        nslots += nu;
        if (nu > plan->max_units) plan->max_units = nu;
        for (uint32_t l = 0; l < levels; ++l) {
            fold_items[l] += outs[l];
            nslots += outs[l];
        }
    }
    if (nslots > 0xFFFFFFF0ull / 64) return PGCM_ERR_ARG;  // set indices are 32-bit
    plan->nunits = (uint32_t)nunits;
    plan->nslots = (uint32_t)nslots;
    plan->nfold = 0;
    for (uint32_t l = 0; l < kMaxLevels; ++l) {
        plan->fold_count[l] = (uint32_t)fold_items[l];
        plan->fold_first[l] = plan->nfold;
        plan->nfold += plan->fold_count[l];
    }
    plan->ncoarse = (plan->nunits >> kCoarseShift) + 1;
    return PGCM_OK;
}

// Byte offsets of the regions of the device workspace.  The regions up to upload_bytes are
// written by the host into a staging buffer of the same layout and uploaded.
struct WorkLayout {
    size_t desc, ubase, coarse, fold, upload_bytes, counter, ekj0, j0, sets, bytes;
};

WorkLayout lay_out(const BatchArgs& a, const BatchPlan& p) {
    WorkLayout w;
    w.desc = 0;
    w.ubase = round_up(w.desc + sizeof(ChunkDesc) * a.n, 256);
    w.coarse = round_up(w.ubase + sizeof(uint32_t) * (a.n + 1), 256);
    w.fold = round_up(w.coarse + sizeof(uint32_t) * (size_t)p.ncoarse, 256);
    w.upload_bytes = round_up(w.fold + sizeof(FoldItem) * (size_t)p.nfold, 256);
    w.counter = w.upload_bytes;
    w.ekj0 = w.counter + 256;
    w.j0 = w.ekj0 + sizeof(Block) * a.n;  // pre-counter blocks: only for IVs not 96 bits long
    w.sets = round_up(w.j0 + (a.iv_len == 12 ? 0 : sizeof(Block) * a.n), 1024);
    w.bytes = w.sets + sizeof(Block) * 64 * (size_t)p.nslots;
    return w;
}

// Upper bounds of a batch's staging and workspace bytes, for any batch of at most n chunks with
// at most `bytes` bytes of payload in all.  False when the numbers are out of range.
bool worst_case_sizes(uint32_t forced_unit_power, uint32_t wave_slots, size_t n, uint64_t bytes,
                      size_t* stage_bytes, size_t* work_bytes) {
    // units: with the unit chosen per batch a batch either has at most wave_slots units or is cut
    // into full-size units, each chunk adding at most one short unit
    const uint32_t up = forced_unit_power ? forced_unit_power : kUnitPower;
    uint64_t units = (bytes >> (up + 4)) + n;
    if (!forced_unit_power && units < wave_slots) units = wave_slots;
    // every fold level leaves at most units / 32 + n sets; four levels
    const uint64_t folds = units / (kFan - 1) + kMaxLevels * (uint64_t)n + 1;
    const uint64_t slots = units + folds;
    if (slots > 0xFFFFFFF0ull / 64 || n > 0x7FFFFFFFull) return false;
    BatchArgs a{};
    a.n = n;
    a.iv_len = 16;  // any length but 12: room for the pre-counter blocks as well
    BatchPlan p{};
    p.nunits = (uint32_t)units;
    p.nslots = (uint32_t)slots;
    p.nfold = (uint32_t)folds;
    p.ncoarse = (p.nunits >> kCoarseShift) + 1;
    const WorkLayout w = lay_out(a, p);
    const size_t small = sizeof(ChunkDesc) * n;  // the small-transfer path stages descriptors only
    *stage_bytes = w.upload_bytes > small ? w.upload_bytes : small;
    *work_bytes = w.bytes;
    return true;
}

// Staging bytes any batch can need that passes the fixed context's other limits: at most
// kFixedMaxChunks descriptors and unit-map entries, and a coarse map and fold list for at most
// kScratchBytes / 1024 partial sets.
constexpr size_t kFixedStageBytes = round_up(
    (sizeof(ChunkDesc) * kFixedMaxChunks + 256) + (4 * (kFixedMaxChunks + 1) + 256) +
        (4 * (kScratchBytes / 1024 / 16 + 1) + 256) +
        (sizeof(FoldItem) * (kScratchBytes / 1024) + 256),
    4096);  // the staging buffers are slices of one block: each must start aligned

// Descriptors, unit maps and fold lists of the batch, written into the staging buffer.
void fill_schedule(const BatchArgs& a, const BatchPlan& p, const WorkLayout& w, uint8_t* stage) {
    ChunkDesc* h_desc = reinterpret_cast<ChunkDesc*>(stage + w.desc);
    uint32_t* h_ubase = reinterpret_cast<uint32_t*>(stage + w.ubase);
    uint32_t* h_coarse = reinterpret_cast<uint32_t*>(stage + w.coarse);
    FoldItem* h_fold = reinterpret_cast<FoldItem*>(stage + w.fold);
    uint32_t unit = 0, slot = p.nunits, coarse_next = 0;
    uint32_t fold_fill[kMaxLevels] = {0, 0, 0, 0};
    for (size_t k = 0; k < a.n; ++k) {
        const size_t i = a.at(k);
        const UnitPlan up = plan_chunk(a.len[i], p.unit_power);
        ChunkDesc& d = h_desc[k];
        describe_chunk(a, i, d);
        d.unit_base = unit;
        d.nunits = up.nunits;
        d.first_blocks = up.first_blocks;
        h_ubase[k] = unit;
        // coarse map: for every 2^kCoarseShift-th unit, the chunk that holds it
        while (coarse_next < p.ncoarse &&
               ((uint64_t)coarse_next << kCoarseShift) < (uint64_t)unit + up.nunits)
            h_coarse[coarse_next++] = (uint32_t)k;
        // fold levels: groups of kFan sets counted back from the end, the first one short
        uint32_t base = unit, count = up.nunits, power = p.unit_power, level = 0;
        while (count > kFan) {
            const uint32_t groups = (count + kFan - 1) / kFan;
            const uint32_t first = count - (groups - 1) * kFan;
            FoldItem* items = h_fold + p.fold_first[level] + fold_fill[level];
            for (uint32_t g = 0; g < groups; ++g) {
                items[g].in_base = base + (g == 0 ? 0 : first + (g - 1) * kFan);
                items[g].in_count = g == 0 ? first : kFan;
                items[g].out_slot = slot + g;
                items[g].pad_ = 0;
            }
            fold_fill[level] += groups;
            base = slot;
            slot += groups;
            count = groups;
            power += kFanPower;
            ++level;
        }
        d.final_base = base;
        d.final_count = count;
        d.final_power = power;
        unit += up.nunits;
    }
    h_ubase[a.n] = unit;
    while (coarse_next < p.ncoarse) h_coarse[coarse_next++] = (uint32_t)a.n - 1;
}

int record_timing_start(pgcm_key* key, hipStream_t stream) {
    if (key->timing) PGCM_HIP(hipEventRecord(key->bulk_start[key->timed % kTimingRing], stream));
    return PGCM_OK;
}

int record_timing_stop(pgcm_key* key, hipStream_t stream) {
    if (key->timing) {
        PGCM_HIP(hipEventRecord(key->bulk_stop[key->timed % kTimingRing], stream));
        ++key->timed;
    }
    return PGCM_OK;
}

// Small-transfer path: one kernel, descriptors read straight from the pinned staging buffer, no
// device workspace.
int run_small_batch(pgcm_key* key, Context* ctx, const BatchArgs& a, bool wide) {
    const uint32_t nchunks = (uint32_t)a.n;
    const int s = ctx->next_stage;
    int rc = ensure_stage(ctx, s, sizeof(ChunkDesc) * a.n);
    if (rc != PGCM_OK) return rc;
    ChunkDesc* h_desc = reinterpret_cast<ChunkDesc*>(ctx->stage[s]);
    for (size_t k = 0; k < a.n; ++k) describe_chunk(a, a.at(k), h_desc[k]);
    const KeyTables* kt = key->tables;
    rc = record_timing_start(key, a.stream);
    if (rc != PGCM_OK) return rc;
    if (a.decrypt)
        launch_small<true>(key->rounds, wide, nchunks, a.stream, kt, (const ChunkDesc*)h_desc,
                           nchunks, a.ivs, a.iv_len, a.tags, a.ok);
    else
        launch_small<false>(key->rounds, wide, nchunks, a.stream, kt, (const ChunkDesc*)h_desc,
                            nchunks, a.ivs, a.iv_len, a.tags, (uint8_t*)nullptr);
    // from here on the stream will read the staging buffer: mark its end even if a later call
    // fails, so that the buffer is not rewritten under a running kernel
    const int rc_end = end_of_batch(ctx, s, a.stream);
    rc = record_timing_stop(key, a.stream);
    if (rc != PGCM_OK) return rc;
    PGCM_HIP(hipGetLastError());
    return rc_end;
}

// Workspace of the one-launch path: arrival words, tag masks, one set per workgroup.
constexpr size_t kSwapArriveBytes = 256, kSwapMaskBytes = sizeof(Block) * kArgChunks;
constexpr size_t kSwapSetsAt = 1024;
static_assert(kSwapArriveBytes + kSwapMaskBytes <= kSwapSetsAt && 4 * kArgChunks <= kSwapArriveBytes,
              "one-launch workspace");

// does the batch take the one-launch path?
// (A chunk of more than 128 workgroups is left to the other kernels: the workgroup that finishes
// it would fold runs of sixteen sets per wavefront, a longer chain of dependent multiplications
// than the fold kernels' trees; measured on one 8 MiB chunk, 45 against 43 us.)
inline bool fits_one_launch(const pgcm_key* key, const BatchArgs& a, const BatchPlan& p) {
    return key->one_launch && a.iv_len == 12 && a.n <= kArgChunks && p.unit_power <= kUnitPower &&
           p.nunits <= key->wave_slots && p.max_units <= 128 * kWavesPerGroup;
}

// A batch of few chunks that does not fill the chip: one kernel, descriptors as its arguments,
// nothing staged and nothing uploaded.
int run_one_launch(pgcm_key* key, Context* ctx, const BatchArgs& a, const BatchPlan& p) {
    ArgBatch batch;
    memset(&batch, 0, sizeof(batch));
    batch.nchunks = (uint32_t)a.n;
    batch.unit_power = p.unit_power;
    uint32_t groups = 0;
    for (size_t k = 0; k < a.n; ++k) {
        const size_t i = a.at(k);
        const UnitPlan up = plan_chunk(a.len[i], p.unit_power);
        ArgChunk& c = batch.c[k];
        c.src = (const uint8_t*)a.src[i];
        c.dst = (uint8_t*)a.dst[i];
        c.len = a.len[i];
        c.aad_len = a.aad_len ? a.aad_len[i] : 0;
        c.aad = c.aad_len ? (const uint8_t*)a.aad[i] : nullptr;
        c.nunits = up.nunits;
        c.first_blocks = up.first_blocks;
        c.index = (uint32_t)i;
        c.group_base = groups;
        c.ngroups = up.nunits == 0 ? 1 : (up.nunits + kWavesPerGroup - 1) / kWavesPerGroup;
        groups += c.ngroups;
    }
    const size_t bytes = kSwapSetsAt + sizeof(Block) * 64 * (size_t)groups;
    int rc = ensure_work(ctx, bytes, a.stream);
    if (rc != PGCM_OK) return rc;
    uint32_t* d_arrive = reinterpret_cast<uint32_t*>(ctx->work);
    Block* d_ekj0 = reinterpret_cast<Block*>(ctx->work + kSwapArriveBytes);
    Block* d_sets = reinterpret_cast<Block*>(ctx->work + kSwapSetsAt);
    // the arrival words are left at zero by every batch of this kind; they need clearing when
    // the workspace is new, was used by a batch of the other kind, or is shared between keys
    if (!ctx->arrive_clean || !ctx->growable)
        hipLaunchKernelGGL(clear_words_kernel, dim3(1), dim3(64), 0, a.stream, d_arrive,
                           (uint32_t)kArgChunks);
    ctx->arrive_clean = false;
    ctx->counter_at = nullptr;  // the unit counter of the other kind of batch may lie under the sets
    int rc_timing = record_timing_start(key, a.stream);
    if (a.decrypt)
        launch_swap<true>(key->rounds, dim3(groups), a.stream, (const KeyTables*)key->tables, batch,
                          a.ivs, d_ekj0, d_sets, d_arrive, a.tags, a.ok);
    else
        launch_swap<false>(key->rounds, dim3(groups), a.stream, (const KeyTables*)key->tables,
                           batch, a.ivs, d_ekj0, d_sets, d_arrive, a.tags, (uint8_t*)nullptr);
    if (rc_timing == PGCM_OK) rc_timing = record_timing_stop(key, a.stream);
    // No staging buffer was used, but the context's workspace was: the batch's end is marked on
    // the event of the stage whose turn it is, without taking the turn.  (If that event still
    // guards an earlier batch's staging buffer, that batch ends before this one on the same
    // stream, so recording it again only moves the guard later.)
    const int s = ctx->next_stage;
    PGCM_HIP(hipEventRecord(ctx->stage_done[s], a.stream));
    ctx->last_stage = s;
    ctx->bound = true;
    if (rc_timing != PGCM_OK) return rc_timing;
    PGCM_HIP(hipGetLastError());
    ctx->arrive_clean = true;
    return PGCM_OK;
}

// The kernels of one batch that goes through the unit schedule, enqueued with context `ctx`.
int run_unit_batch(pgcm_key* key, Context* ctx, const BatchArgs& a, const BatchPlan& p) {
    const uint32_t nchunks = (uint32_t)a.n;
    const WorkLayout w = lay_out(a, p);
    if (!ctx->growable && (a.n > kFixedMaxChunks || w.bytes > ctx->work_cap))
        return PGCM_ERR_CAPACITY;
    const int s = ctx->next_stage;
    int rc = ensure_stage(ctx, s, w.upload_bytes);
    if (rc != PGCM_OK) return rc;
    rc = ensure_work(ctx, w.bytes, a.stream);
    if (rc != PGCM_OK) return rc;
    fill_schedule(a, p, w, ctx->stage[s]);
    ctx->arrive_clean = false;  // the descriptors land where the one-launch path counts arrivals
    uint32_t* d_counter = reinterpret_cast<uint32_t*>(ctx->work + w.counter);
    {
        // the unit counter is left at zero by the last kernel of every batch; it only needs
        // clearing when the workspace is new, the counter's place in it has moved, an earlier
        // batch was cut short, or the workspace is shared with other keys (the fixed context)
        const bool clear = ctx->counter_at != d_counter || ctx->counter_dirty || !ctx->growable;
        ctx->counter_at = d_counter;
        ctx->counter_dirty = true;
        const uint32_t n16 = (uint32_t)(w.upload_bytes / 16);
        uint32_t groups = (n16 + 255) / 256;
        if (groups > 1024) groups = 1024;
        hipLaunchKernelGGL(upload_kernel, dim3(groups), dim3(256), 0, a.stream,
                           reinterpret_cast<uint4*>(ctx->work),
                           reinterpret_cast<const uint4*>(ctx->stage[s]), n16,
                           clear ? d_counter : (uint32_t*)nullptr);
    }

    const KeyTables* kt = key->tables;
    const ChunkDesc* d_desc = reinterpret_cast<const ChunkDesc*>(ctx->work + w.desc);
    const uint32_t* d_ubase = reinterpret_cast<const uint32_t*>(ctx->work + w.ubase);
    const uint32_t* d_coarse = reinterpret_cast<const uint32_t*>(ctx->work + w.coarse);
    const FoldItem* d_fold = reinterpret_cast<const FoldItem*>(ctx->work + w.fold);
    Block* d_ekj0 = reinterpret_cast<Block*>(ctx->work + w.ekj0);
    Block* d_sets = reinterpret_cast<Block*>(ctx->work + w.sets);
    Block* d_j0 = a.iv_len == 12 ? nullptr : reinterpret_cast<Block*>(ctx->work + w.j0);
    if (d_j0 != nullptr)
        hipLaunchKernelGGL(j0_kernel, dim3((nchunks + 63) / 64), dim3(64), 0, a.stream, kt, d_desc,
                           a.ivs, a.iv_len, nchunks, d_j0);

    int rc_timing = PGCM_OK;
    if (p.nunits > 0) {
        uint32_t groups = (p.nunits + kWavesPerGroup - 1) / kWavesPerGroup;
        if (groups > (uint32_t)key->num_cu) groups = (uint32_t)key->num_cu;
        rc_timing = record_timing_start(key, a.stream);
        if (a.decrypt)
            launch_bulk<true>(key->rounds, key->matrix_hash, dim3(groups), a.stream, kt, d_desc,
                              d_ubase, d_coarse, p.nunits, p.unit_power, d_counter, a.ivs,
                              (const Block*)d_j0, d_ekj0, d_sets);
        else
            launch_bulk<false>(key->rounds, key->matrix_hash, dim3(groups), a.stream, kt, d_desc,
                               d_ubase, d_coarse, p.nunits, p.unit_power, d_counter, a.ivs,
                               (const Block*)d_j0, d_ekj0, d_sets);
        if (rc_timing == PGCM_OK) rc_timing = record_timing_stop(key, a.stream);
    }
    for (uint32_t l = 0; l < kMaxLevels; ++l) {
        if (p.fold_count[l] == 0) continue;
        const uint32_t power = p.unit_power + kFanPower * l;
        // few items: a workgroup each, folding as a tree; many: a wavefront each, as a chain
        if (p.fold_count[l] <= kFoldTreeMaxItems)
            hipLaunchKernelGGL(fold_tree_kernel, dim3(p.fold_count[l]), dim3(kFoldTreeWaves * 64),
                               0, a.stream, kt, d_fold + p.fold_first[l], power, d_sets);
        else
            hipLaunchKernelGGL(fold_kernel, dim3(p.fold_count[l]), dim3(64), 0, a.stream, kt,
                               d_fold + p.fold_first[l], power, d_sets);
    }
    // one wavefront per chunk; few chunks are spread over the compute units rather than packed
    // sixteen to a workgroup
    uint32_t per_group = (nchunks + (uint32_t)key->num_cu - 1) / (uint32_t)key->num_cu;
    if (per_group > kFinalWaves) per_group = kFinalWaves;
    const dim3 final_grid((nchunks + per_group - 1) / per_group);
    if (a.decrypt)
        hipLaunchKernelGGL(final_kernel<true>, final_grid, dim3(kFinalWaves * 64), 0, a.stream, kt,
                           d_desc, nchunks, a.ivs, d_j0, d_ekj0, d_sets, a.tags, a.ok,
                           p.unit_power, d_counter, per_group);
    else
        hipLaunchKernelGGL(final_kernel<false>, final_grid, dim3(kFinalWaves * 64), 0, a.stream,
                           kt, d_desc, nchunks, a.ivs, d_j0, d_ekj0, d_sets, a.tags,
                           (uint8_t*)nullptr, p.unit_power, d_counter, per_group);
    // the stream now reads the staging buffer and the workspace: their end is marked whatever
    // else fails below
    const int rc_end = end_of_batch(ctx, s, a.stream);
    if (rc_timing != PGCM_OK) return rc_timing;
    PGCM_HIP(hipGetLastError());
    if (rc_end != PGCM_OK) return rc_end;
    ctx->counter_dirty = false;
    return PGCM_OK;
}

// One batch under one key: validate everything, pick a context, then enqueue upload, J0 (if
// needed), bulk, fold levels and final kernels on the stream.
int run_batch(pgcm_key* key, const BatchArgs& a) {
    if (key == nullptr || key->tables == nullptr) return PGCM_ERR_ARG;
    int rc = check_batch(a);
    if (rc != PGCM_OK || a.n == 0) return rc;
    BatchPlan p;
    rc = plan_batch(key->forced_unit_power, key->wave_slots, a, &p);  // nothing touched so far
    if (rc != PGCM_OK) return rc;
    int cur_device = -1;
    PGCM_HIP(hipGetDevice(&cur_device));
    if (cur_device != key->device) return PGCM_ERR_ARG;  // the key lives on another GPU
    Context* ctx = nullptr;
    if (a.fixed) {
        if (a.n > kFixedMaxChunks) return PGCM_ERR_CAPACITY;
        ctx = &key->fixed;
        key->fixed_used = true;
    } else {
        rc = acquire_context(key, a.stream, &ctx);
        if (rc != PGCM_OK) return rc;
    }
    if (p.all_one_row)
        rc = run_small_batch(key, ctx, a, false);
    else if (p.all_small && a.n <= kSmallWideMaxChunks)
        rc = run_small_batch(key, ctx, a, true);
    else if (fits_one_launch(key, a, p))
        rc = run_one_launch(key, ctx, a, p);
    else
        rc = run_unit_batch(key, ctx, a, p);
    release_context(key, ctx);
    return rc;
}

// A batch whose chunks name their key: the chunks are grouped by key (keeping their order) and
// every group runs as one batch of its key, one after the other on the stream.
int run_batch_keys(pgcm_key* const* keys, size_t nkeys, const uint32_t* key_index,
                   const BatchArgs& all) {
    if (keys == nullptr || nkeys == 0 || nkeys > 0x7FFFFFFFull) return PGCM_ERR_ARG;
    int cur_device = -1;
    PGCM_HIP(hipGetDevice(&cur_device));
    for (size_t k = 0; k < nkeys; ++k)
        if (keys[k] == nullptr || keys[k]->tables == nullptr || keys[k]->device != cur_device)
            return PGCM_ERR_ARG;
    int rc = check_batch(all);
    if (rc != PGCM_OK || all.n == 0) return rc;
    if (key_index == nullptr) return PGCM_ERR_ARG;
    // every chunk is checked before the first group is enqueued
    std::vector<uint32_t> first, fill, order;
    try {
        first.assign(nkeys + 1, 0);
        fill.assign(nkeys, 0);
        order.resize(all.n);
    } catch (const std::bad_alloc&) {
        return PGCM_ERR_NOMEM;
    }
    for (size_t i = 0; i < all.n; ++i) {
        if (key_index[i] >= nkeys) return PGCM_ERR_ARG;
        rc = check_chunk(all, i);
        if (rc != PGCM_OK) return rc;
        ++first[key_index[i] + 1];
    }
    for (size_t k = 0; k < nkeys; ++k) first[k + 1] += first[k];
    for (size_t k = 0; k < nkeys; ++k) fill[k] = first[k];
    for (size_t i = 0; i < all.n; ++i) order[fill[key_index[i]]++] = (uint32_t)i;
    for (size_t k = 0; k < nkeys; ++k) {
        BatchArgs group = all;
        group.n = first[k + 1] - first[k];
        group.order = order.data() + first[k];
        if (group.n == 0) continue;
        rc = run_batch(keys[k], group);
        if (rc != PGCM_OK) return rc;
    }
    return PGCM_OK;
}

}  // namespace

extern "C" {
#pragma GCC visibility push(default)

int pgcm_expand_key(const uint8_t key[32], void* hip_stream, pgcm_key_t** out) {
    return pgcm_expand_key_bytes(key, 32, hip_stream, out);
}

int pgcm_expand_key_bytes(const uint8_t* key, uint32_t key_bytes, void* hip_stream,
                          pgcm_key_t** out) {
    if (key == nullptr || out == nullptr) return PGCM_ERR_ARG;
    *out = nullptr;
    if (key_bytes != 16 && key_bytes != 24 && key_bytes != 32) return PGCM_ERR_ARG;
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
        k->wave_slots = (uint32_t)k->num_cu * kWavesPerGroup;
        // the fixed context: one pinned block cut into the staging buffers, the device's static
        // scratch array as workspace; nothing of it ever grows
        k->fixed.growable = false;
        if ((rc = create_stage_events(&k->fixed)) != PGCM_OK) break;
        {
            void* p = nullptr;
            if (hip_failed(hipHostMalloc(&p, kStages * kFixedStageBytes, hipHostMallocDefault))) {
                rc = PGCM_ERR_NOMEM;
                break;
            }
            for (int s = 0; s < kStages; ++s) {
                k->fixed.stage[s] = static_cast<uint8_t*>(p) + (size_t)s * kFixedStageBytes;
                k->fixed.stage_cap[s] = kFixedStageBytes;
            }
        }
        if ((rc = scratch_of_device(k->device, &k->fixed.work)) != PGCM_OK) break;
        k->fixed.work_cap = kScratchBytes;
        // a pageable copy of at most 32 bytes: staged by the runtime, complete on return for this size
        if (hip_failed(hipMemcpyAsync(d_key, key, key_bytes, hipMemcpyHostToDevice, stream))) { rc = PGCM_ERR_HIP; break; }
        k->rounds = (int)(key_bytes / 4 + 6);
        hipLaunchKernelGGL(expand_key_kernel, dim3(1), dim3(1024), 0, stream, k->tables, d_key,
                           key_bytes / 4);
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
    for (Context* c : k->contexts) {
        destroy_context(c, true);
        delete c;
    }
    // the fixed context: its staging buffers are slices of one allocation, and its workspace is
    // the device's static array, which is wiped (it holds tag masks and partial hashes) but stays
    if (k->fixed.work && k->fixed_used) (void)hipMemset(k->fixed.work, 0, kScratchBytes);
    if (k->fixed.stage[0]) {
        memset(k->fixed.stage[0], 0, kStages * kFixedStageBytes);
        (void)hipHostFree(k->fixed.stage[0]);
    }
    for (int s = 0; s < kStages; ++s)
        if (k->fixed.stage_done[s]) (void)hipEventDestroy(k->fixed.stage_done[s]);
    for (uint32_t i = 0; i < kTimingRing; ++i) {
        if (k->bulk_start[i]) (void)hipEventDestroy(k->bulk_start[i]);
        if (k->bulk_stop[i]) (void)hipEventDestroy(k->bulk_stop[i]);
    }
    delete k;
}

int pgcm_encrypt_batch(pgcm_key_t* key, size_t n, const uint8_t* ivs, const void* const* aad,
                       const uint32_t* aad_len, const void* const* src, const uint64_t* len,
                       void* const* dst, uint8_t* tags, void* hip_stream) {
    return run_batch(key, BatchArgs{false, n, nullptr, ivs, 12, aad, aad_len, src, len, dst, tags,
                                    nullptr, (hipStream_t)hip_stream});
}

int pgcm_encrypt_batch_iv(pgcm_key_t* key, size_t n, const uint8_t* ivs, uint32_t iv_bytes,
                          const void* const* aad, const uint32_t* aad_len, const void* const* src,
                          const uint64_t* len, void* const* dst, uint8_t* tags, void* hip_stream) {
    return run_batch(key, BatchArgs{false, n, nullptr, ivs, iv_bytes, aad, aad_len, src, len, dst,
                                    tags, nullptr, (hipStream_t)hip_stream});
}

int pgcm_encrypt_batch_static(pgcm_key_t* key, size_t n, const uint8_t* ivs,
                              const void* const* aad, const uint32_t* aad_len,
                              const void* const* src, const uint64_t* len, void* const* dst,
                              uint8_t* tags, void* hip_stream) {
    BatchArgs a{false, n, nullptr, ivs, 12, aad, aad_len, src, len, dst, tags, nullptr,
                (hipStream_t)hip_stream};
    a.fixed = true;
    return run_batch(key, a);
}

int pgcm_reserve(pgcm_key_t* key, void* hip_stream, size_t n_max, uint64_t payload_bytes_max) {
    if (key == nullptr || key->tables == nullptr || n_max > 0x7FFFFFFFull) return PGCM_ERR_ARG;
    int cur_device = -1;
    PGCM_HIP(hipGetDevice(&cur_device));
    if (cur_device != key->device) return PGCM_ERR_ARG;
    size_t stage_bytes = 0, work_bytes = 0;
    if (!worst_case_sizes(key->forced_unit_power, key->wave_slots, n_max, payload_bytes_max,
                          &stage_bytes, &work_bytes))
        return PGCM_ERR_ARG;
    const hipStream_t stream = (hipStream_t)hip_stream;
    Context* ctx = nullptr;
    int rc = acquire_context(key, stream, &ctx);
    if (rc != PGCM_OK) return rc;
    for (int s = 0; s < kStages && rc == PGCM_OK; ++s) rc = ensure_stage(ctx, s, stage_bytes);
    if (rc == PGCM_OK) rc = ensure_work(ctx, work_bytes, stream);
    if (rc == PGCM_OK) {
        // the context now belongs to this stream, so that the stream's batches find it
        std::lock_guard<std::mutex> lock(key->mu);
        ctx->bound = true;
    }
    release_context(key, ctx);
    return rc;
}

int pgcm_decrypt_verify_batch(pgcm_key_t* key, size_t n, const uint8_t* ivs,
                              const void* const* aad, const uint32_t* aad_len,
                              const void* const* src, const uint64_t* len, void* const* dst,
                              const uint8_t* tags, uint8_t* ok, void* hip_stream) {
    return run_batch(key, BatchArgs{true, n, nullptr, ivs, 12, aad, aad_len, src, len, dst,
                                    const_cast<uint8_t*>(tags), ok, (hipStream_t)hip_stream});
}

int pgcm_decrypt_verify_batch_iv(pgcm_key_t* key, size_t n, const uint8_t* ivs, uint32_t iv_bytes,
                                 const void* const* aad, const uint32_t* aad_len,
                                 const void* const* src, const uint64_t* len, void* const* dst,
                                 const uint8_t* tags, uint8_t* ok, void* hip_stream) {
    return run_batch(key, BatchArgs{true, n, nullptr, ivs, iv_bytes, aad, aad_len, src, len, dst,
                                    const_cast<uint8_t*>(tags), ok, (hipStream_t)hip_stream});
}

int pgcm_encrypt_batch_keys(pgcm_key_t* const* keys, size_t nkeys, const uint32_t* key_index,
                            size_t n, const uint8_t* ivs, uint32_t iv_bytes,
                            const void* const* aad, const uint32_t* aad_len,
                            const void* const* src, const uint64_t* len, void* const* dst,
                            uint8_t* tags, void* hip_stream) {
    return run_batch_keys(keys, nkeys, key_index,
                          BatchArgs{false, n, nullptr, ivs, iv_bytes, aad, aad_len, src, len, dst,
                                    tags, nullptr, (hipStream_t)hip_stream});
}

int pgcm_decrypt_verify_batch_keys(pgcm_key_t* const* keys, size_t nkeys,
                                   const uint32_t* key_index, size_t n, const uint8_t* ivs,
                                   uint32_t iv_bytes, const void* const* aad,
                                   const uint32_t* aad_len, const void* const* src,
                                   const uint64_t* len, void* const* dst, const uint8_t* tags,
                                   uint8_t* ok, void* hip_stream) {
    return run_batch_keys(keys, nkeys, key_index,
                          BatchArgs{true, n, nullptr, ivs, iv_bytes, aad, aad_len, src, len, dst,
                                    const_cast<uint8_t*>(tags), ok, (hipStream_t)hip_stream});
}

const char* pgcm_strerror(int status) {
    switch (status) {
        case PGCM_OK: return "success";
        case PGCM_ERR_ARG: return "invalid argument";
        case PGCM_ERR_ALIGN: return "src or dst pointer not 16-byte aligned";
        case PGCM_ERR_LEN: return "chunk longer than the GCM limit of 2^36 - 32 bytes, or too long for a forced unit size";
        case PGCM_ERR_NOMEM: return "out of host or device memory";
        case PGCM_ERR_HIP: return "a HIP runtime call failed";
        case PGCM_ERR_BUSY: return "every buffer of the pool is held";
        case PGCM_ERR_CAPACITY: return "the batch needs more than the fixed buffers of an entry point that does not allocate";
        default: return "unknown status";
    }
}

int pgcm_last_hip_error(void) { return g_last_hip_error; }

int64_t pgcm_plan_units(size_t n, const uint64_t* len, uint32_t* nunits, uint32_t* first_blocks,
                        uint32_t* unit_base, uint32_t* final_count, uint32_t* final_power) {
    if (n != 0 && len == nullptr) return PGCM_ERR_ARG;
    uint64_t total = 0;
    const uint32_t unit_power = choose_unit_power(n, nullptr, len, kWaveSlots);
    for (size_t i = 0; i < n; ++i) {
        if (len[i] > PGCM_MAX_CHUNK_BYTES) return PGCM_ERR_LEN;
        UnitPlan p = plan_chunk(len[i], unit_power);
        uint32_t outs[kMaxLevels];
        const uint32_t levels = fold_levels(p.nunits, outs);
        if (levels > kMaxLevels) return PGCM_ERR_LEN;  // cannot happen with the chosen unit
        if (nunits) nunits[i] = p.nunits;
        if (first_blocks) first_blocks[i] = p.first_blocks;
        if (unit_base) unit_base[i] = (uint32_t)total;
        if (final_count) final_count[i] = levels ? outs[levels - 1] : p.nunits;
        if (final_power) final_power[i] = unit_power + kFanPower * levels;
        total += p.nunits;
        if (total > 0xFFFFFFF0ull / 64) return PGCM_ERR_ARG;
    }
    return (int64_t)total;
}

uint32_t pgcm_unit_bytes(void) { return kUnitBytes; }

uint32_t pgcm_batch_unit_bytes(size_t n, const uint64_t* len) {
    if (n != 0 && len == nullptr) return 0;
    return 16u << choose_unit_power(n, nullptr, len, kWaveSlots);
}

int pgcm_describe_schedule(size_t n, const uint64_t* len, uint32_t unit_bytes, uint32_t wave_slots,
                           pgcm_schedule_info* info, void* image, size_t image_capacity) {
    if (info == nullptr || (n != 0 && len == nullptr) || n > 0x7FFFFFFFull) return PGCM_ERR_ARG;
    uint32_t forced = 0;
    if (unit_bytes != 0) {
        for (uint32_t u = kMinUnitPower; u <= kMaxUnitPower; ++u)
            if (unit_bytes == (16u << u)) forced = u;
        if (forced == 0) return PGCM_ERR_ARG;
    }
    memset(info, 0, sizeof(*info));
    // stand-ins for the device pointers a real batch carries (16-byte aligned, never followed)
    std::vector<const void*> ptrs;
    try {
        ptrs.assign(n, reinterpret_cast<const void*>((uintptr_t)4096));
    } catch (const std::bad_alloc&) {
        return PGCM_ERR_NOMEM;
    }
    BatchArgs a{false, n, nullptr, reinterpret_cast<const uint8_t*>((uintptr_t)4096), 12, nullptr,
                nullptr, ptrs.data(), len, const_cast<void* const*>(ptrs.data()),
                reinterpret_cast<uint8_t*>((uintptr_t)4096), nullptr, nullptr};
    BatchPlan p{};
    int rc = plan_batch(forced, wave_slots ? wave_slots : kWaveSlots, a, &p);
    if (rc != PGCM_OK) return rc;
    const WorkLayout w = lay_out(a, p);
    info->desc_offset = w.desc;
    info->unit_base_offset = w.ubase;
    info->coarse_map_offset = w.coarse;
    info->fold_items_offset = w.fold;
    info->image_bytes = w.upload_bytes;
    info->workspace_bytes = w.bytes;
    info->unit_power = p.unit_power;
    info->nunits = p.nunits;
    info->nslots = p.nslots;
    info->ncoarse = p.ncoarse;
    info->nfold = p.nfold;
    for (uint32_t l = 0; l < kMaxLevels; ++l) {
        info->fold_count[l] = p.fold_count[l];
        info->fold_first[l] = p.fold_first[l];
    }
    info->path = n == 0 ? 0 : p.all_one_row ? 1 : (p.all_small && n <= kSmallWideMaxChunks) ? 2 : 0;
    if (image != nullptr) {
        if (image_capacity < w.upload_bytes) return PGCM_ERR_CAPACITY;
        memset(image, 0, w.upload_bytes);
        if (n != 0) fill_schedule(a, p, w, static_cast<uint8_t*>(image));
    }
    return PGCM_OK;
}

size_t pgcm_key_tables_bytes(void) { return sizeof(KeyTables); }

int pgcm_copy_key_tables(pgcm_key_t* key, void* out, size_t bytes) {
    if (key == nullptr || key->tables == nullptr || (out == nullptr && bytes != 0))
        return PGCM_ERR_ARG;
    if (bytes > sizeof(KeyTables)) bytes = sizeof(KeyTables);
    PGCM_HIP(hipDeviceSynchronize());
    if (bytes != 0) PGCM_HIP(hipMemcpy(out, key->tables, bytes, hipMemcpyDeviceToHost));
    return PGCM_OK;
}

int pgcm_set_unit_bytes(pgcm_key_t* key, uint32_t unit_bytes) {
    if (key == nullptr) return PGCM_ERR_ARG;
    if (unit_bytes == 0) {
        key->forced_unit_power = 0;
        return PGCM_OK;
    }
    for (uint32_t u = kMinUnitPower; u <= kMaxUnitPower; ++u)
        if (unit_bytes == (16u << u)) {
            key->forced_unit_power = u;
            return PGCM_OK;
        }
    return PGCM_ERR_ARG;
}

int pgcm_bitsliced_keystream(pgcm_key_t* key, const uint8_t iv[12], uint32_t ctr_base,
                             uint64_t nblocks, void* out, void* hip_stream) {
    constexpr uint64_t kPerGroup = pgcm_bitsliced::kLaneBlocks * pgcm_bitsliced::kGroupLanes;
    if (key == nullptr || key->tables == nullptr || iv == nullptr || out == nullptr)
        return PGCM_ERR_ARG;
    if (ctr_base % pgcm_bitsliced::kLaneBlocks != 0 || nblocks % kPerGroup != 0 ||
        nblocks > ((uint64_t)1 << 31) || ((uintptr_t)out & 15))
        return PGCM_ERR_ARG;
    if (nblocks == 0) return PGCM_OK;
    int cur_device = -1;
    PGCM_HIP(hipGetDevice(&cur_device));
    if (cur_device != key->device) return PGCM_ERR_ARG;
    uint32_t w[3];
    memcpy(w, iv, 12);  // little-endian loads of the IV bytes, like the round-key words
    const dim3 grid((uint32_t)(nblocks / kPerGroup)), block(pgcm_bitsliced::kGroupLanes);
    const hipStream_t stream = (hipStream_t)hip_stream;
    const KeyTables* kt = key->tables;
    uint32_t* o = static_cast<uint32_t*>(out);
    if (key->rounds == 10)
        hipLaunchKernelGGL(pgcm_bitsliced::keystream_kernel<10>, grid, block, 0, stream, kt, w[0],
                           w[1], w[2], ctr_base, o);
    else if (key->rounds == 12)
        hipLaunchKernelGGL(pgcm_bitsliced::keystream_kernel<12>, grid, block, 0, stream, kt, w[0],
                           w[1], w[2], ctr_base, o);
    else
        hipLaunchKernelGGL(pgcm_bitsliced::keystream_kernel<14>, grid, block, 0, stream, kt, w[0],
                           w[1], w[2], ctr_base, o);
    PGCM_HIP(hipGetLastError());
    return PGCM_OK;
}

int pgcm_set_matrix_hash(pgcm_key_t* key, int enable) {
    if (key == nullptr) return PGCM_ERR_ARG;
    key->matrix_hash = enable != 0;
    return PGCM_OK;
}

int pgcm_set_one_launch(pgcm_key_t* key, int enable) {
    if (key == nullptr) return PGCM_ERR_ARG;
    key->one_launch = enable != 0;
    return PGCM_OK;
}

int pgcm_set_timing(pgcm_key_t* key, int enable) {
    if (key == nullptr) return PGCM_ERR_ARG;
    if (enable && key->bulk_start[0] == nullptr) {
        for (uint32_t i = 0; i < kTimingRing; ++i) {
            PGCM_HIP(hipEventCreate(&key->bulk_start[i]));
            PGCM_HIP(hipEventCreate(&key->bulk_stop[i]));
        }
    }
    key->timing = enable != 0;
    key->timed = 0;
    return PGCM_OK;
}

int pgcm_measure_passes(pgcm_key_t* key, size_t n, const uint8_t* ivs, uint32_t iv_bytes,
                        const void* const* aad,
                        const uint32_t* aad_len, const void* const* src, const uint64_t* len,
                        void* const* cipher, void* const* back, uint8_t* tags, uint8_t* ok,
                        void* hip_stream, uint32_t steps, int direction, double* host_ms) {
    if (host_ms == nullptr || direction < 0 || direction > 2) return PGCM_ERR_ARG;
    const hipStream_t stream = (hipStream_t)hip_stream;
    PGCM_HIP(hipStreamSynchronize(stream));
    const auto t0 = std::chrono::steady_clock::now();
    for (uint32_t k = 0; k < steps; ++k) {
        int rc = PGCM_OK;
        if (direction != 2)
            rc = pgcm_encrypt_batch_iv(key, n, ivs, iv_bytes, aad, aad_len, src, len, cipher, tags,
                                       hip_stream);
        if (rc == PGCM_OK && direction != 1)
            rc = pgcm_decrypt_verify_batch_iv(key, n, ivs, iv_bytes, aad, aad_len,
                                              reinterpret_cast<const void* const*>(cipher), len,
                                              back, tags, ok, hip_stream);
        if (rc != PGCM_OK) return rc;
    }
    PGCM_HIP(hipStreamSynchronize(stream));
    *host_ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0)
                   .count();
    return PGCM_OK;
}

int pgcm_last_bulk_kernel_ms(pgcm_key_t* key, float* ms) {
    if (key == nullptr || ms == nullptr || key->timed == 0) return PGCM_ERR_ARG;
    const uint32_t slot = (uint32_t)((key->timed - 1) % kTimingRing);
    PGCM_HIP(hipEventSynchronize(key->bulk_stop[slot]));
    PGCM_HIP(hipEventElapsedTime(ms, key->bulk_start[slot], key->bulk_stop[slot]));
    return PGCM_OK;
}

int64_t pgcm_bulk_kernel_ms_history(pgcm_key_t* key, float* ms, size_t max) {
    if (key == nullptr || (ms == nullptr && max != 0)) return PGCM_ERR_ARG;
    uint64_t count = key->timed < kTimingRing ? key->timed : kTimingRing;
    if (count > max) count = max;
    for (uint64_t i = 0; i < count; ++i) {
        const uint32_t slot = (uint32_t)((key->timed - count + i) % kTimingRing);
        PGCM_HIP(hipEventSynchronize(key->bulk_stop[slot]));
        PGCM_HIP(hipEventElapsedTime(&ms[i], key->bulk_start[slot], key->bulk_stop[slot]));
    }
    return (int64_t)count;
}

#pragma GCC visibility pop
}  // extern "C"
