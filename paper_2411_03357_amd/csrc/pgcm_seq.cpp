// Host-side state machine of the paper's speculative pipelined encryption (sections 4.3, 5.1-5.3):
// see include/pgcm_seq.h.  Plain C++, no GPU calls.
#include "../../include/pgcm_seq.h"

#include <algorithm>
#include <deque>
#include <new>
#include <unordered_map>
#include <utility>
#include <vector>

#include "../../include/pgcm.h"

namespace {

struct Chunk {
    uint64_t addr, len;
    bool operator==(const Chunk& o) const { return addr == o.addr && len == o.len; }
};

struct ChunkHash {
    size_t operator()(const Chunk& c) const {
        uint64_t h = c.addr * 0x9E3779B97F4A7C15ull ^ (c.len + 0x7F4A7C15ull) * 0xC2B2AE3D27D4EB4Full;
        return (size_t)(h ^ (h >> 29));
    }
};

enum class Ends { kFifo, kLifo };

}  // namespace

struct pgcm_seq {
    uint64_t iv_cur = 0;
    uint32_t depth = 1, leeway = 0, history_limit = 1;
    uint64_t threshold = 0;
    std::deque<Chunk> swapped_in;                          // past swap-ins, oldest first (bounded)
    std::vector<Chunk> swapped_out;                        // not yet back, oldest first
    std::unordered_map<Chunk, uint64_t, ChunkHash> kept;   // pre-encrypted: chunk -> its IV
    std::vector<std::pair<Chunk, uint64_t>> held;          // requests waiting for the sync
    Ends ends = Ends::kFifo;                               // which end of swapped_out was taken last
    std::deque<pgcm_seq_action> actions;

    void emit(uint32_t kind, const Chunk& c, uint64_t iv) {
        actions.push_back(pgcm_seq_action{kind, 0, c.addr, c.len, iv});
    }
    bool is_held(const Chunk& c) const {
        for (const auto& h : held)
            if (h.first == c) return true;
        return false;
    }
    std::vector<std::pair<uint64_t, Chunk>> kept_by_iv() const {
        std::vector<std::pair<uint64_t, Chunk>> v;
        v.reserve(kept.size());
        for (const auto& e : kept) v.emplace_back(e.second, e.first);
        std::sort(v.begin(), v.end(),
                  [](const auto& a, const auto& b) { return a.first < b.first; });
        return v;
    }

    // kept ciphertexts whose IV has passed can never be delivered
    void drop_passed() {
        for (const auto& e : kept_by_iv()) {
            if (e.first < iv_cur && !is_held(e.second)) {
                kept.erase(e.second);
                emit(PGCM_SEQ_DROP, e.second, e.first);
            }
        }
    }

    // delivering one transfer may make a held request's IV current
    void release_held() {
        for (bool moved = true; moved;) {
            moved = false;
            for (size_t i = 0; i < held.size(); ++i) {
                if (held[i].second == iv_cur) {
                    const Chunk c = held[i].first;
                    held.erase(held.begin() + (long)i);
                    kept.erase(c);
                    emit(PGCM_SEQ_SEND, c, iv_cur);
                    ++iv_cur;
                    moved = true;
                    break;
                }
            }
        }
    }

    void record_swap_in(const Chunk& c) {
        swapped_in.push_back(c);
        while (swapped_in.size() > history_limit) swapped_in.pop_front();
        auto it = std::find(swapped_out.begin(), swapped_out.end(), c);
        if (it != swapped_out.end()) {
            if (swapped_out.size() > 1) {
                if (it == swapped_out.begin())
                    ends = Ends::kFifo;
                else if (it + 1 == swapped_out.end())
                    ends = Ends::kLifo;
            }
            swapped_out.erase(it);
        }
    }

    // the predictor f: next chunk to come back, given the (possibly extended) history `seen`,
    // the candidates `away` and the chunks already spoken for
    bool predict(const std::vector<Chunk>& seen, const std::vector<Chunk>& away,
                 const std::unordered_map<Chunk, uint64_t, ChunkHash>& spoken, Chunk* next) const {
        if (!seen.empty()) {
            // repetitive pattern: what followed the latest chunk the last time it came by
            const Chunk& last = seen.back();
            for (size_t k = seen.size() - 1; k-- > 0;) {
                if (seen[k] == last) {
                    if (spoken.find(seen[k + 1]) == spoken.end()) {
                        *next = seen[k + 1];
                        return true;
                    }
                    break;
                }
            }
        }
        if (ends == Ends::kFifo) {
            for (size_t i = 0; i < away.size(); ++i)
                if (spoken.find(away[i]) == spoken.end()) {
                    *next = away[i];
                    return true;
                }
        } else {
            for (size_t i = away.size(); i-- > 0;)
                if (spoken.find(away[i]) == spoken.end()) {
                    *next = away[i];
                    return true;
                }
        }
        return false;
    }

    // keep `depth` predicted swaps pre-encrypted, each under the IV it is expected to meet
    void speculate() {
        if (kept.size() >= depth) return;
        // what is already kept is the predicted near future: predictions continue from it
        std::vector<Chunk> seen(swapped_in.begin(), swapped_in.end());
        uint64_t next_iv = iv_cur;
        for (const auto& e : kept_by_iv()) {
            seen.push_back(e.second);
            next_iv = std::max(next_iv, e.first + 1);
        }
        std::vector<Chunk> away;
        for (const Chunk& c : swapped_out)
            if (kept.find(c) == kept.end()) away.push_back(c);
        while (kept.size() < depth) {
            Chunk c;
            if (!predict(seen, away, kept, &c)) break;
            const uint64_t iv = next_iv + leeway;
            kept.emplace(c, iv);
            emit(PGCM_SEQ_PRE, c, iv);
            seen.push_back(c);
            auto it = std::find(away.begin(), away.end(), c);
            if (it != away.end()) away.erase(it);
            next_iv = iv + 1;
        }
    }
};

#pragma GCC visibility push(default)
extern "C" {

int pgcm_seq_create(uint64_t iv_start, uint32_t depth, uint32_t leeway, uint64_t swap_threshold,
                    uint32_t history_limit, pgcm_seq_t** out) {
    if (out == nullptr || depth == 0 || history_limit == 0) return PGCM_ERR_ARG;
    pgcm_seq* s = new (std::nothrow) pgcm_seq();
    if (s == nullptr) return PGCM_ERR_NOMEM;
    s->iv_cur = iv_start;
    s->depth = depth;
    s->leeway = leeway;
    s->threshold = swap_threshold;
    s->history_limit = history_limit;
    *out = s;
    return PGCM_OK;
}

void pgcm_seq_destroy(pgcm_seq_t* seq) { delete seq; }

int pgcm_seq_swap_out(pgcm_seq_t* s, uint64_t addr, uint64_t len) {
    if (s == nullptr) return PGCM_ERR_ARG;
    try {
        // only swaps are pipelined: a chunk too short to be one is not tracked
        if (len < s->threshold) return PGCM_OK;
        const Chunk c{addr, len};
        auto it = std::find(s->swapped_out.begin(), s->swapped_out.end(), c);
        if (it != s->swapped_out.end()) s->swapped_out.erase(it);
        s->swapped_out.push_back(c);
        s->speculate();
    } catch (const std::bad_alloc&) {
        return PGCM_ERR_NOMEM;
    }
    return PGCM_OK;
}

int pgcm_seq_notify_write(pgcm_seq_t* s, uint64_t addr, uint64_t len) {
    if (s == nullptr) return PGCM_ERR_ARG;
    try {
        bool served = false;
        for (const auto& e : s->kept_by_iv()) {
            const Chunk& c = e.second;
            if (c.addr < addr + len && addr < c.addr + c.len) {
                s->kept.erase(c);
                s->emit(PGCM_SEQ_DROP, c, e.first);
                if (s->is_held(c)) {
                    // a held request loses its ciphertext: it is served on the spot instead
                    s->held.erase(std::remove_if(s->held.begin(), s->held.end(),
                                                 [&](const auto& h) { return h.first == c; }),
                                  s->held.end());
                    s->emit(PGCM_SEQ_NOW, c, s->iv_cur);
                    ++s->iv_cur;
                    served = true;
                }
            }
        }
        if (served) {
            s->release_held();
            s->drop_passed();
        }
        s->speculate();
    } catch (const std::bad_alloc&) {
        return PGCM_ERR_NOMEM;
    }
    return PGCM_OK;
}

int pgcm_seq_request(pgcm_seq_t* s, uint64_t addr, uint64_t len) {
    if (s == nullptr) return PGCM_ERR_ARG;
    try {
        const Chunk c{addr, len};
        if (len < s->threshold) {
            // small transfer: never pipelined, takes the current IV (which may bring the wire to
            // the IV a held request waits for)
            s->emit(PGCM_SEQ_NOW, c, s->iv_cur);
            ++s->iv_cur;
            s->release_held();
            s->drop_passed();
            return PGCM_OK;
        }
        s->record_swap_in(c);
        auto it = s->kept.find(c);
        const bool usable = it != s->kept.end() && !s->is_held(c) && it->second >= s->iv_cur;
        if (!usable) {
            // wrong guess: give up what was prepared (held requests keep theirs), serve this
            // request on the critical path, start again from what really happened
            for (const auto& e : s->kept_by_iv()) {
                if (!s->is_held(e.second)) {
                    s->kept.erase(e.second);
                    s->emit(PGCM_SEQ_DROP, e.second, e.first);
                }
            }
            s->emit(PGCM_SEQ_NOW, c, s->iv_cur);
            ++s->iv_cur;
            s->release_held();
            s->drop_passed();
        } else if (it->second == s->iv_cur) {
            s->kept.erase(it);
            s->emit(PGCM_SEQ_SEND, c, s->iv_cur);
            ++s->iv_cur;
            s->release_held();
        } else {
            s->held.emplace_back(c, it->second);
        }
        s->speculate();
    } catch (const std::bad_alloc&) {
        return PGCM_ERR_NOMEM;
    }
    return PGCM_OK;
}

int pgcm_seq_sync(pgcm_seq_t* s) {
    if (s == nullptr) return PGCM_ERR_ARG;
    try {
        // Inside a batch the order is free (section 5.3, swap re-ordering): held requests whose
        // IV still lies ahead are committed first, in IV order, NOPs filling the gaps, so that
        // none of them is overtaken by the others; those the wire had already passed are
        // encrypted afresh after them.
        std::stable_sort(s->held.begin(), s->held.end(),
                         [](const auto& a, const auto& b) { return a.second < b.second; });
        std::vector<std::pair<Chunk, uint64_t>> late;
        for (const auto& h : s->held) {
            if (h.second < s->iv_cur) {
                late.push_back(h);
                continue;
            }
            while (s->iv_cur < h.second) {
                s->emit(PGCM_SEQ_NOP, Chunk{0, 1}, s->iv_cur);
                ++s->iv_cur;
            }
            s->kept.erase(h.first);
            s->emit(PGCM_SEQ_SEND, h.first, h.second);
            ++s->iv_cur;
        }
        for (const auto& h : late) {
            s->kept.erase(h.first);
            s->emit(PGCM_SEQ_DROP, h.first, h.second);
            s->emit(PGCM_SEQ_NOW, h.first, s->iv_cur);
            ++s->iv_cur;
        }
        s->held.clear();
        s->drop_passed();
        s->speculate();
    } catch (const std::bad_alloc&) {
        return PGCM_ERR_NOMEM;
    }
    return PGCM_OK;
}

size_t pgcm_seq_take_actions(pgcm_seq_t* s, pgcm_seq_action* out, size_t cap) {
    if (s == nullptr || out == nullptr) return 0;
    size_t n = 0;
    while (n < cap && !s->actions.empty()) {
        out[n++] = s->actions.front();
        s->actions.pop_front();
    }
    return n;
}

uint64_t pgcm_seq_current_iv(const pgcm_seq_t* s) { return s ? s->iv_cur : 0; }

void pgcm_seq_iv_bytes(const uint8_t iv0[12], uint64_t n, uint8_t out[12]) {
    unsigned carry = 0;
    for (int i = 11; i >= 0; --i) {
        unsigned add = (11 - i) < 8 ? (unsigned)((n >> (8 * (11 - i))) & 0xFF) : 0u;
        unsigned v = iv0[i] + add + carry;
        out[i] = (uint8_t)v;
        carry = v >> 8;
    }
}

}  // extern "C"
#pragma GCC visibility pop
