// Host-side residency manager for the GPU slots of a worker (no device code in this file).
//
// The paper's serving section separates what can be named (a catalog of up to 10^6 adapter
// revisions), what a worker holds near its engine, and what can run in one batch (<= 64 distinct
// adapters), and treats a cache miss as scheduled service work: concurrent misses on the same
// adapter share one load, different adapters are separate load jobs, the number of jobs in flight
// and the queue behind them are bounded, and a request that finds both full is rejected in a way
// the caller can retry (Section 4, cache tiers and cold loading; Appendix cold-load table: with one
// job in flight and a queue of one, a burst of four cold requests loads two and rejects two).  It
// also separates registered / prewarming / ready: a revision the control plane knows is exposed to
// traffic only once its load has completed.
//
// This object keeps exactly that state for the slot tables of this library: catalog id -> state and
// slot, least-recently-used eviction among ready slots that the current batch has not pinned, a
// FIFO of waiting load jobs.  It moves no bytes: on MLORA_R_LOAD the caller uploads the adapter into
// the returned slot of each of its sites (lora_slots_upload) and then calls
// mlora_resident_complete.
#include <cstdint>
#include <deque>
#include <list>
#include <mutex>
#include <new>
#include <unordered_map>
#include <vector>
#include "../../include/mlora.h"

namespace {
enum State : int32_t { kRegistered = 0, kQueued = 1, kPrewarming = 2, kReady = 3 };
struct Entry {
    State state = kRegistered;
    int32_t slot = -1;
    std::list<int64_t>::iterator lru;      // valid while ready
};
}

struct mlora_resident {
    std::mutex mu;
    int32_t n_slots = 0, max_in_flight = 0, max_queue = 0, in_flight = 0;
    std::unordered_map<int64_t, Entry> ids;
    std::vector<int64_t> slot_id;          // catalog id per slot, -1 = free
    std::vector<uint8_t> pinned;
    std::list<int64_t> lru;                // ready ids, most recently used first
    std::deque<int64_t> queue;             // ids waiting for a load job
    int64_t stats[MLORA_RESIDENT_STATS] = {0};

    // A slot a new load may take: a free one, else the least recently used ready slot that is not
    // pinned.  Returns -1 if there is none.  *evicted = the id that lost its slot, or -1.
    int32_t take_slot(int64_t *evicted)
    {
        *evicted = -1;
        for (int32_t s = 0; s < n_slots; ++s)
            if (slot_id[s] < 0) return s;
        for (auto it = lru.rbegin(); it != lru.rend(); ++it) {
            Entry &v = ids[*it];
            if (pinned[v.slot]) continue;
            const int32_t s = v.slot;
            *evicted = *it;
            lru.erase(v.lru);
            v.state = kRegistered; v.slot = -1;
            slot_id[s] = -1;
            stats[MLORA_STAT_EVICTIONS] += 1;
            return s;
        }
        return -1;
    }
    bool start(int64_t id, Entry &e, int32_t *slot, int64_t *evicted)
    {
        if (in_flight >= max_in_flight) return false;
        const int32_t s = take_slot(evicted);
        if (s < 0) return false;
        e.state = kPrewarming; e.slot = s;
        slot_id[s] = id;
        in_flight += 1;
        stats[MLORA_STAT_LOADS] += 1;
        *slot = s;
        return true;
    }
};

extern "C" {

int32_t mlora_resident_create(int32_t n_slots, int32_t max_in_flight, int32_t max_queue, mlora_resident **out)
{
    if (!out || n_slots <= 0 || max_in_flight <= 0 || max_queue < 0) return MLORA_E_INVALID;
    mlora_resident *r = new (std::nothrow) mlora_resident();
    if (!r) return MLORA_E_INVALID;
    r->n_slots = n_slots; r->max_in_flight = max_in_flight; r->max_queue = max_queue;
    r->slot_id.assign((size_t)n_slots, -1);
    r->pinned.assign((size_t)n_slots, 0);
    *out = r;
    return MLORA_OK;
}

void mlora_resident_destroy(mlora_resident *r) { delete r; }

int32_t mlora_resident_register(mlora_resident *r, int64_t catalog_id)
{
    if (!r || catalog_id < 0) return MLORA_E_INVALID;
    std::lock_guard<std::mutex> g(r->mu);
    r->ids.emplace(catalog_id, Entry());        // keeps an existing entry
    return MLORA_OK;
}

int32_t mlora_resident_lookup(mlora_resident *r, int64_t catalog_id)
{
    if (!r) return -1;
    std::lock_guard<std::mutex> g(r->mu);
    auto it = r->ids.find(catalog_id);
    return it != r->ids.end() && it->second.state == kReady ? it->second.slot : -1;
}

int32_t mlora_resident_request(mlora_resident *r, int64_t catalog_id, int32_t *slot, int64_t *evicted_id)
{
    if (!r || !slot || !evicted_id) return MLORA_E_INVALID;
    std::lock_guard<std::mutex> g(r->mu);
    *slot = -1; *evicted_id = -1;
    auto it = r->ids.find(catalog_id);
    if (it == r->ids.end()) return MLORA_E_INVALID;          // not registered: the control plane does not know it
    Entry &e = it->second;
    switch (e.state) {
        case kReady:
            r->lru.splice(r->lru.begin(), r->lru, e.lru);
            *slot = e.slot;
            r->stats[MLORA_STAT_HITS] += 1;
            return MLORA_R_READY;
        case kPrewarming:
        case kQueued:
            r->stats[MLORA_STAT_SHARED] += 1;                // rides on the load that is already scheduled
            return MLORA_R_PENDING;
        case kRegistered:
            break;
    }
    if (r->start(catalog_id, e, slot, evicted_id)) return MLORA_R_LOAD;
    if ((int32_t)r->queue.size() < r->max_queue) {
        e.state = kQueued;
        r->queue.push_back(catalog_id);
        return MLORA_R_QUEUED;
    }
    r->stats[MLORA_STAT_REJECTS] += 1;
    return MLORA_R_REJECTED;
}

// Ends the load job of catalog_id (ok != 0: the adapter is now ready; ok == 0: the load failed and
// the id falls back to registered).  If a queued job can start now, it is returned through next_*.
int32_t mlora_resident_complete(mlora_resident *r, int64_t catalog_id, int32_t ok, int64_t *next_id,
                                int32_t *next_slot, int64_t *evicted_id)
{
    if (!r || !next_id || !next_slot || !evicted_id) return MLORA_E_INVALID;
    std::lock_guard<std::mutex> g(r->mu);
    *next_id = -1; *next_slot = -1; *evicted_id = -1;
    auto it = r->ids.find(catalog_id);
    if (it == r->ids.end() || it->second.state != kPrewarming) return MLORA_E_INVALID;
    Entry &e = it->second;
    r->in_flight -= 1;
    if (ok) {
        e.state = kReady;
        r->lru.push_front(catalog_id);
        e.lru = r->lru.begin();
    } else {
        r->slot_id[e.slot] = -1;
        e.state = kRegistered; e.slot = -1;
    }
    while (!r->queue.empty()) {
        const int64_t id = r->queue.front();
        Entry &q = r->ids[id];
        if (!r->start(id, q, next_slot, evicted_id)) break;  // no slot can be taken yet: it stays queued
        r->queue.pop_front();
        *next_id = id;
        break;
    }
    return MLORA_OK;
}

int32_t mlora_resident_pin(mlora_resident *r, int32_t slot, int32_t pinned)
{
    if (!r || slot < 0 || slot >= r->n_slots) return MLORA_E_SLOT;
    std::lock_guard<std::mutex> g(r->mu);
    r->pinned[slot] = pinned ? 1 : 0;
    return MLORA_OK;
}

int32_t mlora_resident_stats(mlora_resident *r, int64_t *out)
{
    if (!r || !out) return MLORA_E_INVALID;
    std::lock_guard<std::mutex> g(r->mu);
    for (int k = 0; k < MLORA_RESIDENT_STATS; ++k) out[k] = r->stats[k];
    return MLORA_OK;
}

}  // extern "C"
