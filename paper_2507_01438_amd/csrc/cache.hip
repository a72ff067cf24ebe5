// The adapter memory manager (Sec. 3.3 / 4.2 of the paper): which adapter sits in which block of the pre-allocated
// pool, least-recently-used replacement, a stack of free blocks, and the events that order adapter loads on one
// stream against linear calls on another.  Host code only; no kernel here.
//
// Recency is a doubly linked list threaded through per-block arrays (head = least recently used), adapter id ->
// block is a hash map: a request costs O(1) unless pinned adapters have to be skipped on the way to a victim.
#include <unordered_map>
#include <vector>

#include "common.h"

using namespace elora;

namespace {
constexpr int kRing = 64;  // loads (batches) whose "done" event is kept; an older one is stood in for by a later one
}

struct elora_cache {
    int capacity = 0;
    std::unordered_map<int, int> block_of;  // adapter id -> block
    std::vector<int> id, prev, next, pins;  // per block: adapter (-1 free), neighbours in recency order, pin count
    std::vector<int> free_stack;
    int head = -1, tail = -1;               // least / most recently used block
    long long hits = 0, requests = 0, evictions = 0;
    // device-side order
    std::vector<long long> last_load;       // per block: number (from 1) of the load call that filled it last, 0 none
    std::vector<long long> last_batch;      // per block: number (from 1) of the last batch that used it, 0 none
    hipEvent_t load_done[kRing] = {}, batch_done[kRing] = {};
    long long n_loads = 0, n_batches = 0;   // load calls and batches so far
    long long compute_waited_load = 0;      // the compute stream has waited for every load up to this number
    long long copy_waited_batch = 0;        // the copy stream has waited for every batch up to this number

    void unlink(int b)
    {
        if (prev[b] >= 0) next[prev[b]] = next[b]; else head = next[b];
        if (next[b] >= 0) prev[next[b]] = prev[b]; else tail = prev[b];
        prev[b] = next[b] = -1;
    }
    void push_most_recent(int b)
    {
        prev[b] = tail;
        next[b] = -1;
        if (tail >= 0) next[tail] = b; else head = b;
        tail = b;
    }
};

extern "C" {

int elora_cache_create(int capacity, elora_cache_t **out)
{
    if (!out) return ELORA_E_NULL;
    if (capacity < 1) return ELORA_E_SHAPE;
    elora_cache *c = new (std::nothrow) elora_cache;
    if (!c) return ELORA_E_STORAGE;
    try {  // (host memory: nothing is thrown across the C boundary)
        c->capacity = capacity;
        c->id.assign(capacity, -1);
        c->prev.assign(capacity, -1);
        c->next.assign(capacity, -1);
        c->pins.assign(capacity, 0);
        c->free_stack.resize(capacity);
        for (int i = 0; i < capacity; ++i) c->free_stack[i] = capacity - 1 - i;  // block 0 comes off first
        c->last_load.assign(capacity, 0);
        c->last_batch.assign(capacity, 0);
        c->block_of.reserve((size_t)capacity * 2);
    } catch (...) {
        delete c;
        return ELORA_E_STORAGE;
    }
    *out = c;
    return ELORA_OK;
}

int elora_cache_destroy(elora_cache_t *c)
{
    if (!c) return ELORA_E_NULL;
    for (hipEvent_t e : c->load_done)
        if (e) (void)hipEventDestroy(e);
    for (hipEvent_t e : c->batch_done)
        if (e) (void)hipEventDestroy(e);
    delete c;
    return ELORA_OK;
}

int elora_cache_acquire(elora_cache_t *c, int adapter_id, int *slot, int *hit, int *evicted_id)
{
    if (!c || !slot || !hit || !evicted_id) return ELORA_E_NULL;
    if (adapter_id < 0) return ELORA_E_SHAPE;
    auto it = c->block_of.find(adapter_id);
    if (it != c->block_of.end()) {
        const int b = it->second;
        c->unlink(b);
        c->push_most_recent(b);
        ++c->pins[b];
        ++c->requests;
        ++c->hits;
        *slot = b;
        *hit = 1;
        *evicted_id = -1;
        return ELORA_OK;
    }
    int b, victim_id = -1;
    if (!c->free_stack.empty()) {
        b = c->free_stack.back();
        c->free_stack.pop_back();
    } else {
        b = c->head;
        while (b >= 0 && c->pins[b] > 0) b = c->next[b];
        if (b < 0) return ELORA_E_BUSY;
        victim_id = c->id[b];
        c->block_of.erase(victim_id);
        c->unlink(b);
        ++c->evictions;
    }
    try {
        c->block_of.emplace(adapter_id, b);
    } catch (...) {  // out of host memory: the block stays free (a victim, if there was one, stays evicted)
        c->id[b] = -1;
        c->pins[b] = 0;
        c->free_stack.push_back(b);
        return ELORA_E_STORAGE;
    }
    c->id[b] = adapter_id;
    c->pins[b] = 1;
    c->push_most_recent(b);
    ++c->requests;
    *slot = b;
    *hit = 0;
    *evicted_id = victim_id;
    return ELORA_OK;
}

int elora_cache_release(elora_cache_t *c, int adapter_id)
{
    if (!c) return ELORA_E_NULL;
    auto it = c->block_of.find(adapter_id);
    if (it == c->block_of.end() || c->pins[it->second] <= 0) return ELORA_E_NOT_LOADED;
    --c->pins[it->second];
    return ELORA_OK;
}

int elora_cache_acquire_batch(elora_cache_t *c, const int *adapter_ids, int n, int *slots, int *miss_ids, int *miss_slots,
                              int *n_miss)
{
    if (!c || !n_miss || (n > 0 && (!adapter_ids || !slots || !miss_ids || !miss_slots))) return ELORA_E_NULL;
    if (n < 0) return ELORA_E_SHAPE;
    int misses = 0;
    const long long hits0 = c->hits, requests0 = c->requests;
    for (int t = 0; t < n; ++t) {
        if (adapter_ids[t] < 0) {
            slots[t] = -1;
            continue;
        }
        int hit = 0, evicted = -1;
        const int rc = elora_cache_acquire(c, adapter_ids[t], &slots[t], &hit, &evicted);
        if (rc != ELORA_OK) {
            // Undo what this call did: its requests are released and not counted, and the adapters it had assigned
            // blocks to leave the cache again (nothing was ever loaded into those blocks: a later request for one of
            // them must not be a hit).  Their blocks go back on the stack, last assigned first.
            for (int u = 0; u < t; ++u)
                if (adapter_ids[u] >= 0) (void)elora_cache_release(c, adapter_ids[u]);
            for (int i = misses - 1; i >= 0; --i) {
                auto it = c->block_of.find(miss_ids[i]);
                if (it == c->block_of.end()) continue;
                const int b = it->second;
                c->block_of.erase(it);
                c->unlink(b);
                c->id[b] = -1;
                c->pins[b] = 0;
                c->free_stack.push_back(b);
            }
            c->hits = hits0;
            c->requests = requests0;
            return rc;
        }
        if (!hit) {
            miss_ids[misses] = adapter_ids[t];
            miss_slots[misses] = slots[t];
            ++misses;
        }
    }
    *n_miss = misses;
    return ELORA_OK;
}

int elora_cache_release_batch(elora_cache_t *c, const int *adapter_ids, int n)
{
    if (!c || (n > 0 && !adapter_ids)) return ELORA_E_NULL;
    if (n < 0) return ELORA_E_SHAPE;
    int rc = ELORA_OK;
    for (int t = 0; t < n; ++t)
        if (adapter_ids[t] >= 0 && elora_cache_release(c, adapter_ids[t]) != ELORA_OK) rc = ELORA_E_NOT_LOADED;
    return rc;
}

int elora_cache_lookup(const elora_cache_t *c, int adapter_id, int *slot)
{
    if (!c || !slot) return ELORA_E_NULL;
    auto it = c->block_of.find(adapter_id);
    *slot = it == c->block_of.end() ? -1 : it->second;
    return ELORA_OK;
}

int elora_cache_drop(elora_cache_t *c, int adapter_id)
{
    if (!c) return ELORA_E_NULL;
    auto it = c->block_of.find(adapter_id);
    if (it == c->block_of.end()) return ELORA_E_NOT_LOADED;
    const int b = it->second;
    if (c->pins[b] > 0) return ELORA_E_BUSY;
    c->block_of.erase(it);
    c->unlink(b);
    c->id[b] = -1;
    c->free_stack.push_back(b);
    return ELORA_OK;
}

int elora_cache_stats(const elora_cache_t *c, long long *hits, long long *requests, long long *evictions)
{
    if (!c) return ELORA_E_NULL;
    if (hits) *hits = c->hits;
    if (requests) *requests = c->requests;
    if (evictions) *evictions = c->evictions;
    return ELORA_OK;
}

int elora_cache_reset_stats(elora_cache_t *c)
{
    if (!c) return ELORA_E_NULL;
    c->hits = c->requests = c->evictions = 0;
    return ELORA_OK;
}

// Algorithm 1 of the paper after the router: an explicit adapter id wins; otherwise the first of the k most confident
// adapters (descending score; equal scores: lower id first; NaN below everything) that is cached, else the most
// confident one.  Looks only: no request is counted and recency does not change.
int elora_cache_select(const elora_cache_t *c, int explicit_id, const float *scores, int n, int k, int *chosen, int *resident)
{
    if (!c || !chosen || !resident) return ELORA_E_NULL;
    if (explicit_id >= 0) {
        *chosen = explicit_id;
        *resident = c->block_of.count(explicit_id) ? 1 : 0;
        return ELORA_OK;
    }
    if (!scores) return ELORA_E_NULL;
    if (n < 1 || k < 1) return ELORA_E_SHAPE;
    if (k > n) k = n;
    auto better = [&](int a, int b) {  // a before b
        const float sa = scores[a], sb = scores[b];
        const bool na = sa != sa, nb = sb != sb;
        if (na != nb) return nb;
        if (!na && sa != sb) return sa > sb;
        return a < b;
    };
    // the k best, in order: k passes of selection (k is small, Sec. 5: three), each looked up as it is found
    int last = -1, first = -1;
    for (int r = 0; r < k; ++r) {
        int best = -1;
        for (int j = 0; j < n; ++j)
            if ((last < 0 || better(last, j)) && (best < 0 || better(j, best))) best = j;
        if (r == 0) first = best;
        if (c->block_of.count(best)) {
            *chosen = best;
            *resident = 1;
            return ELORA_OK;
        }
        last = best;
    }
    *chosen = first;
    *resident = 0;
    return ELORA_OK;
}

// ---- device-side order ------------------------------------------------------------------------------------------
// Loads all run on one stream and batches all on another, each in the order of the calls here, so "the compute
// stream has waited for load number q" covers every earlier load as well, and likewise for batches: one wait per
// call is enough, and none if an earlier call already waited that far.  Events sit in rings; when a ring comes
// round, the event object of an old load (batch) is recorded again for a new one, and whoever still names the old
// one waits for the new one instead, which ends later on the same stream: never too early.  Every wait refers to
// records made earlier in host order, so the two streams cannot wait for each other in a circle.

static int check_slots(const elora_cache *c, const int *slots, int n)
{
    if (!c || (n > 0 && !slots)) return ELORA_E_NULL;
    if (n < 0) return ELORA_E_SHAPE;
    for (int i = 0; i < n; ++i)
        if (slots[i] >= c->capacity) return ELORA_E_SLOT;  // negative: a row without adapter, skipped
    return ELORA_OK;
}

int elora_cache_load_begin(elora_cache_t *c, const int *slots, int n, elora_stream_t copy_stream)
{
    const int rc = check_slots(c, slots, n);
    if (rc != ELORA_OK) return rc;
    long long latest = 0;  // number (from 1) of the last batch that used any of these blocks
    for (int i = 0; i < n; ++i)
        if (slots[i] >= 0 && c->last_batch[slots[i]] > latest) latest = c->last_batch[slots[i]];
    if (latest > c->copy_waited_batch) {
        ELORA_HIP_TRY(hipStreamWaitEvent(static_cast<hipStream_t>(copy_stream), c->batch_done[(latest - 1) % kRing], 0));
        c->copy_waited_batch = latest;
    }
    return ELORA_OK;
}

int elora_cache_load_end(elora_cache_t *c, const int *slots, int n, elora_stream_t copy_stream)
{
    const int rc = check_slots(c, slots, n);
    if (rc != ELORA_OK) return rc;
    if (n == 0) return ELORA_OK;
    const int r = (int)(c->n_loads % kRing);
    if (!c->load_done[r]) ELORA_HIP_TRY(hipEventCreateWithFlags(&c->load_done[r], hipEventDisableTiming));
    ELORA_HIP_TRY(hipEventRecord(c->load_done[r], static_cast<hipStream_t>(copy_stream)));
    ++c->n_loads;
    for (int i = 0; i < n; ++i)
        if (slots[i] >= 0) c->last_load[slots[i]] = c->n_loads;
    return ELORA_OK;
}

int elora_cache_batch_begin(elora_cache_t *c, const int *slots, int n, elora_stream_t compute_stream)
{
    const int rc = check_slots(c, slots, n);
    if (rc != ELORA_OK) return rc;
    long long latest = 0;
    for (int i = 0; i < n; ++i)
        if (slots[i] >= 0 && c->last_load[slots[i]] > latest) latest = c->last_load[slots[i]];
    if (latest > c->compute_waited_load) {
        ELORA_HIP_TRY(hipStreamWaitEvent(static_cast<hipStream_t>(compute_stream), c->load_done[(latest - 1) % kRing], 0));
        c->compute_waited_load = latest;
    }
    return ELORA_OK;
}

int elora_cache_batch_end(elora_cache_t *c, const int *slots, int n, elora_stream_t compute_stream)
{
    const int rc = check_slots(c, slots, n);
    if (rc != ELORA_OK) return rc;
    if (n == 0) return ELORA_OK;
    const int r = (int)(c->n_batches % kRing);
    if (!c->batch_done[r]) ELORA_HIP_TRY(hipEventCreateWithFlags(&c->batch_done[r], hipEventDisableTiming));
    ELORA_HIP_TRY(hipEventRecord(c->batch_done[r], static_cast<hipStream_t>(compute_stream)));
    ++c->n_batches;
    for (int i = 0; i < n; ++i)
        if (slots[i] >= 0) c->last_batch[slots[i]] = c->n_batches;
    return ELORA_OK;
}

}  // extern "C"
