// Text-keyed index of stored KV chunks (include/kdn_pool.h): the storage module's map
// from a text to its KV cache (Sec. 3.1) behind the store / retrieve interface (Sec. 3.2).  Host code only: a hash map from token-id sequences to chunk descriptors,
// a recency list, use counters, and eviction to a byte capacity.
#include <cstdint>
#include <cstring>
#include <list>
#include <mutex>
#include <new>
#include <unordered_map>
#include <vector>

#include "kdn_pool.h"

namespace {

struct Entry {
    std::vector<int32_t> ids;
    kdn_chunk chunk;
    uint64_t uses;      // lookups that hit, plus the insert
    uint64_t stamp;     // logical time of the last use
};

using Order = std::list<Entry>; // front = most recently used

} // namespace

struct kdn_pool {
    std::mutex mu;
    uint64_t capacity = 0;
    int32_t policy = KDN_POOL_LRU;
    uint64_t clock = 0;
    Order order;
    std::unordered_multimap<uint64_t, Order::iterator> index; // hash -> entries (full ids compared)
    kdn_pool_stats stats = {};

    Order::iterator find(uint64_t h, const int32_t *ids, int32_t n)
    {
        auto range = index.equal_range(h);
        for (auto it = range.first; it != range.second; ++it) {
            const Entry &e = *it->second;
            if ((int32_t)e.ids.size() == n && std::memcmp(e.ids.data(), ids, (size_t)n * 4) == 0)
                return it->second;
        }
        return order.end();
    }

    void unlink(Order::iterator e)
    {
        const uint64_t h = kdn_pool_hash(e->ids.data(), (int32_t)e->ids.size());
        auto range = index.equal_range(h);
        for (auto it = range.first; it != range.second; ++it)
            if (it->second == e) {
                index.erase(it);
                break;
            }
        stats.bytes -= e->chunk.bytes;
        stats.entries -= 1;
        order.erase(e);
    }
};

extern "C" {

uint64_t kdn_pool_hash(const int32_t *token_ids, int32_t n_tokens)
{
    uint64_t h = 1469598103934665603ull;
    const unsigned char *p = reinterpret_cast<const unsigned char *>(token_ids);
    for (int64_t i = 0; token_ids && i < (int64_t)n_tokens * 4; ++i) {
        h ^= p[i];
        h *= 1099511628211ull;
    }
    return h;
}

kdn_status kdn_pool_create(uint64_t capacity_bytes, int32_t policy, kdn_pool **out)
{
    if (!out || capacity_bytes == 0 || (policy != KDN_POOL_LRU && policy != KDN_POOL_LFU))
        return KDN_EINVAL;
    kdn_pool *p = new (std::nothrow) kdn_pool;
    if (!p)
        return KDN_EDEVICE;
    p->capacity = capacity_bytes;
    p->policy = policy;
    *out = p;
    return KDN_OK;
}

void kdn_pool_destroy(kdn_pool *pool) { delete pool; }

kdn_status kdn_pool_lookup(kdn_pool *pool, const int32_t *token_ids, int32_t n_tokens, kdn_chunk *out)
{
    if (!pool || !token_ids || n_tokens <= 0)
        return KDN_EINVAL;
    std::lock_guard<std::mutex> lock(pool->mu);
    auto e = pool->find(kdn_pool_hash(token_ids, n_tokens), token_ids, n_tokens);
    if (e == pool->order.end()) {
        pool->stats.misses += 1;
        return KDN_ENOTFOUND;
    }
    pool->stats.hits += 1;
    e->uses += 1;
    e->stamp = ++pool->clock;
    pool->order.splice(pool->order.begin(), pool->order, e);
    if (out)
        *out = e->chunk;
    return KDN_OK;
}

kdn_status kdn_pool_insert(kdn_pool *pool, const int32_t *token_ids, int32_t n_tokens,
                           const kdn_chunk *chunk, kdn_chunk *evicted, int32_t max_evicted,
                           int32_t *n_evicted)
{
    if (n_evicted)
        *n_evicted = 0;
    if (!pool || !token_ids || n_tokens <= 0 || !chunk || max_evicted < 0 || (max_evicted > 0 && !evicted))
        return KDN_EINVAL;
    std::lock_guard<std::mutex> lock(pool->mu);
    if (chunk->bytes > pool->capacity)
        return KDN_ESIZE;
    const uint64_t h = kdn_pool_hash(token_ids, n_tokens);
    auto same = pool->find(h, token_ids, n_tokens);
    // plan the evictions first so that a failure changes nothing
    std::vector<Order::iterator> out;
    uint64_t bytes = pool->stats.bytes;
    if (same != pool->order.end()) {
        out.push_back(same);
        bytes -= same->chunk.bytes;
    }
    if (bytes + chunk->bytes > pool->capacity) {
        if (pool->policy == KDN_POOL_LRU) {
            for (auto it = pool->order.end(); it != pool->order.begin() && bytes + chunk->bytes > pool->capacity;) {
                --it;
                if (it == same)
                    continue;
                out.push_back(it);
                bytes -= it->chunk.bytes;
            }
        } else {
            // fewest uses first, oldest first among equals
            std::vector<Order::iterator> cand;
            for (auto it = pool->order.begin(); it != pool->order.end(); ++it)
                if (it != same)
                    cand.push_back(it);
            while (bytes + chunk->bytes > pool->capacity && !cand.empty()) {
                size_t best = 0;
                for (size_t i = 1; i < cand.size(); ++i)
                    if (cand[i]->uses < cand[best]->uses
                        || (cand[i]->uses == cand[best]->uses && cand[i]->stamp < cand[best]->stamp))
                        best = i;
                out.push_back(cand[best]);
                bytes -= cand[best]->chunk.bytes;
                cand.erase(cand.begin() + (long)best);
            }
        }
    }
    if (bytes + chunk->bytes > pool->capacity || (int32_t)out.size() > max_evicted)
        return KDN_ESIZE;
    for (size_t i = 0; i < out.size(); ++i) {
        evicted[i] = out[i]->chunk;
        pool->unlink(out[i]);
        pool->stats.evictions += 1;
    }
    if (n_evicted)
        *n_evicted = (int32_t)out.size();
    Entry e;
    e.ids.assign(token_ids, token_ids + n_tokens);
    e.chunk = *chunk;
    e.uses = 1;
    e.stamp = ++pool->clock;
    pool->order.push_front(std::move(e));
    pool->index.emplace(h, pool->order.begin());
    pool->stats.bytes += chunk->bytes;
    pool->stats.entries += 1;
    pool->stats.inserts += 1;
    return KDN_OK;
}

kdn_status kdn_pool_remove(kdn_pool *pool, const int32_t *token_ids, int32_t n_tokens, kdn_chunk *out)
{
    if (!pool || !token_ids || n_tokens <= 0)
        return KDN_EINVAL;
    std::lock_guard<std::mutex> lock(pool->mu);
    auto e = pool->find(kdn_pool_hash(token_ids, n_tokens), token_ids, n_tokens);
    if (e == pool->order.end())
        return KDN_ENOTFOUND;
    if (out)
        *out = e->chunk;
    pool->unlink(e);
    return KDN_OK;
}

kdn_status kdn_pool_get_stats(kdn_pool *pool, kdn_pool_stats *out)
{
    if (!pool || !out)
        return KDN_EINVAL;
    std::lock_guard<std::mutex> lock(pool->mu);
    *out = pool->stats;
    return KDN_OK;
}

} // extern "C"
