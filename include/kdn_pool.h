/*
 * kdn_pool.h -- the text-keyed index of stored KV chunks.
 *
 * The paper's storage module keeps KV caches under the texts they belong to (Sec. 3.1),
 * and the engine-facing interface names a KV cache by its text both when it hands one in
 * and when it asks for one (Sec. 3.2, interface (i) and (ii)).  This is that index: a host-side map from a token-id sequence to the descriptor of a stored chunk,
 * bounded by a byte capacity, with recency- or frequency-based eviction (the paper
 * argues that a small part of the knowledge serves most requests, Sec. 2.2).
 *
 * The index holds descriptors only.  Chunk buffers stay owned by the caller: an insert
 * hands back the descriptors it evicted so that the caller can release their memory.
 * All pointers are [host].  Calls on one pool are serialised by an internal mutex.
 * No GPU work happens here.
 */
#ifndef KDN_POOL_H
#define KDN_POOL_H

#include "kdn.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct kdn_pool kdn_pool;

typedef enum {
    KDN_POOL_LRU = 0, /* evict the entry used longest ago */
    KDN_POOL_LFU = 1  /* evict the entry with the fewest uses, oldest first among equals */
} kdn_pool_policy;

typedef struct {
    uint64_t hits, misses, inserts, evictions;
    uint64_t bytes;   /* sum of chunk.bytes of the resident entries */
    uint64_t entries;
} kdn_pool_stats;

/* A pool that keeps at most capacity_bytes of chunks (by their `bytes` field).
 * KDN_EINVAL on a NULL out pointer, zero capacity or unknown policy. */
kdn_status kdn_pool_create(uint64_t capacity_bytes, int32_t policy, kdn_pool **out);

/* Destroys the index (not the chunk buffers).  NULL is allowed. */
void kdn_pool_destroy(kdn_pool *pool);

/* 64-bit FNV-1a hash of the token ids' bytes, the hash the pool buckets by (exposed so
 * that callers can shard by it).  Lookups compare the full sequence, not the hash. */
uint64_t kdn_pool_hash(const int32_t *token_ids, int32_t n_tokens);

/* Retrieve by text.  On a hit copies the descriptor to *out (may be NULL), counts a use
 * and returns KDN_OK; on a miss returns KDN_ENOTFOUND. */
kdn_status kdn_pool_lookup(kdn_pool *pool, const int32_t *token_ids, int32_t n_tokens, kdn_chunk *out);

/* Store with text.  Registers *chunk under the token ids; an entry already present under
 * the same ids is replaced (and reported as evicted).  Entries are evicted by the policy
 * until the new total fits the capacity; their descriptors are written to evicted[0 ..
 * *n_evicted) (evicted: array of max_evicted, may be NULL when max_evicted is 0).
 * KDN_ESIZE if the chunk alone exceeds the capacity, or if more than max_evicted entries
 * would have to go (then nothing is changed). */
kdn_status kdn_pool_insert(kdn_pool *pool, const int32_t *token_ids, int32_t n_tokens,
                           const kdn_chunk *chunk, kdn_chunk *evicted, int32_t max_evicted,
                           int32_t *n_evicted);

/* Removes an entry; its descriptor goes to *out (may be NULL).  KDN_ENOTFOUND on a miss. */
kdn_status kdn_pool_remove(kdn_pool *pool, const int32_t *token_ids, int32_t n_tokens, kdn_chunk *out);

kdn_status kdn_pool_get_stats(kdn_pool *pool, kdn_pool_stats *out);

#ifdef __cplusplus
}
#endif
#endif /* KDN_POOL_H */
