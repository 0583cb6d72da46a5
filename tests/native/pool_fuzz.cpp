// Host-only stress of the text-keyed index, meant to be built with
// -fsanitize=address,undefined: random lookups, inserts, replacements and removals with
// invariants checked after every call.  Exit code 0 means no violation and no report.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <map>
#include <random>
#include <vector>

#include "kdn_pool.h"

static int fail(const char *what, int step)
{
    std::fprintf(stderr, "pool_fuzz: %s at step %d\n", what, step);
    return 1;
}

int main()
{
    for (int policy = 0; policy < 2; ++policy) {
        kdn_pool *pool = nullptr;
        if (kdn_pool_create(5000, policy, &pool) != KDN_OK)
            return fail("create", -1);
        std::mt19937 rng(1234 + policy);
        std::map<int, uint64_t> resident; // key id -> bytes
        uint64_t bytes = 0;
        for (int step = 0; step < 20000; ++step) {
            const int key = (int)(rng() % 40);
            std::vector<int32_t> ids(3 + key % 7);
            for (size_t i = 0; i < ids.size(); ++i)
                ids[i] = key * 131 + (int32_t)i;
            const unsigned op = rng() % 10;
            kdn_chunk c = {};
            if (op < 5) {
                const kdn_status st = kdn_pool_lookup(pool, ids.data(), (int32_t)ids.size(), &c);
                const bool have = resident.count(key) != 0;
                if ((st == KDN_OK) != have)
                    return fail("lookup disagrees with the shadow map", step);
                if (have && c.bytes != resident[key])
                    return fail("lookup returned another entry", step);
            } else if (op < 9) {
                c.bytes = 100 + rng() % 900;
                c.data = reinterpret_cast<void *>((uintptr_t)(key + 1) << 12);
                kdn_chunk ev[64];
                int32_t n_ev = 0;
                const kdn_status st = kdn_pool_insert(pool, ids.data(), (int32_t)ids.size(), &c, ev, 64, &n_ev);
                if (st != KDN_OK)
                    return fail("insert refused", step);
                for (int i = 0; i < n_ev; ++i) {
                    const int k = (int)(((uintptr_t)ev[i].data >> 12) - 1);
                    if (!resident.count(k) || resident[k] != ev[i].bytes)
                        return fail("evicted an entry that was not resident", step);
                    bytes -= resident[k];
                    resident.erase(k);
                }
                if (resident.count(key))
                    return fail("replaced entry was not reported", step);
                resident[key] = c.bytes;
                bytes += c.bytes;
            } else {
                const kdn_status st = kdn_pool_remove(pool, ids.data(), (int32_t)ids.size(), &c);
                if ((st == KDN_OK) != (resident.count(key) != 0))
                    return fail("remove disagrees with the shadow map", step);
                if (st == KDN_OK) {
                    bytes -= resident[key];
                    resident.erase(key);
                }
            }
            kdn_pool_stats s;
            kdn_pool_get_stats(pool, &s);
            if (s.bytes != bytes || s.entries != resident.size() || s.bytes > 5000)
                return fail("byte or entry accounting", step);
        }
        kdn_pool_destroy(pool);
    }
    std::puts("pool_fuzz ok");
    return 0;
}
