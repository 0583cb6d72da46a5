// The arena's block list against a page map: random takes and gives, every answer compared
// with a model that marks 4 KiB pages one by one.  Run under ASan/UBSan by test_sanitizers.py.
#include "kdn_blocklist.h"

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

namespace {

constexpr size_t kPage = 4096;

struct Model {
    std::vector<int> owner; // per page: 0 free, else block id
    std::vector<std::pair<size_t, size_t>> blocks; // id -> (first page, pages), pages 0 = gone

    explicit Model(size_t pages) : owner(pages, 0) { blocks.push_back({0, 0}); }

    // first fit by scanning
    bool take(size_t want, size_t *off, int *id)
    {
        const size_t need = (want + kPage - 1) / kPage;
        if (want == 0 || need > owner.size())
            return false;
        size_t run = 0;
        for (size_t p = 0; p < owner.size(); ++p) {
            run = owner[p] ? 0 : run + 1;
            if (run == need) {
                const size_t first = p + 1 - need;
                *id = (int)blocks.size();
                blocks.push_back({first, need});
                for (size_t q = first; q <= p; ++q)
                    owner[q] = *id;
                *off = first * kPage;
                return true;
            }
        }
        return false;
    }

    bool give(size_t off)
    {
        if (off % kPage || off / kPage >= owner.size())
            return false;
        const int id = owner[off / kPage];
        if (!id || blocks[id].first != off / kPage)
            return false;
        for (size_t q = blocks[id].first; q < blocks[id].first + blocks[id].second; ++q)
            owner[q] = 0;
        blocks[id].second = 0;
        return true;
    }

    size_t in_use() const
    {
        size_t n = 0;
        for (int o : owner)
            n += o != 0;
        return n * kPage;
    }

    size_t largest_free(size_t *stretches) const
    {
        size_t best = 0, run = 0, count = 0;
        for (size_t p = 0; p <= owner.size(); ++p) {
            if (p < owner.size() && !owner[p]) {
                ++run;
            } else {
                count += run != 0;
                best = run > best ? run : best;
                run = 0;
            }
        }
        *stretches = count;
        return best * kPage;
    }
};

uint64_t rng_state = 88172645463325252ull;
uint64_t rnd()
{
    rng_state ^= rng_state << 13;
    rng_state ^= rng_state >> 7;
    rng_state ^= rng_state << 17;
    return rng_state;
}

#define CHECK(c)                                                              \
    do {                                                                      \
        if (!(c)) {                                                           \
            std::printf("blocklist_fuzz: line %d: %s\n", __LINE__, #c);       \
            return 1;                                                         \
        }                                                                     \
    } while (0)

} // namespace

int main()
{
    for (int round = 0; round < 20; ++round) {
        const size_t pages = 64 + rnd() % 400;
        kdn_impl::BlockList list(pages * kPage, kPage);
        Model model(pages);
        std::vector<size_t> live;
        for (int step = 0; step < 3000; ++step) {
            const uint64_t what = rnd() % 100;
            if (what < 55) { // take: mostly small, sometimes more than is left
                const size_t want = what < 5 ? rnd() % (pages * kPage * 2) : 1 + rnd() % (24 * kPage);
                size_t a = 0, b = 0;
                int id = 0;
                const bool got = list.take(want, &a), exp = model.take(want, &b, &id);
                CHECK(got == exp);
                if (got) {
                    CHECK(a == b);
                    live.push_back(a);
                }
            } else if (what < 95 && !live.empty()) { // give one back
                const size_t k = rnd() % live.size();
                CHECK(list.give(live[k]) && model.give(live[k]));
                live[k] = live.back();
                live.pop_back();
            } else { // something that is no live block: inside one, freed already, outside the range
                const size_t off = (rnd() % (pages + 8)) * kPage + (rnd() % 3 == 0 ? 8 : 0);
                bool is_live = false;
                for (size_t x : live)
                    is_live = is_live || x == off;
                if (!is_live)
                    CHECK(!list.give(off) && !model.give(off));
            }
            size_t stretches = 0;
            CHECK(list.in_use() == model.in_use());
            CHECK(list.largest_free() == model.largest_free(&stretches));
            CHECK(list.free_stretches() == stretches); // free neighbours are always joined
        }
        for (size_t x : live)
            CHECK(list.give(x));
        CHECK(list.in_use() == 0 && list.largest_free() == pages * kPage && list.free_stretches() == 1);
    }
    kdn_impl::BlockList none;
    size_t off = 0;
    CHECK(!none.take(1, &off) && !none.give(0) && none.largest_free() == 0);
    std::printf("blocklist_fuzz ok\n");
    return 0;
}
