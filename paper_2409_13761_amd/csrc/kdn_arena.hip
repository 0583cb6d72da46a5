// The striped device arena of kdn_arena.h: host code over HIP's virtual memory calls; the
// only device work is the library's own bandwidth yardstick (kdn_probe_stream), used to
// find the memory's regions.
#include "kdn_arena.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <cstring>
#include <map>
#include <mutex>
#include <random>
#include <utility>
#include <vector>

namespace {

using Handle = hipMemGenericAllocationHandle_t;

constexpr size_t kMiB = (size_t)1 << 20, kGiB = (size_t)1 << 30;
constexpr size_t kSideBytes = 512 * kMiB;  // a timed pair is two runs of this size, mapped side by side
constexpr size_t kRunBytes = kGiB;         // the unit of the bisection: a region boundary is found to within one
constexpr int32_t kTileKib = 32;           // the tile of the Llama shapes at block size 16
constexpr uint32_t kProbeTiles = 16384;    // tiles written per launch: half of the pair's tiles, drawn at random
constexpr size_t kMargin = 2 * kGiB;       // left free while the regions are measured
constexpr double kSameFactor = 1.12;       // a pair slower than this times the same-region rate lies in one region
                                           // (measured: 5.0 TB/s inside one region, 6.2 and more across two)
constexpr size_t kAlign = 4096;

struct Arena {
    size_t bytes = 0, granule = 0;
    void *va = nullptr;
    std::vector<Handle> handles;          // one per granule, in address order
    std::map<size_t, size_t> free_at;     // offset -> length, disjoint, never adjacent
    std::map<size_t, size_t> used_at;     // offset -> length
    kdn_arena_info info{};
};

std::mutex g_mu;
std::map<int, Arena> g_arena;

double now()
{
    return std::chrono::duration<double>(std::chrono::steady_clock::now().time_since_epoch()).count();
}

// Times scattered tile writes over two runs of granules mapped side by side.
struct Prober {
    size_t granule = 0;
    size_t per_side = 0;                  // granules per run
    const std::vector<Handle> *h = nullptr;
    hipMemAccessDesc access{};
    void *window = nullptr;               // 2 * kSideBytes of reserved addresses
    void *src = nullptr;                  // kProbeTiles half tiles, read in order
    int32_t *ids = nullptr;               // kProbeTiles distinct tiles of the window
    hipEvent_t t0 = nullptr, t1 = nullptr;
    int probes = 0;
    bool failed = false;

    bool setup(size_t g, const std::vector<Handle> *handles, int device)
    {
        granule = g;
        per_side = kSideBytes / g;
        h = handles;
        access.location.type = hipMemLocationTypeDevice;
        access.location.id = device;
        access.flags = hipMemAccessFlagsProtReadWrite;
        std::vector<int32_t> perm(2 * kSideBytes / ((size_t)kTileKib << 10));
        for (size_t i = 0; i < perm.size(); ++i)
            perm[i] = (int32_t)i;
        std::mt19937_64 rng(20240913);
        for (size_t i = perm.size() - 1; i > 0; --i)
            std::swap(perm[i], perm[rng() % (i + 1)]);
        const size_t src_bytes = (size_t)kProbeTiles * ((size_t)kTileKib << 9);
        return hipMalloc(&src, src_bytes) == hipSuccess && hipMemset(src, 0x3c, src_bytes) == hipSuccess
               && hipMalloc(reinterpret_cast<void **>(&ids), kProbeTiles * sizeof(int32_t)) == hipSuccess
               && hipMemcpy(ids, perm.data(), kProbeTiles * sizeof(int32_t), hipMemcpyHostToDevice) == hipSuccess
               && hipEventCreate(&t0) == hipSuccess && hipEventCreate(&t1) == hipSuccess
               && hipMemAddressReserve(&window, 2 * kSideBytes, 0, nullptr, 0) == hipSuccess;
    }

    // GB/s of algorithmic bytes over granules [g0, g0 + per_side) and [g1, g1 + per_side); 0 after a failure
    double rate(size_t g0, size_t g1)
    {
        if (failed)
            return 0.0;
        char *base = static_cast<char *>(window);
        size_t mapped = 0;
        bool ok = true;
        for (size_t i = 0; ok && i < 2 * per_side; ++i) {
            const Handle x = (*h)[i < per_side ? g0 + i : g1 + (i - per_side)];
            ok = hipMemMap(base + i * granule, granule, 0, x, 0) == hipSuccess;
            mapped += ok;
        }
        ok = ok && hipMemSetAccess(window, 2 * kSideBytes, &access, 1) == hipSuccess;
        float ms = 0.0f;
        if (ok) {
            constexpr int kTimed = 3;
            ok = kdn_probe_stream(src, window, ids, kProbeTiles, kTileKib, 0, 0, nullptr) == KDN_OK
                 && hipEventRecord(t0, nullptr) == hipSuccess;
            for (int r = 0; ok && r < kTimed; ++r)
                ok = kdn_probe_stream(src, window, ids, kProbeTiles, kTileKib, 0, 0, nullptr) == KDN_OK;
            ok = ok && hipEventRecord(t1, nullptr) == hipSuccess;
            // the window is not unmapped under running work, whatever failed above
            ok = (hipDeviceSynchronize() == hipSuccess) && ok && hipEventElapsedTime(&ms, t0, t1) == hipSuccess;
            ms /= kTimed;
        }
        for (size_t i = 0; i < mapped; ++i)
            ok = (hipMemUnmap(base + i * granule, granule) == hipSuccess) && ok;
        ++probes;
        if (!ok || !(ms > 0.0f)) {
            (void)hipGetLastError();
            failed = true;
            return 0.0;
        }
        return kProbeTiles * ((size_t)kTileKib << 10) * 1.5 / (ms * 1e6);
    }

    void teardown()
    {
        if (window)
            (void)hipMemAddressFree(window, 2 * kSideBytes);
        if (t0)
            (void)hipEventDestroy(t0);
        if (t1)
            (void)hipEventDestroy(t1);
        if (ids)
            (void)hipFree(ids);
        if (src)
            (void)hipFree(src);
        window = src = nullptr;
        ids = nullptr;
        t0 = t1 = nullptr;
    }
};

struct Region {
    size_t first, last; // runs of kRunBytes, inclusive
};

// The regions along the allocation order.  Region membership is taken to be monotone along
// it (a region is one stretch of runs), which the caller checks afterwards on other runs.
std::vector<Region> find_regions(Prober &p, size_t n_runs, size_t run, kdn_arena_info &info)
{
    std::vector<Region> out;
    const double base = p.rate(0, p.per_side); // the two halves of the first run
    if (p.failed)
        return out;
    info.same_region_gbs = (float)base;
    const double limit = kSameFactor * base;
    auto same = [&](size_t ref, size_t r) { return p.rate(ref * run, r * run) < limit; };
    size_t ref = 0;
    while (ref + 1 < n_runs && out.size() < KDN_ARENA_MAX_REGIONS && !p.failed) {
        size_t lo = ref, hi = n_runs - 1; // same(ref, lo) holds
        if (same(ref, hi))
            lo = hi;
        while (lo + 1 < hi && !p.failed) {
            const size_t mid = lo + (hi - lo) / 2;
            if (same(ref, mid))
                lo = mid;
            else
                hi = mid;
        }
        out.push_back({ref, lo});
        ref = lo + 2; // the run after a region's last one may lie across the boundary
    }
    if (p.failed)
        out.clear();
    return out;
}

// Runs that the bisection did not start from: one third and two thirds into each region.
bool check_regions(Prober &p, const std::vector<Region> &regions, size_t run, kdn_arena_info &info)
{
    const double limit = kSameFactor * info.same_region_gbs;
    double lowest_cross = 0.0;
    std::vector<std::pair<size_t, size_t>> at;
    for (const Region &r : regions) {
        const size_t len = r.last - r.first + 1;
        at.push_back({r.first + len / 3, r.first + (2 * len) / 3});
    }
    for (size_t i = 0; i < regions.size(); ++i) {
        if (at[i].first != at[i].second && !(p.rate(at[i].first * run, at[i].second * run) < limit))
            return false;
        for (size_t j = i + 1; j < regions.size(); ++j) {
            const double x = p.rate(at[i].first * run, at[j].second * run);
            if (!(x >= limit))
                return false;
            lowest_cross = lowest_cross == 0.0 ? x : std::min(lowest_cross, x);
        }
    }
    info.cross_region_gbs = (float)lowest_cross;
    return !p.failed;
}

void release_all(std::vector<Handle> &h, const std::vector<char> *keep = nullptr)
{
    for (size_t i = 0; i < h.size(); ++i)
        if (!keep || !(*keep)[i])
            (void)hipMemRelease(h[i]);
}

size_t largest_free(const Arena &a)
{
    size_t m = 0;
    for (const auto &kv : a.free_at)
        m = std::max(m, kv.second);
    return m;
}

void fill_info(const Arena &a, kdn_arena_info *out)
{
    *out = a.info;
    out->in_use = 0;
    for (const auto &kv : a.used_at)
        out->in_use += kv.second;
    out->largest_free = largest_free(a);
}

} // namespace

extern "C" {

kdn_status kdn_arena_create(uint64_t bytes, int32_t granule_mib, kdn_arena_info *info_out)
{
    const double t_start = now();
    if (bytes == 0 || granule_mib < 0 || granule_mib > 512 || (granule_mib & (granule_mib - 1)) != 0)
        return KDN_EINVAL;
    std::lock_guard<std::mutex> lock(g_mu);
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess) {
        (void)hipGetLastError();
        return KDN_EDEVICE;
    }
    if (g_arena.count(device))
        return KDN_EINVAL;

    hipMemAllocationProp prop{};
    prop.type = hipMemAllocationTypePinned;
    prop.location.type = hipMemLocationTypeDevice;
    prop.location.id = device;
    size_t min_granule = 0, free_b = 0, total_b = 0;
    if (hipMemGetAllocationGranularity(&min_granule, &prop, hipMemAllocationGranularityRecommended) != hipSuccess
        || min_granule == 0 || hipMemGetInfo(&free_b, &total_b) != hipSuccess) {
        (void)hipGetLastError();
        return KDN_EDEVICE;
    }
    const size_t G = (size_t)(granule_mib ? granule_mib : 16) * kMiB;
    if (G % min_granule != 0)
        return KDN_EINVAL;
    if (bytes > total_b)
        return KDN_ESIZE;
    const size_t n = (size_t)((bytes + G - 1) / G); // granules of the arena

    Arena a;
    a.bytes = n * G;
    a.granule = G;
    a.info.bytes = a.bytes;
    a.info.granule = G;
    a.info.regions = 1;

    // what the measurement needs is taken before the free memory is
    std::vector<Handle> h;
    Prober p;
    const size_t run = kRunBytes / G;
    bool measure = p.setup(G, &h, device);
    if (!measure) {
        (void)hipGetLastError();
        p.teardown();
    }
    if (hipMemGetInfo(&free_b, &total_b) != hipSuccess || free_b < kMargin + n * G) {
        (void)hipGetLastError();
        p.teardown();
        return KDN_ESIZE;
    }
    const size_t take = measure ? (free_b - kMargin) / G : n;
    h.reserve(take);
    for (size_t i = 0; i < take; ++i) {
        Handle x;
        if (hipMemCreate(&x, G, &prop, 0) != hipSuccess) {
            (void)hipGetLastError();
            break;
        }
        h.push_back(x);
    }
    if (h.size() < n) {
        release_all(h);
        p.teardown();
        return KDN_ESIZE;
    }

    // regions, as lists of granules in allocation order
    std::vector<std::vector<size_t>> by;
    const size_t n_runs = h.size() / run;
    if (measure && n_runs >= 4) {
        std::vector<Region> regions = find_regions(p, n_runs, run, a.info);
        // a stretch of a few runs between two boundaries is no region to stripe over
        regions.erase(std::remove_if(regions.begin(), regions.end(),
                                     [&](const Region &r) { return (r.last - r.first + 1) * 10 < n_runs; }),
                      regions.end());
        if (regions.size() >= 2 && check_regions(p, regions, run, a.info)) {
            a.info.verified = 1;
            a.info.regions = (int32_t)regions.size();
            for (size_t i = 0; i < regions.size(); ++i) {
                by.emplace_back();
                for (size_t g = regions[i].first * run; g < (regions[i].last + 1) * run; ++g)
                    by.back().push_back(g);
                a.info.region_bytes[i] = by.back().size() * G;
            }
        } else if (regions.size() == 1 && !p.failed) {
            a.info.verified = 1; // one region is all that is free
        }
    }
    a.info.probes = p.probes;
    p.teardown();
    std::vector<char> taken(h.size(), 0);
    if (by.empty()) {
        a.info.regions = 1;
        a.info.cross_region_gbs = 0.0f;
        std::memset(a.info.region_bytes, 0, sizeof a.info.region_bytes);
        a.info.region_bytes[0] = h.size() * G;
    }

    // granule i of the arena comes from region i mod R; a region that runs out is passed over,
    // and what no region holds is taken from the granules left over, in order
    std::vector<size_t> order;
    order.reserve(n);
    {
        std::vector<size_t> next(by.size(), 0);
        size_t exhausted = 0, turn = 0;
        while (order.size() < n && exhausted < by.size()) {
            const size_t r = turn++ % by.size();
            if (next[r] < by[r].size()) {
                order.push_back(by[r][next[r]++]);
                taken[order.back()] = 1;
                if (next[r] == by[r].size())
                    ++exhausted;
            }
        }
        for (size_t g = 0; g < h.size() && order.size() < n; ++g)
            if (!taken[g]) {
                order.push_back(g);
                taken[g] = 1;
            }
    }
    release_all(h, &taken);

    kdn_status rc = KDN_OK;
    size_t mapped = 0;
    if (hipMemAddressReserve(&a.va, a.bytes, 0, nullptr, 0) != hipSuccess) {
        a.va = nullptr;
        rc = KDN_EDEVICE;
    }
    for (size_t i = 0; rc == KDN_OK && i < n; ++i) {
        if (hipMemMap(static_cast<char *>(a.va) + i * G, G, 0, h[order[i]], 0) != hipSuccess)
            rc = KDN_EDEVICE;
        else
            ++mapped;
    }
    if (rc == KDN_OK) {
        hipMemAccessDesc access{};
        access.location = prop.location;
        access.flags = hipMemAccessFlagsProtReadWrite;
        if (hipMemSetAccess(a.va, a.bytes, &access, 1) != hipSuccess)
            rc = KDN_EDEVICE;
    }
    if (rc != KDN_OK) {
        (void)hipGetLastError();
        for (size_t i = 0; i < mapped; ++i)
            (void)hipMemUnmap(static_cast<char *>(a.va) + i * G, G);
        if (a.va)
            (void)hipMemAddressFree(a.va, a.bytes);
        for (size_t g : order)
            (void)hipMemRelease(h[g]);
        return rc;
    }
    a.handles.reserve(n);
    for (size_t g : order)
        a.handles.push_back(h[g]);
    a.free_at[0] = a.bytes;
    a.info.seconds = (float)(now() - t_start);
    if (info_out)
        fill_info(a, info_out);
    g_arena.emplace(device, std::move(a));
    return KDN_OK;
}

kdn_status kdn_arena_alloc(uint64_t bytes, void **ptr_out)
{
    if (bytes == 0 || !ptr_out)
        return KDN_EINVAL;
    std::lock_guard<std::mutex> lock(g_mu);
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess) {
        (void)hipGetLastError();
        return KDN_EDEVICE;
    }
    auto it = g_arena.find(device);
    if (it == g_arena.end())
        return KDN_ENOTFOUND;
    Arena &a = it->second;
    if (bytes > a.bytes)
        return KDN_ESIZE;
    const size_t want = ((size_t)bytes + kAlign - 1) / kAlign * kAlign;
    for (auto f = a.free_at.begin(); f != a.free_at.end(); ++f) {
        if (f->second < want)
            continue;
        const size_t off = f->first, len = f->second;
        a.free_at.erase(f);
        if (len > want)
            a.free_at[off + want] = len - want;
        a.used_at[off] = want;
        *ptr_out = static_cast<char *>(a.va) + off;
        return KDN_OK;
    }
    return KDN_ESIZE;
}

kdn_status kdn_arena_free(void *ptr_dev)
{
    if (!ptr_dev)
        return KDN_EINVAL;
    std::lock_guard<std::mutex> lock(g_mu);
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess) {
        (void)hipGetLastError();
        return KDN_EDEVICE;
    }
    auto it = g_arena.find(device);
    if (it == g_arena.end())
        return KDN_ENOTFOUND;
    Arena &a = it->second;
    const char *p = static_cast<const char *>(ptr_dev), *base = static_cast<const char *>(a.va);
    if (p < base || p >= base + a.bytes)
        return KDN_EINVAL;
    auto u = a.used_at.find((size_t)(p - base));
    if (u == a.used_at.end())
        return KDN_EINVAL;
    size_t off = u->first, len = u->second;
    a.used_at.erase(u);
    auto after = a.free_at.lower_bound(off);
    if (after != a.free_at.end() && after->first == off + len) { // joins the free stretch behind it
        len += after->second;
        after = a.free_at.erase(after);
    }
    if (after != a.free_at.begin()) {
        auto before = std::prev(after);
        if (before->first + before->second == off) { // and the one in front
            off = before->first;
            len += before->second;
            a.free_at.erase(before);
        }
    }
    a.free_at[off] = len;
    return KDN_OK;
}

kdn_status kdn_arena_query(kdn_arena_info *info_out)
{
    if (!info_out)
        return KDN_EINVAL;
    std::lock_guard<std::mutex> lock(g_mu);
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess) {
        (void)hipGetLastError();
        return KDN_EDEVICE;
    }
    auto it = g_arena.find(device);
    if (it == g_arena.end())
        return KDN_ENOTFOUND;
    fill_info(it->second, info_out);
    return KDN_OK;
}

kdn_status kdn_arena_destroy(void)
{
    std::lock_guard<std::mutex> lock(g_mu);
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess) {
        (void)hipGetLastError();
        return KDN_EDEVICE;
    }
    auto it = g_arena.find(device);
    if (it == g_arena.end())
        return KDN_ENOTFOUND;
    Arena &a = it->second;
    kdn_status rc = hipDeviceSynchronize() == hipSuccess ? KDN_OK : KDN_EDEVICE;
    for (size_t i = 0; i < a.handles.size(); ++i)
        if (hipMemUnmap(static_cast<char *>(a.va) + i * a.granule, a.granule) != hipSuccess)
            rc = KDN_EDEVICE;
    for (Handle x : a.handles)
        if (hipMemRelease(x) != hipSuccess)
            rc = KDN_EDEVICE;
    if (hipMemAddressFree(a.va, a.bytes) != hipSuccess)
        rc = KDN_EDEVICE;
    if (rc != KDN_OK)
        (void)hipGetLastError();
    g_arena.erase(it);
    return rc;
}

} // extern "C"
