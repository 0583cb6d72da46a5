// The striped device arena of kdn_arena.h: host code over HIP's virtual memory calls; the
// only device work is the library's own bandwidth yardstick (kdn_probe_stream), used to
// report what the striping gained.
#include "kdn_arena.h"
#include "kdn_blocklist.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <cstring>
#include <map>
#include <mutex>
#include <numeric>
#include <random>
#include <utility>
#include <vector>

namespace {

using Handle = hipMemGenericAllocationHandle_t;

constexpr size_t kMiB = (size_t)1 << 20, kGiB = (size_t)1 << 30;
constexpr int32_t kTileKib = 32;           // the tile of the Llama shapes at block size 16
constexpr size_t kTileBytes = (size_t)kTileKib << 10;
constexpr size_t kWindowMax = kGiB;        // the rates are measured over at most this much
constexpr size_t kWindowMin = 64 * kMiB;   // and not at all on an arena smaller than this
constexpr size_t kMargin = 2 * kGiB;       // left free while the granules are held
constexpr double kGolden = 0.3819660112501051; // 2 - golden ratio: the stride, as a share of the free granules
constexpr size_t kAlign = 4096;

struct Arena {
    size_t bytes = 0, granule = 0;
    void *va = nullptr;
    std::vector<Handle> handles;          // one per granule, in address order
    kdn_impl::BlockList blocks;           // what is handed out
    kdn_arena_info info{};
};

std::mutex g_mu;
std::map<int, Arena> g_arena;

double now()
{
    return std::chrono::duration<double>(std::chrono::steady_clock::now().time_since_epoch()).count();
}

// Scattered tile writes over a mapped window, timed: half of the window's tiles, drawn at
// random, each written once per launch from a source that is read in order.
struct Prober {
    size_t window = 0;                    // bytes
    uint32_t tiles = 0;
    void *src = nullptr;
    int32_t *ids = nullptr;
    hipEvent_t t0 = nullptr, t1 = nullptr;

    bool setup(size_t window_bytes)
    {
        window = window_bytes;
        const size_t all = window / kTileBytes;
        tiles = (uint32_t)(all / 2);
        std::vector<int32_t> perm(all);
        std::iota(perm.begin(), perm.end(), 0);
        std::mt19937_64 rng(20240913);
        for (size_t i = all - 1; i > 0; --i)
            std::swap(perm[i], perm[rng() % (i + 1)]);
        const size_t src_bytes = (size_t)tiles * (kTileBytes / 2);
        return hipMalloc(&src, src_bytes) == hipSuccess && hipMemset(src, 0x3c, src_bytes) == hipSuccess
               && hipMalloc(reinterpret_cast<void **>(&ids), tiles * sizeof(int32_t)) == hipSuccess
               && hipMemcpy(ids, perm.data(), tiles * sizeof(int32_t), hipMemcpyHostToDevice) == hipSuccess
               && hipEventCreate(&t0) == hipSuccess && hipEventCreate(&t1) == hipSuccess;
    }

    // GB/s of algorithmic bytes (16 KiB read and 32 KiB written per tile); 0 after a failure.
    // Returns with the device idle, so the caller may unmap the window.
    double rate(void *mapped)
    {
        constexpr int kTimed = 4;
        bool ok = kdn_probe_stream(src, mapped, ids, tiles, kTileKib, 0, 0, nullptr) == KDN_OK
                  && hipEventRecord(t0, nullptr) == hipSuccess;
        for (int r = 0; ok && r < kTimed; ++r)
            ok = kdn_probe_stream(src, mapped, ids, tiles, kTileKib, 0, 0, nullptr) == KDN_OK;
        ok = ok && hipEventRecord(t1, nullptr) == hipSuccess;
        float ms = 0.0f;
        ok = (hipDeviceSynchronize() == hipSuccess) && ok && hipEventElapsedTime(&ms, t0, t1) == hipSuccess;
        if (!ok || !(ms > 0.0f)) {
            (void)hipGetLastError();
            return 0.0;
        }
        return (double)tiles * kTileBytes * 1.5 / (ms / kTimed * 1e6);
    }

    void teardown()
    {
        if (t0)
            (void)hipEventDestroy(t0);
        if (t1)
            (void)hipEventDestroy(t1);
        if (ids)
            (void)hipFree(ids);
        if (src)
            (void)hipFree(src);
        src = nullptr;
        ids = nullptr;
        t0 = t1 = nullptr;
    }
};

void release_all(std::vector<Handle> &h, const std::vector<char> *keep = nullptr)
{
    for (size_t i = 0; i < h.size(); ++i)
        if (!keep || !(*keep)[i])
            (void)hipMemRelease(h[i]);
}

void fill_info(const Arena &a, kdn_arena_info *out)
{
    *out = a.info;
    out->in_use = a.blocks.in_use();
    out->largest_free = a.blocks.largest_free();
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
    hipMemAccessDesc access{};
    access.location = prop.location;
    access.flags = hipMemAccessFlagsProtReadWrite;
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

    // the measuring buffers are taken before the free memory is
    const size_t window = std::min(kWindowMax, a.bytes) / G * G;
    Prober p;
    bool measure = window >= kWindowMin && window % kTileBytes == 0 && p.setup(window);
    if (!measure) {
        (void)hipGetLastError();
        p.teardown();
    }
    if (hipMemGetInfo(&free_b, &total_b) != hipSuccess || free_b < kMargin + n * G) {
        (void)hipGetLastError();
        p.teardown();
        return KDN_ESIZE;
    }

    // every free granule, in the order the driver hands them out
    std::vector<Handle> h;
    const size_t take = (free_b - kMargin) / G;
    h.reserve(take);
    for (size_t i = 0; i < take; ++i) {
        Handle x;
        if (hipMemCreate(&x, G, &prop, 0) != hipSuccess) {
            (void)hipGetLastError();
            break;
        }
        h.push_back(x);
    }
    const size_t N = h.size();
    if (N < n) {
        release_all(h);
        p.teardown();
        return KDN_ESIZE;
    }

    // granule i of the arena is free granule (i * stride) mod N: neighbours in the arena lie
    // 0.38 of the free memory apart, and no granule is taken twice because the stride shares
    // no factor with N
    size_t stride = std::max<size_t>(1, (size_t)(kGolden * (double)N));
    while (std::gcd(stride, N) != 1)
        ++stride;
    std::vector<char> taken(N, 0);
    a.handles.reserve(n);
    for (size_t i = 0; i < n; ++i) {
        const size_t g = (size_t)(((unsigned __int128)i * stride) % N);
        taken[g] = 1;
        a.handles.push_back(h[g]);
    }
    a.info.free_granules = N;
    a.info.stride = stride;

    kdn_status rc = KDN_OK;
    size_t mapped = 0;
    if (hipMemAddressReserve(&a.va, a.bytes, 0, nullptr, 0) != hipSuccess) {
        a.va = nullptr;
        rc = KDN_EDEVICE;
    }
    for (size_t i = 0; rc == KDN_OK && i < n; ++i) {
        if (hipMemMap(static_cast<char *>(a.va) + i * G, G, 0, a.handles[i], 0) != hipSuccess)
            rc = KDN_EDEVICE;
        else
            ++mapped;
    }
    if (rc == KDN_OK && hipMemSetAccess(a.va, a.bytes, &access, 1) != hipSuccess)
        rc = KDN_EDEVICE;
    if (rc != KDN_OK) {
        (void)hipGetLastError();
        for (size_t i = 0; i < mapped; ++i)
            (void)hipMemUnmap(static_cast<char *>(a.va) + i * G, G);
        if (a.va)
            (void)hipMemAddressFree(a.va, a.bytes);
        release_all(h);
        p.teardown();
        return rc;
    }

    // what the striping gained, for the record: the same scattered writes over the head of the
    // arena and over as many granules that follow one another in the driver's order
    if (measure) {
        a.info.striped_gbs = (float)p.rate(a.va);
        std::vector<size_t> run; // the first untaken granules, in the driver's order
        const size_t want = window / G;
        for (size_t g = 0; g < N && run.size() < want; ++g)
            if (!taken[g])
                run.push_back(g);
        void *w = nullptr;
        if (run.size() == want && hipMemAddressReserve(&w, window, 0, nullptr, 0) == hipSuccess) {
            size_t m = 0;
            bool ok = true;
            for (; ok && m < want; ++m)
                ok = hipMemMap(static_cast<char *>(w) + m * G, G, 0, h[run[m]], 0) == hipSuccess;
            if (!ok)
                --m;
            if (ok && hipMemSetAccess(w, window, &access, 1) == hipSuccess)
                a.info.packed_gbs = (float)p.rate(w);
            for (size_t i = 0; i < m; ++i)
                (void)hipMemUnmap(static_cast<char *>(w) + i * G, G);
            (void)hipMemAddressFree(w, window);
        }
        (void)hipGetLastError();
    }
    p.teardown();
    release_all(h, &taken);

    a.blocks = kdn_impl::BlockList(a.bytes, kAlign);
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
    size_t off = 0;
    if (!a.blocks.take((size_t)bytes, &off))
        return KDN_ESIZE;
    *ptr_out = static_cast<char *>(a.va) + off;
    return KDN_OK;
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
    return a.blocks.give((size_t)(p - base)) ? KDN_OK : KDN_EINVAL;
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
