// Host planner of the KDN library: argument checks, per-device tables (cos/sin rows,
// segment tables, copy stream), kernel dispatch and the compose plan.  Included by
// kdn.hip only.
#ifndef KDN_PLANNER_H
#define KDN_PLANNER_H

#include <algorithm>
#include <cmath>
#include <cstring>
#include <mutex>
#include <unordered_map>
#include <map>
#include <tuple>
#include <vector>

#include "kdn_kernels.h"

namespace kdn_impl {

constexpr int kFormats = 4; // kdn_format values
constexpr int kPerTokenMaxBlock = 3; // block sizes served by per-token block lookup
constexpr int kFewPasses = 4;        // tiles of at most this many wavefront passes take the narrow place flavour

// Resolved RoPE variant of one call: frequencies either derived from `base` or given.
struct RopeSpec {
    double base = 0.0;
    std::vector<double> freq; // rot/2 explicit frequencies, empty: base^(-2j/rot)
    int32_t rot = 0;
    int32_t pairing = KDN_ROPE_HALF_SPLIT;
};

// cos/sin rows of one (frequencies, rot) pair, one row per offset seen so far.  A row that
// kdn_rope_prepare made resident is pinned: it keeps its place and its contents until
// kdn_rope_release or kdn_shutdown, so a captured graph that holds its index stays valid.
// Rows that a compose brought in by itself are transient and go when the table fills up.
struct RopeTable {
    f32x2 *dev = nullptr;
    double base = 0.0;
    std::vector<double> freq;
    int32_t rot = 0;
    std::unordered_map<int32_t, int32_t> row_of;
    std::vector<uint8_t> pinned;    // per row
    std::vector<int32_t> free_rows; // rows that hold nothing
    int32_t n_pinned = 0;
};

// One direction of the host link: a copy stream and, per half of the caller's staging
// buffer, a "filled" and a "drained" event; the staging range of the direction's last call,
// so that a call in the other direction that reuses the memory can wait for it.
struct LinkDir {
    hipStream_t stream = nullptr;
    hipEvent_t entry = nullptr; // recorded on the caller's stream when a call begins
    hipEvent_t filled[2] = {};
    hipEvent_t drained[2] = {};
    bool drained_valid[2] = {};
    const uint8_t *last_lo = nullptr, *last_hi = nullptr;
};

struct DeviceState {
    std::vector<RopeTable> rope;
    uint8_t *seg_dev = nullptr;                   // kSegSlots * kSegSlotBytes
    uint8_t *seg_host = nullptr;                  // pinned mirror
    hipEvent_t seg_done[kSegSlots] = {};
    bool seg_used[kSegSlots] = {};
    int next_slot = 0;
    LinkDir to_device, to_host; // the link is full duplex: the directions do not share a stream
    uint8_t *static_scratch = nullptr; // this device's copy of the library's static scratch array
};

inline std::mutex g_mu; // guards g_dev and everything in it
inline std::unordered_map<int, DeviceState> g_dev;

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline kdn_status check_shape(int32_t L, int32_t H, int32_t D)
{
    if (L <= 0 || H <= 0 || D <= 0 || L > 32767)
        return KDN_EINVAL;
    if (D % 16 != 0 || D > kMaxHeadDim)
        return KDN_EUNSUPPORTED;
    return KDN_OK;
}

inline kdn_status check_cache(const kdn_cache_desc *c)
{
    if (!c || !c->k_base || !c->v_base)
        return KDN_EINVAL;
    kdn_status st = check_shape(c->num_layers, c->num_kv_heads, c->head_dim);
    if (st != KDN_OK)
        return st;
    if (c->block_size <= 0 || c->num_blocks <= 0)
        return KDN_EINVAL;
    if (c->head_stride < c->head_dim || c->token_stride < 0 || c->block_stride < 0
        || c->layer_stride < 0)
        return KDN_EINVAL;
    if (!aligned16(c->k_base) || !aligned16(c->v_base) || c->head_stride % 8 || c->token_stride % 8
        || c->block_stride % 8 || c->layer_stride % 8)
        return KDN_EALIGN;
    return KDN_OK;
}

inline bool known_format(int32_t fmt)
{
    return fmt == KDN_FMT_RAW_BF16 || fmt == KDN_FMT_INT8_ROWSCALE || fmt == KDN_FMT_INT4_GROUP32
           || fmt == KDN_FMT_FP8_ROWSCALE;
}

inline kdn_status check_chunk(const kdn_chunk *ch, const kdn_cache_desc *c)
{
    if (!ch || !ch->data)
        return KDN_EINVAL;
    if (!known_format(ch->fmt))
        return KDN_EINVAL;
    if (ch->fmt == KDN_FMT_INT4_GROUP32 && ch->head_dim % 32 != 0)
        return KDN_EUNSUPPORTED;
    if (ch->num_layers != c->num_layers || ch->num_kv_heads != c->num_kv_heads
        || ch->head_dim != c->head_dim)
        return KDN_EINVAL;
    if (!aligned16(ch->data))
        return KDN_EALIGN;
    if (ch->parent_tokens <= 0 || ch->num_tokens <= 0 || ch->token_start < 0)
        return KDN_EINVAL;
    if ((int64_t)ch->token_start + ch->num_tokens > ch->parent_tokens)
        return KDN_ERANGE;
    if (ch->bytes < kdn_chunk_bytes(ch->num_layers, ch->num_kv_heads, ch->head_dim,
                                    ch->parent_tokens, ch->fmt))
        return KDN_ESIZE;
    return KDN_OK;
}

inline CacheP make_cache_p(const kdn_cache_desc *c)
{
    CacheP p;
    p.k = static_cast<uint16_t *>(c->k_base);
    p.v = static_cast<uint16_t *>(c->v_base);
    p.layer_stride = c->layer_stride;
    p.block_stride = c->block_stride;
    p.token_stride = c->token_stride;
    p.head_stride = c->head_stride;
    p.L = c->num_layers;
    p.H = c->num_kv_heads;
    p.D = c->head_dim;
    p.bs = c->block_size;
    // token group: 16-token pieces of a block, or a whole block of another size; blocks of
    // a few tokens would leave most of a workgroup idle, so there a group is 16 tokens
    // whose rows each look their own block up
    p.G = (c->block_size > 16 && c->block_size % 16 == 0) ? 16 : c->block_size;
    p.dense = (c->head_stride == c->head_dim
               && c->token_stride == (int64_t)c->num_kv_heads * c->head_dim);
    p.per_token = 0;
    if (c->block_size <= kPerTokenMaxBlock) {
        p.G = 16;
        p.per_token = 1;
        p.dense = 0;
    }
    return p;
}

// number of token groups touched by tokens [s, s+t)
inline int64_t groups_spanned(int64_t s, int64_t t, int32_t G) { return (s + t - 1) / G - s / G + 1; }

inline kdn_status hip_status(hipError_t e) { return e == hipSuccess ? KDN_OK : KDN_EDEVICE; }

inline DeviceState *device_state(int *dev_out)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess)
        return nullptr;
    if (dev_out)
        *dev_out = dev;
    return &g_dev[dev];
}

// The stream and events of one link direction, created on first use.
inline kdn_status ensure_link(LinkDir &ln)
{
    if (ln.stream)
        return KDN_OK;
    if (hipStreamCreateWithFlags(&ln.stream, hipStreamNonBlocking) != hipSuccess)
        return KDN_EDEVICE;
    if (hipEventCreateWithFlags(&ln.entry, hipEventDisableTiming) != hipSuccess)
        return KDN_EDEVICE;
    for (int b = 0; b < 2; ++b)
        if (hipEventCreateWithFlags(&ln.filled[b], hipEventDisableTiming) != hipSuccess
            || hipEventCreateWithFlags(&ln.drained[b], hipEventDisableTiming) != hipSuccess)
            return KDN_EDEVICE;
    return KDN_OK;
}

// Orders a call's first writes to its staging memory [staging, staging + need) behind what
// earlier calls still do there.  Within a direction the stage loop waits per half, which is
// exact only when the halves are the same memory as last time; otherwise, and when the
// other direction's last call used overlapping memory, `first_writer` waits until those
// calls have let go of both halves.
inline kdn_status begin_staging(LinkDir &ln, const LinkDir &other, const uint8_t *staging, uint64_t need,
                                hipStream_t first_writer)
{
    const uint8_t *hi = staging + need;
    const bool same_halves = ln.last_lo == staging && ln.last_hi == hi;
    const bool other_overlaps = other.last_lo && staging < other.last_hi && other.last_lo < hi;
    for (int b = 0; b < 2; ++b) {
        if (!same_halves && ln.drained_valid[b] && hipStreamWaitEvent(first_writer, ln.drained[b], 0) != hipSuccess)
            return KDN_EDEVICE;
        if (other_overlaps && other.drained_valid[b]
            && hipStreamWaitEvent(first_writer, other.drained[b], 0) != hipSuccess)
            return KDN_EDEVICE;
    }
    ln.last_lo = staging;
    ln.last_hi = hi;
    return KDN_OK;
}

inline void destroy_link(LinkDir &ln)
{
    if (!ln.stream)
        return;
    (void)hipStreamDestroy(ln.stream);
    if (ln.entry)
        (void)hipEventDestroy(ln.entry);
    for (int b = 0; b < 2; ++b) {
        if (ln.filled[b])
            (void)hipEventDestroy(ln.filled[b]);
        if (ln.drained[b])
            (void)hipEventDestroy(ln.drained[b]);
    }
    ln = LinkDir();
}

// Validates a caller's RoPE variant for head_dim D.  NULL selects the default
// (all of D rotary, half-split pairs, frequencies from `base`).
inline kdn_status resolve_spec(const kdn_rope_spec *in, double base, int32_t D, RopeSpec &out)
{
    out = RopeSpec();
    out.base = in ? in->base : base;
    out.rot = in && in->rot_dim ? in->rot_dim : D;
    out.pairing = in ? in->pairing : (int32_t)KDN_ROPE_HALF_SPLIT;
    if (out.pairing != KDN_ROPE_HALF_SPLIT && out.pairing != KDN_ROPE_INTERLEAVED)
        return KDN_EINVAL;
    if (out.rot <= 0 || out.rot > D)
        return KDN_EINVAL;
    if (out.rot % 16 != 0) // a lane rotates 8 pairs
        return KDN_EUNSUPPORTED;
    if (in && in->inv_freq) {
        out.freq.assign(in->inv_freq, in->inv_freq + out.rot / 2);
        for (double f : out.freq)
            if (!std::isfinite(f))
                return KDN_EINVAL;
    }
    return KDN_OK;
}

// Returns the cos/sin table of the variant and fills rows[i] for offsets[i] (-1 for a
// zero offset).  New rows are computed in double and uploaded before returning.  With
// `pin` the rows of this call become pinned.  When no row is free, the device is
// synchronised (nothing can still read the table) and every transient row is dropped;
// pinned rows keep their index and contents.  KDN_EFULL when the call needs more rows
// than are not pinned by others.
inline kdn_status rope_rows(DeviceState *ds, const RopeSpec &spec, const int32_t *offsets, int32_t n,
                            int32_t *rows, const f32x2 **table, bool pin = false)
{
    *table = nullptr;
    bool any = false;
    for (int32_t i = 0; i < n; ++i)
        any = any || offsets[i] != 0;
    if (!any) {
        for (int32_t i = 0; i < n; ++i)
            rows[i] = -1;
        return KDN_OK;
    }
    if (spec.freq.empty() && (!(spec.base > 0.0) || !std::isfinite(spec.base)))
        return KDN_EINVAL;
    size_t ti = 0;
    for (; ti < ds->rope.size(); ++ti) {
        const RopeTable &t = ds->rope[ti];
        if (t.rot == spec.rot && t.freq == spec.freq && (!spec.freq.empty() || t.base == spec.base))
            break;
    }
    if (ti == ds->rope.size()) {
        RopeTable t;
        t.base = spec.base;
        t.freq = spec.freq;
        t.rot = spec.rot;
        ds->rope.push_back(std::move(t));
    }
    RopeTable &rt = ds->rope[ti];
    {
        // rows this call needs beyond the pinned ones it can share
        std::unordered_map<int32_t, int32_t> distinct;
        for (int32_t i = 0; i < n; ++i)
            if (offsets[i] != 0)
                distinct.emplace(offsets[i], 0);
        if ((int32_t)distinct.size() > kRopeRowsCap)
            return KDN_ESIZE;
        int32_t fresh = 0;
        for (const auto &kv : distinct) {
            auto it = rt.row_of.find(kv.first);
            if (it == rt.row_of.end() || !rt.pinned[(size_t)it->second])
                ++fresh;
        }
        if (fresh > kRopeRowsCap - rt.n_pinned)
            return KDN_EFULL;
    }
    const int32_t half = spec.rot / 2;
    if (!rt.dev) {
        if (hipMalloc(reinterpret_cast<void **>(&rt.dev), (size_t)kRopeRowsCap * half * sizeof(f32x2)) != hipSuccess)
            return KDN_EDEVICE;
        rt.pinned.assign((size_t)kRopeRowsCap, 0);
        rt.free_rows.resize((size_t)kRopeRowsCap);
        for (int32_t r = 0; r < kRopeRowsCap; ++r)
            rt.free_rows[(size_t)r] = kRopeRowsCap - 1 - r; // handed out from row 0 up
    }
    std::vector<float> row((size_t)half * 2);
    for (int32_t i = 0; i < n; ++i) {
        const int32_t d = offsets[i];
        if (d == 0) {
            rows[i] = -1;
            continue;
        }
        auto it = rt.row_of.find(d);
        if (it != rt.row_of.end()) {
            rows[i] = it->second;
            if (pin && !rt.pinned[(size_t)it->second]) {
                rt.pinned[(size_t)it->second] = 1;
                ++rt.n_pinned;
            }
            continue;
        }
        if (rt.free_rows.empty()) {
            // table full: wait until nothing can still read it, then drop the transient rows
            if (hipDeviceSynchronize() != hipSuccess)
                return KDN_EDEVICE;
            for (auto e = rt.row_of.begin(); e != rt.row_of.end();) {
                if (rt.pinned[(size_t)e->second]) {
                    ++e;
                } else {
                    rt.free_rows.push_back(e->second);
                    e = rt.row_of.erase(e);
                }
            }
            for (int32_t k = 0; k < i; ++k) // transient rows handed out earlier in this call are gone
                if (offsets[k] != 0 && rt.row_of.find(offsets[k]) == rt.row_of.end())
                    rows[k] = -2;
            if (rt.free_rows.empty())
                return KDN_EFULL;
        }
        for (int32_t j = 0; j < half; ++j) {
            const double theta = spec.freq.empty() ? std::pow(spec.base, -(double)(2 * j) / (double)spec.rot)
                                                   : spec.freq[(size_t)j];
            const double phi = (double)d * theta;
            row[2 * j] = (float)std::cos(phi);
            row[2 * j + 1] = (float)std::sin(phi);
        }
        const int32_t r = rt.free_rows.back();
        if (hipMemcpy(rt.dev + (size_t)r * half, row.data(), row.size() * sizeof(float),
                      hipMemcpyHostToDevice)
            != hipSuccess)
            return KDN_EDEVICE;
        rt.free_rows.pop_back();
        rt.row_of.emplace(d, r);
        if (pin) {
            rt.pinned[(size_t)r] = 1;
            ++rt.n_pinned;
        }
        rows[i] = r;
    }
    for (int32_t i = 0; i < n; ++i)
        if (rows[i] == -2) // only after the transient rows were dropped inside this call
            return rope_rows(ds, spec, offsets, n, rows, table, pin);
    *table = rt.dev;
    return KDN_OK;
}

// Threads of a workgroup: whole wavefronts, enough for every thread to hold `per_thread`
// items of a full tile in flight, at most kThreads.  Small tiles (few or short heads) thus
// run as more, narrower workgroups instead of leaving lanes without work.
inline unsigned block_threads(int64_t items, int per_thread)
{
    int64_t t = (items + per_thread - 1) / per_thread;
    t = (t + 63) / 64 * 64;
    return (unsigned)std::min<int64_t>(std::max<int64_t>(t, 64), kThreads);
}

template <int DT, int FMT, int P>
void launch_store(const StoreP &p, dim3 grid, hipStream_t st)
{
    const dim3 block(block_threads((int64_t)p.c.G * p.c.H * P, 2)); // 2 rather than kStoreU items each: measured
    if (p.c.dense && !p.tokens)
        hipLaunchKernelGGL((k_store<DT, FMT, P, true>), grid, block, 0, st, p);
    else
        hipLaunchKernelGGL((k_store<DT, FMT, P, false>), grid, block, 0, st, p);
}

template <int FMT>
void launch_store_d(const StoreP &p, dim3 grid, hipStream_t st)
{
    switch (p.c.D) {
    case 64: launch_store<64, FMT, 8>(p, grid, st); return;
    case 128: launch_store<128, FMT, 16>(p, grid, st); return;
    default: break;
    }
    switch (log2_ceil(p.c.D >> 3)) { // lane group: D/8 lanes rounded up to a power of two
    case 1: launch_store<0, FMT, 2>(p, grid, st); break;
    case 2: launch_store<0, FMT, 4>(p, grid, st); break;
    case 3: launch_store<0, FMT, 8>(p, grid, st); break;
    case 4: launch_store<0, FMT, 16>(p, grid, st); break;
    case 5: launch_store<0, FMT, 32>(p, grid, st); break;
    default: launch_store<0, FMT, 64>(p, grid, st); break;
    }
}

template <int DT, int FMT, bool DENSE, bool VAR, bool REUSE>
void launch_place_v(const PlaceP &p, const Seg *segs, int32_t n, const Seg *segs_dev, dim3 grid,
                    hipStream_t st)
{
    const int lanes_per_row = 1 << log2_ceil(p.c.D >> 4);
    const dim3 block(block_threads((int64_t)p.c.G * p.c.H * lanes_per_row, FMT == KDN_FMT_RAW_BF16 ? 2 : 4));
    if (segs_dev) {
        SegsDevice sd{segs_dev};
        hipLaunchKernelGGL((k_place<DT, FMT, DENSE, VAR, REUSE, SegsDevice>), grid, block, 0, st, p, sd);
    } else {
        SegsInline si;
        std::memset(&si, 0, sizeof si);
        std::memcpy(si.s, segs, (size_t)n * sizeof(Seg));
        hipLaunchKernelGGL((k_place<DT, FMT, DENSE, VAR, REUSE, SegsInline>), grid, block, 0, st, p, si);
    }
}

template <int DT, int FMT>
void launch_place(const PlaceP &p, const Seg *segs, int32_t n, const Seg *segs_dev, dim3 grid,
                  hipStream_t st)
{
    const bool var = p.rot != p.c.D || p.pairing != KDN_ROPE_HALF_SPLIT;
    // the cache-friendly load flavour exists for the common serving case only (dense
    // layout, default RoPE variant); elsewhere shared rows are streamed like any other
    if (p.c.dense) {
        if (var)
            launch_place_v<DT, FMT, true, true, false>(p, segs, n, segs_dev, grid, st);
        else if (p.reuse)
            launch_place_v<DT, FMT, true, false, true>(p, segs, n, segs_dev, grid, st);
        else
            launch_place_v<DT, FMT, true, false, false>(p, segs, n, segs_dev, grid, st);
    } else {
        if (var)
            launch_place_v<DT, FMT, false, true, false>(p, segs, n, segs_dev, grid, st);
        else
            launch_place_v<DT, FMT, false, false, false>(p, segs, n, segs_dev, grid, st);
    }
}

// the row-contiguous kernel; the RoPE variant is a run-time matter there
template <int DT, int FMT>
void launch_place_c(const PlaceP &p, const Seg *segs, int32_t n, const Seg *segs_dev, dim3 grid,
                    hipStream_t st)
{
    const int flavour = !p.c.dense ? 0 : p.reuse ? 2 : 1;
    // a wavefront takes 64/(D/8) rows per pass and keeps 8 (raw: 4) passes in flight; a tile of
    // at most 4 passes (one head of 128, two of 64: a block's rows are 4 KiB, one wavefront's
    // work) goes to the flavour that keeps 4: 68 registers instead of 87, 7 wavefronts per SIMD
    // instead of 5, and such tiles are bound by how many of them are in flight (one head of 128:
    // compose 4.7 -> 4.9-5.1 TB/s, load 4.6 -> 5.4; at 8 passes, two heads of 128, it loses)
    const int64_t passes = ((int64_t)p.c.G * p.c.H + 64 / (p.c.D >> 3) - 1) / (64 / (p.c.D >> 3));
    const bool few = FMT != KDN_FMT_RAW_BF16 && passes <= kFewPasses;
    const dim3 block(block_threads(passes * 64, FMT == KDN_FMT_RAW_BF16 || few ? 4 : 8));
    SegsDevice sd{segs_dev};
    SegsInline si;
    if (!segs_dev) {
        std::memset(&si, 0, sizeof si);
        std::memcpy(si.s, segs, (size_t)n * sizeof(Seg));
    }
#define KDN_PLACE_C(DENSE, REUSE, UQ)                                                                           \
    do {                                                                                                        \
        if (segs_dev)                                                                                           \
            hipLaunchKernelGGL((k_place_c<DT, FMT, DENSE, REUSE, UQ, SegsDevice>), grid, block, 0, st, p, sd);  \
        else                                                                                                    \
            hipLaunchKernelGGL((k_place_c<DT, FMT, DENSE, REUSE, UQ, SegsInline>), grid, block, 0, st, p, si);  \
    } while (0)
    if (few) {
        if (flavour == 0)
            KDN_PLACE_C(false, false, 4);
        else if (flavour == 1)
            KDN_PLACE_C(true, false, 4);
        else
            KDN_PLACE_C(true, true, 4);
    } else {
        if (flavour == 0)
            KDN_PLACE_C(false, false, 8);
        else if (flavour == 1)
            KDN_PLACE_C(true, false, 8);
        else
            KDN_PLACE_C(true, true, 8);
    }
#undef KDN_PLACE_C
}

// Which place kernel serves a head_dim, by measurement on pools that span the device memory
// (4096 tokens, 32 layers, TB/s of algorithmic bytes, k_place / k_place_c): the row-contiguous
// kernel wins at head_dim 128 for the quantised forms (int8 5.75 / 6.0-6.3, int4 5.6 / 6.1),
// ties for raw bf16 (6.35), and loses where every row looks its own block up (blocks of one to
// three tokens: 5.65 / 4.8); at 256 and 512 the pair-owning kernel is ahead for int8
// (6.13 / 6.03, 5.87 / 5.70).  Head dims that are not a multiple of 128 always take k_place_c
// (there a pair-owning lane would write runs that are not whole 128-byte lines).
template <int FMT>
void launch_place_d(const PlaceP &p, const Seg *segs, int32_t n, const Seg *segs_dev, dim3 grid,
                    hipStream_t st)
{
    if (p.c.D == 128 && !p.c.per_token && FMT != KDN_FMT_RAW_BF16)
        launch_place_c<128, FMT>(p, segs, n, segs_dev, grid, st);
    else if (p.c.D == 128)
        launch_place<128, FMT>(p, segs, n, segs_dev, grid, st);
    else if (p.c.D % 128 == 0)
        launch_place<0, FMT>(p, segs, n, segs_dev, grid, st);
    else if (p.c.D == 64)
        launch_place_c<64, FMT>(p, segs, n, segs_dev, grid, st);
    else
        launch_place_c<0, FMT>(p, segs, n, segs_dev, grid, st);
}

// Enqueue the placement of `segs` (all of one format).  Up to kMaxInlineSegs travel
// in the kernel arguments; more go through a ring of device tables.
// max_workgroups > 0 caps the launch; the workgroups then stride over the tiles.
// resident: the same records already in device memory (the caller put them there on `st`);
// the kernel then reads them from there and nothing is copied or allocated here.
// heads: the first `heads` records get workgroups of their own (a row of the grid each); the
// others are reached through the `next` links of the records before them (0 = all of them).
inline kdn_status place_segments(DeviceState *ds, const PlaceP &p_in, int32_t fmt, const std::vector<Seg> &segs,
                                 hipStream_t st, int32_t max_workgroups = 0, const Seg *resident = nullptr,
                                 size_t heads = 0)
{
    if (segs.empty())
        return KDN_OK;
    if (heads == 0)
        heads = segs.size();
    if (heads > 65535 || heads > segs.size() || segs.size() * sizeof(Seg) > kSegSlotBytes)
        return KDN_ESIZE;
    for (size_t i = 0; i < segs.size(); ++i) // a chain only ever moves forward, into the records without a row of their own
        if (segs[i].next != 0 && ((size_t)segs[i].next <= i || (size_t)segs[i].next < heads || (size_t)segs[i].next >= segs.size()))
            return KDN_EINVAL;
    int64_t max_groups = 0;
    for (const Seg &s : segs)
        max_groups = std::max(max_groups, groups_spanned(s.S, s.T, p_in.c.G));
    if (max_groups * 2 * p_in.c.L > 0x7fffffff / kThreads)
        return KDN_ESIZE;
    PlaceP p = p_in;
    p.tiles_x = (uint32_t)(max_groups * 2 * p.c.L);
    uint32_t gx = p.tiles_x;
    if (max_workgroups > 0)
        gx = std::min<uint32_t>(gx, std::max<uint32_t>(1u, (uint32_t)max_workgroups / (uint32_t)heads));
    dim3 grid(gx, (unsigned)heads, 1);

    const Seg *segs_dev = resident;
    int slot = -1;
    if (!resident && (int)segs.size() > kMaxInlineSegs) {
        if (!ds->seg_dev) {
            if (hipMalloc(reinterpret_cast<void **>(&ds->seg_dev), kSegSlots * kSegSlotBytes) != hipSuccess)
                return KDN_EDEVICE;
            if (hipHostMalloc(reinterpret_cast<void **>(&ds->seg_host), kSegSlots * kSegSlotBytes,
                              hipHostMallocDefault)
                != hipSuccess)
                return KDN_EDEVICE;
            for (int i = 0; i < kSegSlots; ++i)
                if (hipEventCreateWithFlags(&ds->seg_done[i], hipEventDisableTiming) != hipSuccess)
                    return KDN_EDEVICE;
        }
        slot = ds->next_slot;
        ds->next_slot = (slot + 1) % kSegSlots;
        if (ds->seg_used[slot] && hipEventSynchronize(ds->seg_done[slot]) != hipSuccess)
            return KDN_EDEVICE;
        uint8_t *h = ds->seg_host + (size_t)slot * kSegSlotBytes;
        uint8_t *d = ds->seg_dev + (size_t)slot * kSegSlotBytes;
        std::memcpy(h, segs.data(), segs.size() * sizeof(Seg));
        if (hipMemcpyAsync(d, h, segs.size() * sizeof(Seg), hipMemcpyHostToDevice, st) != hipSuccess)
            return KDN_EDEVICE;
        segs_dev = reinterpret_cast<const Seg *>(d);
    }
    if (fmt == KDN_FMT_RAW_BF16)
        launch_place_d<KDN_FMT_RAW_BF16>(p, segs.data(), (int32_t)segs.size(), segs_dev, grid, st);
    else if (fmt == KDN_FMT_INT8_ROWSCALE)
        launch_place_d<KDN_FMT_INT8_ROWSCALE>(p, segs.data(), (int32_t)segs.size(), segs_dev, grid, st);
    else if (fmt == KDN_FMT_FP8_ROWSCALE)
        launch_place_d<KDN_FMT_FP8_ROWSCALE>(p, segs.data(), (int32_t)segs.size(), segs_dev, grid, st);
    else
        launch_place_d<KDN_FMT_INT4_GROUP32>(p, segs.data(), (int32_t)segs.size(), segs_dev, grid, st);
    kdn_status rc = hip_status(hipGetLastError());
    if (slot >= 0) {
        if (hipEventRecord(ds->seg_done[slot], st) != hipSuccess)
            return KDN_EDEVICE;
        ds->seg_used[slot] = true;
    }
    return rc;
}

// The bookkeeping of a (batched) compose, host only: every chunk view becomes one segment
// placed at the running sum of the token counts before it in its request; segments are
// grouped by stored form (one launch each).  `request`, `chunk` and `offset` say where a
// segment came from; its cos/sin row is filled in later.
struct PlannedSeg {
    Seg seg;
    int32_t request, chunk, offset;
    int32_t follows; // record of the same launch whose workgroups place this view as well, -1: its own
};
struct ComposePlan {
    std::vector<PlannedSeg> segs[kFormats];
    int32_t reuse[kFormats] = {};
    size_t heads[kFormats] = {}; // records with workgroups of their own: the first heads[f] of segs[f]
};

// Views of exactly the same stored rows whose tiles cut them the same way (same rows of the
// same buffer, destinations congruent modulo the token group) are chained: the first keeps
// its workgroups, the others follow it through Seg::next and are moved behind all records
// that have workgroups.  Order is otherwise kept.  Returns the number of records with
// workgroups.
inline size_t chain_views(std::vector<PlannedSeg> &v, int32_t G)
{
    using Key = std::tuple<const uint8_t *, int32_t, int32_t, int32_t, int32_t>;
    std::map<Key, size_t> last; // key -> position in `v` of the latest view with that key
    std::vector<size_t> before(v.size(), SIZE_MAX);
    std::vector<size_t> order, tail;
    for (size_t i = 0; i < v.size(); ++i) {
        const Seg &s = v[i].seg;
        const Key key{s.data, s.Tp, s.tok0, s.T, s.S % G};
        auto it = last.find(key);
        if (it == last.end()) {
            order.push_back(i);
            last.emplace(key, i);
        } else {
            before[i] = it->second;
            it->second = i;
            tail.push_back(i);
        }
    }
    const size_t heads = order.size();
    order.insert(order.end(), tail.begin(), tail.end());
    std::vector<size_t> where(v.size());
    for (size_t k = 0; k < order.size(); ++k)
        where[order[k]] = k;
    std::vector<PlannedSeg> out(v.size());
    for (size_t k = 0; k < order.size(); ++k) {
        out[k] = v[order[k]];
        out[k].seg.next = 0;
        out[k].follows = -1;
    }
    for (size_t i = 0; i < v.size(); ++i)
        if (before[i] != SIZE_MAX) {
            out[where[before[i]]].seg.next = (int32_t)where[i];
            out[where[i]].follows = (int32_t)where[before[i]];
        }
    v.swap(out);
    return heads;
}

inline kdn_status plan_compose(const kdn_request *reqs, int32_t n_reqs, const kdn_cache_desc *cache,
                               ComposePlan &plan)
{
    if (!reqs || n_reqs <= 0)
        return KDN_EINVAL;
    kdn_status st = check_cache(cache);
    if (st != KDN_OK)
        return st;
    for (int32_t r = 0; r < n_reqs; ++r) {
        const kdn_request &q = reqs[r];
        if (!q.chunks || !q.offsets || q.n_chunks <= 0 || !q.block_table_dev || q.table_len <= 0
            || q.dest_token_start < 0)
            return KDN_EINVAL;
        int64_t total = q.dest_token_start;
        for (int32_t i = 0; i < q.n_chunks; ++i) {
            st = check_chunk(&q.chunks[i], cache);
            if (st != KDN_OK)
                return st;
            total += q.chunks[i].num_tokens;
        }
        if (total > (int64_t)q.table_len * cache->block_size || total > 0x7fffffff)
            return KDN_ERANGE; // token indices are 32-bit in the kernels
    }
    for (int32_t r = 0; r < n_reqs; ++r) {
        const kdn_request &q = reqs[r];
        int32_t S = q.dest_token_start;
        for (int32_t i = 0; i < q.n_chunks; ++i) {
            const kdn_chunk &ch = q.chunks[i];
            PlannedSeg ps;
            ps.seg.data = static_cast<const uint8_t *>(ch.data);
            ps.seg.bt = q.block_table_dev;
            ps.seg.Tp = ch.parent_tokens;
            ps.seg.tok0 = ch.token_start;
            ps.seg.T = ch.num_tokens;
            ps.seg.S = S;
            ps.seg.rope_row = 0;
            ps.seg.next = 0;
            ps.follows = -1;
            ps.request = r;
            ps.chunk = i;
            ps.offset = q.offsets[i];
            plan.segs[ch.fmt].push_back(ps);
            S += ch.num_tokens;
        }
    }
    const int32_t G = make_cache_p(cache).G;
    for (int f = 0; f < kFormats; ++f) {
        // Segments that read the same stored rows run back to back, so that a popular
        // chunk is fetched from HBM once and from the last-level cache afterwards; views
        // that are the very same rows are chained onto one set of workgroups.
        plan.reuse[f] = 0;
        std::vector<PlannedSeg> &v = plan.segs[f];
        plan.heads[f] = v.size();
        if (n_reqs <= 1) { // one request: its order is kept; a view it holds twice is still read once
            plan.heads[f] = chain_views(v, G);
            plan.reuse[f] = plan.heads[f] < v.size();
            continue;
        }
        std::stable_sort(v.begin(), v.end(), [](const PlannedSeg &a, const PlannedSeg &b) {
            return a.seg.data != b.seg.data ? a.seg.data < b.seg.data : a.seg.tok0 < b.seg.tok0;
        });
        // sorted by first row, so a view overlaps an earlier one exactly when it starts
        // before the furthest end seen so far in its buffer
        int64_t reach = 0;
        for (size_t i = 0; i < v.size(); ++i) {
            if (i == 0 || v[i].seg.data != v[i - 1].seg.data)
                reach = 0;
            else if (v[i].seg.tok0 < reach)
                plan.reuse[f] = 1;
            reach = std::max<int64_t>(reach, (int64_t)v[i].seg.tok0 + v[i].seg.T);
        }
        plan.heads[f] = chain_views(v, G);
        if (plan.heads[f] < v.size())
            plan.reuse[f] = 1;
    }
    return KDN_OK;
}

inline kdn_status compose_impl(const kdn_request *reqs, int32_t n_reqs, const kdn_cache_desc *cache,
                               double rope_base, const kdn_rope_spec *variant, void *stream,
                               int32_t max_workgroups = 0)
{
    ComposePlan plan;
    kdn_status st = plan_compose(reqs, n_reqs, cache, plan);
    if (st != KDN_OK)
        return st;
    RopeSpec spec;
    st = resolve_spec(variant, rope_base, cache->head_dim, spec);
    if (st != KDN_OK)
        return st;
    std::vector<int32_t> offs;
    for (int f = 0; f < kFormats; ++f)
        for (const PlannedSeg &ps : plan.segs[f])
            offs.push_back(ps.offset);
    std::lock_guard<std::mutex> lock(g_mu);
    DeviceState *ds = device_state(nullptr);
    if (!ds)
        return KDN_EDEVICE;
    PlaceP p;
    p.c = make_cache_p(cache);
    p.layer0 = 0;
    p.rot = spec.rot;
    p.pairing = spec.pairing;
    std::vector<int32_t> rows(offs.size());
    st = rope_rows(ds, spec, offs.data(), (int32_t)offs.size(), rows.data(), &p.rope);
    if (st != KDN_OK)
        return st;
    size_t k = 0;
    for (int f = 0; f < kFormats; ++f) {
        std::vector<Seg> segs;
        segs.reserve(plan.segs[f].size());
        for (const PlannedSeg &ps : plan.segs[f]) {
            segs.push_back(ps.seg);
            segs.back().rope_row = rows[k++];
        }
        p.reuse = plan.reuse[f];
        st = place_segments(ds, p, f, segs, static_cast<hipStream_t>(stream), max_workgroups, nullptr, plan.heads[f]);
        if (st != KDN_OK)
            return st;
    }
    return KDN_OK;
}

// bytes of one stored row's codes, and of its scales, per format
inline uint64_t row_code_bytes(int32_t fmt, int32_t D)
{
    return fmt == KDN_FMT_RAW_BF16 ? (uint64_t)D * 2 : fmt == KDN_FMT_INT4_GROUP32 ? (uint64_t)D / 2 : (uint64_t)D;
}
inline uint64_t row_scale_bytes(int32_t fmt, int32_t D)
{
    return fmt == KDN_FMT_RAW_BF16 ? 0 : fmt == KDN_FMT_INT4_GROUP32 ? (uint64_t)(D / 32) * 4 : 4;
}

// Views of the same host buffer are staged once: the token range [lo, hi) that the
// views of one buffer span crosses the link as one copy per stage.
struct HostParent {
    const uint8_t *data;
    uint64_t bytes; // size of the host buffer
    int32_t fmt, L, H, D, Tp, lo, hi;
};

inline void plan_host_parents(const kdn_chunk *chunks, int32_t n, std::vector<HostParent> &parents,
                              std::vector<int32_t> &parent_of)
{
    parents.clear();
    parent_of.assign((size_t)n, 0);
    for (int32_t i = 0; i < n; ++i) {
        const kdn_chunk &ch = chunks[i];
        size_t k = 0;
        for (; k < parents.size(); ++k)
            if (parents[k].data == ch.data && parents[k].fmt == ch.fmt && parents[k].Tp == ch.parent_tokens)
                break;
        if (k == parents.size())
            parents.push_back({static_cast<const uint8_t *>(ch.data), ch.bytes, ch.fmt, ch.num_layers,
                               ch.num_kv_heads, ch.head_dim, ch.parent_tokens, ch.token_start,
                               ch.token_start + ch.num_tokens});
        parents[k].bytes = std::min<uint64_t>(parents[k].bytes, ch.bytes);
        parents[k].lo = std::min(parents[k].lo, ch.token_start);
        parents[k].hi = std::max(parents[k].hi, ch.token_start + ch.num_tokens);
        parent_of[(size_t)i] = (int32_t)k;
    }
}

// The copies of one stage (cache layers [l0, l0+Lg)) of a compose from host memory.  Per host
// buffer: 2*Lg planes of Tu*H rows, Tp*H rows apart, once for the codes and (if the form has
// any) once for the scales, packed back to back; the staged image is a chunk of Lg layers and
// Tu tokens.  `staged_at[k]` is where buffer k's image starts within the staging half.  Every
// copy is checked to stay inside its host buffer and inside `half_bytes` of staging.
struct StageCopy {
    int32_t parent;
    uint64_t rows, src_off, src_pitch, width, dst_off;
};

inline kdn_status plan_stage_copies(const std::vector<HostParent> &parents, int32_t l0, int32_t Lg,
                                    uint64_t half_bytes, std::vector<StageCopy> &copies,
                                    std::vector<uint64_t> &staged_at)
{
    copies.clear();
    staged_at.assign(parents.size(), 0);
    uint64_t at = 0;
    for (size_t k = 0; k < parents.size(); ++k) {
        const HostParent &hp = parents[k];
        if (l0 < 0 || Lg <= 0 || l0 + Lg > hp.L || hp.lo < 0 || hp.hi <= hp.lo || hp.hi > hp.Tp)
            return KDN_ERANGE;
        const uint64_t Tu = (uint64_t)(hp.hi - hp.lo), Tp = (uint64_t)hp.Tp, H = (uint64_t)hp.H;
        const uint64_t cb = row_code_bytes(hp.fmt, hp.D), sb = row_scale_bytes(hp.fmt, hp.D);
        const uint64_t planes = (uint64_t)2 * Lg;
        const uint64_t first_row = (uint64_t)l0 * 2 * Tp + (uint64_t)hp.lo; // in units of H rows
        staged_at[k] = at;
        StageCopy c = {(int32_t)k, planes, first_row * H * cb, Tp * H * cb, Tu * H * cb, at};
        StageCopy s = {(int32_t)k, planes, (uint64_t)hp.L * 2 * Tp * H * cb + first_row * H * sb, Tp * H * sb,
                       Tu * H * sb, at + planes * c.width};
        if (s.dst_off + planes * s.width > half_bytes
            || c.src_off + (planes - 1) * c.src_pitch + c.width > hp.bytes
            || (sb && s.src_off + (planes - 1) * s.src_pitch + s.width > hp.bytes))
            return KDN_ESIZE;
        copies.push_back(c);
        if (sb)
            copies.push_back(s);
        at += (planes * (c.width + s.width) + 255) & ~(uint64_t)255;
    }
    return KDN_OK;
}

} // namespace kdn_impl
#endif // KDN_PLANNER_H
