// C ABI of the KDN library (include/kdn.h) for MI355X (gfx950).  The kernels live in
// kdn_kernels.h, the host planner in kdn_planner.h; this file validates arguments,
// builds launch parameters and calls them.
#include <new>

#include "kdn_planner.h"

using namespace kdn_impl;

// Scratch of kdn_compose_batch_static: cos/sin rows, then segment records.  Every device the
// library runs on holds its own copy of this array until the process ends; in host code the
// name is only a handle for hipGetSymbolAddress, never a device address.
constexpr int kStaticMaxSegs = 4096;   // chunk views per call
constexpr int kStaticMaxRopeRows = 64; // distinct non-zero offsets per call
constexpr size_t kStaticRopeBytes = (size_t)kStaticMaxRopeRows * (kMaxHeadDim / 2) * sizeof(f32x2);
constexpr size_t kStaticSegBytes = (size_t)kStaticMaxSegs * sizeof(Seg);
static __device__ __align__(256) unsigned char g_static_scratch[kStaticRopeBytes + kStaticSegBytes];
static_assert(kStaticRopeBytes % 256 == 0 && sizeof(Seg) % 4 == 0, "scratch layout");

// ---------------------------------------------------------------------------------
// C ABI

extern "C" {

uint64_t kdn_chunk_bytes(int32_t L, int32_t H, int32_t D, int32_t T, int32_t fmt)
{
    if (L <= 0 || H <= 0 || D <= 0 || T <= 0)
        return 0;
    const uint64_t rows = (uint64_t)L * 2 * (uint64_t)T * (uint64_t)H;
    if (fmt == KDN_FMT_RAW_BF16)
        return rows * (uint64_t)D * 2;
    if (fmt == KDN_FMT_INT8_ROWSCALE || fmt == KDN_FMT_FP8_ROWSCALE)
        return rows * ((uint64_t)D + 4);
    if (fmt == KDN_FMT_INT4_GROUP32 && D % 32 == 0)
        return rows * ((uint64_t)D / 2 + (uint64_t)D / 32 * 4);
    return 0;
}

kdn_status kdn_chunk_init(kdn_chunk *out, void *data_dev, uint64_t bytes, int32_t fmt, int32_t L,
                          int32_t H, int32_t D, int32_t T)
{
    if (!out || !data_dev || T <= 0)
        return KDN_EINVAL;
    if (!known_format(fmt))
        return KDN_EINVAL;
    kdn_status st = check_shape(L, H, D);
    if (st != KDN_OK)
        return st;
    if (fmt == KDN_FMT_INT4_GROUP32 && D % 32 != 0)
        return KDN_EUNSUPPORTED;
    if (!aligned16(data_dev))
        return KDN_EALIGN;
    if (bytes < kdn_chunk_bytes(L, H, D, T, fmt))
        return KDN_ESIZE;
    out->data = data_dev;
    out->bytes = bytes;
    out->fmt = fmt;
    out->num_layers = L;
    out->num_kv_heads = H;
    out->head_dim = D;
    out->parent_tokens = T;
    out->token_start = 0;
    out->num_tokens = T;
    return KDN_OK;
}

kdn_status kdn_chunk_slice(const kdn_chunk *chunk, int32_t token_start, int32_t num_tokens,
                           kdn_chunk *out)
{
    if (!chunk || !out || num_tokens <= 0 || token_start < 0)
        return KDN_EINVAL;
    if ((int64_t)token_start + num_tokens > chunk->num_tokens)
        return KDN_ERANGE;
    kdn_chunk v = *chunk;
    v.token_start = chunk->token_start + token_start;
    v.num_tokens = num_tokens;
    *out = v;
    return KDN_OK;
}

// Validates a store request (shared by the device and host destinations).
static kdn_status store_check(const kdn_cache_desc *cache, const int32_t *block_table_dev,
                              int32_t table_len, int32_t token_start, int32_t num_tokens,
                              const int32_t *tokens_dev, const kdn_chunk *out)
{
    kdn_status st = check_cache(cache);
    if (st != KDN_OK)
        return st;
    if (!block_table_dev || !out || !out->data || table_len <= 0 || num_tokens <= 0 || token_start < 0)
        return KDN_EINVAL;
    if (!known_format(out->fmt))
        return KDN_EINVAL;
    if (out->fmt == KDN_FMT_INT4_GROUP32 && cache->head_dim % 32 != 0)
        return KDN_EUNSUPPORTED;
    if (!aligned16(out->data))
        return KDN_EALIGN;
    const int64_t limit = (int64_t)table_len * cache->block_size;
    if (!tokens_dev && ((int64_t)token_start + num_tokens > limit || (int64_t)token_start + num_tokens > 0x7fffffff))
        return KDN_ERANGE; // token indices are 32-bit in the kernels
    const uint64_t need = kdn_chunk_bytes(cache->num_layers, cache->num_kv_heads, cache->head_dim,
                                          num_tokens, out->fmt);
    if (out->bytes < need)
        return KDN_ESIZE;
    return KDN_OK;
}

// Enqueues the store of layers [layer0, layer0 + n_layers) into `dst`, laid out as a chunk
// of n_layers layers.
static kdn_status store_launch(const kdn_cache_desc *cache, const int32_t *block_table_dev,
                               int32_t table_len, int32_t token_start, int32_t num_tokens,
                               const int32_t *tokens_dev, int32_t fmt, void *dst, int32_t layer0,
                               int32_t n_layers, hipStream_t hs, int32_t max_workgroups = 0)
{
    StoreP p;
    p.c = make_cache_p(cache);
    p.c.L = n_layers;
    p.layer0 = layer0;
    p.bt = block_table_dev;
    p.out = static_cast<uint8_t *>(dst);
    p.t0 = token_start;
    p.T = num_tokens;
    p.tokens = tokens_dev;
    p.limit = (int32_t)std::min<int64_t>((int64_t)table_len * cache->block_size, 0x7fffffff);
    if (tokens_dev)
        p.c.G = std::max(p.c.G, 16); // list entries need no block alignment
    const int64_t groups = groups_spanned(token_start, num_tokens, p.c.G);
    if (groups * 2 * p.c.L > 0x7fffffff / kThreads)
        return KDN_ESIZE;
    p.tiles_x = (uint32_t)(groups * 2 * p.c.L);
    dim3 grid(max_workgroups > 0 ? std::min<uint32_t>(p.tiles_x, (uint32_t)max_workgroups) : p.tiles_x, 1, 1);
    if (fmt == KDN_FMT_RAW_BF16)
        launch_store_d<KDN_FMT_RAW_BF16>(p, grid, hs);
    else if (fmt == KDN_FMT_INT8_ROWSCALE)
        launch_store_d<KDN_FMT_INT8_ROWSCALE>(p, grid, hs);
    else if (fmt == KDN_FMT_FP8_ROWSCALE)
        launch_store_d<KDN_FMT_FP8_ROWSCALE>(p, grid, hs);
    else
        launch_store_d<KDN_FMT_INT4_GROUP32>(p, grid, hs);
    return hip_status(hipGetLastError());
}

static void describe_stored(const kdn_cache_desc *cache, int32_t num_tokens, kdn_chunk *out)
{
    out->num_layers = cache->num_layers;
    out->num_kv_heads = cache->num_kv_heads;
    out->head_dim = cache->head_dim;
    out->parent_tokens = num_tokens;
    out->token_start = 0;
    out->num_tokens = num_tokens;
}

static kdn_status store_impl(const kdn_cache_desc *cache, const int32_t *block_table_dev,
                             int32_t table_len, int32_t token_start, int32_t num_tokens,
                             const int32_t *tokens_dev, kdn_chunk *out, void *stream, int32_t max_workgroups = 0)
{
    kdn_status st = store_check(cache, block_table_dev, table_len, token_start, num_tokens, tokens_dev, out);
    if (st != KDN_OK)
        return st;
    st = store_launch(cache, block_table_dev, table_len, token_start, num_tokens, tokens_dev, out->fmt,
                      out->data, 0, cache->num_layers, static_cast<hipStream_t>(stream), max_workgroups);
    if (st != KDN_OK)
        return st;
    describe_stored(cache, num_tokens, out);
    return KDN_OK;
}

kdn_status kdn_store_chunk(const kdn_cache_desc *cache, const int32_t *block_table_dev,
                           int32_t table_len, int32_t token_start, int32_t num_tokens,
                           kdn_chunk *out, void *stream)
{
    return store_impl(cache, block_table_dev, table_len, token_start, num_tokens, nullptr, out, stream);
}

kdn_status kdn_store_tokens(const kdn_cache_desc *cache, const int32_t *block_table_dev,
                            int32_t table_len, const int32_t *tokens_dev, int32_t num_tokens,
                            kdn_chunk *out, void *stream)
{
    if (!tokens_dev)
        return KDN_EINVAL;
    return store_impl(cache, block_table_dev, table_len, 0, num_tokens, tokens_dev, out, stream);
}

kdn_status kdn_store_chunk_opts(const kdn_cache_desc *cache, const int32_t *block_table_dev,
                                int32_t table_len, int32_t token_start, int32_t num_tokens,
                                kdn_chunk *out, const kdn_launch_opts *opts, void *stream)
{
    if (opts && opts->max_workgroups < 0)
        return KDN_EINVAL;
    return store_impl(cache, block_table_dev, table_len, token_start, num_tokens, nullptr, out, stream,
                      opts ? opts->max_workgroups : 0);
}

uint64_t kdn_store_staging_bytes(const kdn_cache_desc *cache, int32_t num_tokens, int32_t fmt,
                                 int32_t layers_per_stage)
{
    if (!cache || layers_per_stage <= 0)
        return 0;
    const uint64_t b = kdn_chunk_bytes(std::min(layers_per_stage, cache->num_layers), cache->num_kv_heads,
                                       cache->head_dim, num_tokens, fmt);
    return b ? 2 * ((b + 255) & ~(uint64_t)255) : 0;
}

kdn_status kdn_store_to_host(const kdn_cache_desc *cache, const int32_t *block_table_dev,
                             int32_t table_len, int32_t token_start, int32_t num_tokens,
                             kdn_chunk *out_host, void *staging_dev, uint64_t staging_bytes,
                             int32_t layers_per_stage, void *stream)
{
    kdn_status st = store_check(cache, block_table_dev, table_len, token_start, num_tokens, nullptr, out_host);
    if (st != KDN_OK)
        return st;
    if (!staging_dev || layers_per_stage <= 0)
        return KDN_EINVAL;
    if (!aligned16(staging_dev))
        return KDN_EALIGN;
    hipPointerAttribute_t attr;
    if (hipPointerGetAttributes(&attr, out_host->data) != hipSuccess) {
        (void)hipGetLastError();
        return KDN_EINVAL; // ordinary pageable memory
    }
    if (attr.type != hipMemoryTypeHost)
        return KDN_EINVAL;
    const uint64_t need = kdn_store_staging_bytes(cache, num_tokens, out_host->fmt, layers_per_stage);
    if (need == 0 || staging_bytes < need)
        return KDN_ESIZE;

    std::lock_guard<std::mutex> lock(g_mu);
    DeviceState *ds = device_state(nullptr);
    if (!ds)
        return KDN_EDEVICE;
    LinkDir &ln = ds->to_host;
    st = ensure_link(ln);
    if (st != KDN_OK)
        return st;
    hipStream_t user = static_cast<hipStream_t>(stream);
    const int32_t L = cache->num_layers, H = cache->num_kv_heads, D = cache->head_dim, T = num_tokens;
    const int32_t fmt = out_host->fmt;
    // bytes of one layer's codes (K and V) and scales in the stored form
    const uint64_t codes_l = (uint64_t)2 * T * H * row_code_bytes(fmt, D);
    const uint64_t scales_l = (uint64_t)2 * T * H * row_scale_bytes(fmt, D);
    const bool scaled = scales_l != 0;
    uint8_t *staging = static_cast<uint8_t *>(staging_dev);
    uint8_t *host = static_cast<uint8_t *>(out_host->data);
    const uint64_t half_bytes = need / 2;
    st = begin_staging(ln, ds->to_device, staging, need, user); // the kernels write the staging memory
    if (st != KDN_OK)
        return st;
    int stage_no = 0;
    for (int32_t l0 = 0; l0 < L; l0 += layers_per_stage, ++stage_no) {
        const int32_t Lg = std::min(layers_per_stage, L - l0);
        const int b = stage_no & 1;
        uint8_t *buf = staging + (uint64_t)b * half_bytes;
        // the kernel may overwrite this half only after the copy that last read it
        if (ln.drained_valid[b] && hipStreamWaitEvent(user, ln.drained[b], 0) != hipSuccess)
            return KDN_EDEVICE;
        if ((uint64_t)Lg * (codes_l + scales_l) > half_bytes
            || (uint64_t)L * codes_l + (uint64_t)(l0 + Lg) * scales_l > out_host->bytes)
            return KDN_ESIZE; // nothing may leave the staging half or the host buffer
        st = store_launch(cache, block_table_dev, table_len, token_start, T, nullptr, fmt, buf, l0, Lg, user);
        if (st != KDN_OK)
            return st;
        if (hipEventRecord(ln.filled[b], user) != hipSuccess
            || hipStreamWaitEvent(ln.stream, ln.filled[b], 0) != hipSuccess)
            return KDN_EDEVICE;
        // staged: codes of Lg layers, then their scales; both are contiguous runs of the host chunk
        if (hipMemcpyAsync(host + (uint64_t)l0 * codes_l, buf, (uint64_t)Lg * codes_l, hipMemcpyDeviceToHost,
                           ln.stream)
            != hipSuccess)
            return KDN_EDEVICE;
        if (scaled
            && hipMemcpyAsync(host + (uint64_t)L * codes_l + (uint64_t)l0 * scales_l, buf + (uint64_t)Lg * codes_l,
                              (uint64_t)Lg * scales_l, hipMemcpyDeviceToHost, ln.stream)
                   != hipSuccess)
            return KDN_EDEVICE;
        if (hipEventRecord(ln.drained[b], ln.stream) != hipSuccess)
            return KDN_EDEVICE;
        ln.drained_valid[b] = true;
    }
    // the caller's stream completes only when the last copies have landed
    for (int b = 0; b < 2; ++b)
        if (ln.drained_valid[b] && hipStreamWaitEvent(user, ln.drained[b], 0) != hipSuccess)
            return KDN_EDEVICE;
    describe_stored(cache, num_tokens, out_host);
    return KDN_OK;
}

kdn_status kdn_load_chunk(const kdn_chunk *chunk, const kdn_cache_desc *cache,
                          const int32_t *block_table_dev, int32_t table_len,
                          int32_t dest_token_start, void *stream)
{
    const int32_t zero = 0;
    kdn_request q = {chunk, &zero, 1, block_table_dev, table_len, dest_token_start};
    if (!chunk)
        return KDN_EINVAL;
    return compose_impl(&q, 1, cache, 1.0, nullptr, stream);
}

kdn_status kdn_compose(const kdn_chunk *chunks, const int32_t *offsets, int32_t n_chunks,
                       const kdn_cache_desc *cache, const int32_t *block_table_dev,
                       int32_t table_len, int32_t dest_token_start, double rope_base, void *stream)
{
    kdn_request q = {chunks, offsets, n_chunks, block_table_dev, table_len, dest_token_start};
    return compose_impl(&q, 1, cache, rope_base, nullptr, stream);
}

kdn_status kdn_compose_batch(const kdn_request *requests, int32_t n_requests,
                             const kdn_cache_desc *cache, double rope_base, void *stream)
{
    return compose_impl(requests, n_requests, cache, rope_base, nullptr, stream);
}

kdn_status kdn_compose_batch_static(const kdn_request *requests, int32_t n_requests,
                                    const kdn_cache_desc *cache, double rope_base, void *stream)
{
    ComposePlan plan;
    kdn_status st = plan_compose(requests, n_requests, cache, plan);
    if (st != KDN_OK)
        return st;
    RopeSpec spec;
    st = resolve_spec(nullptr, rope_base, cache->head_dim, spec);
    if (st != KDN_OK)
        return st;
    size_t n_segs = 0;
    for (int f = 0; f < kFormats; ++f)
        n_segs += plan.segs[f].size();
    if (n_segs > (size_t)kStaticMaxSegs)
        return KDN_ESIZE;
    // cos/sin rows of this call, in order of first appearance
    std::vector<int32_t> row_offsets;
    for (int f = 0; f < kFormats; ++f)
        for (PlannedSeg &ps : plan.segs[f]) {
            ps.seg.rope_row = -1;
            if (ps.offset == 0)
                continue;
            size_t r = 0;
            while (r < row_offsets.size() && row_offsets[r] != ps.offset)
                ++r;
            if (r == row_offsets.size()) {
                if ((int)r == kStaticMaxRopeRows)
                    return KDN_ESIZE;
                row_offsets.push_back(ps.offset);
            }
            ps.seg.rope_row = (int32_t)r;
        }
    if (!row_offsets.empty() && (!(spec.base > 0.0) || !std::isfinite(spec.base)))
        return KDN_EINVAL;

    std::lock_guard<std::mutex> lock(g_mu);
    DeviceState *ds = device_state(nullptr);
    if (!ds)
        return KDN_EDEVICE;
    if (!ds->static_scratch) { // once per device, with that device current
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(g_static_scratch)) != hipSuccess || !ptr)
            return KDN_EDEVICE;
        ds->static_scratch = static_cast<uint8_t *>(ptr);
    }
    uint8_t *scratch = ds->static_scratch;
    hipStream_t hs = static_cast<hipStream_t>(stream);

    // host image of what the kernels will read: the rows, then the records grouped by stored form
    const int32_t half = spec.rot / 2;
    std::vector<uint32_t> rope_words((size_t)row_offsets.size() * half * 2);
    for (size_t r = 0; r < row_offsets.size(); ++r)
        for (int32_t j = 0; j < half; ++j) {
            const double theta = std::pow(spec.base, -(double)(2 * j) / (double)spec.rot);
            const double phi = (double)row_offsets[r] * theta;
            const float c = (float)std::cos(phi), sn = (float)std::sin(phi);
            std::memcpy(&rope_words[(r * half + j) * 2], &c, 4);
            std::memcpy(&rope_words[(r * half + j) * 2 + 1], &sn, 4);
        }
    std::vector<Seg> all;
    all.reserve(n_segs);
    size_t first[kFormats];
    for (int f = 0; f < kFormats; ++f) {
        first[f] = all.size();
        for (const PlannedSeg &ps : plan.segs[f])
            all.push_back(ps.seg);
    }
    // the records and rows ride in kernel arguments: no copy call, nothing allocated
    auto upload = [&](const uint32_t *words, size_t n_words, size_t dst_byte) -> kdn_status {
        ScratchWords a;
        for (size_t at = 0; at < n_words; at += kScratchWords) {
            a.first = (uint32_t)(dst_byte / 4 + at);
            a.n = (uint32_t)std::min<size_t>(kScratchWords, n_words - at);
            std::memcpy(a.w, words + at, (size_t)a.n * 4);
            hipLaunchKernelGGL(k_scratch_write, dim3(1), dim3(kThreads), 0, hs,
                               reinterpret_cast<uint32_t *>(scratch), a);
            if (hipGetLastError() != hipSuccess)
                return KDN_EDEVICE;
        }
        return KDN_OK;
    };
    st = upload(rope_words.data(), rope_words.size(), 0);
    if (st != KDN_OK)
        return st;
    st = upload(reinterpret_cast<const uint32_t *>(all.data()), all.size() * sizeof(Seg) / 4, kStaticRopeBytes);
    if (st != KDN_OK)
        return st;

    PlaceP p;
    p.c = make_cache_p(cache);
    p.layer0 = 0;
    p.rot = spec.rot;
    p.pairing = spec.pairing;
    p.rope = reinterpret_cast<const f32x2 *>(scratch);
    for (int f = 0; f < kFormats; ++f) {
        if (plan.segs[f].empty())
            continue;
        std::vector<Seg> segs(all.begin() + (long)first[f], all.begin() + (long)(first[f] + plan.segs[f].size()));
        p.reuse = plan.reuse[f];
        st = place_segments(ds, p, f, segs, hs, 0,
                            reinterpret_cast<const Seg *>(scratch + kStaticRopeBytes) + first[f], plan.heads[f]);
        if (st != KDN_OK)
            return st;
    }
    return KDN_OK;
}

kdn_status kdn_compose_opts(const kdn_chunk *chunks, const int32_t *offsets, int32_t n_chunks,
                            const kdn_cache_desc *cache, const int32_t *block_table_dev,
                            int32_t table_len, int32_t dest_token_start, double rope_base,
                            const kdn_rope_spec *rope, const kdn_launch_opts *opts, void *stream)
{
    if (opts && opts->max_workgroups < 0)
        return KDN_EINVAL;
    kdn_request q = {chunks, offsets, n_chunks, block_table_dev, table_len, dest_token_start};
    return compose_impl(&q, 1, cache, rope_base, rope, stream, opts ? opts->max_workgroups : 0);
}

kdn_status kdn_compose_plan(const kdn_request *requests, int32_t n_requests, const kdn_cache_desc *cache,
                            kdn_placement *out, int32_t cap, int32_t *n_out)
{
    if (!n_out || cap < 0 || (cap > 0 && !out))
        return KDN_EINVAL;
    ComposePlan plan;
    kdn_status st = plan_compose(requests, n_requests, cache, plan);
    if (st != KDN_OK)
        return st;
    size_t n = 0;
    for (int f = 0; f < kFormats; ++f)
        n += plan.segs[f].size();
    if (n > 0x7fffffff)
        return KDN_ESIZE;
    *n_out = (int32_t)n;
    if (cap == 0)
        return KDN_OK; // the count alone
    if ((size_t)cap < n)
        return KDN_ESIZE;
    size_t k = 0;
    int32_t launch = 0;
    for (int f = 0; f < kFormats; ++f) {
        const size_t base = k; // `follows` counts within a launch; the output numbers all records
        for (const PlannedSeg &ps : plan.segs[f])
            out[k++] = {ps.request, ps.chunk, f, launch, ps.seg.S, ps.seg.T, ps.offset, plan.reuse[f],
                        ps.follows < 0 ? -1 : (int32_t)(base + (size_t)ps.follows)};
        launch += plan.segs[f].empty() ? 0 : 1;
    }
    return KDN_OK;
}

int32_t kdn_tile_tokens(const kdn_cache_desc *cache)
{
    return check_cache(cache) == KDN_OK ? make_cache_p(cache).G : 0;
}

kdn_status kdn_compose_rope(const kdn_chunk *chunks, const int32_t *offsets, int32_t n_chunks,
                            const kdn_cache_desc *cache, const int32_t *block_table_dev,
                            int32_t table_len, int32_t dest_token_start, const kdn_rope_spec *rope,
                            void *stream)
{
    if (!rope)
        return KDN_EINVAL;
    kdn_request q = {chunks, offsets, n_chunks, block_table_dev, table_len, dest_token_start};
    return compose_impl(&q, 1, cache, rope->base, rope, stream);
}

kdn_status kdn_compose_batch_rope(const kdn_request *requests, int32_t n_requests,
                                  const kdn_cache_desc *cache, const kdn_rope_spec *rope, void *stream)
{
    if (!rope)
        return KDN_EINVAL;
    return compose_impl(requests, n_requests, cache, rope->base, rope, stream);
}

kdn_status kdn_patch_rows(const void *rows_dev, const int32_t *tokens_dev, int32_t n_tokens,
                          const kdn_cache_desc *cache, const int32_t *block_table_dev,
                          int32_t table_len, void *stream)
{
    kdn_status st = check_cache(cache);
    if (st != KDN_OK)
        return st;
    if (!rows_dev || !tokens_dev || !block_table_dev || n_tokens <= 0 || table_len <= 0)
        return KDN_EINVAL;
    if (!aligned16(rows_dev))
        return KDN_EALIGN;
    if ((int64_t)n_tokens * 2 * cache->num_layers > 0x7fffffff / kThreads)
        return KDN_ESIZE;
    PatchP p;
    p.c = make_cache_p(cache);
    p.rows = static_cast<const uint16_t *>(rows_dev);
    p.tokens = tokens_dev;
    p.bt = block_table_dev;
    p.n = n_tokens;
    p.limit = (int64_t)table_len * cache->block_size > 0x7fffffff ? 0x7fffffff
                                                                   : table_len * cache->block_size;
    dim3 grid((unsigned)(n_tokens * 2 * cache->num_layers), 1, 1);
    hipLaunchKernelGGL(k_patch, grid, dim3(kThreads), 0, static_cast<hipStream_t>(stream), p);
    return hip_status(hipGetLastError());
}

uint64_t kdn_staging_bytes(const kdn_chunk *chunks, int32_t n_chunks, int32_t layers_per_stage)
{
    if (!chunks || n_chunks <= 0 || layers_per_stage <= 0)
        return 0;
    std::vector<HostParent> parents;
    std::vector<int32_t> parent_of;
    plan_host_parents(chunks, n_chunks, parents, parent_of);
    uint64_t stage = 0;
    for (const HostParent &hp : parents) {
        const uint64_t b = kdn_chunk_bytes(std::min(layers_per_stage, hp.L), hp.H, hp.D, hp.hi - hp.lo, hp.fmt);
        if (b == 0)
            return 0;
        stage += (b + 255) & ~(uint64_t)255;
    }
    return 2 * stage;
}

kdn_status kdn_host_stage_plan(const kdn_chunk *chunks, int32_t n_chunks, int32_t layers_per_stage,
                               int32_t stage, kdn_stage_copy *copies_out, int32_t cap, int32_t *n_copies,
                               uint64_t *view_offsets)
{
    if (!chunks || n_chunks <= 0 || layers_per_stage <= 0 || stage < 0 || !n_copies || cap < 0
        || (cap > 0 && !copies_out))
        return KDN_EINVAL;
    for (int32_t i = 0; i < n_chunks; ++i) {
        const kdn_chunk &ch = chunks[i];
        if (!ch.data || check_shape(ch.num_layers, ch.num_kv_heads, ch.head_dim) != KDN_OK || !known_format(ch.fmt)
            || ch.num_layers != chunks[0].num_layers || ch.num_kv_heads != chunks[0].num_kv_heads
            || ch.head_dim != chunks[0].head_dim)
            return KDN_EINVAL;
        if (ch.token_start < 0 || ch.num_tokens <= 0 || ch.parent_tokens <= 0
            || (int64_t)ch.token_start + ch.num_tokens > ch.parent_tokens)
            return KDN_ERANGE;
        if (ch.bytes < kdn_chunk_bytes(ch.num_layers, ch.num_kv_heads, ch.head_dim, ch.parent_tokens, ch.fmt))
            return KDN_ESIZE;
    }
    const int32_t L = chunks[0].num_layers;
    const int64_t l0 = (int64_t)stage * layers_per_stage;
    if (l0 >= L)
        return KDN_ERANGE;
    const uint64_t need = kdn_staging_bytes(chunks, n_chunks, layers_per_stage);
    if (need == 0)
        return KDN_ESIZE;
    std::vector<HostParent> parents;
    std::vector<int32_t> parent_of;
    plan_host_parents(chunks, n_chunks, parents, parent_of);
    std::vector<StageCopy> copies;
    std::vector<uint64_t> staged_at;
    kdn_status st = plan_stage_copies(parents, (int32_t)l0, std::min<int32_t>(layers_per_stage, L - (int32_t)l0),
                                      need / 2, copies, staged_at);
    if (st != KDN_OK)
        return st;
    *n_copies = (int32_t)copies.size();
    if ((int32_t)copies.size() > cap)
        return cap == 0 ? KDN_OK : KDN_ESIZE; // cap 0 asks for the count only
    for (size_t c = 0; c < copies.size(); ++c) {
        // name the first chunk that views the host buffer
        int32_t first = 0;
        while (parent_of[(size_t)first] != copies[c].parent)
            ++first;
        copies_out[c] = {first, (int32_t)copies[c].rows, copies[c].src_off, copies[c].src_pitch,
                         copies[c].width, copies[c].dst_off};
    }
    if (view_offsets)
        for (int32_t i = 0; i < n_chunks; ++i)
            view_offsets[i] = staged_at[(size_t)parent_of[(size_t)i]];
    return KDN_OK;
}

} // extern "C"

// stage_done: null, or one caller-owned event per stage, recorded behind the stage's kernels
static kdn_status compose_from_host_impl(const kdn_chunk *chunks, const int32_t *offsets, int32_t n_chunks,
                                         const kdn_cache_desc *cache, const int32_t *block_table_dev,
                                         int32_t table_len, int32_t dest_token_start, double rope_base,
                                         void *staging_dev, uint64_t staging_bytes, int32_t layers_per_stage,
                                         void *const *stage_done, void *stream)
{
    if (!chunks || !offsets || n_chunks <= 0 || !block_table_dev || table_len <= 0
        || dest_token_start < 0 || !staging_dev || layers_per_stage <= 0)
        return KDN_EINVAL;
    kdn_status st = check_cache(cache);
    if (st != KDN_OK)
        return st;
    if (!aligned16(staging_dev))
        return KDN_EALIGN;
    int64_t total = dest_token_start;
    for (int32_t i = 0; i < n_chunks; ++i) {
        st = check_chunk(&chunks[i], cache);
        if (st != KDN_OK)
            return st;
        hipPointerAttribute_t attr;
        if (hipPointerGetAttributes(&attr, chunks[i].data) != hipSuccess) {
            (void)hipGetLastError();
            return KDN_EINVAL; // ordinary pageable memory
        }
        if (attr.type != hipMemoryTypeHost)
            return KDN_EINVAL;
        total += chunks[i].num_tokens;
    }
    if (total > (int64_t)table_len * cache->block_size || total > 0x7fffffff)
        return KDN_ERANGE; // token indices are 32-bit in the kernels
    const uint64_t need = kdn_staging_bytes(chunks, n_chunks, layers_per_stage);
    if (need == 0 || staging_bytes < need)
        return KDN_ESIZE;
    std::vector<HostParent> parents;
    std::vector<int32_t> parent_of;
    plan_host_parents(chunks, n_chunks, parents, parent_of);

    std::lock_guard<std::mutex> lock(g_mu);
    DeviceState *ds = device_state(nullptr);
    if (!ds)
        return KDN_EDEVICE;
    LinkDir &ln = ds->to_device;
    st = ensure_link(ln);
    if (st != KDN_OK)
        return st;
    hipStream_t user = static_cast<hipStream_t>(stream);
    PlaceP p;
    p.c = make_cache_p(cache);
    RopeSpec spec;
    st = resolve_spec(nullptr, rope_base, cache->head_dim, spec);
    if (st != KDN_OK)
        return st;
    p.rot = spec.rot;
    p.pairing = spec.pairing;
    p.reuse = 0;
    std::vector<int32_t> rows((size_t)n_chunks);
    st = rope_rows(ds, spec, offsets, n_chunks, rows.data(), &p.rope);
    if (st != KDN_OK)
        return st;

    const int32_t L = cache->num_layers;
    uint8_t *staging = static_cast<uint8_t *>(staging_dev);
    const uint64_t half_bytes = need / 2;
    std::vector<StageCopy> copies;
    std::vector<uint64_t> staged_at;
    // The copies read the host chunks and write the staging memory on the library's copy
    // stream: order them behind everything the caller's stream holds so far (a store that
    // is still landing in the same host chunk, kernels that still use the staging memory).
    if (hipEventRecord(ln.entry, user) != hipSuccess || hipStreamWaitEvent(ln.stream, ln.entry, 0) != hipSuccess)
        return KDN_EDEVICE;
    st = begin_staging(ln, ds->to_host, staging, need, ln.stream); // the copies write the staging memory
    if (st != KDN_OK)
        return st;
    int stage_no = 0;
    for (int32_t l0 = 0; l0 < L; l0 += layers_per_stage, ++stage_no) {
        const int32_t Lg = std::min(layers_per_stage, L - l0);
        const int b = stage_no & 1;
        uint8_t *buf = staging + (uint64_t)b * half_bytes;
        // the copy may overwrite this half only after the kernel that last read it
        if (ln.drained_valid[b] && hipStreamWaitEvent(ln.stream, ln.drained[b], 0) != hipSuccess)
            return KDN_EDEVICE;
        st = plan_stage_copies(parents, l0, Lg, half_bytes, copies, staged_at);
        if (st != KDN_OK)
            return st;
        for (const StageCopy &c : copies) {
            const uint8_t *from = parents[(size_t)c.parent].data + c.src_off;
            hipError_t e;
            if (c.width == c.src_pitch) // whole chunk: the planes adjoin
                e = hipMemcpyAsync(buf + c.dst_off, from, c.width * c.rows, hipMemcpyHostToDevice, ln.stream);
            else
                e = hipMemcpy2DAsync(buf + c.dst_off, c.width, from, c.src_pitch, c.width, (size_t)c.rows,
                                     hipMemcpyHostToDevice, ln.stream);
            if (e != hipSuccess)
                return KDN_EDEVICE;
        }
        std::vector<Seg> segs[kFormats];
        int32_t S = dest_token_start;
        for (int32_t i = 0; i < n_chunks; ++i) {
            const kdn_chunk &ch = chunks[i];
            const HostParent &hp = parents[parent_of[i]];
            Seg s;
            s.data = buf + staged_at[(size_t)parent_of[i]];
            s.bt = block_table_dev;
            s.Tp = hp.hi - hp.lo;
            s.tok0 = ch.token_start - hp.lo;
            s.T = ch.num_tokens;
            s.S = S;
            s.rope_row = rows[i];
            s.next = 0;
            segs[ch.fmt].push_back(s);
            S += ch.num_tokens;
        }
        if (hipEventRecord(ln.filled[b], ln.stream) != hipSuccess
            || hipStreamWaitEvent(user, ln.filled[b], 0) != hipSuccess)
            return KDN_EDEVICE;
        p.c.L = Lg;
        p.layer0 = l0;
        for (int f = 0; f < kFormats; ++f) {
            st = place_segments(ds, p, f, segs[f], user);
            if (st != KDN_OK)
                return st;
        }
        if (hipEventRecord(ln.drained[b], user) != hipSuccess)
            return KDN_EDEVICE;
        ln.drained_valid[b] = true;
        if (stage_done && hipEventRecord(static_cast<hipEvent_t>(stage_done[stage_no]), user) != hipSuccess)
            return KDN_EDEVICE;
    }
    return KDN_OK;
}

extern "C" {

kdn_status kdn_compose_from_host(const kdn_chunk *chunks, const int32_t *offsets, int32_t n_chunks,
                                 const kdn_cache_desc *cache, const int32_t *block_table_dev,
                                 int32_t table_len, int32_t dest_token_start, double rope_base,
                                 void *staging_dev, uint64_t staging_bytes, int32_t layers_per_stage,
                                 void *stream)
{
    return compose_from_host_impl(chunks, offsets, n_chunks, cache, block_table_dev, table_len, dest_token_start,
                                  rope_base, staging_dev, staging_bytes, layers_per_stage, nullptr, stream);
}

kdn_status kdn_compose_from_host_staged(const kdn_chunk *chunks, const int32_t *offsets, int32_t n_chunks,
                                        const kdn_cache_desc *cache, const int32_t *block_table_dev,
                                        int32_t table_len, int32_t dest_token_start, double rope_base,
                                        void *staging_dev, uint64_t staging_bytes, int32_t layers_per_stage,
                                        void *const *stage_done, int32_t n_stage_events, void *stream)
{
    if (!stage_done || !cache || layers_per_stage <= 0 || cache->num_layers <= 0)
        return KDN_EINVAL;
    const int32_t stages = (cache->num_layers + layers_per_stage - 1) / layers_per_stage;
    if (n_stage_events != stages)
        return KDN_EINVAL;
    for (int32_t s = 0; s < stages; ++s)
        if (!stage_done[s])
            return KDN_EINVAL;
    return compose_from_host_impl(chunks, offsets, n_chunks, cache, block_table_dev, table_len, dest_token_start,
                                  rope_base, staging_dev, staging_bytes, layers_per_stage, stage_done, stream);
}

static kdn_status rope_prepare_impl(const kdn_rope_spec *variant, double rope_base, int32_t head_dim,
                                    const int32_t *offsets, int32_t n)
{
    if (!offsets || n <= 0)
        return KDN_EINVAL;
    kdn_status st = check_shape(1, 1, head_dim);
    if (st != KDN_OK)
        return st;
    RopeSpec spec;
    st = resolve_spec(variant, rope_base, head_dim, spec);
    if (st != KDN_OK)
        return st;
    std::lock_guard<std::mutex> lock(g_mu);
    DeviceState *ds = device_state(nullptr);
    if (!ds)
        return KDN_EDEVICE;
    std::vector<int32_t> rows((size_t)n);
    const f32x2 *table;
    return rope_rows(ds, spec, offsets, n, rows.data(), &table, /*pin=*/true);
}

kdn_status kdn_rope_prepare(double rope_base, int32_t head_dim, const int32_t *offsets, int32_t n)
{
    return rope_prepare_impl(nullptr, rope_base, head_dim, offsets, n);
}

kdn_status kdn_rope_prepare_spec(const kdn_rope_spec *rope, int32_t head_dim, const int32_t *offsets,
                                 int32_t n)
{
    if (!rope)
        return KDN_EINVAL;
    return rope_prepare_impl(rope, rope->base, head_dim, offsets, n);
}

kdn_status kdn_rope_release(void)
{
    std::lock_guard<std::mutex> lock(g_mu);
    DeviceState *ds = device_state(nullptr);
    if (!ds)
        return KDN_EDEVICE;
    if (hipDeviceSynchronize() != hipSuccess) // nothing may still read a row that is about to go
        return KDN_EDEVICE;
    for (RopeTable &rt : ds->rope) {
        rt.row_of.clear();
        rt.n_pinned = 0;
        if (rt.dev) {
            rt.pinned.assign((size_t)kRopeRowsCap, 0);
            rt.free_rows.resize((size_t)kRopeRowsCap);
            for (int32_t r = 0; r < kRopeRowsCap; ++r)
                rt.free_rows[(size_t)r] = kRopeRowsCap - 1 - r;
        }
    }
    return KDN_OK;
}

kdn_status kdn_validate_block_table(const int32_t *block_table_dev, int32_t table_len,
                                    int32_t num_blocks, void *stream)
{
    if (!block_table_dev || table_len <= 0 || num_blocks <= 0)
        return KDN_EINVAL;
    hipStream_t hs = static_cast<hipStream_t>(stream);
    uint32_t *scratch = nullptr;
    const size_t bytes = ((size_t)num_blocks + 1) * sizeof(uint32_t);
    if (hipMalloc(reinterpret_cast<void **>(&scratch), bytes) != hipSuccess)
        return KDN_EDEVICE;
    kdn_status rc = KDN_OK;
    uint32_t flags = 0;
    if (hipMemsetAsync(scratch, 0, bytes, hs) != hipSuccess)
        rc = KDN_EDEVICE;
    if (rc == KDN_OK) {
        hipLaunchKernelGGL(k_validate, dim3((table_len + 255) / 256), dim3(256), 0, hs, block_table_dev,
                           table_len, num_blocks, scratch + 1, scratch);
        if (hipGetLastError() != hipSuccess
            || hipMemcpyAsync(&flags, scratch, sizeof flags, hipMemcpyDeviceToHost, hs) != hipSuccess
            || hipStreamSynchronize(hs) != hipSuccess)
            rc = KDN_EDEVICE;
    }
    (void)hipFree(scratch);
    if (rc != KDN_OK)
        return rc;
    return flags ? KDN_ERANGE : KDN_OK;
}

kdn_status kdn_probe_stream(void *small_dev, void *big_dev, const int32_t *tile_ids_dev, uint32_t tiles,
                            int32_t tile_kib, int32_t direction, int32_t max_workgroups, void *stream)
{
    if (!small_dev || !big_dev || tiles == 0 || max_workgroups < 0 || direction < 0 || direction > 3)
        return KDN_EINVAL;
    if (tile_kib != 4 && (tile_kib < 8 || tile_kib > 4096 || tile_kib % 8 != 0))
        return KDN_EINVAL;
    if (!aligned16(small_dev) || !aligned16(big_dev))
        return KDN_EALIGN;
    const uint32_t chunks = tile_kib == 4 ? 1u : (uint32_t)tile_kib / 8; // the 4 KiB tile: one run of half the width
    const uint32_t grid = max_workgroups > 0 ? std::min<uint32_t>(tiles, (uint32_t)max_workgroups) : tiles;
    hipStream_t hs = static_cast<hipStream_t>(stream);
    u32x4 *sm = static_cast<u32x4 *>(small_dev), *bg = static_cast<u32x4 *>(big_dev);
    const dim3 g(grid), b(tile_kib == 4 ? kThreads / 2 : kThreads);
    const bool fixed = chunks == 4; // the 32 KiB tile has a kernel of its own with nothing predicated
#define KDN_PROBE(DIR)                                                                                      \
    case DIR:                                                                                               \
        if (fixed)                                                                                          \
            hipLaunchKernelGGL((k_probe_stream<DIR, 4>), g, b, 0, hs, sm, bg, tile_ids_dev, tiles, chunks); \
        else                                                                                                \
            hipLaunchKernelGGL((k_probe_stream<DIR, 0>), g, b, 0, hs, sm, bg, tile_ids_dev, tiles, chunks); \
        break;
    switch (direction) {
        KDN_PROBE(0)
        KDN_PROBE(1)
        KDN_PROBE(2)
        KDN_PROBE(3)
    }
#undef KDN_PROBE
    return hip_status(hipGetLastError());
}

kdn_status kdn_f32_to_bf16(const float *in_dev, uint16_t *out_dev, uint64_t n, void *stream)
{
    if (!in_dev || !out_dev)
        return KDN_EINVAL;
    if ((reinterpret_cast<uintptr_t>(in_dev) & 7u) || (reinterpret_cast<uintptr_t>(out_dev) & 3u))
        return KDN_EALIGN;
    if (n == 0)
        return KDN_OK;
    const uint64_t pairs = (n + 1) / 2;
    const unsigned blocks = (unsigned)std::min<uint64_t>((pairs + 255) / 256, 256 * 32);
    hipLaunchKernelGGL(k_f32_to_bf16, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                       in_dev, out_dev, n);
    return hip_status(hipGetLastError());
}

kdn_status kdn_shutdown(void)
{
    std::lock_guard<std::mutex> lock(g_mu);
    int cur = 0;
    (void)hipGetDevice(&cur);
    kdn_status rc = KDN_OK;
    for (auto &kv : g_dev) {
        if (hipSetDevice(kv.first) != hipSuccess || hipDeviceSynchronize() != hipSuccess) {
            rc = KDN_EDEVICE;
            continue;
        }
        DeviceState &ds = kv.second;
        for (auto &rt : ds.rope)
            if (rt.dev)
                (void)hipFree(rt.dev);
        if (ds.seg_dev)
            (void)hipFree(ds.seg_dev);
        if (ds.seg_host)
            (void)hipHostFree(ds.seg_host);
        for (int i = 0; i < kSegSlots; ++i)
            if (ds.seg_done[i])
                (void)hipEventDestroy(ds.seg_done[i]);
        destroy_link(ds.to_device);
        destroy_link(ds.to_host);
    }
    g_dev.clear();
    (void)hipSetDevice(cur);
    return rc;
}

const char *kdn_status_str(kdn_status s)
{
    switch (s) {
    case KDN_OK: return "ok";
    case KDN_EINVAL: return "invalid argument";
    case KDN_EALIGN: return "pointer or stride not 16-byte aligned";
    case KDN_ERANGE: return "token range or block id out of range";
    case KDN_ESIZE: return "buffer too small or too many segments";
    case KDN_EDEVICE: return "HIP call failed";
    case KDN_EUNSUPPORTED: return "head_dim must be a multiple of 16 (32 for int4), at most 512";
    case KDN_ENOTFOUND: return "no entry under this key";
    case KDN_EFULL: return "every cos/sin row is pinned by kdn_rope_prepare (kdn_rope_release frees them)";
    }
    return "unknown status";
}

#ifndef KDN_SRC_HASH
#error "build with -DKDN_SRC_HASH=\"<fingerprint of the sources>\" (paper_2409_13761_amd/build.py does)"
#endif
const char *kdn_version(void) { return "kdn-gfx950 0.2 src:" KDN_SRC_HASH; }

} // extern "C"
