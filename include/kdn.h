/*
 * kdn.h -- C ABI of the KDN KV-cache movement library for AMD MI355X (gfx950).
 *
 * The library moves precomputed KV caches between an inference engine's paged
 * KV memory and a compact stored form, the data-parallel core of the paper's
 * Knowledge Delivery Network:
 *   - kdn_store_chunk   : the engine hands a KV cache to the KDN (Sec. 3.2, interface (i));
 *                         the stored form is the compressed KV of the delivery
 *                         module (Sec. 3.1).
 *   - kdn_load_chunk    : the engine gets a KV cache back (Sec. 3.2, interface (ii));
 *                         it is decompressed on the GPU (Sec. 3.1).
 *   - kdn_compose[_batch]: the blending module puts several independently
 *                         precomputed KV caches together in one context (Sec. 3.1),
 *                         at positions other than the prefix (Sec. 3, the limitation
 *                         on prefix-only reuse; Sec. 3.2, KV-cache blending).
 * The paper defines no data format or arithmetic; the formats and rules below
 * are this library's definitions.
 *
 * General conventions
 *   - Pointers marked [device] are HIP device memory on the current device and are
 *     owned by the caller; pointers marked [host] are ordinary host memory, read
 *     before the call returns.  The library allocates no KV memory.  It owns only a
 *     small per-device table store (RoPE cos/sin rows, segment tables), created
 *     lazily and released by kdn_shutdown().
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All
 *     work is enqueued on it; calls return after enqueueing; results are valid once
 *     the stream has been synchronised.
 *   - Every call returns a kdn_status.  Argument errors are detected on the host
 *     and reported with nothing enqueued.  Nothing throws or aborts across the ABI.
 *   - Block ids inside a [device] block table are NOT checked on the fast path: an
 *     id outside [0, num_blocks) or a destination block listed twice is undefined
 *     behaviour.  kdn_validate_block_table() is the opt-in check.
 *   - KV values must be finite.
 *   - HIP graph capture: kdn_store_chunk, kdn_store_tokens, kdn_load_chunk,
 *     kdn_patch_rows, and kdn_compose / kdn_compose_rope with at most 64 chunks whose
 *     cos/sin rows are resident (kdn_rope_prepare) enqueue kernels only and may be
 *     captured.  The rows that kdn_rope_prepare made resident are pinned: the captured
 *     kernels keep reading the right cos/sin values on every replay, also after other
 *     calls have filled and recycled the rest of the table; only kdn_rope_release and
 *     kdn_shutdown end that.  Composes with more chunks (their segment table is copied from pinned
 *     memory and guarded by events), the staged host paths (kdn_store_to_host,
 *     kdn_compose_from_host, kdn_compose_from_host_staged: copies and events on
 *     library streams) and kdn_validate_block_table must not be captured.
 *   - Calls may come from several host threads and target several streams; the
 *     library serialises its own bookkeeping.  Two calls that write the same
 *     destination blocks race like any two kernels would.
 *
 * Paged cache layout (kdn_cache_desc).  For layer l, side K or V, physical block b,
 * slot s (token within the block), kv-head h and dimension j the bf16 element is
 *     base[l*layer_stride + b*block_stride + s*token_stride + h*head_stride + j]
 * with strides in elements and j contiguous.  Token t of a request whose block
 * table is bt lives in block bt[t / block_size], slot t % block_size.
 *
 * Stored forms (kdn_format).  A chunk stored with Tp tokens is one byte buffer:
 *   KDN_FMT_RAW_BF16       bf16 [L][2][Tp][H][D]             (side 0 = K, 1 = V)
 *   KDN_FMT_INT8_ROWSCALE  int8 [L][2][Tp][H][D]  codes, followed at byte
 *                          L*2*Tp*H*D by fp32 [L][2][Tp][H]  scales,
 *                          one scale per (token, kv-head) row.
 * int8 rule per row x[0..D): amax = max|x_j|.  If amax < 2^-121 (this includes the
 * all-zero row) the scale is 0 and all codes are 0.  Otherwise scale = amax/127,
 * inv = 127/amax (IEEE fp32 divisions) and code_j = clamp(rint(x_j*inv), -127, 127),
 * rint rounding halves to even; -128 is never produced.  Dequantisation is the
 * single fp32 product (float)code_j * scale, rounded to bf16 (nearest even).
 *   KDN_FMT_INT4_GROUP32   uint8 [L][2][Tp][H][D/2] packed codes, followed at byte
 *                          L*2*Tp*H*D/2 by fp32 [L][2][Tp][H][D/32] scales, one per
 *                          group of 32 consecutive elements (head_dim % 32 == 0).
 * int4 rule per group: amax over the group; amax < 2^-121 gives scale 0, codes 0;
 * otherwise scale = amax/7, inv = 7/amax, code_j = clamp(rint(x_j*inv), -7, 7), two
 * codes per byte as two's-complement nibbles, the even element in the low nibble;
 * dequantisation (float)code_j * scale_group.  5 bits per element instead of 8.25: a
 * tighter form toward the footprint reductions of Sec. 3.2, "KV-cache delivery".
 *   KDN_FMT_FP8_ROWSCALE   the int8 layout with e4m3 codes (4 exponent bits, bias 7, 3
 *                          mantissa bits, no infinities, largest finite value 448):
 *                          amax < 2^-119 gives scale 0, codes 0; otherwise scale =
 *                          amax/448, inv = 448/amax, code_j = e4m3(x_j*inv) rounded to
 *                          nearest even; dequantisation value(code_j) * scale.  Same
 *                          footprint as int8, relative instead of absolute precision.
 *
 * RoPE shift.  Keys carry rotary position embedding with half-split pairing:
 * element j pairs with j + D/2, j in [0, D/2), at frequency
 * theta_j = rope_base^(-2j/D).  Shifting a chunk by d positions maps
 *     lo' = fma(-hi, s_j, lo*c_j),   hi' = fma(lo, s_j, hi*c_j)
 * in fp32, where c_j = (float)cos(d*theta_j), s_j = (float)sin(d*theta_j) are
 * evaluated on the host in double as pow(rope_base, -(double)(2*j)/(double)D),
 * multiplied by (double)d, passed to cos/sin and rounded once to fp32.  A shift of
 * 0 skips the rotation (bit-identical to a load).  Values are never rotated.
 */
#ifndef KDN_H
#define KDN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    KDN_OK = 0,
    KDN_EINVAL = -1,       /* NULL pointer, non-positive size, unknown format, shape mismatch */
    KDN_EALIGN = -2,       /* a base pointer or stride is not 16-byte aligned */
    KDN_ERANGE = -3,       /* token range outside the block table / chunk, bad block id (validator) */
    KDN_ESIZE = -4,        /* chunk buffer too small, too many chunks, grid limit exceeded */
    KDN_EDEVICE = -5,      /* a HIP call failed, or no usable device */
    KDN_EUNSUPPORTED = -6, /* head_dim not a multiple of 16 (32 for int4) or above 512 */
    KDN_ENOTFOUND = -7,    /* no entry under this key (text-keyed pool) */
    KDN_EFULL = -8         /* the call needs more cos/sin rows than kdn_rope_prepare has left unpinned */
} kdn_status;

typedef enum {
    KDN_FMT_RAW_BF16 = 0,
    KDN_FMT_INT8_ROWSCALE = 1,
    KDN_FMT_INT4_GROUP32 = 2,
    KDN_FMT_FP8_ROWSCALE = 3
} kdn_format;

/* The engine's paged KV memory.  k_base, v_base: [device] bf16, 16-byte aligned;
 * all strides in elements and multiples of 8. */
typedef struct {
    void *k_base;
    void *v_base;
    int32_t num_layers, num_kv_heads, head_dim, block_size, num_blocks;
    int64_t layer_stride, block_stride, token_stride, head_stride;
} kdn_cache_desc;

/* A stored chunk, or a token view of one.  data: [device], 16-byte aligned, at
 * least kdn_chunk_bytes(..., parent_tokens, fmt) bytes.  A view covers tokens
 * [token_start, token_start + num_tokens) of the parent_tokens the buffer holds.
 * For kdn_store_chunk, kdn_store_tokens, kdn_load_chunk and the kdn_compose* calls,
 * data may instead be pinned host memory that the device can address (hipHostMalloc,
 * a pinned torch tensor): the kernels then read or write the stored rows across the
 * link themselves, with no staging buffer and no copy, at the link's rate and with
 * the same results; only the compact form crosses (Sec. 3.1, delivery module).  The
 * staged calls (kdn_store_to_host, kdn_compose_from_host) move the same bytes with
 * the copy engines instead and leave the compute units free meanwhile. */
typedef struct {
    void *data;
    uint64_t bytes;
    int32_t fmt; /* kdn_format */
    int32_t num_layers, num_kv_heads, head_dim;
    int32_t parent_tokens;
    int32_t token_start;
    int32_t num_tokens;
} kdn_chunk;

/* RoPE variants for composes (what real models need before a chunk can be reused at
 * another position, Sec. 3.2 "KV-cache blending"). */
typedef enum {
    KDN_ROPE_HALF_SPLIT = 0,  /* element j pairs with j + rot_dim/2 */
    KDN_ROPE_INTERLEAVED = 1  /* element 2j pairs with 2j + 1 */
} kdn_rope_pairing;

/* base: frequencies theta_j = base^(-2j/rot_dim), used when inv_freq is NULL.
 * inv_freq: [host] rot_dim/2 explicit frequencies in double (for models whose
 * frequencies are rescaled), or NULL.  rot_dim: only the first rot_dim elements of a
 * row are rotary, the rest pass through unrotated; a multiple of 16, at most head_dim;
 * 0 means head_dim.  pairing: kdn_rope_pairing.  The rotation is the one defined above,
 * applied to the pairs the variant names. */
typedef struct {
    double base;
    const double *inv_freq;
    int32_t rot_dim;
    int32_t pairing;
} kdn_rope_spec;

/* One request of a batched compose: chunks [host array of n_chunks], offsets [host
 * array of n_chunks RoPE position deltas], the request's block table [device], and
 * the first request token to write. */
typedef struct {
    const kdn_chunk *chunks;
    const int32_t *offsets;
    int32_t n_chunks;
    const int32_t *block_table_dev;
    int32_t table_len;
    int32_t dest_token_start;
} kdn_request;

/* Bytes of a stored chunk of num_tokens tokens: L*2*T*H*D*2 (raw), L*2*T*H*(D+4)
 * (int8, fp8) or L*2*T*H*(D/2 + D/8) (int4).  Returns 0 on invalid arguments. */
uint64_t kdn_chunk_bytes(int32_t num_layers, int32_t num_kv_heads, int32_t head_dim,
                         int32_t num_tokens, int32_t fmt);

/* Describe a whole stored chunk over a caller-owned buffer (no device work). */
kdn_status kdn_chunk_init(kdn_chunk *out, void *data_dev, uint64_t bytes, int32_t fmt,
                          int32_t num_layers, int32_t num_kv_heads, int32_t head_dim,
                          int32_t num_tokens);

/* View of tokens [token_start, token_start+num_tokens) of `chunk`, relative to the
 * chunk's own view (no device work).  KDN_ERANGE if the range leaves the chunk. */
kdn_status kdn_chunk_slice(const kdn_chunk *chunk, int32_t token_start, int32_t num_tokens,
                           kdn_chunk *out);

/* Store (Sec. 3.2, interface (i)).  Gathers request tokens [token_start,
 * token_start+num_tokens) through block_table_dev [device, table_len int32 entries]
 * from the paged cache into out->data in the format out->fmt.  In: out->data,
 * out->bytes, out->fmt.  Out: the remaining fields of *out (a whole chunk of
 * num_tokens tokens).  KDN_ESIZE if out->bytes is too small. */
kdn_status kdn_store_chunk(const kdn_cache_desc *cache, const int32_t *block_table_dev,
                           int32_t table_len, int32_t token_start, int32_t num_tokens,
                           kdn_chunk *out, void *stream);

/* Store of a token list: row t of the chunk holds request token tokens_dev[t] ([device]
 * int32, num_tokens entries, each in [0, table_len*block_size); an entry outside is
 * clamped into that range).  The gather a token-dropping compressor needs: only the
 * tokens it keeps are stored (Sec. 3.2, "KV-cache delivery").  Otherwise as
 * kdn_store_chunk. */
kdn_status kdn_store_tokens(const kdn_cache_desc *cache, const int32_t *block_table_dev,
                            int32_t table_len, const int32_t *tokens_dev, int32_t num_tokens,
                            kdn_chunk *out, void *stream);

/* Launch options.  max_workgroups > 0 caps the workgroups of the call's kernels, which
 * then stride over the tiles; 0 (or a NULL options pointer) launches one workgroup per
 * tile.  The cap is for chunks in pinned host memory: a few dozen workgroups keep the
 * link busy (the link, not the device, bounds such a call), and the rest of the device
 * stays free for the kernels of other streams, where an uncapped launch would sit on
 * every wave slot while it waits for the link.  Results do not depend on the cap. */
typedef struct kdn_launch_opts {
    int32_t max_workgroups;
} kdn_launch_opts;

/* kdn_store_chunk with launch options. */
kdn_status kdn_store_chunk_opts(const kdn_cache_desc *cache, const int32_t *block_table_dev,
                                int32_t table_len, int32_t token_start, int32_t num_tokens,
                                kdn_chunk *out, const kdn_launch_opts *opts, void *stream);

/* kdn_compose / kdn_compose_rope with launch options.  rope: NULL selects the default
 * variant at rope_base; otherwise rope_base is ignored.  Kernels only when the cos/sin
 * rows are resident and there are at most 64 chunks, hence capturable into a HIP graph,
 * chunks in host memory included. */
kdn_status kdn_compose_opts(const kdn_chunk *chunks, const int32_t *offsets, int32_t n_chunks,
                            const kdn_cache_desc *cache, const int32_t *block_table_dev,
                            int32_t table_len, int32_t dest_token_start, double rope_base,
                            const kdn_rope_spec *rope, const kdn_launch_opts *opts, void *stream);

/* Store into pinned HOST memory: the way out of the engine toward the storage device
 * (Sec. 3.1, storage module; CPU memory as the KV store, Sec. 3 "Limited storage").
 * out_host->data: [host], allocated with hipHostMalloc (or a pinned torch tensor), at
 * least kdn_chunk_bytes(...) bytes; in: data, bytes, fmt; out: the other fields.  The
 * kernels write layers_per_stage layers at a time, already in the stored form, into
 * staging_dev [device, 16-byte aligned, kdn_store_staging_bytes(...) bytes], and a copy
 * stream the library owns moves each stage to the host while the next is produced.  The
 * host chunk is complete once `stream` has been synchronised.  Same bytes as
 * kdn_store_chunk followed by a device-to-host copy. */
kdn_status kdn_store_to_host(const kdn_cache_desc *cache, const int32_t *block_table_dev,
                             int32_t table_len, int32_t token_start, int32_t num_tokens,
                             kdn_chunk *out_host, void *staging_dev, uint64_t staging_bytes,
                             int32_t layers_per_stage, void *stream);

/* Staging bytes kdn_store_to_host needs (two stages); 0 on invalid arguments. */
uint64_t kdn_store_staging_bytes(const kdn_cache_desc *cache, int32_t num_tokens, int32_t fmt,
                                 int32_t layers_per_stage);

/* Load (Sec. 3.2, interface (ii); decompression on the GPU, Sec. 3.1).  Writes the
 * chunk view's tokens to request tokens [dest_token_start, dest_token_start +
 * chunk->num_tokens) of the paged cache.  No rotation.  Slots and blocks outside
 * that token range are not written. */
kdn_status kdn_load_chunk(const kdn_chunk *chunk, const kdn_cache_desc *cache,
                          const int32_t *block_table_dev, int32_t table_len,
                          int32_t dest_token_start, void *stream);

/* Compose (blending module, Sec. 3.1).  Chunk i is written to request tokens
 * [dest_token_start + S_i, dest_token_start + S_i + T_i), S_i = sum of T_j, j < i, in
 * the order given; its K rows are shifted by offsets[i] positions (signed; only the
 * RoPE delta, independent of placement).  chunks, offsets: [host] arrays of
 * n_chunks.  Chunks may differ in format.  The first use of a new (rope_base,
 * head_dim, offset) uploads its cos/sin row synchronously; see kdn_rope_prepare. */
kdn_status kdn_compose(const kdn_chunk *chunks, const int32_t *offsets, int32_t n_chunks,
                       const kdn_cache_desc *cache, const int32_t *block_table_dev,
                       int32_t table_len, int32_t dest_token_start, double rope_base,
                       void *stream);

/* Many independent composes in one launch.  requests: [host] array of n_requests.
 * Block tables of different requests must not share destination blocks.  The
 * segment table is copied to the device on `stream` before the kernel. */
kdn_status kdn_compose_batch(const kdn_request *requests, int32_t n_requests,
                             const kdn_cache_desc *cache, double rope_base, void *stream);

/* kdn_compose_batch for callers that cannot allocate: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, same result.  The call
 * allocates no device memory, frees none, copies nothing and creates no event or stream:
 * the segment records and the cos/sin rows of the call ride in kernel arguments into a
 * scratch array that is part of the library's image (288 KiB per device, held until the
 * process ends), and the place kernels read them from there; only kernels are enqueued on
 * `stream`, whatever the number of chunks and whether or not kdn_rope_prepare was called.
 * Limits: at most 4096 chunk views in all requests together and at most 64 distinct
 * non-zero offsets per call; beyond either, KDN_ESIZE with nothing enqueued.  Every call
 * on a device uses that device's one scratch array, which keeps the last call's contents
 * (each call overwrites the part it uses; nothing has to start at zero): calls on ONE
 * stream are ordered like any kernels, calls that overlap on two streams of one device
 * race on it and must be ordered by the caller.  The first call on a device looks the
 * array's address up (hipGetSymbolAddress) and keeps it: make that call outside a capture. */
kdn_status kdn_compose_batch_static(const kdn_request *requests, int32_t n_requests,
                                    const kdn_cache_desc *cache, double rope_base, void *stream);

/* kdn_compose / kdn_compose_batch with a RoPE variant (rope: [host], not NULL).
 * KDN_EUNSUPPORTED if rot_dim is not a multiple of 16. */
kdn_status kdn_compose_rope(const kdn_chunk *chunks, const int32_t *offsets, int32_t n_chunks,
                            const kdn_cache_desc *cache, const int32_t *block_table_dev,
                            int32_t table_len, int32_t dest_token_start, const kdn_rope_spec *rope,
                            void *stream);
kdn_status kdn_compose_batch_rope(const kdn_request *requests, int32_t n_requests,
                                  const kdn_cache_desc *cache, const kdn_rope_spec *rope, void *stream);

/* The bookkeeping of kdn_compose_batch without the launch, for callers that want to
 * inspect or log a plan (host only: no device is touched, no pointer is dereferenced
 * beyond the request and chunk records).  One record per chunk view, in the order the
 * kernels take them: grouped by stored form (one launch per form present, `launch`
 * counts them), and, when there is more than one request, views of the same stored rows
 * next to each other.  Views that are exactly the same stored rows (same buffer, same token
 * range) and whose destinations are congruent modulo the tile's token count
 * (kdn_tile_tokens) are read once: the first such view has
 * workgroups of its own, each later one names in `follows` the record it is chained behind
 * (the workgroup that read a tile for that record places it for this one next, out of the
 * caches), and chained records come after all records with workgroups in their launch.
 * dest_token is the request token that receives the view's first
 * row: dest_token_start plus the token counts of the views before it in its request.
 * shares_rows is 1 when some stored rows are read by more than one view of that launch
 * (the kernels then keep them in the cache hierarchy).  Argument checks and status
 * codes are those of kdn_compose_batch.  out: [host] array of `cap` records; *n_out
 * receives the count (cap 0 asks for the count alone); KDN_ESIZE if cap is too small. */
typedef struct kdn_placement {
    int32_t request, chunk; /* indices into requests[] and its chunks[] */
    int32_t fmt;
    int32_t launch;
    int32_t dest_token;
    int32_t num_tokens;
    int32_t offset;         /* RoPE position delta of the view */
    int32_t shares_rows;
    int32_t follows;        /* index in `out` of the record this view is chained behind, -1: none */
} kdn_placement;
kdn_status kdn_compose_plan(const kdn_request *requests, int32_t n_requests, const kdn_cache_desc *cache,
                            kdn_placement *out, int32_t cap, int32_t *n_out);

/* Tokens whose rows (one layer, one side) one workgroup moves at a time for this cache: 16
 * for block sizes 1 to 3 and multiples of 16, else the block size.  Host only.  0 if the
 * descriptor is not valid. */
int32_t kdn_tile_tokens(const kdn_cache_desc *cache);

/* Patch: the write-back half of selective recompute after a blend (Sec. 3.2, "KV-cache
 * blending": recomputing a small part of the composed KV).  rows_dev [device, 16-byte
 * aligned]: bf16 [L][2][n_tokens][H][D] recomputed K and V rows; row i replaces request
 * token tokens_dev[i] ([device] int32, distinct) through block_table_dev.  Bit copy, no
 * arithmetic.  A token index outside [0, table_len*block_size) is skipped. */
kdn_status kdn_patch_rows(const void *rows_dev, const int32_t *tokens_dev, int32_t n_tokens,
                          const kdn_cache_desc *cache, const int32_t *block_table_dev,
                          int32_t table_len, void *stream);

/* Compose from chunks held in pinned HOST memory: the delivery module's path from a
 * storage device to the GPU (Sec. 3.1; bandwidth of loading KV into GPU memory, Sec. 3
 * "Limited storage"; transfer over links, Sec. 3.2).  Same result as kdn_compose.
 * chunks[i].data: [host], allocated with hipHostMalloc (or a pinned torch tensor), in the
 * stored form; it must stay unchanged until `stream` has run the call.  The stored rows
 * cross the link in their compact form, layers_per_stage layers at a time, into
 * staging_dev [device, 16-byte aligned, at least kdn_staging_bytes(...) bytes] on a
 * copy stream the library owns, while the previous stage is dequantised, rotated and
 * scattered on `stream`: copy and kernels overlap, and the two halves of the staging
 * buffer alternate.  The staging buffer may be reused by the next call on any stream.
 * KDN_EINVAL if a chunk is not in pinned host memory, KDN_ESIZE if the staging buffer is
 * too small.  Choosing layers_per_stage: the kernels are about a hundred times faster
 * than the link, so a handful of stages already hides them; each stage enqueues one or
 * two copies per host buffer, and calls issued back to back run slower once more than
 * about a dozen copies are outstanding (measured: 32 layers in 8 stages 6.5 ms per call,
 * in 4 stages or fewer 5.0 ms). */
kdn_status kdn_compose_from_host(const kdn_chunk *chunks, const int32_t *offsets, int32_t n_chunks,
                                 const kdn_cache_desc *cache, const int32_t *block_table_dev,
                                 int32_t table_len, int32_t dest_token_start, double rope_base,
                                 void *staging_dev, uint64_t staging_bytes, int32_t layers_per_stage,
                                 void *stream);

/* kdn_compose_from_host that also tells the engine when each stage is in place, so that
 * it can run the layers of a stage while later stages are still crossing the link
 * (loading overlapped with inference; Sec. 3 "Limited storage", the bandwidth of loading
 * KV into GPU memory).  stage_done: [host] array of n_stage_events hipEvent_t (as void*),
 * created and owned by the caller; event s is recorded on `stream` behind the kernels
 * that place layers [s*layers_per_stage, min(L, (s+1)*layers_per_stage)): once it has
 * completed, those layers of the request hold their final values.  n_stage_events must be
 * ceil(num_layers / layers_per_stage), else KDN_EINVAL.  Everything else as above. */
kdn_status kdn_compose_from_host_staged(const kdn_chunk *chunks, const int32_t *offsets, int32_t n_chunks,
                                        const kdn_cache_desc *cache, const int32_t *block_table_dev,
                                        int32_t table_len, int32_t dest_token_start, double rope_base,
                                        void *staging_dev, uint64_t staging_bytes, int32_t layers_per_stage,
                                        void *const *stage_done, int32_t n_stage_events, void *stream);

/* Bytes of staging memory kdn_compose_from_host needs for these chunk views at this
 * stage depth: two stages of compact rows; views of one host buffer share one staged
 * copy of the token range they span; each copy is padded to 256 bytes.  0 on invalid
 * arguments.  chunks: [host] array; the data they point to is not read. */
uint64_t kdn_staging_bytes(const kdn_chunk *chunks, int32_t n_chunks, int32_t layers_per_stage);

/* The link transfers of one stage of kdn_compose_from_host, for callers that account for
 * link bytes or want to check a plan before running it.  Host only: no device is touched
 * and the chunks' data is not read (any non-null pointer serves).  Stage s covers layers
 * [s*layers_per_stage, min(L, (s+1)*layers_per_stage)).  One kdn_stage_copy is `rows` runs
 * of `width` bytes that lie `src_pitch` apart starting `src_offset` bytes into the data of
 * chunks[chunk] (the first view of that host buffer), packed back to back from
 * `dst_offset` of the stage's staging half.  The staged image of a host buffer is a stored
 * chunk of the stage's layers and the token range its views span; view_offsets[i] ([host]
 * array of n_chunks, may be null) is where the image that chunks[i] reads starts.
 * copies_out: [host] array of `cap` records; *n_copies receives the count (cap 0 asks for
 * the count alone).  KDN_ERANGE when the stage is past the last layer, KDN_ESIZE when cap
 * is too small or a chunk's bytes do not cover its layout. */
typedef struct kdn_stage_copy {
    int32_t chunk;
    int32_t rows;
    uint64_t src_offset, src_pitch, width, dst_offset;
} kdn_stage_copy;
kdn_status kdn_host_stage_plan(const kdn_chunk *chunks, int32_t n_chunks, int32_t layers_per_stage,
                               int32_t stage, kdn_stage_copy *copies_out, int32_t cap, int32_t *n_copies,
                               uint64_t *view_offsets);

/* Make the cos/sin rows of the given offsets resident, so that later composes with them
 * enqueue no copy (needed before capturing composes into a HIP graph), and pin them: a
 * pinned row keeps its place and contents until kdn_rope_release or kdn_shutdown, so a
 * captured graph that holds its index replays correctly whatever happens in between.
 * Rows that a compose brings in by itself are transient: when the table of a (frequencies,
 * rotary width) pair has no free row (it holds 4096), the device is synchronised and the
 * transient rows are dropped; pinned rows are not touched.  KDN_EFULL when the offsets
 * need more rows than are left unpinned (nothing is changed then).  offsets: [host] array
 * of n. */
kdn_status kdn_rope_prepare(double rope_base, int32_t head_dim, const int32_t *offsets,
                            int32_t n);

/* The same for a RoPE variant (rope: [host], not NULL). */
kdn_status kdn_rope_prepare_spec(const kdn_rope_spec *rope, int32_t head_dim, const int32_t *offsets,
                                 int32_t n);

/* Drops every cos/sin row of the current device, pinned ones included (synchronises the
 * device first).  Graphs captured earlier that hold composes with a non-zero offset must
 * not be replayed afterwards: prepare and capture again. */
kdn_status kdn_rope_release(void);

/* Debug check, synchronous: KDN_ERANGE if any of the table_len entries of
 * block_table_dev [device] is outside [0, num_blocks) or occurs twice. */
kdn_status kdn_validate_block_table(const int32_t *block_table_dev, int32_t table_len,
                                    int32_t num_blocks, void *stream);

/* A measuring aid, not a step of the path: moves bytes in the patterns of this library with no
 * arithmetic and no table walk, as the yardstick its kernels are held against.  A tile is
 * tile_kib KiB of big_dev and tile_kib/2 KiB of small_dev (tile_kib 4 or a multiple of 8, at
 * most 4096; 32 is the tile of the Llama shapes at block size 16, 4 that of one KV head of 128).  direction 0, the pattern of load
 * and compose: a workgroup reads tile i of small_dev and writes tile i of big_dev, or, with
 * tile_ids_dev [device, `tiles` distinct int32], tile tile_ids_dev[i] (destination tiles
 * scattered like the blocks of a random block table).  direction 1, the pattern of store: reads
 * that tile of big_dev, writes tile i of small_dev.  direction 2 writes that tile of big_dev and
 * reads nothing, direction 3 reads it and writes nothing (small_dev is then only a place the
 * kernel could write to): the two directions of the memory on their own.  max_workgroups > 0 caps
 * the launch (the workgroups then stride over the tiles).  small_dev: [device] tiles * tile_kib/2
 * KiB; big_dev: [device], holds every tile that is named.  Ids are not checked. */
kdn_status kdn_probe_stream(void *small_dev, void *big_dev, const int32_t *tile_ids_dev, uint32_t tiles,
                            int32_t tile_kib, int32_t direction, int32_t max_workgroups, void *stream);

/* fp32 -> bf16, round to nearest even, n elements, in_dev/out_dev [device], the
 * conversion every load and compose ends with. */
kdn_status kdn_f32_to_bf16(const float *in_dev, uint16_t *out_dev, uint64_t n, void *stream);

/* Release the library's device tables on every device (synchronises them). */
kdn_status kdn_shutdown(void);

const char *kdn_status_str(kdn_status status);

/* "kdn-gfx950 <version> src:<16 hex digits>": the digits are a hash of the sources and
 * compiler flags the library was built from, so that a caller (the Python binding does)
 * can refuse a binary that does not belong to the sources beside it. */
const char *kdn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* KDN_H */
