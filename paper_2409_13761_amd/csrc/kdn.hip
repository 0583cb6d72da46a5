// KDN KV-cache movement for MI355X (gfx950): kernels, host planner and the C ABI
// declared in include/kdn.h.
//
// Three data-parallel operations of the paper's Knowledge Delivery Network:
// store (Sec. 3.2, interface (i)), load (interface (ii), decompression on the GPU,
// Sec. 3.1) and compose (blending module, Sec. 3.1).  All of them stream rows of
// head_dim elements between two layouts; none is a contraction, so the kernels are
// organised around 64-wide wavefronts issuing full-width global loads and stores,
// and the per-row reductions use cross-lane operations.
//
// Work decomposition (both directions): a workgroup owns one (layer, K|V, token
// group) tile.  A token group is a run of at most G consecutive request tokens that
// lies inside one paged block, so a tile is contiguous in the paged cache (for the
// dense layout) and contiguous in the stored chunk.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <mutex>
#include <new>
#include <unordered_map>
#include <vector>

#include "kdn.h"

namespace {

constexpr int kThreads = 256;      // 4 wavefronts per workgroup
constexpr int kMaxInlineSegs = 64; // segments that travel in the kernel arguments
constexpr int kMaxHeadDim = 512;
constexpr int kStoreU = 4;         // 16-byte loads a store thread keeps in flight
constexpr int kRopeRowsCap = 4096; // cos/sin rows kept per (base, head_dim)
constexpr int kSegSlots = 8;       // ring of device segment tables for batched composes
constexpr size_t kSegSlotBytes = 1u << 20;

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// One placed chunk view: rows of tokens [tok0, tok0+T) of a stored buffer that
// holds Tp tokens go to request tokens [S, S+T) of the request whose table is bt.
struct Seg {
    const uint8_t *data;
    const int32_t *bt;
    int32_t Tp, tok0, T, S;
    int32_t rope_row; // row of the cos/sin table, -1: no rotation
    int32_t pad;
};
static_assert(sizeof(Seg) == 40, "Seg layout");

struct SegsInline {
    Seg s[kMaxInlineSegs];
    __device__ const Seg &at(int i) const { return s[i]; }
};
struct SegsDevice {
    const Seg *s;
    __device__ const Seg &at(int i) const { return s[i]; }
};

struct CacheP {
    uint16_t *k, *v;
    int64_t layer_stride, block_stride, token_stride, head_stride;
    int32_t L, H, D, bs;
    int32_t G;     // tokens per group; divides bs
    int32_t dense; // head_stride == D and token_stride == H*D
};

struct StoreP {
    CacheP c;
    const int32_t *bt;
    uint8_t *out;
    int32_t t0, T;
    const int32_t *tokens; // token-list store: row t holds request token tokens[t]; else NULL
    int32_t limit;         // request tokens the block table covers (list entries are clamped to it)
};

struct PlaceP {
    CacheP c;          // c.L counts the layers the stored rows hold (and the grid covers)
    const f32x2 *rope; // [rows][rot/2] (cos, sin)
    int32_t layer0;    // cache layer that stored layer 0 goes to
    int32_t rot;       // rotary leading dimensions (head_dim unless partial rotary)
    int32_t pairing;   // kdn_rope_pairing
    int32_t reuse;     // some stored rows are read by more than one segment: let them stay cached
};

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

__device__ __forceinline__ float code_f32(uint32_t w, int byte)
{
    return (float)(int8_t)(w >> (8 * byte));
}

constexpr __host__ __device__ int log2_ceil(int x)
{
    int l = 0;
    while ((1 << l) < x)
        ++l;
    return l;
}

// ---------------------------------------------------------------------------------
// store: gather paged rows, per-row amax, quantise.
// Lane group: D/8 lanes own one row, 8 consecutive elements (one 16-byte load) each;
// the group is padded to a power of two so the row reduction is a butterfly of
// cross-lane moves (DPP within 16 lanes, wavefront shuffles beyond).
// Grid: x = group * 2L + (layer, side).

// max over the P lanes of a row's lane group; every lane of the group gets the result
template <int P>
__device__ __forceinline__ uint32_t group_max(uint32_t m)
{
    if (P >= 2) // lane ^ 1
        m = max(m, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)m, 0xB1, 0xf, 0xf, true));
    if (P >= 4) // lane ^ 2
        m = max(m, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)m, 0x4E, 0xf, 0xf, true));
    if (P >= 8) // mirror within 8 lanes: the other quad
        m = max(m, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)m, 0x141, 0xf, 0xf, true));
    if (P >= 16) // mirror within 16 lanes: the other half
        m = max(m, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)m, 0x140, 0xf, 0xf, true));
    if (P >= 32)
        m = max(m, (uint32_t)__shfl_xor((int)m, 16));
    if (P >= 64)
        m = max(m, (uint32_t)__shfl_xor((int)m, 32));
    return m;
}

// Row maximum of |x| over the 8 bf16 values a lane holds, as the 15-bit pattern.
__device__ __forceinline__ uint32_t lane_absmax_bits(u32x4 w)
{
    typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
    u16x2 a = __builtin_bit_cast(u16x2, w[0] & 0x7fff7fffu);
#pragma unroll
    for (int i = 1; i < 4; ++i)
        a = __builtin_elementwise_max(a, __builtin_bit_cast(u16x2, w[i] & 0x7fff7fffu));
    const uint32_t m = __builtin_bit_cast(uint32_t, a);
    return max(m & 0xffffu, m >> 16);
}

// Codes of 4 values: rint(x * inv) by the add-a-large-constant rule, which rounds the
// (already rounded) product to the nearest integer, ties to even, exactly as rintf
// does for |value| < 2^22; the code is then the low byte of the sum's bit pattern.
// The clamp to [-127, 127] of the format's definition can never bind for finite
// input: |x| <= amax and inv = RN(127/amax) <= (127/amax)(1 + 2^-24) give
// |x*inv| <= 127(1 + 2^-24), whose fp32 rounding is at most the float just above
// 127, and that still rounds to the integer 127.
__device__ __forceinline__ uint32_t quantise4(uint32_t w0, uint32_t w1, float inv)
{
    const float magic = 12582912.0f; // 1.5 * 2^23
    const uint32_t t0 = __float_as_uint(bf16_lo(w0) * inv + magic);
    const uint32_t t1 = __float_as_uint(bf16_hi(w0) * inv + magic);
    const uint32_t t2 = __float_as_uint(bf16_lo(w1) * inv + magic);
    const uint32_t t3 = __float_as_uint(bf16_hi(w1) * inv + magic);
    const uint32_t p01 = __builtin_amdgcn_perm(t1, t0, 0x0c0c0400u); // bytes: t0.b0, t1.b0, 0, 0
    const uint32_t p23 = __builtin_amdgcn_perm(t3, t2, 0x04000c0cu); // bytes: 0, 0, t2.b0, t3.b0
    return p01 | p23;
}

template <int DT, int FMT, int P, bool DENSE>
__global__ __launch_bounds__(kThreads) void k_store(StoreP p)
{
    constexpr int U = kStoreU;
    constexpr int LOGP = log2_ceil(P);
    // with at least 8 lanes per row the 2*U divisions of a batch are spread over the
    // lanes of the row's group (one division sequence per batch instead of 2*U)
    constexpr bool SPREAD = P >= 8 && U == 4;
    const int D = DT ? DT : p.c.D;
    const int R = D >> 3;
    const int H = p.c.H, G = p.c.G, bs = p.c.bs;
    const int L2 = 2 * p.c.L;

    const int piece = blockIdx.x / L2;
    const int ls = blockIdx.x - piece * L2;
    const int gi = p.t0 / G + piece;
    const int tok_lo = max(p.t0, gi * G);
    const int tok_hi = min(p.t0 + p.T, (gi + 1) * G);
    if (tok_lo >= tok_hi)
        return;
    // a token list (strided instantiation only) resolves every row's token by itself
    const bool listed = !DENSE && p.tokens != nullptr;
    const uint16_t *plane = ((ls & 1) ? p.c.v : p.c.k) + (int64_t)(ls >> 1) * p.c.layer_stride;
    const int blk = listed ? 0 : p.bt[tok_lo / bs];
    const int slot0 = listed ? 0 : tok_lo % bs;
    const uint16_t *tile = plane + (int64_t)blk * p.c.block_stride + (int64_t)slot0 * p.c.token_stride;
    const int64_t row_base = ((int64_t)ls * p.T + (tok_lo - p.t0)) * H;
    const int n_items = ((tok_hi - tok_lo) * H) << LOGP;
    const int64_t total_rows = (int64_t)p.c.L * 2 * p.T * H;
    constexpr int W = FMT == KDN_FMT_RAW_BF16 ? 4 : FMT == KDN_FMT_INT8_ROWSCALE ? 2 : 1; // words per 8 stored elements
    const int spr = FMT == KDN_FMT_INT4_GROUP32 ? D >> 5 : 1;                              // scales per row
    uint8_t *codes = p.out + ((row_base * D * W) >> 1);
    float *scales = reinterpret_cast<float *>(p.out + ((total_rows * D * W) >> 1)) + row_base * spr;

    const int sub = threadIdx.x & (P - 1);
    const int lane = __lane_id();
    const int grp_addr = (lane & ~(P - 1)) << 2; // byte address of the group's first lane for bpermute

    for (int base = 0; base < n_items; base += kThreads * U) {
        u32x4 w[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int it = base + u * kThreads + threadIdx.x;
            const int r = it >> LOGP;
            w[u] = u32x4{0, 0, 0, 0};
            if (it < n_items && sub < R) {
                const uint16_t *src;
                if (DENSE) {
                    src = tile + (uint32_t)(r * D + sub * 8);
                } else {
                    const int tok = r / H, h = r - tok * H;
                    if (listed) {
                        const int t = min(max(p.tokens[tok_lo + tok], 0), p.limit - 1);
                        src = plane + (int64_t)p.bt[t / bs] * p.c.block_stride + (int64_t)(t % bs) * p.c.token_stride
                              + (int64_t)h * p.c.head_stride + sub * 8;
                    } else {
                        src = tile + (int64_t)tok * p.c.token_stride + (int64_t)h * p.c.head_stride + sub * 8;
                    }
                }
                w[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(src));
            }
        }
        if (FMT == KDN_FMT_RAW_BF16) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int it = base + u * kThreads + threadIdx.x;
                const int r = it >> LOGP;
                if (it < n_items && sub < R)
                    __builtin_nontemporal_store(
                        w[u], reinterpret_cast<u32x4 *>(codes + (uint32_t)(r * D + sub * 8) * 2));
            }
            continue;
        }
        if (FMT == KDN_FMT_INT4_GROUP32) {
            // a group of 32 elements is a quad of lanes; lane (sub & 3) of the quad forms
            // 7/amax and amax/7 of item (sub & 3): two division sequences serve the batch
            uint32_t m4[U];
#pragma unroll
            for (int u = 0; u < U; ++u)
                m4[u] = group_max<4>(lane_absmax_bits(w[u]));
            const int us = sub & 3;
            const uint32_t msel = us == 0 ? m4[0] : us == 1 ? m4[1] : us == 2 ? m4[2] : m4[U - 1];
            const float amax = __uint_as_float(msel << 16);
            const bool keep = amax >= 0x1p-121f;
            const float q_inv = keep ? 7.0f / amax : 0.0f;
            const float q_scale = keep ? amax / 7.0f : 0.0f;
            const int it_s = base + us * kThreads + threadIdx.x;
            if (it_s < n_items && sub < R)
                scales[(it_s >> LOGP) * spr + (sub >> 2)] = q_scale;
            float inv4[U];
            inv4[0] = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(q_inv), 0x00, 0xf, 0xf, true));
            inv4[1] = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(q_inv), 0x55, 0xf, 0xf, true));
            inv4[2] = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(q_inv), 0xAA, 0xf, 0xf, true));
            inv4[U - 1] = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(q_inv), 0xFF, 0xf, 0xf, true));
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int it = base + u * kThreads + threadIdx.x;
                const int r = it >> LOGP;
                if (it < n_items && sub < R) {
                    const float magic = 12582912.0f; // see quantise4: rint by adding 1.5 * 2^23
                    uint32_t acc = 0;
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const uint32_t word = w[u][e >> 1];
                        const float x = (e & 1) ? bf16_hi(word) : bf16_lo(word);
                        acc |= (__float_as_uint(x * inv4[u] + magic) & 0xfu) << (4 * e);
                    }
                    __builtin_nontemporal_store(acc, reinterpret_cast<uint32_t *>(codes + (((uint32_t)(r * D + sub * 8)) >> 1)));
                }
            }
            continue;
        }
        // |x| of a bf16 orders like its low 15 bits
        uint32_t m[U];
#pragma unroll
        for (int u = 0; u < U; ++u)
            m[u] = group_max<P>(lane_absmax_bits(w[u]));
        float inv[U];
        if (SPREAD) {
            // lane sub of the group: item (sub & 3); lanes 0..3 form inv = 127/amax,
            // lanes 4..7 form scale = amax/127 (lanes 8.. repeat, unused)
            const int us = sub & 3;
            const uint32_t msel = us == 0 ? m[0] : us == 1 ? m[1] : us == 2 ? m[2] : m[U - 1];
            const float amax = __uint_as_float(msel << 16);
            const bool is_scale = (sub & 4) != 0;
            const float q = (is_scale ? amax : 127.0f) / (is_scale ? 127.0f : amax);
            const float quot = amax >= 0x1p-121f ? q : 0.0f;
#pragma unroll
            for (int u = 0; u < U; ++u)
                inv[u] = __int_as_float(__builtin_amdgcn_ds_bpermute(grp_addr + 4 * u, __float_as_int(quot)));
            const int it_s = base + us * kThreads + threadIdx.x; // same row as every lane of the group
            if (is_scale && sub < 8 && it_s < n_items)
                scales[it_s >> LOGP] = quot;
        } else {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const float amax = __uint_as_float(m[u] << 16);
                const bool keep = amax >= 0x1p-121f;
                inv[u] = keep ? 127.0f / amax : 0.0f;
                const int it = base + u * kThreads + threadIdx.x;
                if (sub == 0 && it < n_items)
                    scales[it >> LOGP] = keep ? amax / 127.0f : 0.0f;
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int it = base + u * kThreads + threadIdx.x;
            const int r = it >> LOGP;
            if (it < n_items && sub < R) {
                const u32x2 q = {quantise4(w[u][0], w[u][1], inv[u]), quantise4(w[u][2], w[u][3], inv[u])};
                __builtin_nontemporal_store(q, reinterpret_cast<u32x2 *>(codes + (uint32_t)(r * D + sub * 8)));
            }
        }
    }
}

// ---------------------------------------------------------------------------------
// place: dequantise (or copy), rotate K pairs, round to bf16, scatter.
// Lane group: D/16 lanes own one row; a lane takes 8 elements of the lower half and
// the 8 elements of the upper half that pair with them, so the rotation needs no
// exchange between lanes and each lane writes two full 16-byte bf16 vectors.
// Each thread issues the loads of U items before it touches the first, and both the
// stored chunk and the paged destination are streamed (non-temporal): nothing here is
// read twice.
// Grid: x = group * 2L + (layer, side), so that neighbouring workgroups write to
// different (layer, side) planes; y = segment.
// Stored rows are streamed past the caches unless several segments read the same rows
// (a popular chunk in a batched compose): then they are loaded normally, so that the
// first reader leaves them in L2 and the last-level cache for the others.
template <typename T, bool REUSE>
__device__ __forceinline__ T load_stored(const uint8_t *ptr)
{
    const T *q = reinterpret_cast<const T *>(ptr);
    if (REUSE)
        return *q;
    return __builtin_nontemporal_load(q);
}

// VAR selects the RoPE variants (partial rotary, interleaved pairs): lanes of the rotary
// part keep the 8 + 8 paired ownership (half-split) or own 16 consecutive elements whose
// pairs are neighbours (interleaved); lanes beyond the rotary part own 16 consecutive
// elements and never rotate.
template <int DT, int FMT, bool DENSE, bool VAR, bool REUSE, typename Segs>
__global__ __launch_bounds__(kThreads) void k_place(PlaceP p, Segs segs)
{
    constexpr int U = FMT == KDN_FMT_RAW_BF16 ? 2 : 4;
    constexpr int W = FMT == KDN_FMT_RAW_BF16 ? 4 : FMT == KDN_FMT_INT8_ROWSCALE ? 2 : 1; // 32-bit words per 8 stored elements
    constexpr int NS = FMT == KDN_FMT_INT4_GROUP32 ? 2 : 1;                                // scales per item
    const int D = DT ? DT : p.c.D;
    const int half = D >> 1;
    const int R = D >> 4;
    const int LOGP = DT ? log2_ceil(DT >> 4) : log2_ceil(R);
    const int P = 1 << LOGP;
    const int H = p.c.H, G = p.c.G, bs = p.c.bs;
    const int L2 = 2 * p.c.L;

    const Seg &sg = segs.at(blockIdx.y);
    const int S = sg.S, T = sg.T;
    const int piece = blockIdx.x / L2;
    const int ls = blockIdx.x - piece * L2;
    const int gi = S / G + piece;
    const int tok_lo = max(S, gi * G);
    const int tok_hi = min(S + T, (gi + 1) * G);
    if (tok_lo >= tok_hi)
        return;
    const int blk = sg.bt[tok_lo / bs];
    const int slot0 = tok_lo % bs;
    uint16_t *tile = ((ls & 1) ? p.c.v : p.c.k) + (int64_t)(p.layer0 + (ls >> 1)) * p.c.layer_stride
                     + (int64_t)blk * p.c.block_stride + (int64_t)slot0 * p.c.token_stride;
    const int Tp = sg.Tp;
    const int64_t row_base = ((int64_t)ls * Tp + sg.tok0 + (tok_lo - S)) * H;
    const int64_t total_rows = (int64_t)p.c.L * 2 * Tp * H;
    const int n_items = ((tok_hi - tok_lo) * H) << LOGP;
    const uint8_t *data = sg.data + ((row_base * D * W) >> 1); // first stored row of this tile
    // int8: one scale per row after the codes; int4: D/32 scales per row after the codes
    const int spr = FMT == KDN_FMT_INT4_GROUP32 ? D >> 5 : 1;
    const float *scales = reinterpret_cast<const float *>(sg.data + ((total_rows * D * W) >> 1)) + row_base * spr;
    const bool rotate = (ls & 1) == 0 && sg.rope_row >= 0;

    const int sub = threadIdx.x & (P - 1);
    // element offsets, within the row, of the two 8-element vectors this lane owns
    int lo_off = sub * 8, hi_off = half + sub * 8;
    bool rot_lane = true, interleaved = false;
    if (VAR) {
        const int rl = p.rot >> 4; // lanes of the rotary part
        interleaved = p.pairing == KDN_ROPE_INTERLEAVED;
        rot_lane = sub < rl;
        if (interleaved) {
            lo_off = sub * 16;
            hi_off = lo_off + 8;
        } else if (rot_lane) {
            hi_off = (p.rot >> 1) + sub * 8;
        } else {
            lo_off = p.rot + (sub - rl) * 16;
            hi_off = lo_off + 8;
        }
    }
    const int rhalf = VAR ? p.rot >> 1 : half; // entries of a cos/sin row
    __shared__ f32x2 s_cs[kMaxHeadDim / 2];
    f32x2 cs[8];
    if (rotate) {
        const f32x2 *row = p.rope + (int64_t)sg.rope_row * rhalf;
        for (int i = threadIdx.x; i < rhalf; i += kThreads)
            s_cs[i] = row[i];
        __syncthreads();
        if (sub < R && rot_lane) {
#pragma unroll
            for (int e = 0; e < 8; ++e)
                cs[e] = s_cs[sub * 8 + e];
        }
    }
    if (sub >= R)
        return;
    const bool rotate_lane = rotate && rot_lane;

    for (int it0 = threadIdx.x; it0 < n_items; it0 += kThreads * U) {
        uint32_t lo[U][W], hi[U][W];
        float sc[U][NS];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int it = it0 + u * kThreads;
            if (it < n_items) {
                const int r = it >> LOGP;
                const uint8_t *src = data + (((uint32_t)(r * D + lo_off) * W) >> 1);
                const uint8_t *src_hi = data + (((uint32_t)(r * D + hi_off) * W) >> 1);
                if (FMT == KDN_FMT_INT4_GROUP32) {
                    lo[u][0] = load_stored<uint32_t, REUSE>(src);
                    hi[u][0] = load_stored<uint32_t, REUSE>(src_hi);
                    sc[u][0] = scales[r * spr + (lo_off >> 5)];
                    sc[u][NS - 1] = scales[r * spr + (hi_off >> 5)];
                } else if (FMT == KDN_FMT_RAW_BF16) {
                    const u32x4 l4 = load_stored<u32x4, REUSE>(src);
                    const u32x4 h4 = load_stored<u32x4, REUSE>(src_hi);
#pragma unroll
                    for (int w = 0; w < W; ++w) {
                        lo[u][w] = l4[w];
                        hi[u][w] = h4[w];
                    }
                } else {
                    const u32x2 l2 = load_stored<u32x2, REUSE>(src);
                    const u32x2 h2 = load_stored<u32x2, REUSE>(src_hi);
#pragma unroll
                    for (int w = 0; w < W; ++w) {
                        lo[u][w] = l2[w & 1];
                        hi[u][w] = h2[w & 1];
                    }
                    sc[u][0] = scales[r];
                }
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int it = it0 + u * kThreads;
            if (it >= n_items)
                continue;
            const int r = it >> LOGP;
            uint16_t *dst; // the row's first element
            if (DENSE) {
                dst = tile + (uint32_t)(r * D);
            } else {
                const int tok = r / H, h = r - tok * H;
                dst = tile + (int64_t)tok * p.c.token_stride + (int64_t)h * p.c.head_stride;
            }
            u32x4 olo, ohi;
            if (FMT == KDN_FMT_RAW_BF16 && !rotate_lane) { // bit copy
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    olo[w] = lo[u][w % W];
                    ohi[w] = hi[u][w % W];
                }
            } else {
                float a[8], b[8];
                if (FMT == KDN_FMT_RAW_BF16) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        a[2 * e] = bf16_lo(lo[u][e % W]);
                        a[2 * e + 1] = bf16_hi(lo[u][e % W]);
                        b[2 * e] = bf16_lo(hi[u][e % W]);
                        b[2 * e + 1] = bf16_hi(hi[u][e % W]);
                    }
                } else if (FMT == KDN_FMT_INT4_GROUP32) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        a[e] = (float)((int32_t)(lo[u][0] << (28 - 4 * e)) >> 28) * sc[u][0];
                        b[e] = (float)((int32_t)(hi[u][0] << (28 - 4 * e)) >> 28) * sc[u][NS - 1];
                    }
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        a[e] = code_f32(lo[u][(e >> 2) % W], e & 3) * sc[u][0];
                        b[e] = code_f32(hi[u][(e >> 2) % W], e & 3) * sc[u][0];
                    }
                }
                if (VAR && rotate_lane && interleaved) {
                    // pairs are neighbours: (a0,a1)..(a6,a7) take cs[0..3], (b0,b1).. cs[4..7]
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float c0 = cs[e].x, s0 = cs[e].y, c1 = cs[4 + e].x, s1 = cs[4 + e].y;
                        const float x0 = a[2 * e], y0 = a[2 * e + 1], x1 = b[2 * e], y1 = b[2 * e + 1];
                        const float x0c = x0 * c0, y0c = y0 * c0, x1c = x1 * c1, y1c = y1 * c1;
                        a[2 * e] = __builtin_fmaf(-y0, s0, x0c);
                        a[2 * e + 1] = __builtin_fmaf(x0, s0, y0c);
                        b[2 * e] = __builtin_fmaf(-y1, s1, x1c);
                        b[2 * e + 1] = __builtin_fmaf(x1, s1, y1c);
                    }
                } else if (rotate_lane) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const float c = cs[e].x, s = cs[e].y;
                        const float ac = a[e] * c, bc = b[e] * c;
                        const float l = __builtin_fmaf(-b[e], s, ac);
                        const float h = __builtin_fmaf(a[e], s, bc);
                        a[e] = l;
                        b[e] = h;
                    }
                }
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    olo[w] = pack_bf16(a[2 * w], a[2 * w + 1]);
                    ohi[w] = pack_bf16(b[2 * w], b[2 * w + 1]);
                }
            }
            __builtin_nontemporal_store(olo, reinterpret_cast<u32x4 *>(dst + lo_off));
            __builtin_nontemporal_store(ohi, reinterpret_cast<u32x4 *>(dst + hi_off));
        }
    }
}

// patch: rows [L][2][n][H][D] replace the rows of n request tokens (bit copy).
// One workgroup per (token, layer, side); a token outside the table is skipped.
struct PatchP {
    CacheP c;
    const uint16_t *rows;
    const int32_t *tokens;
    const int32_t *bt;
    int32_t n, limit;
};

__global__ __launch_bounds__(kThreads) void k_patch(PatchP p)
{
    const int L2 = 2 * p.c.L;
    const int i = blockIdx.x / L2;
    const int ls = blockIdx.x - i * L2;
    const int tok = p.tokens[i];
    if (tok < 0 || tok >= p.limit)
        return;
    const int blk = p.bt[tok / p.c.bs];
    const int slot = tok % p.c.bs;
    uint16_t *dst = ((ls & 1) ? p.c.v : p.c.k) + (int64_t)(ls >> 1) * p.c.layer_stride
                    + (int64_t)blk * p.c.block_stride + (int64_t)slot * p.c.token_stride;
    const int D = p.c.D, H = p.c.H;
    const uint16_t *src = p.rows + ((int64_t)ls * p.n + i) * H * D;
    const int vec_per_row = D >> 3;
    for (int v = threadIdx.x; v < H * vec_per_row; v += kThreads) {
        const int h = v / vec_per_row, j = (v - h * vec_per_row) * 8;
        const u32x4 w = *reinterpret_cast<const u32x4 *>(src + (int64_t)h * D + j);
        *reinterpret_cast<u32x4 *>(dst + (int64_t)h * p.c.head_stride + j) = w;
    }
}

__global__ void k_f32_to_bf16(const float *__restrict__ in, uint16_t *__restrict__ out, uint64_t n)
{
    const uint64_t pairs = n >> 1;
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < pairs; i += stride) {
        const f32x2 v = reinterpret_cast<const f32x2 *>(in)[i];
        reinterpret_cast<uint32_t *>(out)[i] = pack_bf16(v.x, v.y);
    }
    if ((n & 1) && blockIdx.x == 0 && threadIdx.x == 0)
        out[n - 1] = (uint16_t)pack_bf16(in[n - 1], 0.0f);
}

// flags: bit 0 = id out of range, bit 1 = id seen twice
__global__ void k_validate(const int32_t *bt, int32_t n, int32_t num_blocks, uint32_t *seen,
                           uint32_t *flags)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n)
        return;
    const int32_t id = bt[i];
    if (id < 0 || id >= num_blocks) {
        atomicOr(flags, 1u);
        return;
    }
    if (atomicAdd(&seen[id], 1u) != 0)
        atomicOr(flags, 2u);
}

// ---------------------------------------------------------------------------------
// host planner

// Resolved RoPE variant of one call: frequencies either derived from `base` or given.
struct RopeSpec {
    double base = 0.0;
    std::vector<double> freq; // rot/2 explicit frequencies, empty: base^(-2j/rot)
    int32_t rot = 0;
    int32_t pairing = KDN_ROPE_HALF_SPLIT;
};

// cos/sin rows of one (frequencies, rot) pair, one row per offset seen so far
struct RopeTable {
    f32x2 *dev = nullptr;
    double base = 0.0;
    std::vector<double> freq;
    int32_t rot = 0;
    std::unordered_map<int32_t, int32_t> row_of;
};

struct DeviceState {
    std::vector<RopeTable> rope;
    uint8_t *seg_dev = nullptr;                   // kSegSlots * kSegSlotBytes
    uint8_t *seg_host = nullptr;                  // pinned mirror
    hipEvent_t seg_done[kSegSlots] = {};
    bool seg_used[kSegSlots] = {};
    int next_slot = 0;
    // streaming of host-resident chunks: a copy stream and, per half of the caller's
    // staging buffer, "filled" and "drained" events
    hipStream_t copy_stream = nullptr;
    hipEvent_t filled[2] = {};
    hipEvent_t drained[2] = {};
    bool drained_valid[2] = {};
};

std::mutex g_mu;
std::unordered_map<int, DeviceState> g_dev;

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

kdn_status check_shape(int32_t L, int32_t H, int32_t D)
{
    if (L <= 0 || H <= 0 || D <= 0 || L > 32767)
        return KDN_EINVAL;
    if (D % 16 != 0 || D > kMaxHeadDim)
        return KDN_EUNSUPPORTED;
    return KDN_OK;
}

kdn_status check_cache(const kdn_cache_desc *c)
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

bool known_format(int32_t fmt)
{
    return fmt == KDN_FMT_RAW_BF16 || fmt == KDN_FMT_INT8_ROWSCALE || fmt == KDN_FMT_INT4_GROUP32;
}

kdn_status check_chunk(const kdn_chunk *ch, const kdn_cache_desc *c)
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

CacheP make_cache_p(const kdn_cache_desc *c)
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
    // token group: a whole block when it is small, else 16-token pieces of it
    p.G = (c->block_size > 16 && c->block_size % 16 == 0) ? 16 : c->block_size;
    p.dense = (c->head_stride == c->head_dim
               && c->token_stride == (int64_t)c->num_kv_heads * c->head_dim);
    return p;
}

// number of token groups touched by tokens [s, s+t)
int64_t groups_spanned(int64_t s, int64_t t, int32_t G) { return (s + t - 1) / G - s / G + 1; }

kdn_status hip_status(hipError_t e) { return e == hipSuccess ? KDN_OK : KDN_EDEVICE; }

DeviceState *device_state(int *dev_out)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess)
        return nullptr;
    if (dev_out)
        *dev_out = dev;
    return &g_dev[dev];
}

// Validates a caller's RoPE variant for head_dim D.  NULL selects the default
// (all of D rotary, half-split pairs, frequencies from `base`).
kdn_status resolve_spec(const kdn_rope_spec *in, double base, int32_t D, RopeSpec &out)
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
// zero offset).  New rows are computed in double and uploaded before returning.
kdn_status rope_rows(DeviceState *ds, const RopeSpec &spec, const int32_t *offsets, int32_t n,
                     int32_t *rows, const f32x2 **table)
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
    {
        std::unordered_map<int32_t, int32_t> distinct;
        for (int32_t i = 0; i < n; ++i)
            if (offsets[i] != 0)
                distinct.emplace(offsets[i], 0);
        if ((int32_t)distinct.size() > kRopeRowsCap)
            return KDN_ESIZE;
    }
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
    const int32_t half = spec.rot / 2;
    if (!rt.dev
        && hipMalloc(reinterpret_cast<void **>(&rt.dev), (size_t)kRopeRowsCap * half * sizeof(f32x2))
               != hipSuccess)
        return KDN_EDEVICE;
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
            continue;
        }
        if ((int32_t)rt.row_of.size() >= kRopeRowsCap) {
            // table full: wait until nothing can still read it, then start over
            if (hipDeviceSynchronize() != hipSuccess)
                return KDN_EDEVICE;
            rt.row_of.clear();
            for (int32_t k = 0; k < i; ++k) // rows handed out earlier in this call are gone
                if (offsets[k] != 0)
                    rows[k] = -2;
        }
        for (int32_t j = 0; j < half; ++j) {
            const double theta = spec.freq.empty() ? std::pow(spec.base, -(double)(2 * j) / (double)spec.rot)
                                                   : spec.freq[(size_t)j];
            const double phi = (double)d * theta;
            row[2 * j] = (float)std::cos(phi);
            row[2 * j + 1] = (float)std::sin(phi);
        }
        const int32_t r = (int32_t)rt.row_of.size();
        if (hipMemcpy(rt.dev + (size_t)r * half, row.data(), row.size() * sizeof(float),
                      hipMemcpyHostToDevice)
            != hipSuccess)
            return KDN_EDEVICE;
        rt.row_of.emplace(d, r);
        rows[i] = r;
    }
    for (int32_t i = 0; i < n; ++i)
        if (rows[i] == -2) // only after a table reset inside this call
            return rope_rows(ds, spec, offsets, n, rows, table);
    *table = rt.dev;
    return KDN_OK;
}

template <int DT, int FMT, int P>
void launch_store(const StoreP &p, dim3 grid, hipStream_t st)
{
    if (p.c.dense && !p.tokens)
        hipLaunchKernelGGL((k_store<DT, FMT, P, true>), grid, dim3(kThreads), 0, st, p);
    else
        hipLaunchKernelGGL((k_store<DT, FMT, P, false>), grid, dim3(kThreads), 0, st, p);
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
    if (segs_dev) {
        SegsDevice sd{segs_dev};
        hipLaunchKernelGGL((k_place<DT, FMT, DENSE, VAR, REUSE, SegsDevice>), grid, dim3(kThreads), 0, st, p, sd);
    } else {
        SegsInline si;
        std::memset(&si, 0, sizeof si);
        std::memcpy(si.s, segs, (size_t)n * sizeof(Seg));
        hipLaunchKernelGGL((k_place<DT, FMT, DENSE, VAR, REUSE, SegsInline>), grid, dim3(kThreads), 0, st, p, si);
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

template <int FMT>
void launch_place_d(const PlaceP &p, const Seg *segs, int32_t n, const Seg *segs_dev, dim3 grid,
                    hipStream_t st)
{
    switch (p.c.D) {
    case 64: launch_place<64, FMT>(p, segs, n, segs_dev, grid, st); break;
    case 128: launch_place<128, FMT>(p, segs, n, segs_dev, grid, st); break;
    default: launch_place<0, FMT>(p, segs, n, segs_dev, grid, st); break;
    }
}

// Enqueue the placement of `segs` (all of one format).  Up to kMaxInlineSegs travel
// in the kernel arguments; more go through a ring of device tables.
kdn_status place_segments(DeviceState *ds, const PlaceP &p, int32_t fmt, const std::vector<Seg> &segs,
                          hipStream_t st)
{
    if (segs.empty())
        return KDN_OK;
    if (segs.size() > 65535 || segs.size() * sizeof(Seg) > kSegSlotBytes)
        return KDN_ESIZE;
    int64_t max_groups = 0;
    for (const Seg &s : segs)
        max_groups = std::max(max_groups, groups_spanned(s.S, s.T, p.c.G));
    if (max_groups * 2 * p.c.L > 0x7fffffff / kThreads)
        return KDN_ESIZE;
    dim3 grid((unsigned)(max_groups * 2 * p.c.L), (unsigned)segs.size(), 1);

    const Seg *segs_dev = nullptr;
    int slot = -1;
    if ((int)segs.size() > kMaxInlineSegs) {
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

kdn_status compose_impl(const kdn_request *reqs, int32_t n_reqs, const kdn_cache_desc *cache,
                        double rope_base, const kdn_rope_spec *variant, void *stream)
{
    if (!reqs || n_reqs <= 0)
        return KDN_EINVAL;
    kdn_status st = check_cache(cache);
    if (st != KDN_OK)
        return st;
    RopeSpec spec;
    st = resolve_spec(variant, rope_base, cache->head_dim, spec);
    if (st != KDN_OK)
        return st;
    std::vector<int32_t> offs;
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
            offs.push_back(q.offsets[i]);
        }
        if (total > (int64_t)q.table_len * cache->block_size)
            return KDN_ERANGE;
    }
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
    std::vector<Seg> segs[3];
    size_t k = 0;
    for (int32_t r = 0; r < n_reqs; ++r) {
        const kdn_request &q = reqs[r];
        int32_t S = q.dest_token_start;
        for (int32_t i = 0; i < q.n_chunks; ++i, ++k) {
            const kdn_chunk &ch = q.chunks[i];
            Seg s;
            s.data = static_cast<const uint8_t *>(ch.data);
            s.bt = q.block_table_dev;
            s.Tp = ch.parent_tokens;
            s.tok0 = ch.token_start;
            s.T = ch.num_tokens;
            s.S = S;
            s.rope_row = rows[k];
            s.pad = 0;
            segs[ch.fmt].push_back(s);
            S += ch.num_tokens;
        }
    }
    for (int f = 0; f < 3; ++f) {
        // Segments that read the same stored rows run back to back, so that a popular
        // chunk is fetched from HBM once and from the last-level cache afterwards.
        p.reuse = 0;
        if (n_reqs > 1) {
            std::stable_sort(segs[f].begin(), segs[f].end(), [](const Seg &a, const Seg &b) {
                return a.data != b.data ? a.data < b.data : a.tok0 < b.tok0;
            });
            for (size_t i = 1; i < segs[f].size(); ++i) {
                const Seg &a = segs[f][i - 1], &b = segs[f][i];
                if (a.data == b.data && b.tok0 < a.tok0 + a.T)
                    p.reuse = 1;
            }
        }
        st = place_segments(ds, p, f, segs[f], static_cast<hipStream_t>(stream));
        if (st != KDN_OK)
            return st;
    }
    return KDN_OK;
}

// Views of the same host buffer are staged once: the token range [lo, hi) that the
// views of one buffer span crosses the link as one copy per stage.
struct HostParent {
    const uint8_t *data;
    int32_t fmt, L, H, D, Tp, lo, hi;
};

void plan_host_parents(const kdn_chunk *chunks, int32_t n, std::vector<HostParent> &parents,
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
            parents.push_back({static_cast<const uint8_t *>(ch.data), ch.fmt, ch.num_layers, ch.num_kv_heads,
                               ch.head_dim, ch.parent_tokens, ch.token_start, ch.token_start + ch.num_tokens});
        parents[k].lo = std::min(parents[k].lo, ch.token_start);
        parents[k].hi = std::max(parents[k].hi, ch.token_start + ch.num_tokens);
        parent_of[(size_t)i] = (int32_t)k;
    }
}

} // namespace

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
    if (fmt == KDN_FMT_INT8_ROWSCALE)
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

static kdn_status store_impl(const kdn_cache_desc *cache, const int32_t *block_table_dev,
                             int32_t table_len, int32_t token_start, int32_t num_tokens,
                             const int32_t *tokens_dev, kdn_chunk *out, void *stream)
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
    if (!tokens_dev && (int64_t)token_start + num_tokens > limit)
        return KDN_ERANGE;
    const uint64_t need = kdn_chunk_bytes(cache->num_layers, cache->num_kv_heads, cache->head_dim,
                                          num_tokens, out->fmt);
    if (out->bytes < need)
        return KDN_ESIZE;
    StoreP p;
    p.c = make_cache_p(cache);
    p.bt = block_table_dev;
    p.out = static_cast<uint8_t *>(out->data);
    p.t0 = token_start;
    p.T = num_tokens;
    p.tokens = tokens_dev;
    p.limit = (int32_t)std::min<int64_t>(limit, 0x7fffffff);
    if (tokens_dev)
        p.c.G = 16; // list entries need no block alignment
    const int64_t groups = groups_spanned(token_start, num_tokens, p.c.G);
    if (groups * 2 * p.c.L > 0x7fffffff / kThreads)
        return KDN_ESIZE;
    dim3 grid((unsigned)(groups * 2 * p.c.L), 1, 1);
    hipStream_t hs = static_cast<hipStream_t>(stream);
    if (out->fmt == KDN_FMT_RAW_BF16)
        launch_store_d<KDN_FMT_RAW_BF16>(p, grid, hs);
    else if (out->fmt == KDN_FMT_INT8_ROWSCALE)
        launch_store_d<KDN_FMT_INT8_ROWSCALE>(p, grid, hs);
    else
        launch_store_d<KDN_FMT_INT4_GROUP32>(p, grid, hs);
    st = hip_status(hipGetLastError());
    if (st != KDN_OK)
        return st;
    out->num_layers = cache->num_layers;
    out->num_kv_heads = cache->num_kv_heads;
    out->head_dim = cache->head_dim;
    out->parent_tokens = num_tokens;
    out->token_start = 0;
    out->num_tokens = num_tokens;
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

kdn_status kdn_compose_from_host(const kdn_chunk *chunks, const int32_t *offsets, int32_t n_chunks,
                                 const kdn_cache_desc *cache, const int32_t *block_table_dev,
                                 int32_t table_len, int32_t dest_token_start, double rope_base,
                                 void *staging_dev, uint64_t staging_bytes, int32_t layers_per_stage,
                                 void *stream)
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
    if (total > (int64_t)table_len * cache->block_size)
        return KDN_ERANGE;
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
    if (!ds->copy_stream) {
        if (hipStreamCreateWithFlags(&ds->copy_stream, hipStreamNonBlocking) != hipSuccess)
            return KDN_EDEVICE;
        for (int b = 0; b < 2; ++b)
            if (hipEventCreateWithFlags(&ds->filled[b], hipEventDisableTiming) != hipSuccess
                || hipEventCreateWithFlags(&ds->drained[b], hipEventDisableTiming) != hipSuccess)
                return KDN_EDEVICE;
    }
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

    const int32_t L = cache->num_layers, H = cache->num_kv_heads, D = cache->head_dim;
    uint8_t *staging = static_cast<uint8_t *>(staging_dev);
    const uint64_t half_bytes = need / 2;
    std::vector<uint8_t *> staged(parents.size());
    int stage_no = 0;
    for (int32_t l0 = 0; l0 < L; l0 += layers_per_stage, ++stage_no) {
        const int32_t Lg = std::min(layers_per_stage, L - l0);
        const int b = stage_no & 1;
        uint8_t *buf = staging + (uint64_t)b * half_bytes;
        // the copy may overwrite this half only after the kernel that last read it
        if (ds->drained_valid[b] && hipStreamWaitEvent(ds->copy_stream, ds->drained[b], 0) != hipSuccess)
            return KDN_EDEVICE;
        uint64_t at = 0;
        for (size_t k = 0; k < parents.size(); ++k) {
            const HostParent &hp = parents[k];
            const int32_t Tu = hp.hi - hp.lo, Tp = hp.Tp;
            const uint64_t esz = hp.fmt == KDN_FMT_RAW_BF16 ? 2 : 1;
            uint8_t *dst = buf + at;
            staged[k] = dst;
            // rows of layers [l0, l0+Lg), both sides, tokens [lo, hi) of this host buffer:
            // 2*Lg planes of Tu*H*D elements, Tp*H*D apart
            const uint64_t w_codes = (uint64_t)Tu * H * D * esz, pitch_codes = (uint64_t)Tp * H * D * esz;
            const uint8_t *src_codes = hp.data + ((uint64_t)l0 * 2 * Tp + hp.lo) * H * D * esz;
            hipError_t e;
            if (Tu == Tp)
                e = hipMemcpyAsync(dst, src_codes, w_codes * 2 * Lg, hipMemcpyHostToDevice, ds->copy_stream);
            else
                e = hipMemcpy2DAsync(dst, w_codes, src_codes, pitch_codes, w_codes, (size_t)2 * Lg,
                                     hipMemcpyHostToDevice, ds->copy_stream);
            if (e != hipSuccess)
                return KDN_EDEVICE;
            if (hp.fmt == KDN_FMT_INT8_ROWSCALE) {
                const uint64_t w_sc = (uint64_t)Tu * H * 4, pitch_sc = (uint64_t)Tp * H * 4;
                const uint8_t *src_sc = hp.data + (uint64_t)L * 2 * Tp * H * D
                                        + ((uint64_t)l0 * 2 * Tp + hp.lo) * H * 4;
                uint8_t *dst_sc = dst + w_codes * 2 * Lg;
                if (Tu == Tp)
                    e = hipMemcpyAsync(dst_sc, src_sc, w_sc * 2 * Lg, hipMemcpyHostToDevice, ds->copy_stream);
                else
                    e = hipMemcpy2DAsync(dst_sc, w_sc, src_sc, pitch_sc, w_sc, (size_t)2 * Lg,
                                         hipMemcpyHostToDevice, ds->copy_stream);
                if (e != hipSuccess)
                    return KDN_EDEVICE;
            }
            const uint64_t bytes = kdn_chunk_bytes(Lg, H, D, Tu, hp.fmt);
            at += (bytes + 255) & ~(uint64_t)255;
        }
        std::vector<Seg> segs[3];
        int32_t S = dest_token_start;
        for (int32_t i = 0; i < n_chunks; ++i) {
            const kdn_chunk &ch = chunks[i];
            const HostParent &hp = parents[parent_of[i]];
            Seg s;
            s.data = staged[parent_of[i]];
            s.bt = block_table_dev;
            s.Tp = hp.hi - hp.lo;
            s.tok0 = ch.token_start - hp.lo;
            s.T = ch.num_tokens;
            s.S = S;
            s.rope_row = rows[i];
            s.pad = 0;
            segs[ch.fmt].push_back(s);
            S += ch.num_tokens;
        }
        if (hipEventRecord(ds->filled[b], ds->copy_stream) != hipSuccess
            || hipStreamWaitEvent(user, ds->filled[b], 0) != hipSuccess)
            return KDN_EDEVICE;
        p.c.L = Lg;
        p.layer0 = l0;
        for (int f = 0; f < 3; ++f) {
            st = place_segments(ds, p, f, segs[f], user);
            if (st != KDN_OK)
                return st;
        }
        if (hipEventRecord(ds->drained[b], user) != hipSuccess)
            return KDN_EDEVICE;
        ds->drained_valid[b] = true;
    }
    return KDN_OK;
}

kdn_status kdn_rope_prepare(double rope_base, int32_t head_dim, const int32_t *offsets, int32_t n)
{
    if (!offsets || n <= 0)
        return KDN_EINVAL;
    kdn_status st = check_shape(1, 1, head_dim);
    if (st != KDN_OK)
        return st;
    std::lock_guard<std::mutex> lock(g_mu);
    DeviceState *ds = device_state(nullptr);
    if (!ds)
        return KDN_EDEVICE;
    std::vector<int32_t> rows((size_t)n);
    const f32x2 *table;
    RopeSpec spec;
    st = resolve_spec(nullptr, rope_base, head_dim, spec);
    if (st != KDN_OK)
        return st;
    return rope_rows(ds, spec, offsets, n, rows.data(), &table);
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
        if (ds.copy_stream) {
            (void)hipStreamDestroy(ds.copy_stream);
            for (int b = 0; b < 2; ++b) {
                (void)hipEventDestroy(ds.filled[b]);
                (void)hipEventDestroy(ds.drained[b]);
            }
        }
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
    }
    return "unknown status";
}

const char *kdn_version(void) { return "kdn-gfx950 0.1"; }

} // extern "C"
