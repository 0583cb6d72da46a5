// Device side of the KDN library for MI355X (gfx950): launch parameters and the store,
// place, patch and utility kernels.  Included by kdn.hip only.
//
// store (Sec. 3.2, interface (i)), load (interface (ii), decompression on the GPU,
// Sec. 3.1) and compose (blending module, Sec. 3.1) all stream rows of head_dim
// elements between two layouts; none is a contraction, so the kernels are organised
// around 64-wide wavefronts issuing full-width global loads and stores, and the per-row
// reductions use cross-lane operations.
//
// Work decomposition (both directions): a workgroup owns one (layer, K|V, token group)
// tile.  A token group is a run of at most G consecutive request tokens that lies inside
// one paged block, so a tile is contiguous in the paged cache (for the dense layout) and
// contiguous in the stored chunk.  Blocks of one to three tokens are the exception: there
// a group is 16 tokens and every row looks its own block up.  The host sizes the workgroup
// to the tile (whole wavefronts, at most kThreads), so the kernels stride by blockDim.x.
#ifndef KDN_KERNELS_H
#define KDN_KERNELS_H

#include <hip/hip_runtime.h>

#include <cstdint>

#include "kdn.h"

namespace kdn_impl {

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
    int32_t next;     // record of another view of exactly these stored rows, placed by the same workgroups
                      // right after this one (its tiles cut the rows the same way); 0: none (record 0
                      // always has workgroups of its own)
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
    int32_t G;         // tokens per group; divides bs unless per_token
    int32_t dense;     // head_stride == D and token_stride == H*D (and one block per group)
    int32_t per_token; // blocks smaller than a group: every row resolves its own token's block
};

struct StoreP {
    CacheP c;
    const int32_t *bt;
    uint8_t *out;
    int32_t t0, T;
    const int32_t *tokens; // token-list store: row t holds request token tokens[t]; else NULL
    int32_t limit;         // request tokens the block table covers (list entries are clamped to it)
    int32_t layer0;        // cache layer that stored layer 0 comes from (c.L layers are stored)
    uint32_t tiles_x;      // tiles along x; a launch with fewer workgroups strides over them
};

struct PlaceP {
    CacheP c;          // c.L counts the layers the stored rows hold (and the grid covers)
    const f32x2 *rope; // [rows][rot/2] (cos, sin)
    int32_t layer0;    // cache layer that stored layer 0 goes to
    int32_t rot;       // rotary leading dimensions (head_dim unless partial rotary)
    int32_t pairing;   // kdn_rope_pairing
    int32_t reuse;     // some stored rows are read by more than one segment: let them stay cached
    uint32_t tiles_x;  // tiles along x; a launch with fewer workgroups strides over them
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

// value of the e4m3 code in byte `byte` of w (exact)
__device__ __forceinline__ float fp8_f32(uint32_t w, int byte)
{
    switch (byte) {
    case 0: return __builtin_amdgcn_cvt_f32_fp8((int)w, 0);
    case 1: return __builtin_amdgcn_cvt_f32_fp8((int)w, 1);
    case 2: return __builtin_amdgcn_cvt_f32_fp8((int)w, 2);
    default: return __builtin_amdgcn_cvt_f32_fp8((int)w, 3);
    }
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
// Grid: x = (layer, side) * groups + group.

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

// e4m3 codes of 4 values: the hardware conversion rounds to nearest even; the products
// never leave the finite range (|x*inv| <= 448(1 + 2^-24), which still rounds to 448).
__device__ __forceinline__ uint32_t quantise4_fp8(uint32_t w0, uint32_t w1, float inv)
{
    int v = __builtin_amdgcn_cvt_pk_fp8_f32(bf16_lo(w0) * inv, bf16_hi(w0) * inv, 0, false);
    v = __builtin_amdgcn_cvt_pk_fp8_f32(bf16_lo(w1) * inv, bf16_hi(w1) * inv, v, true);
    return (uint32_t)v;
}

template <int DT, int FMT, int P, bool DENSE>
__device__ __forceinline__ void store_tile(const StoreP &p, const uint32_t bx)
{
    constexpr int U = kStoreU;
    constexpr int LOGP = log2_ceil(P);
    // with at least 8 lanes per row the 2*U divisions of a batch are spread over the
    // lanes of the row's group (one division sequence per batch instead of 2*U)
    constexpr bool SPREAD = P >= 8 && U == 4;
    // largest code magnitude, and the smallest amax whose reciprocal scale is finite
    constexpr float QMAX = FMT == KDN_FMT_FP8_ROWSCALE ? 448.0f : 127.0f;
    constexpr float TINY = FMT == KDN_FMT_FP8_ROWSCALE ? 0x1p-119f : 0x1p-121f;
    const int D = DT ? DT : p.c.D;
    const int R = D >> 3;
    const int H = p.c.H, G = p.c.G, bs = p.c.bs;
    const int L2 = 2 * p.c.L;

    // group-fastest order: neighbouring workgroups write neighbouring rows of the chunk
    const int n_groups = p.tiles_x / L2;
    const int ls = bx / n_groups;
    const int piece = bx - ls * n_groups;
    const int gi = p.t0 / G + piece;
    const int tok_lo = max(p.t0, gi * G);
    const int tok_hi = min(p.t0 + p.T, (gi + 1) * G);
    if (tok_lo >= tok_hi)
        return;
    // a token list, or blocks smaller than the group (strided instantiation only): every
    // row resolves its token by itself
    const bool listed = !DENSE && (p.tokens != nullptr || p.c.per_token);
    const uint16_t *plane = ((ls & 1) ? p.c.v : p.c.k) + (int64_t)(p.layer0 + (ls >> 1)) * p.c.layer_stride;
    const int blk = listed ? 0 : p.bt[tok_lo / bs];
    const int slot0 = listed ? 0 : tok_lo % bs;
    const uint16_t *tile = plane + (int64_t)blk * p.c.block_stride + (int64_t)slot0 * p.c.token_stride;
    const int64_t row_base = ((int64_t)ls * p.T + (tok_lo - p.t0)) * H;
    const int n_items = ((tok_hi - tok_lo) * H) << LOGP;
    const int64_t total_rows = (int64_t)p.c.L * 2 * p.T * H;
    constexpr int W = FMT == KDN_FMT_RAW_BF16 ? 4 : FMT == KDN_FMT_INT4_GROUP32 ? 1 : 2; // words per 8 stored elements
    const int spr = FMT == KDN_FMT_INT4_GROUP32 ? D >> 5 : 1;                              // scales per row
    uint8_t *codes = p.out + ((row_base * D * W) >> 1);
    float *scales = reinterpret_cast<float *>(p.out + ((total_rows * D * W) >> 1)) + row_base * spr;

    const int sub = threadIdx.x & (P - 1);
    const int lane = __lane_id();
    const int grp_addr = (lane & ~(P - 1)) << 2; // byte address of the group's first lane for bpermute
    const int NT = blockDim.x; // a small tile is launched with fewer wavefronts

    for (int base = 0; base < n_items; base += NT * U) {
        u32x4 w[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int it = base + u * NT + threadIdx.x;
            const int r = it >> LOGP;
            w[u] = u32x4{0, 0, 0, 0};
            if (it < n_items && sub < R) {
                const uint16_t *src;
                if (DENSE) {
                    src = tile + (uint32_t)(r * D + sub * 8);
                } else {
                    const int tok = r / H, h = r - tok * H;
                    if (listed) {
                        const int t = p.tokens ? min(max(p.tokens[tok_lo + tok], 0), p.limit - 1) : tok_lo + tok;
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
                const int it = base + u * NT + threadIdx.x;
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
            const int it_s = base + us * NT + threadIdx.x;
            if (it_s < n_items && sub < R)
                scales[(it_s >> LOGP) * spr + (sub >> 2)] = q_scale;
            float inv4[U];
            inv4[0] = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(q_inv), 0x00, 0xf, 0xf, true));
            inv4[1] = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(q_inv), 0x55, 0xf, 0xf, true));
            inv4[2] = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(q_inv), 0xAA, 0xf, 0xf, true));
            inv4[U - 1] = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(q_inv), 0xFF, 0xf, 0xf, true));
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int it = base + u * NT + threadIdx.x;
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
            const float q = (is_scale ? amax : QMAX) / (is_scale ? QMAX : amax);
            const float quot = amax >= TINY ? q : 0.0f;
#pragma unroll
            for (int u = 0; u < U; ++u)
                inv[u] = __int_as_float(__builtin_amdgcn_ds_bpermute(grp_addr + 4 * u, __float_as_int(quot)));
            const int it_s = base + us * NT + threadIdx.x; // same row as every lane of the group
            if (is_scale && sub < 8 && it_s < n_items)
                scales[it_s >> LOGP] = quot;
        } else {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const float amax = __uint_as_float(m[u] << 16);
                const bool keep = amax >= TINY;
                inv[u] = keep ? QMAX / amax : 0.0f;
                const int it = base + u * NT + threadIdx.x;
                if (sub == 0 && it < n_items)
                    scales[it >> LOGP] = keep ? amax / QMAX : 0.0f;
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int it = base + u * NT + threadIdx.x;
            const int r = it >> LOGP;
            if (it < n_items && sub < R) {
                u32x2 q;
                if (FMT == KDN_FMT_FP8_ROWSCALE) {
                    // a flushed row (inv == 0) stores code 0, not the -0 code of a negative element
                    const uint32_t live = inv[u] != 0.0f ? 0xffffffffu : 0u;
                    q = u32x2{quantise4_fp8(w[u][0], w[u][1], inv[u]) & live,
                              quantise4_fp8(w[u][2], w[u][3], inv[u]) & live};
                } else {
                    q = u32x2{quantise4(w[u][0], w[u][1], inv[u]), quantise4(w[u][2], w[u][3], inv[u])};
                }
                __builtin_nontemporal_store(q, reinterpret_cast<u32x2 *>(codes + (uint32_t)(r * D + sub * 8)));
            }
        }
    }
}

// One workgroup per tile; a launch capped below the tile count (chunks in host memory: a few
// workgroups keep the link busy and leave the rest of the device to other work) strides.
template <int DT, int FMT, int P, bool DENSE>
__global__ __launch_bounds__(kThreads) void k_store(StoreP p)
{
    store_tile<DT, FMT, P, DENSE>(p, blockIdx.x); // the common launch ends here
    for (uint32_t bx = blockIdx.x + gridDim.x; bx < p.tiles_x; bx += gridDim.x)
        store_tile<DT, FMT, P, DENSE>(p, bx);
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
// Serves head dims that are multiples of 128, where each of the two stores of a lane group
// fills whole 128-byte lines: raw bf16 and per-token block lookup at 128, everything at 256
// and 512; k_place_c below serves the others (the host planner holds the measurements).
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

// VAR selects the RoPE variants (partial rotary, interleaved pairs).  Every lane keeps the
// 8 + 8 ownership, so that a store instruction writes whole runs whatever the variant: a
// lane of the rotary part owns 8 elements of its lower half and the 8 at the same place of
// its upper half (half-split: these pair up; interleaved: each vector holds 4 neighbouring
// pairs of its own); the part behind the rotary one is split into halves the same way and
// never rotates.
template <int DT, int FMT, bool DENSE, bool VAR, bool REUSE>
__device__ __forceinline__ void place_tile(const PlaceP &p, const Seg &sg, const uint32_t bx)
{
    constexpr int U = FMT == KDN_FMT_RAW_BF16 ? 2 : 4;
    constexpr int W = FMT == KDN_FMT_RAW_BF16 ? 4 : FMT == KDN_FMT_INT4_GROUP32 ? 1 : 2; // 32-bit words per 8 stored elements
    constexpr int NS = FMT == KDN_FMT_INT4_GROUP32 ? 2 : 1;                                // scales per item
    const int D = DT ? DT : p.c.D;
    const int half = D >> 1;
    const int R = D >> 4;
    const int LOGP = DT ? log2_ceil(DT >> 4) : log2_ceil(R);
    const int P = 1 << LOGP;
    const int H = p.c.H, G = p.c.G, bs = p.c.bs;
    const int L2 = 2 * p.c.L;
    const int NT = blockDim.x; // a small tile is launched with fewer wavefronts

    const int S = sg.S, T = sg.T;
    const int piece = bx / L2;
    const int ls = bx - piece * L2;
    const int gi = S / G + piece;
    const int tok_lo = max(S, gi * G);
    const int tok_hi = min(S + T, (gi + 1) * G);
    if (tok_lo >= tok_hi)
        return;
    const int blk = sg.bt[tok_lo / bs];
    const int slot0 = tok_lo % bs;
    uint16_t *plane = ((ls & 1) ? p.c.v : p.c.k) + (int64_t)(p.layer0 + (ls >> 1)) * p.c.layer_stride;
    uint16_t *tile = plane + (int64_t)blk * p.c.block_stride + (int64_t)slot0 * p.c.token_stride;
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
        if (rot_lane) {
            hi_off = (p.rot >> 1) + sub * 8;
        } else { // the part behind the rotary one is split into halves the same way
            lo_off = p.rot + (sub - rl) * 8;
            hi_off = lo_off + ((D - p.rot) >> 1);
        }
    }
    const int rhalf = VAR ? p.rot >> 1 : half; // entries of a cos/sin row
    __shared__ f32x2 s_cs[kMaxHeadDim / 2];
    f32x2 cs[8];
    if (rotate) {
        const f32x2 *row = p.rope + (int64_t)sg.rope_row * rhalf;
        for (int i = threadIdx.x; i < rhalf; i += NT)
            s_cs[i] = row[i];
        __syncthreads();
        if (sub < R && rot_lane) {
            if (VAR && interleaved) {
                // each 8-element vector holds 4 whole pairs: pairs sub*4.. of the lower
                // half of the rotary part, and the same of its upper half
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    cs[e] = s_cs[sub * 4 + e];
                    cs[4 + e] = s_cs[(p.rot >> 2) + sub * 4 + e];
                }
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    cs[e] = s_cs[sub * 8 + e];
            }
        }
    }
    if (sub >= R)
        return;
    const bool rotate_lane = rotate && rot_lane;

    for (int it0 = threadIdx.x; it0 < n_items; it0 += NT * U) {
        uint32_t lo[U][W], hi[U][W];
        float sc[U][NS];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int it = it0 + u * NT;
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
            const int it = it0 + u * NT;
            if (it >= n_items)
                continue;
            const int r = it >> LOGP;
            uint16_t *dst; // the row's first element
            if (DENSE) {
                dst = tile + (uint32_t)(r * D);
            } else {
                const int tok = r / H, h = r - tok * H;
                if (p.c.per_token) {
                    const int t = tok_lo + tok;
                    dst = plane + (int64_t)sg.bt[t / bs] * p.c.block_stride + (int64_t)(t % bs) * p.c.token_stride
                          + (int64_t)h * p.c.head_stride;
                } else {
                    dst = tile + (int64_t)tok * p.c.token_stride + (int64_t)h * p.c.head_stride;
                }
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
                } else if (FMT == KDN_FMT_FP8_ROWSCALE) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        a[e] = fp8_f32(lo[u][(e >> 2) % W], e & 3) * sc[u][0];
                        b[e] = fp8_f32(hi[u][(e >> 2) % W], e & 3) * sc[u][0];
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

// One workgroup per tile, or fewer workgroups striding over the tiles (see k_store).  A row
// of the grid (blockIdx.y) is a view with workgroups of its own; the views chained behind it
// (Seg::next) read exactly the same stored rows, so the workgroup that has just read a tile
// places it again for each of them, through the caches, before it moves on: a chunk that
// many requests of a batch draw crosses the memory interface once.  The barrier between
// tiles keeps a fast wavefront from restaging the cos/sin row while a slow one still reads
// the previous tile's.
template <int DT, int FMT, bool DENSE, bool VAR, bool REUSE, typename Segs>
__global__ __launch_bounds__(kThreads) void k_place(PlaceP p, Segs segs)
{
    bool first = true;
    for (uint32_t bx = blockIdx.x; bx < p.tiles_x; bx += gridDim.x) { // the common launch has one tile per workgroup
        int at = blockIdx.y;
        do {
            if (!first)
                __syncthreads();
            first = false;
            const Seg &sg = segs.at(at);
            place_tile<DT, FMT, DENSE, VAR, REUSE>(p, sg, bx);
            at = sg.next;
        } while (at != 0);
    }
}

// the 8 values that the stored words of 8 consecutive elements stand for
template <int FMT>
__device__ __forceinline__ void dequantise8(const uint32_t *w, float scale, float *x)
{
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        if (FMT == KDN_FMT_RAW_BF16)
            x[e] = (e & 1) ? bf16_hi(w[e >> 1]) : bf16_lo(w[e >> 1]);
        else if (FMT == KDN_FMT_INT4_GROUP32)
            x[e] = (float)((int32_t)(w[0] << (28 - 4 * e)) >> 28) * scale;
        else if (FMT == KDN_FMT_FP8_ROWSCALE)
            x[e] = fp8_f32(w[e >> 2], e & 3) * scale;
        else
            x[e] = code_f32(w[e >> 2], e & 3) * scale;
    }
}

// place with row-contiguous ownership: for head dims where half a row is not a whole
// number of 128-byte lines (head_dim not a multiple of 128), and for the quantised forms at
// head_dim 128, where its loads (a wavefront reads 512 contiguous bytes of codes instead of
// 64-byte pieces of 8 rows) make it the faster one on pools that span the device memory.
// D/8 lanes own a row, 8 consecutive elements each, and a wavefront takes 64/(D/8) whole
// rows at a time, so every load and store instruction covers rows back to back.  A lane
// of a half-split rotary pair fetches the stored words of its partner, the lane rot/16
// places away, with ds_bpermute, dequantises both and forms its own 8 outputs:
// out = fma(partner, -+sin, own*cos), which is the pair rotation read from either side.
// Interleaved pairs lie inside a lane's own 8 elements.  All lanes stay active through
// the exchange; loads and stores are predicated instead.
// Grid as k_place.
// UQ: rows a lane of a quantised form keeps in flight: 8, or 4 for tiles of so few rows that
// a wavefront could not fill 8 (short rows: few or narrow heads) and is better off with the
// smaller register footprint, i.e. more wavefronts per SIMD.
template <int DT, int FMT, bool DENSE, bool REUSE, int UQ>
__device__ __forceinline__ void place_tile_c(const PlaceP &p, const Seg &sg, const uint32_t bx)
{
    constexpr int U = FMT == KDN_FMT_RAW_BF16 ? 4 : UQ;
    constexpr int W = FMT == KDN_FMT_RAW_BF16 ? 4 : FMT == KDN_FMT_INT4_GROUP32 ? 1 : 2; // words per 8 stored elements
    const int D = DT ? DT : p.c.D;
    const int R8 = D >> 3;   // lanes per row
    const int RW = 64 / R8;  // rows per wavefront and pass
    const int H = p.c.H, G = p.c.G, bs = p.c.bs;
    const int L2 = 2 * p.c.L;
    const int NT = blockDim.x; // a small tile is launched with fewer wavefronts

    const int S = sg.S, T = sg.T;
    const int piece = bx / L2;
    const int ls = bx - piece * L2;
    const int gi = S / G + piece;
    const int tok_lo = max(S, gi * G);
    const int tok_hi = min(S + T, (gi + 1) * G);
    if (tok_lo >= tok_hi)
        return;
    const int blk = sg.bt[tok_lo / bs];
    const int slot0 = tok_lo % bs;
    uint16_t *plane = ((ls & 1) ? p.c.v : p.c.k) + (int64_t)(p.layer0 + (ls >> 1)) * p.c.layer_stride;
    uint16_t *tile = plane + (int64_t)blk * p.c.block_stride + (int64_t)slot0 * p.c.token_stride;
    const int Tp = sg.Tp;
    const int64_t row_base = ((int64_t)ls * Tp + sg.tok0 + (tok_lo - S)) * H;
    const int64_t total_rows = (int64_t)p.c.L * 2 * Tp * H;
    const int n_rows = (tok_hi - tok_lo) * H;
    const uint8_t *data = sg.data + ((row_base * D * W) >> 1); // first stored row of this tile
    const int spr = FMT == KDN_FMT_INT4_GROUP32 ? D >> 5 : 1;  // scales per row
    const float *scales = reinterpret_cast<const float *>(sg.data + ((total_rows * D * W) >> 1)) + row_base * spr;
    const bool rotate = (ls & 1) == 0 && sg.rope_row >= 0;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int rw = lane / R8; // row of the wavefront's batch that this lane serves
    const int sub = lane - rw * R8;
    const bool lane_ok = rw < RW;
    // the lane's part in the rotation
    const bool interleaved = p.pairing == KDN_ROPE_INTERLEAVED;
    const bool rot_lane = rotate && lane_ok && sub < (p.rot >> 3);
    const int hl = p.rot >> 4; // lanes of half the rotary part
    const bool lo_lane = sub < hl;
    const bool exchange = rotate && !interleaved; // uniform over the workgroup
    const int partner = (rot_lane && !interleaved) ? (lo_lane ? lane + hl : lane - hl) : lane;
    __shared__ f32x2 s_cs[kMaxHeadDim / 2];
    f32x2 cs[8];
    if (rotate) {
        const int rhalf = p.rot >> 1;
        const f32x2 *row = p.rope + (int64_t)sg.rope_row * rhalf;
        for (int i = threadIdx.x; i < rhalf; i += NT)
            s_cs[i] = row[i];
        __syncthreads();
        if (rot_lane) {
            if (interleaved) {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    cs[e] = s_cs[sub * 4 + e];
            } else {
                const int j0 = (lo_lane ? sub : sub - hl) * 8;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    cs[e] = s_cs[j0 + e];
                    if (lo_lane)
                        cs[e].y = -cs[e].y; // lower element: own*cos - partner*sin
                }
            }
        }
    }

    const int rows_pass = (NT / 64) * RW;
    for (int b = 0; b < n_rows; b += rows_pass * U) { // same trip count for every lane
        uint32_t w[U][W];
        float sc[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int r = b + u * rows_pass + wave * RW + rw;
#pragma unroll
            for (int i = 0; i < W; ++i)
                w[u][i] = 0;
            sc[u] = 0.0f;
            if (lane_ok && r < n_rows) {
                const uint8_t *src = data + (((uint32_t)(r * D + sub * 8) * W) >> 1);
                if (FMT == KDN_FMT_INT4_GROUP32) {
                    w[u][0] = load_stored<uint32_t, REUSE>(src);
                    sc[u] = scales[r * spr + (sub >> 2)];
                } else if (FMT == KDN_FMT_RAW_BF16) {
                    const u32x4 v4 = load_stored<u32x4, REUSE>(src);
#pragma unroll
                    for (int i = 0; i < W; ++i)
                        w[u][i] = v4[i & 3];
                } else {
                    const u32x2 v2 = load_stored<u32x2, REUSE>(src);
#pragma unroll
                    for (int i = 0; i < W; ++i)
                        w[u][i] = v2[i & 1];
                    sc[u] = scales[r];
                }
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int r = b + u * rows_pass + wave * RW + rw;
            uint32_t pw[W];
            float psc = sc[u];
            if (exchange) {
#pragma unroll
                for (int i = 0; i < W; ++i)
                    pw[i] = (uint32_t)__builtin_amdgcn_ds_bpermute(partner << 2, (int)w[u][i]);
                if (FMT == KDN_FMT_INT4_GROUP32) // the partner's group has a scale of its own
                    psc = __int_as_float(__builtin_amdgcn_ds_bpermute(partner << 2, __float_as_int(sc[u])));
            } else {
#pragma unroll
                for (int i = 0; i < W; ++i)
                    pw[i] = 0;
            }
            if (!lane_ok || r >= n_rows)
                continue;
            uint16_t *dst; // the row's first element
            if (DENSE) {
                dst = tile + (uint32_t)(r * D);
            } else {
                const int tok = r / H, h = r - tok * H;
                if (p.c.per_token) {
                    const int t = tok_lo + tok;
                    dst = plane + (int64_t)sg.bt[t / bs] * p.c.block_stride + (int64_t)(t % bs) * p.c.token_stride
                          + (int64_t)h * p.c.head_stride;
                } else {
                    dst = tile + (int64_t)tok * p.c.token_stride + (int64_t)h * p.c.head_stride;
                }
            }
            u32x4 out;
            if (FMT == KDN_FMT_RAW_BF16 && !rot_lane) { // bit copy
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    out[i] = w[u][i % W];
            } else {
                float x[8];
                dequantise8<FMT>(w[u], sc[u], x);
                if (rot_lane && interleaved) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float c = cs[e].x, s = cs[e].y;
                        const float x0 = x[2 * e], x1 = x[2 * e + 1];
                        const float x0c = x0 * c, x1c = x1 * c;
                        x[2 * e] = __builtin_fmaf(-x1, s, x0c);
                        x[2 * e + 1] = __builtin_fmaf(x0, s, x1c);
                    }
                } else if (rot_lane) {
                    float y[8];
                    dequantise8<FMT>(pw, psc, y);
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const float xc = x[e] * cs[e].x;
                        x[e] = __builtin_fmaf(y[e], cs[e].y, xc);
                    }
                }
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    out[i] = pack_bf16(x[2 * i], x[2 * i + 1]);
            }
            __builtin_nontemporal_store(out, reinterpret_cast<u32x4 *>(dst + sub * 8));
        }
    }
}

// Grid rows, chained views and the barrier as in k_place.
template <int DT, int FMT, bool DENSE, bool REUSE, int UQ, typename Segs>
__global__ __launch_bounds__(kThreads) void k_place_c(PlaceP p, Segs segs)
{
    bool first = true;
    for (uint32_t bx = blockIdx.x; bx < p.tiles_x; bx += gridDim.x) { // the common launch has one tile per workgroup
        int at = blockIdx.y;
        do {
            if (!first)
                __syncthreads();
            first = false;
            const Seg &sg = segs.at(at);
            place_tile_c<DT, FMT, DENSE, REUSE, UQ>(p, sg, bx);
            at = sg.next;
        } while (at != 0);
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

// Bandwidth yardstick with the byte patterns of this library and none of its work.  A tile is
// `chunks` * 8 KiB of the big buffer and half that of the small one (launched with 128 threads
// and chunks = 1: 4 KiB and 2 KiB, the tile of one KV head of 128).  DIR 0 (the pattern of load
// and compose): a workgroup reads tile t of `small` (contiguous, in order) and writes tile
// ids[t] of `big` (tile t when ids is null): with ids, destination tiles scattered like the
// blocks of a random block table.  DIR 1 (the pattern of store): reads tile ids[t] of `big`,
// writes tile t of `small`.  DIR 2 writes that tile of `big` and reads nothing (each 16 bytes
// hold tile, 4 KiB run, lane and a constant); DIR 3 reads it and writes nothing: the two
// directions of the memory on their own.  16 bytes per lane and instruction, up to four 4 KiB
// loads of a thread issued before its first store, everything streamed; fewer workgroups than
// tiles stride over them.
constexpr uint32_t kProbeMark = 0x4b444e21u;
template <int DIR, int CH> // CH: chunks of 4 KiB per small tile when known at compile time (4: the 32 KiB tile), else 0
__global__ __launch_bounds__(kThreads) void k_probe_stream(u32x4 *__restrict__ small, u32x4 *__restrict__ big,
                                                          const int32_t *__restrict__ ids, uint32_t tiles,
                                                          uint32_t chunks_arg)
{
    constexpr bool FULL = CH > 0; // nothing is predicated
    const uint32_t chunks = CH ? CH : chunks_arg;
    const uint32_t NT = CH ? kThreads : blockDim.x; // lanes of a run: 256, or 128 for the 4 KiB tile (2 KiB runs)
    u32x4 seen = {0u, 0u, 0u, 0u};
    for (uint32_t t = blockIdx.x; t < tiles; t += gridDim.x) {
        u32x4 *s = small + (size_t)t * chunks * NT;
        const uint32_t tile = ids ? (uint32_t)ids[t] : t;
        u32x4 *b = big + (size_t)tile * chunks * (2 * NT);
        for (uint32_t c0 = 0; c0 < chunks; c0 += 4) {
            u32x4 v[4], w[4];
#pragma unroll
            for (uint32_t u = 0; u < 4; ++u) {
                if (FULL || c0 + u < chunks) {
                    if (DIR == 0) {
                        v[u] = __builtin_nontemporal_load(s + (c0 + u) * NT + threadIdx.x);
                    } else if (DIR == 1 || DIR == 3) {
                        v[u] = __builtin_nontemporal_load(b + (2 * (c0 + u)) * NT + threadIdx.x);
                        w[u] = __builtin_nontemporal_load(b + (2 * (c0 + u) + 1) * NT + threadIdx.x);
                    }
                }
            }
#pragma unroll
            for (uint32_t u = 0; u < 4; ++u) {
                if (FULL || c0 + u < chunks) {
                    if (DIR == 0) {
                        u32x4 x = v[u];
                        x.x ^= 0x80008000u; // the second vector differs from the first, as an upper half row would
                        __builtin_nontemporal_store(v[u], b + (2 * (c0 + u)) * NT + threadIdx.x);
                        __builtin_nontemporal_store(x, b + (2 * (c0 + u) + 1) * NT + threadIdx.x);
                    } else if (DIR == 1) {
                        __builtin_nontemporal_store(v[u] ^ w[u], s + (c0 + u) * NT + threadIdx.x);
                    } else if (DIR == 2) {
                        const u32x4 x = {tile, 2 * (c0 + u), threadIdx.x, kProbeMark};
                        u32x4 y = x;
                        y.y += 1;
                        __builtin_nontemporal_store(x, b + (2 * (c0 + u)) * NT + threadIdx.x);
                        __builtin_nontemporal_store(y, b + (2 * (c0 + u) + 1) * NT + threadIdx.x);
                    } else {
                        seen ^= v[u] ^ w[u];
                    }
                }
            }
        }
    }
    // keeps the loads of DIR 3 alive; the small buffer is written only if what was read folds
    // to one particular 128-bit value
    if (DIR == 3 && seen.x == kProbeMark && seen.y == ~kProbeMark && seen.z == 0x5eed5eedu && seen.w == 0xfeedf00du)
        small[(size_t)blockIdx.x * NT + threadIdx.x] = seen;
}

// Writes up to kScratchWords 32-bit words that travel in the kernel arguments to
// dst[first .. first + n): how small host tables reach device memory with no copy call.
constexpr int kScratchWords = 960;
struct ScratchWords {
    uint32_t first, n;
    uint32_t w[kScratchWords];
};

__global__ __launch_bounds__(kThreads) void k_scratch_write(uint32_t *dst, ScratchWords a)
{
    for (uint32_t i = threadIdx.x; i < a.n; i += blockDim.x)
        dst[a.first + i] = a.w[i];
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

} // namespace kdn_impl
#endif // KDN_KERNELS_H
