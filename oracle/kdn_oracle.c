/*
 * kdn_oracle.c -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, scalar CPU definition of what the KDN hot path computes:
 * moving KV caches between an engine's paged KV memory and a stored form
 * (store), back (load), and composing several stored chunks into one request
 * with the keys re-rotated to their new positions (compose).
 *
 * The paper (Sec. 3.1 "Knowledge Delivery Architecture": storage, delivery,
 * blending modules; Sec. 3.2 "Interface with LLM serving engines": the store
 * and retrieve APIs; Sec. 3 "Limitations": prefix-only reuse) fixes only the
 * framing.  It prints no equation, listing or number for this path, so every
 * numeric rule below is a stated reading (block comments marked READING).
 *
 * This file shares no code with the HIP library.  Only tests, the smoke check
 * and the bench's cpu_baseline leg may use it.  All pointers are HOST memory.
 *
 * Build: gcc -O2 -std=c11 -ffp-contract=off -fPIC -shared kdn_oracle.c -lm
 *
 * Pinned by tests/test_oracle_pins.py: address resolution by brute force with
 * tagged fills, bf16 rounding against a float64 formulation, scales and codes
 * against float64 arithmetic, the error bound (per row, and of a whole store
 * against the source rows), which source row feeds which stored row and scale
 * slot for every quantised form, the rotation against complex multiplication /
 * the shift identity R(d)K(p) = K(p+d), zero-offset compose against
 * concatenation.  tests/test_oracle_mutants.py plants one mistake at a time in
 * a copy of this file and requires a pin to fail.  Absolute output values of the five workloads are
 * not printed anywhere in the paper: for those, parity is unpinned by the
 * paper and rests on the pins above.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

enum { KDNO_FMT_RAW_BF16 = 0, KDNO_FMT_INT8_ROWSCALE = 1, KDNO_FMT_INT4_GROUP32 = 2, KDNO_FMT_FP8_ROWSCALE = 3 };
enum { KDNO_GROUP = 32 };

/* Engine paged KV memory (Sec. 3.2, "paged memory" of the serving engine).
 * READING: per layer l and side (K or V) an array addressed as
 *   base[l*layer_stride + block*block_stride + slot*token_stride + h*head_stride + j]
 * in bf16 elements, j in [0, D) contiguous. */
typedef struct {
    uint16_t *k;
    uint16_t *v;
    int32_t L, H, D, bs, nb;
    int64_t layer_stride, block_stride, token_stride, head_stride;
} kdno_cache;

/* ---- bf16 <-> fp32 ------------------------------------------------------
 * READING: bf16 is the upper half of an IEEE binary32.  Widening is exact.
 * Narrowing rounds to nearest, ties to even, on the 16 dropped bits; a NaN
 * stays a (quiet) NaN. */
float kdno_bf16_to_f32(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

uint16_t kdno_f32_to_bf16(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    if ((u & 0x7fffffffu) > 0x7f800000u)
        return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t keep_lsb = (u >> 16) & 1u;
    u += 0x7fffu + keep_lsb;
    return (uint16_t)(u >> 16);
}

void kdno_f32_to_bf16_array(const float *in, uint16_t *out, int64_t n)
{
    for (int64_t i = 0; i < n; ++i)
        out[i] = kdno_f32_to_bf16(in[i]);
}

/* ---- stored form ----------------------------------------------------------
 * READING (the "compressed" KV of the delivery module, Sec. 3.1).  A chunk
 * that holds Tp tokens is one byte buffer:
 *   raw  : bf16  [L][2][Tp][H][D]                      (side 0 = K, 1 = V)
 *   int8 : int8  [L][2][Tp][H][D]   codes, then
 *          fp32  [L][2][Tp][H]      one scale per (token, kv-head) row.
 *   int4 : uint8 [L][2][Tp][H][D/2] two codes per byte (element 2k in the low
 *                                   nibble, 2k+1 in the high nibble, two's
 *                                   complement), then
 *          fp32  [L][2][Tp][H][D/32] one scale per group of 32 elements.
 *   fp8  : uint8 [L][2][Tp][H][D]   e4m3 codes, then fp32 [L][2][Tp][H] row scales
 *                                   (the int8 layout with other codes).
 * Tokens stay sliceable: a view is (Tp, tok_start, T). */
int64_t kdno_chunk_bytes(int32_t L, int32_t H, int32_t D, int32_t Tp, int32_t fmt)
{
    int64_t rows = (int64_t)L * 2 * Tp * H;
    if (fmt == KDNO_FMT_RAW_BF16)
        return rows * D * 2;
    if (fmt == KDNO_FMT_INT4_GROUP32)
        return rows * (D / 2) + rows * (D / KDNO_GROUP) * 4;
    return rows * D + rows * 4;
}

static int64_t row_index(int32_t l, int32_t side, int32_t Tp, int32_t t, int32_t H, int32_t h)
{
    return (((int64_t)l * 2 + side) * Tp + t) * H + h;
}

static uint16_t *cache_row(const kdno_cache *c, int32_t l, int32_t side,
                           int32_t block, int32_t slot, int32_t h)
{
    uint16_t *base = side == 0 ? c->k : c->v;
    return base + (int64_t)l * c->layer_stride + (int64_t)block * c->block_stride
                + (int64_t)slot * c->token_stride + (int64_t)h * c->head_stride;
}

/* ---- per-row symmetric int8 -----------------------------------------------
 * READING: amax = max|x_j| over the D elements of one (token, kv-head) row.
 * A row with amax < 2^-121 (which includes the all-zero row; below that bound
 * 127/amax is not a finite fp32) is stored as scale 0 and codes 0.
 * Otherwise scale = amax/127 and inv = 127/amax, one IEEE fp32 division each,
 * and q_j = clamp(rint(x_j * inv), -127, 127) with round-half-to-even.
 * -128 never appears. */
void kdno_quantise_row(const uint16_t *x, int32_t D, int8_t *q, float *scale)
{
    float amax = 0.0f;
    for (int32_t j = 0; j < D; ++j) {
        float a = fabsf(kdno_bf16_to_f32(x[j]));
        if (a > amax)
            amax = a;
    }
    if (amax < 0x1p-121f) {
        *scale = 0.0f;
        for (int32_t j = 0; j < D; ++j)
            q[j] = 0;
        return;
    }
    *scale = amax / 127.0f;
    float inv = 127.0f / amax;
    for (int32_t j = 0; j < D; ++j) {
        float r = rintf(kdno_bf16_to_f32(x[j]) * inv);
        if (r > 127.0f)
            r = 127.0f;
        if (r < -127.0f)
            r = -127.0f;
        q[j] = (int8_t)r;
    }
}

/* READING: y_j = (float)q_j * scale, one fp32 multiply. */
void kdno_dequantise_row(const int8_t *q, float scale, int32_t D, float *y)
{
    for (int32_t j = 0; j < D; ++j)
        y[j] = (float)q[j] * scale;
}

/* ---- group-wise symmetric int4 ----------------------------------------------
 * READING (a tighter stored form toward the footprint reductions of Sec. 3.2,
 * "KV-cache delivery"): the row is cut into groups of 32 consecutive elements.
 * Per group: amax = max|x_j|; a group with amax < 2^-121 is stored as scale 0,
 * codes 0; otherwise scale = amax/7, inv = 7/amax (IEEE fp32 divisions) and
 * q_j = clamp(rint(x_j * inv), -7, 7), ties to even.  Codes are packed two per
 * byte as two's-complement nibbles, the even element in the low nibble.  D must
 * be a multiple of 32. */
void kdno_quantise_row_int4(const uint16_t *x, int32_t D, uint8_t *packed, float *scales)
{
    for (int32_t g = 0; g < D / KDNO_GROUP; ++g) {
        const uint16_t *xg = x + g * KDNO_GROUP;
        float amax = 0.0f;
        for (int32_t j = 0; j < KDNO_GROUP; ++j) {
            float a = fabsf(kdno_bf16_to_f32(xg[j]));
            if (a > amax)
                amax = a;
        }
        int keep = !(amax < 0x1p-121f);
        scales[g] = keep ? amax / 7.0f : 0.0f;
        float inv = keep ? 7.0f / amax : 0.0f;
        for (int32_t j = 0; j < KDNO_GROUP; j += 2) {
            int q[2];
            for (int32_t e = 0; e < 2; ++e) {
                float r = keep ? rintf(kdno_bf16_to_f32(xg[j + e]) * inv) : 0.0f;
                if (r > 7.0f)
                    r = 7.0f;
                if (r < -7.0f)
                    r = -7.0f;
                q[e] = (int)r;
            }
            packed[(g * KDNO_GROUP + j) / 2] = (uint8_t)((q[0] & 0xF) | ((q[1] & 0xF) << 4));
        }
    }
}

/* READING: y_j = (float)q_j * scale_group(j), one fp32 multiply. */
void kdno_dequantise_row_int4(const uint8_t *packed, const float *scales, int32_t D, float *y)
{
    for (int32_t j = 0; j < D; ++j) {
        int nib = (packed[j / 2] >> (4 * (j & 1))) & 0xF;
        int q = nib >= 8 ? nib - 16 : nib;
        y[j] = (float)q * scales[j / KDNO_GROUP];
    }
}

/* ---- fp8 (e4m3) with a row scale ------------------------------------------------
 * READING: the 8-bit float with 4 exponent bits (bias 7), 3 mantissa bits, no
 * infinities, all-ones = NaN, largest finite value 448, subnormals below 2^-6 in steps
 * of 2^-9.  Conversion rounds to nearest, ties to the even code, and saturates at 448.
 * Per row: amax < 2^-119 (448/amax would not be a finite fp32) gives scale 0 and codes
 * 0; otherwise scale = amax/448, inv = 448/amax, code_j = e4m3(x_j * inv); the
 * dequantised value is e4m3_value(code_j) * scale, one fp32 multiply. */
uint8_t kdno_f32_to_e4m3(float f)
{
    uint8_t sign = signbit(f) ? 0x80 : 0;
    float a = fabsf(f);
    if (a != a)
        return (uint8_t)(sign | 0x7f);
    if (a >= 448.0f)
        return (uint8_t)(sign | 0x7e);
    if (a < 0x1p-6f) {                         /* subnormal range: multiples of 2^-9 */
        int q = (int)rintf(a * 0x1p9f);        /* 0..8; 8 is the smallest normal's code */
        return (uint8_t)(sign | q);
    }
    int e;
    float m = frexpf(a, &e);                   /* a = m * 2^e, m in [0.5, 1) */
    m *= 2.0f;
    e -= 1;                                    /* a = m * 2^e, m in [1, 2) */
    int q = (int)rintf((m - 1.0f) * 8.0f);     /* 0..8 */
    if (q == 8) {
        q = 0;
        e += 1;
    }
    return (uint8_t)(sign | ((e + 7) << 3) | q);
}

float kdno_e4m3_to_f32(uint8_t c)
{
    int e = (c >> 3) & 0xf, q = c & 7;
    float v;
    if (e == 0xf && q == 7)
        v = NAN;
    else if (e == 0)
        v = ldexpf((float)q, -9);
    else
        v = ldexpf(1.0f + (float)q / 8.0f, e - 7);
    return (c & 0x80) ? -v : v;
}

void kdno_quantise_row_fp8(const uint16_t *x, int32_t D, uint8_t *q, float *scale)
{
    float amax = 0.0f;
    for (int32_t j = 0; j < D; ++j) {
        float a = fabsf(kdno_bf16_to_f32(x[j]));
        if (a > amax)
            amax = a;
    }
    if (amax < 0x1p-119f) {
        *scale = 0.0f;
        for (int32_t j = 0; j < D; ++j)
            q[j] = 0;
        return;
    }
    *scale = amax / 448.0f;
    float inv = 448.0f / amax;
    for (int32_t j = 0; j < D; ++j)
        q[j] = kdno_f32_to_e4m3(kdno_bf16_to_f32(x[j]) * inv);
}

void kdno_dequantise_row_fp8(const uint8_t *q, float scale, int32_t D, float *y)
{
    for (int32_t j = 0; j < D; ++j)
        y[j] = kdno_e4m3_to_f32(q[j]) * scale;
}

/* ---- RoPE shift -------------------------------------------------------------
 * READING (a chunk reused at a position other than the one it was computed at,
 * Sec. 3.2 blending): keys
 * carry rotary position embedding; moving a chunk by d positions multiplies
 * each pair (j, j + D/2) by the rotation of angle d * theta_j,
 * theta_j = base^(-2j/D).  theta, the angle, cos and sin are evaluated in
 * double; cos and sin are rounded once to fp32.  Table layout [D/2][2] =
 * (cos, sin). */
void kdno_rope_table(double base, int32_t D, int32_t d, float *cs)
{
    for (int32_t j = 0; j < D / 2; ++j) {
        double theta = pow(base, -(double)(2 * j) / (double)D);
        double phi = (double)d * theta;
        cs[2 * j] = (float)cos(phi);
        cs[2 * j + 1] = (float)sin(phi);
    }
}

/* ---- RoPE variants ------------------------------------------------------------
 * READING (what real models need before a chunk can be reused at another
 * position, Sec. 3.2 blending): only the first rot_dim elements of a row may be
 * rotary (partial rotary; rot_dim == D is the plain case), pairs may be half-split
 * (j, j + rot_dim/2) or interleaved (2j, 2j + 1), and the rot_dim/2 frequencies may
 * be given explicitly (for rescaled-frequency models) instead of base^(-2j/rot_dim).
 * Elements at and beyond rot_dim are never changed. */
enum { KDNO_PAIR_HALF_SPLIT = 0, KDNO_PAIR_INTERLEAVED = 1 };

void kdno_rope_table_spec(double base, const double *inv_freq, int32_t rot_dim, int32_t d, float *cs)
{
    for (int32_t j = 0; j < rot_dim / 2; ++j) {
        double theta = inv_freq ? inv_freq[j] : pow(base, -(double)(2 * j) / (double)rot_dim);
        double phi = (double)d * theta;
        cs[2 * j] = (float)cos(phi);
        cs[2 * j + 1] = (float)sin(phi);
    }
}

/* Same two-operation form as kdno_rotate_row, on the pairs the variant names:
 * first' = fma(-second, s, first*c), second' = fma(first, s, second*c). */
void kdno_rotate_row_spec(float *y, int32_t rot_dim, int32_t pairing, const float *cs)
{
    int32_t half = rot_dim / 2;
    for (int32_t j = 0; j < half; ++j) {
        int32_t ia = pairing == KDNO_PAIR_INTERLEAVED ? 2 * j : j;
        int32_t ib = pairing == KDNO_PAIR_INTERLEAVED ? 2 * j + 1 : j + half;
        float c = cs[2 * j], s = cs[2 * j + 1];
        float a = y[ia], b = y[ib];
        float ac = a * c;
        float bc = b * c;
        y[ia] = fmaf(-b, s, ac);
        y[ib] = fmaf(a, s, bc);
    }
}

/* Rotate one row held in fp32, in place:
 *   lo' = fma(-hi, s, lo*c)     hi' = fma(lo, s, hi*c)
 * (one rounded product, then one fused multiply-add, per output). */
void kdno_rotate_row(float *y, int32_t D, const float *cs)
{
    int32_t half = D / 2;
    for (int32_t j = 0; j < half; ++j) {
        float c = cs[2 * j], s = cs[2 * j + 1];
        float a = y[j], b = y[j + half];
        float ac = a * c;
        float bc = b * c;
        y[j] = fmaf(-b, s, ac);
        y[j + half] = fmaf(a, s, bc);
    }
}

/* ---- store (the "store" API, Sec. 3.2) ----------------------------------------
 * Gathers tokens [t0, t0+T) of the request whose block table is bt into the
 * stored form of a chunk of exactly T tokens.  Layers [l0, l1) only, so that
 * callers may split layers over threads.  Returns 0, or -1 on a bad range. */
int kdno_store(const kdno_cache *c, const int32_t *bt, int32_t table_len,
               int32_t t0, int32_t T, int32_t fmt, void *out,
               int32_t l0, int32_t l1)
{
    if (t0 < 0 || T < 0 || (int64_t)t0 + T > (int64_t)table_len * c->bs)
        return -1;
    const int32_t H = c->H, D = c->D;
    if (fmt == KDNO_FMT_INT4_GROUP32 && D % KDNO_GROUP != 0)
        return -1;
    int64_t n_rows = (int64_t)c->L * 2 * T * H;
    uint16_t *raw = (uint16_t *)out;
    int8_t *codes = (int8_t *)out;
    float *scales = (float *)((char *)out + n_rows * D);
    uint8_t *codes4 = (uint8_t *)out;
    float *scales4 = (float *)((char *)out + n_rows * (D / 2));
    for (int32_t l = l0; l < l1; ++l)
        for (int32_t side = 0; side < 2; ++side)
            for (int32_t t = 0; t < T; ++t) {
                int32_t tok = t0 + t;
                int32_t block = bt[tok / c->bs];
                int32_t slot = tok % c->bs;
                if (block < 0 || block >= c->nb)
                    return -1;
                for (int32_t h = 0; h < H; ++h) {
                    const uint16_t *src = cache_row(c, l, side, block, slot, h);
                    int64_t r = row_index(l, side, T, t, H, h);
                    if (fmt == KDNO_FMT_RAW_BF16)
                        memcpy(raw + r * D, src, (size_t)D * 2);
                    else if (fmt == KDNO_FMT_INT4_GROUP32)
                        kdno_quantise_row_int4(src, D, codes4 + r * (D / 2), scales4 + r * (D / KDNO_GROUP));
                    else if (fmt == KDNO_FMT_FP8_ROWSCALE)
                        kdno_quantise_row_fp8(src, D, (uint8_t *)codes + r * D, scales + r);
                    else
                        kdno_quantise_row(src, D, codes + r * D, scales + r);
                }
            }
    return 0;
}

/* Store of a token list: row t of the chunk holds request token tokens[t] (the gather
 * a token-dropping compressor needs, Sec. 3.2 "KV-cache delivery": only the tokens it
 * keeps are stored).  Same per-row rules as kdno_store. */
int kdno_store_tokens(const kdno_cache *c, const int32_t *bt, int32_t table_len,
                      const int32_t *tokens, int32_t n, int32_t fmt, void *out,
                      int32_t l0, int32_t l1)
{
    const int32_t H = c->H, D = c->D;
    if (fmt == KDNO_FMT_INT4_GROUP32 && D % KDNO_GROUP != 0)
        return -1;
    for (int32_t t = 0; t < n; ++t)
        if (tokens[t] < 0 || tokens[t] >= (int64_t)table_len * c->bs)
            return -1;
    int64_t n_rows = (int64_t)c->L * 2 * n * H;
    for (int32_t l = l0; l < l1; ++l)
        for (int32_t side = 0; side < 2; ++side)
            for (int32_t t = 0; t < n; ++t) {
                int32_t block = bt[tokens[t] / c->bs], slot = tokens[t] % c->bs;
                if (block < 0 || block >= c->nb)
                    return -1;
                for (int32_t h = 0; h < H; ++h) {
                    const uint16_t *src = cache_row(c, l, side, block, slot, h);
                    int64_t r = row_index(l, side, n, t, H, h);
                    if (fmt == KDNO_FMT_RAW_BF16)
                        memcpy((uint16_t *)out + r * D, src, (size_t)D * 2);
                    else if (fmt == KDNO_FMT_INT4_GROUP32)
                        kdno_quantise_row_int4(src, D, (uint8_t *)out + r * (D / 2),
                                               (float *)((char *)out + n_rows * (D / 2)) + r * (D / KDNO_GROUP));
                    else if (fmt == KDNO_FMT_FP8_ROWSCALE)
                        kdno_quantise_row_fp8(src, D, (uint8_t *)out + r * D,
                                              (float *)((char *)out + n_rows * D) + r);
                    else
                        kdno_quantise_row(src, D, (int8_t *)out + r * D,
                                          (float *)((char *)out + n_rows * D) + r);
                }
            }
    return 0;
}

/* Place tokens [tok_start, tok_start+T) of a stored chunk (parent length Tp)
 * at request tokens [dest, dest+T), with RoPE offset d applied to K rows.
 * READING: d == 0 skips the rotation altogether (it is not a multiply by
 * cos 0), so a zero-offset compose is bit-identical to a load; V rows are
 * never rotated; raw-format rows with d == 0 are bit copies. */
static int place(const void *data, int32_t fmt, int32_t Tp, int32_t tok_start,
                 int32_t T, int32_t d, const float *cs, int32_t rot_dim, int32_t pairing,
                 const kdno_cache *c, const int32_t *bt, int32_t dest, int32_t l0, int32_t l1)
{
    const int32_t H = c->H, D = c->D;
    int64_t n_rows = (int64_t)c->L * 2 * Tp * H;
    const uint16_t *raw = (const uint16_t *)data;
    const int8_t *codes = (const int8_t *)data;
    const float *scales = (const float *)((const char *)data + n_rows * D);
    const uint8_t *codes4 = (const uint8_t *)data;
    const float *scales4 = (const float *)((const char *)data + n_rows * (D / 2));
    float y[4096];
    if (D > 4096 || (fmt == KDNO_FMT_INT4_GROUP32 && D % KDNO_GROUP != 0))
        return -1;
    for (int32_t l = l0; l < l1; ++l)
        for (int32_t side = 0; side < 2; ++side)
            for (int32_t t = 0; t < T; ++t) {
                int32_t tok = dest + t;
                int32_t block = bt[tok / c->bs];
                int32_t slot = tok % c->bs;
                if (block < 0 || block >= c->nb)
                    return -1;
                for (int32_t h = 0; h < H; ++h) {
                    uint16_t *dst = cache_row(c, l, side, block, slot, h);
                    int64_t r = row_index(l, side, Tp, tok_start + t, H, h);
                    int rotate = (side == 0 && d != 0);
                    if (fmt == KDNO_FMT_RAW_BF16 && !rotate) {
                        memcpy(dst, raw + r * D, (size_t)D * 2);
                        continue;
                    }
                    if (fmt == KDNO_FMT_RAW_BF16) {
                        for (int32_t j = 0; j < D; ++j)
                            y[j] = kdno_bf16_to_f32(raw[r * D + j]);
                    } else if (fmt == KDNO_FMT_INT4_GROUP32) {
                        kdno_dequantise_row_int4(codes4 + r * (D / 2), scales4 + r * (D / KDNO_GROUP), D, y);
                    } else if (fmt == KDNO_FMT_FP8_ROWSCALE) {
                        kdno_dequantise_row_fp8((const uint8_t *)codes + r * D, scales[r], D, y);
                    } else {
                        kdno_dequantise_row(codes + r * D, scales[r], D, y);
                    }
                    if (rotate && rot_dim == D && pairing == KDNO_PAIR_HALF_SPLIT)
                        kdno_rotate_row(y, D, cs);
                    else if (rotate)
                        kdno_rotate_row_spec(y, rot_dim, pairing, cs);
                    for (int32_t j = 0; j < D; ++j)
                        dst[j] = kdno_f32_to_bf16(y[j]);
                }
            }
    return 0;
}

/* ---- load (the retrieve API, Sec. 3.2; decompression on the GPU, Sec. 3.1)
 * Dequantise and scatter a chunk view into the request's blocks; never rotates. */
int kdno_load(const void *data, int32_t fmt, int32_t Tp, int32_t tok_start,
              int32_t T, const kdno_cache *c, const int32_t *bt,
              int32_t table_len, int32_t dest, int32_t l0, int32_t l1)
{
    if (tok_start < 0 || T < 0 || tok_start + (int64_t)T > Tp || dest < 0
        || (int64_t)dest + T > (int64_t)table_len * c->bs)
        return -1;
    return place(data, fmt, Tp, tok_start, T, 0, 0, c->D, KDNO_PAIR_HALF_SPLIT, c, bt, dest, l0, l1);
}

/* ---- compose (the blending module, Sec. 3.1) -------------------------------------
 * Chunk i goes to request tokens [dest + S_i, dest + S_i + T_i) with
 * S_i = sum_{j<i} T_j; offsets[i] is only the RoPE position delta of chunk i.
 * Slots past the last token and blocks outside the table are not touched. */
int kdno_compose(int32_t n, const void *const *data, const int32_t *fmt,
                 const int32_t *Tp, const int32_t *tok_start, const int32_t *T,
                 const int32_t *offsets, const kdno_cache *c, const int32_t *bt,
                 int32_t table_len, int32_t dest, double rope_base,
                 int32_t l0, int32_t l1)
{
    int64_t total = 0;
    for (int32_t i = 0; i < n; ++i) {
        if (tok_start[i] < 0 || T[i] < 0 || tok_start[i] + (int64_t)T[i] > Tp[i])
            return -1;
        total += T[i];
    }
    if (dest < 0 || (int64_t)dest + total > (int64_t)table_len * c->bs)
        return -1;
    float cs[4096];
    if (c->D > 4096)
        return -1;
    int32_t S = dest;
    for (int32_t i = 0; i < n; ++i) {
        if (offsets[i] != 0)
            kdno_rope_table(rope_base, c->D, offsets[i], cs);
        int rc = place(data[i], fmt[i], Tp[i], tok_start[i], T[i], offsets[i],
                       cs, c->D, KDNO_PAIR_HALF_SPLIT, c, bt, S, l0, l1);
        if (rc)
            return rc;
        S += T[i];
    }
    return 0;
}

/* Compose with a RoPE variant: rot_dim (even, <= D; 0 means D), pairing, and either
 * rope_base or rot_dim/2 explicit frequencies. */
int kdno_compose_spec(int32_t n, const void *const *data, const int32_t *fmt,
                      const int32_t *Tp, const int32_t *tok_start, const int32_t *T,
                      const int32_t *offsets, const kdno_cache *c, const int32_t *bt,
                      int32_t table_len, int32_t dest, double rope_base,
                      const double *inv_freq, int32_t rot_dim, int32_t pairing,
                      int32_t l0, int32_t l1)
{
    if (rot_dim == 0)
        rot_dim = c->D;
    if (rot_dim < 0 || rot_dim > c->D || rot_dim % 2 != 0 || c->D > 4096)
        return -1;
    int64_t total = 0;
    for (int32_t i = 0; i < n; ++i) {
        if (tok_start[i] < 0 || T[i] < 0 || tok_start[i] + (int64_t)T[i] > Tp[i])
            return -1;
        total += T[i];
    }
    if (dest < 0 || (int64_t)dest + total > (int64_t)table_len * c->bs)
        return -1;
    float cs[4096];
    int32_t S = dest;
    for (int32_t i = 0; i < n; ++i) {
        if (offsets[i] != 0)
            kdno_rope_table_spec(rope_base, inv_freq, rot_dim, offsets[i], cs);
        int rc = place(data[i], fmt[i], Tp[i], tok_start[i], T[i], offsets[i],
                       cs, rot_dim, pairing, c, bt, S, l0, l1);
        if (rc)
            return rc;
        S += T[i];
    }
    return 0;
}

/* ---- patch (the write-back half of selective recompute, Sec. 3.2 blending) -------
 * READING: after a compose, an engine may recompute the K/V of a few tokens and must
 * put them over the composed ones.  rows holds bf16 [L][2][n][H][D]; row i replaces
 * request token tokens[i] (bit copy).  Token indices must be distinct. */
int kdno_patch_rows(const uint16_t *rows, const int32_t *tokens, int32_t n,
                    const kdno_cache *c, const int32_t *bt, int32_t table_len)
{
    for (int32_t i = 0; i < n; ++i)
        if (tokens[i] < 0 || tokens[i] >= (int64_t)table_len * c->bs)
            return -1;
    for (int32_t l = 0; l < c->L; ++l)
        for (int32_t side = 0; side < 2; ++side)
            for (int32_t i = 0; i < n; ++i) {
                int32_t block = bt[tokens[i] / c->bs], slot = tokens[i] % c->bs;
                if (block < 0 || block >= c->nb)
                    return -1;
                for (int32_t h = 0; h < c->H; ++h)
                    memcpy(cache_row(c, l, side, block, slot, h),
                           rows + ((((int64_t)l * 2 + side) * n + i) * c->H + h) * c->D,
                           (size_t)c->D * 2);
            }
    return 0;
}
