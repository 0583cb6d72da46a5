/* Host-only run of the CPU oracle over ragged shapes, meant to be built together with
 * oracle/kdn_oracle.c under -fsanitize=address,undefined: every buffer is allocated at
 * its exact size, so an index past a buffer or a misaligned or overflowing access is
 * reported.  Exit code 0 means no report. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    uint16_t *k, *v;
    int32_t L, H, D, bs, nb;
    int64_t layer_stride, block_stride, token_stride, head_stride;
} kdno_cache;

int64_t kdno_chunk_bytes(int32_t L, int32_t H, int32_t D, int32_t Tp, int32_t fmt);
int kdno_store(const kdno_cache *c, const int32_t *bt, int32_t table_len, int32_t t0, int32_t T,
               int32_t fmt, void *out, int32_t l0, int32_t l1);
int kdno_compose_spec(int32_t n, const void *const *data, const int32_t *fmt, const int32_t *Tp,
                      const int32_t *tok_start, const int32_t *T, const int32_t *offsets,
                      const kdno_cache *c, const int32_t *bt, int32_t table_len, int32_t dest,
                      double rope_base, const double *inv_freq, int32_t rot_dim, int32_t pairing,
                      int32_t l0, int32_t l1);
int kdno_patch_rows(const uint16_t *rows, const int32_t *tokens, int32_t n, const kdno_cache *c,
                    const int32_t *bt, int32_t table_len);

static uint32_t rnd(uint32_t *s) { *s = *s * 1664525u + 1013904223u; return *s >> 8; }

int main(void)
{
    uint32_t seed = 99;
    const int32_t dims[] = {32, 64, 96, 128};
    for (int trial = 0; trial < 24; ++trial) {
        kdno_cache c;
        c.L = 1 + trial % 3; c.H = 1 + trial % 4; c.D = dims[trial % 4]; c.bs = 1 + (trial * 5) % 17; c.nb = 12;
        c.head_stride = c.D; c.token_stride = (int64_t)c.H * c.D;
        c.block_stride = c.token_stride * c.bs; c.layer_stride = c.block_stride * c.nb;
        size_t n = (size_t)c.L * c.layer_stride;
        c.k = malloc(n * 2); c.v = malloc(n * 2);
        for (size_t i = 0; i < n; ++i) {       /* finite bf16 patterns only */
            c.k[i] = (uint16_t)((rnd(&seed) & 0x80ff) | 0x3f00);
            c.v[i] = (uint16_t)((rnd(&seed) & 0x80ff) | 0x3e00);
        }
        int32_t bt[6] = {7, 2, 9, 0, 11, 4};
        int32_t cap = 6 * c.bs;
        for (int fmt = 0; fmt < 3; ++fmt) {
            int32_t t0 = (int32_t)(rnd(&seed) % (uint32_t)(cap / 2 + 1));
            int32_t T = 1 + (int32_t)(rnd(&seed) % (uint32_t)(cap - t0));
            void *chunk = malloc((size_t)kdno_chunk_bytes(c.L, c.H, c.D, T, fmt));
            if (kdno_store(&c, bt, 6, t0, T, fmt, chunk, 0, c.L)) return 2;
            int32_t ts = (int32_t)(rnd(&seed) % (uint32_t)T), Tv = 1 + (int32_t)(rnd(&seed) % (uint32_t)(T - ts));
            int32_t dest = (int32_t)(rnd(&seed) % (uint32_t)(cap - Tv + 1));
            int32_t off = (int32_t)(rnd(&seed) % 5000) - 2500;
            const void *data[1] = {chunk};
            int32_t rot = (trial % 2) ? c.D : c.D / 2, pairing = trial % 2;
            if (kdno_compose_spec(1, data, &fmt, &T, &ts, &Tv, &off, &c, bt, 6, dest, 10000.0, 0, rot,
                                  pairing, 0, c.L))
                return 3;
            free(chunk);
        }
        int32_t tokens[3] = {0, cap - 1, cap / 2};
        uint16_t *rows = calloc((size_t)c.L * 2 * 3 * c.H * c.D, 2);
        if (kdno_patch_rows(rows, tokens, cap > 2 ? 3 : 1, &c, bt, 6)) return 4;
        free(rows); free(c.k); free(c.v);
    }
    puts("oracle_check ok");
    return 0;
}
