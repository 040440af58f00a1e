/* Drives every entry point of tq_oracle.c over ragged sizes, bucketed and not, both dtypes and
 * all code widths, for a build with -fsanitize=address,undefined: any out-of-bounds access,
 * misaligned access, signed overflow or invalid shift in the oracle aborts the program. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../oracle/tq_oracle.c"

static uint32_t lcg(uint32_t *s) { *s = *s * 1664525u + 1013904223u; return *s; }

static void make_params(tqo_params_t *P, int bits, int grid, float alpha)
{
    memset(P, 0, sizeof *P);
    const int s = (1 << bits) - 1;
    P->alpha = alpha; P->bits = (uint32_t)bits; P->s = (uint32_t)s; P->grid = (uint32_t)grid;
    for (int k = 0; k <= s; ++k) {
        double t = -1.0 + 2.0 * k / s;
        if (grid != TQO_GRID_UNIFORM) t = t * fabs(t);          /* denser near zero */
        P->level[k] = (float)(alpha * t);
    }
    P->level[0] = -alpha; P->level[s] = alpha;
    for (int k = 0; k < s; ++k)
        P->inv_w[k] = grid == TQO_GRID_UNIFORM ? (float)(s / (2.0 * alpha))
                                               : (float)(1.0 / ((double)P->level[k + 1] - (double)P->level[k]));
}

int main(void)
{
    uint32_t seed = 12345u;
    const uint64_t sizes[] = {1, 7, 8, 9, 41, 127, 128, 129, 2049, 5000};
    const uint64_t buckets[] = {0, 128, 1024};
    unsigned long long cases = 0;
    for (size_t si = 0; si < sizeof sizes / sizeof *sizes; ++si)
        for (size_t bi = 0; bi < sizeof buckets / sizeof *buckets; ++bi)
            for (int dtype = 0; dtype < 2; ++dtype)
                for (int bits = 2; bits <= 4; ++bits)
                    for (int grid = 0; grid < 2; ++grid) {
                        const uint64_t d = sizes[si], be = buckets[bi];
                        const uint64_t nb = tqo_num_buckets(d, be);
                        float *gf = malloc(d * sizeof *gf);
                        uint16_t *gh = malloc(d * sizeof *gh);
                        for (uint64_t e = 0; e < d; ++e) {
                            float x = ((int32_t)lcg(&seed) / 2147483648.0f);
                            x = x * x * x * 3.0f;
                            if (e % 97 == 5) x = NAN;
                            if (e % 101 == 7) x = -INFINITY;
                            gf[e] = x;
                            uint32_t u; memcpy(&u, &x, 4); gh[e] = (uint16_t)(u >> 16);
                        }
                        const void *g = dtype == TQO_F32 ? (const void *)gf : (const void *)gh;
                        tqo_stats_t *S = malloc(nb * sizeof *S);
                        if (tqo_stats(g, dtype, d, be, 0.01f, S)) return 2;
                        tqo_params_t *P[3];
                        uint8_t *pay[3];
                        const uint64_t pb = tqo_payload_bytes(d, bits);
                        for (int w = 0; w < 3; ++w) {
                            P[w] = malloc(nb * sizeof **P);
                            for (uint64_t b = 0; b < nb; ++b) make_params(&P[w][b], bits, grid, 0.5f + 0.25f * w);
                            pay[w] = malloc(pb);                  /* exactly the documented size */
                            if (tqo_compress(g, dtype, d, be, P[w], 77 + w, (uint32_t)w, 3, pay[w])) return 3;
                        }
                        float *out = malloc(d * sizeof *out), *theta = calloc(d, sizeof *theta),
                              *vel = calloc(d, sizeof *vel);
                        const float wts[3] = {0.5f, 0.25f, 0.25f};
                        if (tqo_decompress_aggregate((const uint8_t *const *)pay, (const tqo_params_t *const *)P, NULL,
                                                     3, d, be, bits, 0, out)) return 4;
                        if (tqo_decompress_aggregate((const uint8_t *const *)pay, (const tqo_params_t *const *)P, wts,
                                                     3, d, be, bits, 1, out)) return 5;
                        if (tqo_decompress_aggregate_update((const uint8_t *const *)pay,
                                                            (const tqo_params_t *const *)P, NULL, 3, d, be, bits,
                                                            0.1f, 0.9f, 5e-4f, theta, vel)) return 6;
                        if (tqo_dequantize(pay[0], P[0], d, be, bits, out)) return 7;
                        uint32_t cnt[16];
                        tqo_enumerate_draws(gf[0], &P[0][0], 0, cnt);
                        tqo_enumerate_draws(gf[d - 1], &P[0][nb - 1], 1, cnt);
                        for (int w = 0; w < 3; ++w) { free(P[w]); free(pay[w]); }
                        free(out); free(theta); free(vel); free(S); free(gf); free(gh);
                        ++cases;
                    }
    printf("ok %llu cases\n", cases);
    return 0;
}
