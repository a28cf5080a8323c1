/* Host-only driver for the sanitizer test: the oracle's arithmetic (oracle/update.c) on ragged
 * lengths, including 0 and 1, with every buffer sized exactly - built with
 * -fsanitize=address,undefined, so that a read or write one element too far is caught. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

void orc_fold_bf16(const uint16_t *const *src, int P, int group_len, int64_t n, float *out);
void orc_fold_f32(const float *const *src, int P, int group_len, int64_t n, float *out);
double orc_sumsq(const float *g, int64_t n);
double orc_clip_coef(double total_sumsq, float grad_scale, float max_norm);
void orc_adam64(int64_t n, const float *g, float *p, float *m, float *v, double sc, float lr, float beta1,
                float beta2, float eps, float wd, int step, int adamw);
void orc_adam32(int64_t n, const float *g, float *p, float *m, float *v, double sc, float lr, float beta1,
                float beta2, float eps, float wd, int step, int adamw);
void orc_bf16_rne(const float *p, int64_t n, uint16_t *out);
void orc_f16_rne(const float *p, int64_t n, uint16_t *out);

static uint32_t rng_state = 12345u;
static uint32_t rnd(void) { rng_state = rng_state * 1664525u + 1013904223u; return rng_state; }

int main(void) {
    const int64_t lens[] = {0, 1, 7, 8, 255, 65536, 65537, 200001};
    const int shapes[][2] = {{1, 1}, {4, 2}, {6, 6}, {16, 8}, {9, 1}};
    double acc = 0.0;
    for (unsigned li = 0; li < sizeof lens / sizeof lens[0]; ++li) {
        const int64_t n = lens[li];
        for (unsigned si = 0; si < sizeof shapes / sizeof shapes[0]; ++si) {
            const int P = shapes[si][0], gl = shapes[si][1];
            uint16_t **hb = malloc((size_t)P * sizeof *hb);
            float **fb = malloc((size_t)P * sizeof *fb);
            for (int q = 0; q < P; ++q) {
                hb[q] = malloc((size_t)n * sizeof(uint16_t) + 1);          /* exact size (+1 so that n = 0 allocates) */
                fb[q] = malloc((size_t)n * sizeof(float) + 1);
                for (int64_t e = 0; e < n; ++e) {
                    hb[q][e] = (uint16_t)(rnd() >> 16);                    /* any bit pattern: NaN and inf included */
                    uint32_t u = rnd();
                    memcpy(&fb[q][e], &u, 4);
                }
            }
            float *g = malloc((size_t)n * 4 + 1), *p = malloc((size_t)n * 4 + 1), *m = malloc((size_t)n * 4 + 1),
                  *v = malloc((size_t)n * 4 + 1);
            uint16_t *q16 = malloc((size_t)n * 2 + 1);
            orc_fold_bf16((const uint16_t *const *)hb, P, gl, n, g);
            acc += orc_sumsq(g, n) > 0 ? 1 : 0;
            orc_fold_f32((const float *const *)fb, P, gl, n, g);
            for (int64_t e = 0; e < n; ++e) {
                g[e] = (float)((int32_t)(rnd() >> 8) - (1 << 23)) * 1e-9f;
                p[e] = (float)((int32_t)(rnd() >> 8) - (1 << 23)) * 1e-8f;
                m[e] = 0.0f;
                v[e] = 0.0f;
            }
            const double coef = orc_clip_coef(orc_sumsq(g, n), 0.25f, 1e-3f);
            for (int step = 1; step <= 2; ++step) {
                orc_adam64(n, g, p, m, v, 0.25 * coef, 1e-4f, 0.9f, 0.999f, 1e-8f, 0.01f, step, step & 1);
                orc_adam32(n, g, p, m, v, 0.25 * coef, 1e-4f, 0.9f, 0.999f, 1e-8f, 0.01f, step, step & 1);
            }
            orc_bf16_rne(p, n, q16);
            orc_f16_rne(p, n, q16);
            orc_bf16_rne(fb[0], n, q16);                                   /* every kind of bit pattern through the packs */
            orc_f16_rne(fb[0], n, q16);
            if (n) acc += q16[n - 1] + (isnan(p[n - 1]) ? 0.0 : p[n - 1]);
            for (int q = 0; q < P; ++q) { free(hb[q]); free(fb[q]); }
            free(hb); free(fb); free(g); free(p); free(m); free(v); free(q16);
        }
    }
    printf("oracle sanitizer run ok (%g)\n", acc);
    return 0;
}
