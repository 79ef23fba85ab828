/*
 * Memory and undefined-behaviour check of the CPU oracle (TEST INFRASTRUCTURE ONLY).
 *
 * Compiled together with dlcx_oracle.c under -fsanitize=address,undefined (oracle/build.py,
 * build_sanitized) into a small program that runs one outer step of Alg. 2 for several shapes,
 * ranks, group sizes and both payload widths through every function of the oracle.  Every array
 * is a heap block of exactly the size the oracle's contract states, so an access one element past
 * any input or output ends the program with a sanitizer report and a non-zero status.  It checks
 * no values (tests/test_oracle_pins.py does that); it prints "sanitize ok" and returns 0 when no
 * report was raised.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

void orc_delta_ef(const float *, const void *, int, const float *, float *, int64_t);
void orc_project_p(int64_t, int64_t, int, const float *, const float *, float *);
void orc_project_q(int64_t, int64_t, int, const float *, const float *, float *);
void orc_project_q_row(int64_t, int64_t, int, const float *, const float *, int64_t, float *);
void orc_reconstruct(int64_t, int64_t, int, const float *, const float *, float *);
void orc_orthonormalize(int64_t, int, float *);
void orc_quantize(const float *, int64_t, int, int, uint8_t *, float *);
void orc_dequantize(const uint8_t *, const float *, int64_t, int, int, float *);
void orc_dequant_average(int, const uint8_t *const *, const float *const *, int64_t, int, int,
                         float *);
void orc_ef_update(float *, const float *, int64_t);
void orc_outer_nesterov(float *, float *, const float *, int64_t, double, double);
void orc_gram_eigenvalues(int64_t, int, const float *, double *);
int orc_effective_rank(int64_t, int, const float *, double);
void orc_adagradcmp(const int32_t *, int32_t, int32_t, int32_t, int32_t, int32_t, int32_t,
                    int32_t *, int32_t *);

static uint64_t state = 0x2506212630000001ull;
static float rnd(void)
{ /* xorshift, values in (-1, 1) */
    state ^= state << 13;
    state ^= state >> 7;
    state ^= state << 17;
    return (float)((double)(state >> 11) / 9007199254740992.0 * 2.0 - 1.0);
}
static float *fresh(size_t count, float scale)
{
    float *p = (float *)malloc(sizeof(float) * (count ? count : 1));
    if (!p) exit(2);
    for (size_t i = 0; i < count; ++i) p[i] = scale * rnd();
    return p;
}

static void one_case(int64_t m, int64_t n, int r, int K, int qbits, int group, int bf16)
{
    const size_t mn = (size_t)m * (size_t)n;
    float *theta = fresh(mn, 0.02f), *v = fresh(mn, 0.0f), *q_in = fresh((size_t)r * n, 1.0f);
    float **delta = (float **)malloc(sizeof(float *) * (size_t)K);
    uint8_t **cp = (uint8_t **)malloc(sizeof(uint8_t *) * (size_t)K);
    uint8_t **cq = (uint8_t **)malloc(sizeof(uint8_t *) * (size_t)K);
    float **sp = (float **)malloc(sizeof(float *) * (size_t)K);
    float **sq = (float **)malloc(sizeof(float *) * (size_t)K);
    const size_t np = (size_t)r * m, nq = (size_t)r * n;
    float *p_bar = fresh(np, 0.0f), *q_bar = fresh(nq, 0.0f), *fac;
    for (int k = 0; k < K; ++k) {
        delta[k] = fresh(mn, 0.0f); /* e = 0 */
        if (bf16) {
            uint16_t *tl = (uint16_t *)malloc(sizeof(uint16_t) * mn);
            for (size_t i = 0; i < mn; ++i) tl[i] = (uint16_t)(0x3C00u + (unsigned)(i % 251));
            orc_delta_ef(theta, tl, 1, delta[k], delta[k], (int64_t)mn);
            free(tl);
        } else {
            float *tl = fresh(mn, 0.02f);
            orc_delta_ef(theta, tl, 0, delta[k], delta[k], (int64_t)mn);
            free(tl);
        }
        fac = fresh(np, 0.0f);
        orc_project_p(m, n, r, delta[k], q_in, fac);
        cp[k] = (uint8_t *)malloc(qbits == 4 ? np / 2 : np);
        sp[k] = (float *)malloc(sizeof(float) * (np / (size_t)group));
        orc_quantize(fac, (int64_t)np, qbits, group, cp[k], sp[k]);
        orc_dequantize(cp[k], sp[k], (int64_t)np, qbits, group, fac);
        free(fac);
    }
    orc_dequant_average(K, (const uint8_t *const *)cp, (const float *const *)sp, (int64_t)np, qbits,
                        group, p_bar);
    orc_orthonormalize(m, r, p_bar);
    for (int k = 0; k < K; ++k) {
        fac = fresh(nq, 0.0f);
        orc_project_q(m, n, r, delta[k], p_bar, fac);
        float *row = fresh((size_t)r, 0.0f);
        orc_project_q_row(m, n, r, delta[k], p_bar, n - 1, row);
        free(row);
        cq[k] = (uint8_t *)malloc(qbits == 4 ? nq / 2 : nq);
        sq[k] = (float *)malloc(sizeof(float) * (nq / (size_t)group));
        orc_quantize(fac, (int64_t)nq, qbits, group, cq[k], sq[k]);
        free(fac);
    }
    orc_dequant_average(K, (const uint8_t *const *)cq, (const float *const *)sq, (int64_t)nq, qbits,
                        group, q_bar);
    float *d_hat = fresh(mn, 0.0f);
    orc_reconstruct(m, n, r, p_bar, q_bar, d_hat);
    for (int k = 0; k < K; ++k) orc_ef_update(delta[k], d_hat, (int64_t)mn);
    orc_outer_nesterov(theta, v, d_hat, (int64_t)mn, 0.7, 0.9);
    double *eig = (double *)malloc(sizeof(double) * (size_t)r);
    orc_gram_eigenvalues(n, r, q_bar, eig);
    (void)orc_effective_rank(n, r, q_bar, 0.99);
    free(eig);
    free(d_hat);
    for (int k = 0; k < K; ++k) {
        free(delta[k]); free(cp[k]); free(cq[k]); free(sp[k]); free(sq[k]);
    }
    free(delta); free(cp); free(cq); free(sp); free(sq);
    free(theta); free(v); free(q_in); free(p_bar); free(q_bar);
}

int main(void)
{
    one_case(64, 48, 5, 2, 4, 16, 0);     /* odd rank, smallest group */
    one_case(128, 256, 32, 3, 8, 64, 1);  /* int8, bf16 replicas */
    one_case(256, 128, 1, 1, 4, 128, 1);  /* rank one, one worker */
    one_case(32, 32, 32, 2, 4, 32, 0);    /* full rank */
    {   /* all-zero pseudo-gradient: dead columns, zero groups, zero trace */
        float *z = (float *)calloc(64 * 64, sizeof(float)), *f = (float *)calloc(4 * 64, sizeof(float));
        uint8_t *c = (uint8_t *)malloc(4 * 64 / 2);
        float *s = (float *)malloc(sizeof(float) * 4 * 64 / 16);
        orc_orthonormalize(64, 4, f);
        orc_quantize(f, 4 * 64, 4, 16, c, s);
        (void)orc_effective_rank(64, 4, f, 0.99);
        free(z); free(f); free(c); free(s);
    }
    {   /* window rule over its whole history */
        int32_t hist[12] = {256, 256, 256, 256, 241, 49, 3, 3, 4, 4, 4, 4}, r = 0, H = 0;
        for (int32_t t = 1; t <= 12; ++t) orc_adagradcmp(hist, t, 5, 256, 4, 256, 125, &r, &H);
        if (r < 4 || r > 256 || H < 1) return 3;
    }
    puts("sanitize ok");
    return 0;
}
