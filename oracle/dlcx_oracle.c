/*
 * CPU oracle for the DiLoCoX outer step (arXiv 2506.21263).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, single-threaded, plainly
 * written definition that the GPU library is checked against.  It shares no
 * code, header, table or helper with the HIP library, and nothing on the
 * product path may call it.
 *
 * Conventions
 *   - A weight matrix is m x n, row-major, fp32 ("delta[i*n + j]").
 *   - A factor (P: m x r, Q: n x r) is stored column by column: column c of a
 *     factor of length len occupies f[c*len .. c*len+len).  Quantisation groups
 *     are `group` consecutive elements of one column.
 *   - Every inner product, norm and elementwise formula is evaluated in fp64
 *     from the fp32 operands and rounded once to fp32 when stored.
 *   - The quantiser takes its integer decisions in fp32 (the precision the
 *     payload is defined in), with IEEE divide, multiply and round-half-even.
 *
 * Parity status of each function against something other than itself is
 * listed in tests/test_oracle_pins.py; the only unpinned quantity is the
 * absolute value of the decompressed average with quantisation switched on
 * (the paper prints no worked example) -- "parity unpinned" for that value,
 * bounded by the half-step property only.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_F32 0
#define ORC_BF16 1

static float bf16_to_f32(uint16_t h)
{
    uint32_t u = ((uint32_t)h) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* ---------------------------------------------------------------------------
 * Pseudo-gradient with error compensation (Alg. 2, the line that forms
 * delta^t_{i,j}; Appendix A.3, first display):
 *     delta = (theta_global - theta_local) + e
 * theta_l is fp32 or bf16 (bf16 widened exactly).  delta may alias e.
 * ------------------------------------------------------------------------- */
void orc_delta_ef(const float *theta_g, const void *theta_l, int theta_l_dtype,
                  const float *e, float *delta, int64_t numel)
{
    for (int64_t x = 0; x < numel; ++x) {
        double tl = (theta_l_dtype == ORC_BF16)
                        ? (double)bf16_to_f32(((const uint16_t *)theta_l)[x])
                        : (double)((const float *)theta_l)[x];
        double d = ((double)theta_g[x] - tl) + (double)e[x];
        delta[x] = (float)d;
    }
}

/* ---------------------------------------------------------------------------
 * LOWRANK step 1 (Alg. 1 step (1), in the shared-basis power-iteration form
 * of the low-rank method the paper cites):  P = M * Q_in.
 *   M    : m x n row-major
 *   q_in : n x r, column-major (column c at q_in + c*n)
 *   p    : m x r, column-major (column c at p + c*m)
 * ------------------------------------------------------------------------- */
void orc_project_p(int64_t m, int64_t n, int r, const float *M,
                   const float *q_in, float *p)
{
    for (int c = 0; c < r; ++c) {
        const float *qc = q_in + (int64_t)c * n;
        for (int64_t i = 0; i < m; ++i) {
            const float *row = M + i * n;
            double acc = 0.0;
            for (int64_t j = 0; j < n; ++j)
                acc += (double)row[j] * (double)qc[j];
            p[(int64_t)c * m + i] = (float)acc;
        }
    }
}

/* LOWRANK step 2:  Q = M^T * P_hat  (P_hat m x r column-major, Q n x r). */
void orc_project_q(int64_t m, int64_t n, int r, const float *M,
                   const float *p_hat, float *q)
{
    double *acc = (double *)malloc(sizeof(double) * (size_t)n);
    for (int c = 0; c < r; ++c) {
        const float *pc = p_hat + (int64_t)c * m;
        for (int64_t j = 0; j < n; ++j)
            acc[j] = 0.0;
        for (int64_t i = 0; i < m; ++i) {
            const float *row = M + i * n;
            double pv = (double)pc[i];
            for (int64_t j = 0; j < n; ++j)
                acc[j] += (double)row[j] * pv;
        }
        for (int64_t j = 0; j < n; ++j)
            q[(int64_t)c * n + j] = (float)acc[j];
    }
    free(acc);
}

/* Column j0 only of Q = M^T P_hat: q_row[c] = sum_i M[i][j0] * p_hat[c][i].
 * Lets a test check single outputs of a matrix too large to sweep. */
void orc_project_q_row(int64_t m, int64_t n, int r, const float *M,
                       const float *p_hat, int64_t j0, float *q_row)
{
    for (int c = 0; c < r; ++c) {
        const float *pc = p_hat + (int64_t)c * m;
        double acc = 0.0;
        for (int64_t i = 0; i < m; ++i)
            acc += (double)M[i * n + j0] * (double)pc[i];
        q_row[c] = (float)acc;
    }
}

/* Decompression:  M_hat = P_hat * Q_bar^T  (rank-r reconstruction). */
void orc_reconstruct(int64_t m, int64_t n, int r, const float *p_hat,
                     const float *q_bar, float *m_hat)
{
    for (int64_t i = 0; i < m; ++i)
        for (int64_t j = 0; j < n; ++j) {
            double acc = 0.0;
            for (int c = 0; c < r; ++c)
                acc += (double)p_hat[(int64_t)c * m + i] *
                       (double)q_bar[(int64_t)c * n + j];
            m_hat[i * n + j] = (float)acc;
        }
}

/* ---------------------------------------------------------------------------
 * Thin-QR Q-factor with positive diagonal of R, by modified Gram-Schmidt with
 * one re-orthogonalisation pass, fp64 throughout.  A column whose residual
 * norm is <= 1e-6 of its original norm (or whose original norm is 0) becomes
 * the zero column, so an all-zero input gives an all-zero output.
 * In place on p (m x r column-major).
 * ------------------------------------------------------------------------- */
void orc_orthonormalize(int64_t m, int r, float *p)
{
    double *Q = (double *)malloc(sizeof(double) * (size_t)m * (size_t)r);
    char *dead = (char *)calloc((size_t)r, 1);
    for (int c = 0; c < r; ++c) {
        double *v = Q + (int64_t)c * m;
        double n0 = 0.0;
        for (int64_t i = 0; i < m; ++i) {
            v[i] = (double)p[(int64_t)c * m + i];
            n0 += v[i] * v[i];
        }
        n0 = sqrt(n0);
        for (int pass = 0; pass < 2; ++pass)
            for (int k = 0; k < c; ++k) {
                if (dead[k])
                    continue;
                const double *qk = Q + (int64_t)k * m;
                double dot = 0.0;
                for (int64_t i = 0; i < m; ++i)
                    dot += qk[i] * v[i];
                for (int64_t i = 0; i < m; ++i)
                    v[i] -= dot * qk[i];
            }
        double n1 = 0.0;
        for (int64_t i = 0; i < m; ++i)
            n1 += v[i] * v[i];
        n1 = sqrt(n1);
        if (n0 == 0.0 || n1 <= 1e-6 * n0) {
            dead[c] = 1;
            for (int64_t i = 0; i < m; ++i)
                v[i] = 0.0;
        } else {
            for (int64_t i = 0; i < m; ++i)
                v[i] /= n1;
        }
    }
    for (int64_t x = 0; x < (int64_t)m * r; ++x)
        p[x] = (float)Q[x];
    free(Q);
    free(dead);
}

/* ---------------------------------------------------------------------------
 * QUANTIZE (Alg. 1 step (2)): symmetric per-group absmax quantiser to q bits,
 * qmax = 2^(q-1) - 1, deterministic round-half-even.
 *   amax = max |x| over the group
 *   amax < 2^-100 : scale 0, all codes 0  (covers the all-zero group; the
 *               cut keeps qmax / amax finite)
 *   else      : inv = qmax / amax ; scale = amax / qmax   (fp32 divides)
 *               code = clamp(rint(x * inv), -qmax, qmax)  (fp32 multiply)
 * int8: one signed byte per element.  int4: element 2j in the low nibble of
 * byte j, element 2j+1 in the high nibble, two's-complement nibbles.
 * `count` elements in consecutive groups of `group` (count % group == 0).
 * ------------------------------------------------------------------------- */
void orc_quantize(const float *x, int64_t count, int qbits, int group,
                  uint8_t *codes, float *scales)
{
    const float qmax = (float)((1 << (qbits - 1)) - 1);
    for (int64_t g = 0; g < count / group; ++g) {
        const float *xg = x + g * group;
        float amax = 0.0f;
        for (int k = 0; k < group; ++k) {
            float a = fabsf(xg[k]);
            if (a > amax)
                amax = a;
        }
        float inv = 0.0f, scale = 0.0f;
        if (amax >= 0x1p-100f) {
            inv = qmax / amax;
            scale = amax / qmax;
        }
        scales[g] = scale;
        for (int k = 0; k < group; ++k) {
            float scaled = xg[k] * inv; /* one fp32 multiply */
            float rn = rintf(scaled);            /* half-to-even */
            if (rn > qmax)
                rn = qmax;
            if (rn < -qmax)
                rn = -qmax;
            int code = (int)rn;
            int64_t e = g * group + k;
            if (qbits == 8) {
                codes[e] = (uint8_t)(int8_t)code;
            } else {
                uint8_t nib = (uint8_t)(code & 0xF);
                if ((e & 1) == 0)
                    codes[e >> 1] = (uint8_t)((codes[e >> 1] & 0xF0) | nib);
                else
                    codes[e >> 1] = (uint8_t)((codes[e >> 1] & 0x0F) | (nib << 4));
            }
        }
    }
}

static int code_at(const uint8_t *codes, int64_t e, int qbits)
{
    if (qbits == 8)
        return (int)(int8_t)codes[e];
    int nib = (e & 1) ? (codes[e >> 1] >> 4) : (codes[e >> 1] & 0xF);
    return (nib & 0x8) ? nib - 16 : nib;
}

/* Dequantise one payload: x_hat = code * scale. */
void orc_dequantize(const uint8_t *codes, const float *scales, int64_t count,
                    int qbits, int group, float *x_hat)
{
    for (int64_t e = 0; e < count; ++e)
        x_hat[e] = (float)((double)code_at(codes, e, qbits) *
                           (double)scales[e / group]);
}

/* ---------------------------------------------------------------------------
 * The AllReduce-average of Alg. 2 over the D (= K) data-parallel workers,
 * Appendix A.3 second display:  mean_k dequant(payload_k), workers summed in
 * index order.
 * ------------------------------------------------------------------------- */
void orc_dequant_average(int K, const uint8_t *const *codes,
                         const float *const *scales, int64_t count, int qbits,
                         int group, float *mean_out)
{
    for (int64_t e = 0; e < count; ++e) {
        double acc = 0.0;
        for (int k = 0; k < K; ++k)
            acc += (double)code_at(codes[k], e, qbits) *
                   (double)scales[k][e / group];
        mean_out[e] = (float)(acc / (double)K);
    }
}

/* Error buffer of Alg. 2:  e <- delta_local - Delta_global.  In place. */
void orc_ef_update(float *ef_inout, const float *delta_hat, int64_t numel)
{
    for (int64_t x = 0; x < numel; ++x)
        ef_inout[x] = (float)((double)ef_inout[x] - (double)delta_hat[x]);
}

/* ---------------------------------------------------------------------------
 * OuterOpt: SGD with Nesterov momentum on the averaged pseudo-gradient
 * (the outer optimiser named in Appendix A.3; the displayed heavy-ball form
 * there has the sign of the opposite pseudo-gradient convention):
 *     v     <- mu * v + g
 *     theta <- theta - lr * (g + mu * v)
 * ------------------------------------------------------------------------- */
void orc_outer_nesterov(float *theta, float *v, const float *g, int64_t numel,
                        double lr, double mu)
{
    for (int64_t x = 0; x < numel; ++x) {
        double vn = mu * (double)v[x] + (double)g[x];
        double tn = (double)theta[x] - lr * ((double)g[x] + mu * vn);
        v[x] = (float)vn;
        theta[x] = (float)tn;
    }
}

/* ---------------------------------------------------------------------------
 * Eigenvalues of the r x r Gram matrix S = Q_bar^T Q_bar by the cyclic
 * two-sided Jacobi method in fp64, sorted in descending order into eig[0..r).
 * With P_hat orthonormal these are the squared singular values of the
 * decompressed average.
 * ------------------------------------------------------------------------- */
void orc_gram_eigenvalues(int64_t n, int r, const float *q_bar, double *eig)
{
    double *S = (double *)malloc(sizeof(double) * (size_t)r * (size_t)r);
    for (int a = 0; a < r; ++a)
        for (int b = a; b < r; ++b) {
            double acc = 0.0;
            for (int64_t j = 0; j < n; ++j)
                acc += (double)q_bar[(int64_t)a * n + j] *
                       (double)q_bar[(int64_t)b * n + j];
            S[a * r + b] = acc;
            S[b * r + a] = acc;
        }
    for (int sweep = 0; sweep < 60; ++sweep) {
        double off = 0.0, diag = 0.0;
        for (int a = 0; a < r; ++a) {
            diag += S[a * r + a] * S[a * r + a];
            for (int b = a + 1; b < r; ++b)
                off += S[a * r + b] * S[a * r + b];
        }
        if (off <= 1e-30 * diag || off == 0.0)
            break;
        for (int p = 0; p < r - 1; ++p)
            for (int q = p + 1; q < r; ++q) {
                double apq = S[p * r + q];
                if (apq == 0.0)
                    continue;
                double app = S[p * r + p], aqq = S[q * r + q];
                double theta = (aqq - app) / (2.0 * apq);
                double t = (theta >= 0.0 ? 1.0 : -1.0) /
                           (fabs(theta) + sqrt(theta * theta + 1.0));
                double c = 1.0 / sqrt(t * t + 1.0), s = t * c;
                for (int k = 0; k < r; ++k) { /* columns p, q */
                    double akp = S[k * r + p], akq = S[k * r + q];
                    S[k * r + p] = c * akp - s * akq;
                    S[k * r + q] = s * akp + c * akq;
                }
                for (int k = 0; k < r; ++k) { /* rows p, q */
                    double apk = S[p * r + k], aqk = S[q * r + k];
                    S[p * r + k] = c * apk - s * aqk;
                    S[q * r + k] = s * apk + c * aqk;
                }
            }
    }
    for (int a = 0; a < r; ++a)
        eig[a] = S[a * r + a];
    for (int a = 1; a < r; ++a) { /* insertion sort, descending */
        double key = eig[a];
        int b = a - 1;
        while (b >= 0 && eig[b] < key) {
            eig[b + 1] = eig[b];
            --b;
        }
        eig[b + 1] = key;
    }
    free(S);
}

/* ---------------------------------------------------------------------------
 * r'_t of Alg. 3 ("calculate r' with the globally averaged gradient"; the
 * paper gives no formula): the smallest k whose k largest eigenvalues carry
 * at least tau of the trace.  Returns 0 when the trace is 0 (the caller maps
 * that to its lower rank bound).  Negative round-off eigenvalues count as 0.
 * ------------------------------------------------------------------------- */
int orc_effective_rank(int64_t n, int r, const float *q_bar, double tau)
{
    double *eig = (double *)malloc(sizeof(double) * (size_t)r);
    orc_gram_eigenvalues(n, r, q_bar, eig);
    double total = 0.0;
    for (int a = 0; a < r; ++a) {
        if (eig[a] < 0.0)
            eig[a] = 0.0;
        total += eig[a];
    }
    int rp = 0;
    if (total > 0.0) {
        double cum = 0.0;
        rp = r;
        for (int a = 0; a < r; ++a) {
            cum += eig[a];
            if (cum >= tau * total) {
                rp = a + 1;
                break;
            }
        }
    }
    free(eig);
    return rp;
}

/* ---------------------------------------------------------------------------
 * Alg. 3 (AdaGradCmp), window rule.  hist[0..t) holds r'_1 .. r'_t (r'_1 is
 * defined as r_1 by the caller).  For t < c: r_t = r_1, H_t = H_1.  Otherwise
 * r_t = mean of the last c entries, alpha = (r_1 - r_t) / r_1, H_t = H_1*alpha,
 * exactly as printed.  The mean is rounded half-up and clamped to
 * [rmin, rmax]; H is rounded half-up and kept >= 1.
 * ------------------------------------------------------------------------- */
void orc_adagradcmp(const int32_t *hist, int32_t t, int32_t c, int32_t r1,
                    int32_t rmin, int32_t rmax, int32_t H1, int32_t *r_out,
                    int32_t *H_out)
{
    if (t < c) {
        *r_out = r1;
        *H_out = H1;
        return;
    }
    int64_t sum = 0;
    for (int32_t i = t - c; i < t; ++i)
        sum += hist[i];
    /* round-half-up of sum / c in integers */
    int32_t rt = (int32_t)((2 * sum + c) / (2 * (int64_t)c));
    if (rt < rmin)
        rt = rmin;
    if (rt > rmax)
        rt = rmax;
    double alpha = ((double)r1 - (double)rt) / (double)r1;
    int32_t H = (int32_t)floor((double)H1 * alpha + 0.5);
    if (H < 1)
        H = 1;
    *r_out = rt;
    *H_out = H;
}
