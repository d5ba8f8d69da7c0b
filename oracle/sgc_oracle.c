/*
 * CPU oracle for the per-step hot path of Sparse Gradient Compression (SGC).
 *
 * THIS FILE IS TEST INFRASTRUCTURE. It is a plain, slow, single-threaded
 * restatement of what the method computes (paper Sec. 4.2-4.4, Alg. 2, eq. 5-11,
 * and the definition of OMP in Sec. 4.3 / App. B), used only by the tests, the
 * smoke check and the cpu_baseline leg of the benchmark. It shares no code with
 * the HIP library and the product path never calls it.
 *
 * Conventions
 *   - "At" is the measurement matrix stored transposed: At[i*r + j] = A[j][i],
 *     so row i of At is column i of A (length r, contiguous).
 *   - every accumulation is done in double; results are rounded to float only
 *     where the method stores a float.
 *   - chunks are independent (MESGC, Sec. 4.4): every batched function is a plain
 *     loop over chunks.
 *
 * Pins (see tests/test_oracle_*.py): full-sort brute force for top-k; dense
 * float64 mat-vec for the projection; published Philox4x32-10 known-answer
 * vectors and an exact Box-Muller evaluation for the generated matrix; the
 * closed form of the first Adam step; exact sparse recovery, exhaustive
 * support search and least-squares identities for OMP; a library least-squares
 * routine and exact joint recovery for the shared-support fit; a dense mat-vec
 * and the eq. 10 invariant across a change of matrix for the re-projection; the
 * closed form of the first full step in the exact-recovery regime; for the
 * outer projection of CESGC a hand-worked example, a library matrix product,
 * the identity projection (which must reproduce the plain update) and the
 * projector identities of a matrix with orthonormal rows.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------ */
/* Sparsify_s (Sec. 4.2; chunk-wise in Def. 1): keep the k entries of largest */
/* magnitude. Order of magnitudes is taken on the bit pattern with the sign   */
/* cleared (identical to comparing |g| for finite values, makes +0/-0 tie);   */
/* among equal magnitudes the lower position wins; output ascending position. */
/* ------------------------------------------------------------------------ */
typedef struct {
    uint32_t key;
    int32_t pos;
} mag_pos;

static int by_mag_desc_pos_asc(const void *a, const void *b)
{
    const mag_pos *x = (const mag_pos *)a, *y = (const mag_pos *)b;
    if (x->key != y->key)
        return x->key > y->key ? -1 : 1;
    return x->pos < y->pos ? -1 : (x->pos > y->pos ? 1 : 0);
}

static int by_pos_asc(const void *a, const void *b)
{
    const mag_pos *x = (const mag_pos *)a, *y = (const mag_pos *)b;
    return x->pos < y->pos ? -1 : (x->pos > y->pos ? 1 : 0);
}

static float f32_from_bits(uint32_t u)
{
    float f;
    memcpy(&f, &u, 4);
    return f;
}

static uint32_t bits_from_f32(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    return u;
}

/* g: [C][d] float, idx: [C][k] chunk-local positions, val: [C][k] signed values */
int oracle_topk_f32(const float *g, int64_t C, int32_t d, int32_t k, int32_t *idx, float *val)
{
    if (k < 0 || k > d)
        return -1;
    mag_pos *w = (mag_pos *)malloc(sizeof(mag_pos) * (size_t)(d > 0 ? d : 1));
    if (!w)
        return -2;
    for (int64_t c = 0; c < C; ++c) {
        const float *gc = g + c * (int64_t)d;
        for (int32_t i = 0; i < d; ++i) {
            w[i].key = bits_from_f32(gc[i]) & 0x7fffffffu;
            w[i].pos = i;
        }
        qsort(w, (size_t)d, sizeof(mag_pos), by_mag_desc_pos_asc);
        qsort(w, (size_t)k, sizeof(mag_pos), by_pos_asc);
        for (int32_t t = 0; t < k; ++t) {
            idx[c * k + t] = w[t].pos;
            val[c * k + t] = gc[w[t].pos];
        }
    }
    free(w);
    return 0;
}

/* same for bfloat16 inputs given as raw 16-bit patterns; values widen exactly */
int oracle_topk_bf16(const uint16_t *g, int64_t C, int32_t d, int32_t k, int32_t *idx, float *val)
{
    if (k < 0 || k > d)
        return -1;
    mag_pos *w = (mag_pos *)malloc(sizeof(mag_pos) * (size_t)(d > 0 ? d : 1));
    if (!w)
        return -2;
    for (int64_t c = 0; c < C; ++c) {
        const uint16_t *gc = g + c * (int64_t)d;
        for (int32_t i = 0; i < d; ++i) {
            w[i].key = (uint32_t)(gc[i] & 0x7fffu);
            w[i].pos = i;
        }
        qsort(w, (size_t)d, sizeof(mag_pos), by_mag_desc_pos_asc);
        qsort(w, (size_t)k, sizeof(mag_pos), by_pos_asc);
        for (int32_t t = 0; t < k; ++t) {
            idx[c * k + t] = w[t].pos;
            val[c * k + t] = f32_from_bits((uint32_t)gc[w[t].pos] << 16);
        }
    }
    free(w);
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Projection (eq. 5-6, Alg. 2 line 1): p = A*Sparsify(G), q = A*Sparsify(G^2) */
/* The square of a kept value is formed in float (it is the value a float     */
/* gradient-squared tensor would hold) and then widened.                      */
/* ------------------------------------------------------------------------ */
int oracle_project(const int32_t *idx, const float *val, int64_t C, int32_t k, const float *At,
                   int32_t d, int32_t r, float *p, float *q)
{
    for (int64_t c = 0; c < C; ++c) {
        for (int32_t j = 0; j < r; ++j) {
            double sp = 0.0, sq = 0.0;
            for (int32_t t = 0; t < k; ++t) {
                int32_t i = idx[c * k + t];
                if (i < 0 || i >= d)
                    return -1;
                double a = (double)At[(int64_t)i * r + j];
                float v = val[c * k + t];
                float v2 = v * v;
                sp += a * (double)v;
                sq += a * (double)v2;
            }
            p[c * r + j] = (float)sp;
            if (q)
                q[c * r + j] = (float)sq;
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Measurement matrix from a counter-based stream (Sec. 4.3: entries iid      */
/* zero-mean normal, standard deviation 1/sqrt(r)).                           */
/*                                                                            */
/* Philox4x32-10 (Salmon et al., SC'11) with key = (seed low, seed high) and  */
/* counter = (i, j/4, 0, 0) yields four 32-bit words for rows 4*(j/4)..+3 of  */
/* column i of A. Words (0,1) and (2,3) each feed one Box-Muller pair. The    */
/* transform is specified in float with explicitly fused multiply-adds and    */
/* fixed polynomials, so that every IEEE-754 implementation produces the same */
/* bits.                                                                      */
/* ------------------------------------------------------------------------ */
static void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                          uint32_t k1, uint32_t out[4])
{
    for (int round = 0; round < 10; ++round) {
        uint64_t m0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
        uint64_t m1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        uint32_t n0 = (uint32_t)(m1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)m1;
        uint32_t n2 = (uint32_t)(m0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)m0;
        c0 = n0;
        c1 = n1;
        c2 = n2;
        c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0;
    out[1] = c1;
    out[2] = c2;
    out[3] = c3;
}

void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    philox4x32_10(ctr[0], ctr[1], ctr[2], ctr[3], key[0], key[1], out);
}

/* t = -2 ln(u), u = n * 2^-24 with n an odd integer in [1, 2^24) */
static float neg2_ln_unit(uint32_t n)
{
    float f = (float)n; /* exact */
    uint32_t b = bits_from_f32(f);
    int32_t e = (int32_t)(b >> 23) - 127;
    uint32_t man = b & 0x7fffffu;
    float m;
    if (man > 0x3504f3u) { /* m > sqrt(2): halve it */
        m = f32_from_bits(man | 0x3f000000u);
        e += 1;
    } else {
        m = f32_from_bits(man | 0x3f800000u);
    }
    float s = m - 1.0f; /* exact */
    float qv = -0x1.4237fep-4f;
    qv = fmaf(qv, s, 0x1.0696e4p-3f);
    qv = fmaf(qv, s, -0x1.0c524cp-3f);
    qv = fmaf(qv, s, 0x1.22973ap-3f);
    qv = fmaf(qv, s, -0x1.548882p-3f);
    qv = fmaf(qv, s, 0x1.99a3ecp-3f);
    qv = fmaf(qv, s, -0x1.000206p-2f);
    qv = fmaf(qv, s, 0x1.55554ep-2f);
    qv = fmaf(qv, s, -0x1.fffffep-2f);
    float s2 = s * s;
    float lnm = fmaf(s2, qv, s);
    float ef = (float)(e - 24);
    float ln_u = fmaf(ef, 0x1.62e430p-1f, lnm);
    return -2.0f * ln_u;
}

/* (cos, sin) of the angle oct*pi/4 + (pi/4)*(f + 0.5)/2^23, where oct is the top three
 * bits of w and f the next 23 bits: a uniform angle on a grid of 2^26 points */
static void unit_circle(uint32_t w, float *c_out, float *s_out)
{
    uint32_t oct = w >> 29;
    uint32_t n = (((w >> 6) & 0x7fffffu) << 1) | 1u; /* odd, < 2^24 */
    if (oct & 1u)
        n = 0x1000000u - n;
    float ph = (float)n * 0x1.0p-24f; /* fraction of the octant, exact */
    float u = ph * ph;
    float sp = -0x1.2d9b7cp-15f;
    sp = fmaf(sp, u, 0x1.465ec4p-9f);
    sp = fmaf(sp, u, -0x1.4abbbap-4f);
    sp = fmaf(sp, u, 0x1.921fb6p-1f);
    float sn = sp * ph;
    float cs = -0x1.4e5e6ep-12f;
    cs = fmaf(cs, u, 0x1.03af5ap-6f);
    cs = fmaf(cs, u, -0x1.3bd392p-2f);
    cs = fmaf(cs, u, 1.0f);
    float c = cs, s = sn;
    if ((oct + 1u) & 2u) { /* octants 1,2,5,6 */
        c = sn;
        s = cs;
    }
    if ((oct + 2u) & 4u) /* octants 2,3,4,5 */
        c = -c;
    if (oct & 4u)
        s = -s;
    *c_out = c;
    *s_out = s;
}

static void normal_pair(uint32_t w0, uint32_t w1, float scale, float *z0, float *z1)
{
    uint32_t n = ((w0 >> 9) << 1) | 1u;
    float t = neg2_ln_unit(n);
    float rad = sqrtf(t) * scale;
    float c, s;
    unit_circle(w1, &c, &s);
    *z0 = rad * c;
    *z1 = rad * s;
}

/* exposed for the tests: the float transform of one pair and its inputs */
void oracle_normal_pair(uint32_t w0, uint32_t w1, float scale, float out[2])
{
    normal_pair(w0, w1, scale, &out[0], &out[1]);
}

/* rows [i0, i0+rows) of At (each of length r, r a multiple of 4) into out[rows][r];
 * scale = (float)(1/sqrt((double)r)) */
int oracle_philox_matrix(uint64_t seed, int32_t r, int64_t i0, int64_t rows, float *out)
{
    if (r <= 0 || (r & 3))
        return -1;
    float scale = (float)(1.0 / sqrt((double)r));
    uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
    for (int64_t ii = 0; ii < rows; ++ii) {
        uint32_t i = (uint32_t)(i0 + ii);
        for (int32_t jb = 0; jb < r / 4; ++jb) {
            uint32_t w[4];
            philox4x32_10(i, (uint32_t)jb, 0u, 0u, k0, k1, w);
            float *o = out + ii * r + 4 * jb;
            normal_pair(w[0], w[1], scale, &o[0], &o[1]);
            normal_pair(w[2], w[3], scale, &o[2], &o[3]);
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Compressed AdamW moments (eq. 7-8 with beta2 in the second, Alg. 2 lines   */
/* 2-5). The stored state is the uncorrected moment; the bias-corrected       */
/* moments are separate outputs handed to the recovery.                       */
/* ------------------------------------------------------------------------ */
int oracle_adam(const float *p, const float *q, float *m, float *v, float *mhat, float *vhat,
                int64_t n, int32_t step, double beta1, double beta2)
{
    if (step < 1)
        return -1;
    double b1 = beta1, b2 = beta2;
    double c1 = 1.0 - pow(b1, (double)step), c2 = 1.0 - pow(b2, (double)step);
    for (int64_t i = 0; i < n; ++i) {
        double mn = b1 * (double)m[i] + (1.0 - b1) * (double)p[i];
        double vn = b2 * (double)v[i] + (1.0 - b2) * (double)q[i];
        m[i] = (float)mn;
        v[i] = (float)vn;
        mhat[i] = (float)(mn / c1);
        vhat[i] = (float)(vn / c2);
    }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* OMP (Sec. 4.3 eq. 9; selection rule and output as in App. B): greedy       */
/* k-sparse recovery of x from y = A x.                                       */
/*   repeat k times:                                                          */
/*     corr_i = <A_:i, res>;  lambda = argmax over unselected i of            */
/*              |corr_i| / ||A_:i||   (lowest i among exact ties)             */
/*     x = argmin || y - A_Lambda x ||_2   (normal equations, Cholesky)       */
/*     res = y - A_Lambda x                                                   */
/* The first n_forced selections can be dictated by the caller (used to check */
/* a single selection of a long run without repeating the whole run).         */
/* ------------------------------------------------------------------------ */
void oracle_colnorms(const float *At, int32_t d, int32_t r, double *norm)
{
    for (int32_t i = 0; i < d; ++i) {
        double s = 0.0;
        for (int32_t j = 0; j < r; ++j) {
            double a = (double)At[(int64_t)i * r + j];
            s += a * a;
        }
        norm[i] = sqrt(s);
    }
}

/* solve G x = b for symmetric positive definite G (n x n, row-major, leading
 * dimension ld) by Cholesky; returns nonzero if a pivot is not positive */
static int spd_solve(const double *G, int32_t ld, int32_t n, const double *b, double *x,
                     double *L /* n*n scratch */)
{
    for (int32_t i = 0; i < n; ++i) {
        for (int32_t j = 0; j <= i; ++j) {
            double s = G[i * ld + j];
            for (int32_t t = 0; t < j; ++t)
                s -= L[i * n + t] * L[j * n + t];
            if (i == j) {
                if (!(s > 0.0))
                    return 1;
                L[i * n + i] = sqrt(s);
            } else {
                L[i * n + j] = s / L[j * n + j];
            }
        }
    }
    for (int32_t i = 0; i < n; ++i) { /* L w = b */
        double s = b[i];
        for (int32_t t = 0; t < i; ++t)
            s -= L[i * n + t] * x[t];
        x[i] = s / L[i * n + i];
    }
    for (int32_t i = n - 1; i >= 0; --i) { /* L^T x = w */
        double s = x[i];
        for (int32_t t = i + 1; t < n; ++t)
            s -= L[t * n + i] * x[t];
        x[i] = s / L[i * n + i];
    }
    return 0;
}

/*
 * y[r]; At[d][r]; norm[d] column norms (from oracle_colnorms) or NULL;
 * forced[n_forced] dictated first selections (n_forced may be 0);
 * outputs: sel[k] in selection order, x[k] aligned with sel (float),
 * x64[k] (may be NULL), res_out[r] final residual (may be NULL),
 * top2[2*k] (may be NULL): per iteration the best and second-best score among
 * the unselected positions (for tie diagnostics).
 * returns 0, or a negative code on a bad argument / singular support.
 */
int oracle_omp(const float *y, const float *At, int32_t d, int32_t r, int32_t k,
               const double *norm, const int32_t *forced, int32_t n_forced, int32_t *sel, float *x,
               double *x64, double *res_out, double *top2)
{
    if (k < 0 || k > d || k > r || n_forced > k)
        return -1;
    int rc = 0;
    double *nrm = NULL;
    if (!norm) {
        nrm = (double *)malloc(sizeof(double) * (size_t)d);
        oracle_colnorms(At, d, r, nrm);
        norm = nrm;
    }
    size_t kk = (size_t)(k > 0 ? k : 1);
    double *res = (double *)malloc(sizeof(double) * (size_t)r);
    double *G = (double *)calloc(kk * kk, sizeof(double));
    double *L = (double *)calloc(kk * kk, sizeof(double));
    double *b = (double *)calloc(kk, sizeof(double));
    double *xs = (double *)calloc(kk, sizeof(double));
    unsigned char *taken = (unsigned char *)calloc((size_t)d, 1);
    for (int32_t j = 0; j < r; ++j)
        res[j] = (double)y[j];

    for (int32_t it = 0; it < k; ++it) {
        int32_t lam = -1;
        double best = -1.0, second = -1.0;
        if (it >= n_forced || top2) {
            for (int32_t i = 0; i < d; ++i) {
                if (taken[i])
                    continue;
                const float *a = At + (int64_t)i * r;
                double corr = 0.0;
                for (int32_t j = 0; j < r; ++j)
                    corr += (double)a[j] * res[j];
                double score = norm[i] > 0.0 ? fabs(corr) / norm[i] : 0.0;
                if (score > best) {
                    second = best;
                    best = score;
                    lam = i;
                } else if (score > second) {
                    second = score;
                }
            }
            if (top2) {
                top2[2 * it] = best;
                top2[2 * it + 1] = second;
            }
        }
        if (it < n_forced)
            lam = forced[it];
        if (lam < 0 || lam >= d || taken[lam]) {
            rc = -3;
            break;
        }
        taken[lam] = 1;
        sel[it] = lam;

        /* extend the Gram matrix of the support and the right-hand side A_L^T y */
        const float *an = At + (int64_t)lam * r;
        for (int32_t t = 0; t <= it; ++t) {
            const float *at = At + (int64_t)sel[t] * r;
            double s = 0.0;
            for (int32_t j = 0; j < r; ++j)
                s += (double)an[j] * (double)at[j];
            G[(size_t)it * kk + t] = s;
            G[(size_t)t * kk + it] = s;
        }
        double by = 0.0;
        for (int32_t j = 0; j < r; ++j)
            by += (double)an[j] * (double)y[j];
        b[it] = by;

        if (spd_solve(G, (int32_t)kk, it + 1, b, xs, L)) {
            rc = -4;
            break;
        }
        for (int32_t j = 0; j < r; ++j)
            res[j] = (double)y[j];
        for (int32_t t = 0; t <= it; ++t) {
            const float *at = At + (int64_t)sel[t] * r;
            double xt = xs[t];
            for (int32_t j = 0; j < r; ++j)
                res[j] -= xt * (double)at[j];
        }
    }
    if (rc == 0) {
        for (int32_t t = 0; t < k; ++t) {
            x[t] = (float)xs[t];
            if (x64)
                x64[t] = xs[t];
        }
        if (res_out)
            memcpy(res_out, res, sizeof(double) * (size_t)r);
    }
    free(res);
    free(G);
    free(L);
    free(b);
    free(xs);
    free(taken);
    free(nrm);
    return rc;
}

/* batched form: N right-hand sides sharing A */
int oracle_omp_batch(const float *y, int32_t N, const float *At, int32_t d, int32_t r, int32_t k,
                     int32_t *sel, float *x)
{
    double *norm = (double *)malloc(sizeof(double) * (size_t)d);
    oracle_colnorms(At, d, r, norm);
    int rc = 0;
    for (int32_t n = 0; n < N && rc == 0; ++n)
        rc = oracle_omp(y + (int64_t)n * r, At, d, r, k, norm, NULL, 0, sel + (int64_t)n * k,
                        x + (int64_t)n * k, NULL, NULL, NULL);
    free(norm);
    return rc;
}

/* ------------------------------------------------------------------------ */
/* Shared-support recovery. Sec. 4.3 (text after eq. 11) argues that the two  */
/* moments have the same sparsity pattern, so that both recovered vectors     */
/* have their non-zeros at the same positions. This variant makes that hold   */
/* by construction: the support Lambda is found by OMP on the first moment    */
/* alone, and the second moment is fitted on that same support,               */
/*     z = argmin || y_v - A_Lambda z ||_2 .                                  */
/* ------------------------------------------------------------------------ */

/* least squares on a given support: x64[k] = argmin || y - A_sel x ||_2 by the normal
 * equations (Gram matrix and right-hand side in double, Cholesky). sel[k] distinct positions.
 * returns 0, -1 on a bad argument, -4 if the Gram matrix is not positive definite */
int oracle_lstsq_support(const float *y, const float *At, int32_t d, int32_t r, const int32_t *sel,
                         int32_t k, double *x64)
{
    if (k < 0 || k > r)
        return -1;
    for (int32_t t = 0; t < k; ++t)
        if (sel[t] < 0 || sel[t] >= d)
            return -1;
    if (k == 0)
        return 0;
    double *G = (double *)calloc((size_t)k * k, sizeof(double));
    double *L = (double *)calloc((size_t)k * k, sizeof(double));
    double *b = (double *)calloc((size_t)k, sizeof(double));
    for (int32_t t = 0; t < k; ++t) {
        const float *at = At + (int64_t)sel[t] * r;
        for (int32_t u = 0; u <= t; ++u) {
            const float *au = At + (int64_t)sel[u] * r;
            double s = 0.0;
            for (int32_t j = 0; j < r; ++j)
                s += (double)at[j] * (double)au[j];
            G[(size_t)t * k + u] = s;
            G[(size_t)u * k + t] = s;
        }
        double by = 0.0;
        for (int32_t j = 0; j < r; ++j)
            by += (double)at[j] * (double)y[j];
        b[t] = by;
    }
    int rc = spd_solve(G, k, k, b, x64, L) ? -4 : 0;
    free(G);
    free(L);
    free(b);
    return rc;
}

/* One iteration of the definition of OMP (Sec. 4.3 eq. 9; selection rule of App. B) given the
 * positions selected so far: x = argmin || y - A_prefix x ||_2 (oracle_lstsq_support), res = y - A_prefix x,
 * and the next position = argmax over the unselected i of |<A_:i, res>| / ||A_:i||, lowest i on ties.
 * This is what iteration n_prefix of oracle_omp computes when its earlier picks were `prefix`; it exists
 * so that a single late pick of a long recovery (n_prefix in the hundreds) can be checked without solving
 * every earlier least-squares problem again. norm[d]: column norms (oracle_colnorms).
 * Outputs: *lam the position, top2[2] the best and second-best score (may be NULL), res_out[r] (may be NULL).
 * returns 0, -1 bad argument, -3 a prefix position repeated or out of range, -4 Gram not positive definite */
int oracle_omp_pick(const float *y, const float *At, int32_t d, int32_t r, const double *norm,
                    const int32_t *prefix, int32_t n_prefix, int32_t *lam, double *top2, double *res_out)
{
    if (n_prefix < 0 || n_prefix >= d || n_prefix > r || !norm || !lam)
        return -1;
    unsigned char *taken = (unsigned char *)calloc((size_t)d, 1);
    for (int32_t t = 0; t < n_prefix; ++t) {
        if (prefix[t] < 0 || prefix[t] >= d || taken[prefix[t]]) {
            free(taken);
            return -3;
        }
        taken[prefix[t]] = 1;
    }
    double *xs = (double *)calloc((size_t)(n_prefix > 0 ? n_prefix : 1), sizeof(double));
    int rc = oracle_lstsq_support(y, At, d, r, prefix, n_prefix, xs);
    if (rc) {
        free(taken);
        free(xs);
        return rc;
    }
    double *res = (double *)malloc(sizeof(double) * (size_t)r);
    for (int32_t j = 0; j < r; ++j)
        res[j] = (double)y[j];
    for (int32_t t = 0; t < n_prefix; ++t) {
        const float *at = At + (int64_t)prefix[t] * r;
        for (int32_t j = 0; j < r; ++j)
            res[j] -= xs[t] * (double)at[j];
    }
    int32_t best_i = -1;
    double best = -1.0, second = -1.0;
    for (int32_t i = 0; i < d; ++i) {
        if (taken[i])
            continue;
        const float *a = At + (int64_t)i * r;
        double corr = 0.0;
        for (int32_t j = 0; j < r; ++j)
            corr += (double)a[j] * res[j];
        const double score = norm[i] > 0.0 ? fabs(corr) / norm[i] : 0.0;
        if (score > best) {
            second = best;
            best = score;
            best_i = i;
        } else if (score > second) {
            second = score;
        }
    }
    *lam = best_i;
    if (top2) {
        top2[0] = best;
        top2[1] = second;
    }
    if (res_out)
        memcpy(res_out, res, sizeof(double) * (size_t)r);
    free(taken);
    free(xs);
    free(res);
    return 0;
}

/* y_m[r], y_v[r]: the two bias-corrected moments of one chunk. sel[k], x[k]: OMP_A(y_m);
 * z[k]: least-squares fit of y_v on the same support, aligned with sel. */
int oracle_omp_shared(const float *y_m, const float *y_v, const float *At, int32_t d, int32_t r,
                      int32_t k, const double *norm, int32_t *sel, float *x, float *z)
{
    int rc = oracle_omp(y_m, At, d, r, k, norm, NULL, 0, sel, x, NULL, NULL, NULL);
    if (rc)
        return rc;
    double *z64 = (double *)calloc((size_t)(k > 0 ? k : 1), sizeof(double));
    rc = oracle_lstsq_support(y_v, At, d, r, sel, k, z64);
    for (int32_t t = 0; t < k && rc == 0; ++t)
        z[t] = (float)z64[t];
    free(z64);
    return rc;
}

/* ------------------------------------------------------------------------ */
/* SGCA re-projection (App. C, Alg. 4 lines 9-12): every T steps a new matrix */
/* A' is drawn and the compressed moments are re-aligned with it,             */
/*     M <- A' OMP_A(M),   V <- A' OMP_A(V).                                  */
/* Given a recovered sparse vector (positions sel, values x) this is          */
/*     out = scale * A' x .                                                   */
/* OMP commutes with a positive scale of its input, so when x was recovered   */
/* from the bias-corrected moment (what the step already computes) and the    */
/* stored state is the uncorrected one, scale = 1 - beta^t gives the          */
/* re-aligned state; with x recovered from the state itself, scale = 1.       */
/* ------------------------------------------------------------------------ */
int oracle_reproject(const int32_t *sel, const float *x, int64_t N, int32_t k, const float *At_new,
                     int32_t d, int32_t r, double scale, float *out)
{
    for (int64_t n = 0; n < N; ++n) {
        for (int32_t j = 0; j < r; ++j) {
            double s = 0.0;
            for (int32_t t = 0; t < k; ++t) {
                int32_t i = sel[n * k + t];
                if (i < 0 || i >= d)
                    return -1;
                s += (double)At_new[(int64_t)i * r + j] * (double)x[n * k + t];
            }
            out[n * r + j] = (float)(scale * s);
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Update (eq. 11, Alg. 2 line 6, eq. 3): the two recovered sparse vectors    */
/* are placed in R^d, N = alpha * x / (sqrt(z) + eps) elementwise, and        */
/* W <- W - lr * N. Positions outside the support of x have N = 0. Where the  */
/* recovered second moment is missing it is 0; a negative recovered second    */
/* moment is taken as 0 before the root.                                      */
/* ------------------------------------------------------------------------ */
int oracle_apply(float *W, int64_t C, int32_t d, int32_t k, const int32_t *sel_m, const float *x_m,
                 const int32_t *sel_v, const float *x_v, double alpha, double eps, double lr)
{
    double *xd = (double *)malloc(sizeof(double) * (size_t)d);
    double *zd = (double *)malloc(sizeof(double) * (size_t)d);
    for (int64_t c = 0; c < C; ++c) {
        for (int32_t i = 0; i < d; ++i) {
            xd[i] = 0.0;
            zd[i] = 0.0;
        }
        for (int32_t t = 0; t < k; ++t) {
            int32_t im = sel_m[c * k + t], iv = sel_v[c * k + t];
            if (im < 0 || im >= d || iv < 0 || iv >= d) {
                free(xd);
                free(zd);
                return -1;
            }
            xd[im] = (double)x_m[c * k + t];
            zd[iv] = (double)x_v[c * k + t];
        }
        for (int32_t i = 0; i < d; ++i) {
            if (xd[i] == 0.0)
                continue;
            double z = zd[i] > 0.0 ? zd[i] : 0.0;
            double nv = alpha * xd[i] / (sqrt(z) + eps);
            W[c * (int64_t)d + i] = (float)((double)W[c * (int64_t)d + i] - lr * nv);
        }
    }
    free(xd);
    free(zd);
    return 0;
}

/* ------------------------------------------------------------------------ */
/* CESGC (Sec. 4.4): the gradient of an m x n weight matrix is first compressed */
/* with a projection B (rho x m, in the paper the leading left singular vectors */
/* of the gradient, refreshed every fixed number of steps and an input here):   */
/* Gc = B G (rho x n). SGC then runs on Gc, read row-major as rho*n/d chunks of  */
/* d entries.                                                                    */
/* ------------------------------------------------------------------------ */
int oracle_outer_project(const float *B, const float *G, int32_t rho, int32_t m, int32_t n, float *Gc)
{
    if (rho <= 0 || m <= 0 || n <= 0)
        return -1;
    for (int32_t a = 0; a < rho; ++a)
        for (int32_t j = 0; j < n; ++j) {
            double s = 0.0;
            for (int32_t i = 0; i < m; ++i)
                s += (double)B[(int64_t)a * m + i] * (double)G[(int64_t)i * n + j];
            Gc[(int64_t)a * n + j] = (float)s;
        }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* CESGC update (Sec. 4.4, the last equation of the paragraph): the update N of */
/* SGC lives in the compressed space (rho x n, built from the two recovered      */
/* sparse vectors of every chunk exactly as in the plain update above) and is    */
/* taken back with the transpose of B: W <- W - lr * B^T N.                      */
/* ------------------------------------------------------------------------ */
int oracle_outer_apply(float *W, const float *B, int32_t rho, int32_t m, int32_t n, int32_t d, int32_t k,
                       const int32_t *sel_m, const float *x_m, const int32_t *sel_v, const float *x_v,
                       double alpha, double eps, double lr)
{
    const int64_t total = (int64_t)rho * n;
    if (rho <= 0 || m <= 0 || n <= 0 || d <= 0 || total % d != 0)
        return -1;
    const int64_t C = total / d;
    double *N = (double *)calloc((size_t)total, sizeof(double));
    double *xd = (double *)malloc(sizeof(double) * (size_t)d);
    double *zd = (double *)malloc(sizeof(double) * (size_t)d);
    int rc = 0;
    for (int64_t c = 0; c < C && rc == 0; ++c) {
        for (int32_t i = 0; i < d; ++i) {
            xd[i] = 0.0;
            zd[i] = 0.0;
        }
        for (int32_t t = 0; t < k; ++t) {
            int32_t im = sel_m[c * k + t], iv = sel_v[c * k + t];
            if (im < 0 || im >= d || iv < 0 || iv >= d) {
                rc = -1;
                break;
            }
            xd[im] = (double)x_m[c * k + t];
            zd[iv] = (double)x_v[c * k + t];
        }
        for (int32_t i = 0; i < d && rc == 0; ++i) {
            if (xd[i] == 0.0)
                continue;
            double z = zd[i] > 0.0 ? zd[i] : 0.0;
            N[c * (int64_t)d + i] = alpha * xd[i] / (sqrt(z) + eps);
        }
    }
    for (int32_t i = 0; i < m && rc == 0; ++i)
        for (int32_t j = 0; j < n; ++j) {
            double s = 0.0;
            for (int32_t a = 0; a < rho; ++a)
                s += (double)B[(int64_t)a * m + i] * N[(int64_t)a * n + j];
            W[(int64_t)i * n + j] = (float)((double)W[(int64_t)i * n + j] - lr * s);
        }
    free(N);
    free(xd);
    free(zd);
    return rc;
}
