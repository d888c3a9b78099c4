/*
 * CPU oracle for GRIFFIN's feed-forward hot path.  TEST INFRASTRUCTURE ONLY.
 *
 * Only the tests, the smoke check and the benchmark's cpu-baseline leg may call this file.
 * It shares no code, header, table or helper with the HIP library and is never a fallback
 * for it.  Every function is the paper's definition written out as plain loops in fp64
 * (inputs are widened exactly by the caller); there is no tiling, fusion or reordering.
 * OpenMP only hands independent outputs to different threads; each output is still one
 * plain left-to-right sum (the `omp simd` reductions may regroup a sum's terms, which in
 * fp64 moves results by ~1e-16 relative).
 *
 * Layout: every weight matrix is neuron-major [n][d]: row j holds neuron j.  Wg and W1 are
 * the paper's W_g, W_1 (D_FF x D, Section 3); W2 is the transpose of the paper's W_2
 * (D x D_FF), so a selected neuron is one row in all three.
 *
 * Readings where the paper is silent: ties in top-k go to the lowest index; the selected
 * set is returned ascending; a prompt row whose activations are all zero contributes
 * nothing to the statistic; GEGLU uses the tanh form of GELU.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_ACT_SILU = 0, ORACLE_ACT_GELU_TANH = 1, ORACLE_ACT_RELU = 2 };

/* sigma of Section 3 (Eq. 2, Eq. 3); the named variants are those of Section 1, item 3. */
static double oracle_act(int act, double a)
{
    switch (act) {
    case ORACLE_ACT_SILU:
        return a / (1.0 + exp(-a));
    case ORACLE_ACT_GELU_TANH:
        return 0.5 * a * (1.0 + tanh(0.79788456080286535588 * (a + 0.044715 * a * a * a)));
    case ORACLE_ACT_RELU:
        return a > 0.0 ? a : 0.0;
    default:
        return NAN;
    }
}

static double oracle_dot(const double *a, const double *b, int64_t d)
{
    double acc = 0.0;
#pragma omp simd reduction(+ : acc)
    for (int64_t c = 0; c < d; ++c)
        acc += a[c] * b[c];
    return acc;
}

/*
 * FF activations of a sequence, Z = FF_1(X) applied to every row of X (Section 3, Eq. 3 and
 * the remark after Eq. 5).  With Wg == NULL it is the non-gated form of Eq. 2.
 * X[S][d], Wg/W1[n][d], bg/b1[n] or NULL, Z[S][n].
 */
int oracle_ff1(int64_t S, int64_t d, int64_t n, const double *X, const double *Wg,
               const double *W1, const double *bg, const double *b1, int act, double *Z)
{
    if (act < 0 || act > 2 || !X || !W1 || !Z)
        return 1;
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < n; ++j) {
        for (int64_t i = 0; i < S; ++i) {
            double u = oracle_dot(X + i * d, W1 + j * d, d) + (b1 ? b1[j] : 0.0);
            if (Wg) {
                double g = oracle_dot(X + i * d, Wg + j * d, d) + (bg ? bg[j] : 0.0);
                Z[i * n + j] = oracle_act(act, g) * u;
            } else {
                Z[i * n + j] = oracle_act(act, u);
            }
        }
    }
    return 0;
}

/*
 * Relative activations and the statistic s (Section 4.1 and Eq. 6): each row of Z is scaled
 * to unit l2 norm, then s_j is the l2 norm of column j of the scaled matrix.
 * Z[S][F] -> s[F]; rnorm[S] (optional) receives the row norms.
 */
int oracle_stat(int64_t S, int64_t F, const double *Z, double *s, double *rnorm)
{
    double *r = (double *)malloc(sizeof(double) * (size_t)(S > 0 ? S : 1));
    if (!r)
        return 2;
    for (int64_t i = 0; i < S; ++i) {
        double acc = 0.0;
        for (int64_t j = 0; j < F; ++j)
            acc += Z[i * F + j] * Z[i * F + j];
        r[i] = sqrt(acc);
        if (rnorm)
            rnorm[i] = r[i];
    }
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < F; ++j) {
        double acc = 0.0;
        for (int64_t i = 0; i < S; ++i) {
            if (r[i] > 0.0) {
                double zb = Z[i * F + j] / r[i];
                acc += zb * zb;
            }
        }
        s[j] = sqrt(acc);
    }
    free(r);
    return 0;
}

/*
 * Batched statistic of Section 5.3 (Eq. 7): s_bar = sum_i s_i / sqrt(S_i) over the samples
 * of a batch.  s_all[n][F], lens[n] -> sbar[F].
 */
int oracle_stat_shared(int64_t n, int64_t F, const double *s_all, const int64_t *lens, double *sbar)
{
    for (int64_t j = 0; j < F; ++j) {
        double acc = 0.0;
        for (int64_t i = 0; i < n; ++i)
            acc += s_all[i * F + j] / sqrt((double)lens[i]);
        sbar[j] = acc;
    }
    return 0;
}

typedef struct {
    double s;
    int32_t j;
} oracle_key;

static int oracle_cmp_desc(const void *pa, const void *pb)
{
    const oracle_key *a = (const oracle_key *)pa, *b = (const oracle_key *)pb;
    if (a->s > b->s) return -1;
    if (a->s < b->s) return 1;
    return (a->j > b->j) - (a->j < b->j);
}

static int oracle_cmp_i32(const void *pa, const void *pb)
{
    int32_t a = *(const int32_t *)pa, b = *(const int32_t *)pb;
    return (a > b) - (a < b);
}

/*
 * Expert set E (Section 4.2): the indices of the k largest entries of s.  A full sort by
 * (value descending, index ascending), its first k entries, returned in ascending order.
 */
int oracle_topk(int64_t F, const double *s, int64_t k, int32_t *idx)
{
    if (k < 0 || k > F)
        return 1;
    oracle_key *keys = (oracle_key *)malloc(sizeof(oracle_key) * (size_t)(F > 0 ? F : 1));
    if (!keys)
        return 2;
    for (int64_t j = 0; j < F; ++j) {
        keys[j].s = s[j];
        keys[j].j = (int32_t)j;
    }
    qsort(keys, (size_t)F, sizeof(oracle_key), oracle_cmp_desc);
    for (int64_t t = 0; t < k; ++t)
        idx[t] = keys[t].j;
    qsort(idx, (size_t)k, sizeof(int32_t), oracle_cmp_i32);
    free(keys);
    return 0;
}

/*
 * Compact weights (Section 3, Eq. 4-5 and Section 4.2): the rows of a neuron-major matrix
 * (or the entries of a per-neuron bias, d = 1) listed in idx, in that order.
 */
int oracle_compact(int64_t n_src, int64_t d, const double *W, int64_t k, const int32_t *idx,
                   double *out)
{
    for (int64_t t = 0; t < k; ++t) {
        if (idx[t] < 0 || idx[t] >= n_src)
            return 1;
        memcpy(out + t * d, W + (int64_t)idx[t] * d, sizeof(double) * (size_t)d);
    }
    return 0;
}

/*
 * One generated token through a (pruned or full) FF block (Eq. 1, Eq. 4-5, Section 4.2):
 * z_j = sigma(wg_j . x + bg_j) * (w1_j . x + b1_j),  y_c = sum_j z_j W2[j][c] + b2_c,
 * the sum over j taken in ascending order.  Wg == NULL gives Eq. 2.  z (optional) gets z.
 */
int oracle_ff_decode(int64_t d, int64_t n, const double *x, const double *Wg, const double *W1,
                     const double *W2, const double *bg, const double *b1, const double *b2,
                     int act, double *y, double *z_out)
{
    if (act < 0 || act > 2)
        return 1;
    double *z = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
    if (!z)
        return 2;
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < n; ++j) {
        double u = oracle_dot(x, W1 + j * d, d) + (b1 ? b1[j] : 0.0);
        if (Wg) {
            double g = oracle_dot(x, Wg + j * d, d) + (bg ? bg[j] : 0.0);
            z[j] = oracle_act(act, g) * u;
        } else {
            z[j] = oracle_act(act, u);
        }
    }
#pragma omp parallel for schedule(static)
    for (int64_t c = 0; c < d; ++c) {
        double acc = 0.0;
        for (int64_t j = 0; j < n; ++j)
            acc += z[j] * W2[j * d + c];
        y[c] = acc + (b2 ? b2[c] : 0.0);
    }
    if (z_out)
        memcpy(z_out, z, sizeof(double) * (size_t)n);
    free(z);
    return 0;
}

/* Prompt-phase output of the full block (Section 5.1: the prompt uses every neuron):
 * Y = Z W2 + b2 row by row.  Z[S][n], W2[n][d] -> Y[S][d]. */
int oracle_ff2(int64_t S, int64_t d, int64_t n, const double *Z, const double *W2,
               const double *b2, double *Y)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < S; ++i) {
        for (int64_t c = 0; c < d; ++c) {
            double acc = 0.0;
            for (int64_t j = 0; j < n; ++j)
                acc += Z[i * n + j] * W2[j * d + c];
            Y[i * d + c] = acc + (b2 ? b2[c] : 0.0);
        }
    }
    return 0;
}

/*
 * Static selector of the paper's magnitude baseline (Section 5.1, "Setup"): one score per
 * neuron from the weights alone, the l2 norm of the neuron's row of W1, multiplied, for GLU
 * blocks, by the l2 norm of its row of Wg.  (The paper says "neuron-wise norms" without
 * naming the norm; l2 is the reading taken.)  Wg may be NULL.
 */
int oracle_weight_norm_score(int64_t n, int64_t d, const double *Wg, const double *W1, double *score)
{
    for (int64_t j = 0; j < n; ++j) {
        double a = 0.0, b = 0.0;
        for (int64_t c = 0; c < d; ++c)
            a += W1[j * d + c] * W1[j * d + c];
        if (Wg)
            for (int64_t c = 0; c < d; ++c)
                b += Wg[j * d + c] * Wg[j * d + c];
        score[j] = Wg ? sqrt(a) * sqrt(b) : sqrt(a);
    }
    return 0;
}

typedef struct {
    double q;
    int32_t j;
} oracle_qkey;

static int oracle_cmp_q_desc(const void *pa, const void *pb)
{
    const oracle_qkey *a = (const oracle_qkey *)pa, *b = (const oracle_qkey *)pb;
    if (a->q > b->q) return -1;
    if (a->q < b->q) return 1;
    return (a->j > b->j) - (a->j < b->j);
}

/*
 * Sampling-based selection (Appendix B): k_top experts by top-k of s, the remaining k - k_top
 * drawn from the other neurons without replacement with probability proportional to s_j
 * (k_top = 0 is the pure "sampling" row of Table 5, k_top = k/2 its "top-k + sampling" row,
 * k_top = k plain top-k).  The paper does not say how the draw is made; the reading taken is
 * the exponential-clocks form of weighted sampling without replacement: neuron j rings at time
 * e_j / s_j, with e_j a unit-rate exponential variate supplied by the caller (the method's
 * random numbers are inputs), and the earliest k - k_top rings win.  The winner of "earliest
 * ring" is decided on q_j = s_j / e_j, largest first, in double precision like everything else
 * here; ties go to the lowest index; s_j = 0 (q_j = 0) never beats a positive weight.  The set
 * is returned ascending.
 */
int oracle_select_sampled(int64_t F, const double *s, const float *e, int64_t k, int64_t k_top, int32_t *idx)
{
    if (k < 0 || k > F || k_top < 0 || k_top > k)
        return 1;
    char *taken = (char *)calloc((size_t)(F > 0 ? F : 1), 1);
    oracle_qkey *keys = (oracle_qkey *)malloc(sizeof(oracle_qkey) * (size_t)(F > 0 ? F : 1));
    if (!taken || !keys)
        return 2;
    int rc = oracle_topk(F, s, k_top, idx);
    if (rc) {
        free(keys);
        free(taken);
        return rc;
    }
    for (int64_t t = 0; t < k_top; ++t)
        taken[idx[t]] = 1;
    int64_t m = 0;
    for (int64_t j = 0; j < F; ++j) {
        if (taken[j])
            continue;
        keys[m].q = s[j] / (double)e[j];
        keys[m].j = (int32_t)j;
        ++m;
    }
    qsort(keys, (size_t)m, sizeof(oracle_qkey), oracle_cmp_q_desc);
    for (int64_t t = k_top; t < k; ++t)
        idx[t] = keys[t - k_top].j;
    qsort(idx, (size_t)k, sizeof(int32_t), oracle_cmp_i32);
    free(keys);
    free(taken);
    return 0;
}

/*
 * Jaccard similarity of two selected sets (Section 4.1, the inter-sample comparison of top-k
 * sets): |A n B| / |A u B|, by comparing every pair of members.  Members of a set are distinct.
 */
int oracle_jaccard(int64_t ka, const int32_t *a, int64_t kb, const int32_t *b, double *out)
{
    int64_t inter = 0;
    for (int64_t i = 0; i < ka; ++i)
        for (int64_t j = 0; j < kb; ++j)
            if (a[i] == b[j])
                ++inter;
    const int64_t uni = ka + kb - inter;
    *out = uni > 0 ? (double)inter / (double)uni : 1.0;
    return 0;
}

int oracle_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        n = omp_get_num_threads();
    }
#endif
    return n;
}
