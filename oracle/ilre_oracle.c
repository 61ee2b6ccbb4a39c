/*
 * CPU oracle for intermediate-layer token recall -- scoring part.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, fp64 definition the
 * GPU path is checked against.  It shares no code with the GPU path and is
 * imported only by the tests, by the smoke check and by the benchmark's
 * cpu_baseline leg.  Nothing on the product path may call it.
 *
 * What it computes (paper Section 3.2, "Observations of Retrieval Tasks"):
 *
 *   Eq. 4   A[h,i,t] = softmax_t( q[h,i,:] . K[g(h),t,:] / sqrt(d_h) )
 *           the softmax runs over all L context positions of the key cache;
 *           no mask (the query tokens come after the whole context) and no
 *           query self-keys (only K^C appears in the argument).
 *   GQA     query head h reads kv head g(h) = floor(h / (Hq/Hkv)): consecutive
 *           grouping (the paper only names GQA; this is the reading taken).
 *   Eq. 5   3-D -> 1-D reduction over the head and query dimensions.
 *           mode 0: score[t] = sum_{h,i} A[h,i,t]   (the reading this build's
 *                   target takes; every softmax row sums to one, so the
 *                   scores total Hq*Lq)
 *           mode 1: score[t] = max_{h,i} A[h,i,t]   (Eq. 5 as printed)
 *
 * Shape of the computation: one (head, query) row at a time.  For a row the
 * L logits are written out as an fp64 vector, then max, exp, sum, divide, in
 * that order, exactly as the definition reads.  No tiling, no online softmax,
 * no two-pass trick.  Inputs are the caller's bf16 or fp32 bit patterns widened
 * exactly to fp64.  Rows of one query head accumulate into that head's own
 * L-vector; the per-head vectors are combined in head order at the end, so the
 * result does not depend on the number of threads.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };
enum { ORACLE_SUM = 0, ORACLE_MAX = 1 };

static inline double widen_bf16(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static inline double elem(const void *base, int dtype, int64_t i)
{
    if (dtype == ORACLE_BF16)
        return widen_bf16(((const uint16_t *)base)[i]);
    return (double)((const float *)base)[i];
}

/* logits[t] = scale * sum_c q[c] * K[g,t,c]  for t = 0..L-1 (Eq. 4 argument). */
static void row_logits(const double *qrow, const void *k, int dtype, int64_t g,
                       int64_t L, int d, double scale, double *logits)
{
    for (int64_t t = 0; t < L; ++t) {
        const int64_t off = (g * L + t) * d;
        double acc = 0.0;
        if (dtype == ORACLE_BF16) {
            const uint16_t *kr = (const uint16_t *)k + off;
            for (int c = 0; c < d; ++c)
                acc += qrow[c] * widen_bf16(kr[c]);
        } else {
            const float *kr = (const float *)k + off;
            for (int c = 0; c < d; ++c)
                acc += qrow[c] * (double)kr[c];
        }
        logits[t] = acc * scale;
    }
}

int ilre_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Row statistics of Eq. 4 for a list of rows: rows[j] = h*Lq + i.
 * row_max[j] = max_t logit, row_sumexp[j] = sum_t exp(logit - row_max[j]).
 * q: [Hq, Lq, d], k: [Hkv, L, d], both contiguous.  Returns 0, or -1 on bad args / alloc.
 */
int ilre_oracle_row_stats(const void *q, const void *k, int dtype,
                          int64_t L, int Lq, int Hq, int Hkv, int d, double scale,
                          const int32_t *rows, int nrows,
                          double *row_max, double *row_sumexp)
{
    if (!q || !k || L < 1 || Lq < 1 || Hq < 1 || Hkv < 1 || d < 1 || Hq % Hkv) return -1;
    const int G = Hq / Hkv;
    int fail = 0;
#pragma omp parallel
    {
        double *logits = (double *)malloc(sizeof(double) * (size_t)L);
        double *qrow = (double *)malloc(sizeof(double) * (size_t)d);
        if (!logits || !qrow) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp barrier
        if (!fail) {
#pragma omp for schedule(dynamic, 1)
            for (int j = 0; j < nrows; ++j) {
                const int h = rows[j] / Lq, i = rows[j] % Lq;
                for (int c = 0; c < d; ++c)
                    qrow[c] = elem(q, dtype, ((int64_t)h * Lq + i) * d + c);
                row_logits(qrow, k, dtype, h / G, L, d, scale, logits);
                double m = logits[0];
                for (int64_t t = 1; t < L; ++t)
                    if (logits[t] > m) m = logits[t];
                double z = 0.0;
                for (int64_t t = 0; t < L; ++t)
                    z += exp(logits[t] - m);
                row_max[j] = m;
                row_sumexp[j] = z;
            }
        }
        free(logits);
        free(qrow);
    }
    return fail ? -1 : 0;
}

/*
 * Full scoring: Eq. 4 for every (head, query) row and the Eq. 5 reduction.
 * Outputs: row_max[Hq*Lq], row_sumexp[Hq*Lq] (either may be NULL), score[L].
 */
int ilre_oracle_scores(const void *q, const void *k, int dtype,
                       int64_t L, int Lq, int Hq, int Hkv, int d, double scale,
                       int mode, double *row_max, double *row_sumexp, double *score)
{
    if (!q || !k || !score || L < 1 || Lq < 1 || Hq < 1 || Hkv < 1 || d < 1 || Hq % Hkv) return -1;
    if (mode != ORACLE_SUM && mode != ORACLE_MAX) return -1;
    const int G = Hq / Hkv;
    double *per_head = (double *)calloc((size_t)Hq * (size_t)L, sizeof(double));
    if (!per_head) return -1;
    int fail = 0;
#pragma omp parallel
    {
        double *logits = (double *)malloc(sizeof(double) * (size_t)L);
        double *qrow = (double *)malloc(sizeof(double) * (size_t)d);
        if (!logits || !qrow) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp barrier
        if (!fail) {
#pragma omp for schedule(dynamic, 1)
            for (int h = 0; h < Hq; ++h) {
                double *acc = per_head + (size_t)h * (size_t)L;
                for (int i = 0; i < Lq; ++i) {
                    for (int c = 0; c < d; ++c)
                        qrow[c] = elem(q, dtype, ((int64_t)h * Lq + i) * d + c);
                    row_logits(qrow, k, dtype, h / G, L, d, scale, logits);
                    double m = logits[0];
                    for (int64_t t = 1; t < L; ++t)
                        if (logits[t] > m) m = logits[t];
                    double z = 0.0;
                    for (int64_t t = 0; t < L; ++t) {
                        logits[t] = exp(logits[t] - m);
                        z += logits[t];
                    }
                    if (row_max) row_max[(size_t)h * Lq + i] = m;
                    if (row_sumexp) row_sumexp[(size_t)h * Lq + i] = z;
                    for (int64_t t = 0; t < L; ++t) {
                        const double p = logits[t] / z;
                        if (mode == ORACLE_SUM) acc[t] += p;
                        else if (p > acc[t]) acc[t] = p;
                    }
                }
            }
        }
        free(logits);
        free(qrow);
    }
    if (!fail) {
        for (int64_t t = 0; t < L; ++t) {
            double s = 0.0;
            for (int h = 0; h < Hq; ++h) {
                const double v = per_head[(size_t)h * (size_t)L + (size_t)t];
                if (mode == ORACLE_SUM) s += v;
                else if (v > s) s = v;
            }
            score[t] = s;
        }
    }
    free(per_head);
    return fail ? -1 : 0;
}
