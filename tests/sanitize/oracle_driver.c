/* Host-sanitizer driver for the C scoring oracle (test infrastructure).  Built by tests/test_sanitizers.py
 * together with oracle/ilre_oracle.c under -fsanitize=address,undefined and run on a small problem read from
 * a file; the results go to another file, where the test compares them with the regular build's.
 *
 * Input file: int64 header[8] = {dtype, L, Lq, Hq, Hkv, d, mode, nrows}, double scale, then q, k (element
 * size 4 for dtype 0, 2 for dtype 1), then nrows int32 row indices.
 * Output file: double score[L], rmax[Hq*Lq], rsum[Hq*Lq], then rmax_sel[nrows], rsum_sel[nrows]. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int ilre_oracle_scores(const void *q, const void *k, int dtype, int64_t L, int Lq, int Hq, int Hkv, int d, double scale,
                       int mode, double *row_max, double *row_sumexp, double *score);
int ilre_oracle_row_stats(const void *q, const void *k, int dtype, int64_t L, int Lq, int Hq, int Hkv, int d, double scale,
                          const int32_t *rows, int nrows, double *row_max, double *row_sumexp);

static void *read_exact(FILE *f, size_t bytes)
{
    void *p = malloc(bytes ? bytes : 1);
    if (!p || fread(p, 1, bytes, f) != bytes) {
        fprintf(stderr, "short read\n");
        exit(3);
    }
    return p;
}

int main(int argc, char **argv)
{
    if (argc != 3) return 2;
    FILE *f = fopen(argv[1], "rb");
    if (!f) return 2;
    int64_t h[8];
    double scale;
    if (fread(h, sizeof h, 1, f) != 1 || fread(&scale, sizeof scale, 1, f) != 1) return 3;
    const int dtype = (int)h[0], Lq = (int)h[2], Hq = (int)h[3], Hkv = (int)h[4], d = (int)h[5], mode = (int)h[6], nrows = (int)h[7];
    const int64_t L = h[1];
    const size_t es = dtype ? 2 : 4;
    void *q = read_exact(f, (size_t)Hq * Lq * d * es);
    void *k = read_exact(f, (size_t)Hkv * (size_t)L * d * es);
    int32_t *rows = (int32_t *)read_exact(f, (size_t)nrows * sizeof(int32_t));
    fclose(f);
    const size_t R = (size_t)Hq * Lq;
    double *score = (double *)malloc(sizeof(double) * (size_t)L);
    double *rmax = (double *)malloc(sizeof(double) * R), *rsum = (double *)malloc(sizeof(double) * R);
    double *smax = (double *)malloc(sizeof(double) * (size_t)(nrows ? nrows : 1)), *ssum = (double *)malloc(sizeof(double) * (size_t)(nrows ? nrows : 1));
    if (!score || !rmax || !rsum || !smax || !ssum) return 4;
    if (ilre_oracle_scores(q, k, dtype, L, Lq, Hq, Hkv, d, scale, mode, rmax, rsum, score) != 0) return 5;
    if (ilre_oracle_row_stats(q, k, dtype, L, Lq, Hq, Hkv, d, scale, rows, nrows, smax, ssum) != 0) return 6;
    /* the argument checks must refuse, not read */
    if (ilre_oracle_scores(NULL, k, dtype, L, Lq, Hq, Hkv, d, scale, mode, rmax, rsum, score) == 0) return 7;
    if (ilre_oracle_scores(q, k, dtype, 0, Lq, Hq, Hkv, d, scale, mode, rmax, rsum, score) == 0) return 7;
    FILE *o = fopen(argv[2], "wb");
    if (!o) return 2;
    fwrite(score, sizeof(double), (size_t)L, o);
    fwrite(rmax, sizeof(double), R, o);
    fwrite(rsum, sizeof(double), R, o);
    fwrite(smax, sizeof(double), (size_t)nrows, o);
    fwrite(ssum, sizeof(double), (size_t)nrows, o);
    fclose(o);
    free(q); free(k); free(rows); free(score); free(rmax); free(rsum); free(smax); free(ssum);
    return 0;
}
