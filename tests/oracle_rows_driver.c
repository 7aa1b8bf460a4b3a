/*
 * Test driver for the row-statistics part of the CPU oracle, built together with it under
 * AddressSanitizer and UndefinedBehaviorSanitizer (see test_oracle_sanitized.py).
 * Input file:  int64 dtype, int64 rows, int64 V, int64 row_stride, then rows * row_stride stored logits.
 * Output file: rows doubles m, rows int64 t, rows doubles S.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

void csd_oracle_rows(const void *z, int dtype, int64_t row_stride, int64_t V, int64_t r0, int64_t r1, double *m, int64_t *t,
                     double *S);

int main(int argc, char **argv)
{
    if (argc != 3) return 2;
    FILE *in = fopen(argv[1], "rb");
    if (!in) return 3;
    int64_t head[4];
    if (fread(head, sizeof(int64_t), 4, in) != 4) return 4;
    const int64_t dtype = head[0], rows = head[1], V = head[2], stride = head[3];
    const size_t esz = dtype == 0 ? 4 : 2;
    const size_t n = (size_t)rows * (size_t)stride;
    /* exactly n elements: a read past the last row's V-th logit is an out-of-bounds access the sanitizer reports */
    void *z = malloc(n * esz ? n * esz : 1);
    if (n && fread(z, esz, n, in) != n) return 5;
    fclose(in);
    double *m = malloc(sizeof(double) * (rows ? rows : 1)), *S = malloc(sizeof(double) * (rows ? rows : 1));
    int64_t *t = malloc(sizeof(int64_t) * (rows ? rows : 1));
    /* in two halves, as the threaded caller splits the rows */
    csd_oracle_rows(z, (int)dtype, stride, V, 0, rows / 2, m, t, S);
    csd_oracle_rows(z, (int)dtype, stride, V, rows / 2, rows, m, t, S);
    FILE *out = fopen(argv[2], "wb");
    if (!out) return 6;
    fwrite(m, sizeof(double), rows, out);
    fwrite(t, sizeof(int64_t), rows, out);
    fwrite(S, sizeof(double), rows, out);
    fclose(out);
    free(z); free(m); free(S); free(t);
    return 0;
}
