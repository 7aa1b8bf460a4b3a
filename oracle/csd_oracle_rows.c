/*
 * CPU oracle for CSD verification: per-row statistics of the target logits.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, fp64 definition the
 * GPU library is checked against.  It shares no code with the GPU path and
 * must never be called from it.
 *
 * What a row needs (Algorithm 1: the target distribution p_i(.) of a verify
 * position, the target token t*, and the probabilities that enter the
 * Semantic Consistency Gating test, Eq. 3):
 *     m  = max_v z_v
 *     t* = the smallest v with z_v == m        (greedy target token; ties -> lowest id)
 *     S  = sum_v exp(z_v - m)                  (softmax normaliser, so p_v = exp(z_v - m) / S)
 * Stored logits (fp32, or bf16 bit patterns) are widened exactly to double and
 * everything is evaluated in double, two passes, ascending v.  No blocking, no
 * reordering, no fast-math.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

#define CSD_ORACLE_F32 0
#define CSD_ORACLE_BF16 1

static double widen(const void *z, int dtype, int64_t v)
{
    if (dtype == CSD_ORACLE_F32) {
        return (double)((const float *)z)[v];
    } else {
        /* bfloat16 is the upper half of an IEEE binary32 */
        uint32_t u = (uint32_t)((const uint16_t *)z)[v] << 16;
        float f;
        memcpy(&f, &u, sizeof f);
        return (double)f;
    }
}

/* One logit, widened. */
double csd_oracle_logit(const void *z, int dtype, int64_t v)
{
    return widen(z, dtype, v);
}

/* Statistics of one row of V logits. */
void csd_oracle_row_stats(const void *z, int dtype, int64_t V, double *m_out, int64_t *t_out, double *S_out)
{
    double m = widen(z, dtype, 0);
    int64_t t = 0;
    for (int64_t v = 1; v < V; ++v) {
        double x = widen(z, dtype, v);
        if (x > m) { /* strict: the first maximum keeps the lowest id */
            m = x;
            t = v;
        }
    }
    double S = 0.0;
    for (int64_t v = 0; v < V; ++v) {
        S += exp(widen(z, dtype, v) - m);
    }
    *m_out = m;
    *t_out = t;
    *S_out = S;
}

/* Rows r0 <= r < r1 of a [rows][row_stride] array (row_stride in elements). */
void csd_oracle_rows(const void *z, int dtype, int64_t row_stride, int64_t V, int64_t r0, int64_t r1, double *m, int64_t *t,
                     double *S)
{
    const int64_t esz = (dtype == CSD_ORACLE_F32) ? 4 : 2;
    for (int64_t r = r0; r < r1; ++r) {
        const char *row = (const char *)z + r * row_stride * esz;
        csd_oracle_row_stats(row, dtype, V, &m[r], &t[r], &S[r]);
    }
}
