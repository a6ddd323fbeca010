/*
 * Reference (oracle) implementation of DeltaLLM's hybrid delta attention.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, double-precision
 * statement of what the method computes.  It shares no code with the GPU
 * library and must never be called from the product path; only the tests, the
 * smoke check and the benchmark's cpu_baseline leg may load it.
 *
 * Everything is fp64 except the one operation the method's bit-exact outputs
 * (mask, nnz) depend on: the threshold decision of Eq. 2, which is evaluated
 * in IEEE binary32 (subtract, abs, strict greater-than) because the inputs and
 * the threshold are binary32/bfloat16 values.
 *
 * Layouts: all matrices are row-major [rows][d] arrays of double.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Delta Network step (i), Sec. II-C Eq. 2-3, applied to the key matrix from
 * its top row downwards (Sec. III-A, strategy 3).
 *
 *   K        [n][d]  keys of one KV head
 *   state_in NULL, or [d]: reference vector k_hat held before row 0 of this
 *            call (decode continuation).  NULL means "start of sequence": the
 *            first row is the basis vector, stored whole (Sec. II-C: the delta
 *            matrix stacks the basis a(0) with the delta vectors; Sec. III-A:
 *            the first key is the basis, so the first score column is exact).
 *   mask     [n][d]  1 where the delta entry is kept, 0 where it is zeroed
 *   dK       [n][d]  the delta matrix (row 0 = basis when state_in == NULL)
 *   Khat     [n][d]  the reference vector after each row (Eq. 3)
 *   knife    out: number of entries where an all-fp64 decision would differ
 *            from the binary32 one (expected 0 for bf16 inputs)
 */
void oracle_delta_scan(const double *K, int64_t n, int64_t d, float theta,
                       const double *state_in, uint8_t *mask, double *dK,
                       double *Khat, int64_t *knife)
{
    double *ref = (double *)malloc((size_t)d * sizeof(double));
    int64_t t0 = 0, edge = 0;
    if (state_in) {
        memcpy(ref, state_in, (size_t)d * sizeof(double));
    } else if (n > 0) {
        for (int64_t c = 0; c < d; ++c) {
            ref[c] = K[c];
            mask[c] = 1;
            dK[c] = K[c];
            Khat[c] = K[c];
        }
        t0 = 1;
    }
    for (int64_t t = t0; t < n; ++t) {
        for (int64_t c = 0; c < d; ++c) {
            const double k = K[t * d + c];
            /* Eq. 2 condition, in binary32 */
            volatile float diff32 = (float)k - (float)ref[c];
            const int fire = fabsf(diff32) > theta;
            const double diff64 = k - ref[c];
            if ((fabs(diff64) > (double)theta) != fire)
                ++edge;
            if (fire) {               /* Eq. 2 first case, Eq. 3 first case */
                dK[t * d + c] = diff64;
                ref[c] = k;
            } else {                  /* second cases: zero delta, hold */
                dK[t * d + c] = 0.0;
            }
            mask[t * d + c] = (uint8_t)fire;
            Khat[t * d + c] = ref[c];
        }
    }
    if (knife)
        *knife = edge;
    free(ref);
}

static double dot(const double *a, const double *b, int64_t d)
{
    double s = 0.0;
    for (int64_t c = 0; c < d; ++c)
        s += a[c] * b[c];
    return s;
}

/*
 * Hybrid attention for query rows [row_begin, row_end) of one query head
 * against one KV head (Sec. III-B prefill; Eq. 4; Eq. 1).
 *
 *   mode 0  prefill: the exact region is the set of squares of side W on the
 *           diagonal, cut by the causal mask: (i, j) exact iff j <= i and
 *           floor(i/W) == floor(j/W).
 *   mode 1  decode-style sliding window: (i, j) exact iff 0 <= i - j < W
 *           (the most recent W keys including the current one).
 *
 * Outside the exact region the score is the Delta Network output R(j)[i] of
 * Eq. 4 with A = K and B = Q^T:  R(0) = dK(0).q_i,  R(j) = R(j-1) + dK(j).q_i.
 *
 *   Q  [nq][d] rows row_begin..row_end-1 are used; row i attends keys 0..i+q_off
 *   q_off: position of query row 0 in the key sequence (0 for prefill).
 *   O  [(row_end-row_begin)][d]
 */
void oracle_hybrid_rows(const double *Q, const double *K, const double *V,
                        const double *dK, int64_t d, int64_t W, int mode,
                        double scale, int64_t q_off, int64_t row_begin,
                        int64_t row_end, double *O)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = row_begin; i < row_end; ++i) {
        const int64_t pos = i + q_off;          /* last visible key */
        const double *q = Q + i * d;
        double *s = (double *)malloc((size_t)(pos + 1) * sizeof(double));
        double R = 0.0;                         /* Eq. 4 running output */
        for (int64_t j = 0; j <= pos; ++j) {
            R += dot(q, dK + j * d, d);
            int inside;
            if (mode == 0)
                inside = (pos / W) == (j / W);
            else
                inside = (pos - j) < W;
            s[j] = (inside ? dot(q, K + j * d, d) : R) * scale;
        }
        /* Eq. 1: softmax over the visible keys, then the weighted sum of V */
        double m = s[0];
        for (int64_t j = 1; j <= pos; ++j)
            if (s[j] > m) m = s[j];
        double z = 0.0;
        for (int64_t j = 0; j <= pos; ++j) {
            s[j] = exp(s[j] - m);
            z += s[j];
        }
        double *o = O + (i - row_begin) * d;
        for (int64_t c = 0; c < d; ++c) o[c] = 0.0;
        for (int64_t j = 0; j <= pos; ++j) {
            const double p = s[j] / z;
            for (int64_t c = 0; c < d; ++c)
                o[c] += p * V[j * d + c];
        }
        free(s);
    }
}

/*
 * Score rows only (no softmax): S[(i-row_begin)][j] for j = 0..nk-1, entries
 * with j > i+q_off are set to -inf.  Used by the tests to look at the hybrid
 * score matrix itself (first column exact, telescoping, window area).
 */
void oracle_hybrid_scores(const double *Q, const double *K, const double *dK,
                          int64_t nk, int64_t d, int64_t W, int mode,
                          double scale, int64_t q_off, int64_t row_begin,
                          int64_t row_end, double *S, uint8_t *exact)
{
    for (int64_t i = row_begin; i < row_end; ++i) {
        const int64_t pos = i + q_off;
        const double *q = Q + i * d;
        double R = 0.0;
        for (int64_t j = 0; j < nk; ++j) {
            double *out = S + (i - row_begin) * nk + j;
            uint8_t *ex = exact + (i - row_begin) * nk + j;
            if (j > pos) { *out = -INFINITY; *ex = 0; continue; }
            R += dot(q, dK + j * d, d);
            int inside = (mode == 0) ? ((pos / W) == (j / W)) : ((pos - j) < W);
            *out = (inside ? dot(q, K + j * d, d) : R) * scale;
            *ex = (uint8_t)inside;
        }
    }
}
