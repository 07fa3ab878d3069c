/*
 * attn_oracle.c -- TEST INFRASTRUCTURE ONLY (never on the product path).
 *
 * Plain, slow, obviously-correct FP64 CPU attention used to check the HIP
 * kernels.  It shares no code, header, table or helper with the GPU library.
 *
 * What it computes (paper section 2.2, "Attention computation":
 * O = softmax(Q K^T / sqrt(d)) V, with the causal / grouped-query variants of
 * section 4.1 "Benchmark Configurations" and section 4.3):
 *
 *   for every batch b, query head h, query row i
 *     g        = h / (Hq / Hkv)                  contiguous head groups
 *     s_j      = scale * sum_d Q[b,i,h,d] * K[b,j,g,d]      j = 0..Skv-1
 *     valid(j) = !causal  ||  j <= i + (Skv - Sq)            bottom-right aligned
 *     mx       = max over valid j of s_j
 *     p_j      = exp(s_j - mx) for valid j, else 0
 *     l        = sum_j p_j                      explicit full-row softmax
 *     O[b,i,h,:] = (sum_j p_j V[b,j,g,:]) / l
 *     LSE[b,h,i] = mx + ln(l)
 *     no valid key at all: O = 0, LSE = -inf
 *
 * The score row is materialised in full (the naive algorithm of section 2.2);
 * there is no tiling, no running max and no running sum.  Everything is FP64.
 *
 * Layouts (all host memory, all double, contiguous):
 *   q [B, Sq,  Hq,  D]    k, v [B, Skv, Hkv, D]
 *   o [B, Sq,  Hq,  D]    lse  [B, Hq, Sq]
 *
 * Readings where the paper is silent (layout, LSE, mask alignment for
 * Sq != Skv, empty rows, head grouping) are the ones stated above.
 *
 * Pins: tests/test_oracle_pins.py (invariants, closed forms, brute force on
 * tiny shapes, a float64 library routine on special cases).
 *
 * Return value: 0 on success, -1 on a bad argument, -2 when out of memory.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static int bad_dims(long B, long Hq, long Hkv, long Sq, long Skv, long D)
{
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || Sq <= 0 || Skv <= 0 || D <= 0) return 1;
    if (Hq % Hkv != 0) return 1;
    return 0;
}

/* One query row.  `s` is caller scratch of Skv doubles and, on return, holds
 * the normalised probabilities p_j / l (zeros where masked).  */
static void one_row(const double *q, const double *k, const double *v,
                    long b, long h, long i,
                    long Hq, long Hkv, long Sq, long Skv, long D,
                    int causal, double scale,
                    double *s, double *o_row, double *lse_out)
{
    const long g = h / (Hq / Hkv);
    const double *qrow = q + ((b * Sq + i) * Hq + h) * D;
    long last = Skv - 1;                       /* last valid key index */
    if (causal) {
        long lim = i + (Skv - Sq);
        if (lim < last) last = lim;
    }
    for (long d = 0; d < D; ++d) o_row[d] = 0.0;
    for (long j = 0; j < Skv; ++j) s[j] = 0.0;
    if (last < 0) {                            /* empty valid set */
        *lse_out = -INFINITY;
        return;
    }
    double mx = -INFINITY;
    for (long j = 0; j <= last; ++j) {
        const double *krow = k + ((b * Skv + j) * Hkv + g) * D;
        double acc = 0.0;
        for (long d = 0; d < D; ++d) acc += qrow[d] * krow[d];
        s[j] = scale * acc;
        if (s[j] > mx) mx = s[j];
    }
    double l = 0.0;
    for (long j = 0; j <= last; ++j) {
        s[j] = exp(s[j] - mx);
        l += s[j];
    }
    for (long j = 0; j <= last; ++j) {
        const double *vrow = v + ((b * Skv + j) * Hkv + g) * D;
        const double p = s[j];
        for (long d = 0; d < D; ++d) o_row[d] += p * vrow[d];
    }
    for (long d = 0; d < D; ++d) o_row[d] /= l;
    for (long j = 0; j <= last; ++j) s[j] /= l;
    *lse_out = mx + log(l);
}

/* Every row of every head. */
int attn_ref_f64(const double *q, const double *k, const double *v,
                 double *o, double *lse,
                 int B, int Hq, int Hkv, int Sq, int Skv, int D,
                 int causal, double scale)
{
    if (!q || !k || !v || !o || !lse) return -1;
    if (bad_dims(B, Hq, Hkv, Sq, Skv, D)) return -1;
    const long nrows = (long)B * Hq * Sq;
    int fail = 0;
#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)Skv);
        if (!s) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp for schedule(dynamic, 16)
        for (long r = 0; r < nrows; ++r) {
            if (!s) continue;
            const long i = r % Sq;
            const long h = (r / Sq) % Hq;
            const long b = r / ((long)Sq * Hq);
            one_row(q, k, v, b, h, i, Hq, Hkv, Sq, Skv, D, causal, scale, s,
                    o + ((b * Sq + i) * Hq + h) * D,
                    lse + (b * Hq + h) * Sq + i);
        }
        free(s);
    }
    return fail ? -2 : 0;
}

/* Only the listed rows: rows[3*n + {0,1,2}] = (b, h, i).
 * o_rows [n, D], lse_rows [n].  Each row is exact and independent of the
 * others, so a sample of rows checks a problem too large to run in full. */
int attn_ref_rows_f64(const double *q, const double *k, const double *v,
                      const int32_t *rows, long n,
                      double *o_rows, double *lse_rows,
                      int B, int Hq, int Hkv, int Sq, int Skv, int D,
                      int causal, double scale)
{
    if (!q || !k || !v || !rows || !o_rows || !lse_rows || n < 0) return -1;
    if (bad_dims(B, Hq, Hkv, Sq, Skv, D)) return -1;
    for (long r = 0; r < n; ++r) {
        if (rows[3 * r] < 0 || rows[3 * r] >= B) return -1;
        if (rows[3 * r + 1] < 0 || rows[3 * r + 1] >= Hq) return -1;
        if (rows[3 * r + 2] < 0 || rows[3 * r + 2] >= Sq) return -1;
    }
    int fail = 0;
#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)Skv);
        if (!s) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp for schedule(dynamic, 16)
        for (long r = 0; r < n; ++r) {
            if (!s) continue;
            one_row(q, k, v, rows[3 * r], rows[3 * r + 1], rows[3 * r + 2],
                    Hq, Hkv, Sq, Skv, D, causal, scale, s,
                    o_rows + r * D, lse_rows + r);
        }
        free(s);
    }
    return fail ? -2 : 0;
}

/* The softmax weights p_j / l of one row, p_out [Skv] (zeros where masked);
 * lets a test look at the probabilities themselves. */
int attn_ref_probs_f64(const double *q, const double *k,
                       int b, int h, int i, double *p_out,
                       int B, int Hq, int Hkv, int Sq, int Skv, int D,
                       int causal, double scale)
{
    if (!q || !k || !p_out) return -1;
    if (bad_dims(B, Hq, Hkv, Sq, Skv, D)) return -1;
    if (b < 0 || b >= B || h < 0 || h >= Hq || i < 0 || i >= Sq) return -1;
    double *o_row = (double *)malloc(sizeof(double) * (size_t)D);
    double *zeros = (double *)calloc((size_t)Skv * Hkv * D * (size_t)B, sizeof(double));
    if (!o_row || !zeros) { free(o_row); free(zeros); return -2; }
    double lse;
    /* V does not enter the weights: feed zeros. */
    one_row(q, k, zeros, b, h, i, Hq, Hkv, Sq, Skv, D, causal, scale,
            p_out, o_row, &lse);
    free(o_row);
    free(zeros);
    return 0;
}

int attn_ref_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
