/* attn_oracle.c -- CPU oracle for the FlashAttention-2 tile recurrence.
 *
 * TEST INFRASTRUCTURE.  Slow, literal reference that the GPU library is checked
 * against.  Nothing in the product path may include, link or call it; it shares no
 * code, header, table or helper with the HIP sources.
 *
 * The paper ("FlashAttention-2 Recurrence") processes keys and values in tiles J_t and keeps,
 * per query i, a running maximum m_i, a running sum l_i and a running output o_i (a d-vector):
 *     S_ij  = alpha * Q_i. K_j.^T               alpha = 1/sqrt(d)
 *     mh    = max(m_i, max_{j in J_t} S_ij)
 *     l_i   = exp(m_i - mh) * l_i + sum_{j in J_t} exp(S_ij - mh)
 *     o_i   = exp(m_i - mh) * o_i + sum_{j in J_t} exp(S_ij - mh) * V_j.
 *     m_i   = mh
 * and finally O_i. = o_i / l_i.  Whatever the tiles, this equals
 *     O_i. = sum_j softmax_j(alpha * Q_i. K_j.^T) * V_j.
 * exactly up to rounding, so the second form is the definition and the first is checked
 * against it.
 *
 *   attn_definition_f64   the softmax form, in fp64 (row maximum subtracted before exp, which
 *                         changes nothing mathematically)
 *   attn_recurrence_f64   the tile recurrence as printed, in fp64, key tiles of `tile` keys
 *                         (the last one may be shorter); m starts at -infinity, l and o at 0
 *
 * Q is N x d, K and V are M x d, O is N x d, row-major doubles.  (The GPU library takes
 * bfloat16 Q, K, V; the tests widen them exactly to fp64 before calling the oracle.)
 *
 * Parity pins (tests/test_attn_oracle_pins.py): hand-worked cases, uniform attention (all scores
 * equal gives the mean of V), one dominant key, one key (O = V_0), tile-size independence,
 * shift invariance of the scores, rows of O inside the convex hull of V, planted mistakes.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

int attn_definition_f64(const double *Q, const double *K, const double *V, double *O, int64_t N, int64_t M, int64_t d)
{
    if (N <= 0 || M <= 0 || d <= 0) return 0;
    const double alpha = 1.0 / sqrt((double)d);
    int failed = 0;
#pragma omp parallel
    {
        double *s = (double *)malloc((size_t)M * sizeof(double));
        if (!s) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp barrier
        int skip;
#pragma omp atomic read
        skip = failed;
        if (!skip) {
#pragma omp for schedule(static)
            for (int64_t i = 0; i < N; ++i) {
                double top = -INFINITY;
                for (int64_t j = 0; j < M; ++j) {
                    double acc = 0.0;
                    for (int64_t c = 0; c < d; ++c) acc += Q[i * d + c] * K[j * d + c];
                    s[j] = alpha * acc;
                    if (s[j] > top) top = s[j];
                }
                double sum = 0.0;
                for (int64_t j = 0; j < M; ++j) {
                    s[j] = exp(s[j] - top);
                    sum += s[j];
                }
                for (int64_t c = 0; c < d; ++c) {
                    double acc = 0.0;
                    for (int64_t j = 0; j < M; ++j) acc += s[j] * V[j * d + c];
                    O[i * d + c] = acc / sum;
                }
            }
        }
        free(s);
    }
    return failed ? -1 : 0;
}

int attn_recurrence_f64(const double *Q, const double *K, const double *V, double *O, int64_t N, int64_t M, int64_t d,
                        int64_t tile)
{
    if (N <= 0 || M <= 0 || d <= 0) return 0;
    if (tile <= 0) return -2;
    const double alpha = 1.0 / sqrt((double)d);
    int failed = 0;
#pragma omp parallel
    {
        double *s = (double *)malloc((size_t)tile * sizeof(double));
        double *o = (double *)malloc((size_t)d * sizeof(double));
        if (!s || !o) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp barrier
        int skip;
#pragma omp atomic read
        skip = failed;
        if (!skip) {
#pragma omp for schedule(static)
            for (int64_t i = 0; i < N; ++i) {
                double m = -INFINITY, l = 0.0;                     /* state of query i */
                for (int64_t c = 0; c < d; ++c) o[c] = 0.0;
                for (int64_t j0 = 0; j0 < M; j0 += tile) {          /* tile J_t */
                    const int64_t nj = j0 + tile <= M ? tile : M - j0;
                    double mh = m;
                    for (int64_t j = 0; j < nj; ++j) {
                        double acc = 0.0;
                        for (int64_t c = 0; c < d; ++c) acc += Q[i * d + c] * K[(j0 + j) * d + c];
                        s[j] = alpha * acc;
                        if (s[j] > mh) mh = s[j];
                    }
                    const double keep = exp(m - mh);               /* exp(-inf) = 0 on the first tile */
                    l = keep * l;
                    for (int64_t c = 0; c < d; ++c) o[c] = keep * o[c];
                    for (int64_t j = 0; j < nj; ++j) {
                        const double p = exp(s[j] - mh);
                        l += p;
                        for (int64_t c = 0; c < d; ++c) o[c] += p * V[(j0 + j) * d + c];
                    }
                    m = mh;
                }
                for (int64_t c = 0; c < d; ++c) O[i * d + c] = o[c] / l;
            }
        }
        free(s);
        free(o);
    }
    return failed ? -1 : 0;
}
