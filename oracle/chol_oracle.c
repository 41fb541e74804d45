/* chol_oracle.c -- CPU oracle for the tiled Cholesky factorisation  A = L L^T  (L lower triangular).
 *
 * TEST INFRASTRUCTURE.  Slow, literal reference that the GPU library is checked
 * against.  Nothing in the product path may include, link or call it; it shares no
 * code, header, table or helper with the HIP sources.
 *
 * What it computes.  The scalar recurrence ("Representative recurrences", Cholesky, lower L):
 *     L_ii = sqrt( A_ii - sum_{k<i} L_ik^2 ),      L_ij = ( A_ij - sum_{k<j} L_ik L_jk ) / L_jj   for j < i,
 * and its tiled form ("Cholesky Recurrence"): with A cut into nb x nb tiles, for every panel j
 *     S_jj = A_jj - sum_{k<j} SYRK(L_jk),          L_jj = CHOL(S_jj),
 *     S_ij = A_ij - sum_{k<j} GEMM(L_ik, L_jk),    L_ij = TRSM(S_ij, L_jj)        for i > j.
 *
 *   chol_scalar_f64   the scalar recurrence as written, in fp64: the definition.
 *   chol_tiled_bf16   the tiled recurrence in the arithmetic of the GPU library:
 *     - A and L are fp32; a finished tile L_ik enters the GEMMs and SYRKs of later panels rounded to
 *       bfloat16 (nearest even); these rounded values are returned as Lh;
 *     - GEMM(L_ik, L_jk) = L_ik L_jk^T is the weight-stationary chain of the matrix-multiply recurrence:
 *       per output a partial sum that starts at +0.0f and takes one fp32 add per term, terms ascending
 *       (the bf16 x bf16 product is exact in fp32); S -= G is one fp32 subtraction per element and tile k,
 *       k ascending.  SYRK(L_jk) is the same with i = j;
 *     - CHOL and TRSM are the scalar recurrence inside the tile column, in fp32, on unrounded values:
 *       for column c ascending, for every row r at or below it,  t = S_rc;  t = fma(-L_rk, L_ck, t) for the
 *       columns k < c of the tile, ascending;  then L_cc = sqrtf(t) on the diagonal and L_rc = t / L_cc
 *       below it (IEEE fp32 square root and division).  The rows of the diagonal tile and of the tiles
 *       under it are treated alike: TRSM(S_ij, L_jj) is exactly the off-diagonal line of the recurrence.
 *   Only the lower triangle of A is read; the strictly upper triangle of L is returned as zero.
 *
 * Readings where the paper is loose: the tiled form prints SYRK(A_jk) and GEMM(A_ik, A_jk); the operands
 * are the finished factor tiles L_jk, L_ik (A overwritten in place), and GEMM(X, Y) = X Y^T.  The paper
 * names no precision: the bf16 / fp32 split follows the matrix-multiply path whose kernel the updates
 * reuse, and the tile size nb is part of the method because it fixes where L is rounded.  A matrix that
 * is not positive definite gives NaNs from the square root, not an error.
 *
 * Parity pins (tests/test_chol_oracle_pins.py): hand-worked factors, the fp64 library Cholesky,
 * L L^T = A, integer factors that are exact in every arithmetic, nb >= n reducing to the scalar
 * recurrence in fp32, diagonal A, planted mistakes.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static inline float widen(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* fp32 -> bfloat16, round to nearest, ties to even; NaN stays NaN */
static inline uint16_t narrow(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

/* The scalar recurrence in fp64.  A and L n x n row-major; the upper triangle of L is set to zero. */
int chol_scalar_f64(const double *A, double *L, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) {
        for (int64_t j = 0; j < i; ++j) {
            double t = A[i * n + j];
            for (int64_t k = 0; k < j; ++k) t -= L[i * n + k] * L[j * n + k];
            L[i * n + j] = t / L[j * n + j];
        }
        double t = A[i * n + i];
        for (int64_t k = 0; k < i; ++k) t -= L[i * n + k] * L[i * n + k];
        L[i * n + i] = sqrt(t);
        for (int64_t j = i + 1; j < n; ++j) L[i * n + j] = 0.0;
    }
    return 0;
}

/* The tiled recurrence.  A, L fp32 n x n row-major; Lh bfloat16 bit patterns of L (lower triangle; zero above). */
int chol_tiled_bf16(const float *A, float *L, uint16_t *Lh, int64_t n, int64_t nb)
{
    if (n <= 0) return 0;
    if (nb <= 0) return -2;
    float *lh = (float *)malloc((size_t)n * (size_t)n * sizeof(float));   /* Lh widened, for the chains */
    if (!lh) return -1;
    for (int64_t i = 0; i < n * n; ++i) {
        L[i] = 0.0f;
        Lh[i] = 0;
        lh[i] = 0.0f;
    }
    for (int64_t j0 = 0; j0 < n; j0 += nb) {                         /* panel j */
        const int64_t j1 = j0 + nb < n ? j0 + nb : n;
        /* S_ij = A_ij - sum_{k<j} GEMM(L_ik, L_jk)  for the rows r >= j0 (tile rows i >= j), columns of the
         * panel at or left of the diagonal; kept in L until the tile column is solved */
#pragma omp parallel for schedule(dynamic, 8)
        for (int64_t r = j0; r < n; ++r)
            for (int64_t c = j0; c < j1 && c <= r; ++c) {
                float x = A[r * n + c];
                for (int64_t k0 = 0; k0 < j0; k0 += nb) {            /* tiles k < j are full */
                    float g = 0.0f;                                  /* the chain enters at 0 */
                    for (int64_t k = k0; k < k0 + nb; ++k) g = g + lh[r * n + k] * lh[c * n + k];
                    x = x - g;
                }
                L[r * n + c] = x;
            }
        /* L_jj = CHOL(S_jj), L_ij = TRSM(S_ij, L_jj): column by column inside the panel */
        for (int64_t c = j0; c < j1; ++c) {
            float t = L[c * n + c];
            for (int64_t k = j0; k < c; ++k) t = fmaf(-L[c * n + k], L[c * n + k], t);
            const float d = sqrtf(t);
            L[c * n + c] = d;
#pragma omp parallel for schedule(static)
            for (int64_t r = c + 1; r < n; ++r) {
                float u = L[r * n + c];
                for (int64_t k = j0; k < c; ++k) u = fmaf(-L[r * n + k], L[c * n + k], u);
                L[r * n + c] = u / d;
            }
        }
        /* publish the panel; its bf16 rounding is what later panels stream */
        for (int64_t r = j0; r < n; ++r)
            for (int64_t c = j0; c < j1 && c <= r; ++c) {
                const uint16_t h = narrow(L[r * n + c]);
                Lh[r * n + c] = h;
                lh[r * n + c] = widen(h);
            }
    }
    free(lh);
    return 0;
}
