/* tri_oracle.c -- CPU oracle for the tiled lower-triangular forward solve  L X = B.
 *
 * TEST INFRASTRUCTURE.  Slow, literal reference that the GPU library is checked
 * against.  Nothing in the product path may include, link or call it; it shares no
 * code, header, table or helper with the HIP sources.
 *
 * What it computes.  The paper's second running example: the forward triangular solve
 * with several right-hand sides,
 *     X_i. = ( B_i. - sum_{j<i} L_ij X_j. ) / L_ii                ("Representative recurrences"),
 * and its tiled form ("Multiple Iteration Spaces"): with rows cut into tiles of nb,
 *     X_I = B_I ;  for J < I, ascending:  X_I -= GEMM(L_IJ, X_J) ;  X_I = TRSM(L_II, X_I).
 *
 *   tri_scalar_f64   the scalar recurrence as written, in fp64: the definition.
 *   tri_tiled_bf16   the tiled recurrence in the arithmetic of the GPU library:
 *     - L holds bfloat16 values (uint16 bit patterns), B and X are fp32;
 *     - a solved tile X_J enters the GEMMs of the tri-space rounded to bfloat16
 *       (nearest even); these rounded values are returned as Xh;
 *     - GEMM(L_IJ, Xh_J) is the weight-stationary chain of the matrix-multiply
 *       recurrence with L_IJ as the stationary weights: per output a partial sum that
 *       starts at +0.0f and takes one fp32 add per k, k ascending (the bf16 x bf16
 *       product is exact in fp32); X_I -= G is one fp32 subtraction per element;
 *     - TRSM(L_II, R) is the scalar recurrence inside the tile, in fp32, on the
 *       unrounded x: t = R_r; t = fma(-L_rj, x_j, t) for j ascending; x_r = t / L_rr
 *       (IEEE fp32 division).
 *   Entries of L above the diagonal are never read.
 *
 * Readings where the paper is loose: the scalar form is printed as X_ri with the
 * right-hand-side index first (X L^T = B); the tiled form and the dataflow figures use
 * block rows of L X = B, which is what is taken here, X and B being n x nrhs row-major.
 * The sum's bound is printed once as k < i; it is j < i.  The paper names no precision:
 * the bf16 / fp32 split follows the matrix-multiply path whose kernel the tri-space
 * reuses, and the tile size nb is part of the method because it fixes where X is rounded.
 *
 * Parity pins (tests/test_tri_oracle_pins.py): fp64 library triangular solve, L = I,
 * diagonal L, integer systems whose solution is exact in every arithmetic, nb >= n
 * reducing to the scalar recurrence, column independence, planted mistakes.
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

/* X_i. = (B_i. - sum_{j<i} L_ij X_j.) / L_ii in fp64.  L n x n, B and X n x nrhs, row-major. */
int tri_scalar_f64(const double *L, const double *B, double *X, int64_t n, int64_t nrhs)
{
    for (int64_t i = 0; i < n; ++i)
        for (int64_t c = 0; c < nrhs; ++c) {
            double t = B[i * nrhs + c];
            for (int64_t j = 0; j < i; ++j) t -= L[i * n + j] * X[j * nrhs + c];
            X[i * nrhs + c] = t / L[i * n + i];
        }
    return 0;
}

/* The tiled recurrence for the columns c0 .. c0+nc-1 of the right-hand side (columns are
 * independent of one another).  x and xh are n x nc scratch, row-major. */
static void tiled_columns(const uint16_t *L, const float *B, float *X, uint16_t *Xh, int64_t n, int64_t nrhs,
                          int64_t nb, int64_t c0, int64_t nc, float *x, float *xh)
{
    for (int64_t i0 = 0; i0 < n; i0 += nb) {                     /* tile I */
        const int64_t i1 = i0 + nb < n ? i0 + nb : n;
        /* X_I = B_I */
        for (int64_t r = i0; r < i1; ++r)
            for (int64_t c = 0; c < nc; ++c) x[r * nc + c] = B[r * nrhs + c0 + c];
        /* for J < I:  X_I -= GEMM(L_IJ, Xh_J) */
        for (int64_t j0 = 0; j0 < i0; j0 += nb) {
            const int64_t j1 = j0 + nb;                          /* tiles before I are full */
            for (int64_t r = i0; r < i1; ++r)
                for (int64_t c = 0; c < nc; ++c) {
                    float g = 0.0f;                              /* the chain enters at 0 */
                    for (int64_t k = j0; k < j1; ++k) g = g + widen(L[r * n + k]) * xh[k * nc + c];
                    x[r * nc + c] = x[r * nc + c] - g;
                }
        }
        /* X_I = TRSM(L_II, X_I) */
        for (int64_t r = i0; r < i1; ++r)
            for (int64_t c = 0; c < nc; ++c) {
                float t = x[r * nc + c];
                for (int64_t j = i0; j < r; ++j) t = fmaf(-widen(L[r * n + j]), x[j * nc + c], t);
                x[r * nc + c] = t / widen(L[r * n + r]);
            }
        /* publish the tile; its bf16 rounding is what later GEMMs stream */
        for (int64_t r = i0; r < i1; ++r)
            for (int64_t c = 0; c < nc; ++c) {
                const uint16_t h = narrow(x[r * nc + c]);
                xh[r * nc + c] = widen(h);
                X[r * nrhs + c0 + c] = x[r * nc + c];
                Xh[r * nrhs + c0 + c] = h;
            }
    }
}

int tri_tiled_bf16(const uint16_t *L, const float *B, float *X, uint16_t *Xh, int64_t n, int64_t nrhs, int64_t nb)
{
    if (n <= 0 || nrhs <= 0) return 0;
    if (nb <= 0) return -2;
    const int64_t CB = 16;                                       /* columns per work item */
    const int64_t nblocks = (nrhs + CB - 1) / CB;
    int failed = 0;
#pragma omp parallel
    {
        float *x = (float *)malloc((size_t)n * CB * sizeof(float));
        float *xh = (float *)malloc((size_t)n * CB * sizeof(float));
        if (!x || !xh) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp barrier
        int skip;
#pragma omp atomic read
        skip = failed;
        if (!skip) {
#pragma omp for schedule(dynamic)
            for (int64_t b = 0; b < nblocks; ++b) {
                const int64_t c0 = b * CB, nc = c0 + CB <= nrhs ? CB : nrhs - c0;
                tiled_columns(L, B, X, Xh, n, nrhs, nb, c0, nc, x, xh);
            }
        }
        free(x);
        free(xh);
    }
    return failed ? -1 : 0;
}
