// cyc_tri.hip -- tiled lower-triangular forward solve  L X = B  on gfx950.
//
// The paper's second running example ("Representative recurrences", "Multiple Iteration
// Spaces"): with the rows cut into tiles of nb,
//     X_I = TRSM( L_II,  B_I - sum_{J<I} GEMM(L_IJ, X_J) ).
// It has two iteration spaces.  The triangular space does the GEMMs: there L_IJ is the
// stationary operand and the solved tile X_J is streamed past it -- the weight-stationary
// matrix-multiply recurrence of this library, whose MFMA kernels are reused as they are (with
// A addressed as a window of L and the result subtracted from the running right-hand side).
// The diagonal space does the small triangular solves, in the kernel below.  The paper's
// hand-offs between the spaces are memory here: a solved tile is published as X (fp32) and as
// Xh, its rounding to bfloat16, which is the form in which it enters later GEMMs.
//
// Schedule.  The paper's tile-by-tile order (for I: for J < I) leaves each GEMM with nb rows,
// far too few to fill 256 compute units.  The same sums are grouped recursively instead:
//     solve rows [r0, mid);  rows [mid, r1) -= L[mid:r1, r0:mid] * Xh[r0:mid];  solve rows [mid, r1)
// so that half of all multiply-adds sit in one n/2 x n/2 x nrhs GEMM, a quarter in two of half
// that size, and so on down to single tiles.  Only the order in which the GEMM terms are
// subtracted from B changes (fp32 rounding); where X is rounded to bfloat16 does not: after
// every tile of nb rows.
#include "cyc_internal.h"

namespace cyc {
namespace {

#define CYC_LDS __attribute__((address_space(3)))

__device__ __forceinline__ float widen_bf16(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }
// fp32 -> bfloat16, nearest, ties to even; NaN stays NaN
__device__ __forceinline__ uint16_t round_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

constexpr int SUB = 8;     // rows a lane carries at a time

// Diagonal space: X_I = TRSM(L_II, R_I) for one tile of `rows` <= NB rows starting at row r0, all
// right-hand sides.  One wave per 64 columns, one lane per column: a column of X is a chain
//     t = R_r;  t = fma(-L_rj, x_j, t)  for j ascending over the tile's earlier rows;  x_r = t / L_rr
// in fp32 on the unrounded x.  A lane works on SUB rows at a time: SUB independent chains take the
// x of all earlier rows of the tile (kept in LDS, one column per lane), then the SUB x SUB corner is
// solved in registers.  L_II is staged in LDS once, transposed ([j][r], fp32), so that the SUB
// coefficients a step needs are two broadcast 16-byte reads; nothing above the diagonal is used.
// FULL: the tile has exactly NB rows and its rows of L are 16-byte aligned (no per-row checks).
template <int NB, bool FULL>
__global__ __launch_bounds__(64) void tri_diag_kernel(const uint16_t *__restrict__ L, int64_t n, const float *Rin,
                                                      float *X, uint16_t *__restrict__ Xh, int64_t nrhs, int64_t r0,
                                                      int rows_arg, int vec_arg)
{
    const int rows = FULL ? NB : rows_arg;
    const bool vec = FULL || vec_arg;
    __shared__ __attribute__((aligned(16))) float Lt[NB][NB];    // Lt[j][r] = L[r0+r][r0+j], j <= r
    __shared__ float xs[NB][64];                                 // xs[j][lane] = x_j of this lane's column
    const int lane = threadIdx.x;
    const int64_t c = (int64_t)blockIdx.x * 64 + lane;

    // stage L_II.  With 16-byte aligned rows each lane fetches 16-byte pieces of rows, all loads in flight
    // together (pieces wholly above the diagonal are skipped; of a piece that straddles it only the part
    // at or below the diagonal is used); otherwise element by element.
    if (vec) {
        const int cpr = rows >> 3;                               // 16-byte pieces per row of the tile
        constexpr int PER_LANE = NB * NB / 8 / 64;
        uint4 piece[PER_LANE];
#pragma unroll
        for (int x = 0; x < PER_LANE; ++x) {
            const int id = lane + 64 * x, r = id / cpr, jc = id - r * cpr;
            piece[x] = make_uint4(0, 0, 0, 0);
            if (r < rows && jc * 8 <= r) piece[x] = *(const uint4 *)(L + (r0 + r) * n + r0 + jc * 8);
        }
#pragma unroll
        for (int x = 0; x < PER_LANE; ++x) {
            const int id = lane + 64 * x, r = id / cpr, jc = id - r * cpr;
            if (r < rows && jc * 8 <= r) {
                const uint32_t w[4] = {piece[x].x, piece[x].y, piece[x].z, piece[x].w};
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int j = jc * 8 + e;
                    if (j <= r) Lt[j][r] = widen_bf16((uint16_t)(w[e >> 1] >> (16 * (e & 1))));
                }
            }
        }
    } else {
        for (int r = lane; r < rows; r += 64)
            for (int j = 0; j <= r; ++j) Lt[j][r] = widen_bf16(L[(r0 + r) * n + r0 + j]);
    }
    __syncthreads();
    if (c >= nrhs) return;        // lanes past the last column only helped staging L; no barrier follows

    // the tile's right-hand side comes in with one round of loads, not one per SUB rows
    const float *rp = Rin + r0 * nrhs + c;
    float *xp = X + r0 * nrhs + c;
    uint16_t *hp = Xh + r0 * nrhs + c;
    float rhs[NB];
#pragma unroll
    for (int r = 0; r < NB; ++r) rhs[r] = r < rows ? rp[r * nrhs] : 0.0f;

#pragma unroll
    for (int rb = 0; rb < NB; rb += SUB) {
        if (rb >= rows) continue;                                // uniform over the wave
        float t[SUB];
#pragma unroll
        for (int q = 0; q < SUB; ++q) t[q] = rhs[rb + q];
        // earlier rows of the tile
#pragma unroll 8
        for (int j = 0; j < rb; ++j) {
            const float x = xs[j][lane];
            const float4 l0 = *(const float4 *)&Lt[j][rb], l1 = *(const float4 *)&Lt[j][rb + 4];
            t[0] = __builtin_fmaf(-l0.x, x, t[0]);
            t[1] = __builtin_fmaf(-l0.y, x, t[1]);
            t[2] = __builtin_fmaf(-l0.z, x, t[2]);
            t[3] = __builtin_fmaf(-l0.w, x, t[3]);
            t[4] = __builtin_fmaf(-l1.x, x, t[4]);
            t[5] = __builtin_fmaf(-l1.y, x, t[5]);
            t[6] = __builtin_fmaf(-l1.z, x, t[6]);
            t[7] = __builtin_fmaf(-l1.w, x, t[7]);
        }
        // the SUB x SUB corner
#pragma unroll
        for (int q = 0; q < SUB; ++q) {
            if (rb + q < rows) {                                 // uniform over the wave
#pragma unroll
                for (int p = 0; p < q; ++p) t[q] = __builtin_fmaf(-Lt[rb + p][rb + q], t[p], t[q]);
                t[q] = t[q] / Lt[rb + q][rb + q];
                xs[rb + q][lane] = t[q];
                xp[(rb + q) * nrhs] = t[q];
                hp[(rb + q) * nrhs] = round_bf16(t[q]);
            }
        }
    }
}

struct Solve {
    const uint16_t *L;
    const float *B;
    float *X;
    uint16_t *Xh;
    int64_t n, nrhs, nb;
    hipStream_t s;
};

// the running right-hand side of rows that no GEMM has touched yet is still B; afterwards it lives in X
inline const float *rhs_of(const Solve &v, int64_t r0) { return r0 == 0 ? v.B : v.X; }

hipError_t diag(const Solve &v, int64_t r0, int64_t r1)
{
    dim3 grid((unsigned)((v.nrhs + 63) / 64));
    const float *R = rhs_of(v, r0);
    const int rows = (int)(r1 - r0);
    // 16-byte pieces of the tile's rows can be fetched whole
    const int vec = ((uintptr_t)v.L % 16 == 0) && v.n % 8 == 0 && r0 % 8 == 0 && rows % 8 == 0;
    if (vec && rows == 64)
        hipLaunchKernelGGL((tri_diag_kernel<64, true>), grid, dim3(64), 0, v.s, v.L, v.n, R, v.X, v.Xh, v.nrhs, r0, rows, vec);
    else if (vec && rows == 128)
        hipLaunchKernelGGL((tri_diag_kernel<128, true>), grid, dim3(64), 0, v.s, v.L, v.n, R, v.X, v.Xh, v.nrhs, r0, rows, vec);
    else if (rows <= 64)
        hipLaunchKernelGGL((tri_diag_kernel<64, false>), grid, dim3(64), 0, v.s, v.L, v.n, R, v.X, v.Xh, v.nrhs, r0, rows, vec);
    else
        hipLaunchKernelGGL((tri_diag_kernel<128, false>), grid, dim3(64), 0, v.s, v.L, v.n, R, v.X, v.Xh, v.nrhs, r0, rows, vec);
    return hipGetLastError();
}

// rows [mid, r1) of the running right-hand side  -=  L[mid:r1, r0:mid] * Xh[r0:mid]
hipError_t update(const Solve &v, int64_t r0, int64_t mid, int64_t r1)
{
    Problem p;
    p.A = v.L + mid * v.n + r0;
    p.lda = v.n;
    p.B = v.Xh + r0 * v.nrhs;
    p.C = v.X + mid * v.nrhs;
    p.Cin = rhs_of(v, r0) + mid * v.nrhs;
    p.batch = 1;
    p.M = r1 - mid;
    p.K = mid - r0;
    p.N = v.nrhs;
    p.strideA = p.strideB = p.strideC = 0;
    p.i8 = false;
    const int tile = choose_mfma_tile(p);
    return tile ? launch_mfma(p, tile, 16, v.s) : launch_generic(p, v.s);
}

hipError_t solve(const Solve &v, int64_t r0, int64_t r1)
{
    if (r1 - r0 <= v.nb) return diag(v, r0, r1);
    const int64_t tiles = (r1 - r0 + v.nb - 1) / v.nb;
    const int64_t mid = r0 + (tiles + 1) / 2 * v.nb;       // the first half takes the odd tile: mid stays a tile boundary
    hipError_t e = solve(v, r0, mid);
    if (e == hipSuccess) e = update(v, r0, mid, r1);
    if (e == hipSuccess) e = solve(v, mid, r1);
    return e;
}

}  // namespace

hipError_t launch_trsm(const void *L, const void *B, void *X, void *Xh, int64_t n, int64_t nrhs, int64_t nb, hipStream_t s)
{
    if (nb < 1 || nb > 128 || (int64_t)((nrhs + 63) / 64) > 0x7fffffff) return hipErrorInvalidValue;
    Solve v{(const uint16_t *)L, (const float *)B, (float *)X, (uint16_t *)Xh, n, nrhs, nb, s};
    return solve(v, 0, n);
}

}  // namespace cyc
