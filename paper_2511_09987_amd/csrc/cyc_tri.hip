// cyc_tri.hip -- tiled lower-triangular forward solve  L X = B  on gfx950.
//
// The paper's second running example ("Representative recurrences", "Multiple Iteration
// Spaces"): with the rows cut into tiles of nb,
//     X_I = TRSM( L_II,  B_I - sum_{J<I} GEMM(L_IJ, X_J) ).
// It has two iteration spaces.  The triangular space does the GEMMs: there L_IJ is the
// stationary operand and the solved tile X_J is streamed past it -- the weight-stationary
// matrix-multiply recurrence of this library, whose MFMA kernels are reused as they are (with
// A addressed as a window of L and the result subtracted from the running right-hand side).
// The diagonal space does the small triangular solves, in the kernels below: by substitution, or,
// for tiles of 64 rows that are well conditioned, as a product with the tile's inverse on the
// matrix cores (the inverses of all diagonal tiles are computed ahead, by that substitution).
// The paper's hand-offs between the spaces are memory here: a solved tile is published as X (fp32) and as
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
#include "cyc_wave.h"

namespace cyc {
namespace {

#define CYC_LDS __attribute__((address_space(3)))

constexpr int SUB = 8;     // rows a lane carries at a time

__device__ __forceinline__ float widen_bf16(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }
// fp32 -> bfloat16 bit pattern, round to nearest, ties to even; NaN stays NaN (the hardware conversion)
__device__ __forceinline__ uint16_t round_bf16(float f) { return __builtin_bit_cast(uint16_t, (__bf16)f); }


// SUB chains take the x of the tile's rows [0, rb): t[q] = fma(-L[rb+q][j], x_j, t[q]) for j ascending.
// rb is a multiple of 8.  The LDS reads of eight steps are issued together and only then consumed (left to
// itself the scheduler, under register pressure, issues them one step at a time and every step then
// waits out the full LDS latency).  Lt[j][r] = L[r][j] (fp32), xs[j][lane] = x_j of this lane's column.
template <int NB>
__device__ __forceinline__ void take_earlier_rows(float (&t)[SUB], const float (*Lt)[NB], const float (*xs)[64], int rb, int lane)
{
#pragma unroll 1
    for (int j0 = 0; j0 < rb; j0 += 8) {
        float x[8];
        float4 l0[8], l1[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            x[u] = xs[j0 + u][lane];
            l0[u] = *(const float4 *)&Lt[j0 + u][rb];
            l1[u] = *(const float4 *)&Lt[j0 + u][rb + 4];
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            t[0] = __builtin_fmaf(-l0[u].x, x[u], t[0]);
            t[1] = __builtin_fmaf(-l0[u].y, x[u], t[1]);
            t[2] = __builtin_fmaf(-l0[u].z, x[u], t[2]);
            t[3] = __builtin_fmaf(-l0[u].w, x[u], t[3]);
            t[4] = __builtin_fmaf(-l1[u].x, x[u], t[4]);
            t[5] = __builtin_fmaf(-l1[u].y, x[u], t[5]);
            t[6] = __builtin_fmaf(-l1[u].z, x[u], t[6]);
            t[7] = __builtin_fmaf(-l1[u].w, x[u], t[7]);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

// The SUB x SUB corner of L_II that couples the rows rb .. rb+SUB-1, fetched in one round before the chains
// over the earlier rows run, so that no LDS read sits inside the dependent chain of the corner solve:
// corner(p, q) = L[rb+q][rb+p] for p <= q.
template <int NB>
struct Corner {
    float4 lo[SUB], hi[SUB];
    __device__ __forceinline__ void fetch(const float (*Lt)[NB], int rb)
    {
#pragma unroll
        for (int p = 0; p < SUB; ++p) {
            lo[p] = *(const float4 *)&Lt[rb + p][rb];
            hi[p] = *(const float4 *)&Lt[rb + p][rb + 4];
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    __device__ __forceinline__ float at(int p, int q) const
    {
        const float4 v = q < 4 ? lo[p] : hi[p];
        const int e = q & 3;
        return e == 0 ? v.x : e == 1 ? v.y : e == 2 ? v.z : v.w;
    }
};

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
    // xs[r][lane] holds R_r until row r is solved and x_r from then on.  (The loop over the row groups
    // below is deliberately not unrolled: a wave runs through this code once, so straight-line code
    // would be fetched from memory instruction by instruction; a loop body stays in the instruction cache.)
#pragma unroll 16
    for (int r = 0; r < rows; ++r) xs[r][lane] = rp[r * nrhs];

#pragma unroll 1
    for (int rb = 0; rb < rows; rb += SUB) {
        float t[SUB];
#pragma unroll
        for (int q = 0; q < SUB; ++q) t[q] = rb + q < rows ? xs[rb + q][lane] : 0.0f;
        Corner<NB> corner;
        corner.fetch(Lt, rb);
        take_earlier_rows<NB>(t, Lt, xs, rb, lane);
        // the SUB x SUB corner
#pragma unroll
        for (int q = 0; q < SUB; ++q) {
            if (rb + q < rows) {                                 // uniform over the wave
#pragma unroll
                for (int p = 0; p < q; ++p) t[q] = __builtin_fmaf(-corner.at(p, q), t[p], t[q]);
                t[q] = t[q] / corner.at(q, q);
                xs[rb + q][lane] = t[q];
                xp[(rb + q) * nrhs] = t[q];
                hp[(rb + q) * nrhs] = round_bf16(t[q]);
            }
        }
    }
}

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x2 __attribute__((ext_vector_type(2)));

// The diagonal solve of one full tile of 64 rows by one wave, one lane per right-hand side, with the lane's column
// in registers (constant indices after unrolling): x[r] holds R_r on entry; xn[r] = -x_r on return (a multiply-add
// without a negated operand has a 4-byte encoding, which a lone wave issues faster).  The chains of tri_diag_kernel as
// the list of steps of cyc_wave.h: four rows at a time, their chains over the rows above the four side by side, then
// the 4 x 4 corner, whose divisions run in phases with steps of the next four rows between them.  Every x still takes
// its terms in ascending j.  The rows of L_tt (D, fp32, row-major in LDS) for a step are requested two steps before
// it runs, since a lone wave has nobody else to hide the LDS latency behind.  emit(r, x_r) is called once per row, in
// order, without conditions on the lane (a branch there would cut the chains into basic blocks, and they would be
// moved apart, each to its own division); middle() is called once, before the last four blocks.
template <int LDD, class Emit, class Middle>
__device__ __forceinline__ void solve_tile64(const float (*D)[LDD], const float (&x)[64], float (&xn)[64], Emit emit, Middle middle)
{
    constexpr int NB = 64;
    static_assert(NBLK * 4 == NB, "the step list is for tiles of 64 rows");
    float tt[4], tn[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    f32x4 q[3][4], qc[2][4];
    auto rows_of_L = [&](int i) __attribute__((always_inline)) {            // operands of bulk step i
        if (STEPS.b[i] >= 0) {
#pragma unroll
            for (int j = 0; j < 4; ++j) q[i % 3][j] = *(const f32x4 *)&D[4 * STEPS.b[i] + j][4 * STEPS.k[i]];
        }
    };
    auto quarter = [&](float(&acc)[4], int i, int kk) __attribute__((always_inline)) {   // a quarter of bulk step i
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[j] = __builtin_fmaf(q[i % 3][j][kk], xn[4 * STEPS.k[i] + kk], acc[j]);
    };
    rows_of_L(0);
    rows_of_L(1);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        qc[0][j] = *(const f32x4 *)&D[j][0];
        tt[j] = x[j];
    }
    int i = 0;                                                              // the next bulk step
    auto block = [&](auto index) __attribute__((always_inline)) {
        constexpr int b = decltype(index)::value;
#pragma unroll
        for (int s = early_of(b); s < b; ++s) {                             // the block's bulk steps taken in turn
            rows_of_L(i + 2);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) quarter(tt, i, kk);
            ++i;
        }
        if (b + 1 < NBLK) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                qc[(b + 1) & 1][j] = *(const f32x4 *)&D[4 * (b + 1) + j][4 * (b + 1)];
                tn[j] = x[4 * (b + 1) + j];
            }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {                                       // the corner, row by row
            const int r = 4 * b + j;
            const bool paired = b + 1 < NBLK && j < early_of(b + 1);
            if (paired) rows_of_L(i + 2);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int e = 0; e < j; ++e) tt[j] = __builtin_fmaf(qc[b & 1][j][e], xn[4 * b + e], tt[j]);
            Division dv;
            dv.phase0(tt[j], qc[b & 1][j][j]);
            __builtin_amdgcn_sched_barrier(0);
            if (paired) quarter(tn, i, 0);
            __builtin_amdgcn_sched_barrier(0);
            dv.phase1();
            __builtin_amdgcn_sched_barrier(0);
            if (paired) quarter(tn, i, 1);
            __builtin_amdgcn_sched_barrier(0);
            dv.phase2();
            __builtin_amdgcn_sched_barrier(0);
            if (paired) quarter(tn, i, 2);
            __builtin_amdgcn_sched_barrier(0);
            const float xr = dv.phase3();
            xn[r] = -xr;
            asm("" : "+v"(xn[r]));                                          // (or the negation is folded back into the multiply-adds)
            emit(r, xr);
            __builtin_amdgcn_sched_barrier(0);
            if (paired) {
                quarter(tn, i, 3);
                ++i;
            }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) tt[j] = tn[j];
    };
    unrolled<NBLK - 4>(block);
    middle();                                                               // (the last four blocks are 58 of the 136 steps)
    unrolled<4>([&](auto index) __attribute__((always_inline)) { block(std::integral_constant<int, NBLK - 4 + decltype(index)::value>{}); });
}

// A panel of up to four full tiles of 64 rows for one slab of 64 right-hand sides, in one kernel:
//     for t = 0 .. tiles-1:   R_t = Rin_t - L[t, 0:t] * Xh[0:t]  (tri-space, inside the panel)
//                             X_t = TRSM(L_tt, R_t)              (diag-space)
// Columns of X do not depend on one another, so a wave can carry its 64 columns through the whole
// panel without waiting for any other wave; what would be seven launches (four diagonal solves, three
// small GEMMs that cannot fill the chip) becomes one.  The panel's GEMMs run on the wave's own MFMAs:
// L[t, 0:t] is the stationary operand, read from memory straight into operand registers; the panel's
// solved tiles, rounded to bfloat16, stay in LDS ([k][column]) and are read as the streamed operand
// through the LDS transpose read.  The product comes out in the MFMA's accumulator layout and crosses
// LDS once to reach the one-lane-per-column layout of the diagonal solve, which is the code above.
// Requires 16-byte aligned rows of L (n and r0 multiples of 8).
__global__ __launch_bounds__(64) void tri_panel_kernel(const uint16_t *__restrict__ L, int64_t n, const float *Rin,
                                                       float *X, uint16_t *__restrict__ Xh, int64_t nrhs, int64_t r0,
                                                       int tiles)
{
    constexpr int NB = 64, LDD = NB + 4;
    // one block, D first: in the first 64 KB of LDS a read reaches its word with the 16-bit offset field from one
    // base register
    __shared__ __attribute__((aligned(16))) struct {
        float D[NB][LDD];                  // L_tt in fp32, row-major, on and below the diagonal
        float G[NB][64 + 1];               // L[t, 0:t] * Xh[0:t], [row][column]
        uint16_t Xb[4 * NB][64];           // solved tiles as bfloat16, [k][column]
    } lds;
    auto &D = lds.D;
    auto &G = lds.G;
    auto &Xb = lds.Xb;
    const int lane = threadIdx.x, lq = lane & 15, g = lane >> 4;
    const int64_t c0 = (int64_t)blockIdx.x * 64;
    const int64_t c = c0 + lane < nrhs ? c0 + lane : nrhs - 1;         // lanes past the last column shadow it
    const bool live = c0 + lane < nrhs;
    const unsigned cl = (unsigned)(c - c0);                            // the lane's column within the slab

    // Everything a tile needs from memory -- L_tt, its right-hand side, the rows of L for its GEMM -- is
    // independent of the solves before it, so it is requested one tile ahead and arrives while the
    // previous tile is being solved.
    constexpr int cpr = NB / 8, PER_LANE = NB * NB / 8 / 64;
    uint4 piece[PER_LANE];        // 16-byte pieces of L_tt
    float rhs[2][NB];             // right-hand side of the tile being solved / of the next one
    i32x4 a[6][4];                // stationary operand of the tile's GEMM: [MFMA k-step][16-row tile]
    auto request = [&](int t) __attribute__((always_inline)) {
        const int64_t rt = r0 + (int64_t)t * NB;
#pragma unroll
        for (int x = 0; x < PER_LANE; ++x) {
            const int id = lane + 64 * x, r = id / cpr, jc = id % cpr;
            piece[x] = make_uint4(0, 0, 0, 0);
            if (jc * 8 <= r) piece[x] = *(const uint4 *)(L + (rt + r) * n + rt + jc * 8);
        }
#pragma unroll
        for (int r = 0; r < NB; ++r) rhs[t & 1][r] = (Rin + (rt + r) * nrhs + c0)[cl];      // uniform row address, 32-bit lane offset
        // row lq of 16-row tile i, k = 32 ks + 8 g .. +7, for every MFMA k-step ks of the GEMM
#pragma unroll
        for (int ks = 0; ks < 6; ++ks)                           // (constant bound: unrolls wherever the call sits)
            if (ks < 2 * t) {
#pragma unroll
                for (int i = 0; i < 4; ++i) a[ks][i] = *(const i32x4 *)(L + (rt + i * 16 + lq) * n + r0 + ks * 32 + g * 8);
            }
    };
    request(0);

#pragma unroll
    for (int t = 0; t < 4; ++t) {                                // unrolled: t is a constant in every copy
        if (t >= tiles) break;
        const int64_t rt = r0 + (int64_t)t * NB;
        // ---- stage L_tt: the 16-byte pieces on and below the diagonal, widened to fp32
#pragma unroll
        for (int x = 0; x < PER_LANE; ++x) {
            const int id = lane + 64 * x, r = id / cpr, jc = id % cpr;
            if (jc * 8 <= r) {
                const uint32_t w[4] = {piece[x].x, piece[x].y, piece[x].z, piece[x].w};
                f32x4 lo, hi;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    lo[e] = widen_bf16((uint16_t)(w[e >> 1] >> (16 * (e & 1))));
                    hi[e] = widen_bf16((uint16_t)(w[2 + (e >> 1)] >> (16 * (e & 1))));
                }
                *(f32x4 *)&D[r][jc * 8] = lo;
                *(f32x4 *)&D[r][jc * 8 + 4] = hi;
            }
        }
        // ---- tri-space inside the panel: G = L[t, 0:t] * Xb[0:t]  (64 x 64t times 64t x 64)
        if (t > 0) {
            f32x4 acc[4][4];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = (f32x4){0, 0, 0, 0};
#pragma unroll
            for (int ks = 0; ks < 2 * t; ++ks) {                 // MFMA k-steps of 32
                i32x4 b[4];
                // streamed operand: column lq of tile j, the same k, through the transpose read
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    CYC_LDS char *p = (CYC_LDS char *)&Xb[ks * 32 + 8 * g + (lq >> 2)][j * 16 + 4 * (lq & 3)];
                    const i32x2 lo = __builtin_bit_cast(i32x2, __builtin_amdgcn_ds_read_tr16_b64_v4bf16((CYC_LDS bf16x4 *)p));
                    const i32x2 hi = __builtin_bit_cast(i32x2, __builtin_amdgcn_ds_read_tr16_b64_v4bf16((CYC_LDS bf16x4 *)(p + 4 * 64 * 2)));
                    b[j] = (i32x4){lo[0], lo[1], hi[0], hi[1]};
                }
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a[ks][i]), __builtin_bit_cast(bf16x8, b[j]), acc[i][j], 0, 0, 0);
            }
            // accumulator register r of lane l is row 4*(l/16) + r, column l%16 of its 16 x 16 tile
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int r = 0; r < 4; ++r) G[i * 16 + 4 * g + r][j * 16 + lq] = acc[i][j][r];
        }
        __syncthreads();                                        // D and G are in place
        float(&x)[NB] = rhs[t & 1];                             // the lane's column: R_r until row r is solved (then xn[r] = -x_r)
        if (t > 0) {
#pragma unroll
            for (int r = 0; r < NB; ++r) x[r] -= G[r][lane];
        }

        // ---- diag-space
        float xn[NB];
        solve_tile64<LDD>(
            D, x, xn, [&](int r, float xr) __attribute__((always_inline)) { Xb[t * NB + r][lane] = round_bf16(xr); },
            // the next tile's operands: late enough to keep the registers free for most of the solve, early enough to
            // land before it ends
            [&]() __attribute__((always_inline)) { if (t + 1 < tiles) request(t + 1); });
        // the tile's results go out in one batch: a store under the lane condition inside the chains would cut them
        // into basic blocks, and the chains of a block would then be moved apart, each to its own division
        if (live) {
#pragma unroll
            for (int r = 0; r < NB; ++r) {                      // uniform row address, 32-bit lane offset
                (X + (rt + r) * nrhs + c0)[cl] = -xn[r];
                (Xh + (rt + r) * nrhs + c0)[cl] = round_bf16(-xn[r]);
            }
        }
        __syncthreads();                                        // Xb of this tile visible; D and G free for the next
    }
}

// The diagonal solve of one full tile of 64 rows by FOUR waves, all on the same 64 right-hand sides (lane = column).
// One wave is bound by its instruction issue; the recurrence itself is shorter: row block s (four rows) needs the
// blocks before it, but the 16 multiply-adds that carry x of block s - 1 into a later block do not wait for the
// corners in between.  So the blocks are dealt out in turn (block b belongs to wave b mod 4, which keeps the running
// right-hand side of its four blocks in registers) and the solve runs in 16 phases.  In phase s every wave waits for
// x of block s - 1 and takes it out of its blocks from s on; the owner of block s does that block first, then solves
// its 4 x 4 corner, writes x to LDS (through emit) and publishes the phase.  Every x receives its terms in ascending
// j as in the one-wave form, so the bits are the same; the path per phase is hand-over, 16 multiply-adds, corner.
// Hand-over is a counter in LDS: the owner stores base + s + 1 (release) after its x, the others poll it (acquire).
// A wave's LDS operations complete in order, and a wave in phase s waits only for the phase before, which waits for
// nothing later, so the waits end; they are bounded anyway (`limit` polls, see wait_limit()).  A wave whose wait ran out sets
// *expired (in LDS) and goes on; the caller then overwrites results with NaN: NaNs instead of a hung GPU or of
// plausible wrong numbers, should this code ever be broken.
// D: L_tt, fp32, row-major; R: the tile's right-hand side and Xs: its solution, both [row][column] in LDS;
// emit(r, x_r), called by the owning wave, must write Xs[r][lane]; spare(q) is called by every wave after its q-th
// corner (q = 0 .. 3), when it has time for other work.
template <int LDD, class Emit, class Spare>
__device__ __forceinline__ void solve_tile64_waves(const float (*D)[LDD], const float (*R)[LDD], const float (*Xs)[LDD], int *ready,
                                                   int *expired, int base, int w, int lane, int limit, Emit emit, Spare spare)
{
    const float(*Dw)[LDD] = D + 4 * w;                    // block w + 4 ob of the tile is rows Dw[16 ob .. 16 ob + 3]
    float tt[4][4];                                       // running right-hand side of the wave's blocks: [ob][row in block]
#pragma unroll
    for (int ob = 0; ob < 4; ++ob)
#pragma unroll
        for (int j = 0; j < 4; ++j) tt[ob][j] = R[4 * w + 16 * ob + j][lane];
    // coefficients (they do not depend on x).  What the owner of a block needs on the path, the block's rows in the
    // columns of the block before (own) and its corner (cc), is requested a phase ahead; the rest (cu, the rows of
    // the wave's other blocks in the columns of block s - 1) in the phase itself, where there is time to wait
    f32x4 own[4], ownn[4], cc[4], ccn[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) cc[j] = own[j] = ownn[j] = ccn[j] = *(const f32x4 *)&D[j][0];
    unrolled<NBLK>([&](auto index) __attribute__((always_inline)) {
        constexpr int s = decltype(index)::value, so = s / 4, sw = s % 4;
        if (s + 1 < NBLK && w == (s + 1) % 4) {           // uniform over the wave: the owner of the next block
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                ownn[j] = *(const f32x4 *)&D[4 * (s + 1) + j][4 * s];
                ccn[j] = *(const f32x4 *)&D[4 * (s + 1) + j][4 * (s + 1)];
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        float xv[4] = {0.0f, 0.0f, 0.0f, 0.0f};           // -x of block s - 1
        if (s >= 1) {
            int polls = 0;
            while (__hip_atomic_load(ready, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) < base + s) {
                if (++polls >= limit) {                   // never taken unless this code is broken
                    *expired = 1;
                    break;
                }
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) xv[i] = -Xs[4 * (s - 1) + i][lane];
        }
        auto take_out = [&](float(&t4)[4], const f32x4(&c4)[4]) __attribute__((always_inline)) {   // x of block s - 1 out of a block
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) t4[j] = __builtin_fmaf(c4[j][i], xv[i], t4[j]);
            // the results are next used inside the branch of the wave's own corner, phases later, and the compiler
            // would move all these multiply-adds down into that branch, onto the path everybody waits for: pin them
            asm volatile("" : "+v"(t4[0]), "+v"(t4[1]), "+v"(t4[2]), "+v"(t4[3]));
        };
        if (w == sw) {                                    // the owner of block s
            if (s >= 1) take_out(tt[so], own);
            float xneg[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
#pragma unroll
                for (int e = 0; e < j; ++e) tt[so][j] = __builtin_fmaf(cc[j][e], xneg[e], tt[so][j]);
                const float xr = tt[so][j] / cc[j][j];
                xneg[j] = -xr;
                emit(4 * s + j, xr);
            }
            __hip_atomic_store(ready, base + s + 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
            spare(so);                                    // its next corner is four phases away
        }
        if (s >= 1) {
            // the wave's later blocks: block w + 4 ob for ob > so, and for ob = so if it comes after block s
            f32x4 cu[4][4];
#pragma unroll
            for (int ob = so; ob < 4; ++ob)
#pragma unroll
                for (int j = 0; j < 4; ++j) cu[ob][j] = *(const f32x4 *)&Dw[16 * ob + j][4 * (s - 1)];
            if (w > sw) take_out(tt[so], cu[so]);
#pragma unroll
            for (int ob = so + 1; ob < 4; ++ob) take_out(tt[ob], cu[ob]);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            own[j] = ownn[j];
            cc[j] = ccn[j];
        }
        __builtin_amdgcn_sched_barrier(0);
    });
}

// The panel with the four waves of solve_tile64_waves.  All four work on the same slab of 64 right-hand sides: they
// solve tile t together and share what else a tile needs: wave w stages a quarter of L_tt, multiplies out rows
// 16w .. 16w+15 of the panel's product for the next tile and stores a quarter of the results.  What tile t + 1 needs
// from memory is requested into registers before tile t is solved, and the part of its product that does not
// involve tile t is multiplied out in the spare time of that solve; between two solves remain the last two k-steps,
// the staging of L_tt and the stores (16-byte pieces from LDS).  With the product off the path a panel can be longer
// than in tri_panel_kernel: up to PANELW = 8 tiles (what LDS holds of solved tiles), which saves the smallest GEMM
// launches of the recursion; the loop over tiles is not unrolled.  The sums are the ones of tri_panel_kernel in the
// same order.  Requires, on top of tri_panel_kernel's conditions, nrhs a multiple of 8 and 16-byte aligned X and Xh
// (whole 16-byte pieces of a row are stored or skipped).
constexpr int PANELW = 8;
// everything the solve reads in the first 64 KB of LDS (16-bit offset field from one base register)
struct PanelLds {
    float D[64][64 + 4];               // L_tt in fp32, row-major, on and below the diagonal
    float R[64][64 + 4];               // right-hand side of the tile with the panel's product taken out, [row][column]
    float Xs[64][64 + 4];              // the tile's solution, [row][column]
    uint16_t Xb[PANELW * 64][64];      // solved tiles as bfloat16, [k][column]
    int ready;                         // hand-over counter of solve_tile64_waves
    int expired;                       // set by a wave of solve_tile64_waves whose bounded wait ran out
};
__device__ __forceinline__ void panel_by_substitution(PanelLds &lds, const uint16_t *__restrict__ L, int64_t n, const float *Rin,
                                                      float *X, uint16_t *__restrict__ Xh, int64_t nrhs, int64_t r0, int tiles, int limit)
{
    constexpr int NB = 64, LDD = NB + 4, NT = 256, NKS = 2 * PANELW - 2;
    int tid = threadIdx.x, lane = tid & 63, lq = lane & 15, g = lane >> 4;                // (not const: see the loop over tiles)
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t c0 = (int64_t)(blockIdx.x >> 1) * 64;             // (two workgroups per slab, see tri_panelw_kernel)
    constexpr int cpr = NB / 8, PP = NB * cpr / NT;                    // 16-byte pieces of L_tt per thread

    uint4 piece[PP];
    float rhs[4][4];                                                   // rows 16w + 4g + r, columns 16j + lq: [j][r]
    i32x4 a[NKS];                                                      // row 16w + lq of L[u, 0:u], k = 32 ks + 8 g .. +7
    auto request = [&](int u) __attribute__((always_inline)) {         // what tile u needs from memory
        const int64_t ru = r0 + (int64_t)u * NB;
#pragma unroll
        for (int p = 0; p < PP; ++p) {
            const int id = tid + NT * p, r = id / cpr, jc = id % cpr;
            piece[p] = make_uint4(0, 0, 0, 0);
            if (jc * 8 <= r) piece[p] = *(const uint4 *)(L + (ru + r) * n + ru + jc * 8);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t col = c0 + 16 * j + lq < nrhs ? c0 + 16 * j + lq : nrhs - 1;   // columns past the last one shadow it
#pragma unroll
            for (int r = 0; r < 4; ++r) rhs[j][r] = Rin[(ru + 16 * w + 4 * g + r) * nrhs + col];
        }
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks)
            if (ks < 2 * u) a[ks] = *(const i32x4 *)(L + (ru + 16 * w + lq) * n + r0 + ks * 32 + g * 8);      // uniform condition
    };
    f32x4 acc[4];                                                      // the wave's rows of the panel's product for the next tile
    auto k_step = [&](int ks) __attribute__((always_inline)) {         // one MFMA k-step of 32 of that product
        i32x4 b[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            CYC_LDS char *p = (CYC_LDS char *)&lds.Xb[ks * 32 + 8 * g + (lq >> 2)][j * 16 + 4 * (lq & 3)];
            const i32x2 lo = __builtin_bit_cast(i32x2, __builtin_amdgcn_ds_read_tr16_b64_v4bf16((CYC_LDS bf16x4 *)p));
            const i32x2 hi = __builtin_bit_cast(i32x2, __builtin_amdgcn_ds_read_tr16_b64_v4bf16((CYC_LDS bf16x4 *)(p + 4 * 64 * 2)));
            b[j] = (i32x4){lo[0], lo[1], hi[0], hi[1]};
        }
#pragma unroll
        for (int j = 0; j < 4; ++j)
            acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a[ks]), __builtin_bit_cast(bf16x8, b[j]), acc[j], 0, 0, 0);
    };
    // tile u into LDS: L_uu, and R = rhs - product, the k-steps before first_ks being in acc already
    auto stage = [&](int u, int first_ks) __attribute__((always_inline)) {
#pragma unroll
        for (int p = 0; p < PP; ++p) {
            const int id = tid + NT * p, r = id / cpr, jc = id % cpr;
            if (jc * 8 <= r) {
                const uint32_t v[4] = {piece[p].x, piece[p].y, piece[p].z, piece[p].w};
                f32x4 lo, hi;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    lo[e] = widen_bf16((uint16_t)(v[e >> 1] >> (16 * (e & 1))));
                    hi[e] = widen_bf16((uint16_t)(v[2 + (e >> 1)] >> (16 * (e & 1))));
                }
                *(f32x4 *)&lds.D[r][jc * 8] = lo;
                *(f32x4 *)&lds.D[r][jc * 8 + 4] = hi;
            }
        }
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks)
            if (ks >= first_ks && ks < 2 * u) k_step(ks);              // uniform condition
        // accumulator register r of lane l is row 4 (l/16) + r, column l%16 of its 16 x 16 tile
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) lds.R[16 * w + 4 * g + r][16 * j + lq] = rhs[j][r] - acc[j][r];
    };
    auto store = [&](int v) __attribute__((always_inline)) {           // results of tile v: 16-byte pieces from LDS to X and Xh
        const int64_t rv = r0 + (int64_t)v * NB;
#pragma unroll
        for (int p = 0; p < NB * 16 / NT; ++p) {
            const int id = tid + NT * p, r = id >> 4, ch = id & 15;
            if (c0 + 4 * ch < nrhs) *(f32x4 *)(X + (rv + r) * nrhs + c0 + 4 * ch) = *(const f32x4 *)&lds.Xs[r][4 * ch];
        }
#pragma unroll
        for (int p = 0; p < NB * 8 / NT; ++p) {
            const int id = tid + NT * p, r = id >> 3, ch = id & 7;
            if (c0 + 8 * ch < nrhs) *(uint4 *)(Xh + (rv + r) * nrhs + c0 + 8 * ch) = *(const uint4 *)&lds.Xb[v * NB + r][8 * ch];
        }
    };

    if (tid == 0) lds.ready = lds.expired = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[j] = (f32x4){0, 0, 0, 0};
    request(0);
    stage(0, 0);
    __syncthreads();
#pragma unroll 1
    for (int t = 0; t < tiles; ++t) {                                  // (not unrolled: t only moves LDS addresses and bounds uniform branches)
        // the thread index is made opaque once per tile: otherwise the hundreds of LDS and memory addresses derived
        // from it are all computed ahead of the loop and kept in registers across it, and the kernel spills
        asm volatile("" : "+v"(tid));
        lane = tid & 63;
        lq = lane & 15;
        g = lane >> 4;
        if (t + 1 < tiles) request(t + 1);                             // lands during the solve
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[j] = (f32x4){0, 0, 0, 0};
        solve_tile64_waves<LDD>(
            lds.D, lds.R, lds.Xs, &lds.ready, &lds.expired, t * NBLK, w, lane, limit,
            [&](int r, float xr) __attribute__((always_inline)) {
                lds.Xb[t * NB + r][lane] = round_bf16(xr);
                lds.Xs[r][lane] = xr;
            },
            // after its second, third and fourth corner a wave multiplies out four k-steps each of the next tile's
            // product over the tiles solved before this one (by then the rows of L requested above have arrived)
            [&](int q) __attribute__((always_inline)) {
                if (q >= 1 && t + 1 < tiles) {
#pragma unroll
                    for (int ks = 0; ks < NKS; ++ks)
                        if (ks / 4 == q - 1 && ks < 2 * t) k_step(ks);
                }
            });
        __syncthreads();                                               // tile t is solved: D and R are free, Xs and Xb complete
        store(t);
        if (t + 1 < tiles) stage(t + 1, 2 * t);
        __syncthreads();                                               // tile t + 1 is staged, Xs is free
    }
    if (__builtin_expect(lds.expired != 0, 0)) {
        // (uniform; checked once, after everything, so that the solves pay nothing for it) a hand-over between waves
        // failed somewhere in this panel: its last tile is overwritten with NaN, which every later row of the solve
        // inherits and any check of the result sees
        const int64_t rv = r0 + (int64_t)(tiles - 1) * NB;
        if (c0 + lane < nrhs)
            for (int r = w * 16; r < w * 16 + 16; ++r) {
                X[(rv + r) * nrhs + c0 + lane] = __builtin_nanf("");
                Xh[(rv + r) * nrhs + c0 + lane] = 0x7fc0;
            }
    }
}

// ---- Diagonal tiles through their inverses.
// X_t = TRSM(L_tt, R_t) is a chain of 64 dependent rows per tile and 128 tiles follow one another at n = 8192; the
// tile operation itself is left open by the paper (a library call there).  The inverses of the diagonal tiles depend
// on L alone, so all of them are computed ahead, side by side (tri_inverse_kernel: the substitution above with the
// identity as right-hand side), and a tile's solve becomes the product X_t = L_tt^-1 R_t on the matrix cores in fp32
// (v_mfma_f32_16x16x4_f32: fp32 operands, fp32 sums), which has no chain.  The product is as good as the substitution
// only for a well-conditioned tile: with kappa = || |L_tt^-1| |L_tt| || its error bound is (kappa^2 + kappa) where the
// substitution's is kappa.  tri_inverse_kernel therefore leaves a verdict per tile, ||L_tt^-1||_1 ||L_tt||_1 <= 8
// (an upper bound of kappa taken in the 1-norm, which costs a column sum per lane), and a panel whose tiles do not all pass takes the
// substitution as before.  Both are deterministic; which one runs depends on L alone.
constexpr int INV_FLOATS = 64 * 64;        // one inverse in the workspace, in the order described at tri_inverse_kernel
// The tiles of L that a panel's own product multiplies (tile (T, S), 0 < T - S < PANEL_BAND + 1) are kept a second time in
// the order in which that product wants them as stationary MFMA operands: eight pieces of 1 KiB per tile, piece
// 2 w + h: lane l holds the 16 bytes L[64 T + 16 w + l%16][64 S + 32 h + 8 (l/16) .. +7].  Read from L itself such a
// fragment is 64 separate cache lines per load; from here it is one contiguous KiB.
constexpr int PANEL_BAND = 7, PACK_PIECES = 8, PACK_BYTES_PER_TILE_ROW = PANEL_BAND * PACK_PIECES * 1024;
constexpr float INV_NORM_LIMIT = 8.0f;

// One wave per full diagonal tile: lane j solves L_tt y = e_j.  Entry (r, j) of the inverse is stored where the panel
// kernel's MFMA wants it as its A operand.  Which k a slot of that MFMA stands for is free as long as both operands
// agree; slot l/16 of k-step ks is k = 16 (ks / 4) + 4 (l / 16) + ks % 4, so that the four rows of R which a k-step
// reads as the other operand lie four rows apart, on disjoint LDS banks.  Operand lane (r % 16) + 16 (j / 4 % 4) thus
// holds entry (r, j) for row block rb = r / 16 and k-step ks = 4 (j / 16) + j % 4.  A tile is 16 pieces of 1 KiB, piece
// 4 rb + ks / 4 holding the four k-steps ks / 4 * 4 .. + 3 of all 64 operand lanes ([lane][ks % 4]), so that a wave
// fetches a piece with one fully coalesced 16-byte load per lane.
__global__ __launch_bounds__(64) void tri_inverse_kernel(const uint16_t *__restrict__ L, int64_t n, float *__restrict__ Winv,
                                                         int *__restrict__ ok, char *__restrict__ packed, int full)
{
    constexpr int NB = 64, LDD = NB + 4, cpr = NB / 8, PER_LANE = NB * NB / 8 / 64;
    if ((int)blockIdx.x >= full) {
        // the workgroups behind the `full` that invert: one piece each of the operand-order copy (see PANEL_BAND)
        const int id = (int)blockIdx.x - full, T = id / (PANEL_BAND * PACK_PIECES), rest = id % (PANEL_BAND * PACK_PIECES);
        const int S = T - 1 - rest / PACK_PIECES, piece = rest % PACK_PIECES, l = threadIdx.x;
        if (S >= 0)
            *(uint4 *)(packed + ((int64_t)id * 64 + l) * 16) =
                *(const uint4 *)(L + ((int64_t)T * 64 + 16 * (piece >> 1) + (l & 15)) * n + (int64_t)S * 64 + 32 * (piece & 1) + 8 * (l >> 4));
        return;
    }
    __shared__ __attribute__((aligned(16))) float D[NB][LDD];
    __shared__ float norms[2][64];
    const int lane = threadIdx.x;
    const int64_t rt = (int64_t)blockIdx.x * NB;
#pragma unroll
    for (int x = 0; x < PER_LANE; ++x) {                         // the 16-byte pieces on and below the diagonal, widened
        const int id = lane + 64 * x, r = id / cpr, jc = id % cpr;
        if (jc * 8 <= r) {
            const uint4 piece = *(const uint4 *)(L + (rt + r) * n + rt + jc * 8);
            const uint32_t v[4] = {piece.x, piece.y, piece.z, piece.w};
            f32x4 lo, hi;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                lo[e] = widen_bf16((uint16_t)(v[e >> 1] >> (16 * (e & 1))));
                hi[e] = widen_bf16((uint16_t)(v[2 + (e >> 1)] >> (16 * (e & 1))));
            }
            *(f32x4 *)&D[r][jc * 8] = lo;
            *(f32x4 *)&D[r][jc * 8 + 4] = hi;
        }
    }
    __syncthreads();
    float colsum_L = 0.0f;                                       // column `lane` of |L_tt|, on and below the diagonal
    for (int i = 0; i < NB; ++i) colsum_L += i >= lane ? __builtin_fabsf(D[i][lane]) : 0.0f;
    float x[NB], xn[NB];
#pragma unroll
    for (int r = 0; r < NB; ++r) x[r] = r == lane ? 1.0f : 0.0f;
    float colsum_inv = 0.0f;
    float *out = Winv + (int64_t)blockIdx.x * INV_FLOATS + (lane >> 4) * 256 + ((lane >> 2) & 3) * 64 + (lane & 3);
    solve_tile64<LDD>(
        D, x, xn,
        [&](int r, float y) __attribute__((always_inline)) {
            out[(r >> 4) * 1024 + (r & 15) * 4] = y;              // rows above the lane's own come out as exact zeros
            colsum_inv += __builtin_fabsf(y);
        },
        []() __attribute__((always_inline)) {});
    norms[0][lane] = colsum_L;
    norms[1][lane] = colsum_inv;
    __syncthreads();
    if (lane == 0) {
        float a = 0.0f, b = 0.0f;
        bool finite = true;
        for (int j = 0; j < 64; ++j) {
            a = __builtin_fmaxf(a, norms[0][j]);
            b = __builtin_fmaxf(b, norms[1][j]);
            finite = finite && norms[0][j] == norms[0][j] && norms[1][j] == norms[1][j];   // fmax drops a NaN
        }
        ok[blockIdx.x] = finite && a * b <= INV_NORM_LIMIT ? 1 : 0;
    }
}

// The panel of tri_panelw_kernel with the diagonal solves as products with the inverses, for 32 right-hand sides (two
// column blocks of 16).  In the panel's product for the next tile wave w multiplies out rows 16w .. 16w+15 of both
// column blocks; in the solve it takes one column block and two of the four row blocks of 16 (see NC below): the
// inverse is lower triangular, so row block rb needs the k-steps 0 .. 4 rb + 3 only, and the streamed operand (R,
// [row][column] in LDS) is one LDS read per k-step.
// Memory traffic is arranged around one wait per tile.  On this chip loads and stores share one counter and complete
// out of order with respect to each other, so while both are outstanding the only wait the compiler can insert is
// the wait for all of them.  What a tile issues to memory -- the stores of the previous tile's results, the loads of
// the next tile's inverse and of the right-hand side and rows of L of the tile after that -- is never waited for
// inside that tile: what was loaded is first touched (an empty asm statement that names the registers) at the top of
// the tile in which it is used, a whole tile later, when it has arrived.  Hence two register sets for everything
// loaded, and two tiles per loop trip so that the sets are named statically.
// Placement of the solved tiles in panel_by_inverses: row k of Xb (128 bytes: eight 16-byte chunks of eight columns) keeps
// its chunk q in slot q ^ xb_swizzle(k).  One transposing read takes 8 bytes per lane from the rows 8 (l/16) + 0 .. 3 of a
// k-step, two adjacent chunks of each: unswizzled those are sixteen rows whose chunks lie on the same 16 of the 64 banks
// (a row is half the banks wide, rows two apart coincide), an eight-way conflict; the swizzle moves each group of eight
// rows to banks of its own, which leaves the two-way conflict that 512 bytes per instruction cannot avoid.
__device__ __forceinline__ constexpr int xb_swizzle(int k) { return ((k >> 3) & 3) << 1; }

__device__ __forceinline__ void panel_by_inverses(PanelLds &lds, const uint16_t *__restrict__ L, int64_t n, const float *Rin,
                                                  float *X, uint16_t *__restrict__ Xh, int64_t nrhs, int64_t r0, int tiles,
                                                  const float *__restrict__ Winv, int64_t c0, const char *__restrict__ packed)
{
    // NC: column blocks of 16 per workgroup.  Two (32 right-hand sides), so that a launch has a workgroup for every compute
    // unit and a wave half the work per tile: in the panel's product wave w has rows 16w .. of both column blocks; in the
    // solve it has one column block (w % 2) and two of the four row blocks (w / 2: blocks 0 and 3, or 1 and 2, five 16 x 16
    // blocks of the triangular inverse either way).
    constexpr int NB = 64, NT = 256, NKS = 2 * PANELW - 2, NC = 2;
    int tid = threadIdx.x, lane = tid & 63, lq = lane & 15, g = lane >> 4;                // (not const: see the loop over tiles)
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int sc = w & 1, rbA = w >> 1 ? 1 : 0, rbB = w >> 1 ? 2 : 3;                    // the solve's column block and row blocks
    struct Operands {
        f32x4 rhs[NC];                                                 // rows 16w + 4g + r, columns 16j + lq: [j][r]
        i32x4 a[NKS];                                                  // row 16w + lq of L[u, 0:u], k = 32 ks + 8 g .. +7
    };
    Operands op0, op1;
    // this lane's values of an inverse: row block rbA, column blocks 0 and 1; row block rbB, column blocks 0 .. 3 (the
    // pieces above the block diagonal are stored as zeros: both halves run the same instructions)
    f32x4 inv0[6], inv1[6];

    // What tile u needs from memory, as a list of single loads (so that they can be dealt out between the MFMAs of a
    // solve): items 0 .. 4 NC - 1 its right-hand side, then NKS items for its rows of L (those of the k-steps it has)
    constexpr int REQUEST_ITEMS = 4 * NC + NKS, INVERSE_ITEMS = 6;
    // Every address is a wave-uniform base plus a 32-bit byte offset of the lane (n < 2^26, nrhs < 2^24, see
    // inverses_wanted): the loads then take their base from scalar registers and cost no vector instruction, where 64-bit
    // address arithmetic per lane took ten per load, more than the 32 cycles of the MFMA each load sits behind.
    uint32_t off_rhs[NC];
    auto lane_offsets = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < NC; ++j) {
            const int64_t col = c0 + 16 * j + lq < nrhs ? c0 + 16 * j + lq : nrhs - 1;   // columns past the last one shadow it
            off_rhs[j] = (uint32_t)((int64_t)(4 * g) * nrhs + col) * 4u;
        }
    };
    lane_offsets();
    // (rows: the wave's first row of tile u's right-hand side, row r0 + 64 u + 16 w.  In the unrolled tiles it is a running
    // pointer: multiplied out per row from the tile number, each load took a dozen scalar instructions of address arithmetic)
    const int64_t row_bytes = nrhs * 4;
    auto rhs_rows_of = [&](int u) __attribute__((always_inline)) { return (const char *)(Rin + (r0 + (int64_t)u * NB + 16 * w) * nrhs); };
    const char *later_rows = rhs_rows_of(2);                           // (of tile t + 2 while tile t runs, in the unrolled tiles)
    auto request_item = [&](int u, Operands &o, int i, const char *rows) __attribute__((always_inline)) {
        if (i < 4 * NC) {
            const int j = i >> 2, r = i & 3;
            o.rhs[j][r] = *(const float *)(rows + r * row_bytes + off_rhs[j]);
        } else {
            const int ks = i - 4 * NC;
            // (tile (T, S) = (r0 / 64 + u, r0 / 64 + ks / 2), piece 2 w + ks % 2 of the operand-order copy)
            if (ks < 2 * u)                                                                                             // uniform condition
                o.a[ks] = *(const i32x4 *)(packed + ((((r0 >> 6) + u) * PANEL_BAND + (u - 1 - ks / 2)) * PACK_PIECES + 2 * w + (ks & 1)) * 1024 +
                                          (uint32_t)lane * 16u);
        }
    };
    auto request = [&](int u, Operands &o) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < REQUEST_ITEMS; ++i) request_item(u, o, i, rhs_rows_of(u));
    };
    // the wave's pieces of an inverse: item p < 2 is piece (rbA, p), item p >= 2 piece (rbB, p - 2)
    auto request_inverse_item = [&](int u, f32x4(&iv)[6], int p) __attribute__((always_inline)) {
        const int rb = p < 2 ? rbA : rbB, q = p < 2 ? p : p - 2;
        iv[p] = *(const f32x4 *)((const char *)(Winv + (int64_t)u * INV_FLOATS + (rb * 4 + q) * 256) + (uint32_t)lane * 16u);
    };
    auto request_inverse = [&](int u, f32x4(&iv)[6]) __attribute__((always_inline)) {
#pragma unroll
        for (int p = 0; p < INVERSE_ITEMS; ++p) request_inverse_item(u, iv, p);
    };
    // what was loaded a tile ago is waited for here and nowhere else
    auto touch = [&](f32x4(&iv)[6], Operands &o) __attribute__((always_inline)) {
        asm volatile("" : "+v"(iv[0]), "+v"(iv[1]), "+v"(iv[2]), "+v"(iv[3]), "+v"(iv[4]), "+v"(iv[5]), "+v"(o.rhs[0]), "+v"(o.rhs[1])
                     :: "memory");
        asm volatile("" : "+v"(o.a[0]), "+v"(o.a[1]), "+v"(o.a[2]), "+v"(o.a[3]), "+v"(o.a[4]), "+v"(o.a[5]), "+v"(o.a[6]),
                          "+v"(o.a[7]), "+v"(o.a[8]), "+v"(o.a[9]), "+v"(o.a[10]), "+v"(o.a[11]), "+v"(o.a[12]), "+v"(o.a[13])
                     :: "memory");
    };
    static_assert(NKS == 14 && NC == 2, "touch names every register of Operands");
    // The panel's product for tile u (its rows of L times the tiles solved before it) in two parts: the k-steps over
    // the tiles before u - 1 are multiplied out ahead, beside the solve of tile u - 1 (early), the two k-steps over
    // tile u - 1 after it (late), and R = right-hand side - product goes to LDS.  The bounds are constants in every
    // copy (the switches below when the tile number is not one), so that each part is straight-line code in which the
    // streamed operand of a k-step is read two k-steps ahead of its MFMAs.
    f32x4 acc[NC];
    auto k_range = [&](auto first, auto last, const Operands &o, auto beside) __attribute__((always_inline)) {
        constexpr int FIRST = decltype(first)::value, LAST = decltype(last)::value;
        i32x4 b[3][NC];
        auto read_b = [&](int ks, i32x4(&dst)[NC]) __attribute__((always_inline)) {
#pragma unroll
            for (int j = 0; j < NC; ++j) {
                // (rows 32 ks + 8 g + 0 .. 7 share the swizzle 2 g, see xb_swizzle)
                const int chunk = (2 * j + ((lq >> 1) & 1)) ^ (2 * g);
                CYC_LDS char *p = (CYC_LDS char *)&lds.Xb[ks * 32 + 8 * g + (lq >> 2)][0] + 16 * chunk + 8 * (lq & 1);
                const i32x2 lo = __builtin_bit_cast(i32x2, __builtin_amdgcn_ds_read_tr16_b64_v4bf16((CYC_LDS bf16x4 *)p));
                const i32x2 hi = __builtin_bit_cast(i32x2, __builtin_amdgcn_ds_read_tr16_b64_v4bf16((CYC_LDS bf16x4 *)(p + 4 * 64 * 2)));
                dst[j] = (i32x4){lo[0], lo[1], hi[0], hi[1]};
            }
        };
        if (FIRST < LAST) read_b(FIRST, b[FIRST % 3]);
        if (FIRST + 1 < LAST) read_b(FIRST + 1, b[(FIRST + 1) % 3]);
#pragma unroll
        for (int ks = FIRST; ks < LAST; ++ks) {
            if (ks + 2 < LAST) read_b(ks + 2, b[(ks + 2) % 3]);
#pragma unroll
            for (int j = 0; j < NC; ++j)
                acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, o.a[ks]), __builtin_bit_cast(bf16x8, b[ks % 3][j]), acc[j], 0, 0, 0);
            beside(ks - FIRST);
        }
    };
    auto early_of = [&](auto tile_c, const Operands &o, auto beside) __attribute__((always_inline)) {
        constexpr int U = decltype(tile_c)::value;
#pragma unroll
        for (int j = 0; j < NC; ++j) acc[j] = (f32x4){0, 0, 0, 0};
        k_range(std::integral_constant<int, 0>{}, std::integral_constant<int, U >= 1 ? 2 * U - 2 : 0>{}, o, beside);
    };
    auto late_of = [&](auto tile_c, const Operands &o, auto beside) __attribute__((always_inline)) {
        constexpr int U = decltype(tile_c)::value;
        k_range(std::integral_constant<int, U >= 1 ? 2 * U - 2 : 0>{}, std::integral_constant<int, 2 * U>{}, o, beside);
#pragma unroll
        for (int j = 0; j < NC; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) lds.R[16 * w + 4 * g + r][16 * j + lq] = o.rhs[j][r] - acc[j][r];
    };
    // (u is uniform and at most PANELW - 1; when the caller's tile number is a constant the switch folds away)
    auto stage_early = [&](int u, const Operands &o, auto beside) __attribute__((always_inline)) {
        switch (u) {
            case 0: early_of(std::integral_constant<int, 0>{}, o, beside); break;
            case 1: early_of(std::integral_constant<int, 1>{}, o, beside); break;
            case 2: early_of(std::integral_constant<int, 2>{}, o, beside); break;
            case 3: early_of(std::integral_constant<int, 3>{}, o, beside); break;
            case 4: early_of(std::integral_constant<int, 4>{}, o, beside); break;
            case 5: early_of(std::integral_constant<int, 5>{}, o, beside); break;
            case 6: early_of(std::integral_constant<int, 6>{}, o, beside); break;
            default: early_of(std::integral_constant<int, PANELW - 1>{}, o, beside); break;
        }
    };
    auto stage_late = [&](int u, const Operands &o, auto beside) __attribute__((always_inline)) {
        switch (u) {
            case 0: late_of(std::integral_constant<int, 0>{}, o, beside); break;
            case 1: late_of(std::integral_constant<int, 1>{}, o, beside); break;
            case 2: late_of(std::integral_constant<int, 2>{}, o, beside); break;
            case 3: late_of(std::integral_constant<int, 3>{}, o, beside); break;
            case 4: late_of(std::integral_constant<int, 4>{}, o, beside); break;
            case 5: late_of(std::integral_constant<int, 5>{}, o, beside); break;
            case 6: late_of(std::integral_constant<int, 6>{}, o, beside); break;
            default: late_of(std::integral_constant<int, PANELW - 1>{}, o, beside); break;
        }
    };
    // results of tile v: 16-byte pieces from LDS (Xs: the buffer of v's parity) to X and Xh
    // (in two steps, so that the reads of LDS and the stores can be placed apart)
    constexpr int X_PIECES = NB * 4 * NC / NT;
    struct Results {
        f32x4 x[X_PIECES];
        uint4 xh;
    };
    auto fetch_results = [&](int v, const float(*Xs)[NB + 4], Results &res) __attribute__((always_inline)) {
#pragma unroll
        for (int p = 0; p < X_PIECES; ++p) {
            const int id = tid + NT * p, r = id / (4 * NC), ch = id % (4 * NC);
            res.x[p] = *(const f32x4 *)&Xs[r][4 * ch];
        }
        static_assert(NB * 2 * NC == NT, "one 16-byte piece of Xh per thread");
        const int r = tid / (2 * NC), ch = tid % (2 * NC);
        res.xh = *(const uint4 *)&lds.Xb[v * NB + r][8 * (ch ^ xb_swizzle(r))];
    };
    // (the thread's place in a tile of X and of Xh as 32-bit offsets from a uniform base, worked out once: nrhs < 2^24)
    static_assert(4 * NC == 8 && NT / (4 * NC) == 32, "piece p of X: row tid / 8 + 32 p, columns 4 (tid % 8) ..");
    const uint32_t put_x = (((uint32_t)threadIdx.x >> 3) * (uint32_t)nrhs + 4 * (threadIdx.x & 7)) * 4u;
    const uint32_t put_xh = (((uint32_t)threadIdx.x >> 2) * (uint32_t)nrhs + 8 * (threadIdx.x & 3)) * 2u;
    const bool put_x_ok = c0 + 4 * (threadIdx.x & 7) < nrhs, put_xh_ok = c0 + 8 * (threadIdx.x & 3) < nrhs;
    auto put_results = [&](int v, const Results &res) __attribute__((always_inline)) {
        const int64_t rv = r0 + (int64_t)v * NB;
#pragma unroll
        for (int p = 0; p < X_PIECES; ++p)
            if (put_x_ok) *(f32x4 *)((char *)(X + (rv + 32 * p) * nrhs + c0) + put_x) = res.x[p];
        if (put_xh_ok) *(uint4 *)((char *)(Xh + rv * nrhs + c0) + put_xh) = res.xh;
    };
    auto store = [&](int v, const float(*Xs)[NB + 4]) __attribute__((always_inline)) {
        Results res;
        fetch_results(v, Xs, res);
        put_results(v, res);
    };
    // X_t = L_tt^-1 R_t for the wave's 16 columns (block sc) and its two row blocks.  A operand lane l: row 16 rb + l%16,
    // k = k(ks, l/16) as laid down at tri_inverse_kernel; B operand: the same k, column l%16; accumulator register r: row
    // 16 rb + 4 (l/16) + r, column l%16.  Row block rbA takes the k-steps over column blocks 0 and 1 of the inverse, rbB
    // over all four: 24 MFMAs, of which four multiply a zero block (rbA = 0: its column block 1; rbB = 2: its column block
    // 3), so that both halves of the workgroup run the same code.
    // beside(i) is called after the i-th of the 24 MFMAs and pinned there: an MFMA occupies the matrix pipe for 32
    // cycles, and what the wave issues meanwhile (the loads of later tiles) costs the solve nothing.
    constexpr int SOLVE_MFMAS = 24;
    auto solve = [&](int t, const f32x4(&iv)[6], float(*Xs)[NB + 4], auto beside) __attribute__((always_inline)) {
        float b[16];
#pragma unroll
        for (int ks = 0; ks < 16; ++ks) b[ks] = lds.R[16 * (ks >> 2) + 4 * g + (ks & 3)][16 * sc + lq];
        f32x4 xa = {0, 0, 0, 0}, xb = {0, 0, 0, 0};
        int issued = 0;
#pragma unroll
        for (int ks = 0; ks < 16; ++ks) {
            if (ks < 8) {
                xa = __builtin_amdgcn_mfma_f32_16x16x4f32(iv[ks / 4][ks % 4], b[ks], xa, 0, 0, 0);
                beside(issued++);
            }
            xb = __builtin_amdgcn_mfma_f32_16x16x4f32(iv[2 + ks / 4][ks % 4], b[ks], xb, 0, 0, 0);
            beside(issued++);
        }
#pragma unroll
        for (int half = 0; half < 2; ++half)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int row = 16 * (half ? rbB : rbA) + 4 * g + r;
                const float v = half ? xb[r] : xa[r];
                Xs[row][16 * sc + lq] = v;
                lds.Xb[t * NB + row][8 * ((2 * sc + (lq >> 3)) ^ xb_swizzle(row)) + (lq & 7)] = round_bf16(v);
            }
    };
    // Tile t of `count`.  `mine` holds its inverse and `next` the operands of tile t + 1's product; `other` takes the
    // inverse of tile t + 1 and `later` the operands of tile t + 2.  The results stay in LDS (lds.Xs for even t, lds.D,
    // which nothing else uses here, for odd t) and are stored at the top of the next tile.
    // `dealt`: t and count are constants here, so the loads can be dealt out between the MFMAs of the solve
    auto tile = [&](int t, int count, bool dealt, f32x4(&mine)[6], f32x4(&other)[6], Operands &next, Operands &later, float(*Xs)[NB + 4],
                    const float(*Xs_before)[NB + 4]) __attribute__((always_inline)) {
        // the thread index is made opaque once per tile (see panel_by_substitution)
        asm volatile("" : "+v"(tid));
        lane = tid & 63;
        lq = lane & 15;
        g = lane >> 4;
        lane_offsets();
        touch(mine, next);
        if (t > 0 && !dealt) store(t - 1, Xs_before);
        if (!dealt) {
            if (t + 1 < count) request_inverse(t + 1, other);
            if (t + 2 < count) request(t + 2, later);
        }
        // `dealt`: the loads of later tiles (item e: 0 .. 5 the inverse of tile t + 1; then tile t + 2's right-hand side, 8
        // items, and its rows of L, item 14 + ks for k-step ks) are spread over the whole tile, one behind a k-step's or a
        // solve step's MFMAs and pinned there: the memory pipeline of the compute unit takes 16 cycles per KiB, and a wave
        // that issues loads faster than that stalls in front of whatever comes next.  Rows of L: the first 2 t behind the
        // k-steps of the product ahead, the last four (k-steps 2 t .. 2 t + 3) behind the two late k-steps; the inverse and
        // the right-hand side behind the first 14 MFMAs of the solve.
        auto load_item = [&](int e) __attribute__((always_inline)) {
            if (e < INVERSE_ITEMS) {
                if (t + 1 < count) request_inverse_item(t + 1, other, e);
            } else if (t + 2 < count && e < INVERSE_ITEMS + REQUEST_ITEMS) {
                request_item(t + 2, later, e - INVERSE_ITEMS, later_rows);
            }
        };
        constexpr int L_ITEMS_FROM = INVERSE_ITEMS + 4 * NC;
        static_assert(L_ITEMS_FROM <= SOLVE_MFMAS, "the inverse and the right-hand side fit behind the MFMAs of the solve");
        auto nothing = [](int) __attribute__((always_inline)) {};
        if (t + 1 < count) {
            if (dealt)
                stage_early(t + 1, next, [&](int i) __attribute__((always_inline)) {
                    load_item(L_ITEMS_FROM + i);
                    __builtin_amdgcn_sched_barrier(0);
                });
            else
                stage_early(t + 1, next, nothing);
        }
        // the previous tile's results go to memory from behind the solve's later MFMAs: read from LDS at one, stored at
        // another (nothing writes that tile's buffers before the next barrier)
        constexpr int FETCH_AT = L_ITEMS_FROM + 1, PUT_AT = FETCH_AT + 5;
        static_assert(PUT_AT < SOLVE_MFMAS, "the stores have an MFMA to sit behind");
        Results before;
        solve(t, mine, Xs, [&](int i) __attribute__((always_inline)) {
            if (!dealt) return;
            if (i < L_ITEMS_FROM) load_item(i);
            if (i == FETCH_AT && t > 0) fetch_results(t - 1, Xs_before, before);
            if (i == PUT_AT && t > 0) put_results(t - 1, before);
            __builtin_amdgcn_sched_barrier(0);
        });
        __syncthreads();                                               // tile t is solved: R is free, Xs and Xb complete
        if (t + 1 < count) {
            if (dealt)
                stage_late(t + 1, next, [&](int i) __attribute__((always_inline)) {
                    load_item(L_ITEMS_FROM + 2 * t + 2 * i);
                    load_item(L_ITEMS_FROM + 2 * t + 2 * i + 1);
                    __builtin_amdgcn_sched_barrier(0);
                });
            else
                stage_late(t + 1, next, nothing);
        }
        __syncthreads();                                               // tile t + 1 is staged
        if (dealt) {
            later_rows += NB * row_bytes;
            asm volatile("" : "+s"(later_rows));                       // (stays a running pointer)
        }
    };

    request(0, op0);
    request_inverse(0, inv0);
    if (tiles > 1) request(1, op1);
    // Every workgroup reads the same inverses and the same tiles of L, all of them at about the same time: whichever
    // asks first for a line that the cache of its part of the chip (32 compute units, workgroup numbers congruent modulo
    // 8) does not hold yet waits for memory, and so do all the others.  So the workgroups of such a part fetch the panel's
    // inverses and operand-order tiles once at the start, 4 KiB pieces dealt out among them; the values are not used.
    constexpr int WARM = 3;
    i32x4 warm[WARM];
    {
        const int parts = 8, sharers = ((int)gridDim.x + parts - 1) / parts, me = (int)blockIdx.x / parts;
        const int n_inv = 4 * tiles, n_all = n_inv + tiles * (tiles - 1);          // tile u of the panel: 2 u pieces of L
#pragma unroll
        for (int i = 0; i < WARM; ++i) {
            int c = me + i * sharers;                                              // uniform
            const char *src = (const char *)Winv;
            if (c < n_inv) {
                src += (int64_t)c * 4096;
            } else if (c < n_all) {
                int d = c - n_inv, u = 1;
                while (d >= 2 * u) { d -= 2 * u; ++u; }
                src = packed + (((r0 >> 6) + u) * PANEL_BAND * PACK_PIECES) * 1024 + (int64_t)d * 4096;
            }
            warm[i] = *(const i32x4 *)(src + (uint32_t)tid * 16u);
        }
    }
    stage_early(0, op0, [](int) {});
    stage_late(0, op0, [](int) {});
    __syncthreads();
    if (tiles == PANELW) {
        // the usual case, every tile number a constant: each tile is straight-line code between its barriers
        unrolled<PANELW / 2>([&](auto half) __attribute__((always_inline)) {
            constexpr int t = 2 * decltype(half)::value;
            tile(t, PANELW, true, inv0, inv1, op1, op0, lds.Xs, lds.D);
            tile(t + 1, PANELW, true, inv1, inv0, op0, op1, lds.D, lds.Xs);
        });
    } else {
#pragma unroll 1
        for (int t = 0; t < tiles; t += 2) {
            tile(t, tiles, false, inv0, inv1, op1, op0, lds.Xs, lds.D);
            if (t + 1 < tiles) tile(t + 1, tiles, false, inv1, inv0, op0, op1, lds.D, lds.Xs);
        }
    }
    store(tiles - 1, (tiles - 1) & 1 ? lds.D : lds.Xs);
    asm volatile("" :: "v"(warm[0]), "v"(warm[1]), "v"(warm[2]));
    static_assert(WARM == 3, "every register of warm is named above");
}

// The four-wave panel: through the inverses when every tile of the panel passed tri_inverse_kernel's check (Winv and ok
// start at the panel's first tile; Winv == nullptr: no inverses were computed), by substitution otherwise.
__global__ __launch_bounds__(256) void tri_panelw_kernel(const uint16_t *__restrict__ L, int64_t n, const float *Rin,
                                                         float *X, uint16_t *__restrict__ Xh, int64_t nrhs, int64_t r0,
                                                         int tiles, const float *__restrict__ Winv, const int *__restrict__ ok, int limit,
                                                         const char *__restrict__ packed)
{
    __shared__ __attribute__((aligned(16))) PanelLds lds;
    bool inverses = Winv != nullptr;
    if (inverses)
        for (int t = 0; t < tiles; ++t) inverses = inverses && ok[t] != 0;          // uniform
    // Two workgroups per slab of 64 right-hand sides: through the inverses each takes 32 of them; the substitution, one
    // lane per right-hand side, is the first one's alone.
    if (inverses) {
        const int64_t c0 = (int64_t)(blockIdx.x >> 1) * 64 + (blockIdx.x & 1) * 32;
        if (c0 < nrhs) panel_by_inverses(lds, L, n, Rin, X, Xh, nrhs, r0, tiles, Winv, c0, packed);
    } else if ((blockIdx.x & 1) == 0) {
        panel_by_substitution(lds, L, n, Rin, X, Xh, nrhs, r0, tiles, limit);
    }
}

struct Solve {
    const uint16_t *L;
    const float *B;
    float *X;
    uint16_t *Xh;
    int64_t n, nrhs, nb;
    hipStream_t s;
    const float *Winv;      // inverses of the full diagonal tiles, tile after tile, or nullptr
    const int *ok;          // per tile: the inverse may stand in for the substitution
    const char *packed;     // the tiles next to the diagonal in operand order (see PANEL_BAND), with Winv
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
    hipError_t launch_err = hipSuccess;
    if (vec && rows == 64)
        launch_err = launch_kernel(tri_diag_kernel<64, true>, grid, dim3(64), v.s, v.L, v.n, R, v.X, v.Xh, v.nrhs, r0, rows, vec);
    else if (vec && rows == 128)
        launch_err = launch_kernel(tri_diag_kernel<128, true>, grid, dim3(64), v.s, v.L, v.n, R, v.X, v.Xh, v.nrhs, r0, rows, vec);
    else if (rows <= 64)
        launch_err = launch_kernel(tri_diag_kernel<64, false>, grid, dim3(64), v.s, v.L, v.n, R, v.X, v.Xh, v.nrhs, r0, rows, vec);
    else
        launch_err = launch_kernel(tri_diag_kernel<128, false>, grid, dim3(64), v.s, v.L, v.n, R, v.X, v.Xh, v.nrhs, r0, rows, vec);
    return launch_err;
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

// the four-wave panel kernel can be used: whole 16-byte pieces of the rows of X and Xh
bool panelw_ok(const Solve &v) { return v.nrhs % 8 == 0 && (uintptr_t)v.X % 16 == 0 && (uintptr_t)v.Xh % 16 == 0; }

// up to four (eight with the four-wave kernel) full 64-row tiles with 16-byte aligned rows of L: one launch for the
// whole range
bool panel_ok(const Solve &v, int64_t r0, int64_t r1)
{
    return v.nb == 64 && (r1 - r0) % 64 == 0 && r1 - r0 <= 64 * (panelw_ok(v) ? PANELW : 4) && (uintptr_t)v.L % 16 == 0 &&
           v.n % 8 == 0 && r0 % 8 == 0;
}

hipError_t panel(const Solve &v, int64_t r0, int64_t r1)
{
    dim3 grid((unsigned)((v.nrhs + 63) / 64));
    const int tiles = (int)((r1 - r0) / 64);
    hipError_t launch_err = hipSuccess;
    if (panelw_ok(v))
        launch_err = launch_kernel(tri_panelw_kernel, dim3(2 * grid.x), dim3(256), v.s, v.L, v.n, rhs_of(v, r0), v.X, v.Xh, v.nrhs, r0, tiles,
                                   v.Winv ? v.Winv + r0 / 64 * INV_FLOATS : nullptr, v.ok ? v.ok + r0 / 64 : nullptr, wait_limit(), v.packed);
    else
        launch_err = launch_kernel(tri_panel_kernel, grid, dim3(64), v.s, v.L, v.n, rhs_of(v, r0), v.X, v.Xh, v.nrhs, r0, tiles);
    return launch_err;
}

hipError_t solve(const Solve &v, int64_t r0, int64_t r1)
{
    if (panel_ok(v, r0, r1)) return panel(v, r0, r1);
    if (r1 - r0 <= v.nb) return diag(v, r0, r1);
    const int64_t tiles = (r1 - r0 + v.nb - 1) / v.nb;
    const int64_t mid = r0 + (tiles + 1) / 2 * v.nb;       // the first half takes the odd tile: mid stays a tile boundary
    hipError_t e = solve(v, r0, mid);
    if (e == hipSuccess) e = update(v, r0, mid, r1);
    if (e == hipSuccess) e = solve(v, mid, r1);
    return e;
}

}  // namespace

// the diagonal tiles are worth inverting ahead: the four-wave panel kernel will run, on tiles of 64 rows
static bool inverses_wanted(const Solve &v)
{
    return v.nb == 64 && v.n >= 64 && panelw_ok(v) && (uintptr_t)v.L % 16 == 0 && v.n % 8 == 0 && v.n < (1 << 26) && v.nrhs < (1 << 24);
}

int64_t trsm_workspace_bytes(const void *L, void *X, void *Xh, int64_t n, int64_t nrhs, int64_t nb)
{
    Solve v{(const uint16_t *)L, nullptr, (float *)X, (uint16_t *)Xh, n, nrhs, nb, nullptr, nullptr, nullptr, nullptr};
    // per full tile: its inverse, the operand-order copy of the tiles left of it, its verdict
    return inverses_wanted(v) ? (n / 64) * (int64_t)(INV_FLOATS * sizeof(float) + PACK_BYTES_PER_TILE_ROW + sizeof(int)) : 0;
}

hipError_t launch_trsm(const void *L, const void *B, void *X, void *Xh, int64_t n, int64_t nrhs, int64_t nb, void *workspace,
                       hipStream_t s)
{
    if (nb < 1 || nb > 128 || (int64_t)((nrhs + 63) / 64) > 0x3fffffff) return hipErrorInvalidValue;
    Solve v{(const uint16_t *)L, (const float *)B, (float *)X, (uint16_t *)Xh, n, nrhs, nb, s, nullptr, nullptr, nullptr};
    if (workspace && inverses_wanted(v)) {
        const int64_t full = n / 64;
        float *Winv = (float *)workspace;
        char *packed = (char *)(Winv + full * INV_FLOATS);
        int *ok = (int *)(packed + full * PACK_BYTES_PER_TILE_ROW);
        const hipError_t e = launch_kernel(tri_inverse_kernel, dim3((unsigned)(full + full * PANEL_BAND * PACK_PIECES)), dim3(64), s, v.L, n, Winv, ok,
                                           packed, (int)full);
        if (e != hipSuccess) return e;
        v.Winv = Winv;
        v.ok = ok;
        v.packed = packed;
    }
    return solve(v, 0, n);
}

}  // namespace cyc
