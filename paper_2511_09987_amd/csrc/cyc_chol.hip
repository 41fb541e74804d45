// cyc_chol.hip -- the tiled Cholesky recurrence  A = L L^T  on gfx950.
//
// Paper, "Cholesky Recurrence": with A cut into nb x nb tiles, for every panel (tile column) j
//     S_jj = A_jj - sum_{k<j} SYRK(L_jk),          L_jj = CHOL(S_jj),
//     S_ij = A_ij - sum_{k<j} GEMM(L_ik, L_jk),    L_ij = TRSM(S_ij, L_jj)      for the tiles i below j,
// where the scalar form ("Representative recurrences") is
//     L_ii = sqrt(A_ii - sum_{k<i} L_ik^2),        L_ij = (A_ij - sum_{k<j} L_ik L_jk) / L_jj.
//
// Mapping, on the caller's stream.  The SYRKs and GEMMs are products of the matrix-multiply recurrence of this
// library (bf16 operands, fp32 sums): rows of the finished factor times the transpose of other rows of it.  The
// transpose costs nothing because the bf16 copy of the factor, Lh, is kept with both triangles filled
// (Lh[c][r] = Lh[r][c]): a stationary operand is a window Lh[r0:, k0:k1], the streamed one the window
// Lh[k0:k1, c0:c1].  Panels are taken in groups of eight (see launch_chol):
//   1. at the first panel of a group, one launch of the GEMM kernel takes all tiles left of the group out of the
//      group's columns: epilogue A - product into L[g0:, g0:g0+512], which holds S until solved;
//   2. per panel, CHOL of the diagonal tile: one lane per row, columns left to right, what a lane needs of other
//      rows read from the tile in LDS, where every lane writes its finished columns;
//   3. per panel, TRSM of the rows below: rows do not depend on one another, so one lane per row (64 rows per
//      workgroup) runs the off-diagonal line of the scalar recurrence against L_jj in LDS, and writes its row of
//      L, of Lh, and the mirrored column of Lh.
//   Both tile kernels are workgroups of four waves: all four move the tile and first take the terms of the group's
//   own earlier panels out of it with MFMAs of their own (TileProduct), which is far cheaper than a launch of the
//   GEMM kernel for so short a k range; the first wave then runs the recurrence.  Step 2 for panel j + 1 is done by
//   the first workgroup of step 3 for panel j (the rows that become tile (j+1, j)), in the same launch, also across
//   a group boundary: the chain diagonal tile - tile below it - next diagonal tile is what the whole factorisation
//   waits for.  On that chain
//   - the diagonal tile's recurrence is shared by two waves: the first keeps the corners (square roots, divisions)
//     and the multiply-adds next to them, the second takes every finished block of four columns out of the columns
//     further right on the matrix cores (trailing_update64);
//   - the TRSM of the tile below a well-conditioned diagonal tile is a product with the diagonal tile's inverse,
//     which a third wave computes beside the factorisation of the tile (inverse_follow64).
// Inside a tile column everything is fp32 on unrounded values, in the order of the scalar recurrence:
// t = S_rc; t = fma(-L_rk, L_ck, t) for k ascending; then sqrt on the diagonal, IEEE division below it.  Four such steps
// are one v_mfma_f32_16x16x4_f32: that instruction adds its products in ascending k with one rounding each.
#include "cyc_internal.h"
#include "cyc_wave.h"

namespace cyc {
namespace {

constexpr int NBMAX = 64;      // largest tile
constexpr int LDT = NBMAX + 4; // row stride of the tiles in LDS: rows stay 16-byte aligned, and 16 consecutive rows
                               // spread over all banks for 16-byte reads
typedef float f32x4 __attribute__((ext_vector_type(4), may_alias));   // read from arrays written as floats

// t - sum_{k<c} x[k] y[k] as the chain t = fma(-x[k], y[k], t), k ascending; x and y are 16-byte aligned rows in LDS.
// Four terms per pair of 16-byte reads, the reads of the next four issued before the current four are used.
__device__ __forceinline__ float chain(float t, const float *x, const float *y, int c)
{
    const int c4 = c & ~3;
    if (c4) {
        f32x4 a = *(const f32x4 *)x, b = *(const f32x4 *)y;
        for (int k = 4; k < c4; k += 4) {
            const f32x4 a2 = *(const f32x4 *)(x + k), b2 = *(const f32x4 *)(y + k);
#pragma unroll
            for (int q = 0; q < 4; ++q) t = __builtin_fmaf(-a[q], b[q], t);
            a = a2;
            b = b2;
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) t = __builtin_fmaf(-a[q], b[q], t);
    }
    for (int k = c4; k < c; ++k) t = __builtin_fmaf(-x[k], y[k], t);
    return t;
}

// fp32 -> bfloat16 bit pattern, round to nearest, ties to even; NaN stays NaN (the hardware conversion)
__device__ __forceinline__ uint16_t round_bf16(float f) { return __builtin_bit_cast(uint16_t, (__bf16)f); }
// two values rounded and packed (a in the low half) by one conversion instruction, where rounding them one by one and
// joining the halves takes four
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) { return __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2_t){a, b}, bf16x2_t)); }

// The same for the diagonal tile, where row c of L is what lane c has just computed.  The chains of block b read the
// rows 4b .. 4b+3 of L from LDS, where every lane writes its finished columns; the step over the columns of block k4 can
// be read once the corner of block k4 is written.
// The first wave takes only the steps close to the diagonal itself: the tile's columns in groups of 16 (four blocks),
// group G handed to it by a second wave (trailing_update64) with all steps up to block 4G - 2 taken out already, on
// the matrix cores.  Of block b it runs the steps first_k(b) .. b - 1: the last one (k4 = b - 1) is requested right
// after the corner of block b - 1, the one before it is held back to cover that request's latency, the others (at most
// two) run beside the corner of block b - 1, one after each of its first columns; all but the last are requested when
// that corner starts, which is after block b - 2 was written.
constexpr int first_k(int b) { return b < 4 ? 0 : 4 * (b / 4) - 1; }
constexpr int own_steps(int b) { return b - first_k(b); }
constexpr int LDF = 20;        // row stride of the hand-over buffer: 16 columns, and 16 consecutive rows on distinct banks

constexpr int NT = 256;        // threads of a tile kernel: four waves move tiles and multiply, the first runs the recurrence

// A 64-row tile of a row-major fp32 matrix (row stride ld) into LDS, by the workgroup: rows 0..nrows-1 (rows past that
// repeat the last one), columns 0..cols-1.  All loads of a thread are in flight together.
__device__ __forceinline__ void load_tile(float (*dst)[LDT], const float *src, int64_t ld, int nrows, int cols, int tid)
{
    if (cols == NBMAX && ld % 4 == 0 && ((uintptr_t)src & 15) == 0) {
        constexpr int PASSES = NBMAX * 16 / NT;
        f32x4 v[PASSES];
#pragma unroll
        for (int i = 0; i < PASSES; ++i) {
            const int r = NT / 16 * i + (tid >> 4);
            v[i] = *(const f32x4 *)(src + (int64_t)(r < nrows ? r : nrows - 1) * ld + 4 * (tid & 15));
        }
#pragma unroll
        for (int i = 0; i < PASSES; ++i) *(f32x4 *)&dst[NT / 16 * i + (tid >> 4)][4 * (tid & 15)] = v[i];
    } else {
        for (int i0 = 0; i0 < NBMAX * cols; i0 += NT * 4) {
            float v[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int i = i0 + NT * q + tid, r = i / cols, c = i - r * cols;
                v[q] = i < NBMAX * cols ? src[(int64_t)(r < nrows ? r : nrows - 1) * ld + c] : 0.0f;
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int i = i0 + NT * q + tid, r = i / cols, c = i - r * cols;
                if (i < NBMAX * cols) dst[r][c] = v[q];
            }
        }
    }
}

// The same in two steps for kernels that fetch several tiles: request() issues the loads of a thread, place() puts
// them into LDS.  With the steps of two tiles interleaved (all requests, then all placements) memory is waited for
// once; load_tile twice in a row waits for the first tile before it asks for the second.
struct TileLoad {
    static constexpr int PASSES = NBMAX * 16 / NT;
    f32x4 v[PASSES];
    bool whole;
    __device__ __forceinline__ void request(const float *src, int64_t ld, int nrows, int cols, int tid)
    {
        whole = cols == NBMAX && ld % 4 == 0 && ((uintptr_t)src & 15) == 0;             // uniform
        if (whole) {
#pragma unroll
            for (int i = 0; i < PASSES; ++i) {
                const int r = NT / 16 * i + (tid >> 4);
                v[i] = *(const f32x4 *)(src + (int64_t)(r < nrows ? r : nrows - 1) * ld + 4 * (tid & 15));
            }
        }
    }
    __device__ __forceinline__ void place(float (*dst)[LDT], const float *src, int64_t ld, int nrows, int cols, int tid)
    {
        if (whole) {
#pragma unroll
            for (int i = 0; i < PASSES; ++i) *(f32x4 *)&dst[NT / 16 * i + (tid >> 4)][4 * (tid & 15)] = v[i];
        } else {
            load_tile(dst, src, ld, nrows, cols, tid);
        }
    }
};

// The reverse for a full-width tile held in LDS: rows 0..nrows-1 to the fp32 matrix L and, rounded, to the bfloat16
// matrix Lh (both with row stride ld), 16 bytes per thread and store.  False when shape or alignment do not allow it.
// LOWER: the tile is a diagonal tile; L gets zeros above the diagonal (Lh gets what the tile holds there).
template <bool LOWER, int NTH = NT>
__device__ __forceinline__ bool store_tile(const float (*src)[LDT], float *L, uint16_t *Lh, int64_t ld, int nrows, int cols,
                                           int tid)
{
    if (cols != NBMAX || ld % 8 != 0 || ((uintptr_t)L & 15) != 0 || ((uintptr_t)Lh & 15) != 0) return false;
    // all LDS reads first, without conditions (rows past nrows hold copies of the last one), then the stores: a read
    // inside the row condition would be waited for on the spot, once per row group
    constexpr int PL = NBMAX * 16 / NTH, PH = NBMAX * 8 / NTH;      // tid counts the NTH threads that take part
    f32x4 v[PL];
#pragma unroll
    for (int i = 0; i < PL; ++i) {
        const int r = NTH / 16 * i + (tid >> 4);
        v[i] = *(const f32x4 *)&src[r][4 * (tid & 15)];
        if (LOWER) {
#pragma unroll
            for (int q = 0; q < 4; ++q) v[i][q] = 4 * (tid & 15) + q <= r ? v[i][q] : 0.0f;
        }
    }
    typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
    u32x4 h[PH];
#pragma unroll
    for (int i = 0; i < PH; ++i) {
        const int r = NTH / 8 * i + (tid >> 3);
        const f32x4 a = *(const f32x4 *)&src[r][8 * (tid & 7)], b = *(const f32x4 *)&src[r][8 * (tid & 7) + 4];
        h[i][0] = pack_bf16(a[0], a[1]);
        h[i][1] = pack_bf16(a[2], a[3]);
        h[i][2] = pack_bf16(b[0], b[1]);
        h[i][3] = pack_bf16(b[2], b[3]);
    }
#pragma unroll
    for (int i = 0; i < PL; ++i) {
        const int r = NTH / 16 * i + (tid >> 4);
        if (r < nrows) *(f32x4 *)(L + (int64_t)r * ld + 4 * (tid & 15)) = v[i];
    }
#pragma unroll
    for (int i = 0; i < PH; ++i) {
        const int r = NTH / 8 * i + (tid >> 3);
        if (r < nrows) *(u32x4 *)(Lh + (int64_t)r * ld + 8 * (tid & 7)) = h[i];
    }
    return true;
}

// The mirror image of 64 finished rows (a tile in LDS) into the upper triangle of Lh, by NTH threads: thread (column c,
// part) gathers 64 * 4 / NTH rows of its column (the rows of the tile are LDT floats apart: 16 of them lie on distinct
// banks) and stores them as 16-byte pieces.  dst: entry (column 0, row 0); requires 16-byte aligned rows of Lh.
template <int NTH>
__device__ __forceinline__ void store_mirror(const float (*src)[LDT], uint16_t *dst, int64_t ld, int tid)
{
    constexpr int PARTS = NTH / 64, ROWS = 64 / PARTS;
    const int c = tid / PARTS, r0 = ROWS * (tid % PARTS);
    uint32_t packed[ROWS / 2];
#pragma unroll
    for (int i = 0; i < ROWS / 2; ++i)
        packed[i] = pack_bf16(src[r0 + 2 * i][c], src[r0 + 2 * i + 1][c]);
    uint4 *out = (uint4 *)(dst + (int64_t)c * ld + r0);
#pragma unroll
    for (int i = 0; i < ROWS / 8; ++i) out[i] = make_uint4(packed[4 * i], packed[4 * i + 1], packed[4 * i + 2], packed[4 * i + 3]);
}

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x2 __attribute__((ext_vector_type(2)));
#define CYC_LDS __attribute__((address_space(3)))
constexpr int KMAX = 7 * NBMAX;           // longest k range a tile kernel multiplies out by itself (a group's earlier panels)

// The update of a 64 x 64 tile by the earlier panels of its group, inside the tile's own kernel (four waves):
//     S[r][c] -= sum_{k0 <= k < k1} Lh[row0 + r][k] * Lh[k][j0 + c]          (the second factor is the mirror image)
// as bf16 MFMAs with fp32 sums, S being a tile in LDS; wave w computes rows 16 w .. 16 w + 15 (one wave alone would
// be bound by the MFMA rate of its one SIMD: 224 MFMAs for seven tiles of k).  The streamed operand,
// Lh[k0:k1, j0:j0+64], is staged in LDS ([k][column], 128 bytes per row, see staged_swizzle) and read through the transpose read; the
// stationary operand, the tile's own rows of Lh, goes from memory straight into operand registers, all k-steps at
// once.  Rows past `nrows` repeat the last one.  Requires 16-byte aligned rows of Lh (n, k0, j0 multiples of 8) and
// k1 - k0 a multiple of 64, at most KM.
// In two parts, so that a kernel can ask for the operands first, then for its tile, and wait for memory once.
// An MFMA operand fragment of k-step ks out of a staged operand ([k][64 columns] in LDS), through the transposing
// read: lane l gets column 16 c + l%16, k = 32 ks + 8 (l/16) .. +7.  As a streamed fragment that is column block c; where
// the staged operand is the mirror image of rows of Lh, the same words are the stationary fragment of row block c.
// Placement of a staged operand: row k (128 bytes: eight 16-byte chunks) at k * 128, its chunk q in slot
// q ^ staged_swizzle(k).  One transposing read takes 8 bytes per lane from the rows 8 (l/16) + 0 .. 3 of a k-step, two
// adjacent chunks of each: unswizzled those are sixteen rows whose chunks lie on the same 16 of the 64 banks (a row is
// half the banks wide, rows two apart coincide), an eight-way conflict; the swizzle moves each group of eight rows to
// banks of its own, which leaves the two-way conflict that 512 bytes per instruction cannot avoid.
__device__ __forceinline__ constexpr int staged_swizzle(int k) { return ((k >> 3) & 3) << 1; }
__device__ __forceinline__ i32x4 staged_fragment(uint16_t (*src)[64], int ks, int c, int lq, int g)
{
    // (rows 32 ks + 8 g + 0 .. 7 share the swizzle 2 g)
    const int chunk = (2 * c + ((lq >> 1) & 1)) ^ (2 * g);
    CYC_LDS char *p = (CYC_LDS char *)&src[ks * 32 + 8 * g + (lq >> 2)][0] + 16 * chunk + 8 * (lq & 1);
    const i32x2 lo = __builtin_bit_cast(i32x2, __builtin_amdgcn_ds_read_tr16_b64_v4bf16((CYC_LDS bf16x4 *)p));
    const i32x2 hi = __builtin_bit_cast(i32x2, __builtin_amdgcn_ds_read_tr16_b64_v4bf16((CYC_LDS bf16x4 *)(p + 4 * 64 * 2)));
    return (i32x4){lo[0], lo[1], hi[0], hi[1]};
}

template <int KM>
struct TileProductT {
    static constexpr int NKS = KM / 32;
    i32x4 a[NKS];
    int nks;

    // start the copies of both operands; nothing is waited for
    // rows_in_lds: the tile's own rows of Lh will be at hand in LDS as their mirror image (see apply): none are loaded
    __device__ __forceinline__ void request(uint16_t (*Bs)[64], const uint16_t *__restrict__ Lh, int64_t n, int64_t row0, int nrows,
                                            int64_t k0, int64_t k1, int64_t j0, int tid, bool rows_in_lds = false)
    {
        const int lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6), lq = lane & 15, g = lane >> 4, K = (int)(k1 - k0);
        nks = K / 32;
        // the streamed operand: 8 rows of 128 bytes per copy, memory to LDS directly, all copies in flight at once
        const uint32_t lds_base = (uint32_t)(uintptr_t)(CYC_LDS char *)&Bs[0][0];
        for (int k = 8 * w; k < K; k += 8 * (NT / 64)) {
            // lane l fills slot l%8 of row k + l/8: with the chunk that belongs there (staged_swizzle)
            const uint32_t voff = (uint32_t)(lane >> 3) * (uint32_t)(n * 2) + (uint32_t)((lane & 7) ^ staged_swizzle(k)) * 16;
            const char *base = (const char *)(Lh + (k0 + k) * n + j0);
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                         :
                         : "s"(lds_base + k * 128), "v"(voff), "s"(base)
                         : "memory", "m0");
        }
        // the stationary operand: row 16 w + lq of the tile, k = 32 ks + 8 g .. +7
        if (rows_in_lds) return;                                           // uniform
        const int r = 16 * w + lq;
        const uint16_t *rowp = Lh + (row0 + (r < nrows ? r : nrows - 1)) * n + k0 + 8 * g;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks)
            if (ks < nks) a[ks] = *(const i32x4 *)(rowp + 32 * ks);        // uniform; a load of 16 rows is 64 line requests: none to spare
    }

    // S -= product; call with the tile S in place in LDS and no barrier needed before: waits for the copies itself
    // As: nullptr, or Lh[k0:k1, row0:row0+64] in LDS, the mirror image of the tile's own rows (request with rows_in_lds):
    // the stationary fragment of rows 16 w .. is then read like a streamed fragment of column block w
    __device__ __forceinline__ void apply(float (*S)[LDT], uint16_t (*Bs)[64], int tid, uint16_t (*As)[64] = nullptr)
    {
        const int lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6), lq = lane & 15, g = lane >> 4;
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        f32x4 acc[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[j] = (f32x4){0, 0, 0, 0};
        if (As) {
            // every fragment from LDS: a loop that reads the fragments of the next k-step before it multiplies the
            // current ones (unrolled with a condition per step, as below, each step would wait for its own reads)
            i32x4 f[2][5];                                                       // [parity of the k-step]: stationary, streamed x 4
            auto read_step = [&](int ks, i32x4(&dst)[5]) __attribute__((always_inline)) {
                dst[0] = staged_fragment(As, ks, w, lq, g);
#pragma unroll
                for (int j = 0; j < 4; ++j) dst[1 + j] = staged_fragment(Bs, ks, j, lq, g);
            };
            auto multiply = [&](const i32x4(&src)[5]) __attribute__((always_inline)) {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, src[0]), __builtin_bit_cast(bf16x8, src[1 + j]), acc[j], 0, 0, 0);
            };
            read_step(0, f[0]);                                                  // (nks is even and at least 2)
            if (nks == 2) {                                                      // (a panel whose earlier terms were taken out ahead)
                read_step(1, f[1]);
                multiply(f[0]);
                multiply(f[1]);
            } else {
                for (int ks = 0; ks < nks; ks += 2) {
                    read_step(ks + 1, f[1]);
                    multiply(f[0]);
                    if (ks + 2 < nks) read_step(ks + 2, f[0]);
                    multiply(f[1]);
                }
            }
        }
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            if (!As && ks < nks) {                                               // uniform over the workgroup
                i32x4 b[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) b[j] = staged_fragment(Bs, ks, j, lq, g);
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a[ks]), __builtin_bit_cast(bf16x8, b[j]), acc[j], 0, 0, 0);
            }
        }
        // accumulator register r of lane l is row 4 (l/16) + r, column l%16 of its 16 x 16 tile
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) S[16 * w + 4 * g + r][16 * j + lq] -= acc[j][r];
        __syncthreads();
    }
};

typedef TileProductT<KMAX> TileProduct;

// ---- The inverse of a diagonal tile, computed beside its factorisation.
// L_ij = TRSM(S_ij, L_jj) for the tile right below the diagonal tile is on the path from one diagonal tile to the
// next: 64 dependent columns.  With W = L_jj^-1 at hand it is the product S_ij W^T on the matrix cores, which has no
// chain; and W can be had off that path: while the first wave factors the tile, the second follows it four rows
// behind, lane j solving L_jj y = e_j by the substitution of the triangular solve (the step list of cyc_wave.h: rows
// 4b .. 4b+3 of L_jj are final once the factorisation has finished block b, which it announces through a counter in
// LDS).  As in the triangular solve the product stands in for the substitution only when the tile is well
// conditioned: the follower leaves ||W||_1 ||L_jj||_1 <= 8 (and everything finite, and no wait expired) as a verdict
// beside W.  W is stored in the order in which the product wants its operand, the one of the triangular solve's
// inverses: entry (r, j) in piece 4 (r / 16) + j / 16 of 1 KiB, at [(r % 16) + 16 (j % 4)][(j / 4) % 4].
constexpr int W_FLOATS = 64 * 64;
constexpr float W_NORM_LIMIT = 8.0f;

// maximum over the 64 lanes of a wave, in every lane
__device__ __forceinline__ float wave_max64(float v)
{
    auto dpp = [](float x, auto ctrl) __attribute__((always_inline)) {
        return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), decltype(ctrl)::value, 0xf, 0xf, true));
    };
    v = __builtin_fmaxf(v, dpp(v, std::integral_constant<int, 0xB1>{}));      // quad_perm 1,0,3,2
    v = __builtin_fmaxf(v, dpp(v, std::integral_constant<int, 0x4E>{}));      // quad_perm 2,3,0,1
    v = __builtin_fmaxf(v, dpp(v, std::integral_constant<int, 0x141>{}));     // row_half_mirror
    v = __builtin_fmaxf(v, dpp(v, std::integral_constant<int, 0x140>{}));     // row_mirror: the maximum of each row of 16
    const unsigned u = __builtin_bit_cast(unsigned, v);
    const auto a = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    const unsigned a0 = a[0], a1 = a[1];
    const unsigned m = __builtin_bit_cast(unsigned, __builtin_fmaxf(__builtin_bit_cast(float, a0), __builtin_bit_cast(float, a1)));
    const auto b = __builtin_amdgcn_permlane32_swap(m, m, false, false);
    const unsigned b0 = b[0], b1 = b[1];
    return __builtin_fmaxf(__builtin_bit_cast(float, b0), __builtin_bit_cast(float, b1));
}

// What the waves of a diagonal tile's factorisation pass to one another in LDS.
constexpr int LDY = 80;        // row stride of Y: 64 columns, and four consecutive rows on disjoint banks
struct DiagLds {
    float F[NBMAX][LDF];       // a group of 16 columns on its way from the second wave to the first (trailing_update64)
    float Y[16][LDY];          // the follower's rows of W of the current group of 16 (inverse_follow64)
    int sync[3];               // blocks of four columns finished; groups handed over; a wait ran out (trailing_update64)
};

// The follower: one wave computes W = L_jj^-1 beside the factorisation, in the order in which its work becomes
// available.  T holds S above the factorisation's progress and L below it; *ready counts the blocks of four columns the
// factorisation has finished.  Block k brings the columns 4k .. 4k+3 of every row of L_jj: the follower then solves
// the rows 4k .. 4k+3 of L_jj W = I (their 4 x 4 corner is complete with that block) and takes them out of all rows
// below at once, so that after the factorisation's last block only a corner is left to do.  The running right-hand
// side is kept in the accumulator layout of v_mfma_f32_16x16x4_f32 (the ten 16 x 16 blocks on and below the block
// diagonal: register r of lane l is row 16 rb + 4 (l/16) + r, column 16 cb + l%16), so that taking four rows out of
// the rows below is one MFMA per block: A operand -L_jj[16 rb + l%16][4k + l/16], straight from T; B operand
// W[4k + l/16][16 cb + l%16], which crosses LDS (Y) from the 16 lanes per column block that have just solved it.  Y
// also collects the 16 rows of a group, which go out to W in the operand order of the product that uses them, 1 KiB
// pieces as 16-byte stores.  Every read of T here is of columns of block k, behind the gate of block k.
// Reciprocals of the diagonal by estimate and one Newton step: W is only ever used as an approximation whose error the
// check at the end bounds.
// Not inlined, and its LDS operands passed as addresses: inside diag_rest it raised that kernel's register count from 228
// to 369 and put the factorisation's own values into accumulation registers, 3k cycles on the path per tile.
__device__ __attribute__((noinline)) void inverse_follow64(uint32_t T_in_lds, uint32_t Y_in_lds, uint32_t ready_in_lds, int lane, int limit,
                                                           float *__restrict__ W, int *__restrict__ ok)
{
    CYC_LDS const float *const T = (CYC_LDS const float *)(uintptr_t)T_in_lds;
    CYC_LDS float *const Y = (CYC_LDS float *)(uintptr_t)Y_in_lds;              // [16][LDY]
    CYC_LDS int *const ready = (CYC_LDS int *)(uintptr_t)ready_in_lds;
    // (as a pointer to global memory: through the generic pointer of a function that is not inlined the stores would be
    // flat instructions, which count as LDS operations too and complete out of order with them, and every wait for
    // an LDS read below would become a wait for all of them)
    typedef __attribute__((address_space(1))) f32x4 global_f32x4;
    global_f32x4 *const out = (global_f32x4 *)W + lane;
    const int i = lane & 15, g = lane >> 4;

    bool expired = false;
    auto gate = [&](int b) __attribute__((always_inline)) {
        int polls = 0;
        while (__hip_atomic_load(ready, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) <= b) {
            if (++polls >= limit) {
                expired = true;
                break;
            }
            __builtin_amdgcn_s_sleep(1);
        }
    };
    auto idx = [](int rb, int cb) __attribute__((always_inline)) { return rb * (rb + 1) / 2 + cb; };
    f32x4 t[10];                                               // the running right-hand side: the identity to begin with
#pragma unroll
    for (int rb = 0; rb < 4; ++rb)
#pragma unroll
        for (int cb = 0; cb <= rb; ++cb)
#pragma unroll
            for (int r = 0; r < 4; ++r) t[idx(rb, cb)][r] = rb == cb && 4 * g + r == i ? 1.0f : 0.0f;
    float colsum_L = 0.0f, colsum_W[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    unrolled<NBLK>([&](auto index) __attribute__((always_inline)) {
        constexpr int k = decltype(index)::value, R = k / 4, gk = k % 4;
        gate(k);
        // the block's corner of L_jj, the lane's own column of it (for ||L_jj||_1), and the block's columns of the rows
        // below as stationary operands
        f32x4 qc[4];
        float mine[4], xm[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            qc[j] = *(CYC_LDS const f32x4 *)&T[(4 * k + j) * LDT + 4 * k];
            mine[j] = T[(4 * k + j) * LDT + lane];
        }
#pragma unroll
        for (int rb = (gk == 3 ? R + 1 : R); rb < 4; ++rb) xm[rb] = -T[(16 * rb + i) * LDT + 4 * k + g];
        float rinv[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            colsum_L += 4 * k + j >= lane ? __builtin_fabsf(mine[j]) : 0.0f;
            const float d = qc[j][j], r0 = __builtin_amdgcn_rcpf(d);
            rinv[j] = __builtin_fmaf(__builtin_fmaf(-d, r0, 1.0f), r0, r0);
        }
        // rows 4k .. 4k+3 of W: in the lanes with l/16 = k%4 the registers of row block R are exactly those rows; the
        // other lanes compute along on rows that are not ready
        f32x4 y[4];
#pragma unroll
        for (int cb = 0; cb <= R; ++cb) {
            const f32x4 rhs = t[idx(R, cb)];
            float xn[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                float v = rhs[j];
#pragma unroll
                for (int e = 0; e < j; ++e) v = __builtin_fmaf(qc[j][e], xn[e], v);
                y[cb][j] = v * rinv[j];
                xn[j] = -y[cb][j];
            }
        }
        if (g == gk) {                                         // (one branch per block; the stores differ by constants only)
#pragma unroll
            for (int cb = 0; cb <= R; ++cb)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    colsum_W[cb] += __builtin_fabsf(y[cb][j]);
                    Y[(4 * gk + j) * LDY + 16 * cb + i] = y[cb][j];
                }
        }
        // and out of every row below (of row block R, too: its rows up to 4k+3 are not used again)
        // (pinned here: the compiler otherwise moves all these additions, with their operands, to the end of the function,
        // behind the factorisation's last block)
        asm volatile("" : "+v"(colsum_L), "+v"(colsum_W[0]), "+v"(colsum_W[1]), "+v"(colsum_W[2]), "+v"(colsum_W[3]));
        constexpr int first_rb = gk == 3 ? R + 1 : R;          // (with its last four rows a row block is finished)
        if (first_rb < 4) {
            float yb[4];
#pragma unroll
            for (int cb = 0; cb <= R; ++cb) yb[cb] = Y[(4 * gk + g) * LDY + 16 * cb + i];
#pragma unroll
            for (int rb = first_rb; rb < 4; ++rb)
#pragma unroll
                for (int cb = 0; cb <= R; ++cb) t[idx(rb, cb)] = __builtin_amdgcn_mfma_f32_16x16x4f32(xm[rb], yb[cb], t[idx(rb, cb)], 0, 0, 0);
        }
        if (gk == 3) {
            // rows 16 R .. 16 R + 15 are complete: piece (R, cb) in the order in which the product wants its operand,
            // lane l: W[16 R + l%16][16 cb + 4 q + l/16], q = 0 .. 3
#pragma unroll
            for (int cb = 0; cb <= R; ++cb) {
                f32x4 piece;
#pragma unroll
                for (int q = 0; q < 4; ++q) piece[q] = Y[i * LDY + 16 * cb + 4 * q + g];
                out[(4 * R + cb) * 64] = piece;
            }
        }
    });
    // ||W||_1: the column sums lie in four parts, one per l/16: add the lanes 16, 32 and 48 apart
    float colsum = 0.0f;
#pragma unroll
    for (int cb = 0; cb < 4; ++cb) {
        const unsigned u = __builtin_bit_cast(unsigned, colsum_W[cb]);
        const auto h = __builtin_amdgcn_permlane16_swap(u, u, false, false);
        const unsigned h0 = h[0], h1 = h[1];
        const unsigned m = __builtin_bit_cast(unsigned, __builtin_bit_cast(float, h0) + __builtin_bit_cast(float, h1));
        const auto f = __builtin_amdgcn_permlane32_swap(m, m, false, false);
        const unsigned f0 = f[0], f1 = f[1];
        const float sum = __builtin_bit_cast(float, f0) + __builtin_bit_cast(float, f1);
        colsum = sum > colsum || sum != sum ? sum : colsum;                    // (keeps a NaN)
    }
    const float a = wave_max64(colsum_L), c = wave_max64(colsum);
    // (a NaN anywhere would be dropped by the maxima: every lane checks its own sums)
    const bool fine = colsum_L == colsum_L && colsum == colsum && a * c <= W_NORM_LIMIT && !expired;
    const bool all_fine = __builtin_amdgcn_ballot_w64(!fine) == 0;
    if (lane == 0) *ok = all_fine ? 1 : 0;
}

// The second wave of the diagonal tile's factorisation.  It keeps the columns 16 .. 63 of the tile (the six 16 x 16
// blocks on and below the block diagonal) in accumulator layout and takes block after block of finished columns out of
// them as soon as the first wave announces it: S_rc <- fma(-L_rk, L_ck, S_rc) for the four k of a block is one
// v_mfma_f32_16x16x4_f32 per 16 x 16 block, which adds its four products in ascending k with one rounding each, the bits of
// the scalar chain (checked against it on 10^7 random elements per exponent range, denormal products included; the
// parity tests on integer and real data cover it as well).  Column group G goes to the first wave, through F, when block
// 4G - 2 is out of it; from then on that group is the first wave's.
// sync: [0] blocks finished by the first wave, [1] groups handed over, [2] set when a bounded wait ran out.
__device__ __attribute__((noinline)) void trailing_update64(uint32_t T_in_lds, uint32_t F_in_lds, uint32_t sync_in_lds, int lane, int limit)
{
    CYC_LDS const float *const T = (CYC_LDS const float *)(uintptr_t)T_in_lds;
    CYC_LDS float *const F = (CYC_LDS float *)(uintptr_t)F_in_lds;
    CYC_LDS int *const sync = (CYC_LDS int *)(uintptr_t)sync_in_lds;
    const int i = lane & 15, kq = lane >> 4;
    // block (cb, rb), 1 <= cb <= rb <= 3: register r of lane l is row 16 rb + 4 (l/16) + r, column 16 cb + l%16
    auto idx = [](int cb, int rb) __attribute__((always_inline)) { return cb == 1 ? rb - 1 : cb == 2 ? rb + 1 : 5; };
    f32x4 c[6];
#pragma unroll
    for (int cb = 1; cb < 4; ++cb)
#pragma unroll
        for (int rb = cb; rb < 4; ++rb)
#pragma unroll
            for (int r = 0; r < 4; ++r) c[idx(cb, rb)][r] = T[(16 * rb + 4 * kq + r) * LDT + 16 * cb + i];
    bool expired = false;
    unrolled<4 * 3 - 1>([&](auto index) __attribute__((always_inline)) {
        constexpr int p = decltype(index)::value;                      // the block of four finished columns to take out
        constexpr int first_cb = p % 4 == 3 ? p / 4 + 2 : p / 4 + 1;   // (group (p + 1) / 4 was handed over before its block 4G - 1)
        constexpr int G = p % 4 == 2 ? (p + 2) / 4 : 0;                // the group to hand over after this block
        if (first_cb <= 3) {
            int polls = 0;
            while (__hip_atomic_load(sync, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) <= p) {
                if (++polls >= limit) {
                    expired = true;
                    break;
                }
                __builtin_amdgcn_s_sleep(1);
            }
            // lane l: L[16 rb + l%16][4p + l/16], the stationary operand (negated) for row block rb and the streamed one
            // for column block rb
            float xr[4], xm[4];
#pragma unroll
            for (int rb = first_cb; rb < 4; ++rb) {
                xr[rb] = T[(16 * rb + i) * LDT + 4 * p + kq];
                xm[rb] = -xr[rb];
            }
            auto column_block = [&](int cb) __attribute__((always_inline)) {
#pragma unroll
                for (int rb = cb; rb < 4; ++rb) c[idx(cb, rb)] = __builtin_amdgcn_mfma_f32_16x16x4f32(xm[rb], xr[cb], c[idx(cb, rb)], 0, 0, 0);
            };
            if (G) {
                column_block(G);
#pragma unroll
                for (int rb = G; rb < 4; ++rb)
#pragma unroll
                    for (int r = 0; r < 4; ++r) F[(16 * rb + 4 * kq + r) * LDF + i] = c[idx(G, rb)][r];
                // (a wave's LDS operations are performed in issue order: whoever sees the counter sees the columns)
                asm volatile("" ::: "memory");
                __hip_atomic_store(sync + 1, G, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            }
#pragma unroll
            for (int cb = first_cb; cb < 4; ++cb)
                if (cb != G) column_block(cb);
        }
    });
    if (expired && lane == 0) sync[2] = 1;
}

// The factorisation proper of a diagonal tile whose S (with everything left of it taken out) is in T: the column
// recurrence by the first wave with the second wave's help (trailing_update64), then L, and Lh in both triangles,
// written out by all.  See diag_tile.
// dl: what the waves pass to one another; its counters zero on entry (with a barrier since).
// W, ok: where the tile's inverse and its verdict go, or nullptr (then, and for tiles of fewer than 64 columns, none
// is computed).
// beside(t): called in the full-tile case by the threads 128 .. 191 (t = 0 .. 63), which otherwise only wait, while
// the tile is being factored.
template <class Beside>
__device__ __forceinline__ void diag_rest(float (*T)[LDT], DiagLds &dl, float *L, uint16_t *Lh, int64_t n, int64_t j0, int cols, int r,
                                          float *W, int *ok, int limit, Beside beside, float *copy = nullptr)
{
    float(*const F)[LDF] = dl.F;
    int *const sync = dl.sync;
    const bool live = r < cols;
    bool mirrored = false;
    if (cols == NBMAX) {
        // Full tile: the lane keeps its row of L in registers (every index below is a constant after unrolling) and
        // writes each finished group of four columns to its row of T in LDS, where the other lanes find row c of L
        // when they come to column c (one wave: its LDS operations complete in program order, so a read sees an
        // earlier write without a barrier).  Inside the 4 x 4 corner the few values from other lanes' registers are
        // fetched with lane reads.  Lanes above the diagonal (r < c) compute values nobody uses.  Every entry takes
        // its terms in ascending k.
        if (r < 64) {
        float x[NBMAX], xn[NBMAX], t[4], tn[4] = {0.0f, 0.0f, 0.0f, 0.0f};      // xn = -x, see chol_panel_kernel
        f32x4 grp[4], q[3][4], ql[4];                                           // grp: the lane's row of the current group of 16 columns
#pragma unroll
        for (int i = 0; i < 4; ++i) grp[i] = *(const f32x4 *)&T[r][4 * i];
        auto request = [&](int b, int k4, f32x4(&o)[4]) __attribute__((always_inline)) {     // operands of step k4 of block b
#pragma unroll
            for (int j = 0; j < 4; ++j) o[j] = *(const f32x4 *)&T[4 * b + j][4 * k4];
        };
        auto step = [&](float(&acc)[4], int k4, const f32x4(&o)[4]) __attribute__((always_inline)) {   // 16 multiply-adds
#pragma unroll
            for (int kk = 0; kk < 4; ++kk)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[j] = __builtin_fmaf(xn[4 * k4 + kk], o[j][kk], acc[j]);
        };
        auto lane_value = [](float v, int l) __attribute__((always_inline)) {
            return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), l));
        };
#pragma unroll
        for (int j = 0; j < 4; ++j) t[j] = grp[0][j];
        unrolled<NBLK>([&](auto block) __attribute__((always_inline)) {
            constexpr int b = decltype(block)::value;
            constexpr int mine = own_steps(b), next = b + 1 < NBLK ? own_steps(b + 1) : 0;
            if (b >= 4 && b % 4 == 0) {
                // a new group of 16 columns, from the second wave: everything up to block b - 2 is out of it
                int polls = 0;
                while (__hip_atomic_load(sync + 1, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) < b / 4) {
                    if (++polls >= limit) {
                        __hip_atomic_store(sync + 2, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                        break;
                    }
                }
#pragma unroll
                for (int i = 0; i < 4; ++i) grp[i] = *(const f32x4 *)&F[r][4 * i];
#pragma unroll
                for (int j = 0; j < 4; ++j) t[j] = grp[0][j];
            }
            if (mine >= 2) step(t, b - 2, q[mine >= 2 ? mine - 2 : 0]);                         // held back: covers the latency of ql
            if (mine >= 1) step(t, b - 1, ql);
            if (next >= 1 && (b + 1) % 4 != 0) {
#pragma unroll
                for (int j = 0; j < 4; ++j) tn[j] = grp[(b + 1) % 4][j];
            }
            // operands of the next block's steps, all but the last: blocks first_k(b + 1) .. b - 1 are written
#pragma unroll
            for (int u = 0; u + 1 < next; ++u) request(b + 1, first_k(b + 1) + u, q[u]);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int c = 4 * b + j;
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int e = 0; e < j; ++e) t[j] = __builtin_fmaf(xn[4 * b + e], lane_value(x[4 * b + e], c), t[j]);
                const float d = lane_value(__builtin_sqrtf(t[j]), c);
                x[c] = r == c ? d : t[j] / d;
                xn[c] = -x[c];
                asm("" : "+v"(xn[c]));                                          // (or the negation is folded back into the multiply-adds)
                if (j + 2 < next) step(tn, first_k(b + 1) + j, q[j]);           // one step of the next block beside this column
            }
            f32x4 done;
#pragma unroll
            for (int j = 0; j < 4; ++j) done[j] = x[4 * b + j];
            *(f32x4 *)&T[r][4 * b] = done;
            // block b is final in LDS.  Every lane stores the same number (a store under a lane condition would cut the
            // chains into basic blocks), and without a release fence, which would wait for the operands requested ahead
            // as well: a wave's LDS operations are performed in the order it issues them, so whoever sees the counter
            // sees the block; the empty asm keeps the compiler from moving the store up.
            asm volatile("" ::: "memory");
            __hip_atomic_store(sync, b + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            if (b + 1 < NBLK) request(b + 1, b, ql);
            if (next >= 1 && (b + 1) % 4 != 0) {
#pragma unroll
                for (int j = 0; j < 4; ++j) t[j] = tn[j];
            }
        });
        // the mirror image into the upper part of the tile (Lh holds both triangles): entry (c, r) for c < r; the other
        // lanes write to the padding of their row (a store under a lane condition is a branch around it: 4k cycles for
        // the 63 of them)
#pragma unroll
        for (int c = 0; c < NBMAX - 1; ++c) *(c < r ? &T[c][r] : &T[r][NBMAX]) = x[c];
        } else if (r >= 192) {
            trailing_update64((uint32_t)(uintptr_t)(CYC_LDS const float *)&T[0][0], (uint32_t)(uintptr_t)(CYC_LDS float *)&F[0][0],
                              (uint32_t)(uintptr_t)(CYC_LDS int *)sync, r - 192, limit);
        } else if (r >= 128) {
            beside(r - 128);
        } else if (W) {
            inverse_follow64((uint32_t)(uintptr_t)(CYC_LDS const float *)&T[0][0], (uint32_t)(uintptr_t)(CYC_LDS float *)&dl.Y[0][0],
                             (uint32_t)(uintptr_t)(CYC_LDS int *)sync, r - 64, limit, W, ok);
        }
        mirrored = true;
        __syncthreads();
        if (__builtin_expect(sync[2] != 0, 0)) {
            // a bounded wait between the two waves ran out (it never should): NaNs instead of a factor that looks
            // like one, and no inverse
            for (int e = r; e < NBMAX * NBMAX; e += NT) T[e / NBMAX][e % NBMAX] = __builtin_nanf("");
            if (r == 0 && W) *ok = 0;
            __syncthreads();
        }
    } else {
        for (int c = 0; c < cols; ++c) {
            float t = 0.0f;
            if (live && r >= c) {
                t = chain(T[r][c], T[r], T[c], c);
                if (r == c) T[c][c] = __builtin_sqrtf(t);
            }
            __syncthreads();
            if (live && r > c) T[r][c] = t / T[c][c];
            __syncthreads();
        }
    }
    // mirror the factor into the upper part of the tile in LDS (Lh holds both triangles), then write the tile out
    if (live && !mirrored)
        for (int c = r + 1; c < cols; ++c) T[r][c] = T[c][r];
    __syncthreads();
    if (copy) {
        // a second copy of the tile as it stands in LDS, rows of 64 floats (see chol_panel_kernel, Dcopy)
#pragma unroll
        for (int i = 0; i < NBMAX * 16 / NT; ++i) {
            const int row = NT / 16 * i + (r >> 4);
            *(f32x4 *)(copy + row * NBMAX + 4 * (r & 15)) = *(const f32x4 *)&T[row][4 * (r & 15)];
        }
    }
    if (store_tile<true>(T, L + j0 * n + j0, Lh + j0 * n + j0, n, cols, cols, r)) return;
    if (live)
        for (int c = 0; c < cols; ++c) {
            L[(j0 + r) * n + j0 + c] = c <= r ? T[r][c] : 0.0f;
            Lh[(j0 + r) * n + j0 + c] = round_bf16(T[r][c]);
        }
}

// L_jj = CHOL(S_jj) for the tile at (j0, j0) with `cols` rows and columns.  S is read from Sm (row stride n: A itself
// for the first panel, L afterwards); L gets the factor below and on the diagonal and zero above it, Lh its bf16
// rounding in both triangles.  One workgroup of NT threads; thread r < 64 owns row r, the other waves only help to
// move and update the tile.  T (first 64 KB of LDS: a read reaches its word with the 16-bit offset field from one
// base register; further up every read needs an address register of its own) and Bs are the workgroup's LDS.
__device__ __forceinline__ void diag_tile(float (*T)[LDT], uint16_t (*Bs)[64], const float *Sm, float *L, uint16_t *Lh, int64_t n,
                                          int64_t j0, int cols, int64_t k0, int r, DiagLds &dl, float *W, int *ok, int limit)
{
    if (r < 3) dl.sync[r] = 0;            // (a barrier follows below, before anyone looks at them)
    // (both operands of the tile's own update are the rows j0 .. of Lh: the staged one, Lh[k0:j0, j0:j0+64], is their
    // mirror image, and the stationary fragments are read from it as well)
    TileProduct product;
    if (k0 < j0) product.request(Bs, Lh, n, j0, cols, k0, j0, j0, r, true);     // k0 < j0 only for full tiles, see launch_chol
    load_tile(T, Sm + j0 * n + j0, n, cols, cols, r);     // the whole square; what lies above the diagonal is not used
    if (k0 < j0) product.apply(T, Bs, r, Bs);
    else __syncthreads();
    diag_rest(T, dl, L, Lh, n, j0, cols, r, W, ok, limit, [](int) {});
}

__global__ __launch_bounds__(NT) void chol_diag_kernel(const float *Sm, float *L, uint16_t *Lh, int64_t n, int64_t j0, int cols,
                                                       int64_t k0, float *W, int *ok, int limit)
{
    __shared__ __attribute__((aligned(16))) struct {
        float T[NBMAX][LDT];          // S on entry, L as columns finish
        uint16_t Bs[KMAX][64];        // streamed operand of the tile's own update
        DiagLds dl;                   // between the waves of the factorisation
    } lds;
    diag_tile(lds.T, lds.Bs, Sm, L, Lh, n, j0, cols, k0, threadIdx.x, lds.dl, W, ok, limit);
}

// L_ij = TRSM(S_ij, L_jj) for all rows below the diagonal tile: row j1 + 64 * blockIdx.x + lane of the first wave; the
// other waves of the NT threads only help to move and update the tile.
// next_Sm != nullptr: the workgroup of the first 64 rows goes on to factor the next diagonal tile, (j1, j1), whose S is
// read from next_Sm: it produces the only part of that tile's update that is still missing, and a launch of its own
// for the tile would first wait for memory again.  That workgroup requests the tile's S and the operands of its
// update over the group's earlier panels with everything else, first thing; the three waves that would idle during
// the recurrence multiply them out (wave 1 rows 0 .. 31 of the tile, waves 2 and 3 sixteen rows each; one strip of
// sixteen rows per wave when the rows come through the inverse and the first wave is free).  Then the k range of
// this panel is added, straight from the solved rows in LDS, and the tile is factored; meanwhile two waves write this
// workgroup's own rows out.
// Win, okin: the inverse of L_jj and its verdict (see inverse_follow64), or nullptr.  When the verdict is good the
// workgroup of the first 64 rows, the one the next diagonal tile waits for, forms its rows as the product S W^T on the
// matrix cores in fp32 instead of running the recurrence; all other workgroups, which nothing waits for, keep the
// recurrence.  Wout, okout: where the inverse of the next diagonal tile and its verdict go when that tile rides along.
__global__ __launch_bounds__(NT) void chol_panel_kernel(const float *Sm, float *L, uint16_t *Lh, int64_t n, int64_t j0, int cols,
                                                        int64_t k0, const float *next_Sm, const float *__restrict__ Win,
                                                        const int *__restrict__ okin, float *Wout, int *okout, const float *Dcopy,
                                                        float *next_copy, int limit, int64_t k0_first, int ahead)
{
    // one block, D and X first (see diag_tile)
    __shared__ __attribute__((aligned(16))) struct {
        float D[NBMAX][LDT];          // L_jj
        float X[64][LDT];             // this workgroup's rows: S on entry, L as columns finish
        uint16_t Bs[KMAX][64];        // streamed operand of the tile's own update
        uint16_t Bs2[KMAX][64];       // streamed operand of the next diagonal tile's update
        DiagLds dl;                   // the next diagonal tile: between the waves of its factorisation (see diag_rest)
    } lds;
    auto &D = lds.D;
    auto &X = lds.X;
    auto &Bs = lds.Bs;
    auto &Bs2 = lds.Bs2;
    const int tid = threadIdx.x, lane = tid & 63;
    // ahead != 0: the last two workgroups of the launch work for the NEXT launch's first workgroup, the one that everything
    // waits for.  Its two tiles, rows j1 + 64 .. of the column blocks j1 and j1 + 64 (its own rows and the diagonal tile that
    // rides along with it), lose the terms of the group's panels left of this one here, in place in S, while this launch
    // runs; that workgroup then starts at k = j0 (its k0_first) instead of at the group's first column, with a quarter of
    // the operands to fetch and two k-steps of each product instead of up to fourteen.  (Per entry the terms are then
    // subtracted in two chains, not one.)  Nothing else in this launch reads or writes those two tiles.
    const int row_blocks = (int)gridDim.x - (ahead ? 2 : 0);
    if ((int)blockIdx.x >= row_blocks) {
        const int64_t row0 = j0 + cols + NBMAX, col0 = j0 + cols + ((int)blockIdx.x - row_blocks) * NBMAX;
        float *tile = L + row0 * n + col0;                                 // (S of a later group's panels lives in L)
        TileProduct product;
        TileLoad of_S;
        product.request(Bs, Lh, n, row0, NBMAX, k0, j0, col0, tid);
        of_S.request(tile, n, NBMAX, NBMAX, tid);
        of_S.place(X, tile, n, NBMAX, NBMAX, tid);
        product.apply(X, Bs, tid);
#pragma unroll
        for (int i = 0; i < NBMAX * 16 / NT; ++i) {
            const int r = NT / 16 * i + (tid >> 4);
            *(f32x4 *)(tile + (int64_t)r * n + 4 * (tid & 15)) = *(const f32x4 *)&X[r][4 * (tid & 15)];
        }
        return;
    }
    if (blockIdx.x == 0) k0 = k0_first;                                    // uniform (see above)
    if (tid < 3) lds.dl.sync[tid] = 0;
    const bool solver = tid < 64;                         // the wave that runs the recurrence
    // The rows of this workgroup through the inverse of L_jj?  W and its verdict are requested here with everything
    // else the kernel needs from memory; the verdict is looked at only where the rows are formed, so that nothing
    // waits for it on its own.
    const bool may_invert = blockIdx.x == 0 && cols == NBMAX && Win != nullptr;        // uniform over the workgroup
    int verdict = 0;
    f32x4 winv[10];                                       // this lane's 40 values of W: pieces (cb, q), q <= cb
    if (may_invert) {
        verdict = *okin;
        int p = 0;
#pragma unroll
        for (int cb = 0; cb < 4; ++cb)
#pragma unroll
            for (int q4 = 0; q4 <= cb; ++q4) winv[p++] = *(const f32x4 *)(Win + (cb * 4 + q4) * 256 + lane * 4);
    }
    const int64_t j1 = j0 + cols, row = j1 + (int64_t)blockIdx.x * 64 + lane;
    const bool live = solver && row < n;
    const int64_t first = j1 + (int64_t)blockIdx.x * 64;
    const int nrows = (int)(n - first < 64 ? n - first : 64);
    // L is zero above the diagonal, and the products of the matrix-multiply kernel have written S there (a group's window
    // starts at the group's first row): every workgroup clears the mirror image of its tile's place, the rows of the
    // panel against its own columns.  Over all panels and workgroups that is everything above the diagonal tiles (which
    // clear their own upper halves), and nothing writes there after the group's product, which precedes its panels.
    // (At the end of the workgroup's work: ahead of its loads these stores would sit in the same queue before them.)
    auto clear_mirror_place = [&](int t, int nth) __attribute__((always_inline)) {
        for (int i = t >> 6; i < cols; i += nth / 64)
            if ((t & 63) < nrows) L[(j0 + i) * n + first + (t & 63)] = 0.0f;
    };
    // ---- the next diagonal tile, first part: its S and the operands of the part of its update that does not involve
    // this panel are requested with everything else (their own LDS buffer, Bs2, so that they need not wait for Bs)
    const bool fused = next_Sm != nullptr && blockIdx.x == 0;          // uniform over the workgroup
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6), lq = lane & 15, g = lane >> 4;
    const int nks_e = fused ? (int)(j0 - k0) / 32 : 0;                 // k-steps of that tile's update that do not involve this panel
    f32x4 sv[4], accn[2][4];                                           // its S (this thread's pieces); its update: [slot][column tile]
    // The four 16-row strips of that update: slot si of this wave holds strip(si), or nothing (-1).  Beside the recurrence
    // the three other waves share them (wave 1 takes two).  When the rows may come through the inverse the first wave
    // is free as a rule and every wave takes one strip; should the verdict then be bad after all, the first wave takes
    // its strip after its recurrence.
    auto strip = [&](int si) __attribute__((always_inline)) {
        return may_invert ? (si == 0 ? w : -1) : (w == 1 ? si : (si == 0 && w >= 2 ? w : -1));
    };
    // rows `first_row` .. +count-1 of the streamed operand Lh[., j1 : j1+64] into Bs2 from row `to` on, 8 rows per copy,
    // the copies dealt out to `waves` waves of which this is number `me`
    auto copy_rows = [&](int64_t first_row, int to, int count, int me, int waves) __attribute__((always_inline)) {
        const uint32_t lds_base = (uint32_t)(uintptr_t)(CYC_LDS char *)&Bs2[0][0];
        for (int k = 8 * me; k < count; k += 8 * waves) {
            const uint32_t voff = (uint32_t)(lane >> 3) * (uint32_t)(n * 2) + (uint32_t)((lane & 7) ^ staged_swizzle(to + k)) * 16;
            const char *base = (const char *)(Lh + (first_row + k) * n + j1);
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                         :
                         : "s"(lds_base + (to + k) * 128), "v"(voff), "s"(base)
                         : "memory", "m0");
        }
    };
    if (fused) {
#pragma unroll
        for (int i = 0; i < 4; ++i) sv[i] = *(const f32x4 *)(next_Sm + (j1 + 16 * i + (tid >> 4)) * n + j1 + 4 * (tid & 15));
        if (nks_e > 0) {
            // (only the streamed operand, Lh[k0:j0, j1:j1+64]: the stationary one, the rows j1 .. j1+63 of Lh over the same k,
            // is its mirror image, and the transposing read that makes a streamed fragment of column block c makes the
            // stationary fragment of row block c out of the same words)
            copy_rows(k0, 0, 32 * nks_e, w, NT / 64);
        }
    }
    TileProduct product;
    // (the workgroup that goes on to the next diagonal tile finds its own rows of Lh over k0 .. j0 in Bs2, mirrored: what
    // is left to fetch are whole rows, and nothing on the path waits for a load of 64 separate cache lines)
    const bool rows_in_lds = fused && nks_e > 0;
    if (k0 < j0) product.request(Bs, Lh, n, first, nrows, k0, j0, j0, tid, rows_in_lds);
    TileLoad of_D, of_X;
    // (Dcopy: L_jj is read from there, rows of 64 floats, because a product launched since it was factored has written over
    // its place in L, which the last workgroup restores)
    const float *Dsrc = Dcopy ? Dcopy : L + j0 * n + j0;
    const int64_t ldD = Dcopy ? NBMAX : n;
    of_D.request(Dsrc, ldD, cols, cols, tid);
    of_X.request(Sm + first * n + j0, n, nrows, cols, tid);
    of_D.place(D, Dsrc, ldD, cols, cols, tid);
    of_X.place(X, Sm + first * n + j0, n, nrows, cols, tid);
    // (nks_e > 0 implies k0 < j0: apply waits for every copy of this wave, Bs2's included, before its barrier)
    if (k0 < j0) product.apply(X, Bs, tid, rows_in_lds ? Bs2 : nullptr);
    else __syncthreads();
    if (Dcopy && (int)blockIdx.x == row_blocks - 1) (void)store_tile<true>(D, L + j0 * n + j0, Lh + j0 * n + j0, n, cols, cols, tid);
    const bool by_inverse = may_invert && __builtin_amdgcn_readfirstlane(verdict) != 0;
#pragma unroll
    for (int si = 0; si < 2; ++si)
#pragma unroll
        for (int j = 0; j < 4; ++j) accn[si][j] = (f32x4){0, 0, 0, 0};
    // (lanes past the last row run along on the repeated last row: they take part in the barrier and in the tile
    // store below, and write nothing of their own)
    bool mirrored = false;
    if (cols == NBMAX) {
        if (by_inverse) {
            // X <- S W^T: wave w takes the rows 16w .. 16w+15 and all 64 columns.  A operand lane l: row 16w + l%16 of
            // S, k = 4 ks + l/16; B operand: W[16 cb + l%16][4 ks + l/16], zero for ks >= 4 (cb + 1); accumulator
            // register r of lane l: row 16w + 4 (l/16) + r, column 16 cb + l%16.  Each wave reads only its own rows
            // of X before it overwrites them.
            float sa[16];
#pragma unroll
            for (int ks = 0; ks < 16; ++ks) sa[ks] = X[16 * w + lq][4 * ks + g];
            f32x4 xo[4];
#pragma unroll
            for (int cb = 0; cb < 4; ++cb) xo[cb] = (f32x4){0, 0, 0, 0};
            // Between the MFMAs of this product (32 cycles of the matrix pipe each) run the k-steps of the next diagonal
            // tile's update over the group's earlier panels (second part, see below; this wave's strip is rows 16w ..):
            // they wait for their fragments from LDS, which the product does not need, and alone they took as long again
            // as the product.  One k-step per step of the product, its fragments read a step ahead.  (nks_e <= 14.)
            const bool early = fused && nks_e > 0;                              // uniform
            i32x4 f[2][5];                                                      // [parity of the k-step]: stationary, streamed x 4
            auto read_step = [&](int ks, i32x4(&dst)[5]) __attribute__((always_inline)) {
                dst[0] = staged_fragment(Bs2, ks, w, lq, g);
#pragma unroll
                for (int j = 0; j < 4; ++j) dst[1 + j] = staged_fragment(Bs2, ks, j, lq, g);
            };
            // (The usual numbers of such k-steps, none and two, have a copy of the loop each in which they are constants:
            // as conditions at run time they cut every step of the product into pieces that wait for their own reads.)
            auto product_loop = [&](auto steps_c) __attribute__((always_inline)) {
                constexpr int NE = decltype(steps_c)::value;                    // that many k-steps, or -1: nks_e of them
                auto has = [&](int ks) __attribute__((always_inline)) { return NE >= 0 ? ks < NE : early && ks < nks_e; };
                if (has(0)) read_step(0, f[0]);
#pragma unroll
                for (int ks = 0; ks < 16; ++ks) {
                    if (has(ks + 1)) read_step(ks + 1, f[(ks + 1) & 1]);
#pragma unroll
                    for (int cb = ks / 4; cb < 4; ++cb)
                        xo[cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(sa[ks], winv[cb * (cb + 1) / 2 + ks / 4][ks % 4], xo[cb], 0, 0, 0);
                    if (has(ks)) {
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            accn[0][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, f[ks & 1][0]), __builtin_bit_cast(bf16x8, f[ks & 1][1 + j]), accn[0][j], 0, 0, 0);
                    }
                }
            };
            if (!early) product_loop(std::integral_constant<int, 0>{});
            else if (nks_e == 2) product_loop(std::integral_constant<int, 2>{});
            else product_loop(std::integral_constant<int, -1>{});
#pragma unroll
            for (int cb = 0; cb < 4; ++cb)
#pragma unroll
                for (int r = 0; r < 4; ++r) X[16 * w + 4 * g + r][16 * cb + lq] = xo[cb][r];
        }
        if (solver && !by_inverse) {
        // The lane's row of S and of L in registers (constant indices after unrolling); the steps of StepList, the
        // rows of L_jj for a step requested from LDS two steps before it runs, since a lone wave has nobody else to
        // hide the LDS latency behind.
        float x[NBMAX], xn[NBMAX], t[4], tn[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        f32x4 sr[NBLK], q[3][4], qc[2][4];
#pragma unroll
        for (int i = 0; i < NBLK; ++i) sr[i] = *(const f32x4 *)&X[lane][4 * i];
        auto request = [&](int i) __attribute__((always_inline)) {              // operands of bulk step i
            if (STEPS.b[i] >= 0) {
#pragma unroll
                for (int j = 0; j < 4; ++j) q[i % 3][j] = *(const f32x4 *)&D[4 * STEPS.b[i] + j][4 * STEPS.k[i]];
            }
        };
        // (xn = -x: a multiply-add without a negated operand has a 4-byte encoding, which a lone wave issues faster)
        auto quarter = [&](float(&acc)[4], int i, int kk) __attribute__((always_inline)) {   // a quarter of bulk step i
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[j] = __builtin_fmaf(xn[4 * STEPS.k[i] + kk], q[i % 3][j][kk], acc[j]);
        };
        request(0);
        request(1);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            qc[0][j] = *(const f32x4 *)&D[j][0];
            t[j] = sr[0][j];
        }
        int i = 0;                                                              // the next bulk step
#pragma unroll
        for (int b = 0; b < NBLK; ++b) {
#pragma unroll
            for (int s = early_of(b); s < b; ++s) {                             // the block's bulk steps taken in turn
                request(i + 2);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) quarter(t, i, kk);
                ++i;
            }
            if (b + 1 < NBLK) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    qc[(b + 1) & 1][j] = *(const f32x4 *)&D[4 * (b + 1) + j][4 * (b + 1)];
                    tn[j] = sr[b + 1][j];
                }
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {                                       // the corner, column by column
                const bool paired = b + 1 < NBLK && j < early_of(b + 1);
                if (paired) request(i + 2);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int c = 0; c < j; ++c) t[j] = __builtin_fmaf(xn[4 * b + c], qc[b & 1][j][c], t[j]);
                Division dv;
                dv.phase0(t[j], qc[b & 1][j][j]);
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
                x[4 * b + j] = dv.phase3();
                xn[4 * b + j] = -x[4 * b + j];
                asm("" : "+v"(xn[4 * b + j]));                                  // (or the negation is folded back into the multiply-adds)
                __builtin_amdgcn_sched_barrier(0);
                if (paired) {
                    quarter(tn, i, 3);
                    ++i;
                }
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) t[j] = tn[j];
        }
#pragma unroll
        for (int c = 0; c < NBMAX; ++c) X[lane][c] = x[c];
        if (live) {
            // the mirror image of the rows, straight from the registers: consecutive lanes, consecutive addresses
            uint16_t *m = Lh + j0 * n + row;
#pragma unroll
            for (int c = 0; c < NBMAX; ++c) m[c * n] = round_bf16(x[c]);
        }
        }
        if (fused && nks_e > 0 && (!solver || may_invert) && !by_inverse) {
            // ---- the next diagonal tile, second part: the k-steps over the group's earlier panels, by the three waves
            // beside the recurrence, or by all four after it when the inverse turned out unusable (when the rows come
            // through the inverse these k-steps run between the MFMAs of that product, above).  (Their operands have
            // arrived: requested first thing and waited for before the barrier that precedes the update of this
            // workgroup's own tile.)
            // Both operands out of Bs2 (see above); the fragments of the next k-step are read before the current ones are
            // multiplied.  (nks_e is even.)
            const int s0 = strip(0), s1 = strip(1);
            i32x4 f[2][6];                                                       // [parity]: stationary of slot 0 and 1, streamed x 4
            auto read_step = [&](int ks, i32x4(&dst)[6]) __attribute__((always_inline)) {
                if (s0 >= 0) dst[0] = staged_fragment(Bs2, ks, s0, lq, g);
                if (s1 >= 0) dst[1] = staged_fragment(Bs2, ks, s1, lq, g);
#pragma unroll
                for (int j = 0; j < 4; ++j) dst[2 + j] = staged_fragment(Bs2, ks, j, lq, g);
            };
            auto multiply = [&](const i32x4(&src)[6]) __attribute__((always_inline)) {
#pragma unroll
                for (int si = 0; si < 2; ++si)
                    if ((si == 0 ? s0 : s1) >= 0) {
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            accn[si][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, src[si]), __builtin_bit_cast(bf16x8, src[2 + j]), accn[si][j], 0, 0, 0);
                    }
            };
            read_step(0, f[0]);
            for (int ks = 0; ks < nks_e; ks += 2) {
                read_step(ks + 1, f[1]);
                multiply(f[0]);
                if (ks + 2 < nks_e) read_step(ks + 2, f[0]);
                multiply(f[1]);
            }
        }
        mirrored = !by_inverse;                            // (the recurrence writes the mirror image from its registers)
    } else if (solver) {
        for (int c = 0; c < cols; ++c) X[lane][c] = chain(X[lane][c], X[lane], D[c], c) / D[c][c];
    }
    __syncthreads();
    // In the workgroup that goes on to the next diagonal tile two waves have nothing to do while that tile is factored:
    // they write this workgroup's rows out then (diag_rest below), off the path.  (There the tile is full and every
    // pointer aligned: the host fuses under those conditions only.)
    const bool deferred = fused && cols == NBMAX;
    const bool stored = deferred || store_tile<false>(X, L + first * n + j0, Lh + first * n + j0, n, nrows, cols, tid);
    if (!deferred && by_inverse && nrows == 64 && n % 8 == 0 && (uintptr_t)Lh % 16 == 0) {
        store_mirror<NT>(X, Lh + j0 * n + first, n, tid);
        mirrored = true;
    }
    if (!deferred && live && !(stored && mirrored))
        for (int c = 0; c < cols; ++c) {
            const float v = X[lane][c];
            const uint16_t h = round_bf16(v);
            if (!stored) {
                L[row * n + j0 + c] = v;
                Lh[row * n + j0 + c] = h;
            }
            if (!mirrored) Lh[(j0 + c) * n + row] = h;
        }
    if (!fused) clear_mirror_place(tid, NT);
    if (fused) {
        // ---- the next diagonal tile, third part: the k range of this panel.  Its operands are the rows this
        // workgroup has just solved, still in X: both are the same fragments of X rounded to bfloat16 (the streamed
        // operand is the mirror image of the stationary one), so nothing has to come back from memory.
        auto fragment = [&](int q, int u) __attribute__((always_inline)) {     // row 16 q + lq, k = 32 u + 8 g .. +7 of the panel
            const float *p = &X[16 * q + lq][32 * u + 8 * g];
            const f32x4 lo = *(const f32x4 *)p, hi = *(const f32x4 *)(p + 4);
            i32x4 f;
            f[0] = (int)pack_bf16(lo[0], lo[1]);
            f[1] = (int)pack_bf16(lo[2], lo[3]);
            f[2] = (int)pack_bf16(hi[0], hi[1]);
            f[3] = (int)pack_bf16(hi[2], hi[3]);
            return f;
        };
#pragma unroll
        for (int i = 0; i < 4; ++i) *(f32x4 *)&D[16 * i + (tid >> 4)][4 * (tid & 15)] = sv[i];      // S into the tile (D is free)
        if (may_invert) {
            // (every wave has one strip, its own: the same code without the conditions, which are not constants and cut it
            // into pieces that each wait for their own reads)
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                i32x4 bq[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) bq[j] = fragment(j, u);
                const i32x4 aq = fragment(w, u);
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    accn[0][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, aq), __builtin_bit_cast(bf16x8, bq[j]), accn[0][j], 0, 0, 0);
            }
            __syncthreads();
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int r = 0; r < 4; ++r) D[16 * w + 4 * g + r][16 * j + lq] -= accn[0][j][r];
        } else {
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                i32x4 bq[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) bq[j] = fragment(j, u);
#pragma unroll
                for (int si = 0; si < 2; ++si)
                    if (strip(si) >= 0) {
                        const i32x4 aq = fragment(strip(si), u);
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            accn[si][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, aq), __builtin_bit_cast(bf16x8, bq[j]), accn[si][j], 0, 0, 0);
                    }
            }
            __syncthreads();
            // accumulator register r of lane l is row 4 (l/16) + r, column l%16 of its 16 x 16 tile
#pragma unroll
            for (int si = 0; si < 2; ++si)
                if (strip(si) >= 0) {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
#pragma unroll
                        for (int r = 0; r < 4; ++r) D[16 * strip(si) + 4 * g + r][16 * j + lq] -= accn[si][j][r];
                }
        }
        __syncthreads();
        diag_rest(D, lds.dl, L, Lh, n, j1, NBMAX, tid, Wout, okout, limit, [&](int t) __attribute__((always_inline)) {
            // this workgroup's own rows, deferred above
            store_tile<false, 64>(X, L + first * n + j0, Lh + first * n + j0, n, nrows, cols, t);
            if (by_inverse) store_mirror<64>(X, Lh + j0 * n + first, n, t);
            clear_mirror_place(t, 64);
        }, next_copy);
    }
}

}  // namespace

int64_t chol_workspace_bytes(int64_t n, int64_t nb)
{
    // one inverse and one verdict per full diagonal tile of 64 (see inverse_follow64)
    // and one tile of 64 x 64 floats (see launch_chol: the first diagonal tile of a group)
    return nb == NBMAX && n >= 2 * NBMAX ? (n / NBMAX) * (int64_t)(W_FLOATS * sizeof(float) + sizeof(int)) + 16 + NBMAX * NBMAX * (int64_t)sizeof(float) : 0;
}

hipError_t launch_chol(const void *A_, void *L_, void *Lh_, int64_t n, int64_t nb, void *workspace, hipStream_t s)
{
    const float *A = (const float *)A_;
    float *L = (float *)L_;
    uint16_t *Lh = (uint16_t *)Lh_;
    if (nb < 1 || nb > NBMAX || n < 1 || n > (1 << 22)) return hipErrorInvalidValue;
    // the inverses of the full diagonal tiles and their verdicts, tile after tile (nullptr: none are computed)
    float *Wall = chol_workspace_bytes(n, nb) > 0 ? (float *)workspace : nullptr;
    int *okall = Wall ? (int *)(Wall + (n / NBMAX) * W_FLOATS) : nullptr;
    auto W_of = [&](int64_t j, int c) { return Wall && c == NBMAX ? Wall + j / NBMAX * W_FLOATS : (float *)nullptr; };
    auto ok_of = [&](int64_t j, int c) { return Wall && c == NBMAX ? okall + j / NBMAX : (int *)nullptr; };
    float *tile_copy = Wall ? (float *)(((uintptr_t)(okall + n / NBMAX) + 15) & ~(uintptr_t)15) : nullptr;
    // One product per panel would have only nb columns and all earlier tiles as its k range: a few workgroups
    // walking a long k loop.  So the panels are taken in groups of GROUP: at the first panel of a group one product
    // covers the columns of the whole group against all tiles left of the group; the later panels of the group
    // then only add the terms of the group's own earlier panels (k range at most (GROUP - 1) * nb).  The terms of a
    // sum are the paper's; they are merely added in two chains instead of one.
    constexpr int GROUP = 8;          // measured at n = 8192: 4: 4.74 ms, 8: 4.22, 12: 4.26, 16: 4.33; with the side stream below 4: 4.11, 8: 3.99
    auto product = [&](int64_t r0, int64_t c0, int64_t ncols, int64_t k0, int64_t k1, const float *src, hipStream_t on) {
        Problem p;                        // L[r0:, c0:c0+ncols] = src[r0:, c0:c0+ncols] - Lh[r0:, k0:k1] * Lh[k0:k1, c0:c0+ncols]
        p.A = Lh + r0 * n + k0;           // finished factor, rows r0.., columns k0..k1
        p.lda = n;
        p.B = Lh + k0 * n + c0;           // its transpose, by mirror storage
        p.ldb = n;
        p.C = L + r0 * n + c0;
        p.Cin = src + r0 * n + c0;
        p.ldc = n;
        p.batch = 1;
        p.M = n - r0;
        p.K = k1 - k0;
        p.N = ncols;
        p.strideA = p.strideB = p.strideC = 0;
        p.i8 = false;
        const int tile = choose_mfma_tile(p);
        return tile ? launch_mfma(p, tile, 16, on) : launch_generic(p, on);
    };
    bool diag_done = false;           // the diagonal tile of this panel was factored by the rows kernel of the panel before
    int64_t prepared_from = -1;       // >= 0: the launch before took the k range [k0, prepared_from) out of this launch's first workgroup's tiles
    bool copied = false;              // ... across a group boundary: L_jj is to be read from the copy in the workspace
    // the side stream is worth its events only when there are at least three groups
    SideStreamLock side_lock;
    SideStream *side = n > 2 * GROUP * nb ? side_lock.acquire() : nullptr;
    int64_t ahead = -1;               // first column of the group whose product over the groups before the last is on the side stream
    bool unjoined = false;            // work is on the side stream that the caller's stream does not wait for yet
    // a refused launch ends the call: what is already on the side stream is first joined back into the caller's stream
    auto fail = [&](hipError_t e) {
        if (unjoined) (void)hipStreamWaitEvent(s, side->join[0], 0);
        return e;
    };
    for (int64_t j0 = 0; j0 < n; j0 += nb) {
        const int cols = (int)(j0 + nb <= n ? nb : n - j0);
        const int64_t j1 = j0 + cols;
        const int64_t g0 = j0 / (GROUP * nb) * (GROUP * nb);      // first column of this panel's group
        const float *Sm = A;                                      // where S of this panel is read from
        if (j0 == g0 && g0 > 0) {
            const int64_t gcols = g0 + GROUP * nb <= n ? GROUP * nb : n - g0;
            if (ahead == g0) {
                // the part over the groups before the last was multiplied out on the side stream while the last group
                // was being factored; what is left is the k range of that group
                if (unjoined) {
                    if (hipError_t e = hipStreamWaitEvent(s, side->join[0], 0); e != hipSuccess) return fail(e);
                    unjoined = false;
                }
                // (when the group's first diagonal tile rode along with the last panel, this product writes over its place
                // in L: a copy of the tile is kept in the workspace, see below)
                if (hipError_t e = product(g0, g0, gcols, g0 - GROUP * nb, g0, L, s); e != hipSuccess) return fail(e);
            } else {
                if (hipError_t e = product(g0, g0, gcols, 0, g0, A, s); e != hipSuccess) return fail(e);
            }
            // The product for the NEXT group over everything left of this group does not depend on this group: it goes
            // to the side stream now and runs on the compute units that the tile kernels of this group (at most one
            // workgroup per 64 rows) leave idle.  Per entry the terms are then subtracted in two chains, not one.
            const int64_t g1 = g0 + GROUP * nb;
            if (side && g1 < n) {
                const int64_t ncols = g1 + GROUP * nb <= n ? GROUP * nb : n - g1;
                if (hipError_t e = hipEventRecord(side->fork, s); e != hipSuccess) return fail(e);
                if (hipError_t e = hipStreamWaitEvent(side->stream, side->fork, 0); e != hipSuccess) return fail(e);
                const hipError_t pe = product(g1, g1, ncols, 0, g0, A, side->stream);
                // whatever reached the side stream is covered by the join event, also when the product was refused
                if (hipError_t e = hipEventRecord(side->join[0], side->stream); e != hipSuccess) return fail(e);
                unjoined = true;
                if (pe != hipSuccess) return fail(pe);
                ahead = g1;
            }
        }
        if (g0 > 0) Sm = L;
        // the terms of the group's own earlier panels: multiplied out by the tile kernels themselves where they can
        // (full 64-column tiles with 16-byte aligned rows of Lh), else by a product of their own
        int64_t k0 = j0;                                          // k range [k0, j0) left to the tile kernels
        if (j0 > g0) {
            if (nb == NBMAX && cols == NBMAX && n % 8 == 0 && (uintptr_t)Lh % 16 == 0 && j0 - g0 <= KMAX) {
                k0 = g0;
            } else {
                if (hipError_t e = product(j0, j0, cols, g0, j0, Sm, s); e != hipSuccess) return fail(e);
                Sm = L;
            }
        }
        if (!diag_done) {
            hipError_t e = launch_kernel(chol_diag_kernel, dim3(1), dim3(NT), s, Sm, L, Lh, n, j0, cols, k0, W_of(j0, cols), ok_of(j0, cols), wait_limit());
            if (e != hipSuccess) return fail(e);
        }
        diag_done = false;
        if (j1 < n) {
            // the next diagonal tile rides along when it is a full tile of the same group whose whole update the tile
            // kernels do themselves: its k range [g0, j1) then starts where this panel's starts
            // (the first diagonal tile of the next group, too, once that group's product over everything left of this
            // group is in, or when nothing lies left of this group: the tile's remaining k range is this group, which is
            // what the rows kernel has at hand)
            const bool next_group = j1 == g0 + GROUP * nb && (ahead == j1 || g0 == 0) && tile_copy != nullptr && j1 + NBMAX < n;
            const bool fuse = k0 == g0 && nb == NBMAX && cols == NBMAX && j1 + NBMAX <= n && (j1 < g0 + GROUP * nb || next_group) &&
                              n % 8 == 0 && (uintptr_t)Lh % 16 == 0 && (uintptr_t)A % 16 == 0 && (uintptr_t)L % 16 == 0 &&
                              j0 - g0 <= KMAX;
            if (fuse && next_group && unjoined) {
                if (hipError_t e = hipStreamWaitEvent(s, side->join[0], 0); e != hipSuccess) return fail(e);
                unjoined = false;
            }
            // (see `ahead` in the kernel: the next launch is a fused one of this group, not its last, S is in L, and there is
            // something left of this panel to take out)
            const bool prepare = fuse && g0 > 0 && j0 > g0 && j1 + NBMAX < g0 + GROUP * nb && j1 + 2 * NBMAX <= n;
            if (prepared_from >= 0 && !(fuse && k0 == g0 && prepared_from == j0 - NBMAX)) return fail(hipErrorUnknown);
            const int64_t k0_first = prepared_from >= 0 ? prepared_from : k0;
            hipError_t e = launch_kernel(chol_panel_kernel, dim3((unsigned)((n - j1 + 63) / 64 + (prepare ? 2 : 0))), dim3(NT), s, Sm, L, Lh, n, j0, cols, k0,
                               fuse ? (g0 > 0 ? (const float *)L : A) : (const float *)nullptr, (const float *)W_of(j0, cols),
                               (const int *)ok_of(j0, cols), fuse ? W_of(j1, NBMAX) : (float *)nullptr, fuse ? ok_of(j1, NBMAX) : (int *)nullptr,
                               copied ? (const float *)tile_copy : (const float *)nullptr, fuse && next_group ? tile_copy : (float *)nullptr, wait_limit(),
                               k0_first, prepare ? 1 : 0);
            if (e != hipSuccess) return fail(e);
            prepared_from = prepare ? j0 : -1;
            diag_done = fuse;
            copied = fuse && next_group;
        }
    }
    return hipSuccess;
}

}  // namespace cyc
