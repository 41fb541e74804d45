/* cyclotron_mm.h -- C ABI of the MI355X (gfx950) weight-stationary recurrence matmul.
 *
 * The operation is the weight-stationary program of the Cyclotron paper
 * (section "Space-time Mappings of Dataflow Recurrences"; per-cell programs in
 * the per-PE figure): a grid of cells (i,k) latches [i,k]_W <- A_ik once; for
 * every time step j the north boundary injects B_kj, B moves down the i axis
 * unchanged, and each cell computes
 *        [i,k]_C <- [i,k-1]_C + [i,k]_W * [i,k]_B ,   [i,-1]_C = 0,
 * handing the partial sum east along k until the last column emits
 *        C_ij <- [i,k_end]_C .
 * The value that leaves the grid is C_ij = sum_k A_ik B_kj (the paper's
 * matrix-multiply recurrence, "Explicit Reduction Dimensions" form).
 *
 * All pointers are DEVICE pointers owned by the caller; the library keeps no
 * reference to them after return.  Work is enqueued on `stream` (a hipStream_t
 * passed as void*; NULL = the default stream); no call synchronises the stream,
 * and none synchronises the device except the rare growth of a workspace
 * described below.  Functions return a cyc_status and never throw or abort.
 * Every argument check, and every resource a call needs, is settled before the
 * first launch: a status other than CYC_OK and CYC_ERR_LAUNCH means nothing
 * has been enqueued.  CYC_ERR_LAUNCH means the HIP runtime refused a launch;
 * for the calls that enqueue several kernels (k in space, triangular solve,
 * Cholesky) earlier kernels of the same call then remain enqueued and the
 * outputs are undefined.
 *
 * State the library keeps (all of it per process, created on first use, kept
 * until the process ends, guarded by locks; calls from several host threads
 * on different streams are safe):
 *   - the kernel forced through cyc_force_kernel() / CYC_FORCE_KERNEL;
 *   - for cyc_recurrence_matmul on problems mapped with k in space and for
 *     cyc_recurrence_trsm and cyc_recurrence_cholesky with tiles of 64 rows
 *     (see below): one workspace of
 *     device memory per (device, stream), allocated with hipMalloc at the
 *     first such call on that stream and replaced by a larger one (hipFree +
 *     hipMalloc, which waits for the device) when a later call needs more.
 *     A call that cannot get it returns CYC_ERR_WORKSPACE.  No other entry
 *     point allocates device memory;
 *   - for cyc_recurrence_cholesky with n > 16 nb: one extra stream and a few
 *     events per device (see there); callers that use it are serialised on
 *     the host by a lock for the duration of the enqueueing.
 *
 * Layout: A is M x K, B is K x N, C is M x N, dense row-major with the row
 * length as leading dimension: A_ik = A[i*K+k], B_kj = B[k*N+j],
 * C_ij = C[i*N+j].  C is overwritten (the chain starts from 0); C must not
 * overlap A or B.
 *
 * Element types (cyc_dtype):
 *   CYC_BF16_F32  A,B bfloat16; products exact, partial sums fp32; C fp32.
 *                 The summation order over k is a fixed function of the shape,
 *                 the alignment of the operands and the kernel in force: the
 *                 same call gives bit-identical results every time, with no
 *                 atomic adds anywhere.  It is not the strictly sequential
 *                 order of the cell chain but agrees with it to within fp32
 *                 rounding of a K-term sum.
 *   CYC_I8_I32    A,B int8; partial sums int32, wrapping modulo 2^32; C int32.
 *                 Bit-exact for any summation order.
 *
 * Degenerate extents: M == 0, N == 0 or batch == 0 do nothing and return
 * CYC_OK; K == 0 fills C with zeros (the initial value of every chain).
 * Any M, K, N >= 1 and any batch >= 1 whose element counts fit (each of
 * M*K, K*N, M*N and the batched spans below 2^46) is accepted.  The fast paths need
 * 16-byte aligned base pointers, batch strides and rows of A and B (K and N
 * multiples of 8 for bfloat16, of 16 for int8) but no particular multiples
 * otherwise; anything else runs on a slower shape-agnostic kernel.
 *
 * Kernel families and when the dispatcher picks them:
 *   narrow   N <= 16, many rows: A streamed once from memory, B resident.
 *   narrowm  M <= 32, B of at least a mebibyte: B streamed once, the rows of
 *            A pass over it ((j,k) in space).
 *   mfmak    unbatched, at most 64 output blocks of 128 x 128, K >= 4096: k in
 *            space; k-slices on different workgroups leave partial sums in the
 *            workspace and a second kernel adds them in ascending slice order.
 *   mfma256 / mfma128  everything else with aligned rows.
 *   generic  the rest.
 */
#ifndef CYCLOTRON_MM_H
#define CYCLOTRON_MM_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    CYC_BF16_F32 = 0,
    CYC_I8_I32 = 1
} cyc_dtype;

typedef enum {
    CYC_OK = 0,
    CYC_ERR_NULL = 1,    /* a required pointer is NULL while its extent is not empty */
    CYC_ERR_SHAPE = 2,   /* negative extent, negative stride, element count overflow, or an argument out of its documented range */
    CYC_ERR_DTYPE = 3,   /* dtype is not a cyc_dtype */
    CYC_ERR_ALIAS = 4,   /* C overlaps A or B */
    CYC_ERR_LAUNCH = 5,  /* the HIP runtime refused a launch */
    CYC_ERR_WORKSPACE = 6 /* the workspace a call needs could not be allocated, or exceeds the fixed one */
} cyc_status;

/* One grid: C (M x N) <- A (M x K) streamed against B (K x N).
 * A, B: device, read only.  C: device, written.  stream: hipStream_t or NULL. */
int cyc_recurrence_matmul(const void *A, const void *B, void *C,
                          int64_t M, int64_t K, int64_t N,
                          int dtype, void *stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc): the same operation, kernels and results as cyc_recurrence_matmul, but a problem that the
 * dispatcher maps with k in space keeps its partial products in a fixed 32 MiB array that is part of the library's
 * device image (every GPU the library runs on holds its own copy until the process ends) instead of the
 * per-stream workspace.  The call allocates and frees nothing.  A problem whose partial products
 * (k-slices x M x N x 4 bytes) exceed the array returns CYC_ERR_WORKSPACE with nothing enqueued; problems served by
 * the other kernel families need no workspace and always run.  All calls on one GPU share that GPU's array: calls
 * whose k-in-space work overlaps in time on one GPU (different streams) race and give undefined results; calls on
 * one stream are ordered and safe.  Nothing in the array needs to be cleared between calls: every element a call
 * reads it has written before. */
int cyc_recurrence_matmul_noalloc(const void *A, const void *B, void *C,
                                  int64_t M, int64_t K, int64_t N,
                                  int dtype, void *stream);

/* `batch` independent grids, each with its own stationary A (not part of the
 * paper; the narrow-stream workload has one weight matrix per batch element).
 * Element b uses A + b*strideA, B + b*strideB, C + b*strideC, strides counted
 * in elements of the respective type.  strideA or strideB may be 0 (operand
 * shared by all grids); strideC must be >= M*N when batch > 1. */
int cyc_recurrence_matmul_batched(const void *A, const void *B, void *C,
                                  int64_t batch, int64_t M, int64_t K, int64_t N,
                                  int64_t strideA, int64_t strideB, int64_t strideC,
                                  int dtype, void *stream);

/* Tiled forward solve of the lower-triangular system  L X = B  with nrhs right-hand sides
 * (paper: "Representative recurrences", triangular solve; "Multiple Iteration Spaces", tiled form
 *     X_I = TRSM(L_II, B_I - sum_{J<I} GEMM(L_IJ, X_J))  over tiles of nb rows).
 * The GEMMs are the matrix-multiply recurrence above with L_IJ as the stationary operand and the solved
 * tile X_J streamed: bfloat16 operands, fp32 partial sums.  A solved tile therefore enters them rounded
 * to bfloat16 (nearest even); inside a tile the solve runs in fp32 on the unrounded values, in one of two
 * ways.  By substitution: t = fma(-L_rj, x_j, t) for j ascending, then one IEEE division by L_rr.  Or, for
 * tiles of 64 rows whose diagonal tile L_II is well conditioned (||L_II^-1||_1 ||L_II||_1 <= 8, decided on
 * the device from L alone), as the product L_II^-1 R_I in fp32, L_II^-1 itself being computed by that
 * substitution; its result differs from the substitution's by fp32 rounding, within
 * 64 * 2^-24 * (kappa^2 + kappa) * max|X_I| for kappa = || |L_II^-1| |L_II| ||_inf.  Either way the result is
 * the same on every call.  nb is part of the result: it fixes where X is rounded.
 *
 * L:  device, read only, n x n bfloat16 row-major; only the diagonal and the entries below it are used
 *     (what lies above the diagonal may hold anything, NaN included).
 * B:  device, read only, n x nrhs fp32 row-major.
 * X:  device, written, n x nrhs fp32 row-major: the solution.  Also used as the running right-hand side
 *     while the call is in flight.
 * Xh: device, written, n x nrhs bfloat16 row-major: X rounded to bfloat16, the values the GEMMs consumed.
 * nb: tile size, 1 <= nb <= 128.  The MFMA kernels serve the GEMMs when n, nrhs and nb are multiples of 8
 *     and the pointers are 16-byte aligned; otherwise a slower shape-agnostic kernel does.
 * stream: hipStream_t or NULL.  The call enqueues a sequence of kernels on it and returns.  With nb == 64,
 *     nrhs a multiple of 8 below 2^24, n a multiple of 8 below 2^26 and 16-byte aligned L, X, Xh it keeps the inverses of the diagonal
 *     tiles (16 KiB per 64 rows) and a second copy of the tiles of L next to the diagonal in the order the
 *     kernels read them (56 KiB per 64 rows) in the workspace that the library holds per device and stream (allocated or
 *     grown on the call that first needs it, as for cyc_recurrence_matmul); otherwise it allocates nothing.
 *     n == 0 or nrhs == 0: CYC_OK, nothing done.  A zero on the diagonal
 *     gives infinities or NaNs as IEEE division does, not an error.  Inside the kernels, waves hand solved rows
 *     to one another through LDS with bounded waits; a wait that ever ran out would leave NaN in X and Xh (in
 *     the last tile of the affected panel, and in every row solved after it) rather than plausible wrong values.
 * Errors (nothing enqueued): CYC_ERR_NULL, CYC_ERR_SHAPE (negative or overflowing extents, nb out of
 * range), CYC_ERR_ALIAS (X or Xh overlaps L, B or each other), CYC_ERR_WORKSPACE (the workspace could not be
 * allocated).  CYC_ERR_LAUNCH: see the top of this file. */
int cyc_recurrence_trsm(const void *L, const void *B, void *X, void *Xh,
                        int64_t n, int64_t nrhs, int64_t nb, void *stream);

/* Tiled Cholesky factorisation  A = L L^T  of a symmetric positive definite matrix, L lower triangular
 * (paper: "Representative recurrences", Cholesky; "Cholesky Recurrence", tiled form: for every panel j
 *     L_jj = CHOL(A_jj - sum_{k<j} SYRK(L_jk)),   L_ij = TRSM(A_ij - sum_{k<j} GEMM(L_ik, L_jk), L_jj)  for i > j,
 * over tiles of nb rows and columns).  The SYRKs and GEMMs are the matrix-multiply recurrence above (bfloat16
 * operands, fp32 partial sums; GEMM(X, Y) = X Y^T): a finished tile therefore enters them rounded to bfloat16
 * (nearest even).  CHOL and TRSM run the scalar recurrence inside the tile column in fp32 on unrounded values
 * (t = fma(-L_rk, L_ck, t) for k ascending, then an IEEE square root on the diagonal, an IEEE division below it).
 * One exception, with nb == 64 and n >= 128: the 64 rows right below a diagonal tile, which the next diagonal tile
 * waits for, are formed as the fp32 product S_ij L_jj^-T when L_jj is well conditioned (||L_jj^-1||_1 ||L_jj||_1 <= 8,
 * decided on the device from L_jj alone; L_jj^-1 computed by substitution beside the factorisation of the tile).
 * They differ from the recurrence's by fp32 rounding, within 64 * 2^-24 * (kappa^2 + kappa) * max|L_ij| for
 * kappa = || |L_jj^-1| |L_jj| ||_inf; the result is the same on every call.
 * nb is part of the result: it fixes where L is rounded.
 *
 * A:  device, read only, n x n fp32 row-major.  Entries above the diagonal outside the diagonal tiles are never
 *     read; those inside a diagonal tile may be read but do not influence the result (NaN allowed).
 * L:  device, written, n x n fp32 row-major: the factor on and below the diagonal, zero above.  Also holds the
 *     updated panels while the call is in flight.
 * Lh: device, written, n x n bfloat16 row-major: L rounded to bfloat16, the values the SYRKs and GEMMs consumed,
 *     with both triangles filled: Lh[r][c] = Lh[c][r] = bf16(L[max(r,c)][min(r,c)]).
 * nb: tile size, 1 <= nb <= 64.  The MFMA kernels serve the updates when n and nb are multiples of 8 and the
 *     pointers are 16-byte aligned; otherwise a slower shape-agnostic kernel does.
 * stream: hipStream_t or NULL.  The call enqueues a sequence of kernels on it and returns.  With nb == 64 and
 *     n >= 128 it keeps the inverses of the diagonal tiles (16 KiB per 64 rows) and a copy of one diagonal tile (16 KiB)
 *     in the workspace that the library holds per device and stream (allocated or grown on the call that first needs it); otherwise it allocates no
 *     device memory.  For n > 16 nb part of the work is enqueued on a second stream that the library creates per device
 *     on first use (default priority, kept until the process ends) and that is forked from and joined back into
 *     `stream` with events inside the call: all of the call's work is ordered after what was on `stream` before
 *     and before what is enqueued on it afterwards; calls that use the second stream are serialised on the host
 *     by a lock.  n == 0: CYC_OK, nothing done.  A matrix that is not positive definite gives NaNs (square root
 *     of a negative number), not an error.
 * Errors (nothing enqueued): CYC_ERR_NULL, CYC_ERR_SHAPE (negative or too large n, nb out of range, A or L not
 * 4-byte or Lh not 2-byte aligned), CYC_ERR_ALIAS (A, L, Lh overlap one another), CYC_ERR_WORKSPACE (the workspace
 * could not be allocated).  CYC_ERR_LAUNCH: see the top of
 * this file; work already on the second stream is joined back into `stream` before the call returns. */
int cyc_recurrence_cholesky(const void *A, void *L, void *Lh, int64_t n, int64_t nb, void *stream);

/* Attention by the tile recurrence of the paper's "FlashAttention-2 Recurrence": per query a running
 * maximum, running sum and running output over tiles of keys; the result is
 *     O_i. = sum_j softmax_j(Q_i. K_j.^T / sqrt(d)) V_j.      (no mask).
 * `batch` independent problems (e.g. batch x heads), stored one after the other.
 *
 * Q: device, read only, batch x N x d bfloat16 row-major.  K, V: device, read only, batch x M x d bfloat16.
 * O: device, written, batch x N x d fp32 row-major.  All pointers 16-byte aligned.
 * d must be 64 or 128; N, M >= 1 arbitrary (M * d < 2^31).  Scores, maxima, sums and outputs are fp32; the
 * exponentials enter the product with V, and their running sum, rounded to bfloat16.  stream: hipStream_t or NULL; asynchronous,
 * allocates nothing.  batch == 0 or N == 0: CYC_OK, nothing done.
 * Errors (nothing enqueued): CYC_ERR_NULL, CYC_ERR_SHAPE (negative extents, M == 0 with N > 0, unsupported d,
 * misaligned pointers, batch > 65535, sizes out of range), CYC_ERR_ALIAS (O overlaps Q, K or V), CYC_ERR_LAUNCH. */
int cyc_recurrence_attention(const void *Q, const void *K, const void *V, void *O,
                             int64_t batch, int64_t N, int64_t M, int64_t d, void *stream);

/* Human-readable name of a cyc_status (static storage, never NULL). */
const char *cyc_status_string(int status);

/* Library version: major*10000 + minor*100 + patch. */
int cyc_version(void);

/* Name of the kernel family the dispatcher would pick for this problem
 * ("mfma256", "mfma128", "mfmak", "narrow", "narrowm", "generic", "zero", "none", or the forced one); static storage.
 * Host only; enqueues nothing.  Pointers are only inspected for alignment. */
const char *cyc_kernel_name(const void *A, const void *B, const void *C,
                            int64_t batch, int64_t M, int64_t K, int64_t N,
                            int64_t strideA, int64_t strideB, int64_t strideC, int dtype);

/* Testing and benchmarking aid: from now on, in every thread, use the named kernel family (generic | mfma256 |
 * mfma128 | mfma256x32 | mfma128x32 | mfmak | narrow | narrowm) wherever it supports the problem; NULL or "" gives the
 * choice back to the dispatcher.  The x32 kernels use the 32x32 MFMA shape instead of the 16x16 one; the dispatcher
 * never picks them by itself.  The environment variable CYC_FORCE_KERNEL, read once when the library first chooses
 * a kernel, supplies the initial value.  Returns CYC_ERR_SHAPE for an unknown name. */
int cyc_force_kernel(const char *name);

/* Measurement aid: one launch of `iters` rounds of back-to-back MFMAs (dtype: a cyc_dtype; mfma_shape 16: 16x16
 * instructions, 32: 32x32) from registers on random-looking operands, four waves on every compute unit, no LDS or
 * memory traffic: what the matrix pipes sustain on this chip when nothing else happens.  *ops (host, may be NULL)
 * receives the operations of one launch; time the launch with events on `stream`.  sink: device, 4 bytes, in
 * practice never written.  iters: a multiple of 8, 8 .. 2^24. */
int cyc_diag_mfma_ceiling(int dtype, int mfma_shape, int64_t iters, void *sink, double *ops, void *stream);

/* Measurement aid: what a SIMD issues beside its MFMAs.  One launch of `iters` (1 .. 2^24) rounds per wave; a round is
 * the matrix work of 256 pipe cycles (mfma_shape 16: 16 bf16 MFMAs of 16x16x32, 32: 8 of 32x32x16) with
 * others_per_round (0, 16, 32, 48, 64 or 96) other instructions spread evenly between them (other_kind 0: v_fma_f32,
 * 1: v_exp_f32, 2: ds_read_b128 of a few LDS words), everything else from registers, on constant operands;
 * waves_per_simd (1 or 2) waves on every SIMD of every compute unit.  *ops (host, may be NULL) receives the MFMA
 * operations of one launch; time the launch with events on `stream`.  sink: device, 4 bytes, in practice never written. */
int cyc_diag_issue_mix(int mfma_shape, int other_kind, int others_per_round, int waves_per_simd, int64_t iters, void *sink,
                       double *ops, void *stream);

/* Test aid.  Inside the tile kernels of the triangular solve and of the Cholesky factorisation waves hand work to one
 * another through counters in LDS; every such wait is bounded, 2^20 polls, and a wave whose wait runs out goes on and
 * marks the tile, which is then written as NaN (and, in the factorisation, its inverse as unusable): NaNs instead of a
 * hung GPU or of plausible wrong numbers, should that code ever be broken.  This call sets the bound for the launches
 * enqueued after it (process-wide; polls: 1 .. 2^30, 0 restores the default), so that the behaviour on a run-out wait
 * can be looked at without breaking the code.  CYC_ERR_SHAPE outside that range. */
int cyc_diag_set_wait_limit(int64_t polls);

/* Verification aid for a property of the chip that the Cholesky kernels build on: D = A B + C on `tiles` independent
 * 16 x 16 x 4 problems in fp32, one v_mfma_f32_16x16x4_f32 each.  All device, row-major, 4-byte aligned: A tiles x 16 x 4,
 * B tiles x 4 x 16, C and D tiles x 16 x 16 (D may be C).  The instruction adds its four products to the accumulator in
 * ascending k with one rounding each, d = fma(a_3, b_3, fma(a_2, b_2, fma(a_1, b_1, fma(a_0, b_0, c)))), denormals
 * included: the bits of the scalar chain of the paper's Cholesky recurrence; the tests compare against exactly that.
 * tiles: 0 .. 2^24. */
int cyc_diag_mfma_f32_tiles(const void *A, const void *B, const void *C, void *D, int64_t tiles, void *stream);

/* Measurement aid: one wave that runs for `microseconds` (1 .. 2000000) and then writes to out (device, two
 * uint64_t, 8-byte aligned) the shader clock cycles and the ticks of the constant 100 MHz counter that went by.
 * Launched on a second stream beside other kernels it gives the engine clock sustained under their load:
 * GHz = out[0] / out[1] / 10. */
int cyc_diag_clock(void *out, int64_t microseconds, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* CYCLOTRON_MM_H */
