// cyc_narrowm.hip -- HBM-bound kernel of the matrix-multiply recurrence for a narrow i axis
// (M <= 32), gfx950.
//
// The paper's third choice of space-time mapping ("Space-time Mappings of Dataflow
// Recurrences"; the Spatial Mapping item of the motivating example): when B dominates, put
// (j,k) in space, so that every B_kj sits still in one cell, and let the few rows of A
// pass over it in time.  On this chip a cell of that grid is one slot of an MFMA operand
// register: every element of B crosses the memory interface once, lands in LDS by the
// DMA path, is moved by one LDS transpose read into the operand slot (k, j) where it
// stays, and is used there for all rows i at once: the 16 rows of the MFMA are the time
// axis i of the mapping, so the whole time loop is one instruction.  The partial sums of
// a column j travel along k inside that wave's accumulator.
//
// A wave owns 128 columns of C (all of its M rows) and walks down k.  Nothing is shared
// between waves: each has a private two-stage LDS ring (per stage 64 bytes of k: the rows
// of B as 1 KiB copies, plus its own copy of the A fragment, a few hundred KiB in all of A
// per batch element, served from L2), so the k loop has no workgroup barrier and a wave
// waits only for its own copies.  A workgroup of 8 waves reads 8 x 128 adjacent columns,
// i.e. one contiguous 1-2 KiB piece of every row of B.  For problems with too few column
// blocks to fill the chip the 8 waves of a workgroup instead take 8 contiguous k-slices of
// the same 128 columns and join their partial sums in slice order through LDS (fixed
// order, no atomics).
#include "cyc_internal.h"

namespace cyc {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x2 __attribute__((ext_vector_type(2)));

#define CYC_LDS __attribute__((address_space(3)))

constexpr int NWAVES = 8;
constexpr int WCOLS = 128;    // columns of C per wave
constexpr int TN = WCOLS / 16;

template <bool I8> struct Mac;
template <> struct Mac<false> {   // 16x16 tile, 32 k per instruction
    typedef f32x4 acc_t;
    typedef float elem;
    static __device__ __forceinline__ acc_t mfma(i32x4 a, i32x4 b, acc_t c)
    { return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0); }
};
template <> struct Mac<true> {    // 16x16 tile, 64 k per instruction
    typedef i32x4 acc_t;
    typedef int elem;
    static __device__ __forceinline__ acc_t mfma(i32x4 a, i32x4 b, acc_t c)
    { return __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, c, 0, 0, 0); }
};

// 64 lanes x 16 bytes from global memory (wave-uniform base + per-lane 32-bit offset) straight into
// LDS at lds_addr + lane*16.  STREAM: non-temporal policy, for B, which is read once.
template <bool STREAM>
__device__ __forceinline__ void dma16(const char *base, uint32_t lane_off, uint32_t lds_addr)
{
    if (STREAM)
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 nt" : : "s"(lds_addr), "v"(lane_off), "s"(base) : "memory", "m0");
    else
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(lds_addr), "v"(lane_off), "s"(base) : "memory", "m0");
}
template <int KEEP> __device__ __forceinline__ void wait_copies() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(KEEP) : "memory"); }
__device__ __forceinline__ void wait_lds() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

// MB: 16-row blocks of A (M <= 16*MB).  KSPLIT: the waves of a workgroup take k-slices of one column block
// (and join at the end) instead of adjacent column blocks.
template <bool I8, int MB, bool KSPLIT>
__global__ __launch_bounds__(NWAVES * 64) void ws_narrowm_kernel(const char *__restrict__ A, const char *__restrict__ B,
                                                                 char *__restrict__ Cout, int M, int K, int N, int64_t sA,
                                                                 int64_t sB, int64_t sC)
{
    constexpr int ES = I8 ? 1 : 2;
    constexpr int KR = 64 / ES;              // rows of B per step (64 bytes of k)
    constexpr int RBW = WCOLS * ES;          // bytes of a B row per wave
    constexpr int CPR = RBW / 16;            // 16-byte chunks of that
    constexpr int RPI = 64 / CPR;            // rows per wave-wide 1 KiB copy
    constexpr int NCP = KR / RPI;            // copies of B per step (8)
    constexpr int STAGE = KR * RBW + MB * 1024;
    static_assert(NCP == 8 && KR * RBW == 8192, "a step of B is 8 KiB per wave");
    typedef typename Mac<I8>::acc_t acc_t;
    typedef typename Mac<I8>::elem elem;

    __shared__ __attribute__((aligned(1024))) char smem[NWAVES * 2 * STAGE];
    const int l = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int s16 = l & 15, g = l >> 4;
    CYC_LDS char *mine = (CYC_LDS char *)smem + w * 2 * STAGE;
    const uint32_t mine_addr = (uint32_t)(uintptr_t)mine;

    A += (int64_t)blockIdx.y * sA * ES;
    B += (int64_t)blockIdx.y * sB * ES;
    elem *C = (elem *)Cout + (int64_t)blockIdx.y * sC;

    const int n0 = KSPLIT ? blockIdx.x * WCOLS : (blockIdx.x * NWAVES + w) * WCOLS;   // first column of this wave
    if (!KSPLIT && n0 >= N) return;          // no barrier in this form: a wave without columns just leaves
    const int nsteps = (K + KR - 1) / KR;
    int s_begin = 0, s_end = nsteps;
    if (KSPLIT) {
        const int per = (nsteps + NWAVES - 1) / NWAVES;
        s_begin = w * per < nsteps ? w * per : nsteps;
        s_end = s_begin + per < nsteps ? s_begin + per : nsteps;
    }

    // LDS placement of a stage: row r of B (RBW bytes) at r*RBW with its 16-byte chunk c in slot c ^ swz(r), the XOR
    // chosen so that the rows one transpose read touches fall on distinct banks; the swizzle is applied by
    // choosing which global chunk each lane copies.  Then MB KiB of A fragments, lane-linear.
    auto swz = [](int r) -> int {
        if (!I8) return ((r & 3) << 1) | (((r >> 3) & 1) << 3);
        return ((r >> 1) & 3) | (((r >> 4) & 1) << 2);
    };
    uint32_t voffB[NCP];
    const int cmax = (N - n0) * ES / 16 - 1;     // last 16-byte chunk of this wave's columns that exists (N*ES % 16 == 0)
#pragma unroll
    for (int x = 0; x < NCP; ++x) {
        const int r = x * RPI + l / CPR;
        int c = (l % CPR) ^ swz(r);
        c = c < cmax ? c : cmax;                 // columns past N re-read the last valid chunk and are never stored
        voffB[x] = (uint32_t)r * (uint32_t)(N * ES) + (uint32_t)c * 16;
    }
    // A fragment of a step: lane holds row l%16 (of block mb) and 16 bytes of k at 16*(l/16); rows past M re-read
    // row M-1 (rows of C are independent, theirs are not stored)
    uint32_t voffA[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        int r = mb * 16 + s16;
        r = r < M ? r : M - 1;
        voffA[mb] = (uint32_t)r * (uint32_t)(K * ES) + 16 * g;
    }
    const char *srcB = B + (int64_t)n0 * ES + (int64_t)s_begin * KR * N * ES;
    const char *srcA = A + (int64_t)s_begin * 64;
    const int64_t stepB = (int64_t)KR * N * ES;

    // Stage `slot` <- step st.  WHOLE: every row of the step lies inside K, all copies unconditional.  Otherwise a
    // copy whose rows (for A: whose 16 bytes of k) lie past K is replaced by zeros in LDS.
    auto fetch = [&](int st, int slot, bool whole) __attribute__((always_inline)) {
        const uint32_t dst = mine_addr + slot * STAGE;
#pragma unroll
        for (int x = 0; x < NCP; ++x) {
            if (whole || st * KR + x * RPI < K) dma16<true>(srcB, voffB[x], dst + x * 1024);
            else *(CYC_LDS i32x4 *)(mine + slot * STAGE + x * 1024 + l * 16) = (i32x4){0, 0, 0, 0};
        }
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            if (whole) {
                dma16<false>(srcA, voffA[mb], dst + KR * RBW + mb * 1024);
            } else {
                // lanes differ here (the last 64 bytes of k may end inside the step): an ordinary load and store
                i32x4 v = {0, 0, 0, 0};
                if ((st * 64 + 16 * g) / ES < K) v = *(const i32x4 *)(srcA + voffA[mb]);
                *(CYC_LDS i32x4 *)(mine + slot * STAGE + KR * RBW + mb * 1024 + l * 16) = v;
            }
        }
        srcB += stepB;
        srcA += 64;
    };

    // transpose-read offsets of the B fragments: in every 16-lane group the lanes point at a (4 k x 16 n) bf16 or
    // (8 k x 16 n) int8 patch and receive consecutive k of one column: lane l gets column l%16, k group l/16
    int offB[TN];
    {
        const int krow = I8 ? 16 * g + (s16 >> 1) : 8 * g + (s16 >> 2);
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            const int byte = (tn * 16 + (I8 ? 8 * (s16 & 1) : 4 * (s16 & 3))) * ES;
            offB[tn] = krow * RBW + (((byte >> 4) ^ swz(krow)) << 4) + (byte & 15);
        }
    }
    constexpr int HI = (I8 ? 8 : 4) * RBW;   // the second half of a lane's k values lies this many bytes further

    acc_t acc[MB][TN];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) acc[mb][tn] = (acc_t){0, 0, 0, 0};

    auto consume = [&](int slot) __attribute__((always_inline)) {
        CYC_LDS char *st = mine + slot * STAGE;
        i32x4 fa[MB];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) fa[mb] = *(CYC_LDS i32x4 *)(st + KR * RBW + mb * 1024 + l * 16);
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            i32x2 lo, hi;
            if (I8) {
                lo = __builtin_amdgcn_ds_read_tr8_b64_v2i32((CYC_LDS i32x2 *)(st + offB[tn]));
                hi = __builtin_amdgcn_ds_read_tr8_b64_v2i32((CYC_LDS i32x2 *)(st + offB[tn] + HI));
            } else {
                lo = __builtin_bit_cast(i32x2, __builtin_amdgcn_ds_read_tr16_b64_v4bf16((CYC_LDS bf16x4 *)(st + offB[tn])));
                hi = __builtin_bit_cast(i32x2, __builtin_amdgcn_ds_read_tr16_b64_v4bf16((CYC_LDS bf16x4 *)(st + offB[tn] + HI)));
            }
            const i32x4 fb = {lo[0], lo[1], hi[0], hi[1]};
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) acc[mb][tn] = Mac<I8>::mfma(fa[mb], fb, acc[mb][tn]);
        }
    };

    // ---- the k loop.  Step st sits in slot (st - s_begin) & 1.  While a step is consumed the next one is in flight
    // into the other slot, whose reads (of the step before) have completed.
    const int whole_end = (K / KR) < s_end ? (K / KR) : s_end;    // steps below this have all their rows inside K
    if (s_begin < s_end) fetch(s_begin, 0, s_begin < whole_end);
    int st = s_begin;
    for (; st + 1 < whole_end; ++st) {
        wait_lds();
        __builtin_amdgcn_sched_barrier(0);
        fetch(st + 1, (st + 1 - s_begin) & 1, true);
        wait_copies<NCP + MB>();              // all but the copies just issued have landed
        __builtin_amdgcn_sched_barrier(0);
        consume((st - s_begin) & 1);
    }
    for (; st < s_end; ++st) {                // the last step or two: the following step is ragged or absent
        wait_lds();
        __builtin_amdgcn_sched_barrier(0);
        if (st + 1 < s_end) fetch(st + 1, (st + 1 - s_begin) & 1, false);
        wait_copies<0>();
        __builtin_amdgcn_sched_barrier(0);
        consume((st - s_begin) & 1);
    }

    // ---- C_ij <- the end of the chain.  Accumulator register r of lane l is row 4*(l/16) + r, column l%16.
    if (!KSPLIT) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) {
                const int col = n0 + tn * 16 + s16;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int row = mb * 16 + 4 * g + r;
                    if (row < M && col < N) C[(int64_t)row * N + col] = acc[mb][tn][r];
                }
            }
        return;
    }
    // k-slices: every wave leaves its partial sums in LDS; wave v then adds up column block v of all slices in
    // slice order and emits it
    wait_copies<0>();
    wait_lds();
    __syncthreads();                          // nobody reads or lands anything in the rings any more
    typedef acc_t part_t[MB][TN][64];
    CYC_LDS part_t *part = (CYC_LDS part_t *)smem;   // NWAVES * MB * 8 KiB <= the rings
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) part[w][mb][tn][l] = acc[mb][tn];
    __syncthreads();
    static_assert(TN == NWAVES, "one column block per wave in the join");
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        acc_t sum = part[0][mb][w][l];
#pragma unroll
        for (int v = 1; v < NWAVES; ++v) sum += part[v][mb][w][l];
        const int col = n0 + w * 16 + s16;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = mb * 16 + 4 * g + r;
            if (row < M && col < N) C[(int64_t)row * N + col] = sum[r];
        }
    }
}

template <bool I8, int MB, bool KSPLIT>
hipError_t launch_one(const Problem &p, hipStream_t s)
{
    const int64_t per_wg = KSPLIT ? WCOLS : (int64_t)WCOLS * NWAVES;
    dim3 grid((unsigned)((p.N + per_wg - 1) / per_wg), (unsigned)p.batch);
    hipError_t launch_err = hipSuccess;
    launch_err = launch_kernel(ws_narrowm_kernel<I8, MB, KSPLIT>, grid, dim3(NWAVES * 64), s, (const char *)p.A,
                       (const char *)p.B, (char *)p.C, (int)p.M, (int)p.K, (int)p.N, p.strideA, p.strideB, p.strideC);
    return launch_err;
}

}  // namespace

bool supports_narrowm(const Problem &p)
{
    const int es = p.i8 ? 1 : 2;
    if (p.M < 1 || p.M > 32 || p.K < 1 || p.N < 1) return false;
    if (p.lda || p.ldb || p.ldc || p.Cin || p.kslices) return false;
    if ((p.K * es) % 16 || (p.N * es) % 16) return false;          // rows of A and B stay 16-byte aligned
    if (p.K > (1 << 30) || p.N > (1 << 30) || p.batch > 65535) return false;
    // per-lane byte offsets (32 rows of A, 64 rows of B) are kept in 32 bits
    if (p.K * es * 32 >= ((int64_t)1 << 32) || p.N * es * 64 >= ((int64_t)1 << 32)) return false;
    if (((uintptr_t)p.A | (uintptr_t)p.B) & 15) return false;
    if (p.batch > 1 && (((p.strideA * es) | (p.strideB * es)) & 15)) return false;
    return true;
}

// column blocks of 1024 fill the chip, or else the k-sliced form does better
static bool narrowm_ksplit(const Problem &p) { return p.batch * ((p.N + WCOLS * NWAVES - 1) / (WCOLS * NWAVES)) < 128; }

bool prefers_narrowm(const Problem &p)
{
    // worth it when B dominates: at least a mebibyte of it per launch
    return supports_narrowm(p) && p.batch * p.K * p.N >= (1 << 20) && p.N >= 64 && p.K >= 256;
}

hipError_t launch_narrowm(const Problem &p, hipStream_t s)
{
    if (!supports_narrowm(p)) return hipErrorInvalidValue;
    const bool ks = narrowm_ksplit(p), two = p.M > 16;
    if (p.i8) {
        if (ks) return two ? launch_one<true, 2, true>(p, s) : launch_one<true, 1, true>(p, s);
        return two ? launch_one<true, 2, false>(p, s) : launch_one<true, 1, false>(p, s);
    }
    if (ks) return two ? launch_one<false, 2, true>(p, s) : launch_one<false, 1, true>(p, s);
    return two ? launch_one<false, 2, false>(p, s) : launch_one<false, 1, false>(p, s);
}

}  // namespace cyc
