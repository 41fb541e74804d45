// cyc_narrow.hip -- HBM-bound kernel of the weight-stationary recurrence for a narrow j
// stream (N <= 16), gfx950.
//
// This is the regime the paper gives as the reason for the weight-stationary mapping
// ("Space-time Mappings of Dataflow Recurrences"): A, the weights, is far larger than B
// and C, so A must cross the memory interface exactly once.  Here the roles on chip are
// therefore inverted relative to the paper's cell grid: the whole B (K x N, a few hundred
// KiB) is what stays resident -- each wave keeps its k-slice of B in registers for the
// life of the workgroup -- and A streams past it at HBM speed, 16 rows at a time, straight
// from global memory into MFMA operand registers.  The k chain [i,k]_C <- [i,k-1]_C + W*B
// is cut into 8 contiguous k-slices, one per wave; each slice is accumulated in an MFMA
// accumulator, and the 8 partial sums of a row block are added in slice order by one wave
// through LDS (fixed order: results are bit-identical run to run, no atomics).
//
// What sets the speed is the shape of the loads.  Measured on this device with the same
// row-sliced traversal and no arithmetic: a wave-wide load that takes 64 bytes from each
// of 16 rows (the MFMA operand layout as it stands) tops out at 6.3 TB/s whatever the
// cache policy; one that takes whole 128-byte lines (8 rows x 128 bytes) with the
// non-temporal policy and a short queue (4-8 loads per lane) reaches 7.0-7.3 TB/s.  So A
// is fetched as whole lines, non-temporally, eight rows at a time, and the loaded register
// is used as a 16-row MFMA operand twice (once per half of the k it holds); the matrix
// pipe has time to spare.
#include "cyc_internal.h"

#include <type_traits>

namespace cyc {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x2 __attribute__((ext_vector_type(2)));

#define CYC_LDS __attribute__((address_space(3)))

constexpr int NWAVES = 8;     // k-slices per workgroup
constexpr int RB = 8;         // rows of A per load and per MFMA pair (one row block)
constexpr int RBK = 4;        // row blocks accumulated between two joins of the k-slices (2 to 8 measure the same)
constexpr int MAX_BURST = 4;  // loads per lane and burst (2: 20 % slower, 8: 4 % slower)
constexpr int NT_POLICY = 2;  // cache-policy bits of the A loads: bit 1 = non-temporal (0, the default policy: 12 % slower)

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

// wait for this wave's LDS traffic only (loads of A stay in flight), then meet the other waves
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// S: MFMA steps of 64 bytes of k that make up a wave's k-slice.  The workgroup covers k < 8*S*64/ES.
// FULL: K is exactly that, so no lane ever needs masking.
template <bool I8, int S, bool FULL>
__global__ __launch_bounds__(NWAVES * 64) void ws_narrow_kernel(const char *__restrict__ A, const char *__restrict__ B,
                                                                char *__restrict__ Cout, int M, int K, int N,
                                                                int64_t sA, int64_t sB, int64_t sC, int rows_per_wg, int b_vec)
{
    constexpr int ES = I8 ? 1 : 2;
    constexpr int KS = 64 / ES;          // k values per step
    constexpr int CH = 16 / ES;          // k values per 16-byte chunk
    constexpr int HALF = S / 2;          // B is staged through LDS in two halves
    constexpr int LPB = S / 2;           // loads per row block: 128-byte pieces in the wave's k-slice
    // A is fetched in bursts of BURST loads per lane into one of two register sets.  The next burst
    // is issued the moment the previous one has landed, before its MFMAs, so the queue never holds
    // more than one burst per wave and is refilled without waiting for the matrix pipe.
    constexpr int BURST = LPB % MAX_BURST == 0 ? MAX_BURST : 2;
    constexpr int BPB = LPB / BURST;                       // bursts per row block
    static_assert(LPB % BURST == 0 && (RBK * BPB) % 2 == 0, "a group of row blocks must be an even number of bursts");
    typedef typename Mac<I8>::acc_t acc_t;
    typedef typename Mac<I8>::elem elem;

    // LDS is used twice: first as eight wave-private patches for staging B, then (after a barrier)
    // as the double-buffered exchange area for the partial sums of the k-slices.
    constexpr int PATCH = HALF * KS * 16 * ES;
    constexpr int RED_BYTES = 2 * NWAVES * RBK * 64 * 16;
    __shared__ __attribute__((aligned(16))) char smem[NWAVES * PATCH > RED_BYTES ? NWAVES * PATCH : RED_BYTES];

    const int l = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lq = l & 15, g = l >> 4;

    A += (int64_t)blockIdx.y * sA * ES;
    B += (int64_t)blockIdx.y * sB * ES;
    elem *C = (elem *)Cout + (int64_t)blockIdx.y * sC;

    const int kw0 = w * S * KS;          // first k of this wave's slice

    // ---- stream A.  The wave's slice of a row block (8 rows x S*64 bytes) is fetched in 128-byte
    // pieces: in load p, lane l reads row l%8 of the block and the 16-byte chunk 2*(l/16) + (l%16)/8
    // of piece p, so one wave-wide load covers eight whole 128-byte lines.  Rows past M re-read row
    // M-1 (their results are never stored).
    const int row_begin = blockIdx.x * rows_per_wg;
    const int row_end = (row_begin + rows_per_wg) < M ? (row_begin + rows_per_wg) : M;
    const int nrb = (row_end - row_begin + RB - 1) / RB;
    const int64_t row_bytes = (int64_t)K * ES;
    const int chunk = 2 * g + (lq >> 3);             // 16-byte chunk of the 128-byte piece
    const uint32_t lane_off = (uint32_t)(kw0 * ES + chunk * 16);
    // A row block is addressed through a buffer descriptor based at its first row (wave-uniform) plus a
    // per-lane offset below 8 rows; buffer loads carry their cache policy explicitly.
    auto block_row = [&](int rb) -> int {
        const int r0 = row_begin + rb * RB;
        return r0 < M ? r0 : M - 1;
    };
    auto block_desc = [&](int rb) -> __amdgpu_buffer_rsrc_t {
        return __builtin_amdgcn_make_buffer_rsrc((void *)(A + (int64_t)block_row(rb) * row_bytes), 0, (int)(RB * row_bytes),
                                                 0x00020000);
    };
    auto lane_voff = [&](int rb) -> uint32_t {
        int r = row_begin + rb * RB + (lq & 7);
        r = r < M ? r : M - 1;
        return (uint32_t)(r - block_row(rb)) * (uint32_t)row_bytes + lane_off;
    };
    // piece p of a row block; non-temporal (bit 1 of the cache policy): A is read once
    auto fetch = [&](__amdgpu_buffer_rsrc_t d, uint32_t voff, int p) -> i32x4 {
        const uint32_t off = voff + (uint32_t)(p * 128);
        if (FULL) return __builtin_bit_cast(i32x4, __builtin_amdgcn_raw_buffer_load_b128(d, off, 0, NT_POLICY));
        i32x4 v = {0, 0, 0, 0};
        if (kw0 + (p * 8 + chunk) * CH < K) v = __builtin_bit_cast(i32x4, __builtin_amdgcn_raw_buffer_load_b128(d, off, 0, NT_POLICY));
        return v;
    };

    // the first loads of A go out before B is staged, so that HBM is busy during the staging
    i32x4 ring[2][BURST];
    __amdgpu_buffer_rsrc_t d_cur = block_desc(0);
    uint32_t v_cur = lane_voff(0);
#pragma unroll
    for (int u = 0; u < BURST; ++u) ring[0][u] = fetch(d_cur, v_cur, u);

    // ---- this wave's slice of B -> MFMA operand registers, once.  Rows of B are copied into a
    // wave-private LDS patch ([k][16 columns], zero beyond N and K) and read back through the
    // LDS transpose read, which hands every lane consecutive k of one column.  Bf[2p+e] holds, in
    // lane group g, the k of chunk 2g+e of piece p.
    i32x4 Bf[S];
    {
        typedef typename std::conditional<I8, int8_t, uint16_t>::type in_t;
        const in_t *Bg = (const in_t *)B;
        CYC_LDS in_t *patch = (CYC_LDS in_t *)(smem + w * PATCH);
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int kh0 = kw0 + h * HALF * KS;
            if (b_vec) {
                // N == 16 and B 16-byte aligned: the slice is contiguous in memory, copy 16 bytes per lane
                constexpr int CPRW = 16 * ES / 16;     // 16-byte chunks per row of B
#pragma unroll 16
                for (int x = l; x < PATCH / 16; x += 64) {
                    const int kk = kh0 + x / CPRW;
                    i32x4 v = {0, 0, 0, 0};
                    if (kk < K) v = *(const i32x4 *)(B + ((int64_t)kh0 * 16 * ES) + (int64_t)x * 16);
                    *(CYC_LDS i32x4 *)((CYC_LDS char *)patch + x * 16) = v;
                }
            } else {
                for (int x = l; x < HALF * KS * 16; x += 64) {
                    const int kk = kh0 + (x >> 4), j = x & 15;
                    patch[x] = (kk < K && j < N) ? Bg[(int64_t)kk * N + j] : (in_t)0;
                }
            }
#pragma unroll
            for (int s = 0; s < HALF; ++s) {
                i32x2 lo, hi;
                if (I8) {
                    CYC_LDS char *p = (CYC_LDS char *)patch + ((s >> 1) * 128 + 32 * g + 16 * (s & 1) + (lq >> 1)) * 16 + 8 * (lq & 1);
                    lo = __builtin_amdgcn_ds_read_tr8_b64_v2i32((CYC_LDS i32x2 *)p);
                    hi = __builtin_amdgcn_ds_read_tr8_b64_v2i32((CYC_LDS i32x2 *)(p + 8 * 16));
                } else {
                    CYC_LDS char *p = (CYC_LDS char *)patch + ((s >> 1) * 64 + 16 * g + 8 * (s & 1) + (lq >> 2)) * 32 + 8 * (lq & 3);
                    lo = __builtin_bit_cast(i32x2, __builtin_amdgcn_ds_read_tr16_b64_v4bf16((CYC_LDS bf16x4 *)p));
                    hi = __builtin_bit_cast(i32x2, __builtin_amdgcn_ds_read_tr16_b64_v4bf16((CYC_LDS bf16x4 *)(p + 4 * 32)));
                }
                Bf[h * HALF + s] = (i32x4){lo[0], lo[1], hi[0], hi[1]};
            }
            // the patch is rewritten by the next half: reads above must have completed
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        }
    }

    lds_barrier();     // every wave has its B fragments: the staging patches may be overwritten
    typedef acc_t red_t[NWAVES][RBK][64];
    CYC_LDS red_t *red = (CYC_LDS red_t *)smem;   // red[parity][wave][row block][lane]

    const int ngroups = (nrb + RBK - 1) / RBK;
    for (int gi = 0; gi < ngroups; ++gi) {
        acc_t part[RBK];
#pragma unroll
        for (int b = 0; b < RBK; ++b) {
            // row blocks past the end of this workgroup's rows stream valid rows whose sums are dropped
            const __amdgpu_buffer_rsrc_t d_next = block_desc(gi * RBK + b + 1);
            const uint32_t v_next = lane_voff(gi * RBK + b + 1);
            // The loaded register is used as the 16-row A operand as it stands.  Its lanes l%16 < 8 hold
            // rows 0..7 with the even chunks of the piece, lanes l%16 >= 8 the same rows with the odd
            // chunks.  Multiplied with the B operand of the even chunks, operand rows 0..7 give the even
            // part of the sums of rows 0..7 (operand rows 8..15 give nothing meaningful and are dropped);
            // with the B operand of the odd chunks, operand rows 8..15 give the odd part.
            acc_t even = {0, 0, 0, 0}, odd = {0, 0, 0, 0};
#pragma unroll
            for (int p0 = 0; p0 < LPB; p0 += BURST) {
                const int set = (b * BPB + p0 / BURST) & 1;   // bursts alternate between the two sets; a group starts on set 0
                // this burst has landed (nothing else of this wave is in flight): ask for the next one
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int u = 0; u < BURST; ++u) {
                    const int p = p0 + BURST + u;
                    ring[set ^ 1][u] = p < LPB ? fetch(d_cur, v_cur, p) : fetch(d_next, v_next, p - LPB);
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int u = 0; u < BURST; ++u) {
                    const i32x4 a = ring[set][u];
                    even = Mac<I8>::mfma(a, Bf[2 * (p0 + u)], even);
                    odd = Mac<I8>::mfma(a, Bf[2 * (p0 + u) + 1], odd);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            d_cur = d_next;
            v_cur = v_next;
            // accumulator register r of lane l is operand row 4*(l/16) + r, column l%16: lanes 0..31 keep
            // the even part, lanes 32..63 the odd part of rows 0..7
#pragma unroll
            for (int r = 0; r < 4; ++r) part[b][r] = l < 32 ? even[r] : odd[r];
        }

        // ---- join the 8 k-slices in slice order; wave gi%8 does it and emits C_ij
#pragma unroll
        for (int b = 0; b < RBK; ++b) red[gi & 1][w][b][l] = part[b];
        lds_barrier();
        if (w == (gi & 7)) {
            // lanes 0..31 finish the even-numbered row block of a pair, lanes 32..63 the odd-numbered one
            const int ll = l & 31;
#pragma unroll
            for (int bp = 0; bp < RBK; bp += 2) {
                const int b = bp + (l >> 5);
                acc_t sum = red[gi & 1][0][b][ll] + red[gi & 1][0][b][ll + 32];
#pragma unroll
                for (int v = 1; v < NWAVES; ++v) sum += red[gi & 1][v][b][ll] + red[gi & 1][v][b][ll + 32];
                if ((ll & 15) < N) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int row = row_begin + (gi * RBK + b) * RB + 4 * (ll >> 4) + r;
                        const elem v = sum[r];
                        if (row < row_end) C[(int64_t)row * N + (ll & 15)] = v;
                    }
                }
            }
        }
    }
}

template <bool I8, int S, bool FULL>
hipError_t launch_one(const Problem &p, int rows_per_wg, hipStream_t s)
{
    const int es = I8 ? 1 : 2;
    const int b_vec = p.N == 16 && ((uintptr_t)p.B & 15) == 0 && (p.batch == 1 || ((p.strideB * es) & 15) == 0);
    dim3 grid((unsigned)((p.M + rows_per_wg - 1) / rows_per_wg), (unsigned)p.batch);
    hipError_t launch_err = hipSuccess;
    launch_err = launch_kernel(ws_narrow_kernel<I8, S, FULL>, grid, dim3(NWAVES * 64), s, (const char *)p.A,
                       (const char *)p.B, (char *)p.C, (int)p.M, (int)p.K, (int)p.N, p.strideA, p.strideB, p.strideC,
                       rows_per_wg, b_vec);
    return launch_err;
}

template <bool I8>
hipError_t launch_dtype(const Problem &p, int rows_per_wg, hipStream_t s)
{
    const int64_t per_step = (int64_t)NWAVES * (I8 ? 64 : 32);   // k covered by one step of all waves
    const int steps = (int)((p.K + per_step - 1) / per_step);
    const bool full = (p.K % per_step) == 0;
    if (steps <= 8) return full && steps == 8 ? launch_one<I8, 8, true>(p, rows_per_wg, s) : launch_one<I8, 8, false>(p, rows_per_wg, s);
    if (steps <= 16) return full && steps == 16 ? launch_one<I8, 16, true>(p, rows_per_wg, s) : launch_one<I8, 16, false>(p, rows_per_wg, s);
    if (steps <= 24) return full && steps == 24 ? launch_one<I8, 24, true>(p, rows_per_wg, s) : launch_one<I8, 24, false>(p, rows_per_wg, s);
    return full && steps == 32 ? launch_one<I8, 32, true>(p, rows_per_wg, s) : launch_one<I8, 32, false>(p, rows_per_wg, s);
}

}  // namespace

bool supports_narrow(const Problem &p)
{
    const int es = p.i8 ? 1 : 2;
    const int64_t kmax = (int64_t)NWAVES * 32 * (p.i8 ? 64 : 32);   // 8192 bf16, 16384 int8
    if (p.N < 1 || p.N > 16 || p.K < 1 || p.K > kmax || p.M < 1) return false;
    if ((p.K * es) % 16) return false;                    // rows of A must stay 16-byte aligned
    if (p.M > (1 << 30) || p.batch > 65535) return false;
    if ((uintptr_t)p.A & 15) return false;
    if (p.batch > 1 && ((p.strideA * es) & 15)) return false;
    return true;
}

bool prefers_narrow(const Problem &p)
{
    // worth it only when A dominates: enough rows to amortise loading B into registers
    return supports_narrow(p) && p.M * p.batch >= 4096 && p.K >= 1024;
}

hipError_t launch_narrow(const Problem &p, hipStream_t s)
{
    if (!supports_narrow(p)) return hipErrorInvalidValue;
    // one workgroup per compute unit when the problem allows: rows_per_wg ~ total rows / 256
    int64_t rows = (p.M * p.batch + 255) / 256;
    rows = (rows + RB - 1) / RB * RB;
    if (rows < 64) rows = 64;
    if (rows > p.M) rows = (p.M + RB - 1) / RB * RB;
    return p.i8 ? launch_dtype<true>(p, (int)rows, s) : launch_dtype<false>(p, (int)rows, s);
}

}  // namespace cyc
