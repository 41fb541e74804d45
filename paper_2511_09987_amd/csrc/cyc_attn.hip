// cyc_attn.hip -- the FlashAttention-2 tile recurrence on gfx950.
//
// Paper, "FlashAttention-2 Recurrence": keys and values arrive in tiles J_t; every query i keeps a
// running maximum m_i, a running sum l_i and a running output o_i,
//     S_ij = alpha Q_i. K_j.^T,   mh = max(m_i, max_j S_ij),
//     l_i <- exp(m_i - mh) l_i + sum_j exp(S_ij - mh),   o_i <- exp(m_i - mh) o_i + sum_j exp(S_ij - mh) V_j.,
// and O_i. = o_i / l_i at the end.  The paper maps it with the query tile stationary on a processing
// element and K, V streaming past; so here: a wave holds 32 queries as MFMA operand registers for the
// whole kernel, a workgroup of eight waves (256 queries, two waves per SIMD) streams tiles of 64 or 128 keys
// of K and V through LDS.
//
// Both products are computed transposed, which removes every shuffle between them:
//   S^T = K_tile Q^T   (A operand: 16 keys x 32 d from LDS; B operand: the stationary Q, whose row-major
//                       rows are exactly the operand layout).  Accumulator lane l then holds, for query
//                       l%16, the keys 4*(l/16) .. +3 of each 16-key block: all statistics of a query
//                       (m, l, the rescale factor) are per lane, and only the maximum needs the other
//                       three lanes of the query (two lane swaps per tile).
//   O^T = V^T P^T      (B operand: P^T straight from those accumulators, rounded to bfloat16 -- two
//                       16-key blocks side by side make the 8 k-slots of a lane, and the sum over keys
//                       does not care in which slot a key sits as long as V uses the same slots; A
//                       operand: V^T through the LDS transpose read, with that same key order.)
//                       Accumulator lane l holds, for query l%16, four consecutive d: the rescale by
//                       exp(m - mh) is a per-lane multiply and the final store is 16 bytes per lane.
// Arithmetic: Q, K, V bfloat16; S, m, l, o fp32; exp through the hardware exp2 with alpha*log2(e) folded
// into the scores; the probabilities enter the second product rounded to bfloat16 (nearest even), and the
// running sum adds up those same rounded values (it rides on the second product as a row of ones).  The maximum that
// the exponentials refer to follows the running maximum lazily: a tile's maximum is taken only after one of its
// weights came out above 2^8 (overflowed / rebase below); o / l does not depend on it.
//
// Schedule: a software pipeline across tiles inside every wave, so that matrix-core and vector-ALU
// instructions of neighbouring tiles are issued interleaved (the loop at the end of the kernel).  The LDS reads of
// the K and V fragments are issued from inline asm a fixed number of fragments ahead of the MFMAs that use them and
// waited for one by one; left to the compiler, which is short of registers here, each read sat right before its use
// and its whole latency was waited out.  The build checks the compiler's output for such reads (check_async_reads.py).
//
// Measured at batch 64, N = M = 4096, TFLOP/s at d = 128 / d = 64 (run-to-run and box-to-box spread about 5 %):
//   64 queries per wave, 4 waves, tile after tile                                    599 / 463
//   32 queries per wave, 8 waves, tile after tile, 128-key / 64-key tiles           1036 / 848
//   the same with the two waves of a SIMD half a tile apart (one or two barriers)    940 / 700
//   software pipeline (this file), maximum followed exactly                          960 / 860
//   software pipeline, maximum followed lazily                                      1050 / 910
//   software pipeline with 64 queries per wave and 4 waves (512 registers)           574 / 540
//   this file: fragment reads a window ahead, maximum only after an overflow   1110-1170 / 850-880
//   the same on the 32 x 32 x 16 MFMA shape (half the MFMA instructions)        1070-1100 / 860-870
// The kernel runs at the socket's power limit: on constant inputs (little switching) the 32 x 32 form needs 5 % fewer
// cycles than this one (1360 against 1290 TFLOP/s), on random inputs its clock drops by as much or more.  Removing
// the exponentials or the overflow check altogether changes nothing measurable; what is left is matrix work and LDS
// traffic (each wave reads the whole K and V tile for its 32 queries), and 64 queries per wave do not fit the registers
// at two waves per SIMD.
#include "cyc_internal.h"

namespace cyc {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x2 __attribute__((ext_vector_type(2)));
typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

#define CYC_LDS __attribute__((address_space(3)))

constexpr int QB = 2;                    // 16-query blocks per wave
constexpr int QW = QB * 16;              // queries per wave
constexpr int NWAVE = 8;                 // waves per workgroup

// 64 lanes x 16 bytes from global memory (wave-uniform base + per-lane offset) into LDS at lds_addr + lane*16
__device__ __forceinline__ void copy16(const char *base, uint32_t lane_off, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_addr), "v"(lane_off), "s"(base)
                 : "memory", "m0");
}

__device__ __forceinline__ i32x4 mfma_frag(i32x2 lo, i32x2 hi) { return (i32x4){lo[0], lo[1], hi[0], hi[1]}; }

template <int... I, class F> __device__ __forceinline__ void static_for_each(std::integer_sequence<int, I...>, F &&f)
{
    (f(std::integral_constant<int, I>{}), ...);
}
// f(integral_constant<int, 0>) .. f(integral_constant<int, N-1>): a loop whose index is a constant expression
template <int N, class F> __device__ __forceinline__ void static_for(F &&f) { static_for_each(std::make_integer_sequence<int, N>{}, f); }

// 16 bytes per lane from LDS address addr + OFF, with no wait: dst is valid only after lds_wait
template <int OFF> __device__ __forceinline__ void lds_read128(i32x4 &dst, uint32_t addr)
{
    static_assert(OFF >= 0 && OFF < 65536, "the offset field of an LDS instruction has 16 bits");
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFF));
}
// wait until at most PENDING LDS operations issued after the read of x are outstanding; x is valid from here on
template <int PENDING> __device__ __forceinline__ void lds_wait(i32x4 &x) { asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(x) : "n"(PENDING)); }
// the transposing read of four 16-bit elements per lane, likewise without a wait
template <int OFF> __device__ __forceinline__ void lds_read_tr64(i32x2 &dst, uint32_t addr)
{
    static_assert(OFF >= 0 && OFF < 65536, "the offset field of an LDS instruction has 16 bits");
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFF));
}
template <int PENDING> __device__ __forceinline__ void lds_wait2(i32x2 &x, i32x2 &y) { asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(x), "+v"(y) : "n"(PENDING)); }

// D: head dimension; KT: keys per tile (a multiple of 32)
template <int D, int KT>
__global__ __launch_bounds__(NWAVE * 64) void attn_kernel(const char *__restrict__ Q, const char *__restrict__ K,
                                                          const char *__restrict__ V, float *__restrict__ O, int N,
                                                          int M, int nqb, float scale_log2e)
{
    constexpr int KB = KT / 16;           // 16-key blocks per tile
    constexpr int ROW = D * 2;            // bytes per row of Q, K, V
    constexpr int CPR = ROW / 16;         // 16-byte chunks per row: 16 (D = 128) or 8 (D = 64)
    constexpr int RPC = 64 / CPR;         // rows per 1 KiB copy
    constexpr int DS = D / 32;            // MFMA k-steps over d
    constexpr int DT = D / 16;            // 16-wide d tiles of the output
    constexpr int TILE_BYTES = KT * ROW;
    constexpr int COPIES = TILE_BYTES / 1024 / NWAVE;   // 1 KiB copies per wave per tile and operand
    // LDS: two stages of the K tile, then two stages of the V tile.  Row r of a tile starts at r*ROW; its
    // 16-byte chunk c sits in slot c ^ swzK(r) resp. c ^ swzV(r), so that the rows one operand read touches
    // fall on distinct banks.
    __shared__ __attribute__((aligned(1024))) char lds_raw[4 * TILE_BYTES];
    CYC_LDS char *lds = (CYC_LDS char *)lds_raw;
    const uint32_t lds_base = (uint32_t)(uintptr_t)lds;
    auto swzK = [](int r) { return CPR == 16 ? (r & 15) : ((r >> 1) & 7); };
    auto swzV = [](int r) { return CPR == 16 ? ((r & 7) << 1) : (((r >> 1) & 3) << 1); };

    const int l = threadIdx.x & 63, lq = l & 15, g = l >> 4;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // Workgroups are handed to the eight XCDs round robin by their linear index, and each XCD has its own L2.
    // The workgroups of one batch element read the same K and V, so they are renumbered to run on one XCD:
    // XCD x takes a contiguous range of (batch element, query block) pairs, in the order it receives them.
    const int total = gridDim.x, xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int logical = xcd * (total >> 3) + (xcd < (total & 7) ? xcd : (total & 7)) + slot;
    const int64_t bz = logical / nqb;
    const int bx = logical - (int)bz * nqb;
    Q += bz * (int64_t)N * ROW;
    K += bz * (int64_t)M * ROW;
    V += bz * (int64_t)M * ROW;
    O += bz * (int64_t)N * D;
    const int q0 = bx * (NWAVE * QW) + w * QW;          // first query of this wave

    // ---- the stationary operand: Q of this wave's queries, for the whole kernel.  B operand of
    // S^T = K Q^T: lane holds query jq*16 + l%16, d = 32 ks + 8 (l/16) .. +7.  Queries past N re-read
    // query N-1 (their results are never stored).
    i32x4 qf[QB][DS];
#pragma unroll
    for (int jq = 0; jq < QB; ++jq) {
        int qi = q0 + jq * 16 + lq;
        qi = qi < N ? qi : N - 1;
#pragma unroll
        for (int ks = 0; ks < DS; ++ks) qf[jq][ks] = *(const i32x4 *)(Q + (int64_t)qi * ROW + ks * 64 + g * 16);
    }

    // ---- copies of a tile of K or of V into a stage.  A copy moves RPC rows (1 KiB); copy x of wave w takes the rows
    // x*NWAVE*RPC + w*RPC .. of the tile, so that a lane's offset within its copy (swizzle included: the row
    // number changes by a multiple of 16 with x) is the same for every x and every full tile.  Keys past M (last
    // tile only) re-read key M-1 and are masked below.
    const int row0 = w * RPC + l / CPR;                             // this lane's row within copy 0
    const uint32_t voffK = (uint32_t)row0 * ROW + (((l % CPR) ^ swzK(row0)) << 4);
    const uint32_t voffV = (uint32_t)row0 * ROW + (((l % CPR) ^ swzV(row0)) << 4);
    const int ntiles = (M + KT - 1) / KT;
    auto issue = [&](const char *src, uint32_t voff, int tile, int stage_index) __attribute__((always_inline)) {
        const char *base = src + (int64_t)tile * TILE_BYTES;
        const uint32_t dst = lds_base + stage_index * TILE_BYTES + w * 1024;
        if ((tile + 1) * KT <= M) {
#pragma unroll
            for (int x = 0; x < COPIES; ++x) copy16(base + x * (NWAVE * 1024), voff, dst + x * (NWAVE * 1024));
        } else {
            const int last = M - 1 - tile * KT;                   // last valid row of the tile
#pragma unroll
            for (int x = 0; x < COPIES; ++x) {
                const int r = x * (NWAVE * RPC) + row0;
                // offsets are unsigned: row min(r, last) counted from the tile's first row, this lane's chunk
                copy16(base, (uint32_t)(r <= last ? r : last) * ROW + (voff - (uint32_t)row0 * ROW), dst + x * (NWAVE * 1024));
            }
        }
    };
    auto issue_K = [&](int tile) __attribute__((always_inline)) { issue(K, voffK, tile, tile & 1); };
    auto issue_V = [&](int tile) __attribute__((always_inline)) { issue(V, voffV, tile, 2 + (tile & 1)); };

    // ---- running state of this lane's queries (one per 16-query block jq): maximum in the log2 domain, this lane's
    // share of the sum, and O^T accumulators [d tile][query tile]
    float m2[QB];
    f32x4 acc_o[DT][QB], acc_l[QB];                                   // acc_l: the running sum l, the same value in all four registers
#pragma unroll
    for (int jq = 0; jq < QB; ++jq) {
        m2[jq] = -__builtin_inff();
        acc_l[jq] = (f32x4){0, 0, 0, 0};
#pragma unroll
        for (int id = 0; id < DT; ++id) acc_o[id][jq] = (f32x4){0, 0, 0, 0};
    }
    f32x4 s[KB][QB], s_next[KB][QB];                                  // S^T of tiles t and t+1: [key block][query block]
    i32x4 pf[QB][KB / 2];                                             // P^T as B operand: [query block][32-key step]
    float tile_max[QB];                                               // maximum of the newest S^T per query, log2 domain
    // this wave's copies have landed and its LDS reads have returned (the stages it read are about to be requested into
    // again by other waves); then meet the other waves
    auto landed_barrier = []() __attribute__((always_inline)) { asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory"); };

    // ---- O^T += V^T P^T for a tile in V stage STAGE.  A operand lane: d = 16 id + l%16; k-slots 0..3 = keys
    // 32 sk + 4 (l/16) .. +3, k-slots 4..7 = the same keys of the next 16-key block (the order P^T was packed in).
    // Fragment i = sk * DT + id is two transposing reads (the two key blocks); like the K fragments they are issued
    // VWIN fragments ahead of their use.  The swizzle of a row depends on the lane alone (4 (l/16) + (l%16)/4 mod 8),
    // so one address register per d tile serves every sk and both key blocks through the offset field.
    constexpr int VWIN = 4;
    constexpr int NVFRAG = (KB / 2) * DT;
    uint32_t vaddr[DT];
#pragma unroll
    for (int id = 0; id < DT; ++id) {
        const int row = 4 * g + (lq >> 2);
        const int chunk = (id * 16 + 4 * (lq & 3)) >> 3, within = ((id * 16 + 4 * (lq & 3)) & 7) * 2;
        vaddr[id] = lds_base + 2 * TILE_BYTES + row * ROW + ((chunk ^ swzV(row)) << 4) + within;
    }
    auto weighted_values = [&](auto stage_c) __attribute__((always_inline)) {
        constexpr int STAGE = decltype(stage_c)::value;
        // the running sum rides along as one more row block of V^T whose every entry is 1: l += 1^T P^T, i.e. the sum of
        // the weights as the second product sees them (rounded to bfloat16), with no vector-ALU additions
        const i32x4 ones = {0x3f803f80, 0x3f803f80, 0x3f803f80, 0x3f803f80};
        i32x2 lo[VWIN], hi[VWIN];
        static_for<VWIN>([&](auto ic) __attribute__((always_inline)) {
            constexpr int i = decltype(ic)::value, off = STAGE * TILE_BYTES + (i / DT) * 32 * ROW;
            lds_read_tr64<off>(lo[i], vaddr[i % DT]);
            lds_read_tr64<off + 16 * ROW>(hi[i], vaddr[i % DT]);
        });
        static_for<NVFRAG>([&](auto ic) __attribute__((always_inline)) {
            constexpr int i = decltype(ic)::value, sk = i / DT, id = i % DT;
            constexpr int later = NVFRAG - 1 - i < VWIN - 1 ? NVFRAG - 1 - i : VWIN - 1;   // fragments requested after i
            if constexpr (id == 0) {
#pragma unroll
                for (int jq = 0; jq < QB; ++jq)
                    acc_l[jq] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ones), __builtin_bit_cast(bf16x8, pf[jq][sk]), acc_l[jq], 0, 0, 0);
            }
            lds_wait2<2 * later>(lo[i % VWIN], hi[i % VWIN]);
            const i32x4 vf = mfma_frag(lo[i % VWIN], hi[i % VWIN]);
#pragma unroll
            for (int jq = 0; jq < QB; ++jq)
                acc_o[id][jq] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vf), __builtin_bit_cast(bf16x8, pf[jq][sk]), acc_o[id][jq], 0, 0, 0);
            if constexpr (i + VWIN < NVFRAG) {
                constexpr int off = STAGE * TILE_BYTES + ((i + VWIN) / DT) * 32 * ROW;
                lds_read_tr64<off>(lo[i % VWIN], vaddr[(i + VWIN) % DT]);
                lds_read_tr64<off + 16 * ROW>(hi[i % VWIN], vaddr[(i + VWIN) % DT]);
            }
        });
    };

    // maximum over lanes l, l^16, l^32, l^48.  The swaps exchange halves (rows 2,3 of the first operand with rows
    // 0,1 of the second) resp. odd rows of the first with even rows of the second; fed the same value twice, the
    // two results together hold the value of both partners.  (The elements are copied to scalars before the bit
    // cast: a bit cast applied to a vector element directly reads element 0 whatever the index.)
    auto as_float = [](unsigned u) __attribute__((always_inline)) { return __builtin_bit_cast(float, u); };
    auto wave_max = [&](float x) __attribute__((always_inline)) {
        const unsigned u = __builtin_bit_cast(unsigned, x);
        const auto a = __builtin_amdgcn_permlane32_swap(u, u, false, false);
        const unsigned a0 = a[0], a1 = a[1];
        const unsigned v = __builtin_bit_cast(unsigned, __builtin_fmaxf(as_float(a0), as_float(a1)));
        const auto b = __builtin_amdgcn_permlane16_swap(v, v, false, false);
        const unsigned b0 = b[0], b1 = b[1];
        return __builtin_fmaxf(as_float(b0), as_float(b1));
    };
    // ---- S^T = K_tile Q^T for a tile in K stage STAGE.  Fragment i = ks * KB + ik (16 keys x 32 d) feeds the QB MFMAs of
    // key block ik and d step ks.  The reads are issued KWIN fragments ahead of their use and waited for one at a time:
    // they are written as asm because the compiler, short of registers here, otherwise issues each read right before
    // the MFMAs that need it and waits out the whole LDS latency every time.  The wait names the fragment as an
    // operand so that no use of it can be moved above the wait.  (LDS reads return in order, so reads the compiler
    // issues in between only make these waits longer than needed, never shorter.)
    constexpr int KWIN = 4;
    constexpr int NFRAG = DS * KB;
    uint32_t kaddr[DS];                                               // this lane's address within stage 0, key block 0
#pragma unroll
    for (int ks = 0; ks < DS; ++ks) kaddr[ks] = lds_base + lq * ROW + (((ks * 4 + g) ^ swzK(lq)) << 4);
    auto scores_into = [&](auto stage_c, f32x4(&sn)[KB][QB]) __attribute__((always_inline)) {
        constexpr int STAGE = decltype(stage_c)::value;
        i32x4 kf[KWIN];
        static_for<KWIN>([&](auto ic) __attribute__((always_inline)) {
            constexpr int i = decltype(ic)::value;
            lds_read128<STAGE * TILE_BYTES + (i % KB) * 16 * ROW>(kf[i], kaddr[i / KB]);
        });
#pragma unroll
        for (int ik = 0; ik < KB; ++ik)
#pragma unroll
            for (int jq = 0; jq < QB; ++jq) sn[ik][jq] = (f32x4){0, 0, 0, 0};
        static_for<NFRAG>([&](auto ic) __attribute__((always_inline)) {
            constexpr int i = decltype(ic)::value, ks = i / KB, ik = i % KB;
            constexpr int later = NFRAG - 1 - i < KWIN - 1 ? NFRAG - 1 - i : KWIN - 1;   // reads issued after fragment i
            lds_wait<later>(kf[i % KWIN]);
#pragma unroll
            for (int jq = 0; jq < QB; ++jq)
                sn[ik][jq] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kf[i % KWIN]), __builtin_bit_cast(bf16x8, qf[jq][ks]), sn[ik][jq], 0, 0, 0);
            if constexpr (i + KWIN < NFRAG)
                lds_read128<STAGE * TILE_BYTES + ((i + KWIN) % KB) * 16 * ROW>(kf[i % KWIN], kaddr[(i + KWIN) / KB]);
        });
    };
    // Maximum of the tile's scores per query, in the log2 domain.  Keys past M were copied from key M-1, so their
    // scores repeat a valid score and leave the maximum alone.
    auto stats = [&](const f32x4(&sn)[KB][QB]) __attribute__((always_inline)) {
#pragma unroll
        for (int jq = 0; jq < QB; ++jq) {
            float top = sn[0][jq][0];
#pragma unroll
            for (int ik = 0; ik < KB; ++ik)
#pragma unroll
                for (int r = 0; r < 4; ++r) top = __builtin_fmaxf(top, sn[ik][jq][r]);
            tile_max[jq] = wave_max(top) * scale_log2e;
        }
    };
    // ---- weights of tile t against the reference m2, their sum, and P^T packed as an operand
    auto probabilities = [&](int t, const f32x4(&sc)[KB][QB], bool mask) __attribute__((always_inline)) {
#pragma unroll
        for (int jq = 0; jq < QB; ++jq)
#pragma unroll
            for (int ik = 0; ik < KB; ++ik)
#pragma unroll
                for (int r = 0; r < 4; r += 2) {
                    float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[ik][jq][r], scale_log2e, -m2[jq]));
                    float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[ik][jq][r + 1], scale_log2e, -m2[jq]));
                    if (mask) {                                   // keys past M take no weight
                        const int key = t * KT + ik * 16 + 4 * g + r;
                        p0 = key < M ? p0 : 0.0f;
                        p1 = key + 1 < M ? p1 : 0.0f;
                    }
                    // one conversion instruction rounds and packs the pair; k-slot: block ik&1 of the 32-key step ik/2
                    const bf16x2 pair = __builtin_convertvector((f32x2){p0, p1}, bf16x2);
                    pf[jq][ik >> 1][(ik & 1) * 2 + (r >> 1)] = __builtin_bit_cast(int, pair);
                }
    };
    // The exponentials are taken against a reference m2 that follows the running maximum lazily: no maximum is taken
    // of a tile whose weights all came out at most 2^LAG.  The packed bfloat16 weights are non-negative, so their bit
    // patterns order like unsigned 16-bit integers (infinity and NaN above every finite value), and one packed
    // integer maximum handles two of them.  Only when some weight of some query of the wave is above 2^LAG (always on
    // the first tile, where m2 = -inf gives infinite weights; hardly ever after the first few) is the tile's maximum
    // taken, the reference moved to it, the sums and outputs so far rescaled by exp(m_old - m_new) and the tile's
    // weights taken again.  The quotient o / l at the end is the same whatever the reference.
    constexpr unsigned short LAG_BITS = 0x4380;                       // 2^8 as bfloat16
    auto overflowed = [&]() __attribute__((always_inline)) {
        u16x2 top = {0, 0};
#pragma unroll
        for (int jq = 0; jq < QB; ++jq)
#pragma unroll
            for (int sk = 0; sk < KB / 2; ++sk)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int word = pf[jq][sk][r];
                    top = __builtin_elementwise_max(top, __builtin_bit_cast(u16x2, word));
                }
        const unsigned short t0 = top[0], t1 = top[1];
        return __builtin_amdgcn_ballot_w64((t0 > t1 ? t0 : t1) > LAG_BITS) != 0;
    };
    auto rebase = [&](const f32x4(&sc)[KB][QB]) __attribute__((always_inline)) {
        stats(sc);
#pragma unroll
        for (int jq = 0; jq < QB; ++jq) {
            const float mh = __builtin_fmaxf(m2[jq], tile_max[jq]);
            const float keep = __builtin_amdgcn_exp2f(m2[jq] - mh);       // exp(m - mh); 0 on the first tile
            m2[jq] = mh;
            acc_l[jq] *= keep;
#pragma unroll
            for (int id = 0; id < DT; ++id) acc_o[id][jq] *= keep;
        }
    };
    // ---- Software pipeline: the matrix-core work of tile t+1's scores is issued between the vector-ALU work of tile
    // t's weights; the second product of tile t follows on its own, and the other wave of the SIMD fills its gaps.
    // One barrier per step: K(t+1) and V(t) have landed and every wave is done with K(t) and V(t-1), whose
    // stages K(t+2) and V(t+1) are then requested into.
    // tile t (of parity PAR), whose scores are in cur, and the scores of tile t+1 into nxt
    auto step = [&](int t, auto par_c, f32x4(&cur)[KB][QB], f32x4(&nxt)[KB][QB]) __attribute__((always_inline)) {
        landed_barrier();
        if (t + 2 < ntiles) issue_K(t + 2);
        issue_V(t + 1);
        scores_into(std::integral_constant<int, 1 - decltype(par_c)::value>{}, nxt);
        probabilities(t, cur, false);
        if (__builtin_expect(overflowed(), 0)) {
            rebase(cur);
            probabilities(t, cur, false);
        }
        weighted_values(par_c);
    };
    auto last_step = [&](int t, auto par_c, f32x4(&cur)[KB][QB]) __attribute__((always_inline)) {
        landed_barrier();
        probabilities(t, cur, true);
        if (__builtin_expect(overflowed(), 0)) {
            rebase(cur);
            probabilities(t, cur, true);
        }
        weighted_values(par_c);
    };
    const std::integral_constant<int, 0> even;
    const std::integral_constant<int, 1> odd;
    issue_K(0);
    landed_barrier();
    issue_V(0);
    if (ntiles > 1) issue_K(1);
    scores_into(even, s);
    // two tiles per trip: the K stage of each is a constant, and the two score arrays swap roles without being copied
    int t = 0;
    for (; t + 2 < ntiles; t += 2) {
        step(t, even, s, s_next);
        step(t + 1, odd, s_next, s);
    }
    if (t + 1 < ntiles) {
        step(t, even, s, s_next);
        last_step(t + 1, odd, s_next);
    } else {
        last_step(t, even, s);
    }

    // ---- O_i. = o_i / l_i.  Accumulator register r of lane l: d = 16 id + 4 (l/16) + r, query 16 jq + l%16.
#pragma unroll
    for (int jq = 0; jq < QB; ++jq) {
        const float tot = acc_l[jq][0];                 // every lane of the query holds the whole sum
        const int qi = q0 + jq * 16 + lq;
        if (qi < N) {
#pragma unroll
            for (int id = 0; id < DT; ++id) {
                const f32x4 o = acc_o[id][jq];
                *(f32x4 *)(O + (int64_t)qi * D + id * 16 + 4 * g) = (f32x4){o[0] / tot, o[1] / tot, o[2] / tot, o[3] / tot};
            }
        }
    }
}

}  // namespace

bool supports_attention(int64_t N, int64_t M, int64_t d)
{
    // per-lane byte offsets of keys are kept in 32 bits
    return (d == 64 || d == 128) && N >= 1 && M >= 1 && N < (1 << 30) && M * d * 2 < ((int64_t)1 << 32);
}

hipError_t launch_attention(const void *Q, const void *K, const void *V, void *O, int64_t batch, int64_t N, int64_t M,
                            int64_t d, hipStream_t s)
{
    if (!supports_attention(N, M, d) || batch < 1 || batch > 65535) return hipErrorInvalidValue;
    const float scale_log2e = (float)(1.4426950408889634 / __builtin_sqrt((double)d));
    const int64_t nqb = (N + NWAVE * QW - 1) / (NWAVE * QW);  // query blocks per batch element
    if (nqb * batch >= ((int64_t)1 << 31)) return hipErrorInvalidValue;
    dim3 grid((unsigned)(nqb * batch));
    hipError_t launch_err = hipSuccess;
    if (d == 128)
        launch_err = launch_kernel(attn_kernel<128, 64>, grid, dim3(NWAVE * 64), s, (const char *)Q, (const char *)K,
                           (const char *)V, (float *)O, (int)N, (int)M, (int)nqb, scale_log2e);
    else
        launch_err = launch_kernel(attn_kernel<64, 128>, grid, dim3(NWAVE * 64), s, (const char *)Q, (const char *)K,
                           (const char *)V, (float *)O, (int)N, (int)M, (int)nqb, scale_log2e);
    return launch_err;
}

}  // namespace cyc
