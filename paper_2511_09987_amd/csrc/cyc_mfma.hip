// cyc_mfma.hip -- MFMA kernels of the weight-stationary recurrence for gfx950.
//
// Mapping of the paper's weight-stationary program ("Space-time Mappings of Dataflow
// Recurrences") onto one compute unit: a workgroup owns a BM x BN block of C.  Its
// share of the stationary operand A (BM rows) is staged through LDS once per 128
// bytes of k and then held in registers while the whole BN-wide slice of the j stream
// passes over it; the B values that the paper moves cell to cell down the i axis are
// one LDS read that every row of the block shares; the partial sums that the paper
// hands east along k never move: they are the MFMA accumulators, and only the value
// leaving the last column, C_ij <- [i,k_end]_C, is written to memory.
//
// Both element types share one byte geometry: a k-tile is 128 bytes of a row of A
// (64 bf16 or 128 int8 values), cut into eight 16-byte chunks.
#include "cyc_internal.h"
#include <algorithm>

namespace cyc {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef int i32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x2 __attribute__((ext_vector_type(2)));

#define CYC_LDS __attribute__((address_space(3)))
#define CYC_GLB __attribute__((address_space(1)))

// accumulator type and MFMA instruction per element type and tile shape MT (MT x MT outputs per
// instruction, 16 bytes of k per lane); operands travel as 4 dwords.  Both shapes have the same peak
// rate, but this chip runs dense GEMMs at its power limit and the 16-wide shape costs less energy per
// flop: issued back to back from registers on random operands it sustains 1.96 PFLOP/s (bf16) against
// 1.71 for the 32-wide shape, and the kernels here run at 1.9 GHz with it against 1.65 GHz.  The
// dispatcher uses the 16-wide shape; the 32-wide one stays selectable for comparison.
template <bool I8, int MT> struct Acc;
template <> struct Acc<false, 32> {
    typedef float elem;
    typedef f32x16 type;   // bf16 x bf16 -> fp32, 32x32 tile, 16 k per instruction
    static __device__ __forceinline__ type mfma(i32x4 a, i32x4 b, type c)
    { return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0); }
};
template <> struct Acc<true, 32> {
    typedef int elem;
    typedef i32x16 type;   // int8 x int8 -> int32, 32x32 tile, 32 k per instruction
    static __device__ __forceinline__ type mfma(i32x4 a, i32x4 b, type c)
    { return __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c, 0, 0, 0); }
};
// The 16-wide forms are written as asm with the accumulator tied to the destination: left to the
// register allocator, a fully occupied accumulator file ends up with destinations that differ from
// their sources and some hundred register moves per k-tile to rotate them back.  The compiler's
// hazard logic does not look inside asm: no accumulator is read by another instruction within 60
// MFMAs of its update, and the kernel waits explicitly before it reads them out.
template <> struct Acc<false, 16> {
    typedef float elem;
    typedef f32x4 type;    // 16x16 tile, 32 k per instruction
    static __device__ __forceinline__ type mfma(i32x4 a, i32x4 b, type c)
    {
        asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
        return c;
    }
};
template <> struct Acc<true, 16> {
    typedef int elem;
    typedef i32x4 type;    // 16x16 tile, 64 k per instruction
    static __device__ __forceinline__ type mfma(i32x4 a, i32x4 b, type c)
    {
        asm volatile("v_mfma_i32_16x16x64_i8 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
        return c;
    }
};

template <bool I8, int BM_, int BN_, int WM_, int WN_, int MT_>
struct Cfg {
    static constexpr bool I8v = I8;
    static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_, MT = MT_;
    static constexpr int NKS = MT == 32 ? 4 : 2;   // MFMA k-steps per k-tile (32 or 64 bytes of k each)
    static constexpr int ACCN = MT * MT / 64;      // accumulator registers per MFMA tile
    static constexpr int NW = WM * WN, NT = NW * 64;
    static constexpr int ES = I8 ? 1 : 2;          // bytes per input element
    static constexpr int BKE = 128 / ES;           // k elements per tile
    static constexpr int KSTEP = 32 / ES;          // k elements per MFMA (32 bytes of k)
    static constexpr int A_BYTES = BM * 128;
    static constexpr int RB = BN * ES;             // bytes per row of the B tile
    static constexpr int B_BYTES = BKE * RB;
    static constexpr int NSA = 2, NSB = 3;         // LDS stages: A is double, B triple buffered
    static constexpr int LDS_BYTES = NSA * A_BYTES + NSB * B_BYTES;
    static constexpr int CPR = RB / 16;            // 16-byte chunks per B row
    static constexpr int RPI = 64 / CPR;           // B rows covered by one wave-wide 1 KiB load
    static constexpr int AI = BM / 8 / NW;         // 1 KiB A loads per wave per k-tile
    static constexpr int BI = B_BYTES / 1024 / NW; // 1 KiB B loads per wave per k-tile
    static constexpr int TM = BM / WM / MT, TN = BN / WN / MT;   // MFMA tiles per wave
    static_assert(BM % (8 * NW) == 0 && B_BYTES % (1024 * NW) == 0, "loads must divide evenly over waves");
    static_assert(CPR <= 64 && LDS_BYTES <= 160 * 1024, "tile does not fit");
};

// LDS placement.  A tile: row r (128 bytes) at r*128, its chunk c stored in slot c ^ swzA(r).
// B tile: row k (RB bytes) at k*RB, its chunk c stored in slot c ^ swzB(k).  The XORs spread
// the rows that one fragment read touches over distinct banks.
__device__ __forceinline__ int swzA(int r) { return (r >> 1) & 7; }
template <class C>
__device__ __forceinline__ int swzB(int k)
{
    if (C::MT == 32) {
        if (!C::I8v) return ((k & 3) << 2) | (C::CPR >= 32 ? ((k >> 3) & 1) << 4 : 0);
        return C::CPR >= 16 ? (k & 7) << 1 : ((k >> 1) & 3) << 1;
    }
    // 16-wide tiles: half a wave reads, per transpose read, 4 rows k..k+3 and 4 rows k+8..k+11 of 32 bytes
    // (bf16), or 8 rows k..k+7 and 8 rows k+16..k+23 of 16 bytes (int8)
    if (!C::I8v) return ((k & 3) << 1) | (((k >> 3) & 1) << 3);
    return C::CPR >= 16 ? (k & 7) | (((k >> 4) & 1) << 3) : ((k >> 1) & 3) | (((k >> 4) & 1) << 2);
}

// 64 lanes x 16 bytes go from global memory (wave-uniform base + per-lane 32-bit offset) straight
// into LDS at lds_addr + lane*16 (lds_addr wave-uniform).  Written as asm so that the compiler does
// not make every later LDS read wait for these copies; completion is awaited with tile_fence().
__device__ __forceinline__ void async_copy16(const char *base, uint32_t lane_off, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_addr), "v"(lane_off), "s"(base)
                 : "memory", "m0");
}
// The same copy in two steps, so that an MFMA can sit between them where the hardware wants one
// instruction between a write of m0 and its use: copy_arm() sets the LDS destination (a + b),
// copy_fire() issues the load.  Nothing else in these kernels touches m0.
__device__ __forceinline__ void copy_arm(uint32_t a, uint32_t b)
{
    asm volatile("s_add_u32 m0, %0, %1" : : "s"(a), "s"(b) : "m0", "scc");
}
__device__ __forceinline__ void copy_fire(const char *base, uint32_t lane_off)
{
    asm volatile("global_load_lds_dwordx4 %0, %1" : : "v"(lane_off), "s"(base) : "memory");
}
// This wave's LDS reads are done and all but its newest `keep` copies have landed (copies retire in
// issue order); then meet the other waves.
template <int KEEP>
__device__ __forceinline__ void tile_fence()
{
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(KEEP) : "memory");
}

// RAGGED: M, N need not be multiples of the block and K need not be a multiple of the k-tile (rows of A
// and B must still be 16-byte aligned).  Rows and columns past the edge re-read the last valid ones
// and are not stored; in the last k-tile, chunks at or past K are not copied but written as zeros.
// EPI: what the epilogue does with the accumulators: EPI_STORE C <- A*B; EPI_MINUS C <- Cin - A*B (Cin may be C).
// A template parameter, so that each form is straight-line code.
enum { EPI_STORE = 0, EPI_MINUS = 1 };
template <class C, bool RAGGED, int EPI>
__global__ __launch_bounds__(C::NT) void ws_mfma_kernel(const char *__restrict__ A, const char *__restrict__ B,
                                                        char *__restrict__ Cout, int M, int K, int N, int64_t sA,
                                                        int64_t sB, int64_t sC, int tiles_m, int tiles_n, int lda,
                                                        int ldb, int ldc, const char *Cin)
{
    constexpr int ES = C::ES, RB = C::RB, TM = C::TM, TN = C::TN;
    __shared__ __attribute__((aligned(1024))) char lds_raw[C::LDS_BYTES];
    CYC_LDS char *lds = (CYC_LDS char *)lds_raw;
    const uint32_t lds_base = (uint32_t)(uintptr_t)lds;

    const int l = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = w / C::WN, wn = w % C::WN;

    // ---- which C block: workgroups are dealt round-robin to the 8 XCDs, so ids congruent
    // mod 8 share an L2.  Give each XCD a contiguous run of blocks, ordered so that the
    // 32 blocks resident at a time form 4 block-rows x 8 block-columns: the 4 row panels
    // of A (the stationary operand) stay in that XCD's L2 while the columns stream by.
    int bid = blockIdx.x, bz = blockIdx.y;              // block of C and batch element (or k-slice) of this workgroup
    const int nblk = tiles_m * tiles_n;
    if ((nblk & 7) == 0) {
        bid = (bid & 7) * (nblk >> 3) + (bid >> 3);
    } else if ((gridDim.y & 7) == 0) {
        // few blocks per batch element (or k-slice): keep the blocks of one element, which share its A and B, on one
        // XCD.  Workgroup number blockIdx.y * nblk + blockIdx.x runs on XCD (number mod 8) as the (number / 8)-th there.
        const int number = blockIdx.y * nblk + blockIdx.x, slot = number >> 3;
        bz = (number & 7) + 8 * (slot / nblk);
        bid = slot % nblk;
    }
    constexpr int GM = 4;
    const int per_group = GM * tiles_n;
    const int group = bid / per_group, in_group = bid % per_group;
    const int rows_here = (tiles_m - group * GM) < GM ? (tiles_m - group * GM) : GM;
    const int tm_blk = group * GM + in_group % rows_here, tn_blk = in_group / rows_here;
    const int m0 = tm_blk * C::BM, n0 = tn_blk * C::BN;

    A += (int64_t)bz * sA * ES;
    B += (int64_t)bz * sB * ES;
    Cout += (int64_t)bz * sC * 4;

    // ---- global source of each 16-byte chunk this lane copies per k-tile: a wave-uniform base
    // that advances with the k-tile, plus a fixed per-lane byte offset (below 2^32, see supports_mfma)
    const char *baseA = A + ((int64_t)m0 * lda) * ES;   // lda: row stride of A in elements (K unless A is a window)
    const char *baseB = B + (int64_t)n0 * ES;
    const int64_t stepB = (int64_t)C::BKE * ldb * ES;   // ldb, ldc: row strides of B and C (N unless windows)
    uint32_t voffA[C::AI], voffB[C::BI];
    const int nkt = RAGGED ? (K + C::BKE - 1) / C::BKE : K / C::BKE;
    const int last = nkt - 1;
    unsigned tail_ok = 0;          // RAGGED: bit x set = this lane's copy x of the last k-tile is inside K
#pragma unroll
    for (int t = 0; t < C::AI; ++t) {
        int r = (w * C::AI + t) * 8 + (l >> 3);
        int c = (l & 7) ^ swzA(r);
        if (RAGGED) {
            if (last * C::BKE + c * (16 / ES) < K) tail_ok |= 1u << t;
            r = m0 + r < M ? r : M - 1 - m0;
        }
        voffA[t] = (uint32_t)r * (uint32_t)(lda * ES) + c * 16;
    }
#pragma unroll
    for (int t = 0; t < C::BI; ++t) {
        int kr = (w * C::BI + t) * C::RPI + l / C::CPR;
        int c = (l % C::CPR) ^ swzB<C>(kr);
        if (RAGGED) {
            if (last * C::BKE + kr < K) tail_ok |= 1u << (C::AI + t);
            const int cmax = (N - n0) * ES / 16 - 1;      // last 16-byte chunk of this block's columns that exists
            c = c < cmax ? c : cmax;
        }
        voffB[t] = (uint32_t)kr * (uint32_t)(ldb * ES) + c * 16;
    }
    // LDS map: NSA stages of the A tile, then NSB stages of the B tile
    constexpr int LDS_B0 = C::NSA * C::A_BYTES;
    // copy number x of this wave's share of k-tile `ktile`: x < AI is a piece of the A tile (into A
    // stage sa), otherwise a piece of the B tile (into B stage sb)
    // (`tail`: this call may be about the last k-tile; false in the bulk of the k loop, where the copy is
    // then unconditional)
    const char *srcA = baseA + 2 * 128, *srcB = baseB + 2 * stepB;   // source of the k-tile being fetched in the loop
    auto issue_one = [&](int x, int sa, int sb, int ktile, bool tail) __attribute__((always_inline)) {
        const uint32_t dst = x < C::AI ? sa * C::A_BYTES + (w * C::AI + x) * 1024
                                       : LDS_B0 + sb * C::B_BYTES + (w * C::BI + x - C::AI) * 1024;
        const char *src = x < C::AI ? baseA + (int64_t)ktile * 128 : baseB + (int64_t)ktile * stepB;
        const uint32_t off = x < C::AI ? voffA[x] : voffB[x - C::AI];
        if (RAGGED && tail && ktile == last) {
            if ((tail_ok >> x) & 1) async_copy16(src, off, lds_base + dst);
            else *(CYC_LDS i32x4 *)(lds + dst + l * 16) = (i32x4){0, 0, 0, 0};
        } else {
            async_copy16(src, off, lds_base + dst);
        }
    };
    // The same for the copies inside the k loop, which fetch from srcA / srcB, in two steps around an
    // MFMA: arm_one() returns whether fire_one() is to follow (a piece wholly past K is zero-filled
    // instead).  `at_last`: srcA / srcB point at the last k-tile of a RAGGED problem.
    auto arm_one = [&](int x, int sa, int sb, bool at_last) __attribute__((always_inline)) -> bool {
        const uint32_t piece = x < C::AI ? (w * C::AI + x) * 1024 : LDS_B0 + (w * C::BI + x - C::AI) * 1024;
        const uint32_t stage = x < C::AI ? sa * C::A_BYTES : sb * C::B_BYTES;
        if (RAGGED && at_last && !((tail_ok >> x) & 1)) {
            *(CYC_LDS i32x4 *)(lds + piece + stage + l * 16) = (i32x4){0, 0, 0, 0};
            return false;
        }
        copy_arm(lds_base + piece, stage);
        return true;
    };
    auto fire_one = [&](int x) __attribute__((always_inline)) {
        copy_fire(x < C::AI ? srcA : srcB, x < C::AI ? voffA[x] : voffB[x - C::AI]);
    };

    // ---- LDS read offsets of this lane's fragments
    constexpr int MT = C::MT, NKS = C::NKS;
    // A fragment (MT rows x 32*64/MT bytes of k): lane holds row l%MT and one 16-byte chunk of the k-step:
    // chunk 2*ks + l/32 (MT = 32, k-steps of 32 bytes) or 4*ks + l/16 (MT = 16, k-steps of 64 bytes).
    int offA[NKS];
    {
        int r = wm * (TM * MT) + (l & (MT - 1));
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) offA[ks] = r * 128 + (((ks * (8 / NKS) + l / MT) ^ swzA(r)) << 4);
    }
    // B fragment through the LDS transpose read.  In every 16-lane group the lanes point
    // at a (4 k x 16 n) bf16 or (8 k x 16 n) int8 patch and receive, per lane, consecutive
    // k of one column: lane l ends up with column l%MT and k group l/MT of the MFMA operand.
    int offB[TN];
    {
        const int lq = l & 15, colhalf = MT == 32 ? (l >> 4) & 1 : 0, kg = l / MT;
        const int krow = C::I8v ? 16 * kg + (lq >> 1) : 8 * kg + (lq >> 2);
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            int ncol = wn * (TN * MT) + tn * MT + colhalf * 16 + (C::I8v ? 8 * (lq & 1) : 4 * (lq & 3));
            int byte = ncol * ES;
            offB[tn] = LDS_B0 + krow * RB + ((((byte >> 4)) ^ swzB<C>(krow)) << 4) + (byte & 15);
        }
    }
    // rows of the B tile per MFMA k-step
    constexpr int KROWS = (128 / ES) / NKS;

    typedef Acc<C::I8v, MT> Mac;
    typename Mac::type acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < C::ACCN; ++r) acc[i][j][r] = 0;

    // ---- main loop.  A k-tile (4 MFMA k-steps) is consumed in two halves.  The fragments of one
    // half (2 k-steps: 2*TM A fragments, 2*TN B fragments) sit in one of two register sets; while the
    // MFMAs of a half run from one set, the LDS reads of the following half fill the other, so the
    // matrix pipe has queued work across the workgroup barrier.  Per k-tile kt:
    //   half 0 of kt from set 0 | read half 1 of kt   -> set 1 | copy B of tile kt+2
    //   fence: tile kt+1 has landed, every wave is done reading tile kt
    //   half 1 of kt from set 1 | read half 0 of kt+1 -> set 0 | copy A of tile kt+2
    // The address unit needs 16 cycles per wave-wide copy, which over all waves is half the MFMA time
    // of a k-tile, and a wave that cannot issue its copy cannot issue its MFMAs either.  Hence the
    // copies are spread over both halves, one per group of MFMAs.  B can be fetched before the fence
    // because it has a third stage: tile kt+2 goes where tile kt-1 was, which nobody reads any more.
    constexpr int KSH = NKS / 2;             // MFMA k-steps per half
    i32x4 fa[2][KSH][TM];
    i32x4 fb[2][KSH][TN];
    constexpr int NREAD = KSH * (TM + TN);   // fragment reads per half
    constexpr int NMMA = KSH * TM * TN;      // MFMAs per half
    constexpr int NG = 8;                  // groups per half
    static_assert(C::AI <= NG && C::BI <= NG, "one copy per group");
    // fragment read number r of a half: k-step q = r / (TM+TN); B fragments first, then A
    auto read_one = [&](int r, int set, int sa, int sb, int h) __attribute__((always_inline)) {
        const int q = r / (TM + TN), e = r % (TM + TN), ks = h * KSH + q;
        if (e < TN) {
            const int o = sb * C::B_BYTES + offB[e];
            i32x2 lo, hi;
            if (C::I8v) {
                lo = __builtin_amdgcn_ds_read_tr8_b64_v2i32((CYC_LDS i32x2 *)(lds + o + (ks * KROWS) * RB));
                hi = __builtin_amdgcn_ds_read_tr8_b64_v2i32((CYC_LDS i32x2 *)(lds + o + (ks * KROWS + 8) * RB));
            } else {
                lo = __builtin_bit_cast(i32x2, __builtin_amdgcn_ds_read_tr16_b64_v4bf16((CYC_LDS bf16x4 *)(lds + o + (ks * KROWS) * RB)));
                hi = __builtin_bit_cast(i32x2, __builtin_amdgcn_ds_read_tr16_b64_v4bf16((CYC_LDS bf16x4 *)(lds + o + (ks * KROWS + 4) * RB)));
            }
            fb[set][q][e] = (i32x4){lo[0], lo[1], hi[0], hi[1]};
        } else {
            fa[set][q][e - TN] = *(CYC_LDS i32x4 *)(lds + sa * C::A_BYTES + offA[ks] + (e - TN) * MT * 128);
        }
    };
    // MFMA number m of a half
    auto mma_one = [&](int m, int set) __attribute__((always_inline)) {
        const int q = m / (TM * TN), i = (m / TN) % TM, j = m % TN;
        acc[i][j] = Mac::mfma(fa[set][q][i], fb[set][q][j], acc[i][j]);
    };
    // One half.  A wave issues at most one instruction every four cycles and an MFMA occupies the
    // matrix pipe for 32, so at most about six other instructions fit between two MFMAs before the
    // pipe starves.  The fragment reads that fill the other register set and this half's copies are
    // therefore dealt out evenly, one small item per MFMA slot, and pinned there.
    auto half = [&](int set, int rd_sa, int rd_sb, int rd_half, int cp_first, int cp_count, int cp_sa, int cp_sb, bool at_last) __attribute__((always_inline)) {
        const int naux = NREAD + cp_count, stride = naux / cp_count;   // every stride-th item is a copy
#pragma unroll
        for (int m = 0; m < NMMA; ++m) {
            // items x with x * NMMA / naux == m go in front of MFMA m; a copy is armed in front of it and
            // fired behind it
            int fire = -1;
            bool go = false;
#pragma unroll
            for (int x = (m * naux + NMMA - 1) / NMMA; x < ((m + 1) * naux + NMMA - 1) / NMMA; ++x) {
                if (x % stride == stride - 1 && x / stride < cp_count) {
                    fire = cp_first + x / stride;
                    go = arm_one(fire, cp_sa, cp_sb, at_last);
                } else {
                    read_one(x - (x / stride < cp_count ? x / stride : cp_count), set ^ 1, rd_sa, rd_sb, rd_half);
                }
            }
            mma_one(m, set);
            if (fire >= 0 && go) fire_one(fire);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // Beyond the last tile there is nothing left to fetch or read: the final tile is copied again
    // into a stage nobody reads and a stale half is read into registers nobody uses, rather than
    // branch around the copies and reads.
    auto tile_at = [&](int t) __attribute__((always_inline)) { return t < last ? t : last; };
#pragma unroll
    for (int x = 0; x < C::AI + C::BI; ++x) issue_one(x, 0, 0, 0, true);
    tile_fence<0>();               // tile 0 in LDS
#pragma unroll
    for (int x = 0; x < C::AI + C::BI; ++x) issue_one(x, 1, 1, tile_at(1), true);
#pragma unroll
    for (int r = 0; r < NREAD; ++r) read_one(r, 0, 0, 0, 0);

    int sb0 = 0;                   // B stage of tile kt; tile kt+1 is in sb1, tile kt+2 goes to sb2
    // `careful`: tile kt+2 may be the last k-tile or beyond it; false in the bulk of the k loop, where
    // srcA / srcB simply move on by one k-tile per iteration and every copy is unconditional.
    auto k_tile = [&](int kt, bool careful) __attribute__((always_inline)) {
        const int sa0 = kt & 1, sa1 = sa0 ^ 1;
        const int sb1 = sb0 == 2 ? 0 : sb0 + 1, sb2 = sb1 == 2 ? 0 : sb1 + 1;
        if (careful) {
            srcA = baseA + (int64_t)tile_at(kt + 2) * 128;
            srcB = baseB + (int64_t)tile_at(kt + 2) * stepB;
        }
        const bool at_last = RAGGED && careful && kt + 2 >= last;
        half(0, sa0, sb0, 1, C::AI, C::BI, 0, sb2, at_last);
        // all but the B copies just issued have landed; reads of tile kt done.  (Once the last k-tile
        // of a RAGGED problem is involved, wait for all copies: a wave whose piece of that tile lies
        // wholly past K issues no copy for it, so counting outstanding copies would be off.)
        if (RAGGED && careful) tile_fence<0>();
        else tile_fence<C::BI>();
        half(1, sa1, sb1, 0, 0, C::AI, sa0, 0, at_last);
        if (!careful) {
            srcA += 128;
            srcB += stepB;
        }
        sb0 = sb1;
    };
    // bulk: tile kt+2 is a whole k-tile (RAGGED: and not the last one); then the two or three k-tiles
    // whose copies touch the last k-tile or have nothing left to fetch
    int kt = 0;
    for (; kt + 2 < (RAGGED ? last : nkt); ++kt) k_tile(kt, false);
    for (; kt < nkt; ++kt) k_tile(kt, true);
    // all copies have landed (none may arrive after the workgroup's LDS is released); the last MFMA
    // results are in the register file 
    asm volatile("s_waitcnt vmcnt(0)\n\ts_nop 15\n\ts_nop 15" ::: "memory");

    // ---- C_ij <- [i,k_end]_C.  32x32 tile: accumulator register r of lane l is row (r/4)*8 + (l/32)*4 + r%4,
    // column l%32 (for fixed r, 32 lanes write 128 contiguous bytes).  16x16 tile: register r of lane l is
    // row (l/16)*4 + r, column l%16.
    typedef typename Mac::elem elem;
    elem *Cw = (elem *)Cout;
    auto row_of = [&](int i, int r) __attribute__((always_inline)) { return m0 + wm * (TM * MT) + i * MT + (l / MT) * 4 + (r >> 2) * 8 + (r & 3); };
    auto col_of = [&](int j) __attribute__((always_inline)) { return n0 + wn * (TN * MT) + j * MT + (l & (MT - 1)); };
    if (EPI == EPI_MINUS) {
        // C <- Cin - A*B, in two passes: first every accumulator becomes Cin - accumulator, Cin fetched a row of MFMA tiles at a
        // time with further rows in flight; then all are stored.  Loads alone retire in issue order
        // and can be waited for group by group; with stores between them every wait would be for everything
        // outstanding, one round trip to memory per row of tiles.  (Cin may be C: no element is stored before all of
        // this wave's elements are read, and no other wave touches them.)
        constexpr int AHEAD = TM >= 3 ? 2 : 1;              // rows of tiles requested beyond the one being applied
        elem cin[AHEAD + 1][TN][C::ACCN];
        auto request = [&](int i) __attribute__((always_inline)) {
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < C::ACCN; ++r) {
                    const int row = row_of(i, r), col = col_of(j);
                    cin[i % (AHEAD + 1)][j][r] = (!RAGGED || (row < M && col < N)) ? ((const elem *)Cin)[(int64_t)row * ldc + col] : (elem)0;
                }
        };
#pragma unroll
        for (int i = 0; i < AHEAD && i < TM; ++i) request(i);
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            // (the barriers keep the compiler from moving every accumulator into the vector registers first, which
            // leaves it room for one load at a time)
            __builtin_amdgcn_sched_barrier(0);
            if (i + AHEAD < TM) request(i + AHEAD);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < C::ACCN; ++r) acc[i][j][r] = cin[i % (AHEAD + 1)][j][r] - acc[i][j][r];
        }
        __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < C::ACCN; ++r) {
                const int row = row_of(i, r), col = col_of(j);
                if (!RAGGED || (row < M && col < N)) Cw[(int64_t)row * ldc + col] = acc[i][j][r];
            }
}

template <class C, int EPI>
hipError_t launch_epi(const Problem &p, hipStream_t s)
{
    const bool ragged = p.M % C::BM || p.N % C::BN || p.K % C::BKE;
    const int tiles_m = (int)((p.M + C::BM - 1) / C::BM), tiles_n = (int)((p.N + C::BN - 1) / C::BN);
    dim3 grid((unsigned)(tiles_m * tiles_n), (unsigned)p.batch);
    hipError_t launch_err = hipSuccess;
    if (ragged)
        launch_err = launch_kernel(ws_mfma_kernel<C, true, EPI>, grid, dim3(C::NT), s, (const char *)p.A, (const char *)p.B,
                           (char *)p.C, (int)p.M, (int)p.K, (int)p.N, p.strideA, p.strideB, p.strideC, tiles_m, tiles_n,
                           (int)row_stride_a(p), (int)row_stride_b(p), (int)row_stride_c(p), (const char *)p.Cin);
    else
        launch_err = launch_kernel(ws_mfma_kernel<C, false, EPI>, grid, dim3(C::NT), s, (const char *)p.A, (const char *)p.B,
                           (char *)p.C, (int)p.M, (int)p.K, (int)p.N, p.strideA, p.strideB, p.strideC, tiles_m, tiles_n,
                           (int)row_stride_a(p), (int)row_stride_b(p), (int)row_stride_c(p), (const char *)p.Cin);
    return launch_err;
}

// EXTRA: also build the EPI_MINUS form (only the 16-wide MFMA shape, which is all its callers use)
template <class C, bool EXTRA>
hipError_t launch_cfg(const Problem &p, hipStream_t s)
{
    if (!p.Cin) return launch_epi<C, EPI_STORE>(p, s);
    if constexpr (EXTRA) return launch_epi<C, EPI_MINUS>(p, s);
    return hipErrorInvalidValue;
}

// C <- slice 0 + slice 1 + ... of the workspace, in that order for every element (the order of the adds is part of
// the result for fp32), four elements per thread.
template <typename V>
__global__ __launch_bounds__(256) void ws_join_slices_kernel(const V *__restrict__ part, V *__restrict__ C, int64_t quads,
                                                             int slices)
{
    const int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (q >= quads) return;
    V sum = part[q];
#pragma unroll 8
    for (int sl = 1; sl < slices; ++sl) sum += part[(int64_t)sl * quads + q];
    C[q] = sum;
}

}  // namespace

// Any M, N, K >= 1 whose rows of A and B are 16-byte aligned (K*es and N*es multiples of 16, aligned
// base pointers and batch strides); shapes that are not multiples of the block take the RAGGED variant.
bool supports_mfma(const Problem &p, int tile)
{
    if (tile != 256 && tile != 128) return false;
    const int es = p.i8 ? 1 : 2;
    if (p.K <= 0 || p.M <= 0 || p.N <= 0) return false;
    const int64_t lda = row_stride_a(p), ldb = row_stride_b(p), ldc = row_stride_c(p);
    if ((p.K * es) % 16 || (p.N * es) % 16 || (lda * es) % 16 || lda < p.K) return false;
    if ((ldb * es) % 16 || ldb < p.N || ldc < p.N || ldb > (1 << 30) || ldc > (1 << 30)) return false;
    if ((p.lda || p.ldb || p.ldc || p.Cin) && p.batch != 1 && !p.kslices) return false;
    if (p.M > (1 << 30) || p.N > (1 << 30) || p.K > (1 << 30) || p.batch > 65535) return false;
    if (((p.M + tile - 1) / tile) * ((p.N + tile - 1) / tile) > (1 << 30)) return false;
    // per-lane byte offsets inside a tile's rows are kept in 32 bits
    if (lda * es * 256 + 128 >= ((int64_t)1 << 32) || ldb * es * 128 + 512 >= ((int64_t)1 << 32)) return false;
    if (((uintptr_t)p.A | (uintptr_t)p.B | (uintptr_t)p.C | (uintptr_t)p.Cin) & 15) return false;
    if (p.batch > 1 && (((p.strideA * es) | (p.strideB * es) | (p.strideC * 4)) & 15)) return false;
    return true;
}

// Block size by a small cost model: a CU runs one 256x256 block or two 128x128 blocks at a time; a 128x128
// block does a quarter of the work at about 3/4 of the efficiency.  Compare the number of rounds each needs.
int choose_mfma_tile(const Problem &p)
{
    if (p.M < 16 || p.N < 16) return 0;      // slivers go to the shape-agnostic kernel
    const int64_t n256 = ((p.M + 255) / 256) * ((p.N + 255) / 256) * p.batch;
    const int64_t n128 = ((p.M + 127) / 128) * ((p.N + 127) / 128) * p.batch;
    const double cost256 = (double)((n256 + 255) / 256);
    const double cost128 = (double)((n128 + 511) / 512) * 0.675;
    const bool ok256 = supports_mfma(p, 256), ok128 = supports_mfma(p, 128);
    if (ok256 && (!ok128 || cost256 <= cost128)) return 256;
    return ok128 ? 128 : 0;
}

// The paper's weight-stationary mapping puts k in space: a cell keeps its A_ik and hands its partial sum east.
// For problems with few output blocks and a long k extent this is the mapping that fills the chip: the k range
// is cut into `ksplit` slices, every (output block, slice) pair is a workgroup that keeps its slice of A's block
// row and of B's block column to itself and leaves its partial sum in its slice of a workspace; the hand-over
// along k is a second kernel that adds the slices of every element in ascending slice order (a fixed order: the
// result is the same bits on every call).
int choose_ksplit(const Problem &p, int *tile)
{
    *tile = 128;
    if (p.batch != 1 || p.lda || p.ldb || p.ldc || p.Cin || p.kslices || !supports_mfma(p, 128)) return 1;
    const int64_t b128 = ((p.M + 127) / 128) * ((p.N + 127) / 128), b256 = ((p.M + 255) / 256) * ((p.N + 255) / 256);
    const int64_t bke = p.i8 ? 128 : 64;
    if (b128 > 64 || p.K < 4096) return 1;
    auto slices = [&](int64_t blocks, int64_t slots) {
        const int64_t want = std::min<int64_t>(slots / blocks, p.K / (8 * bke));   // at least eight k-tiles per slice
        int ks = 1;
        while (2 * ks <= want && 2 * ks <= 256 && p.K % (2 * ks * bke) == 0) ks *= 2;
        return ks;
    };
    // 256 x 256 blocks (one per CU) re-read A and B half as often as 128 x 128 blocks (two per CU) but cost more to
    // start and to finish: take them when they compute little padding, still fill the chip and keep long slices
    const int ks256 = supports_mfma(p, 256) ? slices(b256, 256) : 1;
    const bool big = b256 * 4 * 5 <= b128 * 6 && b256 * ks256 >= 200 && p.K / ks256 >= 4096;
    const int ks = big ? ks256 : slices(b128, 256);
    *tile = big ? 256 : 128;
    return ks;
}

hipError_t launch_mfma_ksplit(const Problem &p, int ksplit, int tile, void *workspace, hipStream_t s)
{
    if (ksplit < 2 || ksplit > 256 || p.batch != 1 || p.K % ksplit || !workspace || (p.M * p.N) % 4) return hipErrorInvalidValue;
    Problem q = p;
    q.batch = ksplit;                    // the batch index of the kernel serves as the slice index
    q.kslices = true;
    q.K = p.K / ksplit;
    q.lda = p.K;
    q.ldb = p.N;
    q.ldc = p.N;
    q.strideA = q.K;                     // slice b starts at column b * K/ksplit of A ...
    q.strideB = q.K * p.N;               // ... and at that row of B ...
    q.C = workspace;
    q.strideC = p.M * p.N;               // ... and leaves its partial product in slice b of the workspace
    if (hipError_t e = launch_mfma(q, tile, 16, s); e != hipSuccess) return e;
    const int64_t quads = p.M * p.N / 4;
    dim3 grid((unsigned)((quads + 255) / 256));
    if (p.i8) return launch_kernel(ws_join_slices_kernel<i32x4>, grid, dim3(256), s, (const i32x4 *)workspace, (i32x4 *)p.C, quads, ksplit);
    return launch_kernel(ws_join_slices_kernel<f32x4>, grid, dim3(256), s, (const f32x4 *)workspace, (f32x4 *)p.C, quads, ksplit);
}

hipError_t launch_mfma(const Problem &p, int tile, int mt, hipStream_t s)
{
    if (!supports_mfma(p, tile) || (mt != 16 && mt != 32)) return hipErrorInvalidValue;
    // 4 waves of 128x128 (256-block) or 64x64 (128-block), one per SIMD; in the 256-block the accumulators
    // fill the 256 AGPRs.  Eight waves of 128x64 read 50 % more LDS per MFMA and measured slower with
    // either MFMA shape.  mt chooses the MFMA shape: 16 is what the dispatcher uses (see the comment at Acc).
    if (mt == 16) {
        if (tile == 256)
            return p.i8 ? launch_cfg<Cfg<true, 256, 256, 2, 2, 16>, true>(p, s) : launch_cfg<Cfg<false, 256, 256, 2, 2, 16>, true>(p, s);
        return p.i8 ? launch_cfg<Cfg<true, 128, 128, 2, 2, 16>, true>(p, s) : launch_cfg<Cfg<false, 128, 128, 2, 2, 16>, true>(p, s);
    }
    if (tile == 256)
        return p.i8 ? launch_cfg<Cfg<true, 256, 256, 2, 2, 32>, false>(p, s) : launch_cfg<Cfg<false, 256, 256, 2, 2, 32>, false>(p, s);
    return p.i8 ? launch_cfg<Cfg<true, 128, 128, 2, 2, 32>, false>(p, s) : launch_cfg<Cfg<false, 128, 128, 2, 2, 32>, false>(p, s);
}

}  // namespace cyc

