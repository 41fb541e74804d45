// cyc_attn.hip -- the FlashAttention-2 tile recurrence on gfx950.
//
// Paper, "FlashAttention-2 Recurrence": keys and values arrive in tiles J_t; every query i keeps a
// running maximum m_i, a running sum l_i and a running output o_i,
//     S_ij = alpha Q_i. K_j.^T,   mh = max(m_i, max_j S_ij),
//     l_i <- exp(m_i - mh) l_i + sum_j exp(S_ij - mh),   o_i <- exp(m_i - mh) o_i + sum_j exp(S_ij - mh) V_j.,
// and O_i. = o_i / l_i at the end.  The paper maps it with the query tile stationary on a processing
// element and K, V streaming past; so here: a wave holds 32 queries as MFMA operand registers for the
// whole kernel, a workgroup of eight waves (256 queries) streams tiles of 64 or 128 keys of K and V through LDS.
//
// Both products are computed transposed, which removes every shuffle between them:
//   S^T = K_tile Q^T   (A operand: 16 keys x 32 d from LDS; B operand: the stationary Q, whose row-major
//                       rows are exactly the operand layout).  Accumulator lane l then holds, for query
//                       l%16, the keys 4*(l/16) .. +3 of each 16-key block: all statistics of a query
//                       (m, l, the rescale factor) are per lane, and only the maximum needs the other
//                       three lanes of the query (two xor-shuffles per tile).
//   O^T = V^T P^T      (B operand: P^T straight from those accumulators, rounded to bfloat16 -- two
//                       16-key blocks side by side make the 8 k-slots of a lane, and the sum over keys
//                       does not care in which slot a key sits as long as V uses the same slots; A
//                       operand: V^T through the LDS transpose read, with that same key order.)
//                       Accumulator lane l holds, for query l%16, four consecutive d: the rescale by
//                       exp(m - mh) is a per-lane multiply and the final store is 16 bytes per lane.
// Arithmetic: Q, K, V bfloat16; S, m, l, o fp32; exp through the hardware exp2 with alpha*log2(e) folded
// into the scores; the probabilities enter the second product rounded to bfloat16 (nearest even), the
// running sum takes them unrounded.
#include "cyc_internal.h"

namespace cyc {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x2 __attribute__((ext_vector_type(2)));

#define CYC_LDS __attribute__((address_space(3)))

// Measured at batch 64, N = M = 4096 (TFLOP/s at d = 128 / d = 64): 64 queries per wave and 4 waves 599 / 463;
// 32 queries per wave and 8 waves (two per SIMD, so one wave's exponentials overlap the other's MFMAs)
// 938 / 848 with 64-key tiles and 1036 / 772 with 128-key tiles; 16 queries per wave and 16 waves 919 / 806.
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

// D: head dimension; KT: keys per tile (a multiple of 32)
template <int D, int KT>
__global__ __launch_bounds__(NWAVE * 64) void attn_kernel(const char *__restrict__ Q, const char *__restrict__ K,
                                                          const char *__restrict__ V, float *__restrict__ O, int N,
                                                          int M, float scale_log2e)
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
    const int64_t bz = blockIdx.y;
    Q += bz * (int64_t)N * ROW;
    K += bz * (int64_t)M * ROW;
    V += bz * (int64_t)M * ROW;
    O += bz * (int64_t)N * D;
    const int q0 = blockIdx.x * (NWAVE * QW) + w * QW;          // first query of this wave

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

    // ---- copies of a tile of K and of V into stage `st`; keys past M re-read key M-1 (masked below)
    uint32_t voffK[COPIES], voffV[COPIES];
    auto set_offsets = [&](int tile) __attribute__((always_inline)) {
#pragma unroll
        for (int x = 0; x < COPIES; ++x) {
            const int r = (w * COPIES + x) * RPC + l / CPR, slot = l % CPR;
            int key = tile * KT + r;
            key = key < M ? key : M - 1;
            voffK[x] = (uint32_t)key * ROW + ((slot ^ swzK(r)) << 4);
            voffV[x] = (uint32_t)key * ROW + ((slot ^ swzV(r)) << 4);
        }
    };
    auto issue_tile = [&](int st) __attribute__((always_inline)) {
#pragma unroll
        for (int x = 0; x < COPIES; ++x) {
            copy16(K, voffK[x], lds_base + st * TILE_BYTES + (w * COPIES + x) * 1024);
            copy16(V, voffV[x], lds_base + (2 + st) * TILE_BYTES + (w * COPIES + x) * 1024);
        }
    };

    // ---- running state of this lane's queries (one per 16-query block jq): maximum in the log2 domain, this lane's
    // share of the sum, and O^T accumulators [d tile][query tile]
    float m2[QB], lsum[QB];
    f32x4 acc_o[DT][QB];
#pragma unroll
    for (int jq = 0; jq < QB; ++jq) {
        m2[jq] = -__builtin_inff();
        lsum[jq] = 0.0f;
#pragma unroll
        for (int id = 0; id < DT; ++id) acc_o[id][jq] = (f32x4){0, 0, 0, 0};
    }

    const int ntiles = (M + KT - 1) / KT;
    set_offsets(0);
    issue_tile(0);
    for (int t = 0; t < ntiles; ++t) {
        const int st = t & 1;
        // tile t has landed in stage st; every wave is done with stage st^1 (tile t-1)
        asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
        if (t + 1 < ntiles) {
            set_offsets(t + 1);
            issue_tile(st ^ 1);
        }
        CYC_LDS char *Kt = lds + st * TILE_BYTES, *Vt = lds + (2 + st) * TILE_BYTES;

        // ---- S^T = K_tile Q^T : [key block ik][query block jq]
        f32x4 s[KB][QB];
#pragma unroll
        for (int ik = 0; ik < KB; ++ik)
#pragma unroll
            for (int jq = 0; jq < QB; ++jq) s[ik][jq] = (f32x4){0, 0, 0, 0};
#pragma unroll
        for (int ks = 0; ks < DS; ++ks) {
            i32x4 kf[KB];
#pragma unroll
            for (int ik = 0; ik < KB; ++ik) {
                const int r = ik * 16 + lq;                       // A operand: key row l%16 of block ik, chunk 4 ks + l/16
                kf[ik] = *(CYC_LDS i32x4 *)(Kt + r * ROW + (((ks * 4 + g) ^ swzK(r)) << 4));
            }
#pragma unroll
            for (int ik = 0; ik < KB; ++ik)
#pragma unroll
                for (int jq = 0; jq < QB; ++jq)
                    s[ik][jq] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kf[ik]), __builtin_bit_cast(bf16x8, qf[jq][ks]), s[ik][jq], 0, 0, 0);
        }
        // accumulator register r of lane l: key 16 ik + 4 (l/16) + r of the tile, query 16 jq + l%16
        if ((t + 1) * KT > M) {                                   // last, ragged tile: keys past M take no weight
#pragma unroll
            for (int ik = 0; ik < KB; ++ik)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (t * KT + ik * 16 + 4 * g + r >= M) {
#pragma unroll
                        for (int jq = 0; jq < QB; ++jq) s[ik][jq][r] = -__builtin_inff();
                    }
        }

        // ---- running maximum, rescale factor, probabilities
        i32x4 pf[QB][KB / 2];                                           // P^T as B operand: [query block][32-key step]
#pragma unroll
        for (int jq = 0; jq < QB; ++jq) {
            float top = s[0][jq][0];
#pragma unroll
            for (int ik = 0; ik < KB; ++ik)
#pragma unroll
                for (int r = 0; r < 4; ++r) top = __builtin_fmaxf(top, s[ik][jq][r]);
            top = __builtin_fmaxf(top, __shfl_xor(top, 16));
            top = __builtin_fmaxf(top, __shfl_xor(top, 32));
            const float mh = __builtin_fmaxf(m2[jq], top * scale_log2e);
            const float keep = __builtin_amdgcn_exp2f(m2[jq] - mh);   // exp(m - mh); 0 on the first tile
            m2[jq] = mh;
            float part = 0.0f;
            bf16x8 pk[KB / 2];
#pragma unroll
            for (int ik = 0; ik < KB; ++ik)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[ik][jq][r], scale_log2e, -mh));
                    part += p;
                    pk[ik >> 1][(ik & 1) * 4 + r] = (__bf16)p;   // k-slot: block ik&1 of the 32-key step ik/2
                }
            lsum[jq] = __builtin_fmaf(keep, lsum[jq], part);
#pragma unroll
            for (int sk = 0; sk < KB / 2; ++sk) pf[jq][sk] = __builtin_bit_cast(i32x4, pk[sk]);
            // most tiles leave the maximum of every query of the wave where it was: nothing to rescale then
            if (!__builtin_amdgcn_ballot_w64(keep != 1.0f)) continue;
#pragma unroll
            for (int id = 0; id < DT; ++id) acc_o[id][jq] *= keep;
        }

        // ---- O^T += V^T P^T : A operand lane: d = 16 id + l%16; k-slots 0..3 = keys 32 sk + 4 (l/16) .. +3,
        // k-slots 4..7 = the same keys of the next 16-key block (the order P^T was packed in)
#pragma unroll
        for (int sk = 0; sk < KB / 2; ++sk)
#pragma unroll
            for (int id = 0; id < DT; ++id) {
                const int klo = sk * 32 + 4 * g + (lq >> 2), khi = klo + 16;      // rows the transpose read points at
                const int chunk = (id * 16 + 4 * (lq & 3)) >> 3, within = ((id * 16 + 4 * (lq & 3)) & 7) * 2;
                const i32x2 lo = __builtin_bit_cast(i32x2, __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
                    (CYC_LDS bf16x4 *)(Vt + klo * ROW + ((chunk ^ swzV(klo)) << 4) + within)));
                const i32x2 hi = __builtin_bit_cast(i32x2, __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
                    (CYC_LDS bf16x4 *)(Vt + khi * ROW + ((chunk ^ swzV(khi)) << 4) + within)));
                const i32x4 vf = mfma_frag(lo, hi);
#pragma unroll
                for (int jq = 0; jq < QB; ++jq)
                    acc_o[id][jq] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vf), __builtin_bit_cast(bf16x8, pf[jq][sk]), acc_o[id][jq], 0, 0, 0);
            }
    }

    // ---- O_i. = o_i / l_i.  Accumulator register r of lane l: d = 16 id + 4 (l/16) + r, query 16 jq + l%16.
#pragma unroll
    for (int jq = 0; jq < QB; ++jq) {
        float tot = lsum[jq];
        tot += __shfl_xor(tot, 16);
        tot += __shfl_xor(tot, 32);
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
    dim3 grid((unsigned)((N + NWAVE * QW - 1) / (NWAVE * QW)), (unsigned)batch);
    if (d == 128)
        hipLaunchKernelGGL((attn_kernel<128, 128>), grid, dim3(NWAVE * 64), 0, s, (const char *)Q, (const char *)K,
                           (const char *)V, (float *)O, (int)N, (int)M, scale_log2e);
    else
        hipLaunchKernelGGL((attn_kernel<64, 64>), grid, dim3(NWAVE * 64), 0, s, (const char *)Q, (const char *)K,
                           (const char *)V, (float *)O, (int)N, (int)M, scale_log2e);
    return hipGetLastError();
}

}  // namespace cyc
