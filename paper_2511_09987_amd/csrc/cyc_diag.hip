// cyc_diag.hip -- two measurement aids exported beside the recurrence kernels (declared in cyclotron_mm.h).
//
// cyc_diag_mfma_ceiling: what the matrix pipes of this chip sustain when nothing else happens.  Every wave keeps its
// operand fragments and 256 accumulator registers in place and issues MFMAs of one shape back to back on
// random-looking operands; no LDS, no memory traffic in the loop.  On a power-limited part this, not the datasheet
// figure, is what a GEMM on dense random data can approach, and it differs between the two MFMA shapes.
//
// cyc_diag_clock: one wave that reads the shader clock counter and the constant 100 MHz counter for a given time
// while other kernels run, which gives the engine clock the chip sustains under that load.
//
// cyc_diag_issue_mix: what a SIMD issues beside its MFMAs.  MFMA, vector-ALU and LDS instructions of a SIMD's waves
// go through one issue port; a kernel whose matrix pipe is not full may be out of issue slots instead.  Rounds of the
// same matrix work (16 MFMAs of 16 x 16 x 32 or 8 of 32 x 32 x 16, bf16: 256 cycles of the matrix pipe) with a given
// number of other instructions spread evenly between them, everything from registers (or a few LDS words), one or
// two waves per SIMD: the time per round against the 256 cycles says what the other instructions cost.
#include "../../include/cyclotron_mm.h"
#include "cyc_internal.h"

namespace cyc {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef int i32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint32_t mix32(uint32_t x)
{
    x ^= x >> 16; x *= 0x7feb352du;
    x ^= x >> 15; x *= 0x846ca68bu;
    return x ^ (x >> 16);
}
// two bf16 values with random sign and mantissa and magnitudes around 0.03 .. 1, or four random int8 values
template <bool I8> __device__ __forceinline__ int operand_word(uint32_t h)
{
    if (I8) return (int)h;
    const uint32_t lo = ((h & 1) << 15) | ((121 + ((h >> 1) % 6)) << 7) | ((h >> 4) & 127);
    const uint32_t hi = (((h >> 11) & 1) << 15) | ((121 + ((h >> 12) % 6)) << 7) | ((h >> 15) & 127);
    return (int)(lo | (hi << 16));
}

// MT = 32: 4 x 4 operand fragments, 16 accumulators of 16 registers.  MT = 16: 8 x 8 fragments, 64 accumulators of
// 4 registers, half as many outer iterations: the same operations per launch.
template <bool I8, int MT>
__global__ __launch_bounds__(256) void mfma_ceiling_kernel(int *sink, int iters)
{
    constexpr int NF = MT == 32 ? 4 : 8;
    const uint32_t t = blockIdx.x * 256 + threadIdx.x;
    i32x4 a[NF], b[NF];
#pragma unroll
    for (int i = 0; i < NF; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            a[i][r] = operand_word<I8>(mix32(t * 64 + i * 4 + r));
            b[i][r] = operand_word<I8>(mix32(t * 64 + 32 + i * 4 + r));
        }
    typedef typename std::conditional<MT == 32, typename std::conditional<I8, i32x16, f32x16>::type,
                                      typename std::conditional<I8, i32x4, f32x4>::type>::type acc_t;
    acc_t acc[NF * NF];
#pragma unroll
    for (int i = 0; i < NF * NF; ++i)
#pragma unroll
        for (int r = 0; r < MT * MT / 64; ++r) acc[i][r] = 0;
    // four rounds over all accumulators per change of the operands: the vector instructions that change them take
    // issue slots from the MFMAs, and the point here is the MFMA rate
    for (int it = 0; it < (MT == 32 ? iters : iters / 2) / 4; ++it) {
#pragma unroll
        for (int rep = 0; rep < 4; ++rep)
#pragma unroll
        for (int i = 0; i < NF; ++i)
#pragma unroll
            for (int j = 0; j < NF; ++j) {
                // written as asm with the accumulator tied to the destination: with all 256 accumulator registers
                // occupied the register allocator otherwise rotates them through moves between the MFMAs
                acc_t &c = acc[i * NF + j];
                if constexpr (MT == 32 && I8) asm volatile("v_mfma_i32_32x32x32_i8 %0, %1, %2, %0" : "+a"(c) : "v"(a[i]), "v"(b[j]));
                else if constexpr (MT == 32) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(a[i]), "v"(b[j]));
                else if constexpr (I8) asm volatile("v_mfma_i32_16x16x64_i8 %0, %1, %2, %0" : "+a"(c) : "v"(a[i]), "v"(b[j]));
                else asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(a[i]), "v"(b[j]));
            }
        // the operands change a little every iteration (low mantissa bits only), as they would in a real k loop
#pragma unroll
        for (int i = 0; i < NF; ++i) a[i] = a[i] ^ (i32x4){it & 0x7f, it & 0x7f, it & 0x7f, it & 0x7f};
    }
    // (the compiler's hazard logic does not look inside asm: wait out the last MFMAs before reading their results)
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
    int s = 0;
#pragma unroll
    for (int i = 0; i < NF * NF; ++i) s += __builtin_bit_cast(int, acc[i][0]);
    if (s == 0x12345678) sink[0] = s;      // keeps the loop alive; practically never true
}

// SHAPE 16 | 32; KIND 0: v_fma_f32, 1: v_exp_f32, 2: ds_read_b128; NV: other instructions per round (a multiple of 16)
template <int SHAPE, int KIND, int NV>
__global__ __launch_bounds__(512) void issue_mix_kernel(int *sink, int iters, float seed)
{
    __shared__ __attribute__((aligned(16))) int words[64 * 4];
    if (threadIdx.x < 256) words[threadIdx.x] = (int)threadIdx.x;
    __syncthreads();
    const i32x4 a = {(int)threadIdx.x, 0x3f803f80, 0x40004000, 0x3f003f00}, b = {0x3f803f80, 0x3fc03fc0, 0x3f803f80, (int)threadIdx.x};
    f32x4 acc4[16];
    f32x16 acc16[8];
#pragma unroll
    for (int i = 0; i < 16; ++i) acc4[i] = (f32x4){0, 0, 0, 0};
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc16[i][r] = 0.0f;
    float v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = seed * (float)(i + 1) + (float)threadIdx.x * 1e-3f;
    i32x4 ld = {0, 0, 0, 0};
    const unsigned ldaddr = (unsigned)(uintptr_t)(__attribute__((address_space(3))) int *)words + (threadIdx.x & 63) * 16;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int m = 0; m < 16; ++m) {
            if (SHAPE == 16) asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc4[m]) : "v"(a), "v"(b));
            else if ((m & 1) == 0) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc16[m / 2]) : "v"(a), "v"(b));
#pragma unroll
            for (int k = 0; k < NV / 16; ++k) {
                float &x = v[(m * (NV / 16) + k) & 7];
                if (KIND == 0) asm volatile("v_fma_f32 %0, %0, %1, %1" : "+v"(x) : "v"(seed));
                else if (KIND == 1) asm volatile("v_exp_f32 %0, %0" : "+v"(x));
                else asm volatile("ds_read_b128 %0, %1" : "=v"(ld) : "v"(ldaddr));
            }
        }
        if (KIND == 2) asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(ld));
    }
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += acc4[i][0];
#pragma unroll
    for (int i = 0; i < 8; ++i) s += acc16[i][0];
#pragma unroll
    for (int i = 0; i < 8; ++i) s += v[i];
    s += (float)ld[0];
    if (s == 1.2345f) sink[0] = 1;         // keeps the loop alive; practically never true
}

template <int SHAPE, int KIND>
hipError_t launch_issue_mix(int per_round, dim3 grid, dim3 block, hipStream_t s, int *sink, int iters)
{
    switch (per_round) {
        case 0: return launch_kernel(issue_mix_kernel<SHAPE, 0, 0>, grid, block, s, sink, iters, 0.37f);
        case 16: return launch_kernel(issue_mix_kernel<SHAPE, KIND, 16>, grid, block, s, sink, iters, 0.37f);
        case 32: return launch_kernel(issue_mix_kernel<SHAPE, KIND, 32>, grid, block, s, sink, iters, 0.37f);
        case 48: return launch_kernel(issue_mix_kernel<SHAPE, KIND, 48>, grid, block, s, sink, iters, 0.37f);
        case 64: return launch_kernel(issue_mix_kernel<SHAPE, KIND, 64>, grid, block, s, sink, iters, 0.37f);
        case 96: return launch_kernel(issue_mix_kernel<SHAPE, KIND, 96>, grid, block, s, sink, iters, 0.37f);
        default: return hipErrorInvalidValue;
    }
}

// D = A B + C, 16 x 16 x 4 per tile, one v_mfma_f32_16x16x4_f32 each.  A: tiles x 16 x 4 (row, k), B: tiles x 4 x 16
// (k, column), C and D: tiles x 16 x 16, all row-major.  Operand lane l: row (column) l%16, k = l/16; accumulator
// register r of lane l: row 4 (l/16) + r, column l%16.
__global__ __launch_bounds__(64) void mfma_f32_tiles_kernel(const float *__restrict__ A, const float *__restrict__ B,
                                                            const float *__restrict__ C, float *__restrict__ D, int64_t tiles)
{
    const int l = threadIdx.x;
    for (int64_t t = blockIdx.x; t < tiles; t += gridDim.x) {
        const float a = A[t * 64 + (l % 16) * 4 + l / 16], b = B[t * 64 + (l / 16) * 16 + l % 16];
        f32x4 c;
#pragma unroll
        for (int r = 0; r < 4; ++r) c[r] = C[t * 256 + (4 * (l / 16) + r) * 16 + l % 16];
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
#pragma unroll
        for (int r = 0; r < 4; ++r) D[t * 256 + (4 * (l / 16) + r) * 16 + l % 16] = c[r];
    }
}

__global__ __launch_bounds__(64) void clock_kernel(uint64_t *out, int64_t ticks)
{
    const uint64_t w0 = wall_clock64(), c0 = clock64();
    uint64_t w1 = w0;
    // a sleep of 32 is 2048 cycles, about a microsecond: the round count is bounded as well, so that the wave ends
    // even if the 100 MHz counter should not advance
    for (int64_t round = 0; (int64_t)(w1 - w0) < ticks && round < ticks / 16 + 4096; ++round) {
        __builtin_amdgcn_s_sleep(32);
        w1 = wall_clock64();
    }
    const uint64_t c1 = clock64();
    if (threadIdx.x == 0) {
        out[0] = c1 - c0;
        out[1] = w1 - w0;
    }
}

}  // namespace
}  // namespace cyc

extern "C" {

int cyc_diag_mfma_ceiling(int dtype, int mfma_shape, int64_t iters, void *sink, double *ops, void *stream)
{
    if (dtype != CYC_BF16_F32 && dtype != CYC_I8_I32) return CYC_ERR_DTYPE;
    if ((mfma_shape != 16 && mfma_shape != 32) || iters < 8 || iters > (1 << 24) || (iters & 7)) return CYC_ERR_SHAPE;
    if (!sink) return CYC_ERR_NULL;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
        return CYC_ERR_LAUNCH;
    const bool i8 = dtype == CYC_I8_I32;
    // per wave and outer iteration 16 MFMAs of 32 x 32 x (16 | 32), i.e. 2 * 32 * 32 * k operations each
    if (ops) *ops = (double)cus * 4 * (double)iters * 16 * 2.0 * 32 * 32 * (i8 ? 32 : 16);
    dim3 grid((unsigned)cus), block(256);
    hipStream_t s = (hipStream_t)stream;
    hipError_t e;
    if (mfma_shape == 32)
        e = i8 ? cyc::launch_kernel(cyc::mfma_ceiling_kernel<true, 32>, grid, block, s, (int *)sink, (int)iters)
               : cyc::launch_kernel(cyc::mfma_ceiling_kernel<false, 32>, grid, block, s, (int *)sink, (int)iters);
    else
        e = i8 ? cyc::launch_kernel(cyc::mfma_ceiling_kernel<true, 16>, grid, block, s, (int *)sink, (int)iters)
               : cyc::launch_kernel(cyc::mfma_ceiling_kernel<false, 16>, grid, block, s, (int *)sink, (int)iters);
    return e == hipSuccess ? CYC_OK : CYC_ERR_LAUNCH;
}

int cyc_diag_issue_mix(int mfma_shape, int other_kind, int others_per_round, int waves_per_simd, int64_t iters, void *sink,
                       double *ops, void *stream)
{
    if ((mfma_shape != 16 && mfma_shape != 32) || other_kind < 0 || other_kind > 2 || (waves_per_simd != 1 && waves_per_simd != 2) ||
        iters < 1 || iters > (1 << 24))
        return CYC_ERR_SHAPE;
    if (others_per_round != 0 && others_per_round != 16 && others_per_round != 32 && others_per_round != 48 && others_per_round != 64 &&
        others_per_round != 96)
        return CYC_ERR_SHAPE;
    if (!sink) return CYC_ERR_NULL;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
        return CYC_ERR_LAUNCH;
    // per wave and round 16 MFMAs of 16 x 16 x 32 (or 8 of twice that): 2 * 16 * 16 * 32 operations each
    if (ops) *ops = (double)cus * 4 * waves_per_simd * (double)iters * 16 * 2.0 * 16 * 16 * 32;
    dim3 grid((unsigned)cus), block(256 * waves_per_simd);
    hipStream_t s = (hipStream_t)stream;
    hipError_t e;
    if (mfma_shape == 16)
        e = other_kind == 0   ? cyc::launch_issue_mix<16, 0>(others_per_round, grid, block, s, (int *)sink, (int)iters)
            : other_kind == 1 ? cyc::launch_issue_mix<16, 1>(others_per_round, grid, block, s, (int *)sink, (int)iters)
                              : cyc::launch_issue_mix<16, 2>(others_per_round, grid, block, s, (int *)sink, (int)iters);
    else
        e = other_kind == 0   ? cyc::launch_issue_mix<32, 0>(others_per_round, grid, block, s, (int *)sink, (int)iters)
            : other_kind == 1 ? cyc::launch_issue_mix<32, 1>(others_per_round, grid, block, s, (int *)sink, (int)iters)
                              : cyc::launch_issue_mix<32, 2>(others_per_round, grid, block, s, (int *)sink, (int)iters);
    return e == hipSuccess ? CYC_OK : CYC_ERR_LAUNCH;
}

int cyc_diag_mfma_f32_tiles(const void *A, const void *B, const void *C, void *D, int64_t tiles, void *stream)
{
    if (tiles < 0 || tiles > (1 << 24)) return CYC_ERR_SHAPE;
    if (tiles == 0) return CYC_OK;
    if (!A || !B || !C || !D) return CYC_ERR_NULL;
    if (((uintptr_t)A | (uintptr_t)B | (uintptr_t)C | (uintptr_t)D) & 3) return CYC_ERR_SHAPE;
    const unsigned blocks = (unsigned)(tiles < 4096 ? tiles : 4096);
    const hipError_t e = cyc::launch_kernel(cyc::mfma_f32_tiles_kernel, dim3(blocks), dim3(64), (hipStream_t)stream, (const float *)A,
                                            (const float *)B, (const float *)C, (float *)D, tiles);
    return e == hipSuccess ? CYC_OK : CYC_ERR_LAUNCH;
}

int cyc_diag_clock(void *out, int64_t microseconds, void *stream)
{
    if (!out) return CYC_ERR_NULL;
    if (microseconds < 1 || microseconds > 2000000 || ((uintptr_t)out & 7)) return CYC_ERR_SHAPE;
    const hipError_t e = cyc::launch_kernel(cyc::clock_kernel, dim3(1), dim3(64), (hipStream_t)stream, (uint64_t *)out,
                                            microseconds * 100);
    return e == hipSuccess ? CYC_OK : CYC_ERR_LAUNCH;
}

}  // extern "C"
