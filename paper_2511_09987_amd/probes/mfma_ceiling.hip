// mfma_ceiling.hip -- stand-alone probe, not part of libcyclotron_mm: how fast can this chip run the
// MFMA instructions of the GEMM kernels when nothing else happens?  Every wave keeps its operand
// fragments and 256 accumulator registers in place and issues MFMAs of one shape (32x32 or 16x16)
// back to back on random-looking operands; no LDS, no global traffic inside the timed loop.  On a
// power-limited part this, not the datasheet number, is the ceiling a real GEMM on dense random
// data can approach, and the two shapes differ: the 16x16 one costs less energy per flop.
//
//   python -m paper_2511_09987_amd.build && ./paper_2511_09987_amd/probes/mfma_ceiling.bin
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <vector>

#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); return 1; } } while (0)

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef int i32x16 __attribute__((ext_vector_type(16)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// MT = 32: 4 x 4 operand fragments, 16 accumulators of 16 registers, 32x32 MFMAs.
// MT = 16: 8 x 8 operand fragments, 64 accumulators of 4 registers, 16x16 MFMAs (half as many
// outer iterations: the same flops per launch).
template <bool I8, int MT>
__global__ __launch_bounds__(256) void mfma_loop(const i32x4 *src, int *out, int iters, unsigned mask)
{
    constexpr int NF = MT == 32 ? 4 : 8;
    const unsigned t = blockIdx.x * 256 + threadIdx.x;
    i32x4 a[NF], b[NF];
#pragma unroll
    for (int i = 0; i < NF; ++i) { a[i] = src[(t * 2 * NF + i) & mask]; b[i] = src[(t * 2 * NF + NF + i) & mask]; }
    typedef typename std::conditional<MT == 32, typename std::conditional<I8, i32x16, f32x16>::type,
                                      typename std::conditional<I8, i32x4, f32x4>::type>::type acc_t;
    acc_t acc[NF * NF];
#pragma unroll
    for (int i = 0; i < NF * NF; ++i)
#pragma unroll
        for (int r = 0; r < MT * MT / 64; ++r) acc[i][r] = 0;
    for (int it = 0; it < (MT == 32 ? iters : iters / 2); ++it) {
#pragma unroll
        for (int i = 0; i < NF; ++i)
#pragma unroll
            for (int j = 0; j < NF; ++j) {
                acc_t &c = acc[i * NF + j];
                if constexpr (MT == 32 && I8) c = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[j], c, 0, 0, 0);
                else if constexpr (MT == 32) c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[i]), __builtin_bit_cast(bf16x8, b[j]), c, 0, 0, 0);
                else if constexpr (I8) c = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[i], b[j], c, 0, 0, 0);
                else c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a[i]), __builtin_bit_cast(bf16x8, b[j]), c, 0, 0, 0);
            }
#pragma unroll
        for (int i = 0; i < NF; ++i) a[i] = a[i] ^ (i32x4){it & 0x7f, it & 0x7f, it & 0x7f, it & 0x7f};   // low mantissa bits only
    }
    int s = 0;
#pragma unroll
    for (int i = 0; i < NF * NF; ++i) s += __builtin_bit_cast(int, acc[i][0]);
    if (s == 0x12345678) out[0] = s;
}

int main()
{
    const size_t n16 = 8u << 20;
    std::vector<unsigned short> hb(n16);
    std::vector<signed char> hi(n16 * 2);
    srand(1);
    for (auto &x : hb) {   // bf16: random sign and mantissa, magnitudes around 0.03 .. 1
        int e = 121 + rand() % 6;
        x = (unsigned short)(((rand() & 1) << 15) | (e << 7) | (rand() & 127));
    }
    for (auto &x : hi) x = (signed char)(rand() % 255 - 127);
    i32x4 *db, *di;
    int *out;
    CK(hipMalloc(&db, n16 * 2)); CK(hipMalloc(&di, n16 * 2)); CK(hipMalloc(&out, 4));
    CK(hipMemcpy(db, hb.data(), n16 * 2, hipMemcpyHostToDevice));
    CK(hipMemcpy(di, hi.data(), n16 * 2, hipMemcpyHostToDevice));
    const unsigned mask = (unsigned)(n16 * 2 / 16 - 1);
    hipDeviceProp_t prop;
    CK(hipGetDeviceProperties(&prop, 0));
    const int blocks = prop.multiProcessorCount, iters = 20000, launches = 10;
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    for (int rep = 0; rep < 2; ++rep)
        for (int mt : {32, 16})
            for (int i8 = 0; i8 < 2; ++i8) {
                auto run = [&] {
                    if (mt == 32 && i8) mfma_loop<true, 32><<<blocks, 256>>>(di, out, iters, mask);
                    else if (mt == 32) mfma_loop<false, 32><<<blocks, 256>>>(db, out, iters, mask);
                    else if (i8) mfma_loop<true, 16><<<blocks, 256>>>(di, out, iters, mask);
                    else mfma_loop<false, 16><<<blocks, 256>>>(db, out, iters, mask);
                };
                run();
                CK(hipDeviceSynchronize());
                CK(hipEventRecord(e0));
                for (int r = 0; r < launches; ++r) run();
                CK(hipEventRecord(e1));
                CK(hipDeviceSynchronize());
                float ms;
                CK(hipEventElapsedTime(&ms, e0, e1));
                const double ops = (double)launches * blocks * 4 * iters * 16 * 2.0 * 32 * 32 * (i8 ? 32 : 16);
                printf("%s %dx%d MFMA, registers only, %d CUs x 4 waves: %.0f %s\n", i8 ? "int8" : "bf16", mt, mt, blocks,
                       ops / ms / 1e9, i8 ? "TOP/s" : "TFLOP/s");
            }
    return 0;
}
