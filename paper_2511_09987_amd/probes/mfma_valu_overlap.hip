// mfma_valu_overlap.hip -- stand-alone probe, not part of libcyclotron_mm: do matrix-core (MFMA) and
// vector-ALU instructions overlap on a SIMD of this chip?  Streams of 16x16x32 bf16 MFMAs, of v_fma_f32 and of
// v_exp_f32, alone, interleaved in one wave, and from separate waves on the same SIMD; 1024 workgroups, so
// every SIMD holds 4 (256 threads) or 8 (512 threads) waves.  Measured on MI355X (ms for 4000 iterations):
//     16 MFMA                   2.06      (16 cycles per MFMA at 2 GHz: the pipe is full)
//     48 fma                    1.00      16 exp   0.98
//     16 x (MFMA, 3 fma)        2.76      one wave issues both      -> 0.70 of the 1.00 is added
//     16 x (MFMA, exp)          2.34                                -> 0.28 of the 0.98 is added
//     MFMA waves + fma waves    2.71      separate waves            -> 0.65 added
//     MFMA waves + exp waves    2.12                                -> 0.07 added
// A plain vector instruction beside MFMAs costs most of what it costs alone, whichever wave issues it; the
// transcendental unit runs beside the matrix cores almost for free.  The attention kernel therefore gains from
// fewer vector instructions, not from moving them away from the MFMAs.
//
//   python -m paper_2511_09987_amd.build && ./paper_2511_09987_amd/probes/mfma_valu_overlap.bin
#include <hip/hip_runtime.h>
#include <cstdio>
#pragma clang diagnostic ignored "-Wunused-value"
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
#define MF(i) acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[i], 0, 0, 0);
#define FMA3(x, y, z) asm volatile("v_fma_f32 %0, %0, %3, %4\n\tv_fma_f32 %1, %1, %3, %4\n\tv_fma_f32 %2, %2, %3, %4" : "+v"(x), "+v"(y), "+v"(z) : "v"(c1), "v"(c2));
#define EXP1(x) asm volatile("v_exp_f32 %0, %0" : "+v"(x));
template <int MODE>
__global__ __launch_bounds__(512) void k(float *out, int iters)
{
    const int w = threadIdx.x >> 6;
    bf16x8 a, b;
    for (int i = 0; i < 8; ++i) { a[i] = (__bf16)(threadIdx.x * 0.001f); b[i] = (__bf16)(i * 0.5f); }
    f32x4 acc[16];
    for (int i = 0; i < 16; ++i) acc[i] = (f32x4){0, 0, 0, 0};
    float v[12];
    for (int i = 0; i < 12; ++i) v[i] = threadIdx.x * 0.01f + i;
    float c1 = 0.999f, c2 = 0.001f;
    const bool do_m = MODE == 0 || MODE == 2 || MODE == 5 || ((MODE == 3 || MODE == 6) && w < 4);
    const bool do_v = MODE == 1 || (MODE == 3 && w >= 4);
    const bool do_e = MODE == 4 || (MODE == 6 && w >= 4);
    for (int it = 0; it < iters; ++it) {
        if (MODE == 2) {
#pragma unroll
            for (int i = 0; i < 16; ++i) { MF(i) FMA3(v[(3 * i) % 12], v[(3 * i + 1) % 12], v[(3 * i + 2) % 12]) }
        } else if (MODE == 5) {
#pragma unroll
            for (int i = 0; i < 16; ++i) { MF(i) EXP1(v[i % 12]) }
        } else {
            if (do_m) {
#pragma unroll
                for (int i = 0; i < 16; ++i) { MF(i) }
            }
            if (do_v) {
#pragma unroll
                for (int i = 0; i < 16; ++i) { FMA3(v[(3 * i) % 12], v[(3 * i + 1) % 12], v[(3 * i + 2) % 12]) }
            }
            if (do_e) {
#pragma unroll
                for (int i = 0; i < 16; ++i) { EXP1(v[i % 12]) }
            }
        }
    }
    float s = 0;
    for (int i = 0; i < 16; ++i) s += acc[i][0] + acc[i][3];
    for (int i = 0; i < 12; ++i) s += v[i];
    if (s == 123.456f) out[threadIdx.x] = s;
}
template <int MODE> void run(const char *name, int threads, float *out)
{
    const int iters = 4000;
    hipEvent_t e0, e1; hipEventCreate(&e0); hipEventCreate(&e1);
    k<MODE><<<1024, threads>>>(out, 100);
    hipDeviceSynchronize();
    hipEventRecord(e0);
    k<MODE><<<1024, threads>>>(out, iters);
    hipEventRecord(e1); hipEventSynchronize(e1);
    float ms; hipEventElapsedTime(&ms, e0, e1);
    // 1024 blocks over 256 CUs: 4 blocks per CU in sequence or together (registers allow); per SIMD: blocks*waves/4
    printf("%-44s threads %3d: %8.3f ms  -> %7.1f ns per iteration per block-wave\n", name, threads, ms, ms * 1e6 / iters);
    fflush(stdout);
}
int main()
{
    float *out; hipMalloc(&out, 4096);
    run<0>("0 mfma only (16/iter), 1 wave/SIMD", 256, out);
    run<1>("1 fma only (48/iter), 1 wave/SIMD", 256, out);
    run<4>("4 exp only (16/iter), 1 wave/SIMD", 256, out);
    run<2>("2 same wave: 16 x (mfma + 3 fma)", 256, out);
    run<5>("5 same wave: 16 x (mfma + exp)", 256, out);
    run<3>("3 two waves/SIMD: mfma wave + fma wave", 512, out);
    run<6>("6 two waves/SIMD: mfma wave + exp wave", 512, out);
    run<0>("0 mfma only, 2 waves/SIMD", 512, out);
    run<1>("1 fma only, 2 waves/SIMD", 512, out);
    hipFree(out);
    return 0;
}
