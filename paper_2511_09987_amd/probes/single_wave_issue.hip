// single_wave_issue.hip -- stand-alone probe, not part of libcyclotron_mm: how fast does ONE wave issue fp32
// multiply-adds when nobody else is on its SIMD?  The column recurrences of the triangular solve and of the
// Cholesky tiles run in one wave per 64 rows (or right-hand sides), so this is the rate that bounds them.
// One workgroup of 64 threads; streams of v_fmac_f32 (4-byte encoding) and v_fma_f32 (8-byte encoding), each
// either one dependent chain or four independent chains side by side; in a loop of 64 instructions that stays
// in the instruction cache, and as straight-line code of 8000 instructions that is fetched once.
// Measured on MI355X (cycles of the shader clock per instruction, three launches each):
//                                         one dependent chain     four chains
//     loop,          fmac (4 bytes)       8.3                     5.4
//     loop,          fma  (8 bytes)       8.3 - 10.7              5.7 - 7.3
//     straight line, fmac (4 bytes)       8.1 - 8.3               5.1 - 5.2
//     straight line, fma  (8 bytes)       8.6 - 10.4              5.3 - 6.9
// A multiply-add that waits for the one before it issues every ~8 cycles, an independent one every ~5; cold
// straight-line code runs as fast as a loop, so long unrolled kernels are fine and dependent chains are not; the
// 8-byte encoding (needed for a negated operand) is up to a quarter slower than the 4-byte one and less steady.
// The tile kernels therefore run four chains side by side, fill the division chains with independent work, and
// keep the negated value of a finished entry so that the multiply-adds take the short encoding.
//
//   python -m paper_2511_09987_amd.build && ./paper_2511_09987_amd/probes/single_wave_issue.bin
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("%s: %s\n", #x, hipGetErrorString(e_)); exit(1); } } while (0)

#define FMAC(t, a, b) asm volatile("v_fmac_f32 %0, %1, %2" : "+v"(t) : "v"(a), "v"(b))
#define FMA3(t, a, b) asm volatile("v_fma_f32 %0, -%1, %2, %0" : "+v"(t) : "v"(a), "v"(b))

// MODE 0: fmac, one chain; 1: fmac, four chains; 2: fma, one chain; 3: fma, four chains
template <int MODE, int N>
__device__ __forceinline__ void body(float (&t)[4], float a, float b)
{
#pragma unroll
    for (int i = 0; i < N / 4; ++i) {
        if (MODE == 0) { FMAC(t[0], a, b); FMAC(t[0], a, b); FMAC(t[0], a, b); FMAC(t[0], a, b); }
        if (MODE == 1) { FMAC(t[0], a, b); FMAC(t[1], a, b); FMAC(t[2], a, b); FMAC(t[3], a, b); }
        if (MODE == 2) { FMA3(t[0], a, b); FMA3(t[0], a, b); FMA3(t[0], a, b); FMA3(t[0], a, b); }
        if (MODE == 3) { FMA3(t[0], a, b); FMA3(t[1], a, b); FMA3(t[2], a, b); FMA3(t[3], a, b); }
    }
}

template <int MODE, int N>
__global__ __launch_bounds__(64) void probe(float *out, long long *cycles, int iters)
{
    float t[4] = {(float)threadIdx.x, 1.0f, 2.0f, 3.0f};
    const float a = 1e-3f * threadIdx.x, b = 0.5f;
    const long long c0 = __builtin_readcyclecounter();
    for (int it = 0; it < iters; ++it) body<MODE, N>(t, a, b);
    const long long c1 = __builtin_readcyclecounter();
    out[threadIdx.x] = t[0] + t[1] + t[2] + t[3];
    if (threadIdx.x == 0) *cycles = c1 - c0;
}

template <int MODE, int N>
void run(const char *name, int iters, float *out, long long *cycles)
{
    for (int rep = 0; rep < 3; ++rep) {
        hipEvent_t e0, e1;
        CK(hipEventCreate(&e0));
        CK(hipEventCreate(&e1));
        CK(hipEventRecord(e0));
        probe<MODE, N><<<1, 64>>>(out, cycles, iters);
        CK(hipEventRecord(e1));
        CK(hipDeviceSynchronize());
        float ms;
        CK(hipEventElapsedTime(&ms, e0, e1));
        long long h;
        CK(hipMemcpy(&h, cycles, 8, hipMemcpyDeviceToHost));
        const double n = (double)N * iters;
        printf("%-46s launch %d: %8.0f instructions  %8.2f us  %.2f cycles / instruction\n", name, rep, n, ms * 1e3, h / n);
    }
}

int main()
{
    float *out;
    long long *cycles;
    CK(hipMalloc(&out, 256));
    CK(hipMalloc(&cycles, 8));
    run<0, 64>("loop 64 x 2000, one chain, fmac (4 bytes)", 2000, out, cycles);
    run<1, 64>("loop 64 x 2000, four chains, fmac (4 bytes)", 2000, out, cycles);
    run<2, 64>("loop 64 x 2000, one chain, fma (8 bytes)", 2000, out, cycles);
    run<3, 64>("loop 64 x 2000, four chains, fma (8 bytes)", 2000, out, cycles);
    run<0, 8000>("straight line 8000, one chain, fmac (4 bytes)", 1, out, cycles);
    run<1, 8000>("straight line 8000, four chains, fmac (4 bytes)", 1, out, cycles);
    run<2, 8000>("straight line 8000, one chain, fma (8 bytes)", 1, out, cycles);
    run<3, 8000>("straight line 8000, four chains, fma (8 bytes)", 1, out, cycles);
    CK(hipFree(out));
    CK(hipFree(cycles));
    return 0;
}
