// phased_division_check.hip -- stand-alone check, not part of libcyclotron_mm: the division that cyc_wave.h writes out
// in phases gives, bit for bit, what the compiler's own operator/ gives, on 2^32 pairs: every numerator pattern
// against a denominator drawn from a counter-based hash, with special values (zeros, infinities, NaN, the smallest
// denormal, the largest and the smallest normal number) mixed in.  Prints the number of mismatches (NaN equals NaN);
// exit status 1 if there is any.  Last run on MI355X: 0.
//
//   python -m paper_2511_09987_amd.build && ./paper_2511_09987_amd/probes/phased_division_check.bin
#include "../csrc/cyc_wave.h"

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("%s: %s\n", #x, hipGetErrorString(e_)); exit(1); } } while (0)

__device__ __forceinline__ bool same(float a, float b)
{
    return __builtin_bit_cast(uint32_t, a) == __builtin_bit_cast(uint32_t, b) || (a != a && b != b);
}

__device__ __forceinline__ uint32_t hash(uint32_t v)
{
    v ^= v >> 16; v *= 0x7feb352dU; v ^= v >> 15; v *= 0x846ca68bU; v ^= v >> 16;
    return v;
}

// thread t checks the numerator patterns t, t + T, t + 2T, ... (T threads in all)
__global__ __launch_bounds__(256) void check(unsigned long long *bad)
{
    const uint32_t T = gridDim.x * blockDim.x, t0 = blockIdx.x * blockDim.x + threadIdx.x;
    const uint32_t special[8] = {0x00000000u, 0x80000000u, 0x7f800000u, 0xff800000u, 0x7fc00000u, 0x00000001u, 0x7f7fffffu, 0x00800000u};
    unsigned long long mismatches = 0;
    for (uint64_t p = t0; p < (1ull << 32); p += T) {
        const float num = __builtin_bit_cast(float, (uint32_t)p);
        const uint32_t h = hash((uint32_t)p);
        const float den = __builtin_bit_cast(float, (h & 0xff) < 8 ? special[h & 7] : h);
        cyc::Division dv;
        dv.phase0(num, den);
        dv.phase1();
        dv.phase2();
        if (!same(dv.phase3(), num / den)) ++mismatches;
    }
    if (mismatches) atomicAdd(bad, mismatches);
}

int main()
{
    unsigned long long *bad, h;
    CK(hipMalloc(&bad, 8));
    CK(hipMemset(bad, 0, 8));
    check<<<4096, 256>>>(bad);
    CK(hipDeviceSynchronize());
    CK(hipMemcpy(&h, bad, 8, hipMemcpyDeviceToHost));
    printf("division: %llu mismatches in 2^32 pairs\n", h);
    CK(hipFree(bad));
    return h ? 1 : 0;
}
