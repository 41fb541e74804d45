// cyc_wave.h -- small device helpers shared by the kernels that run a scalar recurrence in one wave
// (the tile kernels of the triangular solve and of the Cholesky factorisation).
#pragma once

#include <hip/hip_runtime.h>

#include <type_traits>
#include <utility>

namespace cyc {

// f(integral_constant<int, 0>), ..., f(integral_constant<int, N - 1>): a loop whose index is a constant in every copy
// from the start (the unrolling pass gives up on bodies as long as those of the tile kernels)
template <class F, int... I>
__device__ __forceinline__ void unrolled(F &&f, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void unrolled(F &&f)
{
    unrolled(f, std::make_integer_sequence<int, N>{});
}

// IEEE fp32 division num / den (correctly rounded, all special cases) in four phases: the instruction sequence the
// compiler itself expands a division into, cut up so that independent work can be placed between the phases of this
// long dependent chain: scale and reciprocal estimate; a Newton step on the reciprocal; quotient and one correction;
// the last correction and the hardware's fix-up of scaling and special cases.
struct Division {
    float num, den, d0, n0, r, q;
    bool flag;
    __device__ __forceinline__ void phase0(float numerator, float denominator)
    {
        num = numerator;
        den = denominator;
        bool unused;
        d0 = __builtin_amdgcn_div_scalef(num, den, false, &unused);
        n0 = __builtin_amdgcn_div_scalef(num, den, true, &flag);
        r = __builtin_amdgcn_rcpf(d0);
    }
    __device__ __forceinline__ void phase1()
    {
        const float e = __builtin_fmaf(-d0, r, 1.0f);
        r = __builtin_fmaf(e, r, r);
    }
    __device__ __forceinline__ void phase2()
    {
        q = n0 * r;
        const float e = __builtin_fmaf(-d0, q, n0);
        q = __builtin_fmaf(e, r, q);
    }
    __device__ __forceinline__ float phase3()
    {
        const float e = __builtin_fmaf(-d0, q, n0);
        return __builtin_amdgcn_div_fixupf(__builtin_amdgcn_div_fmasf(e, r, q, flag), den, num);
    }
};

// The column recurrence of a 64-wide tile as a fixed list of steps, for the kernels that run it in one wave with
// the lane's row in registers.  The 64 columns go in 16 blocks of four.  The four chains of block b first take the
// columns left of the block (b "bulk" steps of four k each: 16 independent multiply-adds), then the 4 x 4 corner
// finishes the four columns one after the other, each with a division: a chain of dependent instructions.  In a lone
// wave a dependent instruction issues every ~8 cycles, an independent one every ~5, so the corner of block b is
// interleaved with bulk steps of block b + 1: its steps over k4 < b do not need the columns the corner is producing,
// and up to EARLY of them are taken out of turn, one beside each corner column.  Every entry still takes its terms
// in ascending k.  StepList is the resulting execution order of all 120 bulk steps.
constexpr int NBLK = 64 / 4, EARLY = 4, NSTEP = NBLK * (NBLK - 1) / 2;
constexpr int early_of(int b) { return b < 1 ? 0 : (b - 1 < EARLY ? b - 1 : EARLY); }
struct StepList {
    signed char b[NSTEP + 2], k[NSTEP + 2];
};
constexpr StepList make_steps()
{
    StepList s{};
    int n = 0;
    for (int b = 0; b < NBLK; ++b) {
        for (int k4 = early_of(b); k4 < b; ++k4) {           // in turn, before the corner of block b
            s.b[n] = (signed char)b;
            s.k[n++] = (signed char)k4;
        }
        if (b + 1 < NBLK)
            for (int k4 = 0; k4 < early_of(b + 1); ++k4) {   // out of turn, beside the corner of block b
                s.b[n] = (signed char)(b + 1);
                s.k[n++] = (signed char)k4;
            }
    }
    s.b[n] = s.b[n + 1] = -1;                                // (requests past the end do nothing)
    return s;
}
constexpr StepList STEPS = make_steps();

}  // namespace cyc
