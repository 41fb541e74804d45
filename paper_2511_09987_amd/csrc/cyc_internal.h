// cyc_internal.h -- declarations shared by the translation units of libcyclotron_mm.
// gfx950 only.  Every launcher enqueues on `stream` and returns the hipError_t of the launch.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cyc {

struct Problem {
    const void *A, *B;
    void *C;
    int64_t batch, M, K, N;
    int64_t strideA, strideB, strideC;   // elements
    bool i8;                             // false: bf16 -> fp32, true: int8 -> int32
};

// any shape, any alignment; one thread per 4x4 block of C, k ascending
hipError_t launch_generic(const Problem &p, hipStream_t s);
// fill C with the chain's initial value (K == 0)
hipError_t launch_zero(const Problem &p, hipStream_t s);
// MFMA tiled GEMM; requires supports_mfma(p, tile)
bool supports_mfma(const Problem &p, int tile);
hipError_t launch_mfma(const Problem &p, int tile, int mt, hipStream_t s);   // mt: MFMA tile width, 16 or 32
// HBM-bound streaming kernel for N <= 16; requires supports_narrow(p)
bool supports_narrow(const Problem &p);
bool prefers_narrow(const Problem &p);   // supported and expected to beat the GEMM kernels
hipError_t launch_narrow(const Problem &p, hipStream_t s);

}  // namespace cyc
