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
    // Extensions used by the triangular solve and the Cholesky factorisation (batch == 1 only; the narrow kernel
    // ignores them): operands and result may be windows of wider matrices
    int64_t lda = 0;                     // row stride of A in elements, 0 = K
    int64_t ldb = 0;                     // row stride of B in elements, 0 = N
    int64_t ldc = 0;                     // row stride of C (and of Cin) in elements, 0 = N
    const void *Cin = nullptr;           // when set, C <- Cin - A*B instead of C <- A*B (same layout as C; may be C)
    bool accumulate = false;             // the epilogue adds its product to C atomically (the k-in-space variant)
};
inline int64_t row_stride_a(const Problem &p) { return p.lda ? p.lda : p.K; }
inline int64_t row_stride_b(const Problem &p) { return p.ldb ? p.ldb : p.N; }
inline int64_t row_stride_c(const Problem &p) { return p.ldc ? p.ldc : p.N; }

// any shape, any alignment; one thread per 4x4 block of C, k ascending
hipError_t launch_generic(const Problem &p, hipStream_t s);
// fill C with the chain's initial value (K == 0)
hipError_t launch_zero(const Problem &p, hipStream_t s);
// MFMA tiled GEMM; requires supports_mfma(p, tile)
bool supports_mfma(const Problem &p, int tile);
hipError_t launch_mfma(const Problem &p, int tile, int mt, hipStream_t s);   // mt: MFMA tile width, 16 or 32
// block edge (256 or 128) of the MFMA kernel that suits the problem best, 0 if neither supports it
int choose_mfma_tile(const Problem &p);
// k in space: number of k-slices (a power of two, 1 = do not split) for problems with few output blocks and a
// long k extent, and the launch that zeroes C and lets one workgroup per (output block, k-slice) add its partial
// product to C atomically
int choose_ksplit(const Problem &p, int *tile);   // *tile: block edge to use, 128 or 256
hipError_t launch_mfma_ksplit(const Problem &p, int ksplit, int tile, hipStream_t s);
// lower-triangular forward solve L X = B in tiles of nb rows (see cyc_tri.hip); arguments validated by the caller
// A second stream per device for work that may run beside what a call enqueues on the caller's stream (forked from
// and joined into that stream with events inside the call).  Created on first use, default priority, kept until the
// process ends.  One lock serialises the callers that use it: SideStreamLock::acquire() takes the lock for the
// lifetime of the object and returns the current device's side stream, or nullptr (creation failed; lock released),
// in which case the caller does without.
struct SideStream {
    hipStream_t stream = nullptr;
    hipEvent_t fork = nullptr;            // recorded on the caller's stream, waited for by the side stream
    hipEvent_t join[8] = {};              // recorded on the side stream, waited for by the caller's stream
    bool tried = false, ok = false;
};
class SideStreamLock {
public:
    SideStream *acquire();
    ~SideStreamLock();

private:
    bool held_ = false;
};

hipError_t launch_trsm(const void *L, const void *B, void *X, void *Xh, int64_t n, int64_t nrhs, int64_t nb, hipStream_t s);
// tiled Cholesky factorisation A = L L^T in tiles of nb (see cyc_chol.hip); arguments validated by the caller
hipError_t launch_chol(const void *A, void *L, void *Lh, int64_t n, int64_t nb, hipStream_t s);
// FlashAttention-2 tile recurrence (see cyc_attn.hip); requires supports_attention(N, M, d)
bool supports_attention(int64_t N, int64_t M, int64_t d);
hipError_t launch_attention(const void *Q, const void *K, const void *V, void *O, int64_t batch, int64_t N, int64_t M,
                            int64_t d, hipStream_t s);
// HBM-bound streaming kernel for N <= 16; requires supports_narrow(p)
bool supports_narrow(const Problem &p);
bool prefers_narrow(const Problem &p);   // supported and expected to beat the GEMM kernels
hipError_t launch_narrow(const Problem &p, hipStream_t s);

}  // namespace cyc
