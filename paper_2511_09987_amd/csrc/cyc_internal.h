// cyc_internal.h -- declarations shared by the translation units of libcyclotron_mm.
// gfx950 only.  Every launcher enqueues on `stream` and returns the hipError_t of the launch.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <tuple>
#include <type_traits>
#include <utility>

namespace cyc {

// Enqueue `kernel` and return the status of this launch itself: unlike the triple-chevron form followed by
// hipGetLastError(), this neither consumes nor reports an error that an earlier call of the application left behind.
template <typename... KArgs, typename... Args>
inline hipError_t launch_kernel(void (*kernel)(KArgs...), dim3 grid, dim3 block, hipStream_t s, Args &&...args)
{
    static_assert(sizeof...(KArgs) == sizeof...(Args), "argument count does not match the kernel's signature");
    std::tuple<std::remove_cv_t<KArgs>...> vals(static_cast<std::remove_cv_t<KArgs>>(args)...);
    void *ptrs[sizeof...(KArgs)];
    std::apply([&](auto &...v) { int i = 0; ((ptrs[i++] = (void *)&v), ...); }, vals);
    return hipLaunchKernel((const void *)kernel, grid, block, ptrs, 0, s);
}

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
    bool kslices = false;                // the batch elements are k-slices of one problem (windows allowed with batch > 1)
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
// long k extent.  One workgroup per (output block, k-slice) writes its partial product to slice `b` of a workspace
// of ksplit x M x N accumulator elements; a second kernel adds the slices in ascending order into C.
int choose_ksplit(const Problem &p, int *tile);   // *tile: block edge to use, 128 or 256
inline int64_t ksplit_workspace_bytes(const Problem &p, int ksplit) { return (int64_t)ksplit * p.M * p.N * 4; }
hipError_t launch_mfma_ksplit(const Problem &p, int ksplit, int tile, void *workspace, hipStream_t s);
// Device memory for the partial products.  cached_workspace: one buffer per (device, stream), allocated with hipMalloc
// on first use, grown when a call needs more, kept until the process ends; nullptr when the allocation fails.
// static_workspace: the library's fixed array in device memory (one per device, *bytes = its size), shared by every
// caller on that device; allocates nothing; nullptr when its address cannot be obtained.
void *cached_workspace(hipStream_t s, int64_t bytes);
void *static_workspace(int64_t *bytes);
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

// Bound, in polls, of the waits by which waves hand work to one another inside the tile kernels of the triangular solve
// and of the Cholesky factorisation (cyc_diag_set_wait_limit; 2^20 unless a test has set it).
int wait_limit();

// workspace: trsm_workspace_bytes() bytes of device memory (inverses of the diagonal tiles), or nullptr: every tile by substitution
int64_t trsm_workspace_bytes(const void *L, void *X, void *Xh, int64_t n, int64_t nrhs, int64_t nb);
hipError_t launch_trsm(const void *L, const void *B, void *X, void *Xh, int64_t n, int64_t nrhs, int64_t nb, void *workspace,
                       hipStream_t s);
// tiled Cholesky factorisation A = L L^T in tiles of nb (see cyc_chol.hip); arguments validated by the caller
// workspace: chol_workspace_bytes() bytes of device memory (inverses of the diagonal tiles), or nullptr: no inverses
int64_t chol_workspace_bytes(int64_t n, int64_t nb);
hipError_t launch_chol(const void *A, void *L, void *Lh, int64_t n, int64_t nb, void *workspace, hipStream_t s);
// FlashAttention-2 tile recurrence (see cyc_attn.hip); requires supports_attention(N, M, d)
bool supports_attention(int64_t N, int64_t M, int64_t d);
hipError_t launch_attention(const void *Q, const void *K, const void *V, void *O, int64_t batch, int64_t N, int64_t M,
                            int64_t d, hipStream_t s);
// HBM-bound streaming kernel for N <= 16; requires supports_narrow(p)
bool supports_narrow(const Problem &p);
bool prefers_narrow(const Problem &p);   // supported and expected to beat the GEMM kernels
hipError_t launch_narrow(const Problem &p, hipStream_t s);
// HBM-bound streaming kernel for M <= 32 (B streamed once, the rows of A pass over it); requires supports_narrowm(p)
bool supports_narrowm(const Problem &p);
bool prefers_narrowm(const Problem &p);
hipError_t launch_narrowm(const Problem &p, hipStream_t s);

}  // namespace cyc
