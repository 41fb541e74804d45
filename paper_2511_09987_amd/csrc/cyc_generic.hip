// cyc_generic.hip -- shape-agnostic kernel of the weight-stationary recurrence
// (paper, "Space-time Mappings of Dataflow Recurrences"): every C_ij is the chain
// acc <- acc + A_ik * B_kj run in ascending k from 0, exactly as the cell row
// (i,0..K-1) produces it for time step j.  Used for ragged extents, unaligned
// pointers and tiny problems; the fast paths live in cyc_mfma.hip / cyc_narrow.hip.
#include "cyc_internal.h"

namespace cyc {
namespace {

constexpr int GT = 64;   // C tile edge per workgroup
constexpr int GK = 16;   // k slab staged in LDS

__device__ inline float widen(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }
__device__ inline int widen(int8_t v) { return (int)v; }

// 256 threads; thread (ty,tx) owns rows ty*4..+3 and columns tx*4..+3 of the tile.
template <typename In, typename Acc>
__global__ __launch_bounds__(256) void ws_generic_kernel(const In *__restrict__ A, const In *__restrict__ B,
                                                         Acc *__restrict__ C, int64_t M, int64_t K, int64_t N,
                                                         int64_t sA, int64_t sB, int64_t sC, int64_t lda, int64_t ldb,
                                                         int64_t ldc, const Acc *Cin)
{
    __shared__ Acc As[GK][GT + 1];   // [k][i]
    __shared__ Acc Bs[GK][GT + 1];   // [k][j]
    const int t = threadIdx.x, tx = t & 15, ty = t >> 4;
    const int64_t i0 = (int64_t)blockIdx.y * GT, j0 = (int64_t)blockIdx.x * GT;
    A += (int64_t)blockIdx.z * sA;
    B += (int64_t)blockIdx.z * sB;
    C += (int64_t)blockIdx.z * sC;

    Acc acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[a][b] = 0;

    for (int64_t k0 = 0; k0 < K; k0 += GK) {
        // stage A[i0..+63][k0..+15] and B[k0..+15][j0..+63], zero outside the matrices
#pragma unroll
        for (int x = t; x < GT * GK; x += 256) {
            int ai = x / GK, ak = x % GK;
            int64_t gi = i0 + ai, gk = k0 + ak;
            As[ak][ai] = (gi < M && gk < K) ? (Acc)widen(A[gi * lda + gk]) : (Acc)0;
            int bk = x / GT, bj = x % GT;
            int64_t gj = j0 + bj;
            gk = k0 + bk;
            Bs[bk][bj] = (gk < K && gj < N) ? (Acc)widen(B[gk * ldb + gj]) : (Acc)0;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < GK; ++k) {
            Acc a[4], b[4];
#pragma unroll
            for (int x = 0; x < 4; ++x) { a[x] = As[k][ty * 4 + x]; b[x] = Bs[k][tx * 4 + x]; }
#pragma unroll
            for (int x = 0; x < 4; ++x)
#pragma unroll
                for (int y = 0; y < 4; ++y) acc[x][y] += a[x] * b[y];
        }
        __syncthreads();
    }
#pragma unroll
    for (int x = 0; x < 4; ++x)
#pragma unroll
        for (int y = 0; y < 4; ++y) {
            int64_t gi = i0 + ty * 4 + x, gj = j0 + tx * 4 + y;
            if (gi < M && gj < N) C[gi * ldc + gj] = Cin ? Cin[gi * ldc + gj] - acc[x][y] : acc[x][y];   // Cin: C <- Cin - A*B
        }
}

template <typename Acc>
__global__ __launch_bounds__(256) void ws_zero_kernel(Acc *__restrict__ C, int64_t count, int64_t sC)
{
    Acc *c = C + (int64_t)blockIdx.y * sC;
    for (int64_t x = (int64_t)blockIdx.x * 256 + threadIdx.x; x < count; x += (int64_t)gridDim.x * 256) c[x] = 0;
}

}  // namespace

hipError_t launch_generic(const Problem &p, hipStream_t s)
{
    // gridDim.y and .z end at 65535: the caller keeps the batch below that; more than 65535 * 64 rows take several
    // launches (rows are independent)
    if (p.batch > 65535) return hipErrorInvalidValue;
    constexpr int64_t ROWS_PER_LAUNCH = (int64_t)65535 * GT;
    const int64_t lda = row_stride_a(p), ldc = row_stride_c(p), es = p.i8 ? 1 : 2;
    for (int64_t r0 = 0; r0 < p.M; r0 += ROWS_PER_LAUNCH) {
        const int64_t rows = p.M - r0 < ROWS_PER_LAUNCH ? p.M - r0 : ROWS_PER_LAUNCH;
        const char *A = (const char *)p.A + r0 * lda * es;
        char *C = (char *)p.C + r0 * ldc * 4;
        const char *Cin = p.Cin ? (const char *)p.Cin + r0 * ldc * 4 : nullptr;
        dim3 grid((unsigned)((p.N + GT - 1) / GT), (unsigned)((rows + GT - 1) / GT), (unsigned)p.batch);
        hipError_t e;
        if (p.i8)
            e = launch_kernel(ws_generic_kernel<int8_t, int>, grid, dim3(256), s, (const int8_t *)A, (const int8_t *)p.B, (int *)C,
                              rows, p.K, p.N, p.strideA, p.strideB, p.strideC, lda, row_stride_b(p), ldc, (const int *)Cin);
        else
            e = launch_kernel(ws_generic_kernel<uint16_t, float>, grid, dim3(256), s, (const uint16_t *)A, (const uint16_t *)p.B,
                              (float *)C, rows, p.K, p.N, p.strideA, p.strideB, p.strideC, lda, row_stride_b(p), ldc,
                              (const float *)Cin);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_zero(const Problem &p, hipStream_t s)
{
    if (p.batch > 65535) return hipErrorInvalidValue;
    int64_t count = p.M * p.N;
    int64_t blocks = (count + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    dim3 grid((unsigned)blocks, (unsigned)p.batch);
    hipError_t launch_err = hipSuccess;
    if (p.i8)
        launch_err = launch_kernel(ws_zero_kernel<int>, grid, dim3(256), s, (int *)p.C, count, p.strideC);
    else
        launch_err = launch_kernel(ws_zero_kernel<float>, grid, dim3(256), s, (float *)p.C, count, p.strideC);
    return launch_err;
}

}  // namespace cyc
