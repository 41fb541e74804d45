// cyc_api.hip -- the C ABI declared in include/cyclotron_mm.h: argument checks and
// the choice of kernel.  No device work happens here except the launches.
#include "../../include/cyclotron_mm.h"
#include "cyc_internal.h"

#include <cstdlib>
#include <cstring>
#include <atomic>

namespace {

constexpr int64_t kMaxElems = (int64_t)1 << 46;   // keeps every byte offset far inside int64

bool mul_ok(int64_t a, int64_t b, int64_t *out)
{
    if (a == 0 || b == 0) { *out = 0; return true; }
    if (a > kMaxElems / b) return false;
    *out = a * b;
    return true;
}

bool overlaps(const void *p, int64_t pbytes, const void *q, int64_t qbytes)
{
    if (!p || !q || pbytes <= 0 || qbytes <= 0) return false;
    uintptr_t a = (uintptr_t)p, b = (uintptr_t)q;
    return a < b + (uintptr_t)qbytes && b < a + (uintptr_t)pbytes;
}

enum Kernel { K_NONE, K_ZERO, K_GENERIC, K_MFMA256, K_MFMA128, K_MFMA256X32, K_MFMA128X32, K_MFMAK, K_NARROW, K_NARROWM };

const char *kernel_label(Kernel k)
{
    switch (k) {
        case K_NONE: return "none";
        case K_ZERO: return "zero";
        case K_GENERIC: return "generic";
        case K_MFMA256: return "mfma256";
        case K_MFMA128: return "mfma128";
        case K_MFMA256X32: return "mfma256x32";
        case K_MFMA128X32: return "mfma128x32";
        case K_MFMAK: return "mfmak";
        case K_NARROW: return "narrow";
        case K_NARROWM: return "narrowm";
    }
    return "none";
}

// The kernel forced by cyc_force_kernel(), or by the environment variable CYC_FORCE_KERNEL, which is read once
// (at the first call that gets as far as choosing a kernel) as the initial value.  K_NONE: the dispatcher decides.
Kernel kernel_by_name(const char *name)
{
    if (!name) return K_NONE;
    for (Kernel k : {K_GENERIC, K_MFMA256, K_MFMA128, K_MFMA256X32, K_MFMA128X32, K_MFMAK, K_NARROW, K_NARROWM})
        if (!std::strcmp(name, kernel_label(k))) return k;
    return K_NONE;
}
std::atomic<int> &forced_kernel()
{
    static std::atomic<int> forced{(int)kernel_by_name(std::getenv("CYC_FORCE_KERNEL"))};
    return forced;
}

std::atomic<int> &wait_limit_value()
{
    static std::atomic<int> v{1 << 20};
    return v;
}

// Validates and fills `p`.  Returns CYC_OK with *k == K_NONE when there is nothing to do.
int plan(const void *A, const void *B, const void *C, int64_t batch, int64_t M, int64_t K, int64_t N,
         int64_t strideA, int64_t strideB, int64_t strideC, int dtype, cyc::Problem *p, Kernel *k)
{
    *k = K_NONE;
    if (dtype != CYC_BF16_F32 && dtype != CYC_I8_I32) return CYC_ERR_DTYPE;
    if (batch < 0 || M < 0 || K < 0 || N < 0 || strideA < 0 || strideB < 0 || strideC < 0) return CYC_ERR_SHAPE;
    int64_t mk, kn, mn;
    if (!mul_ok(M, K, &mk) || !mul_ok(K, N, &kn) || !mul_ok(M, N, &mn)) return CYC_ERR_SHAPE;
    if (batch > 1) {
        int64_t t;
        if (strideC < mn) return CYC_ERR_SHAPE;
        if (!mul_ok(batch, strideA > mk ? strideA : mk, &t) || !mul_ok(batch, strideB > kn ? strideB : kn, &t) ||
            !mul_ok(batch, strideC, &t))
            return CYC_ERR_SHAPE;
        if ((strideA != 0 && strideA < mk) || (strideB != 0 && strideB < kn)) return CYC_ERR_SHAPE;
    }
    if (batch == 0 || M == 0 || N == 0) return CYC_OK;
    if (!C) return CYC_ERR_NULL;
    if (K > 0 && (!A || !B)) return CYC_ERR_NULL;

    const bool i8 = dtype == CYC_I8_I32;
    const int64_t es = i8 ? 1 : 2;
    const int64_t spanA = ((batch - 1) * strideA + mk) * es, spanB = ((batch - 1) * strideB + kn) * es;
    const int64_t spanC = ((batch - 1) * strideC + mn) * 4;
    if (K > 0 && (overlaps(C, spanC, A, spanA) || overlaps(C, spanC, B, spanB))) return CYC_ERR_ALIAS;

    p->A = A; p->B = B; p->C = const_cast<void *>(C);
    p->batch = batch; p->M = M; p->K = K; p->N = N;
    p->strideA = strideA; p->strideB = strideB; p->strideC = strideC;
    p->i8 = i8;

    if (K == 0) { *k = K_ZERO; return CYC_OK; }

    // a forced kernel overrides the heuristic when it supports the problem (testing and benchmarking aid).  The x32
    // names are the MFMA kernels built on the 32x32 instruction shape, which the dispatcher never picks by itself.
    const Kernel force = (Kernel)forced_kernel().load(std::memory_order_relaxed);
    int ktile = 0;
    switch (force) {
        case K_GENERIC: *k = K_GENERIC; return CYC_OK;
        case K_MFMA256: case K_MFMA256X32: if (cyc::supports_mfma(*p, 256)) { *k = force; return CYC_OK; } break;
        case K_MFMA128: case K_MFMA128X32: if (cyc::supports_mfma(*p, 128)) { *k = force; return CYC_OK; } break;
        case K_NARROW: if (cyc::supports_narrow(*p)) { *k = force; return CYC_OK; } break;
        case K_NARROWM: if (cyc::supports_narrowm(*p)) { *k = force; return CYC_OK; } break;
        case K_MFMAK: if (cyc::choose_ksplit(*p, &ktile) > 1) { *k = force; return CYC_OK; } break;
        default: break;
    }
    if (cyc::prefers_narrow(*p)) { *k = K_NARROW; return CYC_OK; }
    if (cyc::prefers_narrowm(*p)) { *k = K_NARROWM; return CYC_OK; }
    // few output blocks, long k: k goes to space (see choose_ksplit)
    if (force == K_NONE && cyc::choose_ksplit(*p, &ktile) > 1) { *k = K_MFMAK; return CYC_OK; }
    // MFMA kernels for everything with 16-byte aligned rows except slivers
    const int tile = cyc::choose_mfma_tile(*p);
    if (tile == 256) { *k = K_MFMA256; return CYC_OK; }
    if (tile == 128) { *k = K_MFMA128; return CYC_OK; }
    *k = K_GENERIC;
    return CYC_OK;
}

int run_chunk(const cyc::Problem &p, Kernel k, void *workspace, hipStream_t s)
{
    hipError_t e = hipSuccess;
    switch (k) {
        case K_NONE: return CYC_OK;
        case K_ZERO: e = cyc::launch_zero(p, s); break;
        case K_GENERIC: e = cyc::launch_generic(p, s); break;
        case K_MFMA256: e = cyc::launch_mfma(p, 256, 16, s); break;
        case K_MFMA128: e = cyc::launch_mfma(p, 128, 16, s); break;
        case K_MFMA256X32: e = cyc::launch_mfma(p, 256, 32, s); break;
        case K_MFMA128X32: e = cyc::launch_mfma(p, 128, 32, s); break;
        case K_MFMAK: {
            int tile = 0;
            const int ks = cyc::choose_ksplit(p, &tile);
            e = cyc::launch_mfma_ksplit(p, ks, tile, workspace, s);
            break;
        }
        case K_NARROW: e = cyc::launch_narrow(p, s); break;
        case K_NARROWM: e = cyc::launch_narrowm(p, s); break;
    }
    return e == hipSuccess ? CYC_OK : CYC_ERR_LAUNCH;
}

// A grid's y extent ends at 65535, which is where a launch's share of the batch ends: longer batches take several
// launches of the same kernel (batch elements are independent).
constexpr int64_t kBatchPerLaunch = 65535;

// fixed_workspace: take the partial products' memory from the library's fixed array instead of the per-stream cache
int run(const cyc::Problem &p, Kernel k, hipStream_t s, bool fixed_workspace = false)
{
    void *workspace = nullptr;
    if (k == K_MFMAK) {
        // everything that can fail before the first launch is settled before it
        int tile = 0;
        const int ks = cyc::choose_ksplit(p, &tile);
        const int64_t need = cyc::ksplit_workspace_bytes(p, ks);
        if (fixed_workspace) {
            int64_t have = 0;
            workspace = cyc::static_workspace(&have);
            if (need > have) return CYC_ERR_WORKSPACE;
        } else {
            workspace = cyc::cached_workspace(s, need);
        }
        if (!workspace) return CYC_ERR_WORKSPACE;
    }
    if (p.batch <= kBatchPerLaunch) return run_chunk(p, k, workspace, s);
    const int64_t es = p.i8 ? 1 : 2;
    for (int64_t b0 = 0; b0 < p.batch; b0 += kBatchPerLaunch) {
        cyc::Problem q = p;
        q.batch = p.batch - b0 < kBatchPerLaunch ? p.batch - b0 : kBatchPerLaunch;
        q.A = (const char *)p.A + b0 * p.strideA * es;
        q.B = (const char *)p.B + b0 * p.strideB * es;
        q.C = (char *)p.C + b0 * p.strideC * 4;
        if (int st = run_chunk(q, k, workspace, s); st != CYC_OK) return st;
    }
    return CYC_OK;
}

}  // namespace

namespace cyc {
int wait_limit() { return wait_limit_value().load(); }
}  // namespace cyc

extern "C" {

int cyc_recurrence_matmul_batched(const void *A, const void *B, void *C, int64_t batch, int64_t M, int64_t K,
                                  int64_t N, int64_t strideA, int64_t strideB, int64_t strideC, int dtype,
                                  void *stream)
{
    cyc::Problem p;
    Kernel k;
    int st = plan(A, B, C, batch, M, K, N, strideA, strideB, strideC, dtype, &p, &k);
    if (st != CYC_OK || k == K_NONE) return st;      // an error, or nothing to do (p is then not filled in)
    return run(p, k, (hipStream_t)stream);
}

int cyc_recurrence_matmul(const void *A, const void *B, void *C, int64_t M, int64_t K, int64_t N, int dtype,
                          void *stream)
{
    return cyc_recurrence_matmul_batched(A, B, C, 1, M, K, N, 0, 0, 0, dtype, stream);
}

int cyc_recurrence_matmul_noalloc(const void *A, const void *B, void *C, int64_t M, int64_t K, int64_t N, int dtype,
                                  void *stream)
{
    cyc::Problem p;
    Kernel k;
    int st = plan(A, B, C, 1, M, K, N, 0, 0, 0, dtype, &p, &k);
    if (st != CYC_OK || k == K_NONE) return st;
    return run(p, k, (hipStream_t)stream, true);
}

int cyc_recurrence_trsm(const void *L, const void *B, void *X, void *Xh, int64_t n, int64_t nrhs, int64_t nb,
                        void *stream)
{
    if (n < 0 || nrhs < 0 || nb < 1 || nb > 128) return CYC_ERR_SHAPE;
    int64_t nn, nr;
    if (!mul_ok(n, n, &nn) || !mul_ok(n, nrhs, &nr)) return CYC_ERR_SHAPE;
    if (n == 0 || nrhs == 0) return CYC_OK;
    if (!L || !B || !X || !Xh) return CYC_ERR_NULL;
    if (overlaps(X, nr * 4, L, nn * 2) || overlaps(X, nr * 4, B, nr * 4) || overlaps(Xh, nr * 2, L, nn * 2) ||
        overlaps(Xh, nr * 2, B, nr * 4) || overlaps(X, nr * 4, Xh, nr * 2))
        return CYC_ERR_ALIAS;
    // the inverses of the diagonal tiles live in the per-stream workspace; it is acquired before the first launch
    void *workspace = nullptr;
    const int64_t need = cyc::trsm_workspace_bytes(L, X, Xh, n, nrhs, nb);
    if (need > 0) {
        workspace = cyc::cached_workspace((hipStream_t)stream, need);
        if (!workspace) return CYC_ERR_WORKSPACE;
    }
    return cyc::launch_trsm(L, B, X, Xh, n, nrhs, nb, workspace, (hipStream_t)stream) == hipSuccess ? CYC_OK : CYC_ERR_LAUNCH;
}

int cyc_recurrence_cholesky(const void *A, void *L, void *Lh, int64_t n, int64_t nb, void *stream)
{
    if (n < 0 || nb < 1 || nb > 64 || n > (1 << 22)) return CYC_ERR_SHAPE;
    int64_t nn;
    if (!mul_ok(n, n, &nn)) return CYC_ERR_SHAPE;
    if (n == 0) return CYC_OK;
    if (!A || !L || !Lh) return CYC_ERR_NULL;
    if (((uintptr_t)A | (uintptr_t)L) & 3 || ((uintptr_t)Lh & 1)) return CYC_ERR_SHAPE;
    if (overlaps(L, nn * 4, A, nn * 4) || overlaps(Lh, nn * 2, A, nn * 4) || overlaps(L, nn * 4, Lh, nn * 2)) return CYC_ERR_ALIAS;
    void *workspace = nullptr;
    const int64_t need = cyc::chol_workspace_bytes(n, nb);
    if (need > 0) {
        workspace = cyc::cached_workspace((hipStream_t)stream, need);
        if (!workspace) return CYC_ERR_WORKSPACE;
    }
    return cyc::launch_chol(A, L, Lh, n, nb, workspace, (hipStream_t)stream) == hipSuccess ? CYC_OK : CYC_ERR_LAUNCH;
}

int cyc_recurrence_attention(const void *Q, const void *K, const void *V, void *O, int64_t batch, int64_t N, int64_t M,
                             int64_t d, void *stream)
{
    if (batch < 0 || N < 0 || M < 0 || d < 0) return CYC_ERR_SHAPE;
    if (batch == 0 || N == 0) return CYC_OK;
    int64_t nq, nk;
    if (!mul_ok(N, d, &nq) || !mul_ok(M, d, &nk) || !mul_ok(batch, nq, &nq) || !mul_ok(batch, nk, &nk)) return CYC_ERR_SHAPE;
    if (M == 0 || batch > 65535 || !cyc::supports_attention(N, M, d)) return CYC_ERR_SHAPE;
    if (!Q || !K || !V || !O) return CYC_ERR_NULL;
    if (((uintptr_t)Q | (uintptr_t)K | (uintptr_t)V | (uintptr_t)O) & 15) return CYC_ERR_SHAPE;
    if (overlaps(O, nq * 4, Q, nq * 2) || overlaps(O, nq * 4, K, nk * 2) || overlaps(O, nq * 4, V, nk * 2)) return CYC_ERR_ALIAS;
    return cyc::launch_attention(Q, K, V, O, batch, N, M, d, (hipStream_t)stream) == hipSuccess ? CYC_OK : CYC_ERR_LAUNCH;
}

const char *cyc_kernel_name(const void *A, const void *B, const void *C, int64_t batch, int64_t M, int64_t K,
                            int64_t N, int64_t strideA, int64_t strideB, int64_t strideC, int dtype)
{
    cyc::Problem p;
    Kernel k;
    if (plan(A, B, C, batch, M, K, N, strideA, strideB, strideC, dtype, &p, &k) != CYC_OK) return "none";
    return kernel_label(k);
}

const char *cyc_status_string(int status)
{
    switch (status) {
        case CYC_OK: return "CYC_OK";
        case CYC_ERR_NULL: return "CYC_ERR_NULL: required pointer is NULL";
        case CYC_ERR_SHAPE: return "CYC_ERR_SHAPE: negative or overflowing extent or stride";
        case CYC_ERR_DTYPE: return "CYC_ERR_DTYPE: unknown element type";
        case CYC_ERR_ALIAS: return "CYC_ERR_ALIAS: C overlaps an input";
        case CYC_ERR_LAUNCH: return "CYC_ERR_LAUNCH: HIP launch failed";
        case CYC_ERR_WORKSPACE: return "CYC_ERR_WORKSPACE: workspace could not be allocated, or the problem needs more than the fixed workspace holds";
    }
    return "unknown cyc_status";
}

int cyc_version(void) { return 200; }

int cyc_diag_set_wait_limit(int64_t polls)
{
    if (polls < 0 || polls > (1 << 30)) return CYC_ERR_SHAPE;
    wait_limit_value().store(polls == 0 ? 1 << 20 : (int)polls);
    return CYC_OK;
}

int cyc_force_kernel(const char *name)
{
    if (!name || !*name) {
        forced_kernel().store((int)K_NONE);
        return CYC_OK;
    }
    const Kernel k = kernel_by_name(name);
    if (k == K_NONE) return CYC_ERR_SHAPE;
    forced_kernel().store((int)k);
    return CYC_OK;
}

}  // extern "C"
