// cyc_workspace.hip -- device memory for the partial products of the k-in-space matmul and for the inverses of the triangular solve (see cyc_internal.h).
//
// Two sources.  cached_workspace(): one hipMalloc'd buffer per (device, stream), so that calls on different
// streams never share one; grown when a call needs more, never shrunk, kept until the process ends.
// static_workspace(): a fixed array in the library's own device image, for callers that must not allocate.
#include "cyc_internal.h"

#include <map>
#include <mutex>
#include <utility>

namespace cyc {
namespace {

constexpr int MAX_DEVICES = 64;

// The fixed workspace of the allocation-free entry point: every device the library runs on holds its own copy
// until the process ends.  In host code the name below is only a handle for hipGetSymbolAddress; kernels are
// given the address obtained from it.
constexpr int64_t SCRATCH_BYTES = (int64_t)32 << 20;
static __device__ __align__(256) unsigned char scratch[SCRATCH_BYTES];

struct PerDevice {
    bool tried = false;
    void *scratch_ptr = nullptr;                        // this device's address of `scratch`
    std::map<hipStream_t, std::pair<void *, int64_t>> cache;   // stream -> (buffer, bytes)
};
PerDevice g_dev[MAX_DEVICES];
std::mutex g_mutex;

PerDevice *current_device()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return nullptr;
    return &g_dev[dev];
}

}  // namespace

void *static_workspace(int64_t *bytes)
{
    *bytes = SCRATCH_BYTES;
    std::lock_guard<std::mutex> hold(g_mutex);
    PerDevice *d = current_device();
    if (!d) return nullptr;
    if (!d->tried) {
        // once per device, with that device current: each device has the array at an address of its own
        d->tried = true;
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) == hipSuccess) d->scratch_ptr = p;
    }
    return d->scratch_ptr;
}

void *cached_workspace(hipStream_t s, int64_t bytes)
{
    std::lock_guard<std::mutex> hold(g_mutex);
    PerDevice *d = current_device();
    if (!d || bytes <= 0) return nullptr;
    auto &slot = d->cache[s];
    if (slot.second >= bytes) return slot.first;
    // hipFree waits for the device, so nothing enqueued earlier still uses the old buffer when it goes
    if (slot.first) (void)hipFree(slot.first);
    slot = {nullptr, 0};
    void *p = nullptr;
    const int64_t want = (bytes + ((int64_t)1 << 20) - 1) >> 20 << 20;
    if (hipMalloc(&p, (size_t)want) != hipSuccess) return nullptr;
    slot = {p, want};
    return p;
}

}  // namespace cyc
