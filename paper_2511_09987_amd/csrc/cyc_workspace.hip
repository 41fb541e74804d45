// cyc_workspace.hip -- device memory for the partial products of the k-in-space matmul (see cyc_internal.h).
//
// cached_workspace(): one hipMalloc'd buffer per (device, stream), so that calls on different streams never share
// one; grown when a call needs more, never shrunk, kept until the process ends.
#include "cyc_internal.h"

#include <map>
#include <mutex>
#include <utility>

namespace cyc {
namespace {

constexpr int MAX_DEVICES = 64;

struct PerDevice {
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
