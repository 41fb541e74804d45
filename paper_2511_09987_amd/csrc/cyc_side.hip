// cyc_side.hip -- the per-device side stream (see cyc_internal.h).
#include "cyc_internal.h"

#include <mutex>

namespace cyc {
namespace {

constexpr int MAX_DEVICES = 64;
SideStream g_side[MAX_DEVICES];
std::mutex g_side_mutex;

}  // namespace

SideStream *SideStreamLock::acquire()
{
    g_side_mutex.lock();
    held_ = true;
    int dev = 0;
    SideStream *v = nullptr;
    if (hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev < MAX_DEVICES) {
        v = &g_side[dev];
        if (!v->tried) {
            v->tried = true;
            v->ok = hipStreamCreateWithFlags(&v->stream, hipStreamNonBlocking) == hipSuccess &&
                    hipEventCreateWithFlags(&v->fork, hipEventDisableTiming | hipEventDisableSystemFence) == hipSuccess;
            for (hipEvent_t &e : v->join) v->ok = v->ok && hipEventCreateWithFlags(&e, hipEventDisableTiming | hipEventDisableSystemFence) == hipSuccess;
            if (!v->ok) (void)hipGetLastError();
        }
        if (!v->ok) v = nullptr;
    }
    if (!v) {
        held_ = false;
        g_side_mutex.unlock();
    }
    return v;
}

SideStreamLock::~SideStreamLock()
{
    if (held_) g_side_mutex.unlock();
}

}  // namespace cyc
