// Scratch areas in which the workgroups that share a row meet (see SplitRow).  One per (device, stream), so that
// calls on different streams never share one; allocated at the first call that needs it and kept until the
// process ends.  A stream that is being captured cannot allocate: it gets an area only if it already has one.
#include <map>
#include <mutex>
#include <utility>

#include "ppv_internal.h"

namespace {
std::mutex g_mu;
std::map<std::pair<int, hipStream_t>, SplitScratch *> g_scratch;
}  // namespace

SplitScratch *ppv_split_scratch(hipStream_t stream) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(g_mu);
    const auto key = std::make_pair(dev, stream);
    const auto it = g_scratch.find(key);
    if (it != g_scratch.end()) return it->second;
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &cs) != hipSuccess || cs != hipStreamCaptureStatusNone) {
        (void)hipGetLastError();
        return nullptr;
    }
    SplitScratch *p = nullptr;
    if (hipMalloc((void **)&p, sizeof(SplitScratch)) != hipSuccess) {
        (void)hipGetLastError();
        return nullptr;
    }
    // the arrival counters start at zero (afterwards every launch leaves them at zero); in stream order before the
    // kernel that is about to be launched
    if (hipMemsetAsync(p->arrivals, 0, sizeof(p->arrivals), stream) != hipSuccess) {
        (void)hipGetLastError();
        (void)hipFree(p);
        return nullptr;
    }
    g_scratch[key] = p;
    return p;
}
