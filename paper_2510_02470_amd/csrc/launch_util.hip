// Launch helpers shared by the kernel launchers.
#include <mutex>
#include <utility>
#include <vector>

#include "sage_internal.h"

namespace sage {

namespace {
std::mutex g_attr_lock;
std::vector<std::pair<int, const void*>> g_attr_done;  // (device, kernel) pairs whose limit has been raised
}  // namespace

// A kernel that asks for more than 64 KB of dynamic LDS needs its limit raised once per device. Thread-safe; the
// runtime's error is returned (and the pair is not recorded, so the next launch tries again).
hipError_t ensure_dynamic_lds(const void* kernel, int bytes) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> hold(g_attr_lock);
    for (const auto& p : g_attr_done)
        if (p.first == dev && p.second == kernel) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e != hipSuccess) return e;
    g_attr_done.emplace_back(dev, kernel);
    return hipSuccess;
}

}  // namespace sage
