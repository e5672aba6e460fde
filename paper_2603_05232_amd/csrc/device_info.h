// Host-side facts about the current device, looked up once per device and kept.
#pragma once
#include <hip/hip_runtime.h>
#include <atomic>
#include <stdint.h>
#include "slidesparse.h"

namespace ss {

constexpr int MAX_TRACKED_DEVICES = 64;

inline int current_device()
{
    int d = 0;
    return hipGetDevice(&d) == hipSuccess ? d : -1;
}

// Compute units of the current device (256, the MI355X count, if the runtime cannot tell: the value only
// steers launch shapes, never correctness).
inline int cu_count()
{
    static std::atomic<int> known[MAX_TRACKED_DEVICES];
    const int d = current_device();
    if (d >= 0 && d < MAX_TRACKED_DEVICES) {
        const int c = known[d].load(std::memory_order_relaxed);
        if (c > 0) return c;
    }
    int cus = 0;
    if (d < 0 || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, d) != hipSuccess || cus <= 0) return 256;
    if (d < MAX_TRACKED_DEVICES) known[d].store(cus, std::memory_order_relaxed);
    return cus;
}

// Opt a kernel in to `bytes` of dynamic LDS, once per kernel and device.
template <auto Kernel> inline ss_status allow_dynamic_lds(int bytes)
{
    static std::atomic<uint64_t> done{0};
    const int d = current_device();
    if (d < 0) return SS_ERR_HIP;
    if (d < MAX_TRACKED_DEVICES && ((done.load(std::memory_order_acquire) >> d) & 1u)) return SS_OK;
    if (hipFuncSetAttribute((const void*)Kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess) return SS_ERR_HIP;
    if (d < MAX_TRACKED_DEVICES) done.fetch_or(1ull << d, std::memory_order_release);
    return SS_OK;
}

}  // namespace ss
