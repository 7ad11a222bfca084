// Small host-side helpers around the HIP runtime shared by the library's translation units.
#ifndef PCMM_HIP_UTIL_HPP
#define PCMM_HIP_UTIL_HPP

#include <hip/hip_runtime.h>

namespace pcmm_hip_util {

// Makes `dev` the current device for the lifetime of the object and restores the previous one.
struct DevGuard {
    int prev;
    bool ok;
    explicit DevGuard(int dev) : prev(-1), ok(false)
    {
        if (hipGetDevice(&prev) != hipSuccess) return;
        if (prev != dev && hipSetDevice(dev) != hipSuccess) return;
        ok = true;
    }
    ~DevGuard()
    {
        int cur = -1;
        if (prev >= 0 && hipGetDevice(&cur) == hipSuccess && cur != prev) (void)hipSetDevice(prev);
    }
};

}  // namespace pcmm_hip_util

#endif  // PCMM_HIP_UTIL_HPP
