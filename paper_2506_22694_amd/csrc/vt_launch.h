// Host-side helper shared by the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>

#include <initializer_list>
#include <mutex>

namespace vt {

// Raises the dynamic-LDS limit of one or more kernels (hipFuncSetAttribute), once per device and safe to call
// from several host threads; a failure is remembered and returned to every later caller on that device.
struct LdsLimitOnce {
    std::once_flag flag[64];
    hipError_t err[64];
};
inline hipError_t allow_dynamic_lds(LdsLimitOnce &state, std::initializer_list<const void *> kernels, int bytes) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    std::call_once(state.flag[dev], [&]() {
        hipError_t r = hipSuccess;
        for (const void *kern : kernels) {
            if (r == hipSuccess) r = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
        }
        state.err[dev] = r;
    });
    return state.err[dev];
}

}  // namespace vt
