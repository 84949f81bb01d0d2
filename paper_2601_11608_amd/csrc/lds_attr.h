// Kernels that ask for more than 64 KB of dynamic LDS have to be allowed to, once per kernel.
#pragma once
#include <hip/hip_runtime.h>

#include <atomic>

// One flag per kernel (the kernel is a template argument: instances that share a function
// type still get their own).  Every thread that finds the flag unset sets the same attribute.
template <auto Kernel>
int fc_allow_full_lds() {
    static std::atomic<bool> allowed{false};
    if (!allowed.load(std::memory_order_acquire)) {
        if (hipFuncSetAttribute((const void *)Kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 163840) != hipSuccess)
            return (int)hipGetLastError();
        allowed.store(true, std::memory_order_release);
    }
    return 0;
}
