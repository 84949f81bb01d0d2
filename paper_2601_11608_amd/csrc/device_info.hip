// Shape of the GPU the calling thread is on (compute units, XCDs, rate of the constant wall clock),
// asked of the runtime once per device.  The launchers size their persistent grids, deal tiles to the
// XCDs and pace their store streams from this instead of from literals; the attribute queries touch no
// stream, so a first call under stream capture is harmless.
#include <hip/hip_runtime.h>

#include <atomic>

#include "launch.h"

namespace {
constexpr int kMaxDevices = 64;
std::atomic<unsigned> g_packed[kMaxDevices];  // cus << 8 | xcds, 0 = not asked yet
std::atomic<unsigned> g_wall_khz[kMaxDevices];  // written before g_packed
}  // namespace

int fc_device(FcDevice *out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return (int)hipGetLastError();
    if (dev < 0 || dev >= kMaxDevices) return (int)hipErrorInvalidDevice;
    unsigned v = g_packed[dev].load(std::memory_order_acquire);
    if (v == 0) {  // every thread that finds 0 computes the same value
        int cus = 0, xcds = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
            return (int)hipGetLastError() ? (int)hipErrorInvalidDevice : (int)hipErrorInvalidDevice;
        if (hipDeviceGetAttribute(&xcds, hipDeviceAttributeNumberOfXccs, dev) != hipSuccess || xcds < 1) {
            (void)hipGetLastError();
            xcds = 1;  // a runtime that cannot say: treat the chip as one partition
        }
        if (xcds > 255 || cus % xcds != 0) xcds = 1;
        int khz = 0;
        if (hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) != hipSuccess || khz < 1) {
            (void)hipGetLastError();
            khz = 0;  // unknown: the launchers then leave their store streams unpaced
        }
        g_wall_khz[dev].store((unsigned)khz, std::memory_order_relaxed);
        v = ((unsigned)cus << 8) | (unsigned)xcds;
        g_packed[dev].store(v, std::memory_order_release);
    }
    out->cus = v >> 8;
    out->xcds = v & 255u;
    out->wall_khz = g_wall_khz[dev].load(std::memory_order_relaxed);
    return 0;
}
