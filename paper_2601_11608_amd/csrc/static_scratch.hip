// foldconv_forward_static: the folded convolution for callers that cannot allocate device memory.
// The kernel-order copy of the expanded filter, which foldconv_forward keeps in a workspace the
// caller brings, lives here in a device array that is part of the library's code object.
#include <hip/hip_runtime.h>

#include <mutex>

#include "launch.h"

// One copy per GPU the library runs on, resident until the process ends.  No kernel names the
// array; it is kept, and made findable by name in the code object, because host code below takes
// its symbol (an explicit "used" attribute would keep it as a local symbol the runtime's lookup
// cannot see).
static __device__ __align__(256) unsigned char scratch[FOLDCONV_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_lock;
void *g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each GPU, resolved on first use

// In host code the array's name is only a handle for the runtime; the address kernels can use
// comes from hipGetSymbolAddress, per device (each GPU holds its own copy at its own address).
int scratch_on_current_device(void **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        return FOLDCONV_ERR_HIP;
    }
    std::lock_guard<std::mutex> hold(g_lock);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return FOLDCONV_ERR_HIP;
        }
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return FOLDCONV_OK;
}
}  // namespace

extern "C" int foldconv_forward_static(foldconv_plan_t plan, const void *x_fold, const void *w_exp, const void *bias,
                                       void *y, unsigned flags, void *stream) {
    if (!plan || plan->magic != FOLDCONV_MAGIC) return FOLDCONV_ERR_BADARG;
    // the scratch is re-written by every call, so there is no earlier content to rely on
    if (flags & (FOLDCONV_FLAG_FILTER_PACKED | FOLDCONV_FLAG_FILTER_COMPACT)) return FOLDCONV_ERR_BADARG;
    const long long need = plan->s.workspace_bytes;
    if (need > (long long)FOLDCONV_STATIC_SCRATCH_BYTES) return FOLDCONV_ERR_SCRATCH;
    if (need == 0)  // the element-gather kernel reads w' as it is: no scratch involved
        return fc_forward(plan, x_fold, w_exp, bias, y, nullptr, 0, flags, stream, false);
    void *ptr = nullptr;
    const int st = scratch_on_current_device(&ptr);
    if (st != FOLDCONV_OK) return st;
    // same kernels as foldconv_forward: pack w' into the scratch, then the convolution reads it
    return fc_forward(plan, x_fold, w_exp, bias, y, ptr, (size_t)FOLDCONV_STATIC_SCRATCH_BYTES, flags, stream, false);
}
