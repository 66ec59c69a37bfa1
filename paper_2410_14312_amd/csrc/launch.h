// Kernel launch helper shared by the .hip files: while profiling is enabled the kernel is launched with a
// start and a stop event of its own, which the runtime stamps with the beginning and the end of that
// kernel's execution on the device.
#pragma once
#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>

#include "profile.h"

namespace tmps {

template <class Kern, class... Args>
static hipError_t launch_timed(int kc, Kern kern, dim3 grid, dim3 block, unsigned lds, hipStream_t s, Args... args) {
    KernelEvents ev;
    if (profile_kernel_begin(ev)) {
        hipExtLaunchKernelGGL(kern, grid, block, lds, s, ev.start, ev.stop, 0, args...);
        profile_kernel_end(kc, ev);
    } else {
        hipLaunchKernelGGL(kern, grid, block, lds, s, args...);
    }
    return hipGetLastError();
}

}  // namespace tmps
