// Shared host-side helpers of libtmps: error text, HIP error mapping.
#pragma once
#include <hip/hip_runtime.h>
#include <stdarg.h>
#include <stdio.h>

#include "../../include/tmps.h"

namespace tmps {

// Sets the thread-local error text and returns `code`.
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

#define TMPS_HIP(expr)                                                                        \
    do {                                                                                      \
        hipError_t e_ = (expr);                                                               \
        if (e_ != hipSuccess)                                                                 \
            return ::tmps::fail(TMPS_EHIP, "%s failed: %s", #expr, hipGetErrorString(e_));    \
    } while (0)

}  // namespace tmps
