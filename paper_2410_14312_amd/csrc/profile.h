// Optional per-kernel-class timing with HIP events recorded on the launching stream.
#pragma once
#include <hip/hip_runtime.h>

namespace tmps {

enum KernelClass {
    kcDenseFwd = 0, kcDenseDgrad, kcDenseWgrad, kcConvFwd, kcConvDgrad, kcConvWgrad, kcSoftmaxCE,
    kcUpdate, kcPoolFwd, kcPoolBwd, kcReluMask, kcReduce, kcCopy, kcCount
};

bool profile_on();
// Record a start/stop event pair around a launch of class `kc` on stream `s`.
void profile_begin(int kc, hipStream_t s);
void profile_end(int kc, hipStream_t s);

struct ProfileScope {
    int kc;
    hipStream_t s;
    bool on;
    ProfileScope(int kc_, hipStream_t s_) : kc(kc_), s(s_), on(profile_on()) {
        if (on) profile_begin(kc, s);
    }
    ~ProfileScope() {
        if (on) profile_end(kc, s);
    }
};

}  // namespace tmps
