// Optional per-kernel-class timing with HIP events recorded on the launching stream.
#pragma once
#include <hip/hip_runtime.h>

namespace tmps {

enum KernelClass {
    kcDenseFwd = 0, kcDenseDgrad, kcDenseWgrad, kcConvFwd, kcConvDgrad, kcConvWgrad, kcSoftmaxCE,
    kcUpdate, kcPoolFwd, kcPoolBwd, kcReluMask, kcReduce, kcCopy, kcEventPair, kcSplitFinish, kcSliceSum, kcLayerNorm,
    kcAttnFwd, kcAttnBwd, kcEmbedding, kcAffine, kcResAdd, kcCount
};

bool profile_on();
// Record a start/stop event pair around a launch of class `kc` on stream `s`.
void profile_begin(int kc, hipStream_t s);
void profile_end(int kc, hipStream_t s);

// Timing of ONE kernel by its own dispatch timestamps: the two events are handed to
// hipExtLaunchKernelGGL, which stamps them with the start and the end of that kernel's execution.
struct KernelEvents {
    hipEvent_t start, stop;
};
bool profile_kernel_begin(KernelEvents& ev);          // false when profiling is off (or no event could be made)
void profile_kernel_end(int kc, const KernelEvents& ev);

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
