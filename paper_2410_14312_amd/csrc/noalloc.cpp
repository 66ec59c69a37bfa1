// tmps_forward_micro_static: the forward pass of one micro-batch for callers that cannot allocate device memory for
// a workspace (code under stream capture, serving loops, harnesses that forbid hipMalloc).  The contractions of a
// forward pass split their k-loop over several workgroups when the output has few tiles; the fp32 partial sums live
// in a workspace, which tmps_forward_micro takes from the stage's caller-owned scratch region.  Here the workspace is
// a fixed array in device memory that belongs to the library's code object: every GPU the library runs on holds its
// own copy from the moment the code object is loaded there until the process ends.
#include <mutex>

#include "stage.h"

using namespace tmps;

namespace {

constexpr size_t kStaticScratchBytes = TMPS_STATIC_SCRATCH_BYTES;

// The workspace.  In host code this name only stands for the symbol: its device address is asked for once per
// device (device_scratch below) and only that address is ever handed to a kernel or a runtime call.
__device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_lock;
void* g_ptr[kMaxDevices];   // device address of `scratch` on device d, null until asked for

// Address of this device's copy of the workspace; the device must be current (it is: the caller's stream lives on it).
int device_scratch(float** out) {
    int dev = -1;
    TMPS_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(TMPS_EUNSUPPORTED, "device ordinal %d outside 0..%d", dev, kMaxDevices - 1);
    std::lock_guard<std::mutex> hold(g_lock);
    if (!g_ptr[dev]) {
        void* p = nullptr;
        hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return fail(TMPS_EHIP, "hipGetSymbolAddress of the static workspace failed on device %d: %s", dev, hipGetErrorString(e));
        g_ptr[dev] = p;
    }
    *out = static_cast<float*>(g_ptr[dev]);
    return TMPS_OK;
}

}  // namespace

extern "C" int tmps_forward_micro_static(tmps_stage* st, int slot, const void* x, void* y, const int32_t* labels,
                                         float* loss_out, void* hip_stream) {
    if (!st) return fail(TMPS_EINVAL, "stage is null");
    if (st->ws_fwd_bytes > kStaticScratchBytes)
        return fail(TMPS_ECAP, "the forward pass of this stage needs %zu bytes of workspace, the static one holds %zu: use tmps_forward_micro",
                    st->ws_fwd_bytes, kStaticScratchBytes);
    float* ws = nullptr;
    int rc = device_scratch(&ws);
    if (rc != TMPS_OK) return rc;
    // Nothing in the workspace has to start at zero: every k-slice writes its whole partial tile before the finishing
    // kernel of the same launch sequence reads it, so what an earlier call left behind is never read.
    return forward_with_workspace(st, slot, x, y, labels, loss_out, hip_stream, ws);
}
