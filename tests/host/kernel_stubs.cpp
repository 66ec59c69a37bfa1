// Stand-ins for the kernel launchers of libtmps (paper_2410_14312_amd/csrc/kernels.h) in host-only sanitizer builds of
// the stage executor: nothing is launched, every launcher reports success, and the workspace sizes are small fixed
// functions of the shape.  Only the host logic of csrc/stage.cpp (layout, argument checks, slot and buffer
// bookkeeping) is exercised by such a build.
#include <string.h>

#include "../../paper_2410_14312_amd/csrc/kernels.h"

namespace tmps {
hipError_t dense_forward(int dtype, const void* x, const void* w, const float* bias, void* y, int B, int Din, int Dout, int act, int out_f32, const void* res, void* zout, float* ws, hipStream_t s) { return hipSuccess; }
hipError_t dense_dgrad(int dtype, const void* dy, const void* w, void* dx, const void* mask, int mask_mode, const void* add, int B, int Din, int Dout, float* ws, hipStream_t s) { return hipSuccess; }
hipError_t dense_wgrad(int dtype, const void* dy, const void* x, float* gw, int B, int Din, int Dout, float* ws, hipStream_t s) { return hipSuccess; }
hipError_t conv_forward(int dtype, const void* x, const void* w, const float* bias, void* y, const ConvShape& c, int relu, float* ws, hipStream_t s) { return hipSuccess; }
hipError_t conv_affine_forward(int dtype, const void* x, const void* w, const float* bias, void* z, const float* gain, const float* shift, void* aout, const void* res, void* yout, int relu, const ConvShape& c, float* ws, hipStream_t s) { return hipSuccess; }
hipError_t conv_dgrad(int dtype, const void* dy, const void* w, void* dx, const void* mask, const void* add, const ConvShape& c, float* ws, hipStream_t s) { return hipSuccess; }
hipError_t conv_wgrad(int dtype, const void* dy, const void* x, float* gw, const ConvShape& c, float* ws, hipStream_t s) { return hipSuccess; }
hipError_t maxpool_forward(int dtype, const void* x, void* y, int B, int H, int W, int C, int k, int stride, int pad, hipStream_t s) { return hipSuccess; }
hipError_t maxpool_backward(int dtype, const void* x, const void* dy, void* dx, int B, int H, int W, int C, int k, int stride, int pad, int relu_mask, hipStream_t s) { return hipSuccess; }
hipError_t affine_forward(int dtype, const void* x, const float* gain, const float* shift, void* y, int64_t rows, int C, int relu, hipStream_t s) { return hipSuccess; }
hipError_t affine_backward(int dtype, const void* dy, const void* x, const float* gain, void* dx, float* dgain_dshift, float* ws, int64_t rows, int C, hipStream_t s) { return hipSuccess; }
hipError_t resadd_forward(int dtype, const void* a, const void* b, void* y, int64_t n, int relu, hipStream_t s) { return hipSuccess; }
hipError_t avgpool_forward(int dtype, const void* x, void* y, int B, int HW, int C, hipStream_t s) { return hipSuccess; }
hipError_t avgpool_backward(int dtype, const void* dy, const void* x, void* dx, int B, int HW, int C, int relu_mask, hipStream_t s) { return hipSuccess; }
hipError_t layernorm_forward(int dtype, const void* x, const float* gamma, const float* beta, void* y, float* stats, int64_t rows, int D, float eps, hipStream_t s) { return hipSuccess; }
hipError_t layernorm_backward(int dtype, const void* dy, const void* x, const float* stats, const float* gamma, const void* add, void* dx, float* dgamma_dbeta, float* ws, int64_t rows, int D, hipStream_t s) { return hipSuccess; }
hipError_t attention_forward(int dtype, const void* qkv, void* o, float* lse, int B, int S, int D, int H, hipStream_t s) { return hipSuccess; }
hipError_t attention_backward(int dtype, const void* qkv, const void* o, const void* dout, const float* lse, float* delta, void* dqkv, int B, int S, int D, int H, hipStream_t s) { return hipSuccess; }
hipError_t embedding_forward(int dtype, const int32_t* tok, const void* wte, const void* wpe, void* y, int64_t rows, int S, int D, int vocab, hipStream_t s) { return hipSuccess; }
hipError_t embedding_backward(int dtype, const int32_t* tok, const void* dy, float* dwte, float* dwpe, int64_t B, int S, int D, int vocab, hipStream_t s) { return hipSuccess; }
hipError_t softmax_ce(int dtype, const float* logits, const int32_t* labels, void* dlogits, float* row_loss, int rows, int C, float inv_M, hipStream_t s) { return hipSuccess; }
hipError_t reduce_scaled_sum(const float* in, int n, float scale, float* out, hipStream_t s) { return hipSuccess; }
hipError_t relu_mask(int dtype, const void* dy, const void* y, void* dz, int64_t n, hipStream_t s) { return hipSuccess; }
hipError_t sgd_momentum(float* w, float* buf, const float* g, void* wcopy_bf16, int64_t n, float lr, float mu, hipStream_t s) { return hipSuccess; }
hipError_t cast_f32_to_bf16(const float* in, void* out, int64_t n, hipStream_t s) { return hipSuccess; }
hipError_t copy_bytes(void* dst, const void* src, size_t bytes, hipStream_t) { memcpy(dst, src, bytes); return hipSuccess; }
GemmPlan plan_gemm(int64_t, int64_t, int64_t) { return GemmPlan{64, 1}; }
size_t gemm_workspace_elems(int64_t M, int64_t N, int64_t, int with_rowsum) { return (size_t)(2 * (M * N + (with_rowsum ? M : 0))); }
size_t affine_workspace_elems(int64_t, int C) { return (size_t)(2 * C * 8); }
size_t layernorm_workspace_elems(int64_t, int D) { return (size_t)(2 * D * 8); }
size_t attention_workspace_elems(int B, int S, int H) { return (size_t)B * S * H; }
}  // namespace tmps

// Profiling is off in these builds, and the three HIP runtime calls the stage executor makes itself are replaced: a
// "device-to-device" copy is a host memcpy here (the regions are host memory), so that the sanitizer also checks the
// bounds of the stash copies.  Nothing in such a build can reach a GPU.
#include <string.h>

#include "../../paper_2410_14312_amd/csrc/profile.h"

namespace tmps {
bool profile_on() { return false; }
void profile_begin(int, hipStream_t) {}
void profile_end(int, hipStream_t) {}
bool profile_kernel_begin(KernelEvents&) { return false; }
void profile_kernel_end(int, const KernelEvents&) {}
}  // namespace tmps

extern "C" hipError_t hipMemcpyAsync(void* dst, const void* src, size_t bytes, hipMemcpyKind, hipStream_t) {
    memcpy(dst, src, bytes);
    return hipSuccess;
}
extern "C" hipError_t hipEventDestroy(hipEvent_t) { return hipSuccess; }
// (graph replay is off in these builds: the calls exist for the linker only)
extern "C" hipError_t hipGraphExecDestroy(hipGraphExec_t) { return hipSuccess; }
extern "C" hipError_t hipGraphDestroy(hipGraph_t) { return hipSuccess; }
extern "C" hipError_t hipGraphLaunch(hipGraphExec_t, hipStream_t) { return hipErrorNotSupported; }
extern "C" hipError_t hipGraphInstantiate(hipGraphExec_t*, hipGraph_t, hipGraphNode_t*, char*, size_t) { return hipErrorNotSupported; }
extern "C" hipError_t hipStreamBeginCapture(hipStream_t, hipStreamCaptureMode) { return hipErrorNotSupported; }
extern "C" hipError_t hipStreamEndCapture(hipStream_t, hipGraph_t*) { return hipErrorNotSupported; }
extern "C" const char* hipGetErrorString(hipError_t) { return "stub"; }
