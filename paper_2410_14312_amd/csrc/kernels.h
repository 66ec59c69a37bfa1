// Host-side launch interface of the HIP kernels (internal to libtmps).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace tmps {

// dtype codes match TMPS_F32 / TMPS_BF16_F32MASTER
constexpr int kF32 = 0;
constexpr int kBF16 = 1;

inline size_t act_bytes(int dtype) { return dtype == kBF16 ? 2 : 4; }

struct ConvShape {
    int B, H, W, Cin, Ho, Wo, Cout, R, S, stride, pad;
};

// Tile edge (64 or 128) and number of k-slices chosen for a [M x N x K] contraction, and the fp32
// workspace elements its partial sums need (0 without a split).  with_rowsum: weight-gradient GEMMs
// also keep M row sums per slice.  Every launcher below takes that workspace as `ws` (may be null:
// then nothing is split).
struct GemmPlan {
    int tile, slices;
};
GemmPlan plan_gemm(int64_t M, int64_t N, int64_t K);
size_t gemm_workspace_elems(int64_t M, int64_t N, int64_t K, int with_rowsum);

// y[B, Dout] = act(x[B, Din] w^T + b).  w is the working copy (bf16 or fp32 per dtype), bias fp32.
// out_f32: write fp32 regardless of dtype (logits).
// act: 0 none, 1 ReLU, 2 exact GELU (then zout, if not null, receives the derivative gelu'(pre-activation) for the backward pass).  res (may be
// null): tensor of y's shape and dtype added after the activation (residual connection).
hipError_t dense_forward(int dtype, const void* x, const void* w, const float* bias, void* y, int B,
                         int Din, int Dout, int act, int out_f32, const void* res, void* zout, float* ws,
                         hipStream_t s);
// dx[B, Din] = dy[B, Dout] w, passed through the activation of the layer below: mask_mode 1: zeroed
// where mask[B, Din] <= 0 (mask = that layer's output); mask_mode 2: times gelu'(mask) (mask = that
// layer's pre-activation).  mask may be null; activation dtype.
hipError_t dense_dgrad(int dtype, const void* dy, const void* w, void* dx, const void* mask, int mask_mode,
                       const void* add, int B, int Din, int Dout, float* ws, hipStream_t s);
// `add` (may be null; may be dx itself): tensor of dx's shape added BEFORE the mask is applied: the
// gradient that other readers of the same input have already contributed.
// gw[Dout, Din] = dy^T x and gb[Dout] = column sums of dy, with gb stored right after gw.
hipError_t dense_wgrad(int dtype, const void* dy, const void* x, float* gw, int B, int Din, int Dout,
                       float* ws, hipStream_t s);

hipError_t conv_forward(int dtype, const void* x, const void* w, const float* bias, void* y,
                        const ConvShape& c, int relu, float* ws, hipStream_t s);
// Convolution (no activation of its own) fused with the per-channel affine layer that follows it and, when res or
// aout is given, with the residual join after that: y -> z (the convolution's result), aout (may be null) the affine
// layer's result, yout = act(affine + res) (res may be null).
hipError_t conv_affine_forward(int dtype, const void* x, const void* w, const float* bias, void* z, const float* gain,
                               const float* shift, void* aout, const void* res, void* yout, int relu, const ConvShape& c,
                               float* ws, hipStream_t s);
hipError_t conv_dgrad(int dtype, const void* dy, const void* w, void* dx, const void* mask, const void* add,
                      const ConvShape& c, float* ws, hipStream_t s);
hipError_t conv_wgrad(int dtype, const void* dy, const void* x, float* gw, const ConvShape& c,
                      float* ws, hipStream_t s);

// 2-D max pooling, channels-last, no padding.  Backward recomputes the winner (first maximum in
// row-major window order) from the stored input; relu_mask: also zero where the input is <= 0.
hipError_t maxpool_forward(int dtype, const void* x, void* y, int B, int H, int W, int C, int k,
                           int stride, int pad, hipStream_t s);
hipError_t maxpool_backward(int dtype, const void* x, const void* dy, void* dx, int B, int H, int W,
                            int C, int k, int stride, int pad, int relu_mask, hipStream_t s);

// Per-channel affine layer on channels-last rows: y[r, c] = gain[c] x[r, c] + shift[c], then ReLU if asked.
hipError_t affine_forward(int dtype, const void* x, const float* gain, const float* shift, void* y, int64_t rows, int C,
                          int relu, hipStream_t s);
// dx (may be null) = gain * dy; dgain_dshift: C gain gradients (sum of dy * x) followed by C shift gradients (sum
// of dy); dy has already passed through the layer's own ReLU; ws: affine_workspace_elems.
hipError_t affine_backward(int dtype, const void* dy, const void* x, const float* gain, void* dx, float* dgain_dshift,
                           float* ws, int64_t rows, int C, hipStream_t s);
size_t affine_workspace_elems(int64_t rows, int C);

// y = act(a + b), n elements.
hipError_t resadd_forward(int dtype, const void* a, const void* b, void* y, int64_t n, int relu, hipStream_t s);

// Global average pooling [B, HW, C] -> [B, C] and its gradient (relu_mask: zero where the stored input is <= 0).
hipError_t avgpool_forward(int dtype, const void* x, void* y, int B, int HW, int C, hipStream_t s);
hipError_t avgpool_backward(int dtype, const void* dy, const void* x, void* dx, int B, int HW, int C, int relu_mask,
                            hipStream_t s);

// Layer normalisation over rows of D features.  stats[rows][2] = (mean, 1/std) of the forward pass.
hipError_t layernorm_forward(int dtype, const void* x, const float* gamma, const float* beta, void* y,
                             float* stats, int64_t rows, int D, float eps, hipStream_t s);
// dx (may be null) = gradient w.r.t. x, plus `add` (may be null: gradient of a residual connection that
// joins x); dgamma_dbeta: D gain gradients followed by D shift gradients; ws: layernorm_workspace_elems.
hipError_t layernorm_backward(int dtype, const void* dy, const void* x, const float* stats, const float* gamma,
                              const void* add, void* dx, float* dgamma_dbeta, float* ws, int64_t rows, int D,
                              hipStream_t s);
size_t layernorm_workspace_elems(int64_t rows, int D);

// Causal multi-head self-attention on packed rows [q | k | v] (3*D features, head h owns features
// h*D/H.. of each part).  o[B*S, D]; lse[B, H, S] = log-sum-exp of the scaled scores of each query.
hipError_t attention_forward(int dtype, const void* qkv, void* o, float* lse, int B, int S, int D, int H,
                             hipStream_t s);
// dqkv[B*S, 3*D] from the gradient dout[B*S, D] of the output; delta: workspace of B*H*S floats.
hipError_t attention_backward(int dtype, const void* qkv, const void* o, const void* dout, const float* lse,
                              float* delta, void* dqkv, int B, int S, int D, int H, hipStream_t s);
size_t attention_workspace_elems(int B, int S, int H);

// y[row] = wte[tok[row]] + wpe[row % S] (tables in the contraction dtype), and the table gradients
// (fp32; dwte cleared, then every occurring token's rows of dy added in row order, no atomic adds; dwpe summed over the batch).
hipError_t embedding_forward(int dtype, const int32_t* tok, const void* wte, const void* wpe, void* y,
                             int64_t rows, int S, int D, int vocab, hipStream_t s);
hipError_t embedding_backward(int dtype, const int32_t* tok, const void* dy, float* dwte, float* dwpe,
                              int64_t B, int S, int D, int vocab, hipStream_t s);

// Softmax cross-entropy of `rows` rows of fp32 logits: row_loss[rows] fp32 and
// dlogits[rows, C] = (softmax - onehot) * inv_M in the gradient dtype.
hipError_t softmax_ce(int dtype, const float* logits, const int32_t* labels, void* dlogits,
                      float* row_loss, int rows, int C, float inv_M, hipStream_t s);
// out[0] = scale * sum(in[0..n))   (deterministic single-block tree)
hipError_t reduce_scaled_sum(const float* in, int n, float scale, float* out, hipStream_t s);

// dz = y > 0 ? dy : 0
hipError_t relu_mask(int dtype, const void* dy, const void* y, void* dz, int64_t n, hipStream_t s);

// buf <- mu*buf + g;  w <- w - lr*buf;  wcopy <- bf16(w) when wcopy != null
hipError_t sgd_momentum(float* w, float* buf, const float* g, void* wcopy_bf16, int64_t n, float lr,
                        float mu, hipStream_t s);
hipError_t cast_f32_to_bf16(const float* in, void* out, int64_t n, hipStream_t s);
// dst[0..bytes) = src[0..bytes), both on the device, by a kernel
hipError_t copy_bytes(void* dst, const void* src, size_t bytes, hipStream_t s);

}  // namespace tmps
