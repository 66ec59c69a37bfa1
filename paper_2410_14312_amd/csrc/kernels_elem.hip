// Bandwidth-bound kernels of the stage step: softmax cross-entropy, momentum update, max pooling,
// ReLU gradient mask, casts and small reductions.
#include "gemm.hip.h"
#include "kernels.h"

namespace tmps {

static inline int cdiv64(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// ------------------------------------------------------------------------- softmax cross-entropy
// One wave per row; 4 rows per block.  dlogits = (softmax - onehot) * inv_M, loss = lse - z[label].
template <typename TG>
__global__ __launch_bounds__(256) void softmax_ce_kernel(const float* __restrict__ logits,
                                                         const int32_t* __restrict__ labels,
                                                         TG* __restrict__ dlogits,
                                                         float* __restrict__ row_loss, int rows, int C,
                                                         float inv_M) {
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const float* z = logits + (int64_t)row * C;
    float mx = -INFINITY;
    for (int c = lane; c < C; c += 64) mx = fmaxf(mx, z[c]);
    mx = wave_max(mx);
    float sum = 0.0f;
    for (int c = lane; c < C; c += 64) sum += expf(z[c] - mx);
    sum = wave_sum(sum);
    const float inv = 1.0f / sum;
    const int label = labels[row];
    const bool label_ok = label >= 0 && label < C;  // an out-of-range label gives a NaN loss, never a wild read
    TG* g = dlogits + (int64_t)row * C;
    for (int c = lane; c < C; c += 64) {
        float p = expf(z[c] - mx) * inv;
        g[c] = from_f32<TG>((p - (c == label ? 1.0f : 0.0f)) * inv_M);
    }
    if (lane == 0) row_loss[row] = label_ok ? logf(sum) - (z[label] - mx) : NAN;
}

// Wide rows (a vocabulary): one 256-thread block per row.  First pass keeps a running (max, sum) per thread
// (online softmax), combined across the block; second pass writes the gradient.
template <typename TG>
__global__ __launch_bounds__(256) void softmax_ce_wide_kernel(const float* __restrict__ logits,
                                                              const int32_t* __restrict__ labels,
                                                              TG* __restrict__ dlogits, float* __restrict__ row_loss,
                                                              int C, float inv_M) {
    __shared__ float sm[4], ss[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t row = blockIdx.x;
    const float* z = logits + row * C;
    float mx = -INFINITY, sum = 0.0f;
    for (int c = tid; c < C; c += 256) {
        const float v = z[c];
        if (v > mx) {
            sum = sum * expf(mx - v) + 1.0f;
            mx = v;
        } else {
            sum += expf(v - mx);
        }
    }
    const float wm = wave_max(mx);
    sum = wave_sum(sum * expf(mx - wm));   // a thread that saw nothing has sum 0 and mx -inf: 0 * exp(-inf) = 0
    if (lane == 0) {
        sm[wave] = wm;
        ss[wave] = sum;
    }
    __syncthreads();
    const float bm = fmaxf(fmaxf(sm[0], sm[1]), fmaxf(sm[2], sm[3]));
    float bs = 0.0f;
#pragma unroll
    for (int w = 0; w < 4; ++w) bs += ss[w] * expf(sm[w] - bm);
    const float inv = 1.0f / bs;
    const int label = labels[row];
    const bool label_ok = label >= 0 && label < C;
    TG* g = dlogits + row * C;
    for (int c = tid; c < C; c += 256) {
        const float p = expf(z[c] - bm) * inv;
        g[c] = from_f32<TG>((p - (c == label ? 1.0f : 0.0f)) * inv_M);
    }
    if (tid == 0) row_loss[row] = label_ok ? logf(bs) - (z[label] - bm) : NAN;
}

// Wide rows that fit in LDS (C fp32 values, C % 4 == 0): one 1024-thread block per row reads the row from HBM ONCE,
// keeps it in LDS for the maximum, the sum and the gradient, and writes the gradient: algorithmic traffic exactly.
// A row of a large vocabulary takes most of a compute unit's LDS, so one workgroup is all a unit holds: 16 waves
// (not 4) keep enough loads in flight.  Exponentials on the hardware exp2 (a few ulp of fp32).
constexpr int kCeThreads = 1024;
template <typename TG>
__global__ __launch_bounds__(kCeThreads) void softmax_ce_lds_kernel(const float* __restrict__ logits, const int32_t* __restrict__ labels,
                                                                    TG* __restrict__ dlogits, float* __restrict__ row_loss, int C,
                                                                    float inv_M) {
    extern __shared__ __attribute__((aligned(16))) float srow[];
    constexpr int NWV = kCeThreads / 64;
    __shared__ float sm[NWV], ss[NWV];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t row = blockIdx.x;
    const float4* z4 = reinterpret_cast<const float4*>(logits + row * C);
    float4* s4 = reinterpret_cast<float4*>(srow);
    const int C4 = C >> 2;
    float mx = -INFINITY;
    for (int c = tid; c < C4; c += kCeThreads) {
        const float4 v = z4[c];
        s4[c] = v;
        mx = fmaxf(fmaxf(mx, fmaxf(v.x, v.y)), fmaxf(v.z, v.w));
    }
    mx = wave_max(mx);
    if (lane == 0) sm[wave] = mx;
    __syncthreads();
    float bm = sm[0];
#pragma unroll
    for (int w = 1; w < NWV; ++w) bm = fmaxf(bm, sm[w]);
    float sum = 0.0f;
    for (int c = tid; c < C4; c += kCeThreads) {
        float4 v = s4[c];
        v.x = __expf(v.x - bm); v.y = __expf(v.y - bm); v.z = __expf(v.z - bm); v.w = __expf(v.w - bm);
        s4[c] = v;   // keep the exponentials: the gradient needs them again
        sum += (v.x + v.y) + (v.z + v.w);
    }
    sum = wave_sum(sum);
    if (lane == 0) ss[wave] = sum;
    __syncthreads();
    float bs = 0.0f;
#pragma unroll
    for (int w = 0; w < NWV; ++w) bs += ss[w];
    const float inv = 1.0f / bs;
    const int label = labels[row];
    const bool label_ok = label >= 0 && label < C;
    TG* g = dlogits + row * C;
    for (int c = tid; c < C4; c += kCeThreads) {
        const float4 e = s4[c];
        float p[4] = {e.x * inv, e.y * inv, e.z * inv, e.w * inv};
        const int c0 = c * 4;
#pragma unroll
        for (int k = 0; k < 4; ++k) p[k] = (p[k] - (c0 + k == label ? 1.0f : 0.0f)) * inv_M;
        if constexpr (sizeof(TG) == 2) {
            union { bf16_t h[4]; uint2 u; } pk;
#pragma unroll
            for (int k = 0; k < 4; ++k) pk.h[k] = (bf16_t)p[k];
            *reinterpret_cast<uint2*>(g + c0) = pk.u;
        } else {
            *reinterpret_cast<float4*>(g + c0) = make_float4(p[0], p[1], p[2], p[3]);
        }
    }
    if (tid == 0) row_loss[row] = label_ok ? logf(bs) - (logits[row * C + label] - bm) : NAN;
}

// The same with the row in registers (C <= 4096 * NV): NV 16-byte pieces per thread, no LDS beyond the block reductions,
// so that a compute unit holds two rows at a time and one row's memory phase overlaps the other's arithmetic (with the row
// in LDS a unit holds one).  The same values are combined in the same order as above: the results are the same bit for bit.
template <typename TG, int NV>
__global__ __launch_bounds__(kCeThreads, 8) void softmax_ce_reg_kernel(const float* __restrict__ logits, const int32_t* __restrict__ labels,
                                                                       TG* __restrict__ dlogits, float* __restrict__ row_loss, int C,
                                                                       float inv_M) {
    constexpr int NWV = kCeThreads / 64;
    __shared__ float sm[NWV], ss[NWV];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t row = blockIdx.x;
    const float4* z4 = reinterpret_cast<const float4*>(logits + row * C);
    const int C4 = C >> 2;
    float4 v[NV];
#pragma unroll
    for (int k = 0; k < NV; ++k) {
        const int c = tid + k * kCeThreads;
        if (c < C4) v[k] = z4[c];
    }
    float mx = -INFINITY;
#pragma unroll
    for (int k = 0; k < NV; ++k)
        if (tid + k * kCeThreads < C4) mx = fmaxf(fmaxf(mx, fmaxf(v[k].x, v[k].y)), fmaxf(v[k].z, v[k].w));
    mx = wave_max(mx);
    if (lane == 0) sm[wave] = mx;
    __syncthreads();
    float bm = sm[0];
#pragma unroll
    for (int w = 1; w < NWV; ++w) bm = fmaxf(bm, sm[w]);
    float sum = 0.0f;
#pragma unroll
    for (int k = 0; k < NV; ++k)
        if (tid + k * kCeThreads < C4) {
            v[k].x = __expf(v[k].x - bm); v[k].y = __expf(v[k].y - bm); v[k].z = __expf(v[k].z - bm); v[k].w = __expf(v[k].w - bm);
            sum += (v[k].x + v[k].y) + (v[k].z + v[k].w);
        }
    sum = wave_sum(sum);
    if (lane == 0) ss[wave] = sum;
    __syncthreads();
    float bs = 0.0f;
#pragma unroll
    for (int w = 0; w < NWV; ++w) bs += ss[w];
    const float inv = 1.0f / bs;
    const int label = labels[row];
    const bool label_ok = label >= 0 && label < C;
    TG* g = dlogits + row * C;
#pragma unroll
    for (int k = 0; k < NV; ++k) {
        const int c = tid + k * kCeThreads;
        if (c < C4) {
            float p[4] = {v[k].x * inv, v[k].y * inv, v[k].z * inv, v[k].w * inv};
            const int c0 = c * 4;
#pragma unroll
            for (int e = 0; e < 4; ++e) p[e] = (p[e] - (c0 + e == label ? 1.0f : 0.0f)) * inv_M;
            if constexpr (sizeof(TG) == 2) {
                union { bf16_t h[4]; uint2 u; } pk;
#pragma unroll
                for (int e = 0; e < 4; ++e) pk.h[e] = (bf16_t)p[e];
                *reinterpret_cast<uint2*>(g + c0) = pk.u;
            } else {
                *reinterpret_cast<float4*>(g + c0) = make_float4(p[0], p[1], p[2], p[3]);
            }
        }
    }
    if (tid == 0) row_loss[row] = label_ok ? logf(bs) - (logits[row * C + label] - bm) : NAN;
}

hipError_t softmax_ce(int dtype, const float* logits, const int32_t* labels, void* dlogits, float* row_loss,
                      int rows, int C, float inv_M, hipStream_t s) {
    if (rows <= 0) return hipSuccess;
    if (C > 2048 && C % 4 == 0 && C <= 4096 * 8 && (reinterpret_cast<uintptr_t>(logits) & 15) == 0 &&
        (reinterpret_cast<uintptr_t>(dlogits) & 15) == 0) {
        const bool small = C <= 4096 * 4;
        if (dtype == kBF16) {
            if (small) hipLaunchKernelGGL((softmax_ce_reg_kernel<bf16_t, 4>), dim3(rows), dim3(kCeThreads), 0, s, logits, labels, (bf16_t*)dlogits, row_loss, C, inv_M);
            else hipLaunchKernelGGL((softmax_ce_reg_kernel<bf16_t, 8>), dim3(rows), dim3(kCeThreads), 0, s, logits, labels, (bf16_t*)dlogits, row_loss, C, inv_M);
        } else {
            if (small) hipLaunchKernelGGL((softmax_ce_reg_kernel<float, 4>), dim3(rows), dim3(kCeThreads), 0, s, logits, labels, (float*)dlogits, row_loss, C, inv_M);
            else hipLaunchKernelGGL((softmax_ce_reg_kernel<float, 8>), dim3(rows), dim3(kCeThreads), 0, s, logits, labels, (float*)dlogits, row_loss, C, inv_M);
        }
        return hipGetLastError();
    }
    if (C > 2048 && C % 4 == 0 && (size_t)C * 4 <= 150 * 1024 && (reinterpret_cast<uintptr_t>(logits) & 15) == 0 &&
        (reinterpret_cast<uintptr_t>(dlogits) & 15) == 0) {
        const unsigned lds = (unsigned)C * 4;
        if (dtype == kBF16) {
            static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(softmax_ce_lds_kernel<bf16_t>),
                                                         hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024);
            if (attr != hipSuccess) return attr;
            hipLaunchKernelGGL(softmax_ce_lds_kernel<bf16_t>, dim3(rows), dim3(kCeThreads), lds, s, logits, labels, (bf16_t*)dlogits,
                               row_loss, C, inv_M);
        } else {
            static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(softmax_ce_lds_kernel<float>),
                                                         hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024);
            if (attr != hipSuccess) return attr;
            hipLaunchKernelGGL(softmax_ce_lds_kernel<float>, dim3(rows), dim3(kCeThreads), lds, s, logits, labels, (float*)dlogits,
                               row_loss, C, inv_M);
        }
        return hipGetLastError();
    }
    if (C > 2048) {
        if (dtype == kBF16)
            hipLaunchKernelGGL(softmax_ce_wide_kernel<bf16_t>, dim3(rows), dim3(256), 0, s, logits, labels,
                               (bf16_t*)dlogits, row_loss, C, inv_M);
        else
            hipLaunchKernelGGL(softmax_ce_wide_kernel<float>, dim3(rows), dim3(256), 0, s, logits, labels,
                               (float*)dlogits, row_loss, C, inv_M);
        return hipGetLastError();
    }
    dim3 grid(cdiv64(rows, 4));
    if (dtype == kBF16)
        hipLaunchKernelGGL(softmax_ce_kernel<bf16_t>, grid, dim3(256), 0, s, logits, labels, (bf16_t*)dlogits,
                           row_loss, rows, C, inv_M);
    else
        hipLaunchKernelGGL(softmax_ce_kernel<float>, grid, dim3(256), 0, s, logits, labels, (float*)dlogits,
                           row_loss, rows, C, inv_M);
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void reduce_scaled_sum_kernel(const float* __restrict__ in, int n,
                                                                float scale, float* __restrict__ out) {
    __shared__ float part[4];
    float a = 0.0f;
    for (int i = threadIdx.x; i < n; i += 256) a += in[i];
    a = wave_sum(a);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = a;
    __syncthreads();
    if (threadIdx.x == 0) out[0] = (part[0] + part[1] + part[2] + part[3]) * scale;
}

hipError_t reduce_scaled_sum(const float* in, int n, float scale, float* out, hipStream_t s) {
    hipLaunchKernelGGL(reduce_scaled_sum_kernel, dim3(1), dim3(256), 0, s, in, n, scale, out);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------- ReLU gradient
template <typename T>
__global__ void relu_mask_kernel(const T* __restrict__ dy, const T* __restrict__ y, T* __restrict__ dz,
                                 int64_t n) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) dz[i] = to_f32(y[i]) > 0.0f ? dy[i] : T(0.0f);
}

// bf16, 8 elements (16 bytes) per thread and access
__global__ __launch_bounds__(256) void relu_mask_bf16x8_kernel(const bf16_t* __restrict__ dy, const bf16_t* __restrict__ y,
                                                               bf16_t* __restrict__ dz, int64_t n8) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n8) return;
    Pack8 g, v;
    g.u = reinterpret_cast<const uint4*>(dy)[i];
    v.u = reinterpret_cast<const uint4*>(y)[i];
#pragma unroll
    for (int e = 0; e < 8; ++e)
        if (!((float)v.h[e] > 0.0f)) g.h[e] = (bf16_t)0.0f;
    reinterpret_cast<uint4*>(dz)[i] = g.u;
}

hipError_t relu_mask(int dtype, const void* dy, const void* y, void* dz, int64_t n, hipStream_t s) {
    if (n <= 0) return hipSuccess;
    if (dtype == kBF16 && n % 8 == 0 && ((reinterpret_cast<uintptr_t>(dy) | reinterpret_cast<uintptr_t>(y) | reinterpret_cast<uintptr_t>(dz)) & 15) == 0) {
        hipLaunchKernelGGL(relu_mask_bf16x8_kernel, dim3(cdiv64(n / 8, 256)), dim3(256), 0, s, (const bf16_t*)dy, (const bf16_t*)y,
                           (bf16_t*)dz, n / 8);
        return hipGetLastError();
    }
    int blocks = cdiv64(n, 256);
    if (blocks > 4096) blocks = 4096;
    if (dtype == kBF16)
        hipLaunchKernelGGL(relu_mask_kernel<bf16_t>, dim3(blocks), dim3(256), 0, s, (const bf16_t*)dy,
                           (const bf16_t*)y, (bf16_t*)dz, n);
    else
        hipLaunchKernelGGL(relu_mask_kernel<float>, dim3(blocks), dim3(256), 0, s, (const float*)dy,
                           (const float*)y, (float*)dz, n);
    return hipGetLastError();
}

// ----------------------------------------------------------------------------- momentum update
// 4 parameters per thread: 16-byte loads of w, buf, g; 16-byte stores of w, buf; 8-byte store of the
// bf16 working copy.  The tail (n % 4) is handled by the last threads one element at a time.
__global__ __launch_bounds__(256) void sgd_momentum_kernel(float* __restrict__ w, float* __restrict__ buf,
                                                           const float* __restrict__ g,
                                                           bf16_t* __restrict__ wc, int64_t n, float lr,
                                                           float mu) {
    const int64_t n4 = n >> 2;
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n4; i += stride) {
        float4 wv = reinterpret_cast<const float4*>(w)[i];
        float4 bv = reinterpret_cast<const float4*>(buf)[i];
        float4 gv = reinterpret_cast<const float4*>(g)[i];
        bv.x = mu * bv.x + gv.x; bv.y = mu * bv.y + gv.y; bv.z = mu * bv.z + gv.z; bv.w = mu * bv.w + gv.w;
        wv.x -= lr * bv.x; wv.y -= lr * bv.y; wv.z -= lr * bv.z; wv.w -= lr * bv.w;
        reinterpret_cast<float4*>(buf)[i] = bv;
        reinterpret_cast<float4*>(w)[i] = wv;
        if (wc) {
            union { bf16_t h[4]; uint2 u; } pk;
            pk.h[0] = (bf16_t)wv.x; pk.h[1] = (bf16_t)wv.y; pk.h[2] = (bf16_t)wv.z; pk.h[3] = (bf16_t)wv.w;
            reinterpret_cast<uint2*>(wc)[i] = pk.u;
        }
    }
    int64_t t = (n4 << 2) + (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < n) {
        float b = mu * buf[t] + g[t];
        float x = w[t] - lr * b;
        buf[t] = b;
        w[t] = x;
        if (wc) wc[t] = (bf16_t)x;
    }
}

hipError_t sgd_momentum(float* w, float* buf, const float* g, void* wcopy_bf16, int64_t n, float lr, float mu,
                        hipStream_t s) {
    if (n <= 0) return hipSuccess;
    int blocks = cdiv64((n >> 2) + 4, 256);
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(sgd_momentum_kernel, dim3(blocks), dim3(256), 0, s, w, buf, g, (bf16_t*)wcopy_bf16, n,
                       lr, mu);
    return hipGetLastError();
}

__global__ void cast_f32_to_bf16_kernel(const float* __restrict__ in, bf16_t* __restrict__ out, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) out[i] = (bf16_t)in[i];
}

hipError_t cast_f32_to_bf16(const float* in, void* out, int64_t n, hipStream_t s) {
    if (n <= 0) return hipSuccess;
    int blocks = cdiv64(n, 256);
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(cast_f32_to_bf16_kernel, dim3(blocks), dim3(256), 0, s, in, (bf16_t*)out, n);
    return hipGetLastError();
}

// dst[0..bytes) = src[0..bytes) as a kernel (a captured graph of the backward pass then holds kernel nodes only):
// 16 bytes per thread and step where both addresses allow it, single bytes for the rest.
__global__ void copy_bytes_kernel(const unsigned char* __restrict__ src, unsigned char* __restrict__ dst, int64_t n16, int64_t bytes) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (int64_t i = t; i < n16; i += stride) reinterpret_cast<uint4*>(dst)[i] = reinterpret_cast<const uint4*>(src)[i];
    for (int64_t i = n16 * 16 + t; i < bytes; i += stride) dst[i] = src[i];
}

hipError_t copy_bytes(void* dst, const void* src, size_t bytes, hipStream_t s) {
    if (bytes == 0) return hipSuccess;
    const bool wide = ((reinterpret_cast<uintptr_t>(dst) | reinterpret_cast<uintptr_t>(src)) & 15) == 0;
    const int64_t n16 = wide ? (int64_t)(bytes / 16) : 0;
    int blocks = cdiv64(wide ? (n16 > 0 ? n16 : 1) : (int64_t)bytes, 256);
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(copy_bytes_kernel, dim3(blocks), dim3(256), 0, s, (const unsigned char*)src, (unsigned char*)dst, n16,
                       (int64_t)bytes);
    return hipGetLastError();
}

// --------------------------------------------------------------------------------- max pooling
// One thread per output element (channels fastest, so a wave reads/writes consecutive channels).
template <typename T>
__global__ void maxpool_fwd_kernel(const T* __restrict__ x, T* __restrict__ y, int B, int H, int W, int C,
                                   int Ho, int Wo, int k, int stride, int pad) {
    int64_t total = (int64_t)B * Ho * Wo * C;
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    int c = (int)(i % C);
    int64_t t = i / C;
    int wo = (int)(t % Wo); t /= Wo;
    int ho = (int)(t % Ho);
    int n = (int)(t / Ho);
    float best = -INFINITY;
    for (int r = 0; r < k; ++r)
        for (int s = 0; s < k; ++s) {
            const int hh = ho * stride - pad + r, ww = wo * stride - pad + s;
            if ((unsigned)hh >= (unsigned)H || (unsigned)ww >= (unsigned)W) continue;   // padding never wins
            float v = to_f32(x[(((int64_t)n * H + hh) * W + ww) * C + c]);
            if (v > best) best = v;
        }
    y[i] = from_f32<T>(best);
}

// The same with 8 channels (16 bytes) per thread and access, bf16, C % 8 == 0.
__global__ __launch_bounds__(256) void maxpool_fwd_bf16x8_kernel(const bf16_t* __restrict__ x, bf16_t* __restrict__ y, int B, int H,
                                                                 int W, int C, int Ho, int Wo, int k, int stride, int pad) {
    const int C8 = C >> 3;
    const int64_t total = (int64_t)B * Ho * Wo * C8;
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const int c8 = (int)(i % C8);
    int64_t t = i / C8;
    const int wo = (int)(t % Wo); t /= Wo;
    const int ho = (int)(t % Ho);
    const int n = (int)(t / Ho);
    float best[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) best[e] = -INFINITY;
    for (int r = 0; r < k; ++r)
        for (int q = 0; q < k; ++q) {
            const int hh = ho * stride - pad + r, ww = wo * stride - pad + q;
            if ((unsigned)hh >= (unsigned)H || (unsigned)ww >= (unsigned)W) continue;   // padding never wins
            Pack8 o;
            o.u = *reinterpret_cast<const uint4*>(x + ((((int64_t)n * H + hh) * W + ww) * C8 + c8) * 8);
#pragma unroll
            for (int e = 0; e < 8; ++e) best[e] = fmaxf(best[e], (float)o.h[e]);
        }
    Pack8 out;
#pragma unroll
    for (int e = 0; e < 8; ++e) out.h[e] = (bf16_t)best[e];
    *reinterpret_cast<uint4*>(y + i * 8) = out.u;
}

// Gather form, one thread per INPUT element: sum dy over the windows whose winner (first maximum in
// row-major window order) it is.  Handles overlapping windows and inputs no window covers.
template <typename T>
__global__ void maxpool_bwd_kernel(const T* __restrict__ x, const T* __restrict__ dy, T* __restrict__ dx,
                                   int B, int H, int W, int C, int Ho, int Wo, int k, int stride, int pad,
                                   int relu_mask) {
    int64_t total = (int64_t)B * H * W * C;
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    int c = (int)(i % C);
    int64_t t = i / C;
    int w = (int)(t % W); t /= W;
    int h = (int)(t % H);
    int n = (int)(t / H);
    float xv = to_f32(x[i]);
    float acc = 0.0f;
    if (!(relu_mask && !(xv > 0.0f))) {
        // windows that contain (h, w): ho * stride - pad <= h <= ho * stride - pad + k - 1
        const int hp = h + pad, wp = w + pad;
        int ho_lo = hp - k + 1 > 0 ? (hp - k + 1 + stride - 1) / stride : 0;
        int wo_lo = wp - k + 1 > 0 ? (wp - k + 1 + stride - 1) / stride : 0;
        for (int ho = ho_lo; ho < Ho && ho * stride <= hp; ++ho)
            for (int wo = wo_lo; wo < Wo && wo * stride <= wp; ++wo) {
                bool win = true;
                for (int r = 0; r < k && win; ++r)
                    for (int s = 0; s < k; ++s) {
                        int hh = ho * stride - pad + r, ww = wo * stride - pad + s;
                        if ((unsigned)hh >= (unsigned)H || (unsigned)ww >= (unsigned)W) continue;
                        float v = to_f32(x[(((int64_t)n * H + hh) * W + ww) * C + c]);
                        bool before = (hh < h) || (hh == h && ww < w);
                        if (v > xv || (before && v == xv)) { win = false; break; }
                    }
                if (win) acc += to_f32(dy[(((int64_t)n * Ho + ho) * Wo + wo) * C + c]);
            }
    }
    dx[i] = from_f32<T>(acc);
}

// The same gather with 8 channels (16 bytes) per thread and access, bf16, C % 8 == 0: any window, stride, padding.
__global__ __launch_bounds__(256) void maxpool_bwd_bf16x8_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ dy,
                                                                 bf16_t* __restrict__ dx, int B, int H, int W, int C, int Ho,
                                                                 int Wo, int k, int stride, int pad, int relu_mask) {
    const int C8 = C >> 3;
    const int64_t total = (int64_t)B * H * W * C8;
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const int c8 = (int)(i % C8);
    int64_t t = i / C8;
    const int w = (int)(t % W); t /= W;
    const int h = (int)(t % H);
    const int n = (int)(t / H);
    Pack8 me, out;
    me.u = *reinterpret_cast<const uint4*>(x + i * 8);
    float xv[8], acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        xv[e] = (float)me.h[e];
        acc[e] = 0.0f;
    }
    const int hp = h + pad, wp = w + pad;
    const int ho_lo = hp - k + 1 > 0 ? (hp - k + 1 + stride - 1) / stride : 0;
    const int wo_lo = wp - k + 1 > 0 ? (wp - k + 1 + stride - 1) / stride : 0;
    for (int ho = ho_lo; ho < Ho && ho * stride <= hp; ++ho)
        for (int wo = wo_lo; wo < Wo && wo * stride <= wp; ++wo) {
            bool win[8] = {true, true, true, true, true, true, true, true};
            for (int r = 0; r < k; ++r)
                for (int s = 0; s < k; ++s) {
                    const int hh = ho * stride - pad + r, ww = wo * stride - pad + s;
                    if ((unsigned)hh >= (unsigned)H || (unsigned)ww >= (unsigned)W) continue;
                    if (hh == h && ww == w) continue;
                    Pack8 o;
                    o.u = *reinterpret_cast<const uint4*>(x + ((((int64_t)n * H + hh) * W + ww) * C8 + c8) * 8);
                    const bool before = (hh < h) || (hh == h && ww < w);
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const float v = (float)o.h[e];
                        if (v > xv[e] || (before && v == xv[e])) win[e] = false;
                    }
                }
            Pack8 g;
            g.u = *reinterpret_cast<const uint4*>(dy + ((((int64_t)n * Ho + ho) * Wo + wo) * C8 + c8) * 8);
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (win[e]) acc[e] += (float)g.h[e];
        }
#pragma unroll
    for (int e = 0; e < 8; ++e) out.h[e] = (bf16_t)((relu_mask && !(xv[e] > 0.0f)) ? 0.0f : acc[e]);
    *reinterpret_cast<uint4*>(dx + i * 8) = out.u;
}

// Large feature maps: a workgroup owns an 8 x 16 tile of input positions of one image and up to 64 channels.
//   1. Every input position that shares a window with the tile (at most k-1 more rows and columns on each side) is
//      copied into LDS, 128 bytes per position: x is read from memory once (plus the halo).
//   2. Every window that touches the tile is scanned ONCE (per 8 channels) in row-major order for its first maximum;
//      the winner's place in the window (r * k + q) is kept in LDS, one byte per channel.
//   3. Every position of the tile looks up the (at most ceil(k / stride)^2) windows that contain it and adds dy where the
//      stored place is its own.
// Scanning a window once instead of once per element it contains is what makes the difference: the per-element gather
// above spends 4 k^2 comparisons per element and channel and is bound by the vector ALUs on large maps.
constexpr int kPoolTH = 8, kPoolTW = 16;
__global__ __launch_bounds__(256) void maxpool_bwd_tiled_bf16_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ dy,
                                                                     bf16_t* __restrict__ dx, int H, int W, int C, int Ho,
                                                                     int Wo, int k, int stride, int pad, int relu_mask,
                                                                     int groups, int patch_bytes) {
    extern __shared__ __attribute__((aligned(16))) unsigned char pool_smem[];
    uint4* const patch = reinterpret_cast<uint4*>(pool_smem);                 // [rows][cols][8 chunks of 8 channels]
    uint2* const place = reinterpret_cast<uint2*>(pool_smem + patch_bytes);   // [windows][8 chunks]: 8 bytes = 8 channels
    const int C8 = C >> 3;
    const int n = blockIdx.z / groups, c8base = (blockIdx.z % groups) * 8;
    const int h0 = blockIdx.y * kPoolTH, w0 = blockIdx.x * kPoolTW;
    const int h1 = min(h0 + kPoolTH, H) - 1, w1 = min(w0 + kPoolTW, W) - 1;   // last position of the tile
    // windows that contain a position of the tile, and the input positions they cover
    const int ho_lo = h0 + pad - k + 1 > 0 ? (h0 + pad - k + 1 + stride - 1) / stride : 0;
    const int wo_lo = w0 + pad - k + 1 > 0 ? (w0 + pad - k + 1 + stride - 1) / stride : 0;
    const int ho_hi = min(Ho - 1, (h1 + pad) / stride), wo_hi = min(Wo - 1, (w1 + pad) / stride);
    const int nwh = max(0, ho_hi - ho_lo + 1), nww = max(0, wo_hi - wo_lo + 1);
    const int ph0 = max(0, ho_lo * stride - pad), pw0 = max(0, wo_lo * stride - pad);
    const int ph1 = min(H - 1, ho_hi * stride - pad + k - 1), pw1 = min(W - 1, wo_hi * stride - pad + k - 1);
    const int nph = max(0, ph1 - ph0 + 1), npw = max(0, pw1 - pw0 + 1);
    const bf16_t* xn = x + (int64_t)n * H * W * C;
    for (int idx = threadIdx.x; idx < nph * npw * 8; idx += 256) {
        const int pos = idx >> 3, ch = idx & 7;
        const int pr = pos / npw, pc = pos - pr * npw;
        if (c8base + ch < C8)
            patch[idx] = *reinterpret_cast<const uint4*>(xn + (((int64_t)(ph0 + pr) * W + pw0 + pc) * C8 + c8base + ch) * 8);
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < nwh * nww * 8; idx += 256) {
        const int wi = idx >> 3, ch = idx & 7;
        if (c8base + ch >= C8) continue;
        const int wr = wi / nww, wc = wi - wr * nww;
        const int hb = (ho_lo + wr) * stride - pad, wb = (wo_lo + wc) * stride - pad;
        float best[8];
        unsigned where[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            best[e] = -INFINITY;
            where[e] = 255u;
        }
        for (int r = 0; r < k; ++r)
            for (int q = 0; q < k; ++q) {
                const int hh = hb + r, ww = wb + q;
                if ((unsigned)hh >= (unsigned)H || (unsigned)ww >= (unsigned)W) continue;
                Pack8 o;
                o.u = patch[((hh - ph0) * npw + (ww - pw0)) * 8 + ch];
                const unsigned me = (unsigned)(r * k + q);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float v = (float)o.h[e];
                    if (v > best[e]) {   // strict: the first maximum in row-major order stays
                        best[e] = v;
                        where[e] = me;
                    }
                }
            }
        uint2 pk;
        pk.x = where[0] | (where[1] << 8) | (where[2] << 16) | (where[3] << 24);
        pk.y = where[4] | (where[5] << 8) | (where[6] << 16) | (where[7] << 24);
        place[idx] = pk;
    }
    __syncthreads();
    for (int it = threadIdx.x; it < kPoolTH * kPoolTW * 8; it += 256) {
        const int pos = it >> 3, ch = it & 7;
        const int h = h0 + pos / kPoolTW, w = w0 + pos % kPoolTW, c8 = c8base + ch;
        if (h >= H || w >= W || c8 >= C8) continue;
        const int64_t i = (((int64_t)n * H + h) * W + w) * C8 + c8;
        float acc[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = 0.0f;
        const int hp = h + pad, wp = w + pad;
        const int a_lo = hp - k + 1 > 0 ? (hp - k + 1 + stride - 1) / stride : 0;
        const int b_lo = wp - k + 1 > 0 ? (wp - k + 1 + stride - 1) / stride : 0;
        for (int ho = a_lo; ho < Ho && ho * stride <= hp; ++ho)
            for (int wo = b_lo; wo < Wo && wo * stride <= wp; ++wo) {
                const unsigned me = (unsigned)((hp - ho * stride) * k + (wp - wo * stride));
                const uint2 pk = place[((ho - ho_lo) * nww + (wo - wo_lo)) * 8 + ch];
                Pack8 g;
                g.u = *reinterpret_cast<const uint4*>(dy + ((((int64_t)n * Ho + ho) * Wo + wo) * C8 + c8) * 8);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const unsigned wv = ((e < 4 ? pk.x : pk.y) >> (8 * (e & 3))) & 255u;
                    if (wv == me) acc[e] += (float)g.h[e];
                }
            }
        Pack8 out;
        if (relu_mask) {
            Pack8 mine;
            mine.u = *reinterpret_cast<const uint4*>(x + i * 8);
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (!((float)mine.h[e] > 0.0f)) acc[e] = 0.0f;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) out.h[e] = (bf16_t)acc[e];
        *reinterpret_cast<uint4*>(dx + i * 8) = out.u;
    }
}

// 2x2 windows with stride 2 on even H, W and C % 8 == 0 (bf16): one thread per window and 8 channels,
// 16-byte loads of the 4 inputs and of dy, 16-byte stores of the 4 gradients.
__global__ __launch_bounds__(256) void maxpool2x2_bwd_bf16_kernel(const bf16_t* __restrict__ x,
                                                                  const bf16_t* __restrict__ dy,
                                                                  bf16_t* __restrict__ dx, int B, int H, int W,
                                                                  int C, int relu_mask) {
    const int Ho = H >> 1, Wo = W >> 1, C8 = C >> 3;
    int64_t total = (int64_t)B * Ho * Wo * C8;
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    int c8 = (int)(i % C8);
    int64_t t = i / C8;
    int wo = (int)(t % Wo); t /= Wo;
    int ho = (int)(t % Ho);
    int n = (int)(t / Ho);
    Pack8 in[4], out[4], g;
    g.u = *reinterpret_cast<const uint4*>(dy + i * 8);
    int64_t base = (((int64_t)n * H + 2 * ho) * W + 2 * wo) * C + c8 * 8;
    const int64_t off[4] = {0, C, (int64_t)W * C, (int64_t)W * C + C};
#pragma unroll
    for (int q = 0; q < 4; ++q) in[q].u = *reinterpret_cast<const uint4*>(x + base + off[q]);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        float v[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) v[q] = (float)in[q].h[e];
        int best = 0;
#pragma unroll
        for (int q = 1; q < 4; ++q)
            if (v[q] > v[best]) best = q;
        const bool pass = !(relu_mask && !(v[best] > 0.0f));
#pragma unroll
        for (int q = 0; q < 4; ++q) out[q].h[e] = (q == best && pass) ? g.h[e] : (bf16_t)0.0f;
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) *reinterpret_cast<uint4*>(dx + base + off[q]) = out[q].u;
}

hipError_t maxpool_forward(int dtype, const void* x, void* y, int B, int H, int W, int C, int k, int stride, int pad,
                           hipStream_t s) {
    int Ho = (H + 2 * pad - k) / stride + 1, Wo = (W + 2 * pad - k) / stride + 1;
    int64_t total = (int64_t)B * Ho * Wo * C;
    if (total <= 0) return hipSuccess;
    if (dtype == kBF16 && C % 8 == 0 && ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(y)) & 15) == 0) {
        hipLaunchKernelGGL(maxpool_fwd_bf16x8_kernel, dim3(cdiv64(total / 8, 256)), dim3(256), 0, s, (const bf16_t*)x, (bf16_t*)y,
                           B, H, W, C, Ho, Wo, k, stride, pad);
        return hipGetLastError();
    }
    dim3 grid(cdiv64(total, 256));
    if (dtype == kBF16)
        hipLaunchKernelGGL(maxpool_fwd_kernel<bf16_t>, grid, dim3(256), 0, s, (const bf16_t*)x, (bf16_t*)y, B, H,
                           W, C, Ho, Wo, k, stride, pad);
    else
        hipLaunchKernelGGL(maxpool_fwd_kernel<float>, grid, dim3(256), 0, s, (const float*)x, (float*)y, B, H, W,
                           C, Ho, Wo, k, stride, pad);
    return hipGetLastError();
}

hipError_t maxpool_backward(int dtype, const void* x, const void* dy, void* dx, int B, int H, int W, int C,
                            int k, int stride, int pad, int relu_mask, hipStream_t s) {
    int Ho = (H + 2 * pad - k) / stride + 1, Wo = (W + 2 * pad - k) / stride + 1;
    int64_t total = (int64_t)B * H * W * C;
    if (total <= 0) return hipSuccess;
    if (dtype == kBF16 && k == 2 && stride == 2 && pad == 0 && H % 2 == 0 && W % 2 == 0 && C % 8 == 0 &&
        (reinterpret_cast<uintptr_t>(x) & 15) == 0 && (reinterpret_cast<uintptr_t>(dy) & 15) == 0 &&
        (reinterpret_cast<uintptr_t>(dx) & 15) == 0) {
        int64_t windows = (int64_t)B * Ho * Wo * (C / 8);
        hipLaunchKernelGGL(maxpool2x2_bwd_bf16_kernel, dim3(cdiv64(windows, 256)), dim3(256), 0, s, (const bf16_t*)x,
                           (const bf16_t*)dy, (bf16_t*)dx, B, H, W, C, relu_mask);
        return hipGetLastError();
    }
    if (dtype == kBF16 && C % 8 == 0 && (reinterpret_cast<uintptr_t>(x) & 15) == 0 && (reinterpret_cast<uintptr_t>(dy) & 15) == 0 &&
        (reinterpret_cast<uintptr_t>(dx) & 15) == 0) {
        // large maps: the LDS-tiled form (its patch of (8 + 2(k-1)) x (16 + 2(k-1)) positions x 128 bytes and the
        // winners of at most (8 + k-1) x (16 + k-1) windows x 64 bytes must fit; a window has at most 255 places)
        const int groups = (C / 8 + 7) / 8;
        const int64_t patch_bytes = (int64_t)(kPoolTH + 2 * (k - 1)) * (kPoolTW + 2 * (k - 1)) * 128;
        const int64_t lds = patch_bytes + (int64_t)(kPoolTH + k - 1) * (kPoolTW + k - 1) * 64;
        const int64_t blocks_z = (int64_t)B * groups;
        if (H >= 2 * kPoolTH && W >= 2 * kPoolTW && lds <= 64 * 1024 && blocks_z <= 65535 && k * k <= 255) {
            dim3 grid((W + kPoolTW - 1) / kPoolTW, (H + kPoolTH - 1) / kPoolTH, (unsigned)blocks_z);
            hipLaunchKernelGGL(maxpool_bwd_tiled_bf16_kernel, grid, dim3(256), (unsigned)lds, s, (const bf16_t*)x, (const bf16_t*)dy,
                               (bf16_t*)dx, H, W, C, Ho, Wo, k, stride, pad, relu_mask, groups, (int)patch_bytes);
            return hipGetLastError();
        }
        hipLaunchKernelGGL(maxpool_bwd_bf16x8_kernel, dim3(cdiv64(total / 8, 256)), dim3(256), 0, s, (const bf16_t*)x,
                           (const bf16_t*)dy, (bf16_t*)dx, B, H, W, C, Ho, Wo, k, stride, pad, relu_mask);
        return hipGetLastError();
    }
    dim3 grid(cdiv64(total, 256));
    if (dtype == kBF16)
        hipLaunchKernelGGL(maxpool_bwd_kernel<bf16_t>, grid, dim3(256), 0, s, (const bf16_t*)x,
                           (const bf16_t*)dy, (bf16_t*)dx, B, H, W, C, Ho, Wo, k, stride, pad, relu_mask);
    else
        hipLaunchKernelGGL(maxpool_bwd_kernel<float>, grid, dim3(256), 0, s, (const float*)x, (const float*)dy,
                           (float*)dx, B, H, W, C, Ho, Wo, k, stride, pad, relu_mask);
    return hipGetLastError();
}

}  // namespace tmps
