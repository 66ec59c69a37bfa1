// Bandwidth-bound kernels of the residual-network stages: per-channel affine layer (a batch-normalisation
// layer with its statistics folded away), residual join, global average pooling.  Channels-last tensors
// [rows, C]; the bf16 kernels move 8 channels (16 bytes) per lane and access when C is a multiple of 8.
#include "gemm.hip.h"
#include "kernels.h"
#include "launch.h"

namespace tmps {

static inline int cdiv_res(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }
static inline bool al16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

// ---------------------------------------------------------------------------------------- affine
template <typename T>
__global__ void affine_fwd_kernel(const T* __restrict__ x, const float* __restrict__ gain, const float* __restrict__ shift,
                                  T* __restrict__ y, int64_t n, int C, int relu) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) {
        const int c = (int)(i % C);
        float v = to_f32(x[i]) * gain[c] + shift[c];
        if (relu) v = v > 0.0f ? v : 0.0f;
        y[i] = from_f32<T>(v);
    }
}

__global__ __launch_bounds__(256) void affine_fwd_bf16x8_kernel(const bf16_t* __restrict__ x, const float* __restrict__ gain,
                                                                const float* __restrict__ shift, bf16_t* __restrict__ y,
                                                                int64_t n8, int C8, int relu) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n8; i += stride) {
        const int c = (int)(i % C8) * 8;
        Pack8 p, o;
        p.u = reinterpret_cast<const uint4*>(x)[i];
        float g[8], b[8];
        load8(gain + c, g);
        load8(shift + c, b);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float v = (float)p.h[e] * g[e] + b[e];
            if (relu) v = v > 0.0f ? v : 0.0f;
            o.h[e] = (bf16_t)v;
        }
        reinterpret_cast<uint4*>(y)[i] = o.u;
    }
}

// dx = gain * dy; partial sums of dgain[c] = sum_r dy[r, c] x[r, c] and dshift[c] = sum_r dy[r, c] over a slab
// of rows: part[slab][0][C], part[slab][1][C].  Block = 64 channel lanes x 4 row lanes.
template <typename T>
__global__ __launch_bounds__(256) void affine_bwd_kernel(const T* __restrict__ dy, const T* __restrict__ x,
                                                         const float* __restrict__ gain, T* __restrict__ dx,
                                                         float* __restrict__ part, int64_t rows, int C, int rows_per_slab) {
    __shared__ float sg[4][64], sb[4][64];
    const int cl = threadIdx.x & 63, rl = threadIdx.x >> 6;
    const int col = blockIdx.x * 64 + cl;
    const int64_t r0 = (int64_t)blockIdx.y * rows_per_slab;
    const int64_t r1 = r0 + rows_per_slab < rows ? r0 + rows_per_slab : rows;
    float dg = 0.0f, db = 0.0f;
    if (col < C) {
        const float g = gain[col];
        for (int64_t r = r0 + rl; r < r1; r += 4) {
            const float d = to_f32(dy[r * C + col]);
            dg += d * to_f32(x[r * C + col]);
            db += d;
            if (dx) dx[r * C + col] = from_f32<T>(d * g);
        }
    }
    sg[rl][cl] = dg;
    sb[rl][cl] = db;
    __syncthreads();
    if (rl == 0 && col < C) {
        part[((int64_t)blockIdx.y * 2 + 0) * C + col] = (sg[0][cl] + sg[1][cl]) + (sg[2][cl] + sg[3][cl]);
        part[((int64_t)blockIdx.y * 2 + 1) * C + col] = (sb[0][cl] + sb[1][cl]) + (sb[2][cl] + sb[3][cl]);
    }
}

// The same with 8 channels per lane: block = 8 channel groups (64 channels) x 32 row lanes.
__global__ __launch_bounds__(256) void affine_bwd_bf16x8_kernel(const bf16_t* __restrict__ dy, const bf16_t* __restrict__ x,
                                                                const float* __restrict__ gain, bf16_t* __restrict__ dx,
                                                                float* __restrict__ part, int64_t rows, int C,
                                                                int rows_per_slab) {
    __shared__ float sg[32][65], sb[32][65];
    const int cg = threadIdx.x & 7, rl = threadIdx.x >> 3;
    const int col = blockIdx.x * 64 + cg * 8;
    const int64_t r0 = (int64_t)blockIdx.y * rows_per_slab;
    const int64_t r1 = r0 + rows_per_slab < rows ? r0 + rows_per_slab : rows;
    float dg[8] = {0, 0, 0, 0, 0, 0, 0, 0}, db[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (col < C) {
        float g[8];
        load8(gain + col, g);
        // several rows' loads in flight per thread: the loop is latency-bound otherwise
#pragma unroll 4
        for (int64_t r = r0 + rl; r < r1; r += 32) {
            Pack8 d, xv, o;
            d.u = *reinterpret_cast<const uint4*>(dy + r * C + col);
            xv.u = *reinterpret_cast<const uint4*>(x + r * C + col);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float dv = (float)d.h[e];
                dg[e] += dv * (float)xv.h[e];
                db[e] += dv;
                o.h[e] = (bf16_t)(dv * g[e]);
            }
            if (dx) *reinterpret_cast<uint4*>(dx + r * C + col) = o.u;
        }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        sg[rl][cg * 8 + e] = dg[e];
        sb[rl][cg * 8 + e] = db[e];
    }
    __syncthreads();
    if (threadIdx.x < 64 && blockIdx.x * 64 + threadIdx.x < C) {
        float a = 0.0f, b = 0.0f;
#pragma unroll 8
        for (int r = 0; r < 32; ++r) {
            a += sg[r][threadIdx.x];
            b += sb[r][threadIdx.x];
        }
        part[((int64_t)blockIdx.y * 2 + 0) * C + blockIdx.x * 64 + threadIdx.x] = a;
        part[((int64_t)blockIdx.y * 2 + 1) * C + blockIdx.x * 64 + threadIdx.x] = b;
    }
}

// out[i] = sum over the slabs of part[slab][i]: 64 outputs per workgroup, sixteen lanes of slabs each, combined through LDS
__global__ __launch_bounds__(1024) void affine_slab_sum_kernel(const float* __restrict__ part, float* __restrict__ out, int count,
                                                               int slabs) {
    __shared__ float sp[16][64];
    const int cl = threadIdx.x & 63, sl = threadIdx.x >> 6;
    const int i = blockIdx.x * 64 + cl;
    float a = 0.0f;
    if (i < count) {
        // eight loads in flight per lane, added in slab order
        const float* p = part + (int64_t)sl * count + i;
        const int64_t step = (int64_t)16 * count;
        int z = sl;
        for (; z + 7 * 16 < slabs; z += 8 * 16) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = p[u * step];
#pragma unroll
            for (int u = 0; u < 8; ++u) a += v[u];
            p += 8 * step;
        }
        for (; z < slabs; z += 16) {
            a += *p;
            p += step;
        }
    }
    sp[sl][cl] = a;
    __syncthreads();
    if (sl == 0 && i < count) {
        float t = 0.0f;
#pragma unroll
        for (int k = 0; k < 16; ++k) t += sp[k][cl];
        out[i] = t;
    }
}

static int affine_slab_rows(int64_t rows) {
    // a few thousand workgroups at most, 64 rows at least (swept 32..1024 on the ResNet-50 workload)
    int64_t r = (rows + 2047) / 2048;
    if (r < 64) r = 64;
    return (int)((r + 31) / 32 * 32);
}

size_t affine_workspace_elems(int64_t rows, int C) {
    return (size_t)cdiv_res(rows, affine_slab_rows(rows)) * 2 * (size_t)C;
}

hipError_t affine_forward(int dtype, const void* x, const float* gain, const float* shift, void* y, int64_t rows, int C,
                          int relu, hipStream_t s) {
    const int64_t n = rows * C;
    if (n <= 0) return hipSuccess;
    if (dtype == kBF16 && C % 8 == 0 && al16(x) && al16(y) && al16(gain) && al16(shift)) {
        int blocks = cdiv_res(n / 8, 256);
        if (blocks > 8192) blocks = 8192;
        return launch_timed(kcAffine, affine_fwd_bf16x8_kernel, dim3(blocks), dim3(256), 0, s, (const bf16_t*)x, gain, shift,
                            (bf16_t*)y, n / 8, C / 8, relu);
    }
    int blocks = cdiv_res(n, 256);
    if (blocks > 8192) blocks = 8192;
    if (dtype == kBF16)
        return launch_timed(kcAffine, affine_fwd_kernel<bf16_t>, dim3(blocks), dim3(256), 0, s, (const bf16_t*)x, gain, shift,
                            (bf16_t*)y, n, C, relu);
    return launch_timed(kcAffine, affine_fwd_kernel<float>, dim3(blocks), dim3(256), 0, s, (const float*)x, gain, shift,
                        (float*)y, n, C, relu);
}

hipError_t affine_backward(int dtype, const void* dy, const void* x, const float* gain, void* dx, float* dgain_dshift,
                           float* ws, int64_t rows, int C, hipStream_t s) {
    if (rows <= 0 || C <= 0) return hipSuccess;
    const int slab = affine_slab_rows(rows);
    const int slabs = cdiv_res(rows, slab);
    dim3 grid(cdiv_res(C, 64), slabs);
    hipError_t e;
    if (dtype == kBF16 && C % 8 == 0 && al16(dy) && al16(x) && al16(gain) && (!dx || al16(dx)))
        e = launch_timed(kcAffine, affine_bwd_bf16x8_kernel, grid, dim3(256), 0, s, (const bf16_t*)dy, (const bf16_t*)x, gain,
                         (bf16_t*)dx, ws, rows, C, slab);
    else if (dtype == kBF16)
        e = launch_timed(kcAffine, affine_bwd_kernel<bf16_t>, grid, dim3(256), 0, s, (const bf16_t*)dy, (const bf16_t*)x, gain,
                         (bf16_t*)dx, ws, rows, C, slab);
    else
        e = launch_timed(kcAffine, affine_bwd_kernel<float>, grid, dim3(256), 0, s, (const float*)dy, (const float*)x, gain,
                         (float*)dx, ws, rows, C, slab);
    if (e != hipSuccess) return e;
    return launch_timed(kcAffine, affine_slab_sum_kernel, dim3(cdiv_res(2 * C, 64)), dim3(1024), 0, s, (const float*)ws,
                        dgain_dshift, 2 * C, slabs);
}

// ---------------------------------------------------------------------------------- residual join
template <typename T>
__global__ void resadd_kernel(const T* __restrict__ a, const T* __restrict__ b, T* __restrict__ y, int64_t n, int relu) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) {
        float v = to_f32(a[i]) + to_f32(b[i]);
        if (relu) v = v > 0.0f ? v : 0.0f;
        y[i] = from_f32<T>(v);
    }
}

__global__ __launch_bounds__(256) void resadd_bf16x8_kernel(const bf16_t* __restrict__ a, const bf16_t* __restrict__ b,
                                                            bf16_t* __restrict__ y, int64_t n8, int relu) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n8; i += stride) {
        Pack8 p, q, o;
        p.u = reinterpret_cast<const uint4*>(a)[i];
        q.u = reinterpret_cast<const uint4*>(b)[i];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float v = (float)p.h[e] + (float)q.h[e];
            if (relu) v = v > 0.0f ? v : 0.0f;
            o.h[e] = (bf16_t)v;
        }
        reinterpret_cast<uint4*>(y)[i] = o.u;
    }
}

hipError_t resadd_forward(int dtype, const void* a, const void* b, void* y, int64_t n, int relu, hipStream_t s) {
    if (n <= 0) return hipSuccess;
    if (dtype == kBF16 && n % 8 == 0 && al16(a) && al16(b) && al16(y)) {
        int blocks = cdiv_res(n / 8, 256);
        if (blocks > 8192) blocks = 8192;
        return launch_timed(kcResAdd, resadd_bf16x8_kernel, dim3(blocks), dim3(256), 0, s, (const bf16_t*)a, (const bf16_t*)b,
                            (bf16_t*)y, n / 8, relu);
    }
    int blocks = cdiv_res(n, 256);
    if (blocks > 8192) blocks = 8192;
    if (dtype == kBF16)
        return launch_timed(kcResAdd, resadd_kernel<bf16_t>, dim3(blocks), dim3(256), 0, s, (const bf16_t*)a, (const bf16_t*)b,
                            (bf16_t*)y, n, relu);
    return launch_timed(kcResAdd, resadd_kernel<float>, dim3(blocks), dim3(256), 0, s, (const float*)a, (const float*)b,
                        (float*)y, n, relu);
}

// ----------------------------------------------------------------------------- global average pooling
// y[b, c] = mean over the HW positions of x[b, :, c]; one thread per (b, c), consecutive c in a wave.
template <typename T>
__global__ void avgpool_fwd_kernel(const T* __restrict__ x, T* __restrict__ y, int B, int HW, int C) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)B * C) return;
    const int c = (int)(i % C);
    const int64_t b = i / C;
    float a = 0.0f;
    for (int p = 0; p < HW; ++p) a += to_f32(x[(b * HW + p) * C + c]);
    y[i] = from_f32<T>(a / (float)HW);
}

// dx[b, p, c] = dy[b, c] / HW, zeroed where the stored input is <= 0 when relu_mask (the layer below ends in a ReLU)
template <typename T>
__global__ void avgpool_bwd_kernel(const T* __restrict__ dy, const T* __restrict__ x, T* __restrict__ dx, int64_t n, int HW,
                                   int C, int relu_mask) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const float inv = 1.0f / (float)HW;
    for (; i < n; i += stride) {
        const int c = (int)(i % C);
        const int64_t b = i / ((int64_t)HW * C);
        float v = to_f32(dy[b * C + c]) * inv;
        if (relu_mask && !(to_f32(x[i]) > 0.0f)) v = 0.0f;
        dx[i] = from_f32<T>(v);
    }
}

hipError_t avgpool_forward(int dtype, const void* x, void* y, int B, int HW, int C, hipStream_t s) {
    const int64_t n = (int64_t)B * C;
    if (n <= 0) return hipSuccess;
    if (dtype == kBF16)
        return launch_timed(kcPoolFwd, avgpool_fwd_kernel<bf16_t>, dim3(cdiv_res(n, 256)), dim3(256), 0, s, (const bf16_t*)x,
                            (bf16_t*)y, B, HW, C);
    return launch_timed(kcPoolFwd, avgpool_fwd_kernel<float>, dim3(cdiv_res(n, 256)), dim3(256), 0, s, (const float*)x,
                        (float*)y, B, HW, C);
}

hipError_t avgpool_backward(int dtype, const void* dy, const void* x, void* dx, int B, int HW, int C, int relu_mask,
                            hipStream_t s) {
    const int64_t n = (int64_t)B * HW * C;
    if (n <= 0) return hipSuccess;
    int blocks = cdiv_res(n, 256);
    if (blocks > 8192) blocks = 8192;
    if (dtype == kBF16)
        return launch_timed(kcPoolBwd, avgpool_bwd_kernel<bf16_t>, dim3(blocks), dim3(256), 0, s, (const bf16_t*)dy,
                            (const bf16_t*)x, (bf16_t*)dx, n, HW, C, relu_mask);
    return launch_timed(kcPoolBwd, avgpool_bwd_kernel<float>, dim3(blocks), dim3(256), 0, s, (const float*)dy, (const float*)x,
                        (float*)dx, n, HW, C, relu_mask);
}

}  // namespace tmps
