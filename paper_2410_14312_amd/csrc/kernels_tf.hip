// Transformer-stage kernels for gfx950: layer normalisation, token + position embedding, causal
// multi-head attention (forward and the three gradient kernels).
//
// Attention has two implementations.  The MFMA path (bf16, 64 features per head) is a flash-style
// kernel: a wave owns 32 query rows (or 32 key rows in the key/value-gradient kernel), streams blocks
// of 64 keys (queries) through LDS and keeps running softmax statistics, so the S x S score matrix
// never exists in memory.  Products are arranged so that the softmax reduction runs over a lane's own
// registers: scores are computed TRANSPOSED (keys along the accumulator registers, queries along the
// lanes), and the probabilities leave the accumulators straight into the B operand of the next MFMA
// with no shuffle.  Operands that the next product needs transposed (V^T, K^T, Q^T, dO^T) are read
// from their row-major LDS tile with the transpose read of gfx950.
// The generic path (any head size, fp32 or bf16) is a plain one-row-per-wave kernel for the fp32
// configuration and odd shapes.
#include <type_traits>
#include <cstdlib>
#include "gemm2.hip.h"
#include "kernels.h"
#include "launch.h"

namespace tmps {

static inline int cdiv_tf(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }

__device__ __forceinline__ float wsum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wmax(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

__global__ void zero_f32_kernel(float* __restrict__ p, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = 0.0f;
}

// ------------------------------------------------------------------------------ layer normalisation
// One wave per row.  The row is read three times (mean, variance, output); it stays in cache.
template <typename T>
__global__ __launch_bounds__(256) void layernorm_fwd_kernel(const T* __restrict__ x, const float* __restrict__ gamma,
                                                            const float* __restrict__ beta, T* __restrict__ y,
                                                            float* __restrict__ stats, int64_t rows, int D, float eps) {
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const T* xr = x + row * D;
    float s = 0.0f;
    for (int i = lane; i < D; i += 64) s += to_f32(xr[i]);
    const float mean = wsum(s) / (float)D;
    float v = 0.0f;
    for (int i = lane; i < D; i += 64) {
        const float d = to_f32(xr[i]) - mean;
        v += d * d;
    }
    const float rstd = 1.0f / sqrtf(wsum(v) / (float)D + eps);
    T* yr = y + row * D;
    for (int i = lane; i < D; i += 64) yr[i] = from_f32<T>((to_f32(xr[i]) - mean) * rstd * gamma[i] + beta[i]);
    if (lane == 0) {
        stats[2 * row] = mean;
        stats[2 * row + 1] = rstd;
    }
}

// The same with 8 bf16 per lane and access (D % 8 == 0, 16-byte aligned rows).
__global__ __launch_bounds__(256) void layernorm_fwd_bf16x8_kernel(const bf16_t* __restrict__ x,
                                                                   const float* __restrict__ gamma,
                                                                   const float* __restrict__ beta, bf16_t* __restrict__ y,
                                                                   float* __restrict__ stats, int64_t rows, int D,
                                                                   float eps) {
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const bf16_t* xr = x + row * D;
    const int nch = D >> 3;
    float s = 0.0f;
    for (int c = lane; c < nch; c += 64) {
        Pack8 p;
        p.u = *reinterpret_cast<const uint4*>(xr + c * 8);
#pragma unroll
        for (int e = 0; e < 8; ++e) s += (float)p.h[e];
    }
    const float mean = wsum(s) / (float)D;
    float v = 0.0f;
    for (int c = lane; c < nch; c += 64) {
        Pack8 p;
        p.u = *reinterpret_cast<const uint4*>(xr + c * 8);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float d = (float)p.h[e] - mean;
            v += d * d;
        }
    }
    const float rstd = 1.0f / sqrtf(wsum(v) / (float)D + eps);
    bf16_t* yr = y + row * D;
    for (int c = lane; c < nch; c += 64) {
        Pack8 p, o;
        p.u = *reinterpret_cast<const uint4*>(xr + c * 8);
        const float4 g0 = *reinterpret_cast<const float4*>(gamma + c * 8), g1 = *reinterpret_cast<const float4*>(gamma + c * 8 + 4);
        const float4 b0 = *reinterpret_cast<const float4*>(beta + c * 8), b1 = *reinterpret_cast<const float4*>(beta + c * 8 + 4);
        const float g[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
        const float b[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
#pragma unroll
        for (int e = 0; e < 8; ++e) o.h[e] = (bf16_t)(((float)p.h[e] - mean) * rstd * g[e] + b[e]);
        *reinterpret_cast<uint4*>(yr + c * 8) = o.u;
    }
    if (lane == 0) {
        stats[2 * row] = mean;
        stats[2 * row + 1] = rstd;
    }
}

// dx = rstd * (g - mean(g) - xhat * mean(g * xhat)) [+ add],  g = dy * gamma, xhat = (x - mean) * rstd with the
// statistics of the forward pass.  `add` is the gradient of a residual connection that joins this layer's input.
template <typename T>
__global__ __launch_bounds__(256) void layernorm_bwd_kernel(const T* __restrict__ dy, const T* __restrict__ x,
                                                            const float* __restrict__ stats,
                                                            const float* __restrict__ gamma, const T* __restrict__ add,
                                                            T* __restrict__ dx, int64_t rows, int D) {
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const T* xr = x + row * D;
    const T* gr = dy + row * D;
    const float mean = stats[2 * row], rstd = stats[2 * row + 1];
    float s1 = 0.0f, s2 = 0.0f;
    for (int i = lane; i < D; i += 64) {
        const float g = to_f32(gr[i]) * gamma[i];
        s1 += g;
        s2 += g * (to_f32(xr[i]) - mean) * rstd;
    }
    const float m1 = wsum(s1) / (float)D, m2 = wsum(s2) / (float)D;
    T* dr = dx + row * D;
    for (int i = lane; i < D; i += 64) {
        const float g = to_f32(gr[i]) * gamma[i];
        const float xh = (to_f32(xr[i]) - mean) * rstd;
        float v = rstd * (g - m1 - xh * m2);
        if (add) v += to_f32(add[row * D + i]);
        dr[i] = from_f32<T>(v);
    }
}

// Gain / shift gradients: block = 64 columns x 4 row lanes over one slab of rows; partial sums
// part[slab][0][D] (gain) and part[slab][1][D] (shift).
template <typename T>
__global__ __launch_bounds__(256) void layernorm_pgrad_kernel(const T* __restrict__ dy, const T* __restrict__ x,
                                                              const float* __restrict__ stats, float* __restrict__ part,
                                                              int64_t rows, int D, int rows_per_slab) {
    __shared__ float sg[4][64], sb[4][64];
    const int cl = threadIdx.x & 63, rl = threadIdx.x >> 6;
    const int col = blockIdx.x * 64 + cl;
    const int64_t r0 = (int64_t)blockIdx.y * rows_per_slab;
    const int64_t r1 = r0 + rows_per_slab < rows ? r0 + rows_per_slab : rows;
    float dg = 0.0f, db = 0.0f;
    if (col < D)
        for (int64_t r = r0 + rl; r < r1; r += 4) {
            const float d = to_f32(dy[r * D + col]);
            dg += d * (to_f32(x[r * D + col]) - stats[2 * r]) * stats[2 * r + 1];
            db += d;
        }
    sg[rl][cl] = dg;
    sb[rl][cl] = db;
    __syncthreads();
    if (rl == 0 && col < D) {
        part[((int64_t)blockIdx.y * 2 + 0) * D + col] = (sg[0][cl] + sg[1][cl]) + (sg[2][cl] + sg[3][cl]);
        part[((int64_t)blockIdx.y * 2 + 1) * D + col] = (sb[0][cl] + sb[1][cl]) + (sb[2][cl] + sb[3][cl]);
    }
}

// Input gradient AND the per-slab partial sums of the gain / shift gradients in one pass over dy and x: bf16, 8 features
// per lane and access, D % 8 == 0 and D <= 1024 (at most two 8-feature chunks per lane).  A wave walks over 8 rows of
// its workgroup's slab of 4 * kLnRowsPerWave rows; the four waves' partial sums are combined through LDS.
constexpr int kLnRowsPerWave = 4;
__global__ __launch_bounds__(256) void layernorm_bwd_fused_bf16x8_kernel(const bf16_t* __restrict__ dy, const bf16_t* __restrict__ x,
                                                                         const float* __restrict__ stats,
                                                                         const float* __restrict__ gamma, const bf16_t* __restrict__ add,
                                                                         bf16_t* __restrict__ dx, float* __restrict__ part,
                                                                         int64_t rows, int D) {
    __shared__ float sred[4][2][1024];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nch = D >> 3;
    float g[2][8], ag[2][8], ab[2][8];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int c = lane + 64 * i;
        if (c < nch) load8(gamma + c * 8, g[i]);
#pragma unroll
        for (int e = 0; e < 8; ++e) ag[i][e] = ab[i][e] = 0.0f;
    }
    const int64_t r0 = (int64_t)blockIdx.x * (4 * kLnRowsPerWave) + wave * kLnRowsPerWave;
#pragma unroll
    for (int rr = 0; rr < kLnRowsPerWave; ++rr) {
        const int64_t row = r0 + rr;
        if (row >= rows) break;   // uniform per wave
        const float mean = stats[2 * row], rstd = stats[2 * row + 1];
        float dyv[2][8], xh[2][8];
        float s1 = 0.0f, s2 = 0.0f;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int c = lane + 64 * i;
            if (c < nch) {
                float xv[8];
                load8(dy + row * D + c * 8, dyv[i]);
                load8(x + row * D + c * 8, xv);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    xh[i][e] = (xv[e] - mean) * rstd;
                    const float t = dyv[i][e] * g[i][e];
                    s1 += t;
                    s2 += t * xh[i][e];
                    ag[i][e] += dyv[i][e] * xh[i][e];
                    ab[i][e] += dyv[i][e];
                }
            }
        }
        const float m1 = wsum(s1) / (float)D, m2 = wsum(s2) / (float)D;
        if (dx) {
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int c = lane + 64 * i;
                if (c < nch) {
                    float v[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) v[e] = rstd * (dyv[i][e] * g[i][e] - m1 - xh[i][e] * m2);
                    if (add) {
                        float a[8];
                        load8(add + row * D + c * 8, a);
#pragma unroll
                        for (int e = 0; e < 8; ++e) v[e] += a[e];
                    }
                    store8(dx + row * D + c * 8, v);
                }
            }
        }
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int c = lane + 64 * i;
        if (c < nch) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                sred[wave][0][c * 8 + e] = ag[i][e];
                sred[wave][1][c * 8 + e] = ab[i][e];
            }
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < 2 * D; i += 256) {
        const int w = i >= D ? 1 : 0, col = i - w * D;
        part[((int64_t)blockIdx.x * 2 + w) * D + col] = (sred[0][w][col] + sred[1][w][col]) + (sred[2][w][col] + sred[3][w][col]);
    }
}

// out[i] = sum over the slabs of part[slab][i]: 64 outputs per workgroup, sixteen lanes of slabs each, combined through LDS
__global__ __launch_bounds__(1024) void slab_sum_kernel(const float* __restrict__ part, float* __restrict__ out, int count,
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

static int ln_slab_rows(int64_t rows) { return rows > 4096 ? 128 : 32; }

size_t layernorm_workspace_elems(int64_t rows, int D) {
    // the fused backward kernel works on slabs of 4 * kLnRowsPerWave rows whatever the row count
    return (size_t)cdiv_tf(rows, 4 * kLnRowsPerWave) * 2 * (size_t)D;
}

hipError_t layernorm_forward(int dtype, const void* x, const float* gamma, const float* beta, void* y, float* stats,
                             int64_t rows, int D, float eps, hipStream_t s) {
    if (rows <= 0) return hipSuccess;
    dim3 grid(cdiv_tf(rows, 4));
    if (dtype == kBF16) {
        const bool vec = D % 8 == 0 && ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(y) |
                                         reinterpret_cast<uintptr_t>(gamma) | reinterpret_cast<uintptr_t>(beta)) & 15) == 0;
        if (vec)
            return launch_timed(kcLayerNorm, layernorm_fwd_bf16x8_kernel, grid, dim3(256), 0, s, (const bf16_t*)x, gamma,
                                beta, (bf16_t*)y, stats, rows, D, eps);
        return launch_timed(kcLayerNorm, layernorm_fwd_kernel<bf16_t>, grid, dim3(256), 0, s, (const bf16_t*)x, gamma, beta,
                            (bf16_t*)y, stats, rows, D, eps);
    }
    return launch_timed(kcLayerNorm, layernorm_fwd_kernel<float>, grid, dim3(256), 0, s, (const float*)x, gamma, beta,
                        (float*)y, stats, rows, D, eps);
}

hipError_t layernorm_backward(int dtype, const void* dy, const void* x, const float* stats, const float* gamma,
                              const void* add, void* dx, float* dgamma_dbeta, float* ws, int64_t rows, int D,
                              hipStream_t s) {
    if (rows <= 0) return hipSuccess;
    hipError_t e;
    if (dtype == kBF16 && D % 8 == 0 && D <= 1024 &&
        ((reinterpret_cast<uintptr_t>(dy) | reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(gamma) |
          reinterpret_cast<uintptr_t>(add) | reinterpret_cast<uintptr_t>(dx)) & 15) == 0) {
        const int slabs32 = cdiv_tf(rows, 4 * kLnRowsPerWave);
        e = launch_timed(kcLayerNorm, layernorm_bwd_fused_bf16x8_kernel, dim3(slabs32), dim3(256), 0, s, (const bf16_t*)dy,
                         (const bf16_t*)x, stats, gamma, (const bf16_t*)add, (bf16_t*)dx, ws, rows, D);
        if (e != hipSuccess) return e;
        return launch_timed(kcLayerNorm, slab_sum_kernel, dim3(cdiv_tf(2 * D, 64)), dim3(1024), 0, s, (const float*)ws,
                            dgamma_dbeta, 2 * D, slabs32);
    }
    const int slab = ln_slab_rows(rows);
    const int slabs = cdiv_tf(rows, slab);
    dim3 g1(cdiv_tf(rows, 4)), g2(cdiv_tf(D, 64), slabs);
    if (dtype == kBF16) {
        if (dx) {
            e = launch_timed(kcLayerNorm, layernorm_bwd_kernel<bf16_t>, g1, dim3(256), 0, s, (const bf16_t*)dy,
                             (const bf16_t*)x, stats, gamma, (const bf16_t*)add, (bf16_t*)dx, rows, D);
            if (e != hipSuccess) return e;
        }
        e = launch_timed(kcLayerNorm, layernorm_pgrad_kernel<bf16_t>, g2, dim3(256), 0, s, (const bf16_t*)dy,
                         (const bf16_t*)x, stats, ws, rows, D, slab);
    } else {
        if (dx) {
            e = launch_timed(kcLayerNorm, layernorm_bwd_kernel<float>, g1, dim3(256), 0, s, (const float*)dy,
                             (const float*)x, stats, gamma, (const float*)add, (float*)dx, rows, D);
            if (e != hipSuccess) return e;
        }
        e = launch_timed(kcLayerNorm, layernorm_pgrad_kernel<float>, g2, dim3(256), 0, s, (const float*)dy, (const float*)x,
                         stats, ws, rows, D, slab);
    }
    if (e != hipSuccess) return e;
    return launch_timed(kcLayerNorm, slab_sum_kernel, dim3(cdiv_tf(2 * D, 64)), dim3(1024), 0, s, (const float*)ws,
                        dgamma_dbeta, 2 * D, slabs);
}

// ----------------------------------------------------------------------------------------- embedding
// y[row] = wte[tok[row]] + wpe[row % S]; a token outside the vocabulary gives a NaN row, never a wild read.
template <typename T>
__global__ __launch_bounds__(256) void embedding_fwd_kernel(const int32_t* __restrict__ tok, const T* __restrict__ wte,
                                                            const T* __restrict__ wpe, T* __restrict__ y, int64_t rows,
                                                            int S, int D, int vocab) {
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const int t = tok[row];
    const bool ok = t >= 0 && t < vocab;
    const T* a = wte + (int64_t)(ok ? t : 0) * D;
    const T* b = wpe + (int64_t)(row % S) * D;
    T* yr = y + row * D;
    for (int i = lane; i < D; i += 64) yr[i] = ok ? from_f32<T>(to_f32(a[i]) + to_f32(b[i])) : from_f32<T>(NAN);
}

template <typename T>
__global__ void embedding_bwd_pos_kernel(const T* __restrict__ dy, float* __restrict__ dwpe, int64_t B, int64_t SD) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= SD) return;
    float a = 0.0f;
    for (int64_t b = 0; b < B; ++b) a += to_f32(dy[b * SD + i]);
    dwpe[i] = a;
}

// Token-table gradient, deterministic: dwte[t] = sum of the rows of dy whose token is t, added in row order.  One wave
// per row.  The wave of a token's FIRST row (no earlier row has the token: a scan of the rows before it) collects the
// later rows with the same token (a scan of the rows after it, 256 tokens per step) and adds them up in increasing row
// order; every other wave leaves.  No atomic adds, so the sum does not depend on which wave arrives first; rows of
// tokens that do not occur are zero (the table gradient is cleared before).
template <typename T>
__global__ __launch_bounds__(256) void embedding_bwd_tok_kernel(const int32_t* __restrict__ tok, const T* __restrict__ dy,
                                                                float* __restrict__ dwte, int64_t rows, int D, int vocab) {
    constexpr int CAP = 128;   // later occurrences kept in LDS per wave; a token with more is summed by rescanning
    __shared__ int later[4][CAP];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t row = (int64_t)blockIdx.x * 4 + wave;
    if (row >= rows) return;
    const int t = tok[row];
    if (t < 0 || t >= vocab) return;
    for (int64_t base = 0; base < row; base += 256) {
        bool hit = false;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t j = base + u * 64 + lane;
            hit |= j < row && tok[j] == t;
        }
        if (__ballot(hit)) return;   // not the first row of this token (uniform over the wave)
    }
    int n = 0;
    for (int64_t base = row + 1; base < rows; base += 256) {
        int v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t j = base + u * 64 + lane;
            v[u] = j < rows ? tok[j] : -1;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            unsigned long long m = __ballot(v[u] == t);
            while (m) {
                const int b = __ffsll((long long)m) - 1;
                m &= m - 1;
                if (n < CAP && lane == 0) later[wave][n] = (int)(base + u * 64 + b);
                ++n;
            }
        }
    }
    // lane 0 wrote the list, every lane reads it: LDS operations of one wave complete in order; keep the compiler
    // from moving the reads up
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_wave_barrier();
    float* dst = dwte + (int64_t)t * D;
    if (n <= CAP) {
        for (int i = lane; i < D; i += 64) {
            float a = to_f32(dy[row * D + i]);
            for (int k = 0; k < n; ++k) a += to_f32(dy[(int64_t)later[wave][k] * D + i]);
            dst[i] = a;
        }
    } else {
        for (int i = lane; i < D; i += 64) {
            float a = to_f32(dy[row * D + i]);
            for (int64_t j = row + 1; j < rows; ++j)
                if (tok[j] == t) a += to_f32(dy[j * D + i]);
            dst[i] = a;
        }
    }
}

hipError_t embedding_forward(int dtype, const int32_t* tok, const void* wte, const void* wpe, void* y, int64_t rows, int S,
                             int D, int vocab, hipStream_t s) {
    if (rows <= 0) return hipSuccess;
    dim3 grid(cdiv_tf(rows, 4));
    if (dtype == kBF16)
        return launch_timed(kcEmbedding, embedding_fwd_kernel<bf16_t>, grid, dim3(256), 0, s, tok, (const bf16_t*)wte,
                            (const bf16_t*)wpe, (bf16_t*)y, rows, S, D, vocab);
    return launch_timed(kcEmbedding, embedding_fwd_kernel<float>, grid, dim3(256), 0, s, tok, (const float*)wte,
                        (const float*)wpe, (float*)y, rows, S, D, vocab);
}

hipError_t embedding_backward(int dtype, const int32_t* tok, const void* dy, float* dwte, float* dwpe, int64_t B, int S,
                              int D, int vocab, hipStream_t s) {
    if (B <= 0) return hipSuccess;
    const int64_t nw = (int64_t)vocab * D, SD = (int64_t)S * D, rows = B * S;
    int zb = cdiv_tf(nw, 256);
    if (zb > 4096) zb = 4096;
    hipError_t e = launch_timed(kcEmbedding, zero_f32_kernel, dim3(zb), dim3(256), 0, s, dwte, nw);
    if (e != hipSuccess) return e;
    if (dtype == kBF16) {
        e = launch_timed(kcEmbedding, embedding_bwd_pos_kernel<bf16_t>, dim3(cdiv_tf(SD, 256)), dim3(256), 0, s,
                         (const bf16_t*)dy, dwpe, B, SD);
        if (e != hipSuccess) return e;
        return launch_timed(kcEmbedding, embedding_bwd_tok_kernel<bf16_t>, dim3(cdiv_tf(rows, 4)), dim3(256), 0, s, tok,
                            (const bf16_t*)dy, dwte, rows, D, vocab);
    }
    e = launch_timed(kcEmbedding, embedding_bwd_pos_kernel<float>, dim3(cdiv_tf(SD, 256)), dim3(256), 0, s, (const float*)dy,
                     dwpe, B, SD);
    if (e != hipSuccess) return e;
    return launch_timed(kcEmbedding, embedding_bwd_tok_kernel<float>, dim3(cdiv_tf(rows, 4)), dim3(256), 0, s, tok,
                        (const float*)dy, dwte, rows, D, vocab);
}

// ------------------------------------------------------------------------- attention, generic path
// qkv rows are [q | k | v] of D features each; head h owns features h*dh .. h*dh+dh-1 of each part.
// One wave per (batch, head, query row).  Dynamic LDS: S floats (probabilities).
template <typename T>
__global__ __launch_bounds__(64) void attn_fwd_row_kernel(const T* __restrict__ qkv, T* __restrict__ o,
                                                          float* __restrict__ lse, int S, int D, int H, float scale) {
    extern __shared__ float sp[];
    const int i = blockIdx.x, h = blockIdx.y, b = blockIdx.z, lane = threadIdx.x;
    const int dh = D / H;
    const int64_t ld = 3 * (int64_t)D;
    const T* base = qkv + (int64_t)b * S * ld + h * dh;
    const T* qi = base + i * ld;
    float mx = -INFINITY;
    for (int j = lane; j <= i; j += 64) {
        const T* kj = base + j * ld + D;
        float a = 0.0f;
        for (int d = 0; d < dh; ++d) a += to_f32(qi[d]) * to_f32(kj[d]);
        a *= scale;
        sp[j] = a;
        mx = fmaxf(mx, a);
    }
    mx = wmax(mx);
    float sum = 0.0f;
    for (int j = lane; j <= i; j += 64) {
        const float e = expf(sp[j] - mx);
        sp[j] = e;
        sum += e;
    }
    sum = wsum(sum);
    __syncthreads();
    const float inv = 1.0f / sum;
    for (int d = lane; d < dh; d += 64) {
        float a = 0.0f;
        for (int j = 0; j <= i; ++j) a += sp[j] * to_f32(base[j * ld + 2 * D + d]);
        o[((int64_t)b * S + i) * D + h * dh + d] = from_f32<T>(a * inv);
    }
    if (lane == 0) lse[((int64_t)b * H + h) * S + i] = mx + logf(sum);
}

// delta[b, h, i] = sum_d dO[i, d] * O[i, d]
template <typename T>
__global__ __launch_bounds__(256) void attn_delta_kernel(const T* __restrict__ o, const T* __restrict__ dout,
                                                         float* __restrict__ delta, int64_t BS, int S, int D, int H) {
    const int lane = threadIdx.x & 63;
    const int64_t idx = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);   // (b*S + i)*H + h
    if (idx >= BS * H) return;
    const int h = (int)(idx % H);
    const int64_t bi = idx / H;
    const int dh = D / H;
    float a = 0.0f;
    for (int d = lane; d < dh; d += 64) a += to_f32(o[bi * D + h * dh + d]) * to_f32(dout[bi * D + h * dh + d]);
    a = wsum(a);
    if (lane == 0) delta[((bi / S) * H + h) * S + (bi % S)] = a;
}

// The same for bf16 and 64 features per head: 8 lanes share a (row, head) pair, 16 bytes per lane and operand.
__global__ __launch_bounds__(256) void attn_delta_bf16x8_kernel(const bf16_t* __restrict__ o, const bf16_t* __restrict__ dout,
                                                                float* __restrict__ delta, int64_t BS, int S, int H) {
    const int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;   // chunk of 8 features; D = 64 H, so g * 8 is its offset
    const bool ok = g < BS * H * 8;
    float a = 0.0f;
    if (ok) {
        const bf16x8_t vo = *reinterpret_cast<const bf16x8_t*>(o + g * 8), vd = *reinterpret_cast<const bf16x8_t*>(dout + g * 8);
#pragma unroll
        for (int e = 0; e < 8; ++e) a += (float)vo[e] * (float)vd[e];
    }
    a += __shfl_xor(a, 1, 64);
    a += __shfl_xor(a, 2, 64);
    a += __shfl_xor(a, 4, 64);
    if (ok && (g & 7) == 0) {
        const int64_t idx = g >> 3;   // (b*S + i)*H + h
        const int h = (int)(idx % H);
        const int64_t bi = idx / H;
        delta[((bi / S) * H + h) * S + (bi % S)] = a;
    }
}

// Query gradient, one wave per (b, h, i).  Dynamic LDS: S floats (dS row).
template <typename T>
__global__ __launch_bounds__(64) void attn_bwd_q_row_kernel(const T* __restrict__ qkv, const T* __restrict__ dout,
                                                            const float* __restrict__ lse, const float* __restrict__ delta,
                                                            T* __restrict__ dqkv, int S, int D, int H, float scale) {
    extern __shared__ float sp[];
    const int i = blockIdx.x, h = blockIdx.y, b = blockIdx.z, lane = threadIdx.x;
    const int dh = D / H;
    const int64_t ld = 3 * (int64_t)D;
    const T* base = qkv + (int64_t)b * S * ld + h * dh;
    const T* qi = base + i * ld;
    const T* doi = dout + ((int64_t)b * S + i) * D + h * dh;
    const float L = lse[((int64_t)b * H + h) * S + i], dl = delta[((int64_t)b * H + h) * S + i];
    for (int j = lane; j <= i; j += 64) {
        const T* kj = base + j * ld + D;
        const T* vj = base + j * ld + 2 * D;
        float a = 0.0f, dp = 0.0f;
        for (int d = 0; d < dh; ++d) {
            a += to_f32(qi[d]) * to_f32(kj[d]);
            dp += to_f32(doi[d]) * to_f32(vj[d]);
        }
        sp[j] = expf(a * scale - L) * (dp - dl);
    }
    __syncthreads();
    for (int d = lane; d < dh; d += 64) {
        float a = 0.0f;
        for (int j = 0; j <= i; ++j) a += sp[j] * to_f32(base[j * ld + D + d]);
        dqkv[((int64_t)b * S + i) * ld + h * dh + d] = from_f32<T>(a * scale);
    }
}

// Key / value gradients, one wave per (b, h, j).  Dynamic LDS: 2*S floats (P and dS columns).
template <typename T>
__global__ __launch_bounds__(64) void attn_bwd_kv_row_kernel(const T* __restrict__ qkv, const T* __restrict__ dout,
                                                             const float* __restrict__ lse, const float* __restrict__ delta,
                                                             T* __restrict__ dqkv, int S, int D, int H, float scale) {
    extern __shared__ float sp[];
    float* sds = sp + S;
    const int j = blockIdx.x, h = blockIdx.y, b = blockIdx.z, lane = threadIdx.x;
    const int dh = D / H;
    const int64_t ld = 3 * (int64_t)D;
    const T* base = qkv + (int64_t)b * S * ld + h * dh;
    const T* kj = base + j * ld + D;
    const T* vj = base + j * ld + 2 * D;
    for (int i = j + lane; i < S; i += 64) {
        const T* qi = base + i * ld;
        const T* doi = dout + ((int64_t)b * S + i) * D + h * dh;
        float a = 0.0f, dp = 0.0f;
        for (int d = 0; d < dh; ++d) {
            a += to_f32(qi[d]) * to_f32(kj[d]);
            dp += to_f32(doi[d]) * to_f32(vj[d]);
        }
        const float p = expf(a * scale - lse[((int64_t)b * H + h) * S + i]);
        sp[i] = p;
        sds[i] = p * (dp - delta[((int64_t)b * H + h) * S + i]);
    }
    __syncthreads();
    for (int d = lane; d < dh; d += 64) {
        float dk = 0.0f, dv = 0.0f;
        for (int i = j; i < S; ++i) {
            dk += sds[i] * to_f32(base[i * ld + d]);
            dv += sp[i] * to_f32(dout[((int64_t)b * S + i) * D + h * dh + d]);
        }
        dqkv[((int64_t)b * S + j) * ld + D + h * dh + d] = from_f32<T>(dk * scale);
        dqkv[((int64_t)b * S + j) * ld + 2 * D + h * dh + d] = from_f32<T>(dv);
    }
}

// ---------------------------------------------------------------------------- attention, MFMA path
// bf16, 64 features per head.  LDS tiles are [64 rows][64 + 8] bf16 (144-byte rows).  Exponentials use the
// hardware exp2 (a few ulp of fp32, far below the bf16 rounding of the results): the library expf costs some
// 25 instructions and made the softmax, not the MFMAs, the bulk of these kernels.
constexpr int kAP = 72;   // LDS row pitch in elements
// 16 bytes in flight between global memory and LDS (a native vector: arrays of it stay in registers)
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

// B-operand / A-operand fragment of a row-major tile: lane holds row (lane % 32), 8 consecutive features
// 16*t + 8*(lane / 32) ..; straight from global memory (rows clamped to the last valid one).
__device__ __forceinline__ bf16x8_t gfrag(const bf16_t* base, int64_t ld, int row, int max_row, int t, int lane) {
    int r = row + (lane & 31);
    r = r < max_row ? r : max_row - 1;
    return *reinterpret_cast<const bf16x8_t*>(base + r * ld + t * 16 + (lane >> 5) * 8);
}
// The same fragment from an LDS tile (rows row0 .. row0+31).
__device__ __forceinline__ bf16x8_t lfrag(const bf16_t* tile, int row0, int t, int lane) {
    return *reinterpret_cast<const bf16x8_t*>(tile + (row0 + (lane & 31)) * kAP + t * 16 + (lane >> 5) * 8);
}
// Transposed fragment: the MFMA row is the FEATURE f0 + lane % 32 and the contraction runs over 16 tile rows
// r0 .. r0+15 in the order in which a 32x32 accumulator holds them: slot (half = lane / 32, e) is tile row
// r0 + 8*(e/4) + 4*half + e%4.  Two transpose reads of 4 rows each.
__device__ __forceinline__ bf16x8_t lfrag_t(const bf16_t* tile, int r0, int f0, int lane) {
    typedef __attribute__((address_space(3))) s16x4_t* lds_ptr_t;
    const int row = r0 + 4 * (lane >> 5) + ((lane & 15) >> 2);
    const int col = f0 + ((lane >> 4) & 1) * 16 + (lane & 3) * 4;
    const bf16_t* p0 = tile + row * kAP + col;
    const bf16_t* p1 = p0 + 8 * kAP;
    union { s16x4_t h[2]; bf16x8_t v; } u;
    u.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(p0));
    u.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(p1));
    return u.v;
}
// Accumulator registers 8*t .. 8*t+7 as a B-operand fragment (bf16).
__device__ __forceinline__ bf16x8_t acc_frag(const f32x16_t& a, int t) {
    bf16x8_t f;
#pragma unroll
    for (int e = 0; e < 8; ++e) f[e] = (bf16_t)a[8 * t + e];
    return f;
}
// Cooperative copy of 64 rows x 64 features (row stride ld) into an LDS tile; rows >= max_row are clamped.
template <int NT>
__device__ __forceinline__ void load_tile(bf16_t* tile, const bf16_t* base, int64_t ld, int row0, int max_row, int tid) {
#pragma unroll
    for (int c = tid; c < 512; c += NT) {
        int r = row0 + (c >> 3);
        r = r < max_row ? r : max_row - 1;
        *reinterpret_cast<uint4*>(tile + (c >> 3) * kAP + (c & 7) * 8) =
            *reinterpret_cast<const uint4*>(base + r * ld + (c & 7) * 8);
    }
}

// The same copy in two halves, so that the global loads of the next tile are in flight while the current one is
// multiplied: fetch() issues the loads into registers, put() writes them to the LDS tile.
template <int NT> struct TileFetch {
    static constexpr int N = 512 / NT;
    u32x4_t r[N];
    __device__ __forceinline__ void fetch(const bf16_t* base, int64_t ld, int row0, int max_row, int tid) {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const int c = tid + i * NT;
            int row = row0 + (c >> 3);
            row = row < max_row ? row : max_row - 1;
            r[i] = *reinterpret_cast<const u32x4_t*>(base + row * ld + (c & 7) * 8);
        }
    }
    __device__ __forceinline__ void put(bf16_t* tile, int tid) const {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const int c = tid + i * NT;
            *reinterpret_cast<u32x4_t*>(tile + (c >> 3) * kAP + (c & 7) * 8) = r[i];
        }
    }
};

// exp2 on the hardware unit; scores are kept in units of log 2 (scale * log2(e) folded into one factor), so that a
// probability costs one fused multiply-add and one exp2.
__device__ __forceinline__ float exp2_hw(float x) { return __builtin_amdgcn_exp2f(x); }
constexpr float kLog2e = 1.4426950408889634f, kLn2 = 0.6931471805599453f;

// One 32-key block of the running softmax of 32 queries (one per lane pair; keys along the registers).  st holds the
// raw scores q.k and leaves as unnormalised probabilities; m_run (in units of log 2) and l_run are the running
// maximum and sum, ot the running output, rescaled here.  MASK: the block straddles the diagonal (or the end of
// the sequence): keys after the query are excluded.  Blocks below the diagonal skip the three mask instructions
// per element.
template <bool MASK>
__device__ __forceinline__ void softmax_block(f32x16_t& st, int kb, int q, int half, float scale2, float& m_run, float& l_run,
                                              f32x16_t (&ot)[2]) {
    float mt = -INFINITY;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        if constexpr (MASK) {
            const int key = kb + 8 * (r >> 2) + 4 * half + (r & 3);
            st[r] = key <= q ? st[r] : -INFINITY;
        }
        mt = fmaxf(mt, st[r]);
    }
    mt = fmaxf(mt, __shfl_xor(mt, 32, 64));
    const float m_new = fmaxf(m_run, mt * scale2);       // scale2 > 0: the maximum commutes with the scaling
    const float m_use = m_new == -INFINITY ? 0.0f : m_new;   // a query with no key yet keeps zeros
    const float alpha = exp2_hw(m_run - m_use);
    float ls = 0.0f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        st[r] = exp2_hw(fmaf(st[r], scale2, -m_use));
        ls += st[r];
    }
    l_run = l_run * alpha + ls;
    m_run = m_new;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) ot[i][r] *= alpha;
}

// Forward.  Block = NW waves = 32*NW query rows of one (batch, head).
// Workgroups go to the 8 XCDs (each with its own L2) round-robin in launch order (x fastest, then y, then z).  Hand
// every XCD a contiguous run of that order instead: the query (or key) blocks of one (batch, head) then sit on one XCD,
// and the keys and values (queries and output gradients) they all read come in from memory once, not once per XCD.
__device__ __forceinline__ void xcd_local_block(int& x, int& y, int& z) {
    const int gx = gridDim.x, gy = gridDim.y, plane = gx * gy, total = plane * gridDim.z;
    x = blockIdx.x; y = blockIdx.y; z = blockIdx.z;
    if (total < 16) return;
    const int lin = (z * gy + y) * gx + x;
    const int xcd = lin & 7, idx = lin >> 3, q = total >> 3, r = total & 7;
    int moved = xcd * q + min(xcd, r) + idx;
    z = moved / plane;
    moved -= z * plane;
    y = moved / gx;
    x = moved - y * gx;
}

template <int NW>
__global__ __launch_bounds__(64 * NW) void attn_fwd_mfma_kernel(const bf16_t* __restrict__ qkv, bf16_t* __restrict__ o,
                                                                float* __restrict__ lse, int S, int D, int H, float scale) {
    __shared__ __attribute__((aligned(16))) bf16_t sKb[2][64 * kAP];
    __shared__ __attribute__((aligned(16))) bf16_t sVb[2][64 * kAP];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, half = lane >> 5;
    int bx, h, b;
    xcd_local_block(bx, h, b);
    const int qb = gridDim.x - 1 - bx;
    const int64_t ld = 3 * (int64_t)D;
    const bf16_t* base = qkv + (int64_t)b * S * ld + h * 64;
    const int q0 = (qb * NW + wave) * 32;
    const int q = q0 + (lane & 31);
    TileFetch<64 * NW> fk, fv;
    fk.fetch(base + D, ld, 0, S, tid);
    fv.fetch(base + 2 * D, ld, 0, S, tid);
    bf16x8_t qf[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) qf[t] = gfrag(base, ld, q0, S, t, lane);
    f32x16_t ot[2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) ot[i][r] = 0.0f;
    float m_run = -INFINITY, l_run = 0.0f;
    const float scale2 = scale * kLog2e;
    const int kv_end = min(S, (qb + 1) * NW * 32);
    fk.put(sKb[0], tid);
    fv.put(sVb[0], tid);
    __syncthreads();
    for (int kv0 = 0, it = 0; kv0 < kv_end; kv0 += 64, ++it) {
        const bf16_t* sK = sKb[it & 1];
        const bf16_t* sV = sVb[it & 1];
        // the next tile's loads fly while this one is multiplied (past the last tile they re-read clamped, valid rows
        // and the copy lands in the buffer that nobody reads again)
        fk.fetch(base + D, ld, kv0 + 64, S, tid);
        fv.fetch(base + 2 * D, ld, kv0 + 64, S, tid);
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            const int kb = kv0 + 32 * sub;
            if (kb > q0 + 31) continue;   // every key of the tile lies after every query of this wave
            f32x16_t st;
#pragma unroll
            for (int r = 0; r < 16; ++r) st[r] = 0.0f;
#pragma unroll
            for (int t = 0; t < 4; ++t)
                st = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lfrag(sK, 32 * sub, t, lane), qf[t], st, 0, 0, 0);
            if (kb + 31 <= q0) softmax_block<false>(st, kb, q, half, scale2, m_run, l_run, ot);
            else softmax_block<true>(st, kb, q, half, scale2, m_run, l_run, ot);
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const bf16x8_t pf = acc_frag(st, t);
#pragma unroll
                for (int i = 0; i < 2; ++i)
                    ot[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lfrag_t(sV, 32 * sub + 16 * t, 32 * i, lane), pf, ot[i], 0, 0, 0);
            }
        }
        fk.put(sKb[(it + 1) & 1], tid);   // the other buffer was last read before the previous barrier
        fv.put(sVb[(it + 1) & 1], tid);
        __syncthreads();
    }
    const float l = l_run + __shfl_xor(l_run, 32, 64);
    if (q < S) {
        const float inv = 1.0f / l;
        bf16_t* orow = o + ((int64_t)b * S + q) * D + h * 64;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                union { bf16_t hv[4]; uint2 u; } pk;
#pragma unroll
                for (int e = 0; e < 4; ++e) pk.hv[e] = (bf16_t)(ot[i][4 * g + e] * inv);
                *reinterpret_cast<uint2*>(orow + 32 * i + 8 * g + 4 * half) = pk.u;
            }
        if (half == 0) lse[((int64_t)b * H + h) * S + q] = m_run * kLn2 + logf(l);
    }
}

// Forward for launches with few (batch, head) pairs, where the kernel above leaves most of the chip idle and its
// longest workgroup walks the whole key range alone.  A workgroup owns 32 query rows; its NW waves take the 32-key
// blocks up to the diagonal in turn (wave w: blocks w, w + NW, ...) with their own running statistics, and the
// partial results are merged at the end: O = sum_w e^{m_w - m} O_w, l = sum_w e^{m_w - m} l_w, m = max_w m_w.
// Nothing is shared between the waves inside the loop, so there is no workgroup barrier in it: K fragments come
// straight from global memory, V passes through a wave-private LDS tile for the transpose read.
template <int NW>
__global__ __launch_bounds__(64 * NW) void attn_fwd_split_kernel(const bf16_t* __restrict__ qkv, bf16_t* __restrict__ o,
                                                                 float* __restrict__ lse, int S, int D, int H, float scale) {
    __shared__ __attribute__((aligned(16))) bf16_t sVw[NW][32 * kAP];
    __shared__ float sOw[NW - 1][32][64];
    __shared__ float sMw[NW - 1][32], sLw[NW - 1][32];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, half = lane >> 5;
    int bx, h, b;
    xcd_local_block(bx, h, b);
    const int qb = gridDim.x - 1 - bx;
    const int64_t ld = 3 * (int64_t)D;
    const bf16_t* base = qkv + (int64_t)b * S * ld + h * 64;
    const int q0 = qb * 32;
    const int q = q0 + (lane & 31);
    bf16_t* const sV = sVw[wave];
    bf16x8_t qf[4], kn[4];
    u32x4_t vn[4];
    auto fetch = [&](int j) {   // rows are clamped: a fetch past the diagonal re-reads valid rows and is never used
#pragma unroll
        for (int t = 0; t < 4; ++t) kn[t] = gfrag(base + D, ld, 32 * j, S, t, lane);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int c = lane + 64 * i;
            int row = 32 * j + (c >> 3);
            row = row < S ? row : S - 1;
            vn[i] = *reinterpret_cast<const u32x4_t*>(base + 2 * D + row * ld + (c & 7) * 8);
        }
    };
    fetch(wave);
#pragma unroll
    for (int t = 0; t < 4; ++t) qf[t] = gfrag(base, ld, q0, S, t, lane);
    f32x16_t ot[2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) ot[i][r] = 0.0f;
    float m_run = -INFINITY, l_run = 0.0f;
    const float scale2 = scale * kLog2e;
    for (int j = wave; j <= qb; j += NW) {
        bf16x8_t kf[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) kf[t] = kn[t];
        // LDS serves a wave's accesses in order: the transpose reads of the previous block are done before these writes
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int c = lane + 64 * i;
            *reinterpret_cast<u32x4_t*>(sV + (c >> 3) * kAP + (c & 7) * 8) = vn[i];
        }
        __builtin_amdgcn_wave_barrier();
        fetch(j + NW);
        const int kb = 32 * j;
        f32x16_t st;
#pragma unroll
        for (int r = 0; r < 16; ++r) st[r] = 0.0f;
#pragma unroll
        for (int t = 0; t < 4; ++t) st = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[t], qf[t], st, 0, 0, 0);
        if (kb + 31 <= q0) softmax_block<false>(st, kb, q, half, scale2, m_run, l_run, ot);
        else softmax_block<true>(st, kb, q, half, scale2, m_run, l_run, ot);
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const bf16x8_t pf = acc_frag(st, t);
#pragma unroll
            for (int i = 0; i < 2; ++i)
                ot[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lfrag_t(sV, 16 * t, 32 * i, lane), pf, ot[i], 0, 0, 0);
        }
    }
    float l = l_run + __shfl_xor(l_run, 32, 64);
    if (wave > 0) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) sOw[wave - 1][16 * i + r][lane] = ot[i][r];
        if (half == 0) {
            sMw[wave - 1][lane] = m_run;
            sLw[wave - 1][lane] = l;
        }
    }
    __syncthreads();
    if (wave != 0) return;
    // wave 0 always owns key block 0, which every query sees: its maximum is finite
    float m = m_run;
#pragma unroll
    for (int w = 0; w < NW - 1; ++w) m = fmaxf(m, sMw[w][lane & 31]);
    const float f0 = exp2_hw(m_run - m);
    l *= f0;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) ot[i][r] *= f0;
#pragma unroll
    for (int w = 0; w < NW - 1; ++w) {
        const float fw = exp2_hw(sMw[w][lane & 31] - m);   // a wave that had no block holds -inf: factor 0
        l += fw * sLw[w][lane & 31];
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) ot[i][r] += fw * sOw[w][16 * i + r][lane];
    }
    if (q < S) {
        const float inv = 1.0f / l;
        bf16_t* orow = o + ((int64_t)b * S + q) * D + h * 64;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                union { bf16_t hv[4]; uint2 u; } pk;
#pragma unroll
                for (int e = 0; e < 4; ++e) pk.hv[e] = (bf16_t)(ot[i][4 * g + e] * inv);
                *reinterpret_cast<uint2*>(orow + 32 * i + 8 * g + 4 * half) = pk.u;
            }
        if (half == 0) lse[((int64_t)b * H + h) * S + q] = m * kLn2 + logf(l);
    }
}

// Query gradient.  Same arrangement as the forward pass: P^T and dS^T have keys along the registers.
template <int NW>
__global__ __launch_bounds__(64 * NW) void attn_bwd_q_mfma_kernel(const bf16_t* __restrict__ qkv,
                                                                  const bf16_t* __restrict__ dout,
                                                                  const float* __restrict__ lse,
                                                                  const float* __restrict__ delta,
                                                                  bf16_t* __restrict__ dqkv, int S, int D, int H,
                                                                  float scale) {
    __shared__ __attribute__((aligned(16))) bf16_t sKb[2][64 * kAP];
    __shared__ __attribute__((aligned(16))) bf16_t sVb[2][64 * kAP];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, half = lane >> 5;
    int bx, h, b;
    xcd_local_block(bx, h, b);
    const int qb = gridDim.x - 1 - bx;
    const int64_t ld = 3 * (int64_t)D;
    const bf16_t* base = qkv + (int64_t)b * S * ld + h * 64;
    const bf16_t* dob = dout + (int64_t)b * S * D + h * 64;
    TileFetch<64 * NW> fk, fv;
    fk.fetch(base + D, ld, 0, S, tid);
    fv.fetch(base + 2 * D, ld, 0, S, tid);
    const int q0 = (qb * NW + wave) * 32;
    const int q = q0 + (lane & 31);
    const int qc = q < S ? q : S - 1;
    bf16x8_t qf[4], dof[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        qf[t] = gfrag(base, ld, q0, S, t, lane);
        dof[t] = gfrag(dob, D, q0, S, t, lane);
    }
    const float L2 = lse[((int64_t)b * H + h) * S + qc] * kLog2e, dl = delta[((int64_t)b * H + h) * S + qc];
    const float scale2 = scale * kLog2e;
    f32x16_t dq[2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) dq[i][r] = 0.0f;
    const int kv_end = min(S, (qb + 1) * NW * 32);
    fk.put(sKb[0], tid);
    fv.put(sVb[0], tid);
    __syncthreads();
    for (int kv0 = 0, it = 0; kv0 < kv_end; kv0 += 64, ++it) {
        const bf16_t* sK = sKb[it & 1];
        const bf16_t* sV = sVb[it & 1];
        fk.fetch(base + D, ld, kv0 + 64, S, tid);
        fv.fetch(base + 2 * D, ld, kv0 + 64, S, tid);
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            const int kb = kv0 + 32 * sub;
            if (kb > q0 + 31) continue;
            f32x16_t st, dp;
#pragma unroll
            for (int r = 0; r < 16; ++r) st[r] = dp[r] = 0.0f;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                st = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lfrag(sK, 32 * sub, t, lane), qf[t], st, 0, 0, 0);
                dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lfrag(sV, 32 * sub, t, lane), dof[t], dp, 0, 0, 0);
            }
            if (kb + 31 <= q0) {   // below the diagonal: no key is excluded
#pragma unroll
                for (int r = 0; r < 16; ++r) st[r] = exp2_hw(fmaf(st[r], scale2, -L2)) * (dp[r] - dl);
            } else {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = kb + 8 * (r >> 2) + 4 * half + (r & 3);
                    const float p = key <= q ? exp2_hw(fmaf(st[r], scale2, -L2)) : 0.0f;
                    st[r] = p * (dp[r] - dl);
                }
            }
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const bf16x8_t df = acc_frag(st, t);
#pragma unroll
                for (int i = 0; i < 2; ++i)
                    dq[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lfrag_t(sK, 32 * sub + 16 * t, 32 * i, lane), df, dq[i], 0, 0, 0);
            }
        }
        fk.put(sKb[(it + 1) & 1], tid);
        fv.put(sVb[(it + 1) & 1], tid);
        __syncthreads();
    }
    if (q < S) {
        bf16_t* drow = dqkv + ((int64_t)b * S + q) * ld + h * 64;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                union { bf16_t hv[4]; uint2 u; } pk;
#pragma unroll
                for (int e = 0; e < 4; ++e) pk.hv[e] = (bf16_t)(dq[i][4 * g + e] * scale);
                *reinterpret_cast<uint2*>(drow + 32 * i + 8 * g + 4 * half) = pk.u;
            }
    }
}

// Key and value gradients.  A wave owns 32 keys (lanes); queries run along the accumulator registers, so the
// per-query statistics (log-sum-exp, delta) are read per register from LDS.
template <int NW>
__global__ __launch_bounds__(64 * NW) void attn_bwd_kv_mfma_kernel(const bf16_t* __restrict__ qkv,
                                                                   const bf16_t* __restrict__ dout,
                                                                   const float* __restrict__ lse,
                                                                   const float* __restrict__ delta,
                                                                   bf16_t* __restrict__ dqkv, int S, int D, int H,
                                                                   float scale) {
    __shared__ __attribute__((aligned(16))) bf16_t sQb[2][64 * kAP];
    __shared__ __attribute__((aligned(16))) bf16_t sOb[2][64 * kAP];
    __shared__ __attribute__((aligned(16))) float sLb[2][64], sDlb[2][64];   // log-sum-exp (in units of log 2) and delta
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, half = lane >> 5;
    int kblk, h, b;
    xcd_local_block(kblk, h, b);
    const int64_t ld = 3 * (int64_t)D;
    const bf16_t* base = qkv + (int64_t)b * S * ld + h * 64;
    const bf16_t* dob = dout + (int64_t)b * S * D + h * 64;
    const int k0 = (kblk * NW + wave) * 32;
    const int key = k0 + (lane & 31);
    const float scale2 = scale * kLog2e;
    bf16x8_t kf[4], vf[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        kf[t] = gfrag(base + D, ld, k0, S, t, lane);
        vf[t] = gfrag(base + 2 * D, ld, k0, S, t, lane);
    }
    f32x16_t dk[2], dv[2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) dk[i][r] = dv[i][r] = 0.0f;
    const int qstart = (kblk * NW * 32) / 64 * 64;   // first query block that can see a key of this workgroup
    TileFetch<64 * NW> fq, fo;
    float pl = 0.0f, pd = 0.0f;   // statistics of query qb0 + tid (threads 0..63)
    auto fetch_stats = [&](int qb0) {
        if (tid < 64) {
            const int qq = qb0 + tid < S ? qb0 + tid : S - 1;
            pl = lse[((int64_t)b * H + h) * S + qq];
            pd = delta[((int64_t)b * H + h) * S + qq];
        }
    };
    auto put_stats = [&](int buf) {
        if (tid < 64) {
            sLb[buf][tid] = pl * kLog2e;
            sDlb[buf][tid] = pd;
        }
    };
    fq.fetch(base, ld, qstart, S, tid);
    fo.fetch(dob, D, qstart, S, tid);
    fetch_stats(qstart);
    fq.put(sQb[0], tid);
    fo.put(sOb[0], tid);
    put_stats(0);
    __syncthreads();
    for (int qb0 = qstart, it = 0; qb0 < S; qb0 += 64, ++it) {
        const bf16_t* sQ = sQb[it & 1];
        const bf16_t* sO = sOb[it & 1];
        const float* sL = sLb[it & 1];
        const float* sDl = sDlb[it & 1];
        fq.fetch(base, ld, qb0 + 64, S, tid);
        fo.fetch(dob, D, qb0 + 64, S, tid);
        fetch_stats(qb0 + 64);
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            const int qs = qb0 + 32 * sub;
            if (qs + 31 < k0) continue;   // every query of the tile lies before every key of this wave
            f32x16_t st, dp;
#pragma unroll
            for (int r = 0; r < 16; ++r) st[r] = dp[r] = 0.0f;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                st = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lfrag(sQ, 32 * sub, t, lane), kf[t], st, 0, 0, 0);
                dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lfrag(sO, 32 * sub, t, lane), vf[t], dp, 0, 0, 0);
            }
            // statistics of the 4 consecutive queries of a register group in one LDS read each
            float4 l4[4], d4[4];
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                l4[g] = *reinterpret_cast<const float4*>(sL + 32 * sub + 8 * g + 4 * half);
                d4[g] = *reinterpret_cast<const float4*>(sDl + 32 * sub + 8 * g + 4 * half);
            }
            const bool inner = k0 + 31 <= qs && qs + 32 <= S;   // every query of the block sees every key of this wave
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float Lq = (r & 3) == 0 ? l4[r >> 2].x : (r & 3) == 1 ? l4[r >> 2].y : (r & 3) == 2 ? l4[r >> 2].z : l4[r >> 2].w;
                const float Dq = (r & 3) == 0 ? d4[r >> 2].x : (r & 3) == 1 ? d4[r >> 2].y : (r & 3) == 2 ? d4[r >> 2].z : d4[r >> 2].w;
                float p = exp2_hw(fmaf(st[r], scale2, -Lq));
                if (!inner) {
                    const int qq = qs + 8 * (r >> 2) + 4 * half + (r & 3);
                    p = (key <= qq && qq < S) ? p : 0.0f;
                }
                st[r] = p;
                dp[r] = p * (dp[r] - Dq);
            }
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const bf16x8_t pf = acc_frag(st, t), df = acc_frag(dp, t);
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    dv[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lfrag_t(sO, 32 * sub + 16 * t, 32 * i, lane), pf, dv[i], 0, 0, 0);
                    dk[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lfrag_t(sQ, 32 * sub + 16 * t, 32 * i, lane), df, dk[i], 0, 0, 0);
                }
            }
        }
        fq.put(sQb[(it + 1) & 1], tid);
        fo.put(sOb[(it + 1) & 1], tid);
        put_stats((it + 1) & 1);
        __syncthreads();
    }
    if (key < S) {
        bf16_t* drow = dqkv + ((int64_t)b * S + key) * ld + h * 64;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                union { bf16_t hv[4]; uint2 u; } pk, pv;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    pk.hv[e] = (bf16_t)(dk[i][4 * g + e] * scale);
                    pv.hv[e] = (bf16_t)dv[i][4 * g + e];
                }
                *reinterpret_cast<uint2*>(drow + D + 32 * i + 8 * g + 4 * half) = pk.u;
                *reinterpret_cast<uint2*>(drow + 2 * D + 32 * i + 8 * g + 4 * half) = pv.u;
            }
    }
}

// Waves per workgroup of the tiled attention kernels.  Every workgroup streams the whole key (query) range of its
// (batch, head) pair through LDS, so the traffic from L2 falls with the number of rows that share a tile: the widest
// workgroup that still leaves about one per compute unit.
static int attn_waves(int B, int S, int H) {
    const int64_t bh = (int64_t)B * H;
    if (cdiv_tf(S, 256) * bh >= 192) return 8;
    if (cdiv_tf(S, 128) * bh >= 192) return 4;
    return 2;
}

static bool attn_mfma_ok(int dtype, const void* a, const void* b, int D, int H) {
    return dtype == kBF16 && H > 0 && D == 64 * H &&
           ((reinterpret_cast<uintptr_t>(a) | reinterpret_cast<uintptr_t>(b)) & 15) == 0;
}

size_t attention_workspace_elems(int B, int S, int H) { return (size_t)B * S * H; }

hipError_t attention_forward(int dtype, const void* qkv, void* o, float* lse, int B, int S, int D, int H, hipStream_t s) {
    if (B <= 0) return hipSuccess;
    const float scale = 1.0f / sqrtf((float)(D / H));
    if (attn_mfma_ok(dtype, qkv, o, D, H)) {
        const bf16_t* in = (const bf16_t*)qkv;
        bf16_t* out = (bf16_t*)o;
        if ((int64_t)cdiv_tf(S, 64) * H * B < 512)   // too few workgroups of the tiled kernel to fill the chip
            return launch_timed(kcAttnFwd, attn_fwd_split_kernel<4>, dim3(cdiv_tf(S, 32), H, B), dim3(256), 0, s, in, out,
                                lse, S, D, H, scale);
        switch (attn_waves(B, S, H)) {
            case 8:
                return launch_timed(kcAttnFwd, attn_fwd_mfma_kernel<8>, dim3(cdiv_tf(S, 256), H, B), dim3(512), 0, s, in, out,
                                    lse, S, D, H, scale);
            case 4:
                return launch_timed(kcAttnFwd, attn_fwd_mfma_kernel<4>, dim3(cdiv_tf(S, 128), H, B), dim3(256), 0, s, in, out,
                                    lse, S, D, H, scale);
            default:
                return launch_timed(kcAttnFwd, attn_fwd_mfma_kernel<2>, dim3(cdiv_tf(S, 64), H, B), dim3(128), 0, s, in, out,
                                    lse, S, D, H, scale);
        }
    }
    const unsigned lds = (unsigned)S * 4;
    if (dtype == kBF16)
        return launch_timed(kcAttnFwd, attn_fwd_row_kernel<bf16_t>, dim3(S, H, B), dim3(64), lds, s, (const bf16_t*)qkv,
                            (bf16_t*)o, lse, S, D, H, scale);
    return launch_timed(kcAttnFwd, attn_fwd_row_kernel<float>, dim3(S, H, B), dim3(64), lds, s, (const float*)qkv, (float*)o,
                        lse, S, D, H, scale);
}

hipError_t attention_backward(int dtype, const void* qkv, const void* o, const void* dout, const float* lse, float* delta,
                              void* dqkv, int B, int S, int D, int H, hipStream_t s) {
    if (B <= 0) return hipSuccess;
    const float scale = 1.0f / sqrtf((float)(D / H));
    const int64_t BS = (int64_t)B * S;
    hipError_t e;
    if (attn_mfma_ok(dtype, o, dout, D, H))
        e = launch_timed(kcAttnBwd, attn_delta_bf16x8_kernel, dim3(cdiv_tf(BS * H * 8, 256)), dim3(256), 0, s, (const bf16_t*)o,
                         (const bf16_t*)dout, delta, BS, S, H);
    else if (dtype == kBF16)
        e = launch_timed(kcAttnBwd, attn_delta_kernel<bf16_t>, dim3(cdiv_tf(BS * H, 4)), dim3(256), 0, s, (const bf16_t*)o,
                         (const bf16_t*)dout, delta, BS, S, D, H);
    else
        e = launch_timed(kcAttnBwd, attn_delta_kernel<float>, dim3(cdiv_tf(BS * H, 4)), dim3(256), 0, s, (const float*)o,
                         (const float*)dout, delta, BS, S, D, H);
    if (e != hipSuccess) return e;
    if (attn_mfma_ok(dtype, qkv, dout, D, H) && (reinterpret_cast<uintptr_t>(dqkv) & 15) == 0) {
        auto go = [&](auto nwc) {
            constexpr int NW = decltype(nwc)::value;
            dim3 grid(cdiv_tf(S, 32 * NW), H, B);
            hipError_t e2 = launch_timed(kcAttnBwd, attn_bwd_q_mfma_kernel<NW>, grid, dim3(64 * NW), 0, s, (const bf16_t*)qkv,
                                         (const bf16_t*)dout, (const float*)lse, (const float*)delta, (bf16_t*)dqkv, S, D, H,
                                         scale);
            if (e2 != hipSuccess) return e2;
            return launch_timed(kcAttnBwd, attn_bwd_kv_mfma_kernel<NW>, grid, dim3(64 * NW), 0, s, (const bf16_t*)qkv,
                                (const bf16_t*)dout, (const float*)lse, (const float*)delta, (bf16_t*)dqkv, S, D, H, scale);
        };
        switch (attn_waves(B, S, H)) {
            case 8: return go(std::integral_constant<int, 8>{});
            case 4: return go(std::integral_constant<int, 4>{});
            default: return go(std::integral_constant<int, 2>{});
        }
    }
    dim3 grid(S, H, B);
    if (dtype == kBF16) {
        e = launch_timed(kcAttnBwd, attn_bwd_q_row_kernel<bf16_t>, grid, dim3(64), (unsigned)S * 4, s, (const bf16_t*)qkv,
                         (const bf16_t*)dout, (const float*)lse, (const float*)delta, (bf16_t*)dqkv, S, D, H, scale);
        if (e != hipSuccess) return e;
        return launch_timed(kcAttnBwd, attn_bwd_kv_row_kernel<bf16_t>, grid, dim3(64), (unsigned)S * 8, s,
                            (const bf16_t*)qkv, (const bf16_t*)dout, (const float*)lse, (const float*)delta, (bf16_t*)dqkv,
                            S, D, H, scale);
    }
    e = launch_timed(kcAttnBwd, attn_bwd_q_row_kernel<float>, grid, dim3(64), (unsigned)S * 4, s, (const float*)qkv,
                     (const float*)dout, (const float*)lse, (const float*)delta, (float*)dqkv, S, D, H, scale);
    if (e != hipSuccess) return e;
    return launch_timed(kcAttnBwd, attn_bwd_kv_row_kernel<float>, grid, dim3(64), (unsigned)S * 8, s, (const float*)qkv,
                        (const float*)dout, (const float*)lse, (const float*)delta, (float*)dqkv, S, D, H, scale);
}

}  // namespace tmps
