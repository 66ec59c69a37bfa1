// Contraction kernels of the stage step for gfx950: one MFMA GEMM skeleton (bf16 in, fp32
// accumulate) and one plain fp32 GEMM skeleton, both parameterised by operand "views" that map
// (row, k) of the GEMM to memory.  Dense forward / input-gradient / weight-gradient and the
// implicit-GEMM forms of convolution are all instances; nothing is materialised (no im2col).
//
// GEMM convention: C[m, n] = sum_k A(m, k) * B(n, k).  A view is "k-contiguous" when
// consecutive k of one row are consecutive in memory (then 8 bf16 are fetched with one 16-byte
// load), otherwise consecutive rows are (then a wave reads 64 consecutive rows per k and the
// transposition happens on the way into LDS).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tmps {

typedef __bf16 bf16_t;
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16_t v) { return (float)v; }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return (bf16_t)v; }

union Pack8 {
    uint4 u;
    bf16_t h[8];
};

// ------------------------------------------------------------------------------------------
// Operand views
// ------------------------------------------------------------------------------------------

// Plain matrix.  KC: element(row, k) = p[row*ld + k];  otherwise element(row, k) = p[k*ld + row].
template <typename T, bool KC> struct DenseView {
    static constexpr bool kContig = KC;
    const T* p;
    int rows, K;
    int64_t ld;
    int vec_ok;  // base 16-byte aligned and ld % 8 == 0
    __device__ __forceinline__ T at(int row, int k) const {
        if (row >= rows || k >= K) return T(0.0f);
        return KC ? p[(int64_t)row * ld + k] : p[(int64_t)k * ld + row];
    }
    __device__ __forceinline__ uint4 load8(int row, int k) const {
        if (KC && vec_ok && row < rows && k + 8 <= K)
            return *reinterpret_cast<const uint4*>(p + (int64_t)row * ld + k);
        Pack8 r;
#pragma unroll
        for (int i = 0; i < 8; ++i) r.h[i] = (bf16_t)at(row, k + i);
        return r.u;
    }
};

struct ConvGeom {
    int B, H, W, Cin, Ho, Wo, Cout, R, S, stride, pad;
};

// Forward A operand: row m = (n, ho, wo), k = (r, s, c) -> x[n, ho*stride+r-pad, wo*stride+s-pad, c].
template <typename T> struct ConvFwdA {
    static constexpr bool kContig = true;
    const T* x;
    ConvGeom g;
    int rows, K, vec_ok;  // vec_ok: Cin % 8 == 0 and base aligned
    __device__ __forceinline__ int64_t addr(int m, int k, bool& ok) const {
        int hw = g.Ho * g.Wo;
        int n = m / hw, rem = m - n * hw;
        int ho = rem / g.Wo, wo = rem - ho * g.Wo;
        int sc = g.S * g.Cin;
        int r = k / sc, rem2 = k - r * sc;
        int s = rem2 / g.Cin, c = rem2 - s * g.Cin;
        int h = ho * g.stride + r - g.pad, w = wo * g.stride + s - g.pad;
        ok = (m < rows) && (k < K) && h >= 0 && h < g.H && w >= 0 && w < g.W;
        return (((int64_t)n * g.H + h) * g.W + w) * g.Cin + c;
    }
    __device__ __forceinline__ T at(int m, int k) const {
        bool ok;
        int64_t a = addr(m, k, ok);
        return ok ? x[a] : T(0.0f);
    }
    __device__ __forceinline__ uint4 load8(int m, int k) const {
        if (vec_ok) {
            bool ok;
            int64_t a = addr(m, k, ok);
            return ok ? *reinterpret_cast<const uint4*>(x + a) : make_uint4(0, 0, 0, 0);
        }
        Pack8 r;
#pragma unroll
        for (int i = 0; i < 8; ++i) r.h[i] = (bf16_t)at(m, k + i);
        return r.u;
    }
};

// Input-gradient A operand: row m = (n, h, w), k = (r, s, co) -> dy[n, (h+pad-r)/stride, (w+pad-s)/stride, co]
// where the divisions are exact and in range, else 0.
template <typename T> struct ConvDgradA {
    static constexpr bool kContig = true;
    const T* dy;
    ConvGeom g;
    int rows, K, vec_ok;  // vec_ok: Cout % 8 == 0 and base aligned
    __device__ __forceinline__ int64_t addr(int m, int k, bool& ok) const {
        int hw = g.H * g.W;
        int n = m / hw, rem = m - n * hw;
        int h = rem / g.W, w = rem - h * g.W;
        int sc = g.S * g.Cout;
        int r = k / sc, rem2 = k - r * sc;
        int s = rem2 / g.Cout, co = rem2 - s * g.Cout;
        int hy = h + g.pad - r, wy = w + g.pad - s;
        int ho = hy / g.stride, wo = wy / g.stride;
        ok = (m < rows) && (k < K) && hy >= 0 && wy >= 0 && ho * g.stride == hy &&
             wo * g.stride == wy && ho < g.Ho && wo < g.Wo;
        return (((int64_t)n * g.Ho + ho) * g.Wo + wo) * g.Cout + co;
    }
    __device__ __forceinline__ T at(int m, int k) const {
        bool ok;
        int64_t a = addr(m, k, ok);
        return ok ? dy[a] : T(0.0f);
    }
    __device__ __forceinline__ uint4 load8(int m, int k) const {
        if (vec_ok) {
            bool ok;
            int64_t a = addr(m, k, ok);
            return ok ? *reinterpret_cast<const uint4*>(dy + a) : make_uint4(0, 0, 0, 0);
        }
        Pack8 r;
#pragma unroll
        for (int i = 0; i < 8; ++i) r.h[i] = (bf16_t)at(m, k + i);
        return r.u;
    }
};

// Input-gradient B operand: row n = ci, k = (r, s, co) -> w[co, r, s, ci]  (rows contiguous).
template <typename T> struct ConvDgradB {
    static constexpr bool kContig = false;
    const T* w;
    ConvGeom g;
    int rows, K;
    __device__ __forceinline__ T at(int ci, int k) const {
        if (ci >= rows || k >= K) return T(0.0f);
        int sc = g.S * g.Cout;
        int r = k / sc, rem = k - r * sc;
        int s = rem / g.Cout, co = rem - s * g.Cout;
        return w[(((int64_t)co * g.R + r) * g.S + s) * g.Cin + ci];
    }
    __device__ __forceinline__ uint4 load8(int ci, int k) const {
        Pack8 r;
#pragma unroll
        for (int i = 0; i < 8; ++i) r.h[i] = (bf16_t)at(ci, k + i);
        return r.u;
    }
};

// Weight-gradient B operand: row = (r, s, ci), k = m = (n, ho, wo) -> x[n, ho*stride+r-pad, wo*stride+s-pad, ci].
template <typename T> struct ConvWgradB {
    static constexpr bool kContig = false;
    const T* x;
    ConvGeom g;
    int rows, K;
    __device__ __forceinline__ T at(int row, int m) const {
        if (row >= rows || m >= K) return T(0.0f);
        int sc = g.S * g.Cin;
        int r = row / sc, rem = row - r * sc;
        int s = rem / g.Cin, c = rem - s * g.Cin;
        int hw = g.Ho * g.Wo;
        int n = m / hw, rem2 = m - n * hw;
        int ho = rem2 / g.Wo, wo = rem2 - ho * g.Wo;
        int h = ho * g.stride + r - g.pad, w = wo * g.stride + s - g.pad;
        if (h < 0 || h >= g.H || w < 0 || w >= g.W) return T(0.0f);
        return x[(((int64_t)n * g.H + h) * g.W + w) * g.Cin + c];
    }
    __device__ __forceinline__ uint4 load8(int row, int m) const {
        Pack8 r;
#pragma unroll
        for (int i = 0; i < 8; ++i) r.h[i] = (bf16_t)at(row, m + i);
        return r.u;
    }
};

// ------------------------------------------------------------------------------------------
// Epilogues: called once per output element with the fp32 accumulator.  `z` is the split-K slice.
// ------------------------------------------------------------------------------------------

// Exact GELU z * Phi(z) and its derivative Phi(z) + z * phi(z), Phi(z) = (1 + erf(z / sqrt 2)) / 2.
// erf by the rational-times-Gaussian formula of Abramowitz & Stegun 7.1.26 (|error| < 1.5e-7, at the level of fp32
// rounding), with the hardware reciprocal and exp2: the library erff costs several dozen instructions per element,
// which made the GELU epilogues longer than the k-loops of the GEMMs they end.  E = exp(-z^2 / 2) serves both the
// erf and the density phi(z) = E / sqrt(2 pi).
__device__ __forceinline__ void gelu_parts(float z, float& Phi, float& E) {
    const float x = fabsf(z) * 0.70710678118654752f;
    const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, x, 1.0f));
    E = __expf(-x * x);
    float p = fmaf(1.061405429f, t, -1.453152027f);
    p = fmaf(p, t, 1.421413741f);
    p = fmaf(p, t, -0.284496736f);
    p = fmaf(p, t, 0.254829592f);
    const float er = 1.0f - p * t * E;             // erf(|z| / sqrt 2)
    Phi = 0.5f * (1.0f + copysignf(er, z));
}
__device__ __forceinline__ float gelu_f(float z) {
    float Phi, E;
    gelu_parts(z, Phi, E);
    return z * Phi;
}
__device__ __forceinline__ float gelu_grad_f(float z) {
    float Phi, E;
    gelu_parts(z, Phi, E);
    return Phi + z * 0.3989422804014327f * E;
}
// both at once: y = gelu(z), d = gelu'(z)
__device__ __forceinline__ void gelu_both(float z, float& y, float& d) {
    float Phi, E;
    gelu_parts(z, Phi, E);
    y = z * Phi;
    d = Phi + z * 0.3989422804014327f * E;
}

enum { kActNone = 0, kActRelu = 1, kActGelu = 2 };

// 8 consecutive elements with 16-byte accesses (the address is 16-byte aligned)
__device__ __forceinline__ void store8(bf16_t* p, const float (&v)[8]) {
    Pack8 pk;
#pragma unroll
    for (int e = 0; e < 8; ++e) pk.h[e] = (bf16_t)v[e];
    *reinterpret_cast<uint4*>(p) = pk.u;
}
__device__ __forceinline__ void store8(float* p, const float (&v)[8]) {
    *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
    *reinterpret_cast<float4*>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
}
__device__ __forceinline__ void load8(const bf16_t* p, float (&v)[8]) {
    Pack8 pk;
    pk.u = *reinterpret_cast<const uint4*>(p);
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = (float)pk.h[e];
}
__device__ __forceinline__ void load8(const float* p, float (&v)[8]) {
    const float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}

// 8 consecutive elements fetched now and converted later: the 8-wide epilogues request what they read from memory
// (a residual source, a mask, the gradient already collected) for several rows at once, BEFORE the results of those
// rows are ready, so that the memory latency is paid once per group of rows and not once per row.
template <typename T> struct Raw8;
template <> struct Raw8<bf16_t> {
    uint4 u;
    __device__ __forceinline__ void load(const bf16_t* p) { u = *reinterpret_cast<const uint4*>(p); }
    __device__ __forceinline__ void get(float (&v)[8]) const {
        Pack8 pk;
        pk.u = u;
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = (float)pk.h[e];
    }
};
template <> struct Raw8<float> {
    float4 a, b;
    __device__ __forceinline__ void load(const float* p) {
        a = *reinterpret_cast<const float4*>(p);
        b = *reinterpret_cast<const float4*>(p + 4);
    }
    __device__ __forceinline__ void get(float (&v)[8]) const {
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    }
};
struct NoCol8 {};
struct NoRow8 {};

// Host-side test for the 8-wide (16-byte) form of an epilogue: every tensor it touches is 16-byte aligned and a row
// start keeps that alignment.
static inline bool epi_al16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

// out[m, n] = act(v + bias[n]) + res[m, n].  With GELU the DERIVATIVE gelu'(v + bias[n]) is stored as well (zout): the
// backward pass then multiplies by a stored factor, as it does for ReLU, instead of evaluating an erf and an
// exponential per element in the epilogue of the input-gradient GEMM (where that cost more than the GEMM's k-loop).
// res: a residual connection's source, same shape as out.
template <typename TOut> struct EpiBiasAct {
    TOut* out;
    const float* bias;  // may be null
    int64_t ld;
    int relu;           // kActNone / kActRelu / kActGelu
    const TOut* res = nullptr;
    TOut* zout = nullptr;
    __device__ __forceinline__ void finish(int64_t idx, float v) const {
        if (relu == kActRelu) v = v > 0.0f ? v : 0.0f;
        else if (relu == kActGelu) {
            float d;
            gelu_both(v, v, d);
            if (zout) zout[idx] = from_f32<TOut>(d);
        }
        if (res) v += to_f32(res[idx]);
        out[idx] = from_f32<TOut>(v);
    }
    __device__ __forceinline__ void operator()(int m, int n, float v, int) const {
        if (bias) v += bias[n];
        finish((int64_t)m * ld + n, v);
    }
    bool wide_ok() const { return ld % 8 == 0 && epi_al16(out) && epi_al16(bias) && epi_al16(res) && epi_al16(zout); }
    // the same in two steps: column(n) fetches the bias once, at() finishes element idx = m*ld + n
    __device__ __forceinline__ float column(int n) const { return bias ? bias[n] : 0.0f; }
    __device__ __forceinline__ void at(float b, int64_t idx, float v, int) const { finish(idx, v + b); }
    // 8 consecutive columns n..n+7 of one row (n and idx multiples of 8; bias, res, zout, out 16-byte aligned)
    __device__ __forceinline__ void at8(int n, int64_t idx, float (&v)[8], int) const {
        if (bias) {
            float b[8];
            load8(bias + n, b);
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] += b[e];
        }
        if (relu == kActRelu) {
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = v[e] > 0.0f ? v[e] : 0.0f;
        } else if (relu == kActGelu) {
            float d[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) gelu_both(v[e], v[e], d[e]);
            if (zout) store8(zout + idx, d);
        }
        if (res) {
            float r[8];
            load8(res + idx, r);
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] += r[e];
        }
        store8(out + idx, v);
    }
    // the same with the column data (bias) and the row data (residual source) requested ahead of time
    struct Col8 { float b[8]; };
    struct Row8 { Raw8<TOut> r; };
    __device__ __forceinline__ Col8 col8(int n) const {
        Col8 c;
        if (bias) load8(bias + n, c.b);
        return c;
    }
    __device__ __forceinline__ Row8 row8(int64_t idx, bool ok) const {
        Row8 p;
        if (res && ok) p.r.load(res + idx);
        return p;
    }
    __device__ __forceinline__ void at8(const Col8& c, const Row8& p, int64_t idx, float (&v)[8], int) const {
        if (bias) {
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] += c.b[e];
        }
        if (relu == kActRelu) {
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = v[e] > 0.0f ? v[e] : 0.0f;
        } else if (relu == kActGelu) {
            float d[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) gelu_both(v[e], v[e], d[e]);
            if (zout) store8(zout + idx, d);
        }
        if (res) {
            float r[8];
            p.r.get(r);
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] += r[e];
        }
        store8(out + idx, v);
    }
    __device__ __forceinline__ void rowsum(int, float, int) const {}
};

// Convolution followed by a per-channel affine layer and, optionally, a residual join, in one epilogue:
//   z = v + bias[n]                        -> out   (the convolution's result, kept for the affine layer's gradient)
//   a = gain[n] * z + shift[n]             -> aout  (null when nothing reads it: the backward pass of the affine layer
//                                                    needs z, that of the join only y)
//   y = act(a + res[m, n])                 -> yout  (res may be null)
// Every stored tensor is rounded to its storage type before the next step reads it, exactly as if the three layers
// had run one after the other.
template <typename TOut> struct EpiConvAffine {
    TOut* out;
    const float* bias;   // may be null
    int64_t ld;
    const float* gain;
    const float* shift;
    TOut* aout;          // affine result; null when the affine layer itself writes yout, or when only the join reads it
    const TOut* res;     // second source of the residual join; may be null
    TOut* yout;
    int relu;
    struct Col { float b, g, s; };
    bool wide_ok() const {
        return ld % 8 == 0 && epi_al16(out) && epi_al16(bias) && epi_al16(gain) && epi_al16(shift) && epi_al16(aout) &&
               epi_al16(res) && epi_al16(yout);
    }
    __device__ __forceinline__ Col column(int n) const { return Col{bias ? bias[n] : 0.0f, gain[n], shift[n]}; }
    __device__ __forceinline__ void at(const Col& c, int64_t idx, float v, int) const {
        const TOut z = from_f32<TOut>(v + c.b);
        out[idx] = z;
        const TOut ar = from_f32<TOut>(c.g * to_f32(z) + c.s);   // rounded as the stored tensor would be, stored or not
        if (aout) aout[idx] = ar;
        float a = to_f32(ar);
        if (res) a += to_f32(res[idx]);
        if (relu) a = a > 0.0f ? a : 0.0f;
        yout[idx] = from_f32<TOut>(a);
    }
    // 8 consecutive columns n..n+7 of one row (n and idx multiples of 8; every tensor and vector 16-byte aligned)
    __device__ __forceinline__ void at8(int n, int64_t idx, float (&v)[8], int) const {
        float g[8], sh[8];
        load8(gain + n, g);
        load8(shift + n, sh);
        if (bias) {
            float b[8];
            load8(bias + n, b);
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] += b[e];
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = to_f32(from_f32<TOut>(v[e]));
        store8(out + idx, v);
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = g[e] * v[e] + sh[e];
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = to_f32(from_f32<TOut>(v[e]));   // rounded as the stored tensor would be
        if (aout) store8(aout + idx, v);
        if (res) {
            float r[8];
            load8(res + idx, r);
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] += r[e];
        }
        if (relu) {
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = v[e] > 0.0f ? v[e] : 0.0f;
        }
        store8(yout + idx, v);
    }
    struct Col8 { float b[8], g[8], s[8]; };
    struct Row8 { Raw8<TOut> r; };
    __device__ __forceinline__ Col8 col8(int n) const {
        Col8 c;
        load8(gain + n, c.g);
        load8(shift + n, c.s);
        if (bias) load8(bias + n, c.b);
        return c;
    }
    __device__ __forceinline__ Row8 row8(int64_t idx, bool ok) const {
        Row8 p;
        if (res && ok) p.r.load(res + idx);
        return p;
    }
    __device__ __forceinline__ void at8(const Col8& c, const Row8& p, int64_t idx, float (&v)[8], int) const {
        if (bias) {
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] += c.b[e];
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = to_f32(from_f32<TOut>(v[e]));
        store8(out + idx, v);
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = to_f32(from_f32<TOut>(c.g[e] * v[e] + c.s[e]));   // rounded as the stored tensor would be
        if (aout) store8(aout + idx, v);
        if (res) {
            float r[8];
            p.r.get(r);
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] += r[e];
        }
        if (relu) {
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = v[e] > 0.0f ? v[e] : 0.0f;
        }
        store8(yout + idx, v);
    }
    __device__ __forceinline__ void operator()(int m, int n, float v, int z) const { at(column(n), (int64_t)m * ld + n, v, z); }
    __device__ __forceinline__ void rowsum(int, float, int) const {}
};

// Gradient through the stored activation of the layer below: mode kActRelu: v where mask[m, n] > 0 else 0
// (mask = that layer's output); mode kActGelu: v * mask[m, n] (mask = the derivative stored by that layer's forward pass).
// add (may be null, may be out itself): what other readers of the same tensor have already contributed to its
// gradient; it joins v before the mask is applied.
template <typename TOut, typename TMask> struct EpiMask {
    TOut* out;
    const TMask* mask;  // may be null
    int64_t ld;
    int mode = kActRelu;
    const TOut* add = nullptr;
    __device__ __forceinline__ void finish(int64_t i, float v) const {
        if (add) v += to_f32(add[i]);
        if (mask) {
            const float t = to_f32(mask[i]);
            if (mode == kActGelu) v *= t;
            else if (!(t > 0.0f)) v = 0.0f;
        }
        out[i] = from_f32<TOut>(v);
    }
    __device__ __forceinline__ void operator()(int m, int n, float v, int) const { finish((int64_t)m * ld + n, v); }
    bool wide_ok() const { return ld % 8 == 0 && epi_al16(out) && epi_al16(mask) && epi_al16(add); }
    __device__ __forceinline__ int column(int) const { return 0; }
    __device__ __forceinline__ void at(int, int64_t i, float v, int) const { finish(i, v); }
    __device__ __forceinline__ void at8(int, int64_t i, float (&v)[8], int) const {
        if (add) {
            float a[8];
            load8(add + i, a);
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] += a[e];
        }
        if (mask) {
            float t[8];
            load8(mask + i, t);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                if (mode == kActGelu) v[e] *= t[e];
                else if (!(t[e] > 0.0f)) v[e] = 0.0f;
            }
        }
        store8(out + i, v);
    }
    typedef NoCol8 Col8;
    struct Row8 { Raw8<TOut> a; Raw8<TMask> t; };
    __device__ __forceinline__ Col8 col8(int) const { return Col8{}; }
    __device__ __forceinline__ Row8 row8(int64_t i, bool ok) const {
        Row8 p;
        if (add && ok) p.a.load(add + i);
        if (mask && ok) p.t.load(mask + i);
        return p;
    }
    __device__ __forceinline__ void at8(const Col8&, const Row8& p, int64_t i, float (&v)[8], int) const {
        if (add) {
            float a[8];
            p.a.get(a);
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] += a[e];
        }
        if (mask) {
            float t[8];
            p.t.get(t);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                if (mode == kActGelu) v[e] *= t[e];
                else if (!(t[e] > 0.0f)) v[e] = 0.0f;
            }
        }
        store8(out + i, v);
    }
    __device__ __forceinline__ void rowsum(int, float, int) const {}
};

// Weight gradient: fp32 [rows, cols] followed by the bias gradient [rows]; slice z writes its own
// copy at out + z*slice_stride (reduced afterwards), or the final location when there is one slice.
struct EpiWgrad {
    float* out;
    int64_t ld;            // cols
    int64_t bias_off;      // rows*cols
    int64_t slice_stride;  // rows*cols + rows
    __device__ __forceinline__ void operator()(int m, int n, float v, int z) const {
        out[z * slice_stride + (int64_t)m * ld + n] = v;
    }
    bool wide_ok() const { return ld % 8 == 0 && slice_stride % 4 == 0 && epi_al16(out); }
    __device__ __forceinline__ int column(int) const { return 0; }
    __device__ __forceinline__ void at(int, int64_t idx, float v, int z) const {
        out[z * slice_stride + idx] = v;
    }
    __device__ __forceinline__ void at8(int, int64_t idx, float (&v)[8], int z) const {
        store8(out + z * slice_stride + idx, v);
    }
    typedef NoCol8 Col8;
    typedef NoRow8 Row8;
    __device__ __forceinline__ Col8 col8(int) const { return Col8{}; }
    __device__ __forceinline__ Row8 row8(int64_t, bool) const { return Row8{}; }
    __device__ __forceinline__ void at8(const Col8&, const Row8&, int64_t idx, float (&v)[8], int z) const {
        store8(out + z * slice_stride + idx, v);
    }
    __device__ __forceinline__ void rowsum(int m, float v, int z) const {
        out[z * slice_stride + bias_off + m] = v;
    }
};

// ------------------------------------------------------------------------------------------
// bf16 MFMA GEMM.  256 threads = 4 waves in a 2x2 arrangement; wave tile (BM/2)x(BN/2) made of
// 32x32 MFMA tiles; BK = 32; LDS double-buffered; next tile's global loads are in flight while
// the current one is multiplied.  ROWSUM: blocks of the first column of tiles also sum A over k
// (the bias gradient of a weight-gradient GEMM, whose A operand is dY transposed).
// ------------------------------------------------------------------------------------------
constexpr int kBK = 32;
constexpr int kLdsLd = kBK + 8;  // bf16 elements per LDS row: 80 bytes, keeps 16-byte reads conflict-free

template <int BM, int BN, bool ROWSUM, class AOp, class BOp, class Epi>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(AOp A, BOp B, Epi epi, int M, int N, int K,
                                                        int k_per_slice) {
    constexpr int TM = BM / 64, TN = BN / 64;  // 32x32 tiles per wave along m and n
    __shared__ __attribute__((aligned(16))) bf16_t sA[2][BM * kLdsLd];
    __shared__ __attribute__((aligned(16))) bf16_t sB[2][BN * kLdsLd];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    const int z = blockIdx.z;
    const int k_begin = z * k_per_slice;
    const int k_end = min(K, k_begin + k_per_slice);
    const int nk = (k_end - k_begin + kBK - 1) / kBK;

    constexpr int A_CH = BM * (kBK / 8) / 256;  // 16-byte chunks per thread
    constexpr int B_CH = BN * (kBK / 8) / 256;
    uint4 ra[A_CH], rb[B_CH];

    // The views zero-fill beyond K, but a slice must not read past its own k range.
    auto gload = [&](int kt) {
        const int kb = k_begin + kt * kBK;
#pragma unroll
        for (int i = 0; i < A_CH; ++i) {
            int c = tid + i * 256;
            int row = AOp::kContig ? (c >> 2) : (c % BM);
            int kc = AOp::kContig ? (c & 3) : (c / BM);
            int k = kb + kc * 8;
            if (k + 8 <= k_end) ra[i] = A.load8(m0 + row, k);
            else {
                Pack8 t;
#pragma unroll
                for (int e = 0; e < 8; ++e) t.h[e] = (k + e < k_end) ? (bf16_t)A.at(m0 + row, k + e) : (bf16_t)0.0f;
                ra[i] = t.u;
            }
        }
#pragma unroll
        for (int i = 0; i < B_CH; ++i) {
            int c = tid + i * 256;
            int row = BOp::kContig ? (c >> 2) : (c % BN);
            int kc = BOp::kContig ? (c & 3) : (c / BN);
            int k = kb + kc * 8;
            if (k + 8 <= k_end) rb[i] = B.load8(n0 + row, k);
            else {
                Pack8 t;
#pragma unroll
                for (int e = 0; e < 8; ++e) t.h[e] = (k + e < k_end) ? (bf16_t)B.at(n0 + row, k + e) : (bf16_t)0.0f;
                rb[i] = t.u;
            }
        }
    };
    auto lstore = [&](int buf) {
#pragma unroll
        for (int i = 0; i < A_CH; ++i) {
            int c = tid + i * 256;
            int row = AOp::kContig ? (c >> 2) : (c % BM);
            int kc = AOp::kContig ? (c & 3) : (c / BM);
            *reinterpret_cast<uint4*>(&sA[buf][row * kLdsLd + kc * 8]) = ra[i];
        }
#pragma unroll
        for (int i = 0; i < B_CH; ++i) {
            int c = tid + i * 256;
            int row = BOp::kContig ? (c >> 2) : (c % BN);
            int kc = BOp::kContig ? (c & 3) : (c / BN);
            *reinterpret_cast<uint4*>(&sB[buf][row * kLdsLd + kc * 8]) = rb[i];
        }
    };

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
    float rsum = 0.0f;

    if (nk > 0) {
        gload(0);
        lstore(0);
    }
    __syncthreads();

    const int frag_row = lane & 31;
    const int frag_k = (lane >> 5) * 8;
    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < nk) gload(kt + 1);
#pragma unroll
        for (int kk = 0; kk < kBK / 16; ++kk) {
            bf16x8_t af[TM], bfr[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                af[i] = *reinterpret_cast<const bf16x8_t*>(
                    &sA[buf][(wm * (BM / 2) + i * 32 + frag_row) * kLdsLd + kk * 16 + frag_k]);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                bfr[j] = *reinterpret_cast<const bf16x8_t*>(
                    &sB[buf][(wn * (BN / 2) + j * 32 + frag_row) * kLdsLd + kk * 16 + frag_k]);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
        }
        if (ROWSUM && blockIdx.x == 0 && tid < BM) {
            const bf16_t* rowp = &sA[buf][tid * kLdsLd];
#pragma unroll
            for (int e = 0; e < kBK; ++e) rsum += (float)rowp[e];
        }
        if (kt + 1 < nk) lstore(buf ^ 1);
        __syncthreads();
    }

    // Accumulator layout of the 32x32 MFMA: lane holds column (lane % 32); register r holds
    // row 8*(r/4) + 4*(lane/32) + r%4.
    const int col_in = lane & 31;
    const int row_in = (lane >> 5) * 4;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            int n = n0 + wn * (BN / 2) + j * 32 + col_in;
            if (n >= N) continue;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                int m = m0 + wm * (BM / 2) + i * 32 + 8 * (r >> 2) + row_in + (r & 3);
                if (m < M) epi(m, n, acc[i][j][r], z);
            }
        }
    if (ROWSUM && blockIdx.x == 0 && tid < BM && m0 + tid < M) epi.rowsum(m0 + tid, rsum, z);
}

// ------------------------------------------------------------------------------------------
// fp32 GEMM (TMPS_F32 stages): 64x64 tile, BK = 16, 256 threads, 4x4 outputs per thread.
// ------------------------------------------------------------------------------------------
template <bool ROWSUM, class AOp, class BOp, class Epi>
__global__ __launch_bounds__(256) void gemm_f32_kernel(AOp A, BOp B, Epi epi, int M, int N, int K,
                                                       int k_per_slice) {
    constexpr int BT = 64, BKF = 16;
    __shared__ float sA[BKF][BT + 4];
    __shared__ float sB[BKF][BT + 4];
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int m0 = blockIdx.y * BT, n0 = blockIdx.x * BT;
    const int z = blockIdx.z;
    const int k_begin = z * k_per_slice;
    const int k_end = min(K, k_begin + k_per_slice);
    float acc[4][4] = {};
    float rsum = 0.0f;
    for (int kb = k_begin; kb < k_end; kb += BKF) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int e = tid + i * 256;
            int row = AOp::kContig ? (e >> 4) : (e & 63);
            int k = AOp::kContig ? (e & 15) : (e >> 6);
            sA[k][row] = (kb + k < k_end) ? to_f32(A.at(m0 + row, kb + k)) : 0.0f;
            row = BOp::kContig ? (e >> 4) : (e & 63);
            k = BOp::kContig ? (e & 15) : (e >> 6);
            sB[k][row] = (kb + k < k_end) ? to_f32(B.at(n0 + row, kb + k)) : 0.0f;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < BKF; ++k) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = sA[k][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = sB[k][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        if (ROWSUM && blockIdx.x == 0 && tid < BT) {
#pragma unroll
            for (int k = 0; k < BKF; ++k) rsum += sA[k][tid];
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int m = m0 + ty * 4 + i;
        if (m >= M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int n = n0 + tx * 4 + j;
            if (n < N) epi(m, n, acc[i][j], z);
        }
    }
    if (ROWSUM && blockIdx.x == 0 && tid < BT && m0 + tid < M) epi.rowsum(m0 + tid, rsum, z);
}

}  // namespace tmps
