// Launchers of the contraction kernels: dense and convolution forward, input gradient and
// weight gradient, in bf16 (MFMA) and fp32.
#include "gemm.hip.h"
#include "kernels.h"

namespace tmps {

static inline int cdiv(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }
static inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

int wgrad_slices(int rows, int cols, int64_t K) {
    int64_t tiles = (int64_t)cdiv(rows, 128) * cdiv(cols, 128);
    if (tiles >= 256 || K <= 512) return 1;
    int64_t want = (512 + tiles - 1) / tiles;
    int64_t by_k = K / 256;
    int64_t by_ws = (int64_t(64) << 20) / (((int64_t)rows * cols + rows) * 4);
    int64_t s = want;
    if (s > by_k) s = by_k;
    if (s > by_ws) s = by_ws;
    if (s > 128) s = 128;
    if (s < 1) s = 1;
    return (int)s;  // upper bound: rounding the slice length up to whole k-tiles can only lower it
}

size_t wgrad_workspace_elems(int rows, int cols, int64_t K) {
    int s = wgrad_slices(rows, cols, K);
    return s <= 1 ? 0 : (size_t)s * ((size_t)rows * cols + rows);
}

__global__ void slice_sum_kernel(const float* __restrict__ part, float* __restrict__ out, int64_t count,
                                 int slices) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= count) return;
    float a = 0.0f;
    for (int z = 0; z < slices; ++z) a += part[(int64_t)z * count + i];
    out[i] = a;
}

template <bool ROWSUM, class AOp, class BOp, class Epi>
static hipError_t launch_bf16(const AOp& A, const BOp& B, const Epi& epi, int M, int N, int K, int slices,
                              hipStream_t s) {
    if (M <= 0 || N <= 0) return hipSuccess;
    int per = cdiv(cdiv(K, slices), kBK) * kBK;
    if (per < kBK) per = kBK;
    int nz = K > 0 ? cdiv(K, per) : 1;
    int64_t tiles128 = (int64_t)cdiv(M, 128) * cdiv(N, 128) * nz;
    if (tiles128 >= 192) {
        dim3 grid(cdiv(N, 128), cdiv(M, 128), nz);
        hipLaunchKernelGGL((gemm_bf16_kernel<128, 128, ROWSUM, AOp, BOp, Epi>), grid, dim3(256), 0, s, A, B,
                           epi, M, N, K, per);
    } else {
        dim3 grid(cdiv(N, 64), cdiv(M, 64), nz);
        hipLaunchKernelGGL((gemm_bf16_kernel<64, 64, ROWSUM, AOp, BOp, Epi>), grid, dim3(256), 0, s, A, B, epi,
                           M, N, K, per);
    }
    return hipGetLastError();
}

template <bool ROWSUM, class AOp, class BOp, class Epi>
static hipError_t launch_f32(const AOp& A, const BOp& B, const Epi& epi, int M, int N, int K, int slices,
                             hipStream_t s) {
    if (M <= 0 || N <= 0) return hipSuccess;
    int per = cdiv(cdiv(K, slices), 16) * 16;
    if (per < 16) per = 16;
    int nz = K > 0 ? cdiv(K, per) : 1;
    dim3 grid(cdiv(N, 64), cdiv(M, 64), nz);
    hipLaunchKernelGGL((gemm_f32_kernel<ROWSUM, AOp, BOp, Epi>), grid, dim3(256), 0, s, A, B, epi, M, N, K,
                       per);
    return hipGetLastError();
}

// Number of slices the launchers will really use for a requested count (slice length is rounded up
// to whole k-tiles, which can shrink the count).
static int real_slices(int64_t K, int slices, int ktile) {
    int per = cdiv(cdiv(K, slices), ktile) * ktile;
    if (per < ktile) per = ktile;
    return K > 0 ? cdiv(K, per) : 1;
}

template <typename T, class AOp, class BOp>
static hipError_t wgrad_common(const AOp& A, const BOp& B, float* gw, int rows, int cols, int64_t K,
                               float* workspace, hipStream_t s) {
    int slices = wgrad_slices(rows, cols, K);
    constexpr int ktile = sizeof(T) == 2 ? kBK : 16;
    slices = real_slices(K, slices, ktile);
    int64_t count = (int64_t)rows * cols + rows;
    EpiWgrad epi{slices > 1 ? workspace : gw, cols, (int64_t)rows * cols, count};
    if (slices > 1 && workspace == nullptr) return hipErrorInvalidValue;
    hipError_t e;
    if constexpr (sizeof(T) == 2)
        e = launch_bf16<true>(A, B, epi, rows, cols, (int)K, slices, s);
    else
        e = launch_f32<true>(A, B, epi, rows, cols, (int)K, slices, s);
    if (e != hipSuccess) return e;
    if (slices > 1) {
        hipLaunchKernelGGL(slice_sum_kernel, dim3(cdiv(count, 256)), dim3(256), 0, s, workspace, gw, count,
                           slices);
        e = hipGetLastError();
    }
    return e;
}

// ---------------------------------------------------------------------------------------- dense
hipError_t dense_forward(int dtype, const void* x, const void* w, const float* bias, void* y, int B, int Din,
                         int Dout, int relu, int out_f32, hipStream_t s) {
    if (dtype == kBF16) {
        int vec = (Din % 8 == 0) && aligned16(x) && aligned16(w);
        DenseView<bf16_t, true> A{(const bf16_t*)x, B, Din, Din, vec};
        DenseView<bf16_t, true> Bv{(const bf16_t*)w, Dout, Din, Din, vec};
        if (out_f32) {
            EpiBiasAct<float> epi{(float*)y, bias, Dout, relu};
            return launch_bf16<false>(A, Bv, epi, B, Dout, Din, 1, s);
        }
        EpiBiasAct<bf16_t> epi{(bf16_t*)y, bias, Dout, relu};
        return launch_bf16<false>(A, Bv, epi, B, Dout, Din, 1, s);
    }
    DenseView<float, true> A{(const float*)x, B, Din, Din, 0};
    DenseView<float, true> Bv{(const float*)w, Dout, Din, Din, 0};
    EpiBiasAct<float> epi{(float*)y, bias, Dout, relu};
    return launch_f32<false>(A, Bv, epi, B, Dout, Din, 1, s);
}

hipError_t dense_dgrad(int dtype, const void* dy, const void* w, void* dx, const void* mask, int B, int Din,
                       int Dout, hipStream_t s) {
    // dx[m, n] = sum_k dy[m, k] * w[k, n]:  A = dy (k-contiguous), B(n, k) = w[k*Din + n] (row-contiguous)
    if (dtype == kBF16) {
        int vec = (Dout % 8 == 0) && aligned16(dy);
        DenseView<bf16_t, true> A{(const bf16_t*)dy, B, Dout, Dout, vec};
        DenseView<bf16_t, false> Bv{(const bf16_t*)w, Din, Dout, Din, 0};
        EpiMask<bf16_t, bf16_t> epi{(bf16_t*)dx, (const bf16_t*)mask, Din};
        return launch_bf16<false>(A, Bv, epi, B, Din, Dout, 1, s);
    }
    DenseView<float, true> A{(const float*)dy, B, Dout, Dout, 0};
    DenseView<float, false> Bv{(const float*)w, Din, Dout, Din, 0};
    EpiMask<float, float> epi{(float*)dx, (const float*)mask, Din};
    return launch_f32<false>(A, Bv, epi, B, Din, Dout, 1, s);
}

hipError_t dense_wgrad(int dtype, const void* dy, const void* x, float* gw, int B, int Din, int Dout,
                       float* workspace, hipStream_t s) {
    // gw[m, n] = sum_k dy[k, m] * x[k, n]: both operands row-contiguous, contraction over the batch
    if (dtype == kBF16) {
        DenseView<bf16_t, false> A{(const bf16_t*)dy, Dout, B, Dout, 0};
        DenseView<bf16_t, false> Bv{(const bf16_t*)x, Din, B, Din, 0};
        return wgrad_common<bf16_t>(A, Bv, gw, Dout, Din, B, workspace, s);
    }
    DenseView<float, false> A{(const float*)dy, Dout, B, Dout, 0};
    DenseView<float, false> Bv{(const float*)x, Din, B, Din, 0};
    return wgrad_common<float>(A, Bv, gw, Dout, Din, B, workspace, s);
}

// ---------------------------------------------------------------------------------- convolution
static ConvGeom geom(const ConvShape& c) {
    return ConvGeom{c.B, c.H, c.W, c.Cin, c.Ho, c.Wo, c.Cout, c.R, c.S, c.stride, c.pad};
}

hipError_t conv_forward(int dtype, const void* x, const void* w, const float* bias, void* y,
                        const ConvShape& c, int relu, hipStream_t s) {
    int M = c.B * c.Ho * c.Wo, K = c.R * c.S * c.Cin;
    if (dtype == kBF16) {
        ConvFwdA<bf16_t> A{(const bf16_t*)x, geom(c), M, K, (c.Cin % 8 == 0) && aligned16(x)};
        DenseView<bf16_t, true> Bv{(const bf16_t*)w, c.Cout, K, K, (K % 8 == 0) && aligned16(w)};
        EpiBiasAct<bf16_t> epi{(bf16_t*)y, bias, c.Cout, relu};
        return launch_bf16<false>(A, Bv, epi, M, c.Cout, K, 1, s);
    }
    ConvFwdA<float> A{(const float*)x, geom(c), M, K, 0};
    DenseView<float, true> Bv{(const float*)w, c.Cout, K, K, 0};
    EpiBiasAct<float> epi{(float*)y, bias, c.Cout, relu};
    return launch_f32<false>(A, Bv, epi, M, c.Cout, K, 1, s);
}

hipError_t conv_dgrad(int dtype, const void* dy, const void* w, void* dx, const void* mask,
                      const ConvShape& c, hipStream_t s) {
    int M = c.B * c.H * c.W, K = c.R * c.S * c.Cout;
    if (dtype == kBF16) {
        ConvDgradA<bf16_t> A{(const bf16_t*)dy, geom(c), M, K, (c.Cout % 8 == 0) && aligned16(dy)};
        ConvDgradB<bf16_t> Bv{(const bf16_t*)w, geom(c), c.Cin, K};
        EpiMask<bf16_t, bf16_t> epi{(bf16_t*)dx, (const bf16_t*)mask, c.Cin};
        return launch_bf16<false>(A, Bv, epi, M, c.Cin, K, 1, s);
    }
    ConvDgradA<float> A{(const float*)dy, geom(c), M, K, 0};
    ConvDgradB<float> Bv{(const float*)w, geom(c), c.Cin, K};
    EpiMask<float, float> epi{(float*)dx, (const float*)mask, c.Cin};
    return launch_f32<false>(A, Bv, epi, M, c.Cin, K, 1, s);
}

hipError_t conv_wgrad(int dtype, const void* dy, const void* x, float* gw, const ConvShape& c,
                      float* workspace, hipStream_t s) {
    int rows = c.Cout, cols = c.R * c.S * c.Cin;
    int64_t K = (int64_t)c.B * c.Ho * c.Wo;
    if (dtype == kBF16) {
        DenseView<bf16_t, false> A{(const bf16_t*)dy, rows, (int)K, c.Cout, 0};
        ConvWgradB<bf16_t> Bv{(const bf16_t*)x, geom(c), cols, (int)K};
        return wgrad_common<bf16_t>(A, Bv, gw, rows, cols, K, workspace, s);
    }
    DenseView<float, false> A{(const float*)dy, rows, (int)K, c.Cout, 0};
    ConvWgradB<float> Bv{(const float*)x, geom(c), cols, (int)K};
    return wgrad_common<float>(A, Bv, gw, rows, cols, K, workspace, s);
}

}  // namespace tmps
