// Launchers of the contraction kernels: dense and convolution forward, input gradient and weight
// gradient.  bf16 stages use the MFMA skeleton of gemm2.hip.h whenever every operand can be fetched
// with aligned 16-byte loads (channel / feature counts that are multiples of 8), and the
// element-wise skeleton of gemm.hip.h otherwise (3-channel input layer, 10-way logits layer);
// fp32 stages use the fp32 skeleton.
#include <cstdlib>
#include <hip/hip_ext.h>

#include "gemm3.hip.h"
#include "kernels.h"
#include "launch.h"
#include "profile.h"

namespace tmps {

static inline int cdiv(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }
static inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

// ------------------------------------------------------------------------------------------
// Tile size and k-split of a [M x N x K] contraction.  Small outputs are split along k until the grid
// has a few hundred workgroups, as long as the fp32 partial sums do not outweigh the operands.
// ------------------------------------------------------------------------------------------
GemmPlan plan_gemm(int64_t M, int64_t N, int64_t K) {
    GemmPlan p;
    const int64_t t128 = (int64_t)cdiv(M, 128) * cdiv(N, 128);
    const int64_t t64 = (int64_t)cdiv(M, 64) * cdiv(N, 64);
    const bool wide = N > 64 && M > 64;
    // An output with fewer 128-tiles than compute units and a contraction that is not long is latency-bound: more,
    // smaller workgroups finish sooner (measured on 1024-row transformer GEMMs: 13 us against 16 us; a row limit of
    // 2048 that used to stand here cost ResNet-50 1.6 % and VGG-16 2.8 % per step).
    const bool short_rows = t128 < 256 && K <= 4096;
    // (a long contraction is cut into slices anyway: then a dozen 128-tiles suffice to fill the device)
    // 128 x 128 tiles for outputs of 512 such tiles or more, for 64 or more with a contraction of 2048 or longer, and
    // for a dozen with a very long one; in between, the smaller tiles (128 x 64 for tall outputs) do better with
    // the stages' kernels sharing the device (swept on the ResNet-50, VGG-16 and GPT-2 workloads: a short contraction
    // is mostly epilogue, which the smaller tiles spread over more workgroups)
    p.tile = (wide && !short_rows && (t128 >= 512 || (t128 >= 64 && K >= 2048) || (K > 4096 && t128 >= 8))) ? 128 : 64;
    const int64_t tiles = p.tile == 128 ? t128 : t64;
    const int64_t target = 384;  // swept 32..2048 on the VGG workload: flat optimum around 384-512
    int64_t s = 1;
    // (short outputs with 64 tiles or more and a short contraction are not split: the finishing kernel costs
    // more than the split saves; swept 1..256)
    if (tiles < target && !(short_rows && tiles >= 64)) {
        s = (target + tiles - 1) / tiles;
        const int64_t by_k = K / 128;
        const int64_t by_bytes = ((M + N) * K) / (2 * M * N);
        if (s > by_k) s = by_k;
        if (s > by_bytes) s = by_bytes;
        if (s > 64) s = 64;
        if (s < 1) s = 1;
    }
    p.slices = (int)s;
    return p;
}

static int g3_wgrad_slices(int64_t M, int64_t N, int64_t K);
static int g3_long_k_slices(int64_t M, int64_t N, int64_t K);

size_t gemm_workspace_elems(int64_t M, int64_t N, int64_t K, int with_rowsum) {
    GemmPlan p = plan_gemm(M, N, K);
    int slices = p.slices;
    if (with_rowsum) {   // a weight gradient may go to the persistent path, with its own number of slices
        const int s3 = g3_wgrad_slices(M, N, K);
        if (s3 > slices) slices = s3;
    } else {             // and so may an input gradient with a very long contraction
        const int s3 = g3_long_k_slices(M, N, K);
        if (s3 > slices) slices = s3;
    }
    if (slices <= 1) return 0;
    return (size_t)(slices + 1) * ((size_t)M * N + (with_rowsum ? (size_t)M : 0));
}

__global__ void slice_sum_kernel(const float* __restrict__ part, float* __restrict__ out, int64_t count,
                                 int slices) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= count) return;
    // eight loads in flight per thread, added in slice order
    const float* p = part + i;
    float a = 0.0f;
    int z = 0;
    for (; z + 8 <= slices; z += 8) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = p[u * count];
#pragma unroll
        for (int u = 0; u < 8; ++u) a += v[u];
        p += 8 * count;
    }
    for (; z < slices; ++z) {
        a += *p;
        p += count;
    }
    out[i] = a;
}

// The same for 4 consecutive elements per thread (count a multiple of 4, both arrays 16-byte aligned).
__global__ __launch_bounds__(256) void slice_sum4_kernel(const float* __restrict__ part, float* __restrict__ out, int64_t count,
                                                         int slices) {
    const int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (i >= count) return;
    const float* p = part + i;
    float4 a = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    int z = 0;
    for (; z + 8 <= slices; z += 8) {
        float4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = *reinterpret_cast<const float4*>(p + u * count);
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            a.x += v[u].x; a.y += v[u].y; a.z += v[u].z; a.w += v[u].w;
        }
        p += 8 * count;
    }
    for (; z < slices; ++z) {
        const float4 v = *reinterpret_cast<const float4*>(p);
        a.x += v.x; a.y += v.y; a.z += v.z; a.w += v.w;
        p += count;
    }
    *reinterpret_cast<float4*>(out + i) = a;
}

static hipError_t slice_sum(const float* part, float* out, int64_t count, int slices, hipStream_t s) {
    if (count % 4 == 0 && aligned16(part) && aligned16(out))
        return launch_timed(kcSliceSum, slice_sum4_kernel, dim3(cdiv(count / 4, 256)), dim3(256), 0, s, part, out, count, slices);
    return launch_timed(kcSliceSum, slice_sum_kernel, dim3(cdiv(count, 256)), dim3(256), 0, s, part, out, count, slices);
}

// slice length (whole k-tiles) and the number of slices really launched
static void slice_geometry(int64_t K, int want, int ktile, int& per, int& nz) {
    if (want < 1) want = 1;
    per = cdiv(cdiv(K, want), ktile) * ktile;
    if (per < ktile) per = ktile;
    nz = K > 0 ? cdiv(K, per) : 1;
}

// ---- MFMA path --------------------------------------------------------------------------------
template <int BM, int BN, int D, bool ROWSUM, class AOp, class BOp, class Epi>
static hipError_t launch2_inst(int kc, const AOp& A, const BOp& B, const Epi& epi, int M, int N, int K, int per,
                               int nz, hipStream_t s) {
    constexpr int lds = gemm2_lds_bytes<BM, BN, AOp, BOp>();
    auto kern = gemm2_kernel<BM, BN, D, ROWSUM, AOp, BOp, Epi>;
    if (lds > 64 * 1024) {
        // more LDS than the default per-workgroup limit: raise it once per kernel instance
        static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (attr != hipSuccess) return attr;
    }
    dim3 grid(cdiv(N, BN), cdiv(M, BM), nz);
    // the XCDs split the operand with more rows between them and each reads the other one whole
    const int col_major = N > M ? 1 : 0;
    return launch_timed(kc, kern, grid, dim3(256), lds, s, A, B, epi, M, N, K, per, col_major,
                        (N % 8 == 0 && epi.wide_ok()) ? 1 : 0, FastDiv(grid.x * grid.y), FastDiv(col_major ? grid.y : grid.x));
}

// tile: the plan's tile edge.  Where it is 64, the output has 512 rows or more and 128 x 64 tiles still make 192
// workgroups, the tiles are 128 rows tall unless the caller needs them square (`square`): a 128 x 64 tile reads a
// quarter less LDS per MFMA than a 64 x 64 one, and with the stages' kernels sharing the device that outweighs
// having half as many workgroups (measured: GPT-2 and ResNet-50 steps 1 % shorter, VGG-16 1-2 %; 128 x 128 and
// 64 x 128 for the same launches did worse; below 192 workgroups the launch itself gets slower and the step no faster).
template <bool ROWSUM, class AOp, class BOp, class Epi>
static hipError_t launch2_tile(int kc, int tile, bool square, const AOp& A, const BOp& B, const Epi& epi, int M, int N,
                               int K, int per, int nz, hipStream_t s) {
    if (tile == 128) return launch2_inst<128, 128, 2, ROWSUM>(kc, A, B, epi, M, N, K, per, nz, s);
    if constexpr (!ROWSUM) {
        if (!square && M >= 512 && (int64_t)cdiv(M, 128) * cdiv(N, 64) * nz >= 192)
            return launch2_inst<128, 64, 2, false>(kc, A, B, epi, M, N, K, per, nz, s);
    }
    return launch2_inst<64, 64, 4, ROWSUM>(kc, A, B, epi, M, N, K, per, nz, s);
}

// Forward / input-gradient style GEMM: epilogue `epi` applied once per output element.
// tile: 0 = the plan's choice, else the edge of the square tiles to use (the slices stay the plan's)
template <class AOp, class BOp, class Epi>
static hipError_t run2(int kc, const AOp& A, const BOp& B, const Epi& epi, int M, int N, int K, float* ws,
                       hipStream_t s, int tile = 0) {
    if (M <= 0 || N <= 0) return hipSuccess;
    GemmPlan p = plan_gemm(M, N, K);
    if (tile) p.tile = tile;
    int per, nz;
    slice_geometry(K, ws ? p.slices : 1, kBK2, per, nz);
    if (nz <= 1) return launch2_tile<false>(kc, p.tile, tile != 0, A, B, epi, M, N, K, per, nz, s);
    EpiPartial part{ws, N, (int64_t)M * N};
    hipError_t e = launch2_tile<false>(kc, p.tile, tile != 0, A, B, part, M, N, K, per, nz, s);
    if (e != hipSuccess) return e;
    int64_t total = (int64_t)M * N;
    if (N % 8 == 0 && epi.wide_ok() && aligned16(ws))
        return launch_timed(kcSplitFinish, splitk_finish8_kernel<Epi>, dim3(cdiv(total / 8, 256)), dim3(256), 0, s,
                            (const float*)ws, epi, M, N, nz);
    return launch_timed(kcSplitFinish, splitk_finish_kernel<Epi>, dim3(cdiv(total, 256)), dim3(256), 0, s,
                        (const float*)ws, epi, M, N, nz);
}

// Weight-gradient style GEMM: fp32 result [rows x cols] followed by the row sums of A (bias gradient).
template <class AOp, class BOp>
static hipError_t run2_wgrad(int kc, const AOp& A, const BOp& B, float* gw, int rows, int cols, int64_t K,
                             float* ws, hipStream_t s) {
    GemmPlan p = plan_gemm(rows, cols, K);
    int per, nz;
    slice_geometry(K, ws ? p.slices : 1, kBK2, per, nz);
    int64_t count = (int64_t)rows * cols + rows;
    EpiWgrad epi{nz > 1 ? ws : gw, cols, (int64_t)rows * cols, count};
    hipError_t e = launch2_tile<true>(kc, p.tile, true, A, B, epi, rows, cols, (int)K, per, nz, s);
    if (e != hipSuccess || nz <= 1) return e;
    return slice_sum((const float*)ws, gw, count, nz, s);
}

static int one_slice(int64_t K, int ktile) {
    int per = cdiv(K, ktile) * ktile;
    return per < ktile ? ktile : per;
}

// ---- persistent MFMA path (gemm3.hip.h): large dense contractions --------------------------------------
static int compute_units() {
    static int n = [] {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v < 1)
            v = 256;
        return v;
    }();
    return n;
}

constexpr int kG3Tile = 256;
static int64_t g3_tiles(int64_t M, int64_t N) { return (int64_t)cdiv(M, kG3Tile) * cdiv(N, kG3Tile); }
// k-slices of a weight-gradient contraction on the persistent path (0: leave it to the other path).  Measured:
// the path pays once a launch has about as many (tile, slice) units as the device has compute units.
static int g3_wgrad_slices(int64_t M, int64_t N, int64_t K) {
    if (K % 64 != 0 || M % 8 != 0 || N % 8 != 0) return 0;
    const int64_t tiles = g3_tiles(M, N);
    int64_t s = tiles >= 192 ? 1 : 256 / tiles;
    if (s > K / 1024) s = K / 1024;
    if (s < 1) s = 1;
    return tiles * s >= 200 ? (int)s : 0;   // (swept: 144..200 units are quicker on the other path, ResNet-50 step -1.7 %)
}
// Not for a contraction of a single k-tile, which is all epilogue (many small workgroups keep more memory requests in
// flight than one persistent workgroup per compute unit), nor when more than a quarter of the 256-wide tiles would be
// padding (measured on the 1x1 convolutions of the residual networks).
static bool g3_forward_ok(int64_t M, int64_t N, int64_t K) {
    return K % 64 == 0 && K >= 128 && N % 8 == 0 && g3_tiles(M, N) >= 192 && (int64_t)cdiv(N, 256) * 256 * 3 <= N * 4;
}

// A tall, narrow output (the 8192 x 768 input gradients of a transformer block: 96 tiles of 256 x 256, which leave most
// of the device idle) goes to the persistent kernel in 256 x 128 tiles with four waves of 128 x 64 each: at least half the
// compute units get a unit, none gets two, and a k-loop of at least 8 k-tiles carries the unit's prologue and epilogue.
// Measured against the 128 x 128 tiles of the other kernel (384 workgroups, two on half the compute units): 45 / 21 /
// 57 us against 52 / 23 / 67 for the contractions over 2304 / 768 / 3072.
static bool g3_narrow_ok(int64_t M, int64_t N, int64_t K) {
    if (K % 64 != 0 || K < 512 || N % 128 != 0) return false;
    const int64_t units = (int64_t)cdiv(M, 256) * (N / 128);
    return units >= compute_units() / 2 && units <= compute_units();
}

// An output of few 256-wide tiles with a very long contraction (the input gradient of a vocabulary-wide output layer:
// 96 tiles, k = 32000) goes to the persistent kernel in k-slices: the slice count is the one whose (tile, slice) units
// fill whole rounds of the device best, weighed against the fp32 partial sums it writes and the finishing pass reads
// (rates measured: 1 PFLOP/s in the k-loop, 5 TB/s for the partial sums).  0: leave it to the tiled kernel.
static int g3_long_k_slices(int64_t M, int64_t N, int64_t K) {
    if (K % 64 != 0 || N % 8 != 0 || K < 8192) return 0;
    const int64_t tiles = g3_tiles(M, N);
    if (tiles >= 192 || tiles < 32 || (int64_t)cdiv(N, 256) * 256 * 3 > N * 4) return 0;
    const int cus = compute_units();
    int best = 0;
    double best_us = 0.0;
    for (int sl = 2; sl <= 16; ++sl) {
        if (K / sl < 2048) break;
        const int64_t units = tiles * sl;
        const double fill = (double)units / (double)((units + cus - 1) / cus * cus);
        const double us = 2.0 * M * N * K / (fill * 1e9) + (double)sl * M * N * 8.0 / 5e6;
        if (best == 0 || us < best_us) {
            best = sl;
            best_us = us;
        }
    }
    return best;
}

static G3Plan g3_plan(int M, int N, int K, int slices, int bm = kG3Tile, int bn = kG3Tile) {
    G3Plan p;
    p.tiles_m = cdiv(M, bm);
    p.tiles_n = cdiv(N, bn);
    int per = cdiv(cdiv(K, slices), 64) * 64;
    p.k_per_slice = per;
    p.slices = cdiv(K, per);
    p.units = p.tiles_m * p.tiles_n * p.slices;
    p.col_major = N > M ? 1 : 0;   // the XCDs split the operand with more rows between them and each reads the other one whole
    p.d_tn = FastDiv(p.col_major ? p.tiles_m : p.tiles_n);
    p.d_tiles = FastDiv(p.tiles_m * p.tiles_n);
    // Blocks of 32 tiles for outputs wide enough that a run of 32 tiles would span few rows and all columns (or the
    // other way round): the squarest block whose sides divide the tile counts.
    p.gm = p.gn = 0;
    if (p.tiles_m >= 8 && p.tiles_n >= 8) {
        for (int gn : {4, 8, 2, 16}) {
            const int gm = 32 / gn;
            if (p.tiles_n % gn == 0 && p.tiles_m % gm == 0) {
                p.gm = gm;
                p.gn = gn;
                break;
            }
        }
    }
    if (p.gm) {
        p.d_blk = FastDiv(32);
        p.d_gn = FastDiv(p.gn);
        p.d_nbn = FastDiv(p.tiles_n / p.gn);
    }
    return p;
}

// 256 x 256 x 64 tiles, 8 waves (2 x 4), two LDS stages: the configuration that did best on every large shape tried.
template <int BM, int BN, int WM, int WN, int NS, int PER_CU, bool AKC, bool BKC, bool ROWSUM, class Epi>
static hipError_t launch3_inst(int kc, const G3Operand<AKC>& A, const G3Operand<BKC>& B, const Epi& epi, int M, int N, int K,
                               const G3Plan& plan, hipStream_t s) {
    constexpr int lds = gemm3_lds_bytes<BM, BN, 64, NS>();
    auto kern = gemm3_kernel<BM, BN, 64, WM, WN, NS, AKC, BKC, ROWSUM, Epi>;
    static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (attr != hipSuccess) return attr;
    const int slots = compute_units() * PER_CU;
    const int grid = plan.units < slots ? plan.units : slots;
    return launch_timed(kc, kern, dim3(grid), dim3(64 * WM * WN), lds, s, A, B, epi, M, N, K, plan);
}

template <bool AKC, bool BKC, bool ROWSUM, class Epi>
static hipError_t launch3(int kc, const G3Operand<AKC>& A, const G3Operand<BKC>& B, const Epi& epi, int M, int N, int K,
                          const G3Plan& plan, hipStream_t s) {
    return launch3_inst<256, 256, 2, 4, 2, 1, AKC, BKC, ROWSUM>(kc, A, B, epi, M, N, K, plan, s);
}

// ---- element-wise fallbacks ------------------------------------------------------------------
template <bool ROWSUM, class AOp, class BOp, class Epi>
static hipError_t launch_bf16(int kc, const AOp& A, const BOp& B, const Epi& epi, int M, int N, int K, int per,
                              int nz, hipStream_t s) {
    if (M <= 0 || N <= 0) return hipSuccess;
    dim3 grid(cdiv(N, 64), cdiv(M, 64), nz);
    return launch_timed(kc, gemm_bf16_kernel<64, 64, ROWSUM, AOp, BOp, Epi>, grid, dim3(256), 0, s, A, B, epi, M, N,
                        K, per);
}

template <bool ROWSUM, class AOp, class BOp, class Epi>
static hipError_t launch_f32(int kc, const AOp& A, const BOp& B, const Epi& epi, int M, int N, int K, int per,
                             int nz, hipStream_t s) {
    if (M <= 0 || N <= 0) return hipSuccess;
    dim3 grid(cdiv(N, 64), cdiv(M, 64), nz);
    return launch_timed(kc, gemm_f32_kernel<ROWSUM, AOp, BOp, Epi>, grid, dim3(256), 0, s, A, B, epi, M, N, K, per);
}

template <typename T, class AOp, class BOp>
static hipError_t wgrad_fallback(int kc, const AOp& A, const BOp& B, float* gw, int rows, int cols, int64_t K, float* ws,
                                 hipStream_t s) {
    GemmPlan p = plan_gemm(rows, cols, K);
    constexpr int ktile = sizeof(T) == 2 ? kBK : 16;
    int per, nz;
    slice_geometry(K, ws ? p.slices : 1, ktile, per, nz);
    int64_t count = (int64_t)rows * cols + rows;
    EpiWgrad epi{nz > 1 ? ws : gw, cols, (int64_t)rows * cols, count};
    hipError_t e;
    if constexpr (sizeof(T) == 2)
        e = launch_bf16<true>(kc, A, B, epi, rows, cols, (int)K, per, nz, s);
    else
        e = launch_f32<true>(kc, A, B, epi, rows, cols, (int)K, per, nz, s);
    if (e != hipSuccess || nz <= 1) return e;
    return slice_sum((const float*)ws, gw, count, nz, s);
}

// ---------------------------------------------------------------------------------------- dense
// The dense contractions with the kernel class they are accounted under as a parameter: a 1x1 convolution with unit
// stride and no padding is the same contraction over its positions.
static hipError_t dense_forward_as(int kc, int dtype, const void* x, const void* w, const float* bias, void* y, int B, int Din,
                                   int Dout, int relu, int out_f32, const void* res, void* zout, float* ws, hipStream_t s) {
    if (dtype == kBF16) {
        const bool fast = (Din % 8 == 0) && aligned16(x) && aligned16(w);
        if (fast && g3_forward_ok(B, Dout, Din) && aligned16(y) && aligned16(bias) && aligned16(res) && aligned16(zout)) {
            G3Operand<true> A{(const bf16_t*)x, B, Din};
            G3Operand<true> Bv{(const bf16_t*)w, Dout, Din};
            const G3Plan plan = g3_plan(B, Dout, Din, 1);
            if (out_f32) return launch3<true, true, false>(kc, A, Bv, EpiBiasAct<float>{(float*)y, bias, Dout, relu}, B, Dout, Din, plan, s);
            return launch3<true, true, false>(kc, A, Bv, EpiBiasAct<bf16_t>{(bf16_t*)y, bias, Dout, relu, (const bf16_t*)res, (bf16_t*)zout}, B, Dout, Din, plan, s);
        }
        if (fast) {
            DenseKC A{(const bf16_t*)x, B, Din, Din};
            DenseKC Bv{(const bf16_t*)w, Dout, Din, Din};
            if (out_f32) return run2(kc, A, Bv, EpiBiasAct<float>{(float*)y, bias, Dout, relu}, B, Dout, Din, ws, s);
            return run2(kc, A, Bv, EpiBiasAct<bf16_t>{(bf16_t*)y, bias, Dout, relu, (const bf16_t*)res, (bf16_t*)zout}, B, Dout, Din, ws, s);
        }
        DenseView<bf16_t, true> A{(const bf16_t*)x, B, Din, Din, 0};
        DenseView<bf16_t, true> Bv{(const bf16_t*)w, Dout, Din, Din, 0};
        if (out_f32) return launch_bf16<false>(kc, A, Bv, EpiBiasAct<float>{(float*)y, bias, Dout, relu}, B, Dout, Din, one_slice(Din, kBK), 1, s);
        return launch_bf16<false>(kc, A, Bv, EpiBiasAct<bf16_t>{(bf16_t*)y, bias, Dout, relu, (const bf16_t*)res, (bf16_t*)zout}, B, Dout, Din, one_slice(Din, kBK), 1, s);
    }
    DenseView<float, true> A{(const float*)x, B, Din, Din, 0};
    DenseView<float, true> Bv{(const float*)w, Dout, Din, Din, 0};
    return launch_f32<false>(kc, A, Bv, EpiBiasAct<float>{(float*)y, bias, Dout, relu, (const float*)res, (float*)zout}, B, Dout, Din, one_slice(Din, 16), 1, s);
}

hipError_t dense_forward(int dtype, const void* x, const void* w, const float* bias, void* y, int B, int Din,
                         int Dout, int relu, int out_f32, const void* res, void* zout, float* ws, hipStream_t s) {
    return dense_forward_as(tmps::kcDenseFwd, dtype, x, w, bias, y, B, Din, Dout, relu, out_f32, res, zout, ws, s);
}

static hipError_t dense_dgrad_as(int kc, int dtype, const void* dy, const void* w, void* dx, const void* mask, int mask_mode,
                                 const void* add, int B, int Din, int Dout, float* ws, hipStream_t s) {
    // dx[m, n] = sum_k dy[m, k] * w[k, n]:  A = dy (k-contiguous), B(n, k) = w[k*Din + n] (row-contiguous)
    if (dtype == kBF16) {
        EpiMask<bf16_t, bf16_t> epi{(bf16_t*)dx, (const bf16_t*)mask, Din, mask_mode, (const bf16_t*)add};
        const bool fast = (Dout % 8 == 0) && (Din % 8 == 0) && aligned16(dy) && aligned16(w);
        if (fast && g3_forward_ok(B, Din, Dout) && aligned16(dx) && aligned16(mask) && aligned16(add)) {
            G3Operand<true> A{(const bf16_t*)dy, B, Dout};
            G3Operand<false> Bv{(const bf16_t*)w, Din, Din};
            return launch3<true, false, false>(kc, A, Bv, epi, B, Din, Dout, g3_plan(B, Din, Dout, 1), s);
        }
        const int s3 = (fast && ws && aligned16(ws) && aligned16(dx) && aligned16(mask) && aligned16(add) && epi.wide_ok())
                           ? g3_long_k_slices(B, Din, Dout) : 0;
        if (s3 > 1) {
            G3Operand<true> A{(const bf16_t*)dy, B, Dout};
            G3Operand<false> Bv{(const bf16_t*)w, Din, Din};
            const G3Plan plan = g3_plan(B, Din, Dout, s3);
            EpiPartial part{ws, Din, (int64_t)B * Din};
            hipError_t e = launch3<true, false, false>(kc, A, Bv, part, B, Din, Dout, plan, s);
            if (e != hipSuccess) return e;
            return launch_timed(kcSplitFinish, splitk_finish8_kernel<EpiMask<bf16_t, bf16_t>>, dim3(cdiv((int64_t)B * Din / 8, 256)),
                                dim3(256), 0, s, (const float*)ws, epi, B, Din, plan.slices);
        }
        if (fast && g3_narrow_ok(B, Din, Dout) && aligned16(dx) && aligned16(mask) && aligned16(add)) {
            G3Operand<true> A{(const bf16_t*)dy, B, Dout};
            G3Operand<false> Bv{(const bf16_t*)w, Din, Din};
            return launch3_inst<256, 128, 2, 2, 2, 1, true, false, false>(kc, A, Bv, epi, B, Din, Dout, g3_plan(B, Din, Dout, 1, 256, 128), s);
        }
        if (fast) {
            DenseKC A{(const bf16_t*)dy, B, Dout, Dout};
            DenseRC Bv{(const bf16_t*)w, Din, Dout, Din};
            return run2(kc, A, Bv, epi, B, Din, Dout, ws, s);
        }
        DenseView<bf16_t, true> A{(const bf16_t*)dy, B, Dout, Dout, 0};
        DenseView<bf16_t, false> Bv{(const bf16_t*)w, Din, Dout, Din, 0};
        return launch_bf16<false>(kc, A, Bv, epi, B, Din, Dout, one_slice(Dout, kBK), 1, s);
    }
    DenseView<float, true> A{(const float*)dy, B, Dout, Dout, 0};
    DenseView<float, false> Bv{(const float*)w, Din, Dout, Din, 0};
    return launch_f32<false>(kc, A, Bv, EpiMask<float, float>{(float*)dx, (const float*)mask, Din, mask_mode, (const float*)add}, B, Din, Dout, one_slice(Dout, 16), 1, s);
}

hipError_t dense_dgrad(int dtype, const void* dy, const void* w, void* dx, const void* mask, int mask_mode,
                       const void* add, int B, int Din, int Dout, float* ws, hipStream_t s) {
    return dense_dgrad_as(tmps::kcDenseDgrad, dtype, dy, w, dx, mask, mask_mode, add, B, Din, Dout, ws, s);
}

static hipError_t dense_wgrad_as(int kc, int dtype, const void* dy, const void* x, float* gw, int B, int Din, int Dout,
                                 float* ws, hipStream_t s) {
    // gw[m, n] = sum_k dy[k, m] * x[k, n]: both operands row-contiguous, contraction over the batch
    if (dtype == kBF16) {
        const bool fast = (Dout % 8 == 0) && (Din % 8 == 0) && aligned16(dy) && aligned16(x);
        const int s3 = fast && aligned16(gw) ? g3_wgrad_slices(Dout, Din, B) : 0;
        if (s3 >= 1 && (s3 == 1 || (ws && aligned16(ws)))) {
            G3Operand<false> A{(const bf16_t*)dy, Dout, Dout};
            G3Operand<false> Bv{(const bf16_t*)x, Din, Din};
            const G3Plan plan = g3_plan(Dout, Din, B, s3);
            const int64_t count = (int64_t)Dout * Din + Dout;
            EpiWgrad epi{plan.slices > 1 ? ws : gw, Din, (int64_t)Dout * Din, count};
            hipError_t e = launch3<false, false, true>(kc, A, Bv, epi, Dout, Din, B, plan, s);
            if (e != hipSuccess || plan.slices <= 1) return e;
            return slice_sum((const float*)ws, gw, count, plan.slices, s);
        }
        if (fast) {
            DenseRC A{(const bf16_t*)dy, Dout, B, Dout};
            DenseRC Bv{(const bf16_t*)x, Din, B, Din};
            return run2_wgrad(kc, A, Bv, gw, Dout, Din, B, ws, s);
        }
        DenseView<bf16_t, false> A{(const bf16_t*)dy, Dout, B, Dout, 0};
        DenseView<bf16_t, false> Bv{(const bf16_t*)x, Din, B, Din, 0};
        return wgrad_fallback<bf16_t>(kc, A, Bv, gw, Dout, Din, B, ws, s);
    }
    DenseView<float, false> A{(const float*)dy, Dout, B, Dout, 0};
    DenseView<float, false> Bv{(const float*)x, Din, B, Din, 0};
    return wgrad_fallback<float>(kc, A, Bv, gw, Dout, Din, B, ws, s);
}

hipError_t dense_wgrad(int dtype, const void* dy, const void* x, float* gw, int B, int Din, int Dout, float* ws,
                       hipStream_t s) {
    return dense_wgrad_as(tmps::kcDenseWgrad, dtype, dy, x, gw, B, Din, Dout, ws, s);
}

// ---------------------------------------------------------------------------------- convolution
static ConvGeom geom(const ConvShape& c) {
    return ConvGeom{c.B, c.H, c.W, c.Cin, c.Ho, c.Wo, c.Cout, c.R, c.S, c.stride, c.pad};
}

// The MFMA loaders index positions with 24-bit multiplies and tensors with 32-bit element offsets.
static bool small_enough(const ConvShape& c) {
    const int64_t pin = (int64_t)c.B * c.H * c.W, pout = (int64_t)c.B * c.Ho * c.Wo;
    const int64_t wel = (int64_t)c.Cout * c.R * c.S * c.Cin;
    return pin < (1 << 24) && pout < (1 << 24) && pin * c.Cin < (int64_t(1) << 31) &&
           pout * c.Cout < (int64_t(1) << 31) && wel < (int64_t(1) << 31) && c.Cin < (1 << 20) && c.Cout < (1 << 20);
}

static ConvGeom2 geom2(const ConvShape& c) {
    ConvGeom2 g;
    g.B = c.B; g.H = c.H; g.W = c.W; g.Cin = c.Cin; g.Ho = c.Ho; g.Wo = c.Wo; g.Cout = c.Cout;
    g.R = c.R; g.S = c.S; g.stride = c.stride; g.pad = c.pad;
    g.d_howo = FastDiv(c.Ho * c.Wo); g.d_wo = FastDiv(c.Wo);
    g.d_hw = FastDiv(c.H * c.W); g.d_w = FastDiv(c.W);
    g.d_scin = FastDiv(c.S * c.Cin); g.d_cin = FastDiv(c.Cin);
    g.d_scout = FastDiv(c.S * c.Cout); g.d_cout = FastDiv(c.Cout);
    g.d_stride = FastDiv(c.stride);
    return g;
}

// A 1x1 convolution with unit stride and no padding on NHWC tensors IS a dense layer over the B*H*W positions
// (weights [Cout][Cin]); bf16 ones take the dense paths, which have plain loaders and the persistent kernel.
static bool pointwise(int dtype, const ConvShape& c) {
    return dtype == kBF16 && c.R == 1 && c.S == 1 && c.stride == 1 && c.pad == 0 &&
           (int64_t)c.B * c.H * c.W < (int64_t(1) << 31);
}

hipError_t conv_forward(int dtype, const void* x, const void* w, const float* bias, void* y, const ConvShape& c,
                        int relu, float* ws, hipStream_t s) {
    int M = c.B * c.Ho * c.Wo, K = c.R * c.S * c.Cin;
    if (pointwise(dtype, c))
        return dense_forward_as(kcConvFwd, dtype, x, w, bias, y, M, c.Cin, c.Cout, relu ? kActRelu : kActNone, 0, nullptr, nullptr,
                                ws, s);
    if (dtype == kBF16) {
        EpiBiasAct<bf16_t> epi{(bf16_t*)y, bias, c.Cout, relu};
        if (c.Cin % 8 == 0 && aligned16(x) && aligned16(w) && small_enough(c)) {
            ConvFwdA2 A{(const bf16_t*)x, geom2(c), M, K};
            DenseKC Bv{(const bf16_t*)w, c.Cout, K, K};
            return run2(kcConvFwd, A, Bv, epi, M, c.Cout, K, ws, s);
        }
        ConvFwdA<bf16_t> A{(const bf16_t*)x, geom(c), M, K, 0};
        DenseView<bf16_t, true> Bv{(const bf16_t*)w, c.Cout, K, K, 0};
        return launch_bf16<false>(kcConvFwd, A, Bv, epi, M, c.Cout, K, one_slice(K, kBK), 1, s);
    }
    ConvFwdA<float> A{(const float*)x, geom(c), M, K, 0};
    DenseView<float, true> Bv{(const float*)w, c.Cout, K, K, 0};
    return launch_f32<false>(kcConvFwd, A, Bv, EpiBiasAct<float>{(float*)y, bias, c.Cout, relu}, M, c.Cout, K, one_slice(K, 16), 1, s);
}

hipError_t conv_affine_forward(int dtype, const void* x, const void* w, const float* bias, void* z, const float* gain,
                               const float* shift, void* aout, const void* res, void* yout, int relu, const ConvShape& c,
                               float* ws, hipStream_t s) {
    int M = c.B * c.Ho * c.Wo, K = c.R * c.S * c.Cin;
    if (dtype == kBF16) {
        EpiConvAffine<bf16_t> epi{(bf16_t*)z, bias, c.Cout, gain, shift, (bf16_t*)aout, (const bf16_t*)res, (bf16_t*)yout, relu};
        if (pointwise(dtype, c) && c.Cin % 8 == 0 && aligned16(x) && aligned16(w)) {
            if (g3_forward_ok(M, c.Cout, K) && aligned16(z) && aligned16(bias) && aligned16(gain) && aligned16(shift) &&
                aligned16(aout) && aligned16(res) && aligned16(yout)) {
                G3Operand<true> A{(const bf16_t*)x, M, K};
                G3Operand<true> Bv{(const bf16_t*)w, c.Cout, K};
                return launch3<true, true, false>(kcConvFwd, A, Bv, epi, M, c.Cout, K, g3_plan(M, c.Cout, K, 1), s);
            }
            DenseKC A{(const bf16_t*)x, M, K, K};
            DenseKC Bv{(const bf16_t*)w, c.Cout, K, K};
            return run2(kcConvFwd, A, Bv, epi, M, c.Cout, K, ws, s);
        }
        if (c.Cin % 8 == 0 && aligned16(x) && aligned16(w) && small_enough(c)) {
            ConvFwdA2 A{(const bf16_t*)x, geom2(c), M, K};
            DenseKC Bv{(const bf16_t*)w, c.Cout, K, K};
            return run2(kcConvFwd, A, Bv, epi, M, c.Cout, K, ws, s);
        }
        ConvFwdA<bf16_t> A{(const bf16_t*)x, geom(c), M, K, 0};
        DenseView<bf16_t, true> Bv{(const bf16_t*)w, c.Cout, K, K, 0};
        return launch_bf16<false>(kcConvFwd, A, Bv, epi, M, c.Cout, K, one_slice(K, kBK), 1, s);
    }
    ConvFwdA<float> A{(const float*)x, geom(c), M, K, 0};
    DenseView<float, true> Bv{(const float*)w, c.Cout, K, K, 0};
    EpiConvAffine<float> epi{(float*)z, bias, c.Cout, gain, shift, (float*)aout, (const float*)res, (float*)yout, relu};
    return launch_f32<false>(kcConvFwd, A, Bv, epi, M, c.Cout, K, one_slice(K, 16), 1, s);
}

hipError_t conv_dgrad(int dtype, const void* dy, const void* w, void* dx, const void* mask, const void* add,
                      const ConvShape& c, float* ws, hipStream_t s) {
    int M = c.B * c.H * c.W, K = c.R * c.S * c.Cout;
    if (pointwise(dtype, c)) return dense_dgrad_as(kcConvDgrad, dtype, dy, w, dx, mask, kActRelu, add, M, c.Cin, c.Cout, ws, s);
    if (dtype == kBF16) {
        EpiMask<bf16_t, bf16_t> epi{(bf16_t*)dx, (const bf16_t*)mask, c.Cin, kActRelu, (const bf16_t*)add};
        if (c.Cin % 8 == 0 && c.Cout % 8 == 0 && aligned16(dy) && aligned16(w) && small_enough(c)) {
            if (c.stride == 2 && c.H % 2 == 0 && c.W % 2 == 0) {
                // Rows ordered by the parity of their position, each class walking only the filter taps that reach it:
                // k extent of the largest class; every class a whole number of tiles; the 16-byte epilogue (the one
                // that asks the loader where a row lies in memory), also for the partial sums of a split.
                const int Kp = ((c.R + 1) / 2) * ((c.S + 1) / 2) * c.Cout;
                const GemmPlan plan = plan_gemm(M, c.Cin, Kp);
                const int Mc = M / 4;
                int per, nz;
                slice_geometry(Kp, ws ? plan.slices : 1, kBK2, per, nz);
                const bool split_ok = nz <= 1 || (aligned16(ws) && ((int64_t)M * c.Cin) % 4 == 0);
                // (where a class is no whole number of the plan's tiles, smaller tiles still pay for a filter with
                // several taps; a 1x1 filter's launch is mostly epilogue either way and keeps the plain order then)
                const int tile = (Mc % plan.tile == 0 || c.R * c.S == 1) ? plan.tile : 64;
                if (Mc % tile == 0 && epi.wide_ok() && split_ok) {
                    ParityGeom pg;
                    pg.Mc = Mc;
                    pg.W2 = c.W / 2;
                    pg.d_mc = FastDiv(Mc);
                    pg.d_h2w2 = FastDiv((c.H / 2) * (c.W / 2));
                    pg.d_w2 = FastDiv(c.W / 2);
                    ConvDgradA2P A{(const bf16_t*)dy, geom2(c), M, Kp, pg, {}};
                    ConvDgradB2P Bv{(const bf16_t*)w, geom2(c), c.Cin, Kp, pg, {}};
                    return run2(kcConvDgrad, A, Bv, epi, M, c.Cin, Kp, ws, s, tile);
                }
            }
            ConvDgradA2 A{(const bf16_t*)dy, geom2(c), M, K};
            ConvDgradB2 Bv{(const bf16_t*)w, geom2(c), c.Cin, K};
            return run2(kcConvDgrad, A, Bv, epi, M, c.Cin, K, ws, s);
        }
        ConvDgradA<bf16_t> A{(const bf16_t*)dy, geom(c), M, K, 0};
        ConvDgradB<bf16_t> Bv{(const bf16_t*)w, geom(c), c.Cin, K};
        return launch_bf16<false>(kcConvDgrad, A, Bv, epi, M, c.Cin, K, one_slice(K, kBK), 1, s);
    }
    ConvDgradA<float> A{(const float*)dy, geom(c), M, K, 0};
    ConvDgradB<float> Bv{(const float*)w, geom(c), c.Cin, K};
    return launch_f32<false>(kcConvDgrad, A, Bv, EpiMask<float, float>{(float*)dx, (const float*)mask, c.Cin, kActRelu, (const float*)add}, M, c.Cin, K, one_slice(K, 16), 1, s);
}

hipError_t conv_wgrad(int dtype, const void* dy, const void* x, float* gw, const ConvShape& c, float* ws,
                      hipStream_t s) {
    int rows = c.Cout, cols = c.R * c.S * c.Cin;
    int64_t K = (int64_t)c.B * c.Ho * c.Wo;
    if (pointwise(dtype, c)) return dense_wgrad_as(kcConvWgrad, dtype, dy, x, gw, (int)K, c.Cin, c.Cout, ws, s);
    if (dtype == kBF16) {
        if (c.Cin % 8 == 0 && c.Cout % 8 == 0 && aligned16(dy) && aligned16(x) && small_enough(c)) {
            DenseRC A{(const bf16_t*)dy, rows, (int)K, c.Cout};
            const int rows64 = kBK2 / c.Wo;
            ConvWgradB2 Bv{(const bf16_t*)x, geom2(c), cols, (int)K, kBK2 % c.Wo, rows64 % c.Ho, rows64 / c.Ho};
            return run2_wgrad(kcConvWgrad, A, Bv, gw, rows, cols, K, ws, s);
        }
        DenseView<bf16_t, false> A{(const bf16_t*)dy, rows, (int)K, c.Cout, 0};
        ConvWgradB<bf16_t> Bv{(const bf16_t*)x, geom(c), cols, (int)K};
        return wgrad_fallback<bf16_t>(kcConvWgrad, A, Bv, gw, rows, cols, K, ws, s);
    }
    DenseView<float, false> A{(const float*)dy, rows, (int)K, c.Cout, 0};
    ConvWgradB<float> Bv{(const float*)x, geom(c), cols, (int)K};
    return wgrad_fallback<float>(kcConvWgrad, A, Bv, gw, rows, cols, K, ws, s);
}

}  // namespace tmps
