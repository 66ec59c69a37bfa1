// Main MFMA GEMM skeleton for gfx950 (bf16 in, fp32 accumulate), used by every contraction whose
// operands can be fetched with aligned 16-byte loads.
//
//   C[m, n] = sum_k A(m, k) * B(n, k)
//
// Each operand is described by a loader that is either
//   k-contiguous   (8 consecutive k of one row are 16 consecutive bytes): the tile is kept in LDS as
//                  [row][k] and MFMA fragments are read with 16-byte LDS reads, or
//   row-contiguous (8 consecutive rows of one k are 16 consecutive bytes): the tile is kept in LDS as
//                  [k][row], exactly as it lies in memory, and fragments are read with the LDS
//                  transpose read of gfx950 (ds_read_b64_tr_b16), which hands each lane 4 consecutive
//                  k of its own row.  No operand is ever transposed in registers or in memory.
// Dense forward (A, B k-contiguous), dense input gradient (B = W row-contiguous), dense weight
// gradient (both row-contiguous) and the three implicit-GEMM forms of convolution are instances.
//
// 256 threads = 4 waves (2x2), wave tile (BM/2)x(BN/2) of 32x32x16 MFMA tiles, BK = 64.  Global loads
// of tile t+1 are in flight while tile t is multiplied (register staging, single LDS buffer).
// blockIdx.z selects a k-slice; with more than one slice the epilogue stores fp32 partial sums that a
// finishing kernel reduces.
#pragma once
#include "gemm.hip.h"

namespace tmps {

typedef short s16x4_t __attribute__((ext_vector_type(4)));

// Division of a non-negative 31-bit integer by a runtime constant through multiply-and-shift.
struct FastDiv {
    uint32_t mul, sh, d;
    __host__ __device__ FastDiv() : mul(0), sh(0), d(1) {}
    __host__ explicit FastDiv(uint32_t div) : d(div) {
        uint32_t l = 0;
        while ((uint64_t(1) << l) < div) ++l;
        sh = 31 + l;
        mul = (uint32_t)(((uint64_t(1) << sh) + div - 1) / div);
    }
    __device__ __forceinline__ uint32_t div(uint32_t n) const { return (uint32_t)(((uint64_t)n * mul) >> sh); }
    __device__ __forceinline__ void divmod(uint32_t n, uint32_t& q, uint32_t& r) const {
        q = div(n);
        r = n - q * d;
    }
};

constexpr int kBK2 = 64;

// ------------------------------------------------------------------------------------------
// Loaders.  KC loaders: init(ctx, row, kc) once per thread-chunk with the global row and the chunk
// index kc (k offset kc*8 inside a tile); load(ctx, kb, k_end) returns the 16 bytes at k = kb + kc*8
// (zeros when out of range).  RC (row-contiguous) loaders: init(ctx, row0, kl) with the first of 8
// consecutive rows and the k offset kl inside a tile; load(ctx, kb, k_end) returns rows row0..row0+7
// at k = kb + kl.
// ------------------------------------------------------------------------------------------
struct DenseKC {
    static constexpr bool kContig = true;
    const bf16_t* p;
    int rows, K;
    int64_t ld;
    struct Ctx { const bf16_t* q; int koff; bool ok; };
    __device__ __forceinline__ void init(Ctx& c, int row, int kc) const {
        c.ok = row < rows;
        c.koff = kc * 8;
        c.q = p + (int64_t)(c.ok ? row : 0) * ld + c.koff;
    }
    __device__ __forceinline__ uint4 load(const Ctx& c, int kb, int k_end) const {
        if (c.ok && kb + c.koff + 8 <= k_end) return *reinterpret_cast<const uint4*>(c.q + kb);
        return make_uint4(0, 0, 0, 0);
    }
};

struct DenseRC {
    static constexpr bool kContig = false;
    const bf16_t* p;  // element(row, k) = p[k*ld + row]
    int rows, K;
    int64_t ld;
    struct Ctx { const bf16_t* q; int kl; bool ok; };
    __device__ __forceinline__ void init(Ctx& c, int row0, int kl) const {
        c.ok = row0 + 8 <= rows;
        c.kl = kl;
        c.q = p + (c.ok ? row0 : 0) + (int64_t)kl * ld;
    }
    __device__ __forceinline__ uint4 load(const Ctx& c, int kb, int k_end) const {
        if (c.ok && kb + c.kl < k_end) return *reinterpret_cast<const uint4*>(c.q + (int64_t)kb * ld);
        return make_uint4(0, 0, 0, 0);
    }
};

struct ConvGeom2 {
    int B, H, W, Cin, Ho, Wo, Cout, R, S, stride, pad;
    FastDiv d_howo, d_wo, d_hw, d_w, d_scin, d_cin, d_scout, d_cout, d_stride;
};

// Forward A: row m = (n, ho, wo), k = (r, s, c) -> x[n, ho*stride + r - pad, wo*stride + s - pad, c].
struct ConvFwdA2 {
    static constexpr bool kContig = true;
    const bf16_t* x;
    ConvGeom2 g;
    int rows, K;
    struct Ctx { int64_t base; int h0, w0, koff; bool ok; };
    __device__ __forceinline__ void init(Ctx& c, int m, int kc) const {
        c.ok = m < rows;
        uint32_t n, rem, ho, wo;
        g.d_howo.divmod(c.ok ? m : 0, n, rem);
        g.d_wo.divmod(rem, ho, wo);
        c.h0 = (int)ho * g.stride - g.pad;
        c.w0 = (int)wo * g.stride - g.pad;
        c.base = (((int64_t)n * g.H + c.h0) * g.W + c.w0) * g.Cin;
        c.koff = kc * 8;
    }
    __device__ __forceinline__ uint4 load(const Ctx& c, int kb, int k_end) const {
        int k = kb + c.koff;
        if (!c.ok || k + 8 > k_end) return make_uint4(0, 0, 0, 0);
        uint32_t r, rem, s, ch;
        g.d_scin.divmod(k, r, rem);
        g.d_cin.divmod(rem, s, ch);
        int h = c.h0 + (int)r, w = c.w0 + (int)s;
        if ((unsigned)h >= (unsigned)g.H || (unsigned)w >= (unsigned)g.W) return make_uint4(0, 0, 0, 0);
        return *reinterpret_cast<const uint4*>(x + c.base + ((int64_t)r * g.W + s) * g.Cin + ch);
    }
};

// Input-gradient A: row m = (n, h, w), k = (r, s, co) -> dy[n, (h+pad-r)/stride, (w+pad-s)/stride, co]
// when both divisions are exact and in range.
struct ConvDgradA2 {
    static constexpr bool kContig = true;
    const bf16_t* dy;
    ConvGeom2 g;
    int rows, K;
    struct Ctx { int n, hp, wp, koff; bool ok; };
    __device__ __forceinline__ void init(Ctx& c, int m, int kc) const {
        c.ok = m < rows;
        uint32_t n, rem, h, w;
        g.d_hw.divmod(c.ok ? m : 0, n, rem);
        g.d_w.divmod(rem, h, w);
        c.n = (int)n;
        c.hp = (int)h + g.pad;
        c.wp = (int)w + g.pad;
        c.koff = kc * 8;
    }
    __device__ __forceinline__ uint4 load(const Ctx& c, int kb, int k_end) const {
        int k = kb + c.koff;
        if (!c.ok || k + 8 > k_end) return make_uint4(0, 0, 0, 0);
        uint32_t r, rem, s, co;
        g.d_scout.divmod(k, r, rem);
        g.d_cout.divmod(rem, s, co);
        int hy = c.hp - (int)r, wy = c.wp - (int)s;
        if (hy < 0 || wy < 0) return make_uint4(0, 0, 0, 0);
        uint32_t ho, hr, wo, wr;
        g.d_stride.divmod(hy, ho, hr);
        g.d_stride.divmod(wy, wo, wr);
        if (hr != 0 || wr != 0 || (int)ho >= g.Ho || (int)wo >= g.Wo) return make_uint4(0, 0, 0, 0);
        return *reinterpret_cast<const uint4*>(dy + (((int64_t)c.n * g.Ho + ho) * g.Wo + wo) * g.Cout + co);
    }
};

// Input-gradient B: row n = ci (8 consecutive), k = (r, s, co) -> w[co, r, s, ci].
struct ConvDgradB2 {
    static constexpr bool kContig = false;
    const bf16_t* w;
    ConvGeom2 g;
    int rows, K;
    struct Ctx { int ci0, kl; bool ok; };
    __device__ __forceinline__ void init(Ctx& c, int row0, int kl) const {
        c.ok = row0 + 8 <= rows;
        c.ci0 = row0;
        c.kl = kl;
    }
    __device__ __forceinline__ uint4 load(const Ctx& c, int kb, int k_end) const {
        int k = kb + c.kl;
        if (!c.ok || k >= k_end) return make_uint4(0, 0, 0, 0);
        uint32_t r, rem, s, co;
        g.d_scout.divmod(k, r, rem);
        g.d_cout.divmod(rem, s, co);
        return *reinterpret_cast<const uint4*>(w + ((((int64_t)co * g.R + r) * g.S + s) * g.Cin + c.ci0));
    }
};

// Weight-gradient B: row = (r, s, ci) (8 consecutive ci), k = m = (n, ho, wo)
// -> x[n, ho*stride + r - pad, wo*stride + s - pad, ci].
struct ConvWgradB2 {
    static constexpr bool kContig = false;
    const bf16_t* x;
    ConvGeom2 g;
    int rows, K;
    struct Ctx { int dr, ds, ci0, kl; bool ok; };
    __device__ __forceinline__ void init(Ctx& c, int row0, int kl) const {
        c.ok = row0 + 8 <= rows;
        uint32_t r, rem, s, ci;
        g.d_scin.divmod(c.ok ? row0 : 0, r, rem);
        g.d_cin.divmod(rem, s, ci);
        c.dr = (int)r - g.pad;
        c.ds = (int)s - g.pad;
        c.ci0 = (int)ci;
        c.kl = kl;
    }
    __device__ __forceinline__ uint4 load(const Ctx& c, int kb, int k_end) const {
        int m = kb + c.kl;
        if (!c.ok || m >= k_end) return make_uint4(0, 0, 0, 0);
        uint32_t n, rem, ho, wo;
        g.d_howo.divmod(m, n, rem);
        g.d_wo.divmod(rem, ho, wo);
        int h = (int)ho * g.stride + c.dr, w = (int)wo * g.stride + c.ds;
        if ((unsigned)h >= (unsigned)g.H || (unsigned)w >= (unsigned)g.W) return make_uint4(0, 0, 0, 0);
        return *reinterpret_cast<const uint4*>(x + (((int64_t)n * g.H + h) * g.W + w) * g.Cin + c.ci0);
    }
};

// ------------------------------------------------------------------------------------------
// LDS tile shapes.  k-contiguous: [rows][64 + 8] (144-byte rows: 16-byte reads of 8 consecutive rows
// hit disjoint banks).  row-contiguous: [64][rows + 16] (row pitch = 32 bytes mod 128, so the 4 k-rows
// a 16-lane group reads in one transpose read hit disjoint banks).
// ------------------------------------------------------------------------------------------
template <int ROWS, bool KC> struct TileShape {
    static constexpr int pitch = KC ? (kBK2 + 8) : (ROWS + 16);
    static constexpr int elems = KC ? ROWS * pitch : kBK2 * pitch;
};

template <int ROWS, bool KC> __device__ __forceinline__ bf16x8_t read_frag(const bf16_t* tile, int row_base, int kk, int lane) {
    if constexpr (KC) {
        const bf16_t* p = tile + (row_base + (lane & 31)) * TileShape<ROWS, true>::pitch + kk * 16 + (lane >> 5) * 8;
        return *reinterpret_cast<const bf16x8_t*>(p);
    } else {
        constexpr int pitch = TileShape<ROWS, false>::pitch;
        const int k = kk * 16 + (lane >> 5) * 8 + ((lane & 15) >> 2);
        const int col = row_base + ((lane >> 4) & 1) * 16 + (lane & 3) * 4;
        typedef __attribute__((address_space(3))) s16x4_t* lds_ptr_t;
        const bf16_t* p0 = tile + k * pitch + col;
        const bf16_t* p1 = p0 + 4 * pitch;
        s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(p0));
        s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(p1));
        union { s16x4_t h[2]; bf16x8_t v; } u;
        u.h[0] = lo;
        u.h[1] = hi;
        return u.v;
    }
}

template <int BM, int BN, bool ROWSUM, class AOp, class BOp, class Epi>
__global__ __launch_bounds__(256) void gemm2_kernel(AOp A, BOp B, Epi epi, int M, int N, int K, int k_per_slice) {
    constexpr bool AKC = AOp::kContig, BKC = BOp::kContig;
    constexpr int TM = BM / 64, TN = BN / 64;
    constexpr int A_CH = BM * (kBK2 / 8) / 256, B_CH = BN * (kBK2 / 8) / 256;
    __shared__ __attribute__((aligned(16))) bf16_t sA[TileShape<BM, AKC>::elems];
    __shared__ __attribute__((aligned(16))) bf16_t sB[TileShape<BN, BKC>::elems];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN, z = blockIdx.z;
    const int k_begin = z * k_per_slice;
    const int k_end = min(K, k_begin + k_per_slice);
    const int nk = (k_end - k_begin + kBK2 - 1) / kBK2;

    typename AOp::Ctx ca[A_CH];
    typename BOp::Ctx cb[B_CH];
    int sa_off[A_CH], sb_off[B_CH];
#pragma unroll
    for (int i = 0; i < A_CH; ++i) {
        int c = tid + i * 256;
        if constexpr (AKC) {
            int row = c >> 3, kc = c & 7;
            A.init(ca[i], m0 + row, kc);
            sa_off[i] = row * TileShape<BM, true>::pitch + kc * 8;
        } else {
            int rc = c % (BM / 8), kl = c / (BM / 8);
            A.init(ca[i], m0 + rc * 8, kl);
            sa_off[i] = kl * TileShape<BM, false>::pitch + rc * 8;
        }
    }
#pragma unroll
    for (int i = 0; i < B_CH; ++i) {
        int c = tid + i * 256;
        if constexpr (BKC) {
            int row = c >> 3, kc = c & 7;
            B.init(cb[i], n0 + row, kc);
            sb_off[i] = row * TileShape<BN, true>::pitch + kc * 8;
        } else {
            int rc = c % (BN / 8), kl = c / (BN / 8);
            B.init(cb[i], n0 + rc * 8, kl);
            sb_off[i] = kl * TileShape<BN, false>::pitch + rc * 8;
        }
    }

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
    float rsum = 0.0f;

    uint4 ra[A_CH], rb[B_CH];
    if (nk > 0) {
#pragma unroll
        for (int i = 0; i < A_CH; ++i) ra[i] = A.load(ca[i], k_begin, k_end);
#pragma unroll
        for (int i = 0; i < B_CH; ++i) rb[i] = B.load(cb[i], k_begin, k_end);
    }
    for (int kt = 0; kt < nk; ++kt) {
        __syncthreads();  // everyone is done reading the previous tile
#pragma unroll
        for (int i = 0; i < A_CH; ++i) *reinterpret_cast<uint4*>(&sA[sa_off[i]]) = ra[i];
#pragma unroll
        for (int i = 0; i < B_CH; ++i) *reinterpret_cast<uint4*>(&sB[sb_off[i]]) = rb[i];
        __syncthreads();
        if (kt + 1 < nk) {
            const int kb = k_begin + (kt + 1) * kBK2;
#pragma unroll
            for (int i = 0; i < A_CH; ++i) ra[i] = A.load(ca[i], kb, k_end);
#pragma unroll
            for (int i = 0; i < B_CH; ++i) rb[i] = B.load(cb[i], kb, k_end);
        }
#pragma unroll
        for (int kk = 0; kk < kBK2 / 16; ++kk) {
            bf16x8_t af[TM], bfr[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) af[i] = read_frag<BM, AKC>(sA, wm * (BM / 2) + i * 32, kk, lane);
#pragma unroll
            for (int j = 0; j < TN; ++j) bfr[j] = read_frag<BN, BKC>(sB, wn * (BN / 2) + j * 32, kk, lane);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
        }
        if (ROWSUM && blockIdx.x == 0 && tid < BM) {
            if constexpr (AKC) {
                const bf16_t* rowp = &sA[tid * TileShape<BM, true>::pitch];
#pragma unroll 8
                for (int e = 0; e < kBK2; ++e) rsum += (float)rowp[e];
            } else {
#pragma unroll 8
                for (int e = 0; e < kBK2; ++e) rsum += (float)sA[e * TileShape<BM, false>::pitch + tid];
            }
        }
    }

    const int col_in = lane & 31, row_in = (lane >> 5) * 4;
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

// Split-k partial sums: slice z stores fp32 at part[z][m][n].
struct EpiPartial {
    float* part;
    int64_t ld, slice_stride;
    __device__ __forceinline__ void operator()(int m, int n, float v, int z) const {
        part[z * slice_stride + (int64_t)m * ld + n] = v;
    }
    __device__ __forceinline__ void rowsum(int, float, int) const {}
};

// Reduce the slices and apply the real epilogue.
template <class Epi>
__global__ void splitk_finish_kernel(const float* __restrict__ part, Epi epi, int M, int N, int slices) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t total = (int64_t)M * N;
    if (i >= total) return;
    float a = 0.0f;
    for (int z = 0; z < slices; ++z) a += part[z * total + i];
    int m = (int)(i / N), n = (int)(i - (int64_t)m * N);
    epi(m, n, a, 0);
}

}  // namespace tmps
