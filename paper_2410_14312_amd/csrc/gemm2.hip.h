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
// 256 threads = 4 waves (2x2), wave tile (BM/2)x(BN/2) of 32x32x16 MFMA tiles, BK = 64.  The global
// loads of the next D k-tiles are in flight in a register ring while the current tile is multiplied
// (these contractions are short and few workgroups share a CU, so memory latency has to be hidden
// inside the workgroup); LDS is double-buffered, one barrier per k-tile.
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

__device__ __forceinline__ uint4 zero16() { return make_uint4(0, 0, 0, 0); }
__device__ __forceinline__ uint4 ld16(const bf16_t* p) { return *reinterpret_cast<const uint4*>(p); }
// Load that is ALWAYS issued: lanes whose chunk lies outside the operand read 16 zero bytes from a
// dummy location instead.  With neither a branch around the load nor a select on its result, the
// compiler counts the loads in flight exactly and a tile is waited for only when it is copied to LDS,
// D tiles after it was requested.
static __device__ __attribute__((aligned(16))) uint4 g_zero_chunk;  // zero-initialised, never written
__device__ __forceinline__ uint4 ld16_if(const bf16_t* base, int64_t off, bool ok) {
    const bf16_t* p = ok ? base + off : reinterpret_cast<const bf16_t*>(&g_zero_chunk);
    return ld16(p);
}
// full-rate 24-bit multiply (both factors below 2^24, product below 2^31)
__device__ __forceinline__ int mul24(int a, int b) { return __mul24(a, b); }

// ------------------------------------------------------------------------------------------
// Loaders.  A thread fetches a fixed set of 16-byte chunks of every k-tile; a loader is an iterator
// over k-tiles, so that the k-loop needs no integer division and no 64-bit multiply:
//   init_thread(ks, k_begin, col)  per-thread state for the first tile; col = the thread's chunk column
//                                  (k offset col*8) for k-contiguous loaders, unused otherwise
//   init(ctx, row, col, k_begin)   per-chunk state.  k-contiguous: row = global row.  row-contiguous:
//                                  row = first of 8 consecutive rows, col = k offset inside a tile.
//   load(ctx, ks, k_end)           the chunk of the current tile (zeros outside the operand); called once
//                                  per tile and chunk, in order; may step per-chunk state
//   next(ks)                       step the per-thread state to the next tile (k += 64)
// Element offsets are 32-bit: every tensor here has fewer than 2^31 elements.
// ------------------------------------------------------------------------------------------
struct DenseKC {
    static constexpr bool kContig = true;
    const bf16_t* p;
    int rows, K;
    int64_t ld;
    struct KS { int k; };
    struct Ctx { int64_t roff; bool ok; };
    __device__ __forceinline__ void init_thread(KS& ks, int k_begin, int col) const { ks.k = k_begin + col * 8; }
    __device__ __forceinline__ void init(Ctx& c, int row, int, int) const {
        c.ok = row < rows;
        c.roff = (int64_t)(c.ok ? row : 0) * ld;
    }
    __device__ __forceinline__ uint4 load(Ctx& c, const KS& ks, int k_end) const {
        return ld16_if(p, c.roff + ks.k, c.ok && ks.k + 8 <= k_end);
    }
    __device__ __forceinline__ void next(KS& ks) const { ks.k += kBK2; }
};

struct DenseRC {
    static constexpr bool kContig = false;
    const bf16_t* p;  // element(row, k) = p[k*ld + row]
    int rows, K;
    int64_t ld;
    struct KS { int kb; };
    struct Ctx { int64_t off; int kl; bool ok; };
    __device__ __forceinline__ void init_thread(KS& ks, int k_begin, int) const { ks.kb = k_begin; }
    __device__ __forceinline__ void init(Ctx& c, int row0, int kl, int k_begin) const {
        c.ok = row0 + 8 <= rows;
        c.kl = kl;
        c.off = (c.ok ? row0 : 0) + (int64_t)(k_begin + kl) * ld;
    }
    __device__ __forceinline__ uint4 load(Ctx& c, const KS& ks, int k_end) const {
        uint4 v = ld16_if(p, c.off, c.ok && ks.kb + c.kl < k_end);
        c.off += kBK2 * ld;
        return v;
    }
    __device__ __forceinline__ void next(KS& ks) const { ks.kb += kBK2; }
};

struct ConvGeom2 {
    int B, H, W, Cin, Ho, Wo, Cout, R, S, stride, pad;
    FastDiv d_howo, d_wo, d_hw, d_w, d_scin, d_cin, d_scout, d_cout, d_stride;
};

// Forward A: row m = (n, ho, wo), k = (r, s, c) -> x[n, ho*stride + r - pad, wo*stride + s - pad, c].
// Per thread: (r, s, c) of its chunk column, stepped by 64 channels per tile.
struct ConvFwdA2 {
    static constexpr bool kContig = true;
    const bf16_t* x;
    ConvGeom2 g;
    int rows, K;
    struct KS { int k, r, s, ch, koff; };
    struct Ctx { int base, h0, w0; bool ok; };
    __device__ __forceinline__ void init_thread(KS& ks, int k_begin, int col) const {
        ks.k = k_begin + col * 8;
        uint32_t r, rem, s, ch;
        g.d_scin.divmod(ks.k, r, rem);
        g.d_cin.divmod(rem, s, ch);
        ks.r = (int)r; ks.s = (int)s; ks.ch = (int)ch;
        ks.koff = mul24(mul24(ks.r, g.W) + ks.s, g.Cin) + ks.ch;
    }
    __device__ __forceinline__ void init(Ctx& c, int m, int, int) const {
        c.ok = m < rows;
        uint32_t n, rem, ho, wo;
        g.d_howo.divmod(c.ok ? m : 0, n, rem);
        g.d_wo.divmod(rem, ho, wo);
        c.h0 = (int)ho * g.stride - g.pad;
        c.w0 = (int)wo * g.stride - g.pad;
        c.base = (((int)n * g.H + c.h0) * g.W + c.w0) * g.Cin;
    }
    __device__ __forceinline__ uint4 load(Ctx& c, const KS& ks, int k_end) const {
        const int h = c.h0 + ks.r, w = c.w0 + ks.s;
        const bool ok = c.ok && ks.k + 8 <= k_end && (unsigned)h < (unsigned)g.H && (unsigned)w < (unsigned)g.W;
        return ld16_if(x, c.base + ks.koff, ok);
    }
    __device__ __forceinline__ void next(KS& ks) const {
        ks.k += kBK2;
        ks.ch += kBK2;
        while (ks.ch >= g.Cin) {
            ks.ch -= g.Cin;
            if (++ks.s == g.S) { ks.s = 0; ++ks.r; }
        }
        ks.koff = mul24(mul24(ks.r, g.W) + ks.s, g.Cin) + ks.ch;
    }
};

// Input-gradient A: row m = (n, h, w), k = (r, s, co) -> dy[n, (h+pad-r)/stride, (w+pad-s)/stride, co]
// when both divisions are exact and in range.
struct ConvDgradA2 {
    static constexpr bool kContig = true;
    const bf16_t* dy;
    ConvGeom2 g;
    int rows, K;
    struct KS { int k, r, s, co, kterm; };
    struct Ctx { int c0, hp, wp, nbase; bool ok; };
    __device__ __forceinline__ void init_thread(KS& ks, int k_begin, int col) const {
        ks.k = k_begin + col * 8;
        uint32_t r, rem, s, co;
        g.d_scout.divmod(ks.k, r, rem);
        g.d_cout.divmod(rem, s, co);
        ks.r = (int)r; ks.s = (int)s; ks.co = (int)co;
        ks.kterm = ks.co - mul24(mul24(ks.r, g.Wo) + ks.s, g.Cout);
    }
    __device__ __forceinline__ void init(Ctx& c, int m, int, int) const {
        c.ok = m < rows;
        uint32_t n, rem, h, w;
        g.d_hw.divmod(c.ok ? m : 0, n, rem);
        g.d_w.divmod(rem, h, w);
        c.hp = (int)h + g.pad;
        c.wp = (int)w + g.pad;
        c.nbase = (int)n * g.Ho * g.Wo * g.Cout;
        c.c0 = c.nbase + (c.hp * g.Wo + c.wp) * g.Cout;  // stride 1: offset = c0 + kterm
    }
    __device__ __forceinline__ uint4 load(Ctx& c, const KS& ks, int k_end) const {
        const bool in_k = c.ok && ks.k + 8 <= k_end;
        const int hy = c.hp - ks.r, wy = c.wp - ks.s;
        if (g.stride == 1) {
            const bool ok = in_k && (unsigned)hy < (unsigned)g.Ho && (unsigned)wy < (unsigned)g.Wo;
            return ld16_if(dy, c.c0 + ks.kterm, ok);
        }
        uint32_t ho, hr, wo, wr;
        g.d_stride.divmod(hy < 0 ? 0 : hy, ho, hr);
        g.d_stride.divmod(wy < 0 ? 0 : wy, wo, wr);
        const bool ok = in_k && hy >= 0 && wy >= 0 && hr == 0 && wr == 0 && (int)ho < g.Ho && (int)wo < g.Wo;
        return ld16_if(dy, c.nbase + ((int)ho * g.Wo + (int)wo) * g.Cout + ks.co, ok);
    }
    __device__ __forceinline__ void next(KS& ks) const {
        ks.k += kBK2;
        ks.co += kBK2;
        while (ks.co >= g.Cout) {
            ks.co -= g.Cout;
            if (++ks.s == g.S) { ks.s = 0; ++ks.r; }
        }
        ks.kterm = ks.co - mul24(mul24(ks.r, g.Wo) + ks.s, g.Cout);
    }
};

// Input-gradient B: row n = ci (8 consecutive), k = (r, s, co) -> w[co, r, s, ci].
// Per thread: (r, s, co) of the tile's first k; a chunk adds its k offset (with carry when the tile
// crosses a filter tap).
struct ConvDgradB2 {
    static constexpr bool kContig = false;
    const bf16_t* w;
    ConvGeom2 g;
    int rows, K;
    struct KS { int kb, r, s, co; };
    struct Ctx { int ci0, kl; bool ok; };
    __device__ __forceinline__ void init_thread(KS& ks, int k_begin, int) const {
        ks.kb = k_begin;
        uint32_t r, rem, s, co;
        g.d_scout.divmod(k_begin, r, rem);
        g.d_cout.divmod(rem, s, co);
        ks.r = (int)r; ks.s = (int)s; ks.co = (int)co;
    }
    __device__ __forceinline__ void init(Ctx& c, int row0, int kl, int) const {
        c.ok = row0 + 8 <= rows;
        c.ci0 = row0;
        c.kl = kl;
    }
    __device__ __forceinline__ uint4 load(Ctx& c, const KS& ks, int k_end) const {
        const bool ok = c.ok && ks.kb + c.kl < k_end;
        int co = ks.co + c.kl, s = ks.s, r = ks.r;
        while (co >= g.Cout) {
            co -= g.Cout;
            if (++s == g.S) { s = 0; ++r; }
        }
        const int off = mul24(mul24(mul24(co, g.R) + r, g.S) + s, g.Cin) + c.ci0;
        return ld16_if(w, off, ok);
    }
    __device__ __forceinline__ void next(KS& ks) const {
        ks.kb += kBK2;
        ks.co += kBK2;
        while (ks.co >= g.Cout) {
            ks.co -= g.Cout;
            if (++ks.s == g.S) { ks.s = 0; ++ks.r; }
        }
    }
};

// Weight-gradient B: row = (r, s, ci) (8 consecutive ci), k = m = (n, ho, wo)
// -> x[n, ho*stride + r - pad, wo*stride + s - pad, ci].
// Per chunk: (ho, wo) of its position and the element offset of that position, stepped by 64
// positions per tile with precomputed carries.
struct ConvWgradB2 {
    static constexpr bool kContig = false;
    const bf16_t* x;
    ConvGeom2 g;
    int rows, K;
    int step_wo, step_ho, step_n;  // 64 positions = step_n images + step_ho rows + step_wo columns
    struct KS { int kb; };
    struct Ctx { int dr, ds, ci0, kl, ho, wo, n; bool ok; };
    __device__ __forceinline__ void init_thread(KS& ks, int k_begin, int) const { ks.kb = k_begin; }
    __device__ __forceinline__ void init(Ctx& c, int row0, int kl, int k_begin) const {
        c.ok = row0 + 8 <= rows;
        uint32_t r, rem, s, ci;
        g.d_scin.divmod(c.ok ? row0 : 0, r, rem);
        g.d_cin.divmod(rem, s, ci);
        c.dr = (int)r - g.pad;
        c.ds = (int)s - g.pad;
        c.ci0 = (int)ci;
        c.kl = kl;
        uint32_t n, rem2, ho, wo;
        g.d_howo.divmod(k_begin + kl, n, rem2);
        g.d_wo.divmod(rem2, ho, wo);
        c.n = (int)n; c.ho = (int)ho; c.wo = (int)wo;
    }
    __device__ __forceinline__ uint4 load(Ctx& c, const KS& ks, int k_end) const {
        const int h = c.ho * g.stride + c.dr, w = c.wo * g.stride + c.ds;
        const bool ok = c.ok && ks.kb + c.kl < k_end && (unsigned)h < (unsigned)g.H && (unsigned)w < (unsigned)g.W;
        uint4 v = ld16_if(x, mul24(mul24(mul24(c.n, g.H) + h, g.W) + w, g.Cin) + c.ci0, ok);
        // advance this chunk's position by 64
        c.wo += step_wo;
        c.ho += step_ho;
        c.n += step_n;
        if (c.wo >= g.Wo) { c.wo -= g.Wo; ++c.ho; }
        if (c.ho >= g.Ho) { c.ho -= g.Ho; ++c.n; }
        return v;
    }
    __device__ __forceinline__ void next(KS& ks) const { ks.kb += kBK2; }
};

// Input gradient of a convolution with stride 2, rows ordered by the PARITY of their position: row
// m = ((a, b), n, h2, w2) stands for position (h, w) = (2 h2 + a, 2 w2 + b) of image n (H and W even, every class
// a whole number of tiles).  Position (h, w) receives gradient only through the filter taps r = h + pad (mod 2),
// s = w + pad (mod 2), so the tiles of one class walk just those taps, k = (r, s, co) over r = r0, r0 + 2, ...,
// s = s0, s0 + 2, ...: a quarter of the products of the natural order, where the other three quarters multiply
// zeros.  The kernel asks the loaders for the k extent of a tile (k_total) and for the memory row of a row (out_row).
struct ParityGeom {
    int Mc, W2;                      // rows per class, half width
    FastDiv d_mc, d_h2w2, d_w2;
};

struct ParityTaps {
    int r0, s0, ns, keff;            // first tap of the class along r and s, taps along s, k extent
    __device__ __forceinline__ void set(int pc, const ConvGeom2& g) {
        r0 = ((pc >> 1) + g.pad) & 1;
        s0 = ((pc & 1) + g.pad) & 1;
        const int nr = r0 < g.R ? (g.R - r0 + 1) >> 1 : 0;
        ns = s0 < g.S ? (g.S - s0 + 1) >> 1 : 0;
        keff = nr * ns * g.Cout;
    }
    // tap and channel of k = (r, s, co) in the class's own order
    __device__ __forceinline__ void locate(int k, const ConvGeom2& g, int& r, int& s, int& co) const {
        const int t = (int)g.d_cout.div((uint32_t)k);
        co = k - t * g.Cout;
        const int ri = ns > 0 ? t / ns : 0;
        r = r0 + 2 * ri;
        s = s0 + 2 * (t - ri * ns);
    }
    __device__ __forceinline__ void carry(int& r, int& s, int& co, const ConvGeom2& g) const {
        while (co >= g.Cout) {
            co -= g.Cout;
            s += 2;
            if (s >= g.S) { s = s0; r += 2; }
        }
    }
};

struct ConvDgradA2P {
    static constexpr bool kContig = true;
    const bf16_t* dy;
    ConvGeom2 g;
    int rows, K;
    ParityGeom p;
    ParityTaps taps;
    struct KS { int k, r, s, co; };
    struct Ctx { int hp, wp, nbase; bool ok; };
    __device__ __forceinline__ void position(int m, int& n, int& h, int& w) const {
        const int pc = (int)p.d_mc.div((uint32_t)m);
        uint32_t n_, rem, h2, w2;
        p.d_h2w2.divmod((uint32_t)(m - pc * p.Mc), n_, rem);
        p.d_w2.divmod(rem, h2, w2);
        n = (int)n_;
        h = 2 * (int)h2 + (pc >> 1);
        w = 2 * (int)w2 + (pc & 1);
    }
    __device__ __forceinline__ void begin_tile(int m0) { taps.set((int)p.d_mc.div((uint32_t)m0), g); }
    __device__ __forceinline__ int k_total(int) const { return taps.keff; }
    __device__ __forceinline__ int out_row(int m) const {
        int n, h, w;
        position(m, n, h, w);
        return (n * g.H + h) * g.W + w;
    }
    __device__ __forceinline__ void init_thread(KS& ks, int k_begin, int col) const {
        ks.k = k_begin + col * 8;
        taps.locate(ks.k, g, ks.r, ks.s, ks.co);
    }
    __device__ __forceinline__ void init(Ctx& c, int m, int, int) const {
        c.ok = m < rows;
        int n, h, w;
        position(c.ok ? m : 0, n, h, w);
        c.hp = h + g.pad;
        c.wp = w + g.pad;
        c.nbase = n * g.Ho * g.Wo * g.Cout;
    }
    __device__ __forceinline__ uint4 load(Ctx& c, const KS& ks, int k_end) const {
        const int hy = c.hp - ks.r, wy = c.wp - ks.s;   // even for the taps of this class
        const int ho = hy >> 1, wo = wy >> 1;
        const bool ok = c.ok && ks.k + 8 <= k_end && hy >= 0 && wy >= 0 && ho < g.Ho && wo < g.Wo;
        return ld16_if(dy, c.nbase + (ho * g.Wo + wo) * g.Cout + ks.co, ok);
    }
    __device__ __forceinline__ void next(KS& ks) const {
        ks.k += kBK2;
        ks.co += kBK2;
        taps.carry(ks.r, ks.s, ks.co, g);
    }
};

// The filter taps in the same order: row n = ci (8 consecutive), k = (r, s, co) of the tile's class -> w[co, r, s, ci].
struct ConvDgradB2P {
    static constexpr bool kContig = false;
    const bf16_t* w;
    ConvGeom2 g;
    int rows, K;
    ParityGeom p;
    ParityTaps taps;
    struct KS { int kb, r, s, co; };
    struct Ctx { int ci0, kl; bool ok; };
    __device__ __forceinline__ void begin_tile(int m0) { taps.set((int)p.d_mc.div((uint32_t)m0), g); }
    __device__ __forceinline__ void init_thread(KS& ks, int k_begin, int) const {
        ks.kb = k_begin;
        taps.locate(k_begin, g, ks.r, ks.s, ks.co);
    }
    __device__ __forceinline__ void init(Ctx& c, int row0, int kl, int) const {
        c.ok = row0 + 8 <= rows;
        c.ci0 = row0;
        c.kl = kl;
    }
    __device__ __forceinline__ uint4 load(Ctx& c, const KS& ks, int k_end) const {
        const bool ok = c.ok && ks.kb + c.kl < k_end;
        int co = ks.co + c.kl, s = ks.s, r = ks.r;
        taps.carry(r, s, co, g);
        const int off = mul24(mul24(mul24(co, g.R) + r, g.S) + s, g.Cin) + c.ci0;
        return ld16_if(w, off, ok);
    }
    __device__ __forceinline__ void next(KS& ks) const {
        ks.kb += kBK2;
        ks.co += kBK2;
        taps.carry(ks.r, ks.s, ks.co, g);
    }
};

// What gemm2_kernel asks of a loader beyond its chunks; loaders without these members get the defaults.
template <class Op> __device__ __forceinline__ auto op_begin_tile(Op& op, int m0, int) -> decltype(op.begin_tile(m0), void()) { op.begin_tile(m0); }
template <class Op> __device__ __forceinline__ void op_begin_tile(Op&, int, long) {}
template <class Op> __device__ __forceinline__ auto op_k_total(const Op& op, int K, int) -> decltype(op.k_total(K)) { return op.k_total(K); }
template <class Op> __device__ __forceinline__ int op_k_total(const Op&, int K, long) { return K; }
template <class Op> __device__ __forceinline__ auto op_out_row(const Op& op, int m, int) -> decltype(op.out_row(m)) { return op.out_row(m); }
template <class Op> __device__ __forceinline__ int op_out_row(const Op&, int m, long) { return m; }

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
        // Transpose read: within 16 lanes, lane j supplies the address of 4 consecutive rows at
        // k = k0 + j/4, rows c0 + 4*(j%4); lane i receives k0..k0+3 of row c0 + i.
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

// LDS bytes of one launch: two buffers of an A tile and a B tile.
template <int BM, int BN, class AOp, class BOp> constexpr int gemm2_lds_bytes() {
    return 2 * (TileShape<BM, AOp::kContig>::elems + TileShape<BN, BOp::kContig>::elems) * (int)sizeof(bf16_t);
}

// D = number of k-tiles whose global loads are in flight per thread (register ring).
// The 64 x 64 tiles are compiled for three waves per SIMD (168 registers, nothing spilled): launches of 500 to 800
// tiles, as the 1024-row transformer GEMMs are, then have all their workgroups resident at once instead of running
// a second, nearly empty round.
template <int BM, int BN, int D, bool ROWSUM, class AOp, class BOp, class Epi>
__global__ __launch_bounds__(256, (BM == 64 && BN == 64) ? 3 : 2) void gemm2_kernel(AOp A, BOp B, Epi epi, int M, int N, int K, int k_per_slice,
                                                    int col_major, int wide, FastDiv d_plane, FastDiv d_minor) {
    constexpr bool AKC = AOp::kContig, BKC = BOp::kContig;
    constexpr int TM = BM / 64, TN = BN / 64;
    constexpr int A_CH = BM * (kBK2 / 8) / 256, B_CH = BN * (kBK2 / 8) / 256;
    constexpr int A_ELEMS = TileShape<BM, AKC>::elems, B_ELEMS = TileShape<BN, BKC>::elems;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    bf16_t* const sA = reinterpret_cast<bf16_t*>(smem_raw);  // [2][A_ELEMS]
    bf16_t* const sB = sA + 2 * A_ELEMS;                      // [2][B_ELEMS]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    // Workgroups are handed to the 8 XCDs (each with its own L2) round-robin in launch order (x fastest, then y, then
    // z).  Renumber them so that the workgroups of one XCD own a contiguous run of (k-slice, tile) pairs, the tiles of
    // a k-slice next to each other: the tiles of one k-slice read the same k-range of both operands (a split
    // weight gradient: the same positions of dY and of X, nine times over for a 3x3 filter), which then comes in
    // from memory once instead of once per XCD.  Within a k-slice, in row-major order the tiles of a row share their
    // A panel and find it in their own L2, but every XCD fetches all of B; in column-major order (col_major, chosen
    // by the host when B is the larger operand) it is the other way round.
    int tile_x = blockIdx.x, tile_y = blockIdx.y, z = blockIdx.z;
    {
        const int gx = gridDim.x, gy = gridDim.y, nb = gx * gy, total = nb * gridDim.z;
        if (total >= 16) {
            const int lin = (z * gy + tile_y) * gx + tile_x;
            const int xcd = lin & 7, idx = lin >> 3;
            const int q = total >> 3, r = total & 7;
            // (d_plane divides by the tiles of a k-slice, d_minor by the tiles along the direction walked first: the host
            // prepares the multipliers, so that the workgroup reaches its first loads without integer divisions)
            int moved = xcd * q + min(xcd, r) + idx;
            z = (int)d_plane.div((uint32_t)moved);
            moved -= z * nb;
            if (col_major) {
                tile_x = (int)d_minor.div((uint32_t)moved);
                tile_y = moved - tile_x * gy;
            } else {
                tile_y = (int)d_minor.div((uint32_t)moved);
                tile_x = moved - tile_y * gx;
            }
        }
    }
    const int m0 = tile_y * BM, n0 = tile_x * BN;
    // (a loader may walk a k range of its own for this tile, and may keep its rows in another order than memory does:
    // the wide epilogue below asks it for the memory row; the host sends such a loader only there)
    op_begin_tile(A, m0, 0);
    op_begin_tile(B, m0, 0);
    const int k_begin = z * k_per_slice;
    const int k_end = min(op_k_total(A, K, 0), k_begin + k_per_slice);
    const int nk = max(0, (k_end - k_begin + kBK2 - 1) / kBK2);

    typename AOp::KS ksa;
    typename BOp::KS ksb;
    typename AOp::Ctx ca[A_CH];
    typename BOp::Ctx cb[B_CH];
    int sa_off[A_CH], sb_off[B_CH];
    A.init_thread(ksa, k_begin, tid & 7);
    B.init_thread(ksb, k_begin, tid & 7);
#pragma unroll
    for (int i = 0; i < A_CH; ++i) {
        int c = tid + i * 256;
        if constexpr (AKC) {
            int row = c >> 3, kc = c & 7;
            A.init(ca[i], m0 + row, kc, k_begin);
            sa_off[i] = row * TileShape<BM, true>::pitch + kc * 8;
        } else {
            int rc = c % (BM / 8), kl = c / (BM / 8);
            A.init(ca[i], m0 + rc * 8, kl, k_begin);
            sa_off[i] = kl * TileShape<BM, false>::pitch + rc * 8;
        }
    }
#pragma unroll
    for (int i = 0; i < B_CH; ++i) {
        int c = tid + i * 256;
        if constexpr (BKC) {
            int row = c >> 3, kc = c & 7;
            B.init(cb[i], n0 + row, kc, k_begin);
            sb_off[i] = row * TileShape<BN, true>::pitch + kc * 8;
        } else {
            int rc = c % (BN / 8), kl = c / (BN / 8);
            B.init(cb[i], n0 + rc * 8, kl, k_begin);
            sb_off[i] = kl * TileShape<BN, false>::pitch + rc * 8;
        }
    }

    // A wave with a single 32x32 output tile alternates between two accumulators (even and odd 16-k steps), so that
    // consecutive MFMAs do not wait for each other's result; they are added at the end.
    constexpr int NACC = TM * TN == 1 ? 2 : 1;
    f32x16_t acc[NACC][TM][TN];
#pragma unroll
    for (int a = 0; a < NACC; ++a)
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[a][i][j][r] = 0.0f;
    // Row sums of A (ROWSUM): the waves of the first tile column's first wave column add up the A fragments they
    // hold anyway: a lane has 8 consecutive k of its row per fragment, the two half-waves the two halves of 16 k.
    float rsum[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) rsum[i] = 0.0f;
    const bool sums_rows = ROWSUM && tile_x == 0 && wn == 0;

    // Register ring: tile t is fetched into slot t % D.
    uint4 ra[D][A_CH], rb[D][B_CH];
    auto fetch = [&](uint4 (&a)[A_CH], uint4 (&b)[B_CH]) {
#pragma unroll
        for (int i = 0; i < A_CH; ++i) a[i] = A.load(ca[i], ksa, k_end);
#pragma unroll
        for (int i = 0; i < B_CH; ++i) b[i] = B.load(cb[i], ksb, k_end);
        A.next(ksa);
        B.next(ksb);
    };
    auto stash = [&](const uint4 (&a)[A_CH], const uint4 (&b)[B_CH], int buf) {
        bf16_t* da = sA + buf * A_ELEMS;
        bf16_t* db = sB + buf * B_ELEMS;
#pragma unroll
        for (int i = 0; i < A_CH; ++i) *reinterpret_cast<uint4*>(da + sa_off[i]) = a[i];
#pragma unroll
        for (int i = 0; i < B_CH; ++i) *reinterpret_cast<uint4*>(db + sb_off[i]) = b[i];
    };
    // Fetches beyond the slice return zeros (the loaders clamp), so the ring is always kept full and the
    // steady-state loop has no branch around a load or a store.
#pragma unroll
    for (int d = 0; d < D; ++d) fetch(ra[d], rb[d]);
    stash(ra[0], rb[0], 0);
    fetch(ra[0], rb[0]);
    __syncthreads();

    auto multiply = [&](int buf) {
        const bf16_t* tA = sA + buf * A_ELEMS;
        const bf16_t* tB = sB + buf * B_ELEMS;
        // every fragment of the k-tile is requested before the first MFMA: the LDS latency is paid once per k-tile,
        // not once per 16-k step
        constexpr int KK = kBK2 / 16;
        bf16x8_t af[KK][TM], bfr[KK][TN];
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
#pragma unroll
            for (int i = 0; i < TM; ++i) af[kk][i] = read_frag<BM, AKC>(tA, wm * (BM / 2) + i * 32, kk, lane);
#pragma unroll
            for (int j = 0; j < TN; ++j) bfr[kk][j] = read_frag<BN, BKC>(tB, wn * (BN / 2) + j * 32, kk, lane);
        }
#pragma unroll
        for (int kk = 0; kk < KK; ++kk)
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[kk % NACC][i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[kk][i], bfr[kk][j], acc[kk % NACC][i][j], 0, 0, 0);
        if (sums_rows) {
#pragma unroll
            for (int kk = 0; kk < KK; ++kk)
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int e = 0; e < 8; ++e) rsum[i] += (float)af[kk][i][e];
        }
    };

    // Rounds of D tiles; the last round may multiply up to D-1 all-zero tiles.
    const int rounds = (nk + D - 1) / D;
    for (int round = 0; round < rounds; ++round) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            const int kt = round * D + d;
            const int dn = (d + 1) % D;  // compile-time after unrolling
            // LDS buffer (kt+1)&1 was last read in iteration kt-1, which ended with a barrier
            stash(ra[dn], rb[dn], (kt + 1) & 1);
            fetch(ra[dn], rb[dn]);
            multiply(kt & 1);
            __syncthreads();
        }
    }

    if constexpr (NACC == 2) {
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[0][0][0][r] += acc[1][0][0][r];
    }
    // Accumulator layout of the 32x32 MFMA: lane holds column (lane % 32); register r holds
    // row 8*(r/4) + 4*(lane/32) + r%4.  Output offsets advance by additions only.
    const int col_in = lane & 31, row_in = (lane >> 5) * 4;
    const int64_t ld = epi.ld;
    if (wide) {
        // 8-wide form (N a multiple of 8, every tensor of the epilogue 16-byte aligned): each wave transposes a 32x32
        // block of results through LDS (the k-loop ended with a barrier, the tiles are free; a wave uses a region of
        // its own) and leaves with 8 consecutive columns of one row per lane, so that the epilogue reads and writes
        // 16 bytes per lane where the element-wise form below moves 2.  Rows are 40 floats apart: the two half-waves,
        // 4 rows apart, then write to disjoint banks.
        constexpr int SP = 40;
        float* const stage = reinterpret_cast<float*>(smem_raw) + wave * (32 * SP);
        static_assert(4 * 32 * SP * 4 <= gemm2_lds_bytes<BM, BN, AOp, BOp>(), "staging area exceeds the tile buffers");
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                // what the epilogue reads from memory for this block's two groups of rows is requested before the
                // block is transposed, so that the loads fly meanwhile
                typename Epi::Row8 prow[2];
                const int pn = n0 + wn * (BN / 2) + j * 32 + (lane & 3) * 8;
                const typename Epi::Col8 pcol = epi.col8(pn < N ? pn : 0);
#pragma unroll
                for (int ps = 0; ps < 2; ++ps) {
                    const int pm = m0 + wm * (BM / 2) + i * 32 + ps * 16 + (lane >> 2);
                    prow[ps] = epi.row8((int64_t)op_out_row(A, pm < M ? pm : 0, 0) * ld + pn, pm < M && pn < N);
                }
#pragma unroll
                for (int r = 0; r < 16; ++r) stage[(8 * (r >> 2) + row_in + (r & 3)) * SP + col_in] = acc[0][i][j][r];
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                const int n = n0 + wn * (BN / 2) + j * 32 + (lane & 3) * 8;
#pragma unroll
                for (int ps = 0; ps < 2; ++ps) {
                    const int row = ps * 16 + (lane >> 2);
                    const float4 lo = *reinterpret_cast<const float4*>(stage + row * SP + (lane & 3) * 8);
                    const float4 hi = *reinterpret_cast<const float4*>(stage + row * SP + (lane & 3) * 8 + 4);
                    float v[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
                    const int m = m0 + wm * (BM / 2) + i * 32 + row;
                    if (m < M && n < N) epi.at8(pcol, prow[ps], (int64_t)op_out_row(A, m, 0) * ld + n, v, z);
                }
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // staged values are in registers before they are overwritten
            }
    } else if (m0 + BM <= M && n0 + BN <= N) {
        // Interior block: no bounds tests, hence no branch between the stores (a branch makes the
        // compiler wait for every earlier store before the next one).
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int n = n0 + wn * (BN / 2) + j * 32 + col_in;
                const int mb = m0 + wm * (BM / 2) + i * 32 + row_in;
                const int64_t idx = (int64_t)mb * ld + n;
                const auto col = epi.column(n);
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    epi.at(col, idx + (int64_t)(8 * (r >> 2) + (r & 3)) * ld, acc[0][i][j][r], z);
            }
    } else {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int n = n0 + wn * (BN / 2) + j * 32 + col_in;
                if (n >= N) continue;
                const int mb = m0 + wm * (BM / 2) + i * 32 + row_in;
                const int64_t idx = (int64_t)mb * ld + n;
                const auto col = epi.column(n);  // whatever depends on the column only (bias), fetched once
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int m = mb + 8 * (r >> 2) + (r & 3);
                    if (m < M) epi.at(col, idx + (int64_t)(8 * (r >> 2) + (r & 3)) * ld, acc[0][i][j][r], z);
                }
            }
    }
    if (sums_rows) {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const float total = rsum[i] + __shfl_xor(rsum[i], 32);
            const int m = m0 + wm * (BM / 2) + i * 32 + (lane & 31);
            if (lane < 32 && m < M) epi.rowsum(m, total, z);
        }
    }
}

// Split-k partial sums: slice z stores fp32 at part[z][m][n].
struct EpiPartial {
    float* part;
    int64_t ld, slice_stride;
    bool wide_ok() const { return ld % 8 == 0 && slice_stride % 4 == 0 && epi_al16(part); }
    __device__ __forceinline__ int column(int) const { return 0; }
    __device__ __forceinline__ void at(int, int64_t idx, float v, int z) const {
        part[z * slice_stride + idx] = v;
    }
    __device__ __forceinline__ void at8(int, int64_t idx, float (&v)[8], int z) const {
        store8(part + z * slice_stride + idx, v);
    }
    typedef NoCol8 Col8;
    typedef NoRow8 Row8;
    __device__ __forceinline__ Col8 col8(int) const { return Col8{}; }
    __device__ __forceinline__ Row8 row8(int64_t, bool) const { return Row8{}; }
    __device__ __forceinline__ void at8(const Col8&, const Row8&, int64_t idx, float (&v)[8], int z) const {
        store8(part + z * slice_stride + idx, v);
    }
    __device__ __forceinline__ void rowsum(int, float, int) const {}
};

// Reduce the slices and apply the real epilogue.
template <class Epi>
__global__ void splitk_finish_kernel(const float* __restrict__ part, Epi epi, int M, int N, int slices) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t total = (int64_t)M * N;
    if (i >= total) return;
    float a0 = 0.0f, a1 = 0.0f, a2 = 0.0f, a3 = 0.0f;
    int z = 0;
    for (; z + 8 <= slices; z += 8) {   // eight loads in flight; the sums are those of two rounds of the loop below
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = part[(z + u) * total + i];
        a0 += v[0]; a1 += v[1]; a2 += v[2]; a3 += v[3];
        a0 += v[4]; a1 += v[5]; a2 += v[6]; a3 += v[7];
    }
    for (; z + 4 <= slices; z += 4) {
        a0 += part[(z + 0) * total + i];
        a1 += part[(z + 1) * total + i];
        a2 += part[(z + 2) * total + i];
        a3 += part[(z + 3) * total + i];
    }
    for (; z < slices; ++z) a0 += part[z * total + i];
    int m = (int)(i / N), n = (int)(i - (int64_t)m * N);
    epi.at(epi.column(n), (int64_t)m * epi.ld + n, (a0 + a1) + (a2 + a3), 0);
}

// The same for 8 consecutive columns per thread (N a multiple of 8, every tensor of the epilogue 16-byte aligned):
// 16-byte loads of the partial sums and of what the epilogue reads, 16-byte stores; sums in the order of the kernel
// above (slice z goes to accumulator z % 4).
template <class Epi>
__global__ __launch_bounds__(256) void splitk_finish8_kernel(const float* __restrict__ part, Epi epi, int M, int N, int slices) {
    const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int n8 = N >> 3;
    if (c >= (int64_t)M * n8) return;
    const int m = (int)(c / n8), n = (int)(c - (int64_t)m * n8) * 8;
    const int64_t total = (int64_t)M * N, idx = (int64_t)m * epi.ld + n;
    const typename Epi::Col8 pcol = epi.col8(n);
    const typename Epi::Row8 prow = epi.row8(idx, true);
    const float* p = part + (int64_t)m * N + n;
    float a[4][8];
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int e = 0; e < 8; ++e) a[k][e] = 0.0f;
    int z = 0;
    for (; z + 4 <= slices; z += 4) {
        float4 lo[4], hi[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            lo[k] = *reinterpret_cast<const float4*>(p + k * total);
            hi[k] = *reinterpret_cast<const float4*>(p + k * total + 4);
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            a[k][0] += lo[k].x; a[k][1] += lo[k].y; a[k][2] += lo[k].z; a[k][3] += lo[k].w;
            a[k][4] += hi[k].x; a[k][5] += hi[k].y; a[k][6] += hi[k].z; a[k][7] += hi[k].w;
        }
        p += 4 * total;
    }
    for (; z < slices; ++z) {
        const float4 lo = *reinterpret_cast<const float4*>(p), hi = *reinterpret_cast<const float4*>(p + 4);
        a[0][0] += lo.x; a[0][1] += lo.y; a[0][2] += lo.z; a[0][3] += lo.w;
        a[0][4] += hi.x; a[0][5] += hi.y; a[0][6] += hi.z; a[0][7] += hi.w;
        p += total;
    }
    float v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = (a[0][e] + a[1][e]) + (a[2][e] + a[3][e]);
    epi.at8(pcol, prow, idx, v, 0);
}

}  // namespace tmps
