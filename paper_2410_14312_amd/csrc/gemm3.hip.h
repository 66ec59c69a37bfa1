// Persistent MFMA GEMM for gfx950 with asynchronous global -> LDS copies (bf16 in, fp32 accumulate), used
// by the dense contractions whose shapes allow it (K a multiple of 64, row counts of row-contiguous
// operands a multiple of 8, 16-byte aligned operands).
//
//   C[m, n] = sum_k A(m, k) * B(n, k)
//
// An operand is k-contiguous (element (row, k) at p[row*ld + k]) or row-contiguous (p[k*ld + row]).
//
// Work decomposition: the output is cut into BM x BN tiles and k into `slices` equal ranges; a work unit
// is (tile, slice).  The grid has one workgroup per compute unit; workgroup b (renumbered so that the workgroups
// of an XCD are neighbours) processes units b, b + grid, b + 2 grid, ...  The k-loop is software-pipelined ACROSS units: the copies of the next
// NS-1 k-tiles are always in flight, also over a unit boundary, so a unit's first tiles arrive while the
// previous unit is still being multiplied and its results are being stored.  Short contractions (a dozen
// k-tiles per unit) therefore pay the memory latency once per workgroup, not once per tile.
//
// Copies: one wave instruction copies 64 x 16 bytes from per-lane global addresses to 1 KB of consecutive
// LDS (global_load_lds_dwordx4); nothing is staged in registers.  LDS tiles are unpadded; bank conflicts
// are avoided by permuting 16-byte chunks with an XOR of the row (k-contiguous tiles, [rows][64]) or of k
// (row-contiguous tiles, [64][rows]), which only changes WHICH global chunk a lane fetches.
// Fragments: k-contiguous tiles are read with 16-byte LDS reads, row-contiguous ones with the transpose
// read of gfx950.  Results are transposed through LDS on their way out, so that every lane stores 16 bytes and
// a store instruction covers whole 128-byte lines: the wave must wait for its stores before it can tell that
// a later copy has landed (both are counted by the same counter), so slow scattered stores would stall the
// k-loop of the next unit.
#pragma once
#include <type_traits>

#include "gemm2.hip.h"

namespace tmps {

// LDS is addressed by 32-bit byte addresses throughout this kernel (lds_t), turned into LDS pointers where a value is
// read or written: generic pointers into LDS make the compiler carry null checks and aperture tests around (and, in
// some arrangements of this kernel's control flow, fail in its instruction verifier).
typedef uint32_t lds_t;
template <class T> __device__ __forceinline__ __attribute__((address_space(3))) T* lds_ptr(lds_t a) {
    return (__attribute__((address_space(3))) T*)(uintptr_t)a;
}

template <bool KC> struct G3Operand {
    static constexpr bool kContig = KC;
    const bf16_t* p;
    int rows;    // valid rows (m or n extent)
    int64_t ld;  // elements between consecutive rows (KC) or consecutive k (RC)
};

// wait until at most N vector-memory operations of this wave are outstanding
// (the trailing comment tells this wait from the ones the compiler inserts, for tests/test_gemm3_isa.py)
template <int N> __device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N <= 63, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0) ; tmps" ::"n"(N) : "memory");
}

// One wave instruction that copies 16 bytes per lane from `src` (per lane) to 1 KB of consecutive LDS at `dst` (the same
// for all lanes).  Written out as instructions rather than through the compiler's builtin: the compiler cannot tell
// which LDS reads a copy in flight may alias and makes the wave wait for ALL its outstanding copies before the next
// LDS read it sees, which serialises the copy pipeline; here the kernel's own counter waits and barriers order copies
// and reads (a stage is read only after the wait and barrier that follow its copies, and refilled only after the
// barrier that follows its last read).
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"   // m0 is reserved: the compiler keeps nothing in it across statements
__device__ __forceinline__ void copy16_to_lds(const void* src, lds_t dst) {
    const uint32_t lds = __builtin_amdgcn_readfirstlane(dst);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds), "v"(src) : "memory", "m0");
}
#pragma clang diagnostic pop

// Makes the compiler treat every 32-bit word of `t` (values requested from memory earlier) as read here, on every
// path: a request whose result is never read stays "in flight" in the compiler's book-keeping, and the wait it then
// inserts wherever the register is next written — in the k-loop of the following unit — would drain the copy pipeline
// on every k-tile.
template <class T> __device__ __forceinline__ void settle(const T& t) {
    if constexpr (!std::is_empty<T>::value) {
        static_assert(sizeof(T) % 4 == 0, "whole registers");
        uint32_t w[sizeof(T) / 4];
        __builtin_memcpy(w, &t, sizeof(T));
#pragma unroll
        for (unsigned i = 0; i < sizeof(T) / 4; ++i) asm volatile("" ::"v"(w[i]));
    }
}

// LDS bytes of one launch
template <int BM, int BN, int BK, int NS> constexpr int gemm3_lds_bytes() { return NS * (BM + BN) * BK * 2; }

// Per-wave copy state of one operand tile of ROWS rows x BK k (BK = 32 or 64): GROUPS 1-KB groups per k-tile.
template <int ROWS, int BK, int NW, bool KC> struct G3Loader {
    static constexpr int GROUPS = ROWS * BK * 2 / 1024 / NW;
    static_assert(GROUPS >= 1 && GROUPS * NW * 1024 == ROWS * BK * 2, "the waves must share a tile evenly");
    static_assert(KC || (ROWS / 8 <= 64 && 64 % (ROWS / 8) == 0), "a 1 KB group of a row-contiguous tile covers whole k-rows");
    const bf16_t* ptr[GROUPS];
    // (re)compute the lane addresses for the tile starting at row0, k range starting at k0
    __device__ __forceinline__ void seek(const G3Operand<KC>& op, int row0, int k0, int wave, int lane) {
#pragma unroll
        for (int g = 0; g < GROUPS; ++g) {
            const int grp = wave + g * NW;
            if constexpr (KC) {
                // LDS tile [ROWS][BK]; a group is 1 KB of consecutive rows; the 16-byte chunk at (r, p) holds global
                // chunk p ^ s(r) of row r, s(r) = (r >> 1) & 7 for BK = 64 (8 chunks per row), (r >> 2) & 3 for BK = 32
                constexpr int CPR = BK / 8;   // chunks per row
                const int r = grp * (64 / CPR) + lane / CPR;
                const int c = (lane % CPR) ^ (BK == 64 ? ((r >> 1) & 7) : ((r >> 2) & 3));
                int gr = row0 + r;
                gr = gr < op.rows ? gr : op.rows - 1;
                ptr[g] = op.p + (int64_t)gr * op.ld + k0 + c * 8;
            } else {
                // LDS tile [BK][ROWS]; the chunk at (k, p) holds rows 8 * (p ^ ((k & 3) << 2)) .. + 7 of k
                constexpr int CPR = ROWS / 8;  // chunks per k-row
                const int k = grp * (64 / CPR) + lane / CPR;
                const int c = (lane % CPR) ^ ((k & 3) << 2);
                int r = row0 + c * 8;
                r = r + 8 <= op.rows ? r : op.rows - 8;
                ptr[g] = op.p + (int64_t)(k0 + k) * op.ld + r;
            }
        }
    }
    // copy this wave's groups of the current k-tile into `tile` (LDS) and step to the next k-tile
    __device__ __forceinline__ void issue(lds_t tile, int64_t ld, int wave) {
#pragma unroll
        for (int g = 0; g < GROUPS; ++g) issue_group(tile, ld, wave, g);
    }
    // the same, one group at a time (every group of a k-tile exactly once, in any order)
    __device__ __forceinline__ void issue_group(lds_t tile, int64_t ld, int wave, int g) {
        copy16_to_lds(ptr[g], tile + (wave + g * NW) * 1024);
        ptr[g] += KC ? BK : BK * ld;
    }
};

// Fragment reader of one operand for a wave whose first row in the tile is wrow0: T fragments of 32 rows.
template <int ROWS, int BK, int T, bool KC> struct G3Frags {
    static constexpr int KK = BK / 16;
    int base[KC ? 1 : T];   // byte offsets that depend on the lane (and, for RC, on the fragment)
    int koff[KC ? KK : 1];
    __device__ __forceinline__ void init(int wrow0, int lane) {
        if constexpr (KC) {
            // s(row) of row = wrow0 + 32 i + lane % 32 depends on the lane only
            const int half = lane >> 5, swz = BK == 64 ? ((lane >> 1) & 7) : ((lane >> 2) & 3);
            base[0] = (wrow0 + (lane & 31)) * (BK * 2);
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) koff[kk] = ((kk * 2 + half) ^ swz) << 4;
        } else {
            // transpose read: lane supplies 4 consecutive rows (8 bytes) at k = 16 kk + 8 half + (lane % 16) / 4,
            // rows rb + 16 ((lane / 16) % 2) + 4 (lane % 4); a second read 4 k further completes the 8 k of a lane
            const int kl = (lane >> 5) * 8 + ((lane & 15) >> 2);
            const int sw = ((lane >> 2) & 3) << 2;   // (k & 3) << 2
            koff[0] = kl * (ROWS * 2);
#pragma unroll
            for (int i = 0; i < T; ++i) {
                const int col = wrow0 + 32 * i + ((lane >> 4) & 1) * 16 + (lane & 3) * 4;
                base[i] = (((col >> 3) ^ sw) << 4) + (col & 7) * 2;
            }
        }
    }
    __device__ __forceinline__ bf16x8_t read(lds_t tile, int i, int kk) const {
        if constexpr (KC) {
            return *lds_ptr<const bf16x8_t>(tile + base[0] + i * (32 * BK * 2) + koff[kk]);
        } else {
            const lds_t p0 = tile + koff[0] + kk * 16 * (ROWS * 2) + base[i];
            const lds_t p1 = p0 + 4 * (ROWS * 2);
            union { s16x4_t h[2]; bf16x8_t v; } u;
            u.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(lds_ptr<s16x4_t>(p0));
            u.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(lds_ptr<s16x4_t>(p1));
            return u.v;
        }
    }
};

// Work geometry, computed on the host.
struct G3Plan {
    int tiles_m, tiles_n, slices, k_per_slice;  // k_per_slice a multiple of the kernel's BK
    int units;                                  // tiles_m * tiles_n * slices
    int col_major;                              // consecutive units walk down a column of tiles (share B) instead of along a row (share A)
    FastDiv d_tn, d_tiles;                      // by tiles_n (tiles_m when col_major) and by tiles_m * tiles_n
    // gm > 0: the tiles of a slice are numbered block by block, a block being gm x gn tiles (gm * gn = 32, the
    // workgroups of one XCD in a round; gm divides tiles_m, gn divides tiles_n): the 32 tiles an XCD works on at a time
    // then share gm + gn operand panels instead of 1 + 32, and most LDS fills find their lines in the XCD's L2.
    int gm, gn;
    FastDiv d_blk, d_gn, d_nbn;                 // by 32, by gn, by tiles_n / gn
};

// ROWSUM: units of the first tile column also sum A over k (bias gradient of a weight-gradient GEMM, whose
// A operand is dY, row-contiguous), from the fragments in registers; the sums go to epi.rowsum(m, v, slice).
template <int BM, int BN, int BK, int WM, int WN, int NS, bool AKC, bool BKC, bool ROWSUM, class Epi>
__global__ __launch_bounds__(64 * WM * WN) void gemm3_kernel(G3Operand<AKC> A, G3Operand<BKC> B, Epi epi, int M, int N,
                                                              int K, G3Plan plan) {
    constexpr int NW = WM * WN, NT = 64 * NW;
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    constexpr int KK = BK / 16;
    constexpr int A_BYTES = BM * BK * 2, STAGE = (BM + BN) * BK * 2;
    typedef G3Loader<BM, BK, NW, AKC> LoaderA;
    typedef G3Loader<BN, BK, NW, BKC> LoaderB;
    constexpr int G = LoaderA::GROUPS + LoaderB::GROUPS;   // copy instructions per wave and k-tile
    static_assert((NS - 1) * G <= 63, "too many copies in flight for the vmcnt counter");
    static_assert(!ROWSUM || !AKC, "row sums are built for a row-contiguous A");
    static_assert(TN % 2 == 0 && G >= 8, "results are staged 32 x 64 at a time through 8 KB of a wave's own copy targets");
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem_raw[];
    const lds_t smem = (lds_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem_raw;

    const int tid = threadIdx.x, lane = tid & 63;
    // (the wave's index as a scalar: what derives from it — LDS addresses of its copies, its place in the tile — then
    // lives in scalar registers and is computed by the scalar unit)
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN, half = lane >> 5;
    const int grid = gridDim.x;
    // Workgroups are handed to the 8 XCDs (each with its own L2) round-robin in launch order.  Renumber them so that
    // the workgroups of one XCD take CONSECUTIVE units of every round: consecutive units are tiles of one row and
    // slice, which share their A panel (and all of them the few B panels), so an XCD fetches a panel once instead
    // of every XCD fetching every panel.
    int vb = blockIdx.x;
    {
        const int xcd = vb & 7, idx = vb >> 3, q = grid >> 3, r = grid & 7;
        vb = xcd * q + min(xcd, r) + idx;
    }

    auto unit_coords = [&](int u, int& tm, int& tn, int& z) {
        uint32_t zz, rem, m_, n_;
        plan.d_tiles.divmod((uint32_t)u, zz, rem);
        if (plan.gm) {
            uint32_t blk, w, bm, bn, i, j;
            plan.d_blk.divmod(rem, blk, w);
            plan.d_nbn.divmod(blk, bm, bn);
            plan.d_gn.divmod(w, i, j);
            m_ = bm * plan.gm + i;
            n_ = bn * plan.gn + j;
        } else if (plan.col_major) plan.d_tn.divmod(rem, n_, m_);
        else plan.d_tn.divmod(rem, m_, n_);
        z = (int)zz; tm = (int)m_; tn = (int)n_;
    };
    auto unit_nk = [&](int z) {
        const int kb = z * plan.k_per_slice;
        const int ke = min(K, kb + plan.k_per_slice);
        return (ke - kb) / BK;
    };

    // ---- copy cursor: runs NS-1 k-tiles ahead of the multiply cursor ----
    LoaderA la;
    LoaderB lb;
    int iu = vb, ikt = 0, ink = 0, istage = 0;
    auto seek_unit = [&]() {
        if (iu < plan.units) {
            int tm, tn, z;
            unit_coords(iu, tm, tn, z);
            ink = unit_nk(z);
            la.seek(A, tm * BM, z * plan.k_per_slice, wave, lane);
            lb.seek(B, tn * BN, z * plan.k_per_slice, wave, lane);
        }
        ikt = 0;
    };
    auto copies_left = [&]() { return iu < plan.units; };
    // copy group g (of G) of the cursor's k-tile into stage `istage`
    auto issue_group = [&](int g) {
        const lds_t st = smem + istage * STAGE;
        if (g < LoaderA::GROUPS) la.issue_group(st, A.ld, wave, g);
        else lb.issue_group(st + A_BYTES, B.ld, wave, g - LoaderA::GROUPS);
    };
    // all G groups of the cursor's k-tile are issued: step the cursor
    auto advance = [&]() {
        istage = istage + 1 == NS ? 0 : istage + 1;
        if (++ikt == ink) {
            iu += grid;
            seek_unit();
        }
    };
    // copy the cursor's whole k-tile (if any is left); returns false when all is issued
    auto issue_next = [&]() -> bool {
        if (!copies_left()) return false;
#pragma unroll
        for (int g = 0; g < G; ++g) issue_group(g);
        advance();
        return true;
    };

    G3Frags<BM, BK, TM, AKC> fa;
    G3Frags<BN, BK, TN, BKC> fb;
    fa.init(wm * (BM / WM), lane);
    fb.init(wn * (BN / WN), lane);

    seek_unit();
    int ahead = 0;   // k-tiles issued beyond the one being multiplied
#pragma unroll
    for (int s = 0; s < NS; ++s)
        if (issue_next()) ++ahead;
    if (ahead == 0) return;   // no unit for this workgroup (uniform)
    --ahead;
    // first k-tile: wait for it, make it visible to all waves, fetch its first fragments
    if (ahead == NS - 1) wait_vmcnt<(NS - 1) * G>();
    else wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    // Fragments are fetched PD multiply steps (of 16 k) ahead of their use.  With two waves per SIMD one step is
    // enough: the other wave's multiplies cover a wave's LDS latency.  With one wave per SIMD (the 4-wave instances)
    // a fragment requested during a step of TM * TN multiplies has not arrived when the next step starts, so these
    // run two steps ahead, with four sets of fragment registers.
    constexpr int PD = NW <= 4 ? 2 : 1, NBUF = PD == 2 ? 4 : 2;
    static_assert(PD < KK && KK % NBUF == 0, "the fragment sets rotate once per k-tile");
    bf16x8_t af[NBUF][TM], bfr[NBUF][TN];
    int cstage = 0;
    {
        const lds_t sa = smem;
#pragma unroll
        for (int p = 0; p < PD; ++p) {
#pragma unroll
            for (int i = 0; i < TM; ++i) af[p][i] = fa.read(sa, i, p);
#pragma unroll
            for (int j = 0; j < TN; ++j) bfr[p][j] = fb.read(sa + A_BYTES, j, p);
        }
    }

    for (int cu = vb; cu < plan.units; cu += grid) {
        int tm, tn, z;
        unit_coords(cu, tm, tn, z);
        const int nk = unit_nk(z);
        const int m0 = tm * BM, n0 = tn * BN;
        f32x16_t acc[TM][TN];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
        // ROWSUM: in units of the first tile column the waves add up the A fragments they multiply with anyway (a lane
        // holds 8 consecutive k of one row: four two-element dot products with ones).  The WN waves of a wave row hold
        // the same fragments: wave column c takes the fragments i with i % WN == c, so that no wave falls behind.
        float rs[TM];
#pragma unroll
        for (int i = 0; i < TM; ++i) rs[i] = 0.0f;
        const bool sum_rows = ROWSUM && tn == 0;

        // What the epilogue reads from memory (a bias per column, a residual source or a mask per element), block by
        // block of 32 rows x 64 columns of this wave's results (block b: rows 32 (b / (TN / 2)), columns 64 (b % (TN / 2))).
        constexpr int NB = TM * (TN / 2);
        const int64_t epi_ld = epi.ld;
        typename Epi::Col8 pcol[TN / 2];
        typename Epi::Row8 prow[NB][4];
        // (ln: the lane's index as the caller has it; see the epilogue)
        auto epi_n = [&](int jp, int ln) { return n0 + wn * (BN / WN) + jp * 64 + (ln & 7) * 8; };
        auto epi_request = [&](int b, int ln) {
            const int i = b / (TN / 2), jp = b % (TN / 2), n = epi_n(jp, ln);
            if (i == 0) pcol[jp] = epi.col8(n < N ? n : 0);
#pragma unroll
            for (int sp = 0; sp < 4; ++sp) {
                const int pm = m0 + wm * (BM / WM) + i * 32 + sp * 8 + (ln >> 3);
                prow[b][sp] = epi.row8((int64_t)pm * epi_ld + n, pm < M && n < N);
            }
        };
        // With registers to spare (the 4-wave instances: 512 per lane) all of it is requested before the k-loop; the
        // 8-wave instances, which would spill, request a block's data when they come to the block.  A wave waits for
        // its requests in issue order, stores included: waiting for data requested after a store means waiting for the
        // store to be acknowledged.
        constexpr bool EARLY = NW <= 4;
        if constexpr (EARLY) {
#pragma unroll
            for (int b = 0; b < NB; ++b) epi_request(b, lane);
        }

        for (int kt = 0; kt < nk; ++kt) {
            // Invariant: the fragments of this k-tile's first PD multiply steps are in registers or on their way
            // (requested during the previous k-tile's last PD steps); `ahead` younger k-tiles are in flight or have landed.
            asm volatile("; tmps k-tile begin");
            const lds_t sa = smem + cstage * STAGE;
            const int nstage = cstage + 1 == NS ? 0 : cstage + 1;
            // After the barrier of this k-tile its stage is free; unless the unit's results go through it first (the
            // unit's last k-tile) it is refilled at once, the copies spread over the multiplies that follow the barrier.
            bool fill = false;
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) {
                const int nx = kk + PD;   // the step whose fragments are requested during this one
                if (nx == KK) {
                    // Every fragment of this k-tile has been requested.  The next k-tile is the oldest copy in
                    // flight: copies complete in issue order, so it has landed once at most (ahead - 1) * G younger
                    // copies are outstanding.  Result stores of an earlier unit are younger than it too and only
                    // make the wait stricter.  While the pipeline drains (ahead < NS - 1) wait for everything.
                    if (ahead > 0) {
                        if (ahead == NS - 1) wait_vmcnt<(NS - 2) * G>();
                        else wait_vmcnt<0>();
                    }
                    __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0): this wave's reads of the current stage are done
                    __builtin_amdgcn_s_barrier();
                    // All waves are past their last read of the current stage, and the next k-tile is visible to all:
                    // its first fragments are fetched under the cover of the remaining multiply steps.  (While the
                    // pipeline drains there is no next k-tile: the reads then fetch stale bytes that nothing uses.)
                    fill = kt + 1 < nk && copies_left();
                }
                // This step in program order, kept by the scheduling barriers: before multiply g, the g-th share of
                // the fragment requests of step nx and, after the barrier, of the copies: a wave has one instruction
                // stream, and what it issues between two multiplies costs nothing while the matrix unit is busy.
                const lds_t ra = nx < KK ? sa : smem + nstage * STAGE;
                const int rk = nx < KK ? nx : nx - KK;
                constexpr int NM = TM * TN, NR = TM + TN, CPS = G / PD;
                static_assert(G % PD == 0, "the copies of a k-tile are spread evenly over the steps after the barrier");
#pragma unroll
                for (int g = 0; g < NM; ++g) {
#pragma unroll
                    for (int r = g * NR / NM; r < (g + 1) * NR / NM; ++r) {
                        if (r < TM) af[nx % NBUF][r] = fa.read(ra, r, rk);
                        else bfr[nx % NBUF][r - TM] = fb.read(ra + A_BYTES, r - TM, rk);
                    }
                    if (nx >= KK) {
                        if (fill) {
#pragma unroll
                            for (int c = g * CPS / NM; c < (g + 1) * CPS / NM; ++c) issue_group((nx - KK) * CPS + c);
                        }
                    }
                    acc[g / TN][g % TN] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[kk % NBUF][g / TN], bfr[kk % NBUF][g % TN], acc[g / TN][g % TN], 0, 0, 0);
                    if constexpr (ROWSUM) {
                        // Behind the fragment's first multiply, so that it is issued while that one runs; written as
                        // instructions because the compiler otherwise turns the branch into selects and moves the
                        // additions, which nothing in the loop depends on, below the multiplies of the k-tile.
                        if (g % TN == 0 && sum_rows && (g / TN) % WN == wn) {
                            typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
                            const u32x4_t f = __builtin_bit_cast(u32x4_t, af[kk % NBUF][g / TN]);
#pragma unroll
                            for (int q = 0; q < 4; ++q)   // rs += f[q].lo * 1 + f[q].hi * 1 (0x3f80 = 1.0 in bf16)
                                asm volatile("v_dot2c_f32_bf16_e32 %0, 0x3f803f80, %1" : "+v"(rs[g / TN]) : "v"(f[q]));
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            if (fill) {
                advance();
                ++ahead;
            }
            if (kt + 1 < nk) {
                --ahead;   // kt + 1 < nk: a next k-tile exists
                cstage = nstage;
            }
            asm volatile("; tmps k-tile end");
        }

        // ---- results ----
        // The stage of the unit's last k-tile is free and not yet refilled: each wave transposes its accumulators
        // through the 8 KB of that stage that its own copies write (so no other wave touches them), one block of
        // 32 rows x 64 columns of fp32 at a time, and leaves with 8 consecutive columns of one row per lane: a store
        // instruction then writes 8 rows of 128 (bf16) or 256 (fp32) consecutive bytes.
        {
            const lds_t stg = smem + cstage * STAGE;
            // piece p (1 KB = 4 staged rows) of this wave: its p-th copy group
            // (computed where it is used: an array of them indexed by the lane's half would live in scratch memory)
            auto piece = [&](int p) {
                return p < LoaderA::GROUPS ? (wave + p * NW) * 1024 : A_BYTES + (wave + (p - LoaderA::GROUPS) * NW) * 1024;
            };
            // Everything the epilogue derives from the lane's index is derived here, from a copy of the index that the
            // compiler cannot trace back: otherwise it computes these offsets before the k-loop and, in the 8-wave
            // instances, whose loop leaves no register free, spills them around it — and every reload from scratch
            // memory is a wait for all of the wave's requests, result stores included.
            int ln = lane;
            asm volatile("" : "+v"(ln));
            const int half = ln >> 5, col_in = ln & 31;
            if constexpr (EARLY) {
#pragma unroll
                for (int b = 0; b < NB; ++b) {
                    if (b < TN / 2) settle(pcol[b]);
#pragma unroll
                    for (int sp = 0; sp < 4; ++sp) settle(prow[b][sp]);
                }
            }
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const int i = b / (TN / 2), jp = b % (TN / 2);
                // (requested before the block is transposed: one memory latency per block, not one per group of rows)
                if constexpr (!EARLY) epi_request(b, ln);
                const int n = epi_n(jp, ln);
                // accumulator register r of a lane: row 8 (r / 4) + 4 half + r % 4, column lane % 32
#pragma unroll
                for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int base = half ? piece(2 * (r >> 2) + 1) : piece(2 * (r >> 2));
                        *lds_ptr<float>(stg + base + (r & 3) * 256 + (jj * 32 + col_in) * 4) = acc[i][2 * jp + jj][r];
                    }
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                if constexpr (!EARLY) {
                    // before the block's first store, where the block's data is the wave's youngest request
                    if (i == 0) settle(pcol[jp]);
#pragma unroll
                    for (int sp = 0; sp < 4; ++sp) settle(prow[b][sp]);
                }
#pragma unroll
                for (int sp = 0; sp < 4; ++sp) {
                    // staged row 8 sp + lane / 8 lies in piece 2 sp + half, at row (lane / 8) % 4 of the piece
                    const int base = half ? piece(2 * sp + 1) : piece(2 * sp);
                    const lds_t src = stg + base + ((ln >> 3) & 3) * 256 + (ln & 7) * 32;
                    typedef float f32x4_t __attribute__((ext_vector_type(4)));
                    const f32x4_t lo = *lds_ptr<const f32x4_t>(src), hi = *lds_ptr<const f32x4_t>(src + 16);
                    float v[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
                    const int m = m0 + wm * (BM / WM) + i * 32 + sp * 8 + (ln >> 3);
                    if (m < M && n < N) epi.at8(pcol[jp], prow[b][sp], (int64_t)m * epi_ld + n, v, z);   // N is a multiple of 8
                }
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // staged values are in registers before they are overwritten
            }
        }
        if constexpr (ROWSUM) {
            if (sum_rows) {
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    if (i % WN != wn) continue;
                    // lanes l and l + 32 hold the two halves of every 16 k of row 32 i + l % 32
                    const float total = rs[i] + __shfl_xor(rs[i], 32, 64);
                    const int m = m0 + wm * (BM / WM) + i * 32 + (lane & 31);
                    if (lane < 32 && m < M) epi.rowsum(m, total, z);
                }
            }
        }
        // refill the stage the results went through, and move on to the next unit's first k-tile
        if (issue_next()) ++ahead;
        if (ahead > 0) {
            --ahead;
            cstage = cstage + 1 == NS ? 0 : cstage + 1;
        }
    }
    (void)NT;
}

}  // namespace tmps
