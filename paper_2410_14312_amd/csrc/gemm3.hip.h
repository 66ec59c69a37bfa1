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
#include "gemm2.hip.h"

namespace tmps {

typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef __attribute__((address_space(1))) const void* global_void_ptr;

template <bool KC> struct G3Operand {
    static constexpr bool kContig = KC;
    const bf16_t* p;
    int rows;    // valid rows (m or n extent)
    int64_t ld;  // elements between consecutive rows (KC) or consecutive k (RC)
};

// wait until at most N vector-memory operations of this wave are outstanding
template <int N> __device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N <= 63, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// LDS bytes of one launch
template <int BM, int BN, int BK, int NS> constexpr int gemm3_lds_bytes() { return NS * (BM + BN) * BK * 2; }

// Per-wave copy state of one operand tile of ROWS rows x BK k (BK = 32 or 64): GROUPS 1-KB groups per k-tile.
template <int ROWS, int BK, int NW, bool KC> struct G3Loader {
    static constexpr int GROUPS = ROWS * BK * 2 / 1024 / NW;
    static_assert(GROUPS >= 1 && GROUPS * NW * 1024 == ROWS * BK * 2, "the waves must share a tile evenly");
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
    __device__ __forceinline__ void issue(unsigned char* tile, int64_t ld, int wave) {
#pragma unroll
        for (int g = 0; g < GROUPS; ++g) {
            __builtin_amdgcn_global_load_lds((global_void_ptr)ptr[g], (lds_void_ptr)(tile + (wave + g * NW) * 1024), 16, 0, 0);
            ptr[g] += KC ? BK : BK * ld;
        }
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
    __device__ __forceinline__ bf16x8_t read(const unsigned char* tile, int i, int kk) const {
        if constexpr (KC) {
            return *reinterpret_cast<const bf16x8_t*>(tile + base[0] + i * (32 * BK * 2) + koff[kk]);
        } else {
            typedef __attribute__((address_space(3))) s16x4_t* lds_ptr_t;
            const unsigned char* p0 = tile + koff[0] + kk * 16 * (ROWS * 2) + base[i];
            const unsigned char* p1 = p0 + 4 * (ROWS * 2);
            union { s16x4_t h[2]; bf16x8_t v; } u;
            u.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(p0));
            u.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(p1));
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
// A operand is dY, row-contiguous); the sums go to epi.rowsum(m, v, slice).
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
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
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
    // copy the next k-tile (if any is left) into stage `istage`; returns false when all is issued
    auto issue_next = [&]() -> bool {
        if (iu >= plan.units) return false;
        unsigned char* st = smem + istage * STAGE;
        la.issue(st, A.ld, wave);
        lb.issue(st + A_BYTES, B.ld, wave);
        istage = istage + 1 == NS ? 0 : istage + 1;
        if (++ikt == ink) {
            iu += grid;
            seek_unit();
        }
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
    bf16x8_t af[2][TM], bfr[2][TN];
    int cstage = 0;
    {
        const unsigned char* sa = smem;
#pragma unroll
        for (int i = 0; i < TM; ++i) af[0][i] = fa.read(sa, i, 0);
#pragma unroll
        for (int j = 0; j < TN; ++j) bfr[0][j] = fb.read(sa + A_BYTES, j, 0);
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
        float rsum = 0.0f;

        for (int kt = 0; kt < nk; ++kt) {
            // Invariant: the fragments of this k-tile's first 16 k are in registers (fetched during the previous
            // k-tile's last multiply step); `ahead` younger k-tiles are in flight or have landed.
            const unsigned char* sa = smem + cstage * STAGE;
            const unsigned char* sb = sa + A_BYTES;
            const int nstage = cstage + 1 == NS ? 0 : cstage + 1;
            if constexpr (ROWSUM) {
                if (tn == 0 && tid < BM) {
                    // column tid of the [BK][BM] tile: chunk (tid / 8) ^ ((k & 3) << 2) of k-row k
#pragma unroll 8
                    for (int k = 0; k < BK; ++k)
                        rsum += (float)*reinterpret_cast<const bf16_t*>(sa + k * (BM * 2) + ((((tid >> 3) ^ ((k & 3) << 2)) << 4) | ((tid & 7) << 1)));
                }
            }
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) {
                if (kk < KK - 1) {
#pragma unroll
                    for (int i = 0; i < TM; ++i) af[(kk + 1) & 1][i] = fa.read(sa, i, kk + 1);
#pragma unroll
                    for (int j = 0; j < TN; ++j) bfr[(kk + 1) & 1][j] = fb.read(sb, j, kk + 1);
                } else {
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
                    // All waves are past their last read of the current stage (it is refilled after this k-tile's last
                    // multiply step, or after the unit's results have been staged through it), and the next k-tile
                    // is visible to all: fetch its first fragments under the cover of that multiply step.  (While the
                    // pipeline drains there is no next k-tile: the reads then fetch stale bytes that nothing uses.)
                    {
                        const unsigned char* na = smem + nstage * STAGE;
#pragma unroll
                        for (int i = 0; i < TM; ++i) af[(kk + 1) & 1][i] = fa.read(na, i, 0);
#pragma unroll
                        for (int j = 0; j < TN; ++j) bfr[(kk + 1) & 1][j] = fb.read(na + A_BYTES, j, 0);
                    }
                }
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[kk & 1][i], bfr[kk & 1][j], acc[i][j], 0, 0, 0);
                {
                    // instruction order of this step: one fragment read of the next step, one multiply of this one, in turn
                    constexpr int READS = (AKC ? TM : 2 * TM) + (BKC ? TN : 2 * TN);
                    constexpr int PER = READS > TM * TN ? (READS + TM * TN - 1) / (TM * TN) : 1;
#pragma unroll
                    for (int g = 0; g < TM * TN; ++g) {
                        __builtin_amdgcn_sched_group_barrier(0x100, PER, 0);
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    }
                }
            }
            if (kt + 1 < nk) {
                if (issue_next()) ++ahead;
                --ahead;   // kt + 1 < nk: a next k-tile exists
                cstage = nstage;
            }
        }

        // ---- results ----
        // The stage of the unit's last k-tile is free and not yet refilled: each wave transposes its accumulators
        // through the 8 KB of that stage that its own copies write (so no other wave touches them), 32 rows x 64
        // columns of fp32 at a time, and leaves with 8 consecutive columns of one row per lane: a store
        // instruction then writes 8 rows of 128 (bf16) or 256 (fp32) consecutive bytes.
        {
            unsigned char* stg = smem + cstage * STAGE;
            // piece p (1 KB = 4 staged rows) of this wave: its p-th copy group
            // (computed where it is used: an array of them indexed by the lane's half would live in scratch memory)
            auto piece = [&](int p) {
                return p < LoaderA::GROUPS ? (wave + p * NW) * 1024 : A_BYTES + (wave + (p - LoaderA::GROUPS) * NW) * 1024;
            };
            const int64_t ld = epi.ld;
            const int col_in = lane & 31;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int jp = 0; jp < TN / 2; ++jp) {
                    // what the epilogue reads from memory for the four groups of 8 rows of this block is requested before
                    // the block is transposed: one memory latency per block, not one per group of rows
                    const int n = n0 + wn * (BN / WN) + jp * 64 + (lane & 7) * 8;
                    const typename Epi::Col8 pcol = epi.col8(n < N ? n : 0);
                    typename Epi::Row8 prow[4];
#pragma unroll
                    for (int sp = 0; sp < 4; ++sp) {
                        const int pm = m0 + wm * (BM / WM) + i * 32 + sp * 8 + (lane >> 3);
                        prow[sp] = epi.row8((int64_t)pm * ld + n, pm < M && n < N);
                    }
                    // accumulator register r of a lane: row 8 (r / 4) + 4 half + r % 4, column lane % 32
#pragma unroll
                    for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int base = half ? piece(2 * (r >> 2) + 1) : piece(2 * (r >> 2));
                            *reinterpret_cast<float*>(stg + base + (r & 3) * 256 + (jj * 32 + col_in) * 4) = acc[i][2 * jp + jj][r];
                        }
                    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
                    for (int sp = 0; sp < 4; ++sp) {
                        // staged row 8 sp + lane / 8 lies in piece 2 sp + half, at row (lane / 8) % 4 of the piece
                        const int base = half ? piece(2 * sp + 1) : piece(2 * sp);
                        const unsigned char* src = stg + base + ((lane >> 3) & 3) * 256 + (lane & 7) * 32;
                        const float4 lo = *reinterpret_cast<const float4*>(src), hi = *reinterpret_cast<const float4*>(src + 16);
                        float v[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
                        const int m = m0 + wm * (BM / WM) + i * 32 + sp * 8 + (lane >> 3);
                        if (m < M && n < N) epi.at8(pcol, prow[sp], (int64_t)m * ld + n, v, z);   // N is a multiple of 8
                    }
                    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // staged values are in registers before they are overwritten
                }
        }
        if constexpr (ROWSUM) {
            if (tn == 0 && tid < BM && m0 + tid < M) epi.rowsum(m0 + tid, rsum, z);
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
