// The block mask of a small grid, drawn inside a GEMM kernel and held in registers (included by the GEMM translation
// units only).
//
// The paper found mask generation to dominate the run time of small layers (Section 3.4).  Here the mask kernel of a
// step and the launch boundary behind it cost about 15 us, a tenth of a 4096^3 step and a fifth of an 8192 x 1024 x 1024
// one.  For block grids of at most 128 rows and 64 columns every workgroup of the forward kernel therefore draws the
// whole mask itself: the generator is counter-based, a block's keep flag depends on (seed, stream, block number, p)
// only, so every workgroup arrives at the same bits without talking to anyone.  A block row's flags are one 64-bit
// word; lane l of every wavefront keeps the words of rows l and l + 64, and everything the forward kernel looks up in a
// mask object (the heaviest-first order of the rows, a row's kept columns) is computed from those registers:
// no dependent chain of global loads at the start of the kernel.  The mask object that the backward kernels read is
// written by the same launch, cut into small independent pieces that the computing wavefronts of all workgroups share
// while they wait for their first operands.
#ifndef SDROP_GEMM_SEEDED_GRID_H
#define SDROP_GEMM_SEEDED_GRID_H
#include "gemm_device_common.h"

namespace sdrop {
namespace {

constexpr int kSeededMaxRows = 128, kSeededMaxCols = 64;

// number of set bits of `mask` that belong to lanes below this one
__device__ __forceinline__ int below_count(uint64_t mask)
{
    return (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}
// Sum of v (0 <= v < 2^BITS) over the lanes below this one, and over all lanes, without LDS traffic or shuffles: one
// ballot per bit of v, whose set bits are counted below the lane and altogether.
template <int BITS> __device__ __forceinline__ int excl_prefix(int v, int &total)
{
    int pre = 0;
    total = 0;
#pragma unroll
    for (int b = 0; b < BITS; ++b) {
        const uint64_t m = __ballot((v >> b) & 1);
        pre += below_count(m) << b;
        total += (int)__popcll(m) << b;
    }
    return pre;
}

struct SeededGrid {
    uint64_t rw[2];     // keep bits of block rows lane and lane + 64 (0 for rows that do not exist)
    int cnt[2];         // kept blocks of those rows
    int ord[2];         // the block rows at places lane and lane + 64 of the heaviest-first order (more kept blocks
                        // first, ties: lower row first)
    int ccnt;           // kept blocks of block column `lane` (0 for columns that do not exist)
    int MB, KB;

    // LDS the draw needs: the row words, the order, the column counts
    static constexpr int kLdsBytes = kSeededMaxRows * 8 + kSeededMaxRows * 4 + kSeededMaxCols * 4;

    // keep bits of block row i (uniform)
    __device__ __forceinline__ uint64_t row_word(int i) const
    {
        const uint64_t v = i < 64 ? rw[0] : rw[1];
        const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, i & 63);
        const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), i & 63);
        return ((uint64_t)hi << 32) | lo;
    }
    __device__ __forceinline__ int row_count(int i) const { return __builtin_amdgcn_readlane(i < 64 ? cnt[0] : cnt[1], i & 63); }
    // the block row at place q of the heaviest-first order (uniform q < MB)
    __device__ __forceinline__ int row_of_rank(int q) const { return __builtin_amdgcn_readlane(q < 64 ? ord[0] : ord[1], q & 63); }

    // Draws the grid.  Every wavefront of the workgroup takes its share of the rows (a wavefront draws 64 / (KB
    // rounded up to a power of two) rows per ballot, so that no lane idles through the Philox rounds) and the row
    // words meet in LDS; every wavefront reads all of them back, ranks its share of the rows (rank = number of
    // rows with a larger key, two ballots per row; the key count * 1024 + (1023 - row) is the one the mask kernel
    // sorts by) and the order meets in LDS the same way.  `lds` (kLdsBytes) must stay untouched by anyone else
    // until every wavefront has passed one more barrier after this call.  Called by all wavefronts of the workgroup.
    __device__ __forceinline__ void draw(const GemmParams &P, char *lds)
    {
        uint64_t *const s_words = reinterpret_cast<uint64_t *>(lds);
        int32_t *const s_order = reinterpret_cast<int32_t *>(lds + kSeededMaxRows * 8);
        int32_t *const s_ccnt = s_order + kSeededMaxRows;
        const int lane = threadIdx.x & 63;
        const int wave = uni((int)(threadIdx.x >> 6)), nwaves = (int)(blockDim.x >> 6);
        MB = P.MB; KB = P.KB;
        int kshift = 0;
        while ((1 << kshift) < KB) ++kshift;
        const int kbp = 1 << kshift, R = 64 >> kshift, sub = lane >> kshift, j = lane & (kbp - 1);
        for (int b = wave; b * R < MB; b += nwaves) {
            const int i = b * R + sub;
            bool keep = false;
            if (i < MB && j < KB) {
                const uint32_t blk = __umul24((uint32_t)i, (uint32_t)KB) + (uint32_t)j;   // the block number b = i KB + j of the generator's counter
                keep = (uint64_t)philox_word0(blk, 0u, P.ctr2, P.ctr3, P.key0, P.key1) >= P.threshold;
            }
            const uint64_t all = __ballot(keep);
            if (j == 0 && i < MB) s_words[i] = kbp == 64 ? all : ((all >> (sub * kbp)) & ((uint64_t(1) << kbp) - 1));
        }
        __syncthreads();
        int key[2];
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const int i = lane + 64 * r;
            rw[r] = i < MB ? s_words[i] : 0;
            cnt[r] = (int)__popcll(rw[r]);
            key[r] = i < MB ? cnt[r] * 1024 + (1023 - i) : -1;
        }
        for (int i = wave; i < MB; i += nwaves) {
            const int ki = __builtin_amdgcn_readlane(i < 64 ? key[0] : key[1], i & 63);
            const int rank = (int)__popcll(__ballot(key[0] > ki)) + (int)__popcll(__ballot(key[1] > ki));
            if (lane == 0) s_order[rank] = i;
        }
        // kept counts of the block columns, shared the same way: a column's keep bits are a ballot over the rows
        for (int jc = wave; jc < KB; jc += nwaves) {
            const int c = (int)__popcll(__ballot((rw[0] >> jc) & 1)) + (int)__popcll(__ballot((rw[1] >> jc) & 1));
            if (lane == 0) s_ccnt[jc] = c;
        }
        __syncthreads();
#pragma unroll
        for (int r = 0; r < 2; ++r) ord[r] = lane + 64 * r < MB ? s_order[lane + 64 * r] : 0;
        ccnt = lane < KB ? s_ccnt[lane] : 0;
    }

    // ---- the mask object, in pieces ----
    // Piece numbers: 0 = header, bits, col_ptr, col_order; 1 = row_ptr, row_order; 2 = the pair list and its length
    // in the header; then one per block row (its part of col_idx / blk_row), one per block column (its part of
    // row_idx), one per group of 8 block rows (its part of loc_row / loc_col).  Every piece is computed from the registers alone and writes a part of the object that no
    // other piece writes; the result is what sdrop_mask builds (same lists, same tie-breaking).
    __device__ __forceinline__ int pieces() const { return 3 + MB + KB + (MB + 7) / 8; }

    // exclusive prefix sums of the rows' kept counts, for this lane's two rows; total = number of kept blocks
    __device__ __forceinline__ void row_starts(int (&start)[2], int &total) const
    {
        int t0, t1;
        start[0] = excl_prefix<7>(cnt[0], t0);
        start[1] = t0;
        t1 = 0;
        if (MB > 64) start[1] += excl_prefix<7>(cnt[1], t1);        // uniform branch
        total = t0 + t1;
    }
    __device__ __forceinline__ int start_of_row(const int (&start)[2], int i) const
    {
        return __builtin_amdgcn_readlane(i < 64 ? start[0] : start[1], i & 63);
    }

    __device__ __forceinline__ void write_piece(const GemmParams &P, int piece) const
    {
        const int lane = threadIdx.x & 63;
        const MaskView &mv = P.mv;
        // the object is this launch's output although the GEMM parameters describe it as an input
        int32_t *const row_ptr = const_cast<int32_t *>(mv.row_ptr), *const col_idx = const_cast<int32_t *>(mv.col_idx);
        int32_t *const blk_row = const_cast<int32_t *>(mv.blk_row), *const col_ptr = const_cast<int32_t *>(mv.col_ptr);
        int32_t *const row_idx = const_cast<int32_t *>(mv.row_idx), *const row_order = const_cast<int32_t *>(mv.row_order);
        int32_t *const col_order = const_cast<int32_t *>(mv.col_order);
        int32_t *const loc_row = const_cast<int32_t *>(mv.loc_row), *const loc_col = const_cast<int32_t *>(mv.loc_col);
        if (piece == 0) {
            int total;
            const int cstart = excl_prefix<8>(ccnt, total);
            if (lane < KB) col_ptr[lane] = cstart;
            if (lane == 0) col_ptr[KB] = total;
            const int key = lane < KB ? ccnt * 1024 + (1023 - lane) : -1;
            int crank = 0;
            for (int q = 0; q < KB; ++q) crank += __builtin_amdgcn_readlane(key, q) > key;
            if (lane < KB) col_order[crank] = lane;
            const uint64_t first_col = __ballot(lane < KB && crank == 0);
            const int max_col = __builtin_amdgcn_readlane(ccnt, first_col ? (int)__builtin_ctzll(first_col) : 0);
            const int max_row = row_count(row_of_rank(0));
            uint64_t *const bits = const_cast<uint64_t *>(mv.bits);
#pragma unroll
            for (int r = 0; r < 2; ++r)
                if (lane + 64 * r < MB) bits[lane + 64 * r] = rw[r];
            if (lane == 0) {
                MaskHeader h = {};
                h.M = P.M; h.K = P.K; h.BM = P.BM; h.BK = P.BK; h.MB = MB; h.KB = KB;
                h.words_per_row = 1;
                h.nnz = total;
                h.magic = kMaskMagic;
                h.max_row_cnt = max_row;
                h.max_col_cnt = max_col;
                h.flags = kMaskDrawn;
                h.p = P.p_call;
                h.seed = ((uint64_t)P.key1 << 32) | P.key0;
                h.rng_stream = ((uint64_t)P.ctr3 << 32) | P.ctr2;
                // everything but n_units, which piece 2 writes
                const uint64_t *const src = reinterpret_cast<const uint64_t *>(&h);
                uint64_t *const dst = reinterpret_cast<uint64_t *>(const_cast<MaskHeader *>(mv.hdr));
                static_assert(offsetof(MaskHeader, n_units) == 80, "the header's eleventh 8 bytes hold n_units");
#pragma unroll
                for (int q = 0; q < 32; ++q)
                    if (q != 10) dst[q] = src[q];
                reinterpret_cast<int32_t *>(dst)[21] = 0;
            }
            return;
        }
        if (piece == 2) {
            const int n = units_apply(MB, KB, P.BM, P.BK) ? build_units(rw[0], rw[1], MB, const_cast<int32_t *>(mv.units)) : 0;
            if (lane == 0) reinterpret_cast<int32_t *>(const_cast<MaskHeader *>(mv.hdr))[20] = n;
            return;
        }
        int start[2], total;
        row_starts(start, total);
        if (piece == 1) {
#pragma unroll
            for (int r = 0; r < 2; ++r)
                if (lane + 64 * r < MB) { row_ptr[lane + 64 * r] = start[r]; row_order[lane + 64 * r] = ord[r]; }
            if (lane == 0) row_ptr[MB] = total;
            return;
        }
        piece -= 3;
        if (piece < MB) {
            // block row `piece`: lane <-> block column
            const uint64_t word = row_word(piece);
            const int base = start_of_row(start, piece);     // read from another lane: outside the divergent branch
            if ((word >> lane) & 1) {
                const int at = base + (int)below_count(word);
                col_idx[at] = lane;
                blk_row[at] = piece;
            }
            return;
        }
        piece -= MB;
        if (piece < KB) {
            // block column `piece`: lane <-> block row; the ballots are the column's keep bits
            const int j = piece;
            const uint64_t c0 = __ballot((rw[0] >> j) & 1), c1 = __ballot((rw[1] >> j) & 1);
            int base;                                         // kept blocks in earlier columns: those columns' counts, summed
            (void)excl_prefix<8>(lane < j ? ccnt : 0, base);
            if ((rw[0] >> j) & 1) row_idx[base + below_count(c0)] = lane;
            if ((rw[1] >> j) & 1) row_idx[base + (int)__popcll(c0) + below_count(c1)] = lane + 64;
            return;
        }
        piece -= KB;
        {
            // group `piece` of 8 block rows, sorted by (column, row): lane <-> block column
            const int i0 = piece * 8, nr = MB - i0 < 8 ? MB - i0 : 8;
            int mine = 0, c = 0;
            for (int r = 0; r < nr; ++r) {
                const int bit = (int)((row_word(i0 + r) >> lane) & 1);
                mine |= bit << r;
                c += bit;
            }
            int in_group;
            int at = start_of_row(start, i0) + excl_prefix<4>(c, in_group);
            for (int r = 0; r < nr; ++r)
                if ((mine >> r) & 1) { loc_row[at] = i0 + r; loc_col[at] = lane; ++at; }
        }
    }

    // wavefront `slot` of `nslots` writes pieces slot, slot + nslots, ...
    __device__ __forceinline__ void write_pieces(const GemmParams &P, int slot, int nslots) const
    {
        const int n = pieces();
        for (int piece = slot; piece < n; piece += nslots) write_piece(P, piece);
    }
};

}  // namespace
}  // namespace sdrop
#endif
