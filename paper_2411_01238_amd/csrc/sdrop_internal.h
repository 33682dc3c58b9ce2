// Internal declarations shared by the translation units of libsdrop.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "sdrop.h"

namespace sdrop {

// First 256 bytes of a mask object (device memory).  nnz sits at byte 36.
struct MaskHeader {
    int64_t M, K;            // 0, 8
    int32_t BM, BK;          // 16, 20
    int32_t MB, KB;          // 24, 28
    int32_t words_per_row;   // 32
    int32_t nnz;             // 36
    uint32_t magic;          // 40
    int32_t max_row_cnt;     // 44
    int32_t max_col_cnt;     // 48
    uint32_t flags;          // 52: kMaskDrawn when the mask was drawn (p, seed, rng_stream below say how)
    double p;                // 56: the dropout probability the mask was drawn with (0 when built from given bits)
    uint64_t seed;           // 64
    uint64_t rng_stream;     // 72
    int32_t n_units;         // 80: entries of the pair list (0 when the grid is too large for one)
    int32_t pad_[43];
};
static_assert(sizeof(MaskHeader) == 256, "mask header is 256 bytes");
static_assert(offsetof(MaskHeader, nnz) == SDROP_MASK_NNZ_OFFSET, "nnz offset is part of the ABI");

constexpr uint32_t kMaskMagic = 0x5344524Fu;  // "SDRO"
constexpr uint32_t kMaskDrawn = 1u;           // MaskHeader::flags

// Does the mask object belong to this call?  Same shape and blocks, and, for a mask that was drawn, the dropout
// probability the call derives its scale from is the one the mask was drawn with.  A kernel that finds a mismatch
// writes nothing; one of its threads records it in the library's status word (see sdrop_status) when there is one.
__device__ __forceinline__ bool mask_header_ok(const MaskHeader *H, int64_t M, int64_t K, int BM, int BK,
                                               bool check_p, double p_call, int *status)
{
    bool ok = H->magic == kMaskMagic && H->M == M && H->K == K && H->BM == BM && H->BK == BK;
    if (ok && check_p && (H->flags & kMaskDrawn) && H->p != p_call) ok = false;
    if (!ok && status && blockIdx.x == 0 && threadIdx.x == 0) atomicOr(status, SDROP_STATUS_MASK_MISMATCH);
    return ok;
}

// Device-side view of a mask object.
struct MaskView {
    const MaskHeader *hdr;
    const uint64_t *bits;
    const int32_t *row_ptr, *col_idx, *blk_row;
    const int32_t *col_ptr, *row_idx, *row_order, *col_order;
    const int32_t *loc_row, *loc_col;
    const int32_t *units;
};

inline MaskView make_view(const void *mask, const sdrop_mask_layout_t &L)
{
    const char *b = static_cast<const char *>(mask);
    MaskView v;
    v.hdr = reinterpret_cast<const MaskHeader *>(b);
    v.bits = reinterpret_cast<const uint64_t *>(b + L.off_bits);
    v.row_ptr = reinterpret_cast<const int32_t *>(b + L.off_row_ptr);
    v.col_idx = reinterpret_cast<const int32_t *>(b + L.off_col_idx);
    v.blk_row = reinterpret_cast<const int32_t *>(b + L.off_blk_row);
    v.col_ptr = reinterpret_cast<const int32_t *>(b + L.off_col_ptr);
    v.row_idx = reinterpret_cast<const int32_t *>(b + L.off_row_idx);
    v.row_order = reinterpret_cast<const int32_t *>(b + L.off_row_order);
    v.col_order = reinterpret_cast<const int32_t *>(b + L.off_col_order);
    v.loc_row = reinterpret_cast<const int32_t *>(b + L.off_loc_row);
    v.loc_col = reinterpret_cast<const int32_t *>(b + L.off_loc_col);
    v.units = reinterpret_cast<const int32_t *>(b + L.off_units);
    return v;
}

// Philox4x32-10 (Salmon et al., SC'11); returns output word 0.
__device__ __forceinline__ uint32_t philox_word0(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                 uint32_t k0, uint32_t k1)
{
    // the two 32 x 32 -> 64-bit products of a round, each as ONE 64-bit multiply (a multiply-add instruction that
    // delivers both halves; written as separate high and low products the round costs four multiplies)
    constexpr uint64_t MUL0 = 0xD2511F53u, MUL1 = 0xCD9E8D57u;
    constexpr uint32_t BUMP0 = 0x9E3779B9u, BUMP1 = 0xBB67AE85u;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = MUL0 * (uint64_t)c0, p1 = MUL1 * (uint64_t)c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        c0 = n0; c1 = (uint32_t)p1; c2 = n2; c3 = (uint32_t)p0;
        k0 += BUMP0; k1 += BUMP1;   // the bump after the last round is unused
    }
    return c0;
}

// ---- The pair list: the kept blocks of a small grid (at most 128 x 64 blocks of 128 x 128) as units of two ----
// eq. (2) computes kept blocks only, and a 128 x 256 tile of two kept blocks costs about 1.6 single 128 x 128 tiles.
// Two kept blocks can share a tile when they share the block row (a wide pair: one dY panel against two W panels)
// or the block column (a tall pair: two dY panels against one W panel, computed as the transposed product).
// The list partitions the kept blocks into such pairs and as few single blocks as it can:
//   rows in ascending order; a row with an odd number of kept blocks gives one of them away: if it keeps a column
//   in which an earlier row's block is still waiting, the lowest such column, and the two form a tall pair; else
//   its own highest kept column, where the block waits.  The rest of a row pairs up left to right.  Blocks
//   still waiting after the last row are singles.
// Order of the list: the wide pairs row by row, the tall pairs in the order they were closed, the singles by column.
// An entry is kind << 30 | x << 16 | y << 8 | z: wide (i, j1, j2), tall (j, i1, i2), single (i, j, j).
constexpr int kUnitWide = 0, kUnitTall = 1, kUnitSingle = 2;
constexpr int kUnitsMaxMB = 128, kUnitsMaxKB = 64;
// (built for 128 x 128 blocks only, the one block size whose eq. 2 kernel walks it: on the 128 x 16 grid of 64 x 64
// blocks of the MLP workload it cost the forward kernel that writes the mask object 5 of 23 us)
__host__ __device__ inline bool units_apply(int64_t MB, int64_t KB, int BM, int BK)
{
    return MB <= kUnitsMaxMB && KB <= kUnitsMaxKB && BM == 128 && BK == 128;
}
__device__ __forceinline__ int32_t unit_entry(int kind, int x, int y, int z) { return (int32_t)((uint32_t)kind << 30 | (uint32_t)x << 16 | (uint32_t)y << 8 | (uint32_t)z); }

// Called by all 64 lanes of one wavefront; lane l passes the keep words of block rows l and l + 64 (0 beyond the
// grid).  Writes the list and returns its length (the same value in every lane).
__device__ inline int build_units(uint64_t rw0, uint64_t rw1, int MB, int32_t *units)
{
    const int lane = threadIdx.x & 63;
    // where each row's wide pairs go: a row has floor(kept / 2) of them whichever block it gives away
    // (prefix sums over the lanes by ballots of the counts' six bits: no trips through the LDS crossbar)
    const int np0 = __popcll(rw0) >> 1, np1 = __popcll(rw1) >> 1;
    const uint64_t below = (uint64_t(1) << lane) - 1;
    int off0 = 0, off1 = 0, tot0 = 0, tot1 = 0;
#pragma unroll
    for (int b = 0; b < 6; ++b) {
        const uint64_t m0 = __ballot((np0 >> b) & 1), m1 = __ballot((np1 >> b) & 1);
        off0 += (int)__popcll(m0 & below) << b;
        off1 += (int)__popcll(m1 & below) << b;
        tot0 += (int)__popcll(m0) << b;
        tot1 += (int)__popcll(m1) << b;
    }
    off1 += tot0;
    const int n_wide = tot0 + tot1;
    // The rows with an odd count in turn (the others give nothing away).  Every lane follows the same chain, in
    // scalar registers and without a branch inside a step (a step with branches took 0.14 us, 18 us for 128 rows):
    // lane c remembers the row waiting in column c, lane i % 64 the column row i gave away, lane t the t-th tall pair.
    const uint32_t lo0 = (uint32_t)rw0, hi0 = (uint32_t)(rw0 >> 32), lo1 = (uint32_t)rw1, hi1 = (uint32_t)(rw1 >> 32);
    uint64_t waiting = 0;
    int pend = 0, gave0 = -1, gave1 = -1, n_tall = 0;
    int32_t tall = 0;
    auto chain = [&](uint64_t odd, uint32_t lo_v, uint32_t hi_v, int base, int &gave) __attribute__((always_inline)) {
        while (odd) {
            const int src = __builtin_ctzll(odd);
            odd &= odd - 1;
            // (the builtin returns a signed int: through uint32_t, or the low word's top bit would spread over the high word)
            const uint64_t w = (uint64_t)(uint32_t)__builtin_amdgcn_readlane(hi_v, src) << 32 | (uint32_t)__builtin_amdgcn_readlane(lo_v, src);
            const uint64_t hit = w & waiting;
            const bool has = hit != 0;                  // an earlier row's block waits in a column this row keeps
            const int c = has ? __builtin_ctzll(hit) : 63 - __builtin_clzll(w);
            const int i1 = __builtin_amdgcn_readlane(pend, c);
            tall = (has && lane == n_tall) ? unit_entry(kUnitTall, c, i1, base + src) : tall;
            n_tall += has ? 1 : 0;
            waiting ^= uint64_t(1) << c;                // taken out of the waiting set, or put into it
            pend = (!has && lane == c) ? base + src : pend;
            gave = lane == src ? c : gave;
        }
    };
    chain(__ballot(__popcll(rw0) & 1), lo0, hi0, 0, gave0);
    chain(__ballot(__popcll(rw1) & 1), lo1, hi1, 64, gave1);
    (void)MB;                                           // (rows beyond the grid hold no bits)
    if (lane < n_tall) units[n_wide + lane] = tall;
    // what still waits is single: lane <-> column
    const int n_single = (int)__popcll(waiting);
    if ((waiting >> lane) & 1)
        units[n_wide + n_tall + (int)__popcll(waiting & ((uint64_t(1) << lane) - 1))] = unit_entry(kUnitSingle, pend, lane, lane);
    // every lane writes the wide pairs of its two rows
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        uint64_t w = h ? rw1 : rw0;
        const int gave = h ? gave1 : gave0, i = lane + 64 * h;
        int at = h ? off1 : off0;
        if (gave >= 0) w &= ~(uint64_t(1) << gave);
        while (w) {
            const int j1 = __builtin_ctzll(w);
            w &= w - 1;
            const int j2 = __builtin_ctzll(w);
            w &= w - 1;
            units[at++] = unit_entry(kUnitWide, i, j1, j2);
        }
    }
    return n_wide + n_tall + n_single;
}

// Host-side argument checks shared by the GEMM entry points.
int check_gemm_args(const void *a, const void *b, const void *mask, void *out,
                    int64_t M, int64_t K, int64_t N, int BM, int BK, double p,
                    int dtype, int out_dtype);

// Records a HIP failure for sdrop_last_hip_error() and returns SDROP_EHIP, or SDROP_OK.
int hip_status(hipError_t e);

inline bool block_size_ok(int b) { return b == 64 || b == 128; }

// Compute units of the current device (256 when the query fails).
int cu_count();

// The current device's status word (device address), or null when it cannot be had.
int *device_status_word();

}  // namespace sdrop
