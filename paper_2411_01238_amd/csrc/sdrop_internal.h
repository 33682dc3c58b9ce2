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
    int32_t pad_[44];
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
