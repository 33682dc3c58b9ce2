// The persistent forms of the three block-sparse GEMMs and the launches that hold both gradients (included by
// the typed GEMM translation units only; the design notes are at the top of that file).
#ifndef SDROP_GEMM_PERSISTENT_KERNELS_H
#define SDROP_GEMM_PERSISTENT_KERNELS_H
#include "gemm_tile_kernel.h"
#include "gemm_seeded_grid.h"

namespace sdrop {
namespace {

// The computing side of a persistent kernel: one wavefront's accumulators and operand registers,
// the MFMA schedule of one slice, and the epilogue.
template <class T, class OutT, bool A_TR, bool B_TR, int TM, int TN, int WM, int WN> struct Compute {
    static constexpr int WTM = TM / WM, WTN = TN / WN, MI = WTM / 32, NI = WTN / 32;
    static constexpr int A_BYTES = TM * TK * 2;
    static constexpr int NM = MI * NI, NOPS = MI + NI;
    // operand reads requested per MFMA (at least what fits the group)
    static constexpr int RPM_MIN = ceil_div(NOPS, NM >= 4 ? NM - 2 : NM), RPM = 2 > RPM_MIN ? 2 : RPM_MIN;
    static constexpr int ESZ = (int)sizeof(OutT);
    static constexpr int STAGING = 32 * 128;         // output staging per wavefront: 32 rows of 128 bytes
    static constexpr int NIP = 128 / (32 * ESZ);     // 32-column accumulator blocks per 128-byte row
    static constexpr int NJ = NI / NIP;              // 128-byte column groups of the wavefront's sub-tile
    static_assert(NI % NIP == 0, "a wavefront's columns must fill whole 128-byte rows");

    typename In<T>::vec fa[2][MI], fb[2][NI];
    f32x16 acc[MI][NI];
    int wm, wn;

    __device__ __forceinline__ void zero()
    {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;
    }
    // operands of the first quarter of the slice in stage `st`
    __device__ __forceinline__ void first(const char *st)
    {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) fa[0][mi] = read_frag<T, A_TR, TM>(st, wm * WTM + mi * 32, 0);
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) fb[0][ni] = read_frag<T, B_TR, TN>(st + A_BYTES, wn * WTN + ni * 32, 0);
    }
    // One slice: 4 quarters of NM MFMAs.  On entry the first quarter's operands are in flight to
    // register set 0; each MFMA is followed by up to RPM operand reads for the next quarter, in the
    // order that quarter's MFMAs (A index major) first use them: A0, B0 .. B(NI-1), A1 .. A(MI-1).
    // After the first MFMAs of the last quarter comes the slice's barrier (every wavefront is done
    // reading `cur`; the slice in `nx1` has landed), then the first operands of `nx1`.
    // SWAP: the MFMAs take the operands the other way round, which leaves the transposed 32 x 32 blocks in the
    // accumulators (lane <-> tile column, registers <-> tile rows); store_t writes such a tile out transposed.
    template <bool SWAP = false> __device__ __forceinline__ void slice(const char *cur, const char *nx1)
    {
        __builtin_amdgcn_sched_barrier(0);
        static_for<4>([&](auto gi) __attribute__((always_inline)) {
            constexpr int g = decltype(gi)::value;
            constexpr int NB = (g == 3 && NM >= 4) ? 2 : 0;   // MFMAs of the last quarter that precede the barrier
            static_for<NM>([&](auto ci) __attribute__((always_inline)) {
                constexpr int c = decltype(ci)::value;
                constexpr int mi = c / NI, ni = c % NI, cb = g & 1, nb = (g + 1) & 1;
                if constexpr (g == 3 && c == NB) {
                    __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(63));
                    __builtin_amdgcn_s_barrier();
                    __builtin_amdgcn_sched_barrier(0);
                }
                if constexpr (SWAP) acc[mi][ni] = In<T>::mfma(fa[cb][mi], fb[cb][ni], acc[mi][ni]);
                else acc[mi][ni] = In<T>::mfma(fb[cb][ni], fa[cb][mi], acc[mi][ni]);
                constexpr int r0 = c < NB ? 0 : (c - NB) * RPM < NOPS ? (c - NB) * RPM : NOPS;
                constexpr int r1 = c < NB ? 0 : (c - NB + 1) * RPM < NOPS ? (c - NB + 1) * RPM : NOPS;
                static_for<r1 - r0>([&](auto ri) __attribute__((always_inline)) {
                    constexpr int r = r0 + decltype(ri)::value;
                    const char *st = g < 3 ? cur : nx1;
                    constexpr int kk = g < 3 ? g + 1 : 0;
                    if constexpr (r == 0) fa[nb][0] = read_frag<T, A_TR, TM>(st, wm * WTM, kk);
                    else if constexpr (r <= NI) fb[nb][r - 1] = read_frag<T, B_TR, TN>(st + A_BYTES, wn * WTN + (r - 1) * 32, kk);
                    else fa[nb][r - NI] = read_frag<T, A_TR, TM>(st, wm * WTM + (r - NI) * 32, kk);
                });
                __builtin_amdgcn_sched_barrier(0);
            });
        });
    }
    // Epilogue: scale in fp32, round once, park 32 rows x 128 bytes at a time in this wavefront's
    // own piece of LDS (`reg`) and write them out as whole 128-byte lines.  The MFMAs took the
    // operands swapped, so accumulator register 4q+e of lane l is row l%32, column 8q + 4(l/32) + e
    // of its 32x32 block.  8-byte slot u of row r lies at slot u ^ (r & 15): the 8-byte writes of 32
    // rows then spread over all banks, and a 16-byte read finds its two halves in one 16-byte
    // piece, exchanged when r is odd.  dst(mi, nj) is the address of row 0 of the 32 x 128-byte
    // piece (mi, nj) of the wavefront's sub-tile, or null if that piece is not to be written.
    // With a tail, dst also reports the global column of the piece's first column.
    //
    // The bias values of a range of pieces are requested by tail_prefetch ahead of the store of that
    // range (see finish): one wait for all of them instead of one per piece.  For 16-bit outputs under
    // a ReLU gate the gate values lie where the outputs go; store requests them a piece ahead.
    uint4 gate_q[MI * NJ][4];
    f32x4 bias_r[NJ][NIP * 4];
    template <int MI0 = 0, int MI1 = MI, int NJ0 = 0, int NJ1 = NJ, class F>
    __device__ __forceinline__ void tail_prefetch(int64_t ldc, const Tail &tl, F &&dst)
    {
        const int lane = threadIdx.x & 63;
        const int whalf = lane >> 5;
#pragma unroll
        for (int mi = MI0; mi < MI1; ++mi)
#pragma unroll
            for (int nj = NJ0; nj < NJ1; ++nj) {
                int64_t gcol0 = 0;
                char *const out = dst(mi, nj, gcol0);
                if (!out) continue;                        // uniform
                if (mi == 0 && tl.bias) {
#pragma unroll
                    for (int i = 0; i < NIP * 4; ++i)
                        bias_r[nj][i] = *(const_f4)(uintptr_t)(tl.bias + gcol0 + (i >> 2) * 32 + 8 * (i & 3) + 4 * whalf);
                }
            }
    }
    // The gate values of one 32 x 128-byte piece, in the layout its rows are written in.
    template <class F> __device__ __forceinline__ void gate_load(int mi, int nj, uint4 (&g)[4], int64_t ldc, const Tail &tl, F &&dst)
    {
        const int lane = threadIdx.x & 63;
        const int rrow = lane >> 3, rch = lane & 7;
        int64_t gcol0 = 0;
        char *const out = dst(mi, nj, gcol0);
        if (!out) return;                                  // uniform
#pragma unroll
        for (int it = 0; it < 4; ++it)
            g[it] = *reinterpret_cast<const uint4 *>(tl.aux + (out - tl.c0) + (int64_t)(it * 8 + rrow) * ldc + rch * 16);
    }
    // MODE: which tail this instance is compiled for (TailMode; the host picks the kernel by it).  The
    // generic form carries every activation and every gate's derivative in each of its 16 to 32
    // unrolled steps, ~200 KB of code of which a tile runs a few KB scattered over all of it: a ReLU
    // then cost 25 us per 128 x 256 tile, mostly instruction fetch.  The common tails have forms of
    // their own that hold one mode's code only.
    // RAGN: the tile may hang over the last column of the output (N not a multiple of the tile);
    // pieces that lie beyond column `ncols` are skipped and the piece that straddles it is written
    // only up to it (N is a multiple of 8, so whole 16-byte chunks).
    int64_t ncols;
    template <int MODE, int MI0 = 0, int MI1 = MI, int NJ0 = 0, int NJ1 = NJ, bool RAGN = false, class F>
    __device__ __forceinline__ void store(char *reg, float scale, int64_t ldc, const Tail &tl, F &&dst)
    {
        constexpr bool TAIL = MODE != kTailNone;
        const int lane = threadIdx.x & 63;
        const int wrow = lane & 31, whalf = lane >> 5;
        const int rrow = lane >> 3, rch = lane & 7;
        // 16-bit outputs under a ReLU gate are gated after rounding, on whole rows; everything else in the accumulator's layout
        const bool gate_rows = MODE == kTailReluGate ? ESZ == 2
                             : MODE == kTailGeneric ? (ESZ == 2 && tl.aux != nullptr && tl.gate_mode == SDROP_GATE_RELU) : false;
        const bool gate_acc = MODE == kTailReluGate ? ESZ == 4 : MODE == kTailGeluErfGate ? true
                            : MODE == kTailGeneric ? (tl.aux != nullptr && !gate_rows) : false;
        const int gate_mode = MODE == kTailGeneric ? tl.gate_mode : MODE == kTailGeluErfGate ? SDROP_GATE_GELU_ERF : SDROP_GATE_RELU;
        // The gate values of a piece are requested AHEAD pieces before it is written.  With 128
        // accumulator registers (a 64 x 128 sub-tile) that is one piece: the values of a whole
        // sub-tile next to its accumulators do not fit the register file (measured on tiles with a
        // 1024-long reduction: 672 -> 619 us).  Smaller sub-tiles request all of them up front
        // (one piece ahead measured 73 -> 79 us at 4096^3).
        constexpr int NJW = NJ1 - NJ0, NP = (MI1 - MI0) * NJW;
        constexpr int AHEAD = MI * NI * 16 >= 128 ? 1 : NP;
        if constexpr (TAIL && ESZ == 2) {
            if (gate_rows) {
#pragma unroll
                for (int q = 0; q < AHEAD && q < NP; ++q) gate_load(MI0 + q / NJW, NJ0 + q % NJW, gate_q[q], ldc, tl, dst);
            }
        }
#pragma unroll
        for (int pc = 0; pc < NP; ++pc) {
            {
                const int mi = MI0 + pc / NJW, nj = NJ0 + pc % NJW;
                if constexpr (TAIL && ESZ == 2) {
                    if (gate_rows && pc + AHEAD < NP)
                        gate_load(MI0 + (pc + AHEAD) / NJW, NJ0 + (pc + AHEAD) % NJW, gate_q[pc + AHEAD], ldc, tl, dst);
                }
                int64_t gcol0 = 0;
                char *const out = dst(mi, nj, gcol0);
                if (!out) continue;                        // uniform
                const int vch = RAGN ? (int)((ncols - gcol0) * ESZ / 16) : 8;      // valid 16-byte chunks of the piece's rows
                if (RAGN && vch <= 0) continue;            // uniform
#pragma unroll
                for (int nl = 0; nl < NIP; ++nl)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const f32x16 &a = acc[mi][nj * NIP + nl];
                        float v[4] = {a[4 * q] * scale, a[4 * q + 1] * scale, a[4 * q + 2] * scale, a[4 * q + 3] * scale};
                        if constexpr (TAIL) {
                            if (tl.bias) {
                                const f32x4 bv = bias_r[nj][nl * 4 + q];
                                v[0] += bv.x; v[1] += bv.y; v[2] += bv.z; v[3] += bv.w;
                            }
                            if constexpr (MODE == kTailLight) {
                                if (tl.act == SDROP_ACT_RELU) act4(SDROP_ACT_RELU, v);       // no activation, or a ReLU
                            } else if constexpr (MODE == kTailGeluErf) {
                                act4(SDROP_ACT_GELU_ERF, v);
                            } else if constexpr (MODE == kTailGeneric) {
                                act4(tl.act, v);
                            }
                            if (gate_acc) {
                                // the gate matrix has 16-bit elements, read here in the accumulator's layout
                                using E = typename In<T>::out16;
                                typedef __attribute__((__vector_size__(4 * sizeof(E)))) E e4;
                                const int c = nl * 32 + 8 * q + 4 * whalf;   // column within the piece
                                const int64_t elem = (out - tl.c0) / ESZ + wrow * (ldc / ESZ) + c;
                                const e4 x = *reinterpret_cast<const e4 *>(tl.aux + elem * (int64_t)sizeof(E));
                                const float xf[4] = {static_cast<float>(x[0]), static_cast<float>(x[1]), static_cast<float>(x[2]), static_cast<float>(x[3])};
                                gate4(gate_mode, v, xf);
                            }
                        }
                        const float v0 = v[0], v1 = v[1], v2 = v[2], v3 = v[3];
                        if constexpr (ESZ == 4) {
                            // 16 bytes per lane: 16-byte slot 2q + half, exchanged as a whole with (row & 7)
                            const int slot = (2 * q + whalf) ^ (wrow & 7);
                            *reinterpret_cast<float4 *>(reg + wrow * 128 + slot * 16) = make_float4(v0, v1, v2, v3);
                        } else {
                            typedef __attribute__((__vector_size__(4 * sizeof(OutT)))) OutT out4;
                            const out4 o = {static_cast<OutT>(v0), static_cast<OutT>(v1), static_cast<OutT>(v2), static_cast<OutT>(v3)};
                            const int slot8 = (nl * 8 + 2 * q + whalf) ^ (wrow & 15);
                            *reinterpret_cast<out4 *>(reg + wrow * 128 + slot8 * 8) = o;
                        }
                    }
                // all four reads of the piece are requested before the first is used (left to itself the compiler
                // waited for each one before it requested the next: four trips to LDS in a row per piece)
                uint4 rv[4];
#pragma unroll
                for (int it = 0; it < 4; ++it) {
                    const int row = it * 8 + rrow;
                    if constexpr (ESZ == 4) rv[it] = *reinterpret_cast<const uint4 *>(reg + row * 128 + ((rch ^ (row & 7)) << 4));
                    else rv[it] = *reinterpret_cast<const uint4 *>(reg + row * 128 + ((rch ^ ((row & 15) >> 1)) << 4));
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int it = 0; it < 4; ++it) {
                    const int row = it * 8 + rrow;
                    uint4 v = rv[it];
                    if constexpr (ESZ != 4) {
                        const uint4 x = rv[it];
                        v = (row & 1) ? make_uint4(x.z, x.w, x.x, x.y) : x;
                        if constexpr (TAIL) {
                            if (gate_rows) v = gate16<T>(v, gate_q[pc][it]);
                        }
                    }
                    if (!RAGN || rch < vch) store_out(out + (int64_t)row * ldc + rch * 16, v);
                }
            }
        }
    }
    // The epilogue of a tile whose slices ran with SWAP, written out transposed (no tail): accumulator block
    // [mi][ni] holds, in the layout `store` expects, the 32 x 32 block (ni, mi) of the transposed sub-tile, so a
    // 32-row x 128-byte piece (r, pj) of the transposed sub-tile is made of blocks [pj NIP + nl][r].
    // dst_t(r, pj) is the address of its row 0, or null.
    template <class F> __device__ __forceinline__ void store_t(char *reg, float scale, int64_t ldc, F &&dst_t)
    {
        static_assert(MI % NIP == 0, "a wavefront's rows must fill whole 128-byte rows of the transposed tile");
        const int lane = threadIdx.x & 63;
        const int wrow = lane & 31, whalf = lane >> 5;
        const int rrow = lane >> 3, rch = lane & 7;
#pragma unroll
        for (int r = 0; r < NI; ++r)
#pragma unroll
            for (int pj = 0; pj < MI / NIP; ++pj) {
                char *const out = dst_t(r, pj);
                if (!out) continue;                        // uniform
#pragma unroll
                for (int nl = 0; nl < NIP; ++nl)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const f32x16 &a = acc[pj * NIP + nl][r];
                        const float v0 = a[4 * q] * scale, v1 = a[4 * q + 1] * scale, v2 = a[4 * q + 2] * scale, v3 = a[4 * q + 3] * scale;
                        if constexpr (ESZ == 4) {
                            const int slot = (2 * q + whalf) ^ (wrow & 7);
                            *reinterpret_cast<float4 *>(reg + wrow * 128 + slot * 16) = make_float4(v0, v1, v2, v3);
                        } else {
                            typedef __attribute__((__vector_size__(4 * sizeof(OutT)))) OutT out4;
                            const out4 o = {static_cast<OutT>(v0), static_cast<OutT>(v1), static_cast<OutT>(v2), static_cast<OutT>(v3)};
                            const int slot8 = (nl * 8 + 2 * q + whalf) ^ (wrow & 15);
                            *reinterpret_cast<out4 *>(reg + wrow * 128 + slot8 * 8) = o;
                        }
                    }
                uint4 rv[4];                               // (all four reads first, as in store)
#pragma unroll
                for (int it = 0; it < 4; ++it) {
                    const int row = it * 8 + rrow;
                    if constexpr (ESZ == 4) rv[it] = *reinterpret_cast<const uint4 *>(reg + row * 128 + ((rch ^ (row & 7)) << 4));
                    else rv[it] = *reinterpret_cast<const uint4 *>(reg + row * 128 + ((rch ^ ((row & 15) >> 1)) << 4));
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int it = 0; it < 4; ++it) {
                    const int row = it * 8 + rrow;
                    const uint4 x = rv[it];
                    const uint4 v = (ESZ == 4 || !(row & 1)) ? x : make_uint4(x.z, x.w, x.x, x.y);
                    store_out(out + (int64_t)row * ldc + rch * 16, v);
                }
            }
    }
    // The epilogue of one tile.  With a tail, the sub-tile goes out in two halves (of its column groups,
    // else of its row blocks when it is one group wide and four blocks tall), each half requesting its
    // own tail operands first: the accumulators and the operands of a whole 64 x 128 or 128 x 64 sub-tile
    // together do not fit the register file, those of a half do.
    template <int MODE, bool RAGN = false, class F> __device__ __forceinline__ void finish(char *reg, float scale, int64_t ldc, const Tail &tl, F &&dst)
    {
        static_assert(!RAGN || MODE == kTailNone, "tiles that hang over the output's edge have no tail forms");
        if constexpr (MODE == kTailNone) {
            store<kTailNone, 0, MI, 0, NJ, RAGN>(reg, scale, ldc, tl, dst);
        } else if constexpr (NJ >= 2) {
            constexpr int H = NJ / 2;
            tail_prefetch<0, MI, 0, H>(ldc, tl, dst);
            store<MODE, 0, MI, 0, H>(reg, scale, ldc, tl, dst);
            tail_prefetch<0, MI, H, NJ>(ldc, tl, dst);
            store<MODE, 0, MI, H, NJ>(reg, scale, ldc, tl, dst);
        } else if constexpr (MI >= 4) {
            constexpr int H = MI / 2;
            tail_prefetch<0, H, 0, NJ>(ldc, tl, dst);
            store<MODE, 0, H, 0, NJ>(reg, scale, ldc, tl, dst);
            tail_prefetch<H, MI, 0, NJ>(ldc, tl, dst);
            store<MODE, H, MI, 0, NJ>(reg, scale, ldc, tl, dst);
        } else {
            tail_prefetch(ldc, tl, dst);
            store<MODE>(reg, scale, ldc, tl, dst);
        }
    }
};

// s_waitcnt immediate that waits only for vector-memory operations (at most `vm` outstanding).
constexpr int waitcnt_vm_only(int vm) { return (vm & 15) | ((vm >> 4) << 14) | (7 << 4) | (15 << 8); }
// s_waitcnt immediate that waits only for LDS / scalar-memory operations (lgkmcnt = 0).
constexpr int waitcnt_lgkm0_only() { return 15 | (3 << 14) | (7 << 4) | (0 << 8); }

// FWD and DW for 128-row tiles without ragged edges, as a persistent kernel: one workgroup per
// CU walks a fixed sequence of tiles, and the slices of consecutive tiles form ONE stream
// through the three LDS stages.  The four loader wavefronts run two slices ahead of the four
// computing wavefronts across tile boundaries, so the first operands of the next tile arrive
// while the current tile is still being multiplied and stored; what the per-tile launch pays
// for every tile (index look-ups, the latency of the first loads: about 4 us, against 25 us of
// MFMAs per tile at 4096^3 with half the blocks kept) is paid once per workgroup.
//
// Tile sequence of workgroup w of G: tiles are numbered in the mask's schedule order (heaviest
// block rows / columns first), and round k takes tile k*G + w (k even) or k*G + G-1-w (k odd),
// so a workgroup that drew a heavy tile in one round draws a light one in the next.
//
// Synchronisation: slice g of the workgroup's stream lives in stage g % 3.  Barrier g is passed
// by the computing wavefronts when they have read all of slice g, and by the loaders when their
// part of slice g+1 has landed; the loaders issue slice g+2 (into the stage of slice g-1) after
// barrier g-1.  One more barrier, before the first slice, publishes slice 0.  Both roles derive
// the number of slices from the same mask lists, so they execute the same number of barriers.
// (The body is a device function of the workgroup's index w among G, so that one launch can hold
// the workgroups of two operations; see bwd_fused_kernel.)
//
// SEEDED (the forward only): there is no mask object to read.  Every workgroup draws the block grid itself and keeps
// it in registers (SeededGrid), so a tile's block row and its kept columns come from a few scalar instructions
// instead of three dependent look-ups, and the computing wavefronts write the mask object for the backward kernels,
// a small piece each, before they meet their first barrier.
//
// W_NK (the forward, whole tile columns, no tail): the weight is given as [N,K], one row per output column, so its
// reduction index is the contiguous one like X's: the B tile of a slice is then 256 rows of W at the slice's column
// offset, loaded and read in the row form that eq. (2) uses for both its operands.
// W_NK for eq. (3): the gradient goes out as [N,K].  Operands and loads are as ever; the MFMAs take their operands the
// other way round, which leaves the transposed 32 x 32 blocks in the accumulators, and the epilogue writes the tile
// transposed (Compute::store_t), into the output or into planes of partial sums laid out [N][K].
template <int OP, class T, class OutT, int TM, int TN, int WM, int WN, int TAIL, bool RAGN = false, bool SEEDED = false,
          bool W_NK = false>
__device__ __forceinline__ void gemm_persistent_body(const GemmParams &P, const int G, const int w)
{
    static_assert(OP == FWD || OP == DW, "output-sparse dX is not handled here");
    static_assert(!SEEDED || OP == FWD, "only the forward kernel draws its own mask");
    static_assert(!W_NK || (!RAGN && TAIL == kTailNone), "[N,K] weights: the plain products on whole tiles");
    static_assert(!W_NK || OP == FWD || (TM / WM / 32) % (128 / (32 * (int)sizeof(OutT))) == 0, "the transposed tile's rows must fill 128-byte pieces");
    constexpr int NW = WM * WN;
    static_assert(NW == 4, "one computing and one loading wavefront per SIMD");
    constexpr int WTM = TM / WM, WTN = TN / WN, MI = WTM / 32, NI = WTN / 32;
    constexpr bool A_KMAJ = (OP == FWD), A_TR = !A_KMAJ, B_TR = !(W_NK && OP == FWD);
    constexpr bool OUT_T = W_NK && OP == DW;             // the output tile is written transposed
    constexpr int A_BYTES = TM * TK * 2, B_BYTES = TN * TK * 2, STAGE_BYTES = A_BYTES + B_BYTES;
    constexpr int STAGES = 3, AHEAD = 2;
    constexpr int ESZ = (int)sizeof(OutT);
    constexpr int STAGING = 32 * 128;           // per computing wavefront: 32 rows of 128 bytes

    extern __shared__ __attribute__((aligned(16))) char smem[];
    char *const staging = smem + STAGES * STAGE_BYTES;

    // A kernel handed a mask built for another problem writes nothing.  The header is tested after
    // the first look-ups have been issued (they are addressed by the tile number alone and stay
    // inside the mask object whatever it holds), so that it costs no round trip of its own.
    const MaskHeader *H = P.mv.hdr;
    auto mask_ok = [&]() __attribute__((always_inline)) -> bool {
        return mask_header_ok(H, P.M, P.K, P.BM, P.BK, true, P.p_call, P.status);
    };

    const int lane = threadIdx.x & 63;
    const int wave_all = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const bool loader = wave_all >= NW;
    const int wave = loader ? wave_all - NW : wave_all;
    const int wm = wave / WN, wn = wave % WN;
    const int total = P.total_tiles;
    const int BLK = (OP == FWD) ? P.BK : P.BM;            // extent of a mask block along the reduction
    const int sub_shift = (BLK == 128), sub_mask = (1 << sub_shift) - 1;
    const int64_t lda = P.lda, ldb = P.ldb, ldc = P.ldc;
    const int32_t *const order = (OP == FWD) ? P.mv.row_order : P.mv.col_order;
    const int32_t *const ptr = (OP == FWD) ? P.mv.row_ptr : P.mv.col_ptr;
    const int32_t *const lists = (OP == FWD) ? P.mv.col_idx : P.mv.row_idx;
    const int per_line = P.n_tiles * P.splits;            // tiles per block row / column

    SeededGrid sg;
    // all eight wavefronts; two barriers inside.  The third stage is free for it: the loaders fill it only after the
    // stream's first barrier, which the computing wavefronts join after they have read the order back
    static_assert(SeededGrid::kLdsBytes <= STAGE_BYTES, "the draw's scratch must fit a stage");
    if constexpr (SEEDED) sg.draw(P, smem + 2 * STAGE_BYTES);

    // tile number of round k (may be >= total: the sequence has ended)
    auto tile_of = [&](int k) __attribute__((always_inline)) -> int { return k * G + ((k & 1) ? G - 1 - w : w); };
    // position in the schedule order; clamped so that look-ahead beyond the end stays in bounds
    auto rank_of = [&](int t) __attribute__((always_inline)) -> int { return (t < total ? t : total - 1) / per_line; };
    // the part of a kept list of `cnt` entries that tile t reduces: [lo, lo + len)
    auto part_of = [&](int t, int cnt, int &lo) __attribute__((always_inline)) -> int {
        if (P.splits == 1) { lo = 0; return cnt; }
        const int part = t % P.splits;
        lo = (int)((int64_t)cnt * part / P.splits);
        return (int)((int64_t)cnt * (part + 1) / P.splits) - lo;
    };
    auto stage_ptr = [&](int st) __attribute__((always_inline)) -> char * { return smem + st * STAGE_BYTES; };

    if (loader) {
        // ---------------- loaders: the stream of slices ----------------
        using DmaA = typename std::conditional<A_KMAJ, DmaK<TM, 1, NW>, DmaT<TM, NW>>::type;
        using DmaB = typename std::conditional<W_NK && OP == FWD, DmaK<TN, 1, NW>, DmaT<TN, NW>>::type;
        DmaA da;
        DmaB db;
        da.init(lda, wave);
        db.init(ldb, wave);
        constexpr int NDMA_A = TM / (8 * NW), NDMA_B = TN / (8 * NW), NDMA = NDMA_A + NDMA_B;

        // Look-ups run three tiles ahead of the tile being issued, one level of indirection per
        // tile, so that no load waits for the one before it: order[] of tile k+3, the list bounds
        // of tile k+2, the first two list entries of tile k+1.
        // The mask lists do not change while the kernel runs: read through the constant address
        // space they keep the scalar load form also after a barrier (which otherwise counts as a
        // possible write to anything in global memory).
        typedef const __attribute__((address_space(4))) int32_t *const_i32;
        const const_i32 k_order = (const_i32)(uintptr_t)order, k_ptr = (const_i32)(uintptr_t)ptr;
        const const_i32 k_lists = (const_i32)(uintptr_t)lists;
        struct Meta { int t, ord, start, len, e0, e1; };
        auto level1 = [&](int k) __attribute__((always_inline)) -> Meta {
            Meta m;
            m.t = tile_of(k);
            m.ord = k_order[rank_of(m.t)];
            m.start = m.len = m.e0 = m.e1 = 0;
            return m;
        };
        auto level2 = [&](Meta &m) __attribute__((always_inline)) {
            const int p0 = k_ptr[m.ord], cnt = k_ptr[m.ord + 1] - p0;
            int lo;
            m.len = part_of(m.t < total ? m.t : total - 1, cnt, lo);
            m.start = p0 + lo;
        };
        auto entry = [&](const Meta &m, int e) __attribute__((always_inline)) -> int {
            const int ec = e < m.len ? e : m.len - 1;
            return k_lists[ec < 0 ? 0 : m.start + ec];
        };
        auto level3 = [&](Meta &m) __attribute__((always_inline)) { m.e0 = entry(m, 0); m.e1 = entry(m, 1); };

        Meta cur, n1, n2, n3;
        if constexpr (!SEEDED) {
            n1 = level1(0); n2 = level1(1); n3 = level1(2);
            if (!mask_ok()) return;
            level2(n1); level3(n1);
            level2(n2);
        }
        uint64_t w_rem = 0;              // SEEDED: kept columns of the current block row that are still to come
        int nt_cur = 0, ord_cur = 0;
        int k = -1;                      // round of the tile being issued
        int s = 0, nsteps = 0;           // next slice of that tile; its number of slices
        int e_cur = 0, e_nxt = 0;        // list entries of slice s and of the block after it
        const char *a_tile = nullptr, *b_tile = nullptr;
        int b_chunks = TN / 8;           // RAGN: 16-byte chunks of B's rows that exist in this tile column
        bool ended = false;

        // issues the next slice of the stream into stage `st`; false when the stream has ended
        auto issue_next = [&](int st) __attribute__((always_inline)) -> bool {
            while (s == nsteps) {
                if (ended) return false;
                ++k;
                if constexpr (SEEDED) {
                    const int t = tile_of(k);
                    if (t >= total) { ended = true; return false; }
                    ord_cur = sg.row_of_rank(t / per_line);
                    nt_cur = t % per_line;
                    const uint64_t word = sg.row_word(ord_cur);
                    s = 0;
                    nsteps = (int)__popcll(word) << sub_shift;
                    e_cur = word ? (int)__builtin_ctzll(word) : 0;
                    w_rem = word & (word - 1);
                } else {
                    cur = n1;
                    if (cur.t >= total) { ended = true; return false; }
                    n1 = n2; level3(n1);
                    n2 = n3; level2(n2);
                    n3 = level1(k + 3);
                    s = 0;
                    nsteps = cur.len << sub_shift;
                    e_cur = cur.e0; e_nxt = cur.e1;
                    ord_cur = cur.ord;
                    nt_cur = (cur.t % per_line) / P.splits;
                }
                const int nt = nt_cur;
                if constexpr (OP == FWD) a_tile = P.A + (int64_t)ord_cur * P.BM * lda;
                else a_tile = P.A + (int64_t)ord_cur * P.BK * 2;
                if constexpr (W_NK && OP == FWD) b_tile = P.B + (int64_t)nt * TN * ldb;      // rows [nt TN, nt TN + TN) of W[N,K]
                else b_tile = P.B + (int64_t)nt * TN * 2;
                if constexpr (RAGN) {
                    const int64_t left = P.N - (int64_t)nt * TN;
                    b_chunks = left < TN ? (int)(left / 8) : TN / 8;
                }
            }
            const int64_t off = (int64_t)e_cur * BLK + (int64_t)(s & sub_mask) * TK;
            const char *const sa[1] = {a_tile + off * (OP == FWD ? 2 : lda)};
            const char *const sb[1] = {(W_NK && OP == FWD) ? b_tile + off * 2 : b_tile + off * ldb};
            char *stp = stage_ptr(st);
#pragma unroll
            for (int j = 0; j < NDMA_A; ++j) da.issue(sa, lda, stp, j);
            if constexpr (RAGN) {
#pragma unroll
                for (int j = 0; j < NDMA_B; ++j) db.issue(sb, ldb, stp + A_BYTES, j, b_chunks);
            } else {
#pragma unroll
                for (int j = 0; j < NDMA_B; ++j) db.issue(sb, ldb, stp + A_BYTES, j);
            }
            ++s;
            if ((s & sub_mask) == 0) {
                if constexpr (SEEDED) {
                    e_cur = w_rem ? (int)__builtin_ctzll(w_rem) : 0;
                    w_rem &= w_rem - 1;
                } else {
                    e_cur = e_nxt;
                    e_nxt = entry(cur, (s >> sub_shift) + 1);
                }
            }
            return true;
        };

        int issued = 0, st_issue = 0;
        for (int i = 0; i < AHEAD; ++i)
            if (issue_next(st_issue)) { ++issued; st_issue = st_issue == STAGES - 1 ? 0 : st_issue + 1; }
        if (issued == 0) return;         // no slice at all: the computing wavefronts meet no barrier either
        if (issued == AHEAD) __builtin_amdgcn_s_waitcnt(waitcnt_vm_only(NDMA));
        else __builtin_amdgcn_s_waitcnt(waitcnt_vm_only(0));
        __builtin_amdgcn_s_barrier();    // slice 0 is in place
        for (int g = 0; g < issued; ++g) {
            const bool more = issue_next(st_issue);
            if (more) {
                ++issued;
                st_issue = st_issue == STAGES - 1 ? 0 : st_issue + 1;
                __builtin_amdgcn_s_waitcnt(waitcnt_vm_only(NDMA));      // all but the slice just issued: g+1 is in
            } else {
                __builtin_amdgcn_s_waitcnt(waitcnt_vm_only(0));
            }
            __builtin_amdgcn_s_barrier();
        }
        return;
    }

    // ---------------- computing wavefronts ----------------
    // Look-ups two tiles ahead (order[] of tile k+2, list bounds of tile k+1), as vector loads:
    // they are waited for with the vector-memory counter, which the main loop never waits on.
    // Every look-up is turned into a scalar right after a tile's slices, BEFORE the tile's stores:
    // the counter is in order, so a wait placed after the stores (the top of the next iteration)
    // would also wait until those stores have drained to memory.
    auto c_order = [&](int k) __attribute__((always_inline)) -> int { return order[rank_of(tile_of(k))]; };
    auto c_count = [&](int o) __attribute__((always_inline)) -> int { return ptr[o + 1] - ptr[o]; };
    auto c_len = [&](int k, int cnt) __attribute__((always_inline)) -> int {
        const int tk = tile_of(k);
        int lo;
        return part_of(tk < total ? tk : total - 1, cnt, lo);
    };
    // scalars: this tile (ord0, len0), the next one's block row / column (ord1);
    // in flight: the next tile's kept count (cnt1_v), order[] of the tile after it (ord2_v)
    int ord0 = 0, len0 = 0, ord1 = 0, ord2 = 0;
    if constexpr (SEEDED) {
        // this wavefront's pieces of the mask object, while the first operands are on their way
        sg.write_pieces(P, w * NW + wave, G * NW);
    } else {
        const int ord0_v = c_order(0), ord1_v = c_order(1), ord2_v = c_order(2);
        if (!mask_ok()) return;
        ord0 = uni(ord0_v);
        len0 = uni(c_len(0, c_count(ord0)));
        ord1 = uni(ord1_v);
        __builtin_amdgcn_s_waitcnt(waitcnt_vm_only(0));
        ord2 = uni(ord2_v);
    }

    Compute<T, OutT, A_TR, B_TR, TM, TN, WM, WN> cw;
    cw.wm = wm; cw.wn = wn;
    cw.ncols = P.N;
    int st0 = 0, st1 = 1, st2 = 2;       // stages of the stream's slices g, g+1, g+2
    bool started = false;
    const float scale = P.scale;
    const Tail tl = make_tail(P);
    char *const reg = staging + wave * STAGING;

    for (int k = 0;; ++k) {
        const int t = tile_of(k);
        if (t >= total) break;
        int cnt1_v = 0, ord3_v = 0;
        if constexpr (SEEDED) {
            ord0 = sg.row_of_rank(t / per_line);
            len0 = sg.row_count(ord0);
        } else {
            // requests for the tiles after this one; consumed after this tile's slices
            cnt1_v = c_count(ord1);
            ord3_v = c_order(k + 3);
        }
        const int ord = ord0, nsteps = len0 << sub_shift;

        cw.zero();
        if (nsteps > 0 && !started) {
            started = true;
            __builtin_amdgcn_s_barrier();                     // slice 0 is in place
            cw.first(stage_ptr(0));
        }
        const int line = t % per_line;
        const int nt = line / P.splits, part = line % P.splits;
        char *c_tile;
        if constexpr (OP == FWD) c_tile = P.C + (int64_t)ord * P.BM * ldc + (int64_t)nt * TN * ESZ;
        else c_tile = P.C + (int64_t)part * P.K * ldc + (int64_t)ord * P.BK * ldc + (int64_t)nt * TN * ESZ;
        c_tile += (int64_t)(wm * WTM) * ldc + (int64_t)(wn * WTN) * ESZ;
        auto dst = [&](int mi, int nj, int64_t &gcol0) __attribute__((always_inline)) -> char * {
            gcol0 = (int64_t)nt * TN + wn * WTN + nj * (128 / ESZ);
            return c_tile + (int64_t)(mi * 32) * ldc + nj * 128;
        };
        for (int s = 0; s < nsteps; ++s) {
            cw.template slice<OUT_T>(stage_ptr(st0), stage_ptr(st1));
            const int t0 = st0; st0 = st1; st1 = st2; st2 = t0;
        }
        if constexpr (!SEEDED) {
            // the look-ups have had the whole tile to arrive and no store is in flight: this wait is free
            __builtin_amdgcn_s_waitcnt(waitcnt_vm_only(0));
            len0 = uni(c_len(k + 1, cnt1_v));
            ord0 = ord1; ord1 = ord2; ord2 = uni(ord3_v);
        }
        if constexpr (OUT_T) {
            // the wavefront's sub-tile, rows [ord BK + wm WTM, +WTM) x columns [nt TN + wn WTN, +WTN) of dW, is rows
            // [nt TN + wn WTN, +WTN) x columns [ord BK + wm WTM, +WTM) of the [N,K] output (or of plane `part`)
            char *const ct = P.C + (int64_t)part * P.N * ldc + ((int64_t)nt * TN + wn * WTN) * ldc
                             + ((int64_t)ord * P.BK + wm * WTM) * ESZ;
            auto dst_t = [&](int r, int pj) __attribute__((always_inline)) -> char * {
                return ct + (int64_t)(r * 32) * ldc + pj * 128;
            };
            cw.store_t(reg, scale, ldc, dst_t);
        } else {
            cw.template finish<TAIL, RAGN>(reg, scale, ldc, tl, dst);
        }
    }
}

template <int OP, class T, class OutT, int TM, int TN, int WM, int WN, int TAIL, bool RAGN = false>
__global__ __launch_bounds__(WM * WN * 128) void gemm_persistent_kernel(GemmParams P)
{
    gemm_persistent_body<OP, T, OutT, TM, TN, WM, WN, TAIL, RAGN>(P, gridDim.x, blockIdx.x);
}

// eq. (3) with the gradient written as [N,K] (see W_NK above).
template <class T, class OutT, int TM>
__global__ __launch_bounds__(512) void dw_nk_kernel(GemmParams P)
{
    gemm_persistent_body<DW, T, OutT, TM, 256, 1, 4, kTailNone, false, false, true>(P, gridDim.x, blockIdx.x);
}

// eq. (1) with the weight as [N,K] (see W_NK above); SEEDED: it draws its own mask as well.
template <class T, class OutT, int TM, bool SEEDED>
__global__ __launch_bounds__(512) void fwd_nk_kernel(GemmParams P)
{
    gemm_persistent_body<FWD, T, OutT, TM, 256, 1, 4, kTailNone, false, SEEDED, true>(P, gridDim.x, blockIdx.x);
}

// The forward kernel that draws its own mask and writes the mask object as well (see SEEDED above).
template <class T, class OutT, int TM, bool RAGN>
__global__ __launch_bounds__(512) void fwd_seeded_kernel(GemmParams P)
{
    gemm_persistent_body<FWD, T, OutT, TM, 256, 1, 4, kTailNone, RAGN, true>(P, gridDim.x, blockIdx.x);
}

// a[i] for a uniform index i in 0..3, as selects (keeps everything in scalar registers)
__device__ __forceinline__ int sel4(const int (&a)[4], int i)
{
    return i == 0 ? a[0] : i == 1 ? a[1] : i == 2 ? a[2] : a[3];
}

// dX for 128-row tiles without a ragged reduction tail, as a persistent kernel (same stream of
// slices, stages and barrier protocol as gemm_persistent_kernel; every tile reduces over all of N,
// so every tile has the same number of slices).
//
// Work units are groups of G = TN / BK consecutive entries of a kept-block list: the locally
// ordered one for G = 1, the row-major one for G > 1 (consecutive entries then share the block
// row).  A group whose entries lie in one block row is one tile; where the row changes inside a
// group it is cut into one tile per run of equal rows.  The groups are dealt out in equal
// contiguous chunks to the XCDs (workgroup w runs on XCD w mod 8) and round-robin inside a
// chunk, so that the tiles an XCD has in flight at one time are neighbours in the list.
// Both roles read the same list entries and derive the same tiles from them.
//
// Zero fill of the dropped blocks: workgroup w owns block positions w, w+G, ...; its loader
// wavefronts write them a kilobyte per slice of the stream, beside the direct loads, and finish
// what is left when the stream has ended.
//
// PAIRS (128 x 128 blocks, 256-wide tiles, no tail, whole slices, dY and W with the same row stride): the work
// units are the entries of the mask's pair list instead.  A wide pair or a single block is a tile as above (two
// block columns of one block row; the single block twice, written once).  A tall pair, blocks (i1, j) and
// (i2, j), is computed as the transposed product: W's panel j takes dY's place as the 128-row operand, the two dY
// panels are the 256-row operand, the MFMAs take their operands the other way round and the epilogue writes the
// two 128 x 128 results transposed.
//
// W_NK (one kept block of 128 x 128 per tile, no tail, whole slices): the weight is given as [N,K].  Its reduction
// index is then the strided one, as in eq. (1): a slice of B is 64 rows of W at the block's column offset, loaded
// and read in eq. 1's transposing form.
template <class T, class OutT, int TM, int TN, int WM, int WN, int TAIL, bool RAGN = false, bool PAIRS = false, bool W_NK = false>
__device__ __forceinline__ void gemm_persistent_dx_body(const GemmParams &P, const int G, const int w)
{
    static_assert(!W_NK || (TN == 128 && TAIL == kTailNone && !RAGN && !PAIRS), "[N,K] weights: plain single-block tiles");
    constexpr int NW = WM * WN;
    static_assert(NW == 4 && TM == 128, "one computing and one loading wavefront per SIMD, 128-row tiles");
    static_assert(!PAIRS || (TN == 256 && TAIL == kTailNone && !RAGN), "the pair list serves plain 128 x 256 tiles");
    constexpr int WTM = TM / WM, WTN = TN / WN;
    constexpr int DXG = TN / 64;                      // 64-column chunks of a tile
    static_assert(DXG <= 4, "tile too wide");
    constexpr int A_BYTES = TM * TK * 2, B_BYTES = TN * TK * 2, STAGE_BYTES = A_BYTES + B_BYTES;
    constexpr int STAGES = 3, AHEAD = 2;
    constexpr int ESZ = (int)sizeof(OutT);
    constexpr int STAGING = 32 * 128;

    extern __shared__ __attribute__((aligned(16))) char smem[];
    char *const staging = smem + STAGES * STAGE_BYTES;

    const MaskHeader *H = P.mv.hdr;
    if (!mask_header_ok(H, P.M, P.K, P.BM, P.BK, true, P.p_call, P.status)) return;

    const int lane = threadIdx.x & 63;
    const int wave_all = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const bool loader = wave_all >= NW;
    const int wave = loader ? wave_all - NW : wave_all;
    const int wm = wave / WN, wn = wave % WN;
    const int GB = TN / P.BK;                          // kept blocks per group: 1, 2 or 4
    const int cshift = (P.BK == 128), cmask = (1 << cshift) - 1;   // 64-column chunks per block
    const int nnz = H->nnz;
    const int ngroups = PAIRS ? H->n_units : (nnz + GB - 1) / GB;
    // slices of the reduction; when N is not a multiple of the slice the last one is ragged: the loaders
    // clear what lies beyond N in LDS (see DmaK::issue), the computing wavefronts see a full slice
    // (RAGN: a form of its own, because the extra case in the loaders cost the whole-slice form 5 %)
    const int nsteps = RAGN ? (int)((P.N + TK - 1) / TK) : (int)(P.N / TK);
    const int last_chunks = RAGN ? (int)(P.N % TK) / 8 : 0;       // valid 16-byte chunks of a ragged last slice, 0 if none
    const int64_t lda = P.lda, ldb = P.ldb, ldc = P.ldc;
    const int32_t *const rows = GB == 1 ? P.mv.loc_row : P.mv.blk_row;
    const int32_t *const cols = GB == 1 ? P.mv.loc_col : P.mv.col_idx;
    // this workgroup's groups: chunk x of the list, local indices r, r + wx, r + 2 wx, ...
    const int nx = G < 8 ? G : 8;
    const int x = w % nx, r = w / nx;
    const int wx = (G - x + nx - 1) / nx;              // workgroups that share chunk x
    const int per_chunk = (ngroups + nx - 1) / nx;
    // group of round k, or -1 when the workgroup has no more
    auto group_of = [&](int k) __attribute__((always_inline)) -> int {
        const int lr = r + k * wx;
        const int u = x * per_chunk + lr;
        return (lr < per_chunk && u < ngroups) ? u : -1;
    };
    auto stage_ptr = [&](int st) __attribute__((always_inline)) -> char * { return smem + st * STAGE_BYTES; };
    struct Group { int u, n; int r[4], c[4]; };        // list entries [u GB, u GB + n)

    if (loader) {
        DmaK<TM, 1, NW> da;
        typename std::conditional<W_NK, DmaT<TN, NW>, DmaK<TN, DXG, NW>>::type db;
        da.init(lda, wave);
        db.init(ldb, wave);
        constexpr int NDMA_A = TM / (8 * NW), NDMA_B = TN / (8 * NW), NDMA = NDMA_A + NDMA_B;
        typedef const __attribute__((address_space(4))) int32_t *const_i32;   // see gemm_persistent_kernel
        const const_i32 k_rows = (const_i32)(uintptr_t)rows, k_cols = (const_i32)(uintptr_t)cols;
        const const_i32 k_units = (const_i32)(uintptr_t)P.mv.units;
        auto load_group = [&](int k) __attribute__((always_inline)) -> Group {
            Group g;
            g.u = group_of(k);
            if constexpr (PAIRS) {
                // one entry of the pair list (c[0]); entry 0 always lies inside the object
                g.n = g.u < 0 ? 0 : 1;
#pragma unroll
                for (int b = 0; b < 4; ++b) g.r[b] = g.c[b] = 0;
                g.c[0] = k_units[g.u < 0 ? 0 : g.u];
                return g;
            }
            const int e0 = (g.u < 0 ? 0 : g.u) * GB;
            g.n = g.u < 0 ? 0 : (nnz - e0 < GB ? nnz - e0 : GB);
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const int e = e0 + (b < g.n ? b : 0);   // always a valid entry (the lists hold at least one slot)
                g.r[b] = k_rows[e < nnz ? e : 0];
                g.c[b] = k_cols[e < nnz ? e : 0];
            }
            return g;
        };
        Group cur, nxt;
        cur.u = -1; cur.n = 0;
#pragma unroll
        for (int b = 0; b < 4; ++b) cur.r[b] = cur.c[b] = 0;
        nxt = load_group(0);
        int k = -1, a = 0;                              // round of `cur`; next unused entry of `cur`
        int s = nsteps;                                 // next slice of the tile being issued
        const char *a_tile = nullptr;
        const char *bgrp[DXG];
#pragma unroll
        for (int g = 0; g < DXG; ++g) bgrp[g] = nullptr;
        bool ended = false;

        auto issue_next = [&](int st) __attribute__((always_inline)) -> bool {
            if (s == nsteps) {
                if (ended) return false;
                if (a >= cur.n) {
                    ++k;
                    cur = nxt;
                    if (cur.u < 0) { ended = true; return false; }
                    nxt = load_group(k + 1);
                    a = 0;
                }
                if constexpr (PAIRS) {
                    const int ent = cur.c[0], kind = (ent >> 30) & 3, x = (ent >> 16) & 255, y = (ent >> 8) & 255, z = ent & 255;
                    // (lda == ldb here, so either matrix can sit on either side)
                    const char *const m128 = kind == kUnitTall ? P.B : P.A, *const m256 = kind == kUnitTall ? P.A : P.B;
                    a_tile = m128 + (int64_t)x * 128 * lda;
#pragma unroll
                    for (int g = 0; g < DXG; ++g) bgrp[g] = m256 + ((int64_t)(g < 2 ? y : z) * 128 + (g & 1) * 64) * ldb;
                    a = 1;
                    s = 0;
                } else {
                const int row = sel4(cur.r, a);
                int nb = 1;
                while (a + nb < cur.n && sel4(cur.r, a + nb) == row) ++nb;
                a_tile = P.A + (int64_t)row * P.BM * lda;
#pragma unroll
                for (int g = 0; g < DXG; ++g) {
                    const int bb = g >> cshift;         // a missing block repeats the last one
                    const int col = sel4(cur.c, a + (bb < nb ? bb : nb - 1));
                    if constexpr (W_NK) bgrp[g] = P.B + (int64_t)col * P.BK * 2;      // columns of W[N,K] (one block per tile)
                    else bgrp[g] = P.B + ((int64_t)col * P.BK + (g & cmask) * 64) * ldb;
                }
                a += nb;
                s = 0;
                }
            }
            const int64_t off = (int64_t)s * TK * 2;
            const char *const sa[1] = {a_tile + off};
            const char *sb[DXG];
#pragma unroll
            for (int g = 0; g < DXG; ++g) sb[g] = bgrp[g] + off;
            char *stp = stage_ptr(st);
            bool whole = true;
            if constexpr (RAGN) {
                if (last_chunks != 0 && s == nsteps - 1) {
                    whole = false;
#pragma unroll
                    for (int j = 0; j < NDMA_A; ++j) da.issue(sa, lda, stp, j, last_chunks);
#pragma unroll
                    for (int j = 0; j < NDMA_B; ++j) db.issue(sb, ldb, stp + A_BYTES, j, last_chunks);
                    // the cleared chunks are ordinary LDS writes: done before this wavefront goes on to
                    // the barrier that publishes the slice (which waits for the direct loads only)
                    __builtin_amdgcn_s_waitcnt(waitcnt_lgkm0_only());
                }
            }
            if (whole) {
#pragma unroll
                for (int j = 0; j < NDMA_A; ++j) da.issue(sa, lda, stp, j);
                if constexpr (W_NK) {
                    const char *const sk[1] = {bgrp[0] + (int64_t)s * TK * ldb};      // rows [64 s, 64 s + 64) of W[N,K]
#pragma unroll
                    for (int j = 0; j < NDMA_B; ++j) db.issue(sk, ldb, stp + A_BYTES, j);
                } else {
#pragma unroll
                    for (int j = 0; j < NDMA_B; ++j) db.issue(sb, ldb, stp + A_BYTES, j);
                }
            }
            ++s;
            return true;
        };

        // Zero fill of the dropped blocks, by the loaders: the workgroup owns positions w, w + G, ...
        // (z-th: w + G z).  One step per slice of the stream: either test the next position's keep
        // bit (its word was requested a step earlier, as a scalar load through the constant address
        // space) or write this wavefront's next kilobyte of the dropped block in hand (a block is
        // TM rows of BK elements; the four loaders share its 16-byte pieces).  The computing
        // wavefronts never stop for it.  The stores go out before the step's direct loads, so the
        // wait that follows those loads still means "the slice issued one step ago has landed".
        typedef const __attribute__((address_space(4))) uint64_t *const_u64;
        const const_u64 k_bits = (const_u64)(uintptr_t)P.mv.bits;
        const int total_pos = P.MB * P.KB;
        const int nz = w < total_pos ? (total_pos - w + G - 1) / G : 0;
        const int wpr = H->words_per_row;
        const int row_chunks = P.BK * ESZ / 16;                      // 16-byte pieces per row of a block
        const int per_wave = TM * row_chunks / (NW * 64);           // store instructions per wavefront and block
        int zpos = 0;                    // next position to test
        int zprog = 0;                   // store instructions already issued for the block in hand
        char *zblock = nullptr;          // the dropped block in hand, or null
        uint64_t zword = 0;              // keep bits around position zpos (valid when zpos < nz)
        auto request_word = [&]() __attribute__((always_inline)) {
            if (zpos < nz) {
                const int pz = w + G * zpos;
                zword = k_bits[(int64_t)(pz / P.KB) * wpr + ((pz % P.KB) >> 6)];
            }
        };
        request_word();
        // true while there is zero fill left
        auto zero_step = [&]() __attribute__((always_inline)) -> bool {
            if (zblock) {
                const int c = (zprog * NW + wave) * 64 + lane;
                store_out(zblock + (c / row_chunks) * ldc + (c % row_chunks) * 16, make_uint4(0, 0, 0, 0));
                if (++zprog == per_wave) zblock = nullptr;
                return true;
            }
            if (zpos >= nz) return false;
            const int pz = w + G * zpos;
            const int zi = pz / P.KB, zj = pz % P.KB;
            if (!((zword >> (zj & 63)) & 1)) {
                zblock = P.C + (int64_t)zi * P.BM * ldc + (int64_t)zj * P.BK * ESZ;
                zprog = 0;
            }
            ++zpos;
            request_word();
            return true;
        };

        int issued = 0, st_issue = 0;
        for (int i = 0; i < AHEAD; ++i)
            if (issue_next(st_issue)) { ++issued; st_issue = st_issue == STAGES - 1 ? 0 : st_issue + 1; }
        if (issued > 0) {
            if (issued == AHEAD) __builtin_amdgcn_s_waitcnt(waitcnt_vm_only(NDMA));
            else __builtin_amdgcn_s_waitcnt(waitcnt_vm_only(0));
            __builtin_amdgcn_s_barrier();
            for (int g = 0; g < issued; ++g) {
                zero_step();
                const bool more = issue_next(st_issue);
                if (more) {
                    ++issued;
                    st_issue = st_issue == STAGES - 1 ? 0 : st_issue + 1;
                    __builtin_amdgcn_s_waitcnt(waitcnt_vm_only(NDMA));
                } else {
                    __builtin_amdgcn_s_waitcnt(waitcnt_vm_only(0));
                }
                __builtin_amdgcn_s_barrier();
            }
        }
        // what the stream left of the zero fill (all of it for a workgroup without tiles)
        while (zero_step()) { }
        return;
    }

    // ---------------- computing wavefronts ----------------
    auto c_load_group = [&](int k) __attribute__((always_inline)) -> Group {
        Group g;
        g.u = group_of(k);
        if constexpr (PAIRS) {
            g.n = g.u < 0 ? 0 : 1;
#pragma unroll
            for (int b = 0; b < 4; ++b) g.r[b] = g.c[b] = 0;
            g.c[0] = P.mv.units[g.u < 0 ? 0 : g.u];
            return g;
        }
        const int e0 = (g.u < 0 ? 0 : g.u) * GB;
        g.n = g.u < 0 ? 0 : (nnz - e0 < GB ? nnz - e0 : GB);
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int e = e0 + (b < g.n ? b : 0);
            g.r[b] = rows[e < nnz ? e : 0];
            g.c[b] = cols[e < nnz ? e : 0];
        }
        return g;
    };
    Compute<T, OutT, false, W_NK, TM, TN, WM, WN> cw;
    cw.wm = wm; cw.wn = wn;
    int st0 = 0, st1 = 1, st2 = 2;
    bool started = false;
    const float scale = P.scale;
    const Tail tl = make_tail(P);
    char *const reg = staging + wave * STAGING;

    // Every look-up (the next group's entries) is turned
    // into scalars right after a tile's slices, BEFORE the tile's stores: the vector-memory counter is
    // in order, so a wait placed after the stores would also wait until they have drained to memory
    // (measured: 2.4 us per tile on 65536 x 4096 x 1024).
    Group nxt = c_load_group(0);
    __builtin_amdgcn_s_waitcnt(waitcnt_vm_only(0));
    int gr[4], gc[4];
#pragma unroll
    for (int b = 0; b < 4; ++b) { gr[b] = uni(nxt.r[b]); gc[b] = uni(nxt.c[b]); }
    int gn = nxt.n, gu = nxt.u;
    for (int k = 0; gu >= 0; ++k) {
        nxt = c_load_group(k + 1);                      // in flight during this group's tiles
        int ngr[4] = {0, 0, 0, 0}, ngc[4] = {0, 0, 0, 0};
        int a = 0;
        if constexpr (PAIRS) {
            // one unit = one tile
            const int ent = gc[0], kind = (ent >> 30) & 3, x = (ent >> 16) & 255, y = (ent >> 8) & 255, z = ent & 255;
            cw.zero();
            if (!started) {
                started = true;
                __builtin_amdgcn_s_barrier();           // slice 0 is in place
                cw.first(stage_ptr(0));
            }
            if (kind == kUnitTall) {
                for (int s = 0; s < nsteps; ++s) {
                    cw.template slice<true>(stage_ptr(st0), stage_ptr(st1));
                    const int t0 = st0; st0 = st1; st1 = st2; st2 = t0;
                }
            } else {
                for (int s = 0; s < nsteps; ++s) {
                    cw.slice(stage_ptr(st0), stage_ptr(st1));
                    const int t0 = st0; st0 = st1; st1 = st2; st2 = t0;
                }
            }
            __builtin_amdgcn_s_waitcnt(waitcnt_vm_only(0));
#pragma unroll
            for (int b = 0; b < 4; ++b) { ngr[b] = uni(nxt.r[b]); ngc[b] = uni(nxt.c[b]); }
            if (kind == kUnitTall) {
                // sub-tile (wm, wn) of the tile [W panel x] x [dY panels y, z] is, transposed, rows [32 r, 32 r + 32)
                // of block row (wn ? z : y) and columns [64 wm, 64 wm + 64) of block column x
                char *const c_blk = P.C + ((int64_t)(wn ? z : y) * 128) * ldc + ((int64_t)x * 128 + wm * WTM) * ESZ;
                auto dst_t = [&](int r, int pj) __attribute__((always_inline)) -> char * {
                    return c_blk + (int64_t)(r * 32) * ldc + pj * 128;
                };
                cw.store_t(reg, scale, ldc, dst_t);
            } else {
                char *const c_rows = P.C + ((int64_t)x * 128 + wm * WTM) * ldc;
                const int cols_valid = kind == kUnitSingle ? 128 : 256;
                auto dst = [&](int mi, int nj, int64_t &gcol0) __attribute__((always_inline)) -> char * {
                    const int col_t = wn * WTN + nj * (128 / ESZ);         // first column of the piece, in the tile
                    if (col_t >= cols_valid) return nullptr;
                    const int64_t col0 = (int64_t)(col_t < 128 ? y : z) * 128 + (col_t & 127);
                    gcol0 = col0;
                    return c_rows + (int64_t)(mi * 32) * ldc + col0 * ESZ;
                };
                cw.template finish<kTailNone>(reg, scale, ldc, tl, dst);
            }
            (void)a;
        } else
        while (a < gn) {
            const int row = sel4(gr, a);
            int nb = 1;
            while (a + nb < gn && sel4(gr, a + nb) == row) ++nb;
            const int chunks_valid = nb << cshift;

            cw.zero();
            if (!started) {
                started = true;
                __builtin_amdgcn_s_barrier();           // slice 0 is in place
                cw.first(stage_ptr(0));
            }
            char *const c_rows = P.C + ((int64_t)row * P.BM + wm * WTM) * ldc;
            auto dst = [&](int mi, int nj, int64_t &gcol0) __attribute__((always_inline)) -> char * {
                const int col_t = wn * WTN + nj * (128 / ESZ);         // first column of the piece, in the tile
                const int g = col_t >> 6;
                if (g >= chunks_valid) return nullptr;
                const int col = sel4(gc, a + (g >> cshift));
                const int64_t col0 = (int64_t)col * P.BK + (g & cmask) * 64 + (col_t & 63);
                gcol0 = col0;
                return c_rows + (int64_t)(mi * 32) * ldc + col0 * ESZ;
            };
            for (int s = 0; s < nsteps; ++s) {
                cw.slice(stage_ptr(st0), stage_ptr(st1));
                const int t0 = st0; st0 = st1; st1 = st2; st2 = t0;
            }
            // the look-ups have had the whole tile to arrive and no store is in flight: this wait is free
            __builtin_amdgcn_s_waitcnt(waitcnt_vm_only(0));
#pragma unroll
            for (int b = 0; b < 4; ++b) { ngr[b] = uni(nxt.r[b]); ngc[b] = uni(nxt.c[b]); }
            if constexpr (TAIL != kTailNone) {
                if (P.C2) {
                    // the producing layer's value before the activation, to the second output
                    const Tail tz = make_tail_preact(P);
                    const int64_t delta = P.C2 - P.C;
                    auto dst2 = [&](int mi, int nj, int64_t &gcol0) __attribute__((always_inline)) -> char * {
                        char *const o = dst(mi, nj, gcol0);
                        return o ? o + delta : nullptr;
                    };
                    cw.template finish<kTailLight>(reg, scale, ldc, tz, dst2);     // bias only
                }
            }
            cw.template finish<TAIL>(reg, scale, ldc, tl, dst);
            a += nb;
        }
#pragma unroll
        for (int b = 0; b < 4; ++b) { gr[b] = ngr[b]; gc[b] = ngc[b]; }
        gn = nxt.n; gu = nxt.u;
    }
}

template <class T, class OutT, int TM, int TN, int WM, int WN, int TAIL, bool RAGN, bool PAIRS = false, bool W_NK = false>
__global__ __launch_bounds__(WM * WN * 128) void gemm_persistent_dx_kernel(GemmParams P)
{
    gemm_persistent_dx_body<T, OutT, TM, TN, WM, WN, TAIL, RAGN, PAIRS, W_NK>(P, gridDim.x, blockIdx.x);
}

// Both gradients of the layer in one launch (eq. 2 and eq. 3 share dY and the mask and do not
// depend on each other): workgroups [0, g_dx) are the persistent dX kernel, the rest the persistent
// dW kernel.  One workgroup fits a CU, so the dW workgroups start one by one on the CUs that the dX
// workgroups leave: no launch boundary (about 5 us of idle chip between dependent launches) and no
// idle tail between the two.  The dX workgroups come first, so dX workgroup w is workgroup w of
// the launch and runs on XCD w % 8, which its schedule assumes; the dW schedule assumes nothing.
// (W_NK: the weight is given and its gradient wanted as [N,K]; both bodies in their in-place forms.)
template <class T, class OutDX, class OutDW, int TN_DX, bool PAIRS = false, bool W_NK = false>
__global__ __launch_bounds__(512) void bwd_fused_kernel(GemmParams Pdx, GemmParams Pdw, int g_dx)
{
    if ((int)blockIdx.x < g_dx)
        gemm_persistent_dx_body<T, OutDX, 128, TN_DX, 2, 2, kTailNone, false, PAIRS, W_NK>(Pdx, g_dx, (int)blockIdx.x);
    else
        gemm_persistent_body<DW, T, OutDW, 128, 256, 1, 4, kTailNone, false, false, W_NK>(Pdw, (int)gridDim.x - g_dx, (int)blockIdx.x - g_dx);
}

// The same where dX runs one workgroup per tile (tiles of two kept blocks that are too few per CU
// for the persistent kernel): workgroups [0, n_dx) are those tiles, in the order of the separate
// launch, the rest the persistent dW kernel.
template <class T, class OutDX, class OutDW>
__global__ __launch_bounds__(512) void bwd_fused_tile_kernel(GemmParams Pdx, GemmParams Pdw, int n_dx)
{
    if ((int)blockIdx.x < n_dx)
        gemm_tile_body<DX, T, OutDX, 128, 256, 2, 2, false, true, false>(Pdx, (int)blockIdx.x);
    else
        gemm_persistent_body<DW, T, OutDW, 128, 256, 1, 4, kTailNone>(Pdw, (int)gridDim.x - n_dx, (int)blockIdx.x - n_dx);
}

// Both gradients in one launch for 64 x 64 blocks with short kept lists, where dX and dW both run one
// workgroup per tile (four wavefronts, several workgroups per CU): workgroups [0, n_dx) are dX's tiles,
// the rest dW's, each in the order of its separate launch.
template <class T, class OutDX, class OutDW, int TN_DX>
__global__ __launch_bounds__(256) void bwd_fused_tile64_kernel(GemmParams Pdx, GemmParams Pdw, int n_dx)
{
    if ((int)blockIdx.x < n_dx)
        gemm_tile_body<DX, T, OutDX, 64, TN_DX, 1, 4, false, false, false>(Pdx, (int)blockIdx.x);
    else
        gemm_tile_body<DW, T, OutDW, 64, 256, 1, 4, false, false, false>(Pdw, (int)blockIdx.x - n_dx);
}

}  // namespace
}  // namespace sdrop
#endif
