// The three block-sparse GEMMs of SparseDrop (arxiv 2411.01238, Section 3.1
// eq. (1)-(3), Section 3.2) as one MFMA main loop with three instantiations.
//
//   FWD  Y  = s (X . m') W        tile (block row i, N tile): walks the kept K-blocks of row i
//   DX   dX = s (dY W^T) . m'     tile = 1, 2 or 4 kept blocks of one block row: reduction over all of N
//   DW   dW = s (X . m')^T dY     tile (block column j, N tile): walks the kept row blocks of column j
//
// Two kernel forms share that loop.  gemm_kernel: one launch per tile (ragged edges, and the shapes
// where several co-resident workgroups or the hardware's dynamic dispatch do better).
// gemm_persistent_kernel / gemm_persistent_dx_kernel: one workgroup per CU walks a sequence of
// tiles as one stream of slices, so that the next tile's operands arrive while the current one is
// still multiplied and stored; the host picks between them per call (dispatch_tile).
// bwd_fused_kernel holds the persistent dX and dW workgroups of one layer in a single launch
// (sdrop_bwd).  Kernels with an element-wise tail (bias, activation, ReLU gate: the sparse
// operators around the dropout of Section 4.3's closing remark) are separate instantiations
// of the same templates, so eq. (1)-(3) proper run the code they would without that feature.
//
// Each workgroup owns one TM x TN output tile and steps through its reduction in slices of
// TK = 64 that rotate through LDS stages (three for 128-row tiles, one workgroup per CU; two for
// 64-row tiles, several workgroups per CU).  The paper names the lack of software pipelining as
// the reason its kernels lose to dense at zero sparsity (Section 5.1); here, while the MFMAs of
// slice t run, slice t+1 is complete in LDS and slice t+2 is on its way.  One barrier per slice,
// placed after the first MFMAs of the slice's last quarter so that the matrix pipe has work
// while the wavefronts meet.  Inside a slice every instruction has a fixed place (compile-time
// loops and scheduling fences), because one computing wavefront per SIMD has no other wavefront
// to hide its issue slots.
//
// For 128-row tiles the workgroup has eight wavefronts: four compute (one per SIMD), four only
// issue loads (again one per SIMD).  A load instruction that the memory pipeline holds up then
// stalls a wavefront that has nothing else to do, not the one feeding the matrix pipe
// (measured: 134 -> 119 us for the dense 4096^3 forward).
//
// The matrix-core instruction is v_mfma_f32_32x32x16_{f16,bf16}: lane l supplies row (l%32) of
// one operand and column (l%32) of the other, each as 8 consecutive reduction indices starting
// at 8*(l/32).
//   - Every operand goes HBM -> LDS directly (global_load_lds_dwordx4): no registers, no LDS
//     store instructions, and the LDS pipe stays free for the reads (an LDS store of 1 KiB was
//     measured at 13 clocks, a read at 5.6).
//   - An operand whose reduction index is contiguous in HBM (X in FWD, dY and W in DX) lies in
//     LDS as [rows][64 reduction indices] with 128-byte rows and is read with one 16-byte
//     ds_read_b128 per lane and MFMA.  The 16-byte slot of chunk c in row r is c ^ swz(r) (see
//     lds_off): the direct loads forbid padding, and with this swizzle the reads are free of
//     bank conflicts.
//   - An operand whose reduction index is the strided one (W in FWD; X and dY in DW) stays in
//     LDS as it lies in HBM, [64 reduction rows][columns], and is read with the transposing
//     read of gfx950 (two ds_read_b64_tr_b16 per operand).
//   - Only a ragged edge (N not a multiple of the tile in FWD / DW, N not a multiple of 64 in
//     DX) sends the affected operand through registers, which zero-fill the tail and, for the
//     strided operand, transpose 8 x NW patches with byte permutes on the way.
// The MFMAs are issued with the operands swapped (B's columns as the instruction's rows), so
// that an accumulator register quad holds four consecutive output columns for the epilogue.
//
// On this chip the loop is limited by power, not by issue slots: the shader clock, read in the
// loop, is ~2.0 GHz with the MFMAs alone, ~1.55 GHz once the operand reads from LDS are added
// and ~1.4 GHz with the loads as well, at 84 % MFMA duty (1214 clocks per slice against 1024).
#include "sdrop_internal.h"
#include <limits.h>
#include <stdlib.h>
#include <type_traits>
#include <utility>

namespace sdrop {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(_Float16)))) _Float16 f16x8;
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(8 * sizeof(short)))) short s16x8;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

struct F16 {};
struct BF16 {};

template <class T> struct In;
template <> struct In<F16> {
    using vec = f16x8;
    using out16 = _Float16;
    __device__ static f32x16 mfma(vec a, vec b, f32x16 c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
    }
};
template <> struct In<BF16> {
    using vec = bf16x8;
    using out16 = __bf16;
    __device__ static f32x16 mfma(vec a, vec b, f32x16 c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
};

// Compile-time loop: f(integral_constant<int, 0>{}), ..., f(integral_constant<int, N-1>{}).
template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F> __device__ __forceinline__ void static_for(F &&f)
{
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

constexpr int TK = 64;           // reduction slice staged per step
constexpr int kThreads = 256;    // 4 wavefronts per workgroup
// LDS stages: three for tiles of 128 rows (one workgroup per CU; the deeper prefetch measured
// faster than two co-resident workgroups with two stages: 93 vs 120 us for dX at 4096^3, p=0.5);
// two for tiles of 64 rows, so that two or three workgroups share a CU (measured faster there).
constexpr int stages_for(int tm, int tn) { return (void)tn, tm <= 64 ? 2 : 3; }

enum Op { FWD = 0, DX = 1, DW = 2 };

// A value that is the same in every lane, told to the compiler (it then lives in a scalar register
// and everything derived from it is scalar arithmetic).
__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }


#ifdef SDROP_GEMM_TIMING   // development aid: per-workgroup phase timestamps
__device__ long long g_ticks[16384 * 16];
#define GEMM_TICK(n) do { if (threadIdx.x == 0 && blockIdx.x < 16384) { g_ticks[blockIdx.x * 16 + (n)] = wall_clock64(); g_ticks[blockIdx.x * 16 + 8 + (n)] = clock64(); } } while (0)
#define GEMM_TICKW(n) do { if (threadIdx.x == 0 && blockIdx.x < 16384 && (n) < 16) g_ticks[blockIdx.x * 16 + (n)] = wall_clock64(); } while (0)
#else
#define GEMM_TICK(n) do { } while (0)
#define GEMM_TICKW(n) do { } while (0)
#endif

struct GemmParams {
    const char *A;      // FWD: X   DX: dY  DW: X
    const char *B;      // FWD: W   DX: W   DW: dY
    char *C;            // FWD: Y   DX: dX  DW: dW
    MaskView mv;
    int64_t M, K, N;
    int32_t BM, BK, MB, KB;
    int32_t n_tiles;    // FWD/DW: TN-wide tiles along N.  DX: groups of kept blocks per block row
    int32_t splits;     // DW: parts the kept-row list of a block column is cut into (1 = no split)
    int32_t total_tiles; // persistent kernels: tiles of the whole launch
    float scale;
    // optional element-wise tail of FWD and DX (see Tail below); all null / 0 for eq. (1)-(3) proper
    const float *bias;
    const char *aux;
    int32_t act;
    double p;           // host only: dropout probability, for choosing tile shapes
};

// 16 bytes of output, as a non-temporal store.  Outputs are written once and not read again by the
// kernel that writes them; stored this way they neither displace operand tiles from the L2s and
// the Infinity Cache nor wait there, dirty, for the write-back at the end of the kernel (4096^3,
// half the blocks kept, operands outside the Infinity Cache: 224 -> 208 us per step).
__device__ __forceinline__ void store_out(char *p, uint4 v)
{
    typedef __attribute__((__vector_size__(4 * sizeof(unsigned)))) unsigned u32x4;
    const u32x4 w = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(w, reinterpret_cast<u32x4 *>(p));
}

// Element-wise tail applied to the scaled fp32 accumulator before the single rounding, for the
// layers around the dropout (Section 4.3, closing remark: sparse operators for the layer before
// the dropout as well):  out = [aux > 0] act(scale * acc + bias[column]).
//   bias  fp32, one value per output column
//   act   SDROP_ACT_RELU: max(v, 0);  SDROP_ACT_GELU_TANH: v / (1 + exp(-2 c (v + 0.044715 v^3))),
//         c = sqrt(2/pi), which is 0.5 v (1 + tanh(c (v + 0.044715 v^3)))
//   aux   matrix of the operands' type and the output's shape; where it is not > 0 the output
//         is 0 (the backward of a ReLU whose output was kept)
struct Tail {
    const float *bias;
    const char *aux;
    const char *c0;     // the output's origin
    int act;
};
__device__ __forceinline__ Tail make_tail(const GemmParams &P)
{
    Tail t;
    t.bias = P.bias; t.aux = P.aux; t.c0 = P.C; t.act = P.act;
    return t;
}
// v: four consecutive columns of one output row, starting at global column `col`; `elem` is the
// index of v[0] in the output matrix (row * columns + col).  col is a multiple of 4.  The gate is
// applied here only with AUX; the persistent kernels gate their 16-bit outputs after rounding
// instead, 16 bytes at a time (gate16), which selects the same values.
// The bias does not change while the kernel runs: read through the constant address space, its
// loads may be moved and merged across the output stores.
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef const __attribute__((address_space(4))) f32x4 *const_f4;
__device__ __forceinline__ void act4(int act, float (&v)[4])
{
    if (act == SDROP_ACT_RELU) {
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = v[e] < 0.f ? 0.f : v[e];
    } else if (act == SDROP_ACT_GELU_TANH) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float x = v[e];
            const float u = 0.7978845608028654f * (x + 0.044715f * x * x * x);
            v[e] = x * __builtin_amdgcn_rcpf(1.f + __expf(-2.f * u));
        }
    }
}
template <class T, bool AUX>
__device__ __forceinline__ void tail4(const Tail &tl, float (&v)[4], int64_t col, int64_t elem)
{
    if (tl.bias) {
        const f32x4 b = *(const_f4)(uintptr_t)(tl.bias + col);
        v[0] += b.x; v[1] += b.y; v[2] += b.z; v[3] += b.w;
    }
    act4(tl.act, v);
    if constexpr (AUX) {
        if (tl.aux) {
            using E = typename In<T>::out16;
            typedef __attribute__((__vector_size__(4 * sizeof(E)))) E e4;
            const e4 x = *reinterpret_cast<const e4 *>(tl.aux + elem * (int64_t)sizeof(E));
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = static_cast<float>(x[e]) > 0.f ? v[e] : 0.f;
        }
    }
}
// Eight 16-bit outputs and the eight gate values at the same place of the gate matrix.
template <class T>
__device__ __forceinline__ uint4 gate16(uint4 out, uint4 gate)
{
    using E = typename In<T>::out16;
    typedef __attribute__((__vector_size__(8 * sizeof(E)))) E e8;
    e8 o = __builtin_bit_cast(e8, out);
    const e8 g = __builtin_bit_cast(e8, gate);
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = static_cast<float>(g[e]) > 0.f ? o[e] : static_cast<E>(0.f);
    return __builtin_bit_cast(uint4, o);
}

// Slot swizzle of an LDS operand row: a 3-bit value XORed into the chunk index.
// With m = (r>>1)&7: rotate m left by one and flip with bits 4,5 of r.  Measured
// conflict-free for ds_read_b128 of 32 consecutive rows x 2 chunks per wavefront,
// for row-wise 16-byte stores and for the transposed stores below.
__device__ __forceinline__ int swz(int r)
{
    const int m = (r >> 1) & 7;
    return (((m & 3) << 1) | (m >> 2)) ^ ((r >> 3) & 6);
}
// Byte offset of 16-byte chunk c (0..7) of row r in an LDS operand tile.
__device__ __forceinline__ int lds_off(int r, int c) { return r * 128 + (((c ^ swz(r)) & 7) << 4); }

// One global_load_lds_dwordx4: every lane moves 16 bytes from sbase + voff (uniform 64-bit base
// plus 32-bit lane offset) to LDS byte address lds_base + 16*lane.  Written as inline assembly on
// purpose: the compiler then does not know that LDS is written behind its back, and does not make
// every later LDS read wait for ALL outstanding vector-memory operations (which is what it does
// for the builtin form as soon as a transposing LDS read is involved, serialising the pipeline).
// The price is that completion is tracked by hand: explicit s_waitcnt vmcnt(n) before the barrier
// that publishes a slice.
__device__ __forceinline__ void dma16(const char *sbase, uint32_t voff, const char *lds)
{
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char *)lds;
    asm volatile("s_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(sbase), "{m0}"(lds_base));
}

// HBM -> LDS without registers, for an operand tile [ROWS][64] whose rows lie ld_bytes
// apart in HBM (reduction index contiguous).  One instruction of one wavefront fills
// 1 KiB = 8 LDS rows: lane l lands in row 8*I + l/8, slot l%8, so it fetches chunk
// (l%8) ^ swz(row) of that row.  Wavefront w of NW issues instructions I = w + NW*i.  Row of
// this lane in pass i is r = 8*NW*i + r0; of the pass offset swz(r) sees only bit 5, so two
// lane offsets serve every pass and the rest of the address is uniform.
template <int ROWS, int NGRP, int NW> struct DmaK {
    static constexpr int PASS_ROWS = 8 * NW;              // rows filled by one pass of the NW wavefronts
    static constexpr int PER_WAVE = ROWS / PASS_ROWS, GROUP_ROWS = ROWS / NGRP;
    static_assert(GROUP_ROWS % PASS_ROWS == 0 && ROWS % PASS_ROWS == 0, "row groups must cover whole passes");
    uint32_t voff_even, voff_odd;
    int wave;
    __device__ __forceinline__ void init(int64_t ld_bytes, int w)
    {
        const int lane = threadIdx.x & 63;
        wave = w;
        const int r0 = 8 * wave + (lane >> 3);
        const uint32_t row_off = (uint32_t)r0 * (uint32_t)ld_bytes;
        voff_even = row_off + (((lane & 7) ^ swz(r0)) << 4);
        voff_odd = row_off + (((lane & 7) ^ swz(r0) ^ 4) << 4);
    }
    // pass i of this wavefront
    __device__ __forceinline__ void issue(const char *const (&base)[NGRP], int64_t ld_bytes, char *lds, int i) const
    {
        const int g = (PASS_ROWS * i) / GROUP_ROWS;       // uniform: pass i covers rows PASS_ROWS*i ..
        const char *sbase = base[g] + (int64_t)(PASS_ROWS * i - g * GROUP_ROWS) * ld_bytes;
        // bit 5 of the row (the only bit of a pass offset that swz() sees) picks the lane offset
        dma16(sbase, ((PASS_ROWS * i) & 32) ? voff_odd : voff_even, lds + (wave + NW * i) * 1024);
    }
};

// Slot swizzle of an LDS tile kept as it lies in HBM when the reduction index is the strided
// one: [64 reduction rows][ROWS contiguous].  The transposing read of one 16-lane group
// touches 4 consecutive rows x 32 bytes; XORing the 64-byte slot index with (row & 3) (with
// (row>>1)&1 for 128-byte rows) keeps those rows on different banks.
template <int ROWS> __device__ __forceinline__ int swz_t(int k)
{
    return ROWS >= 128 ? ((k & 3) << 2) : (((k >> 1) & 1) << 2);
}

// HBM -> LDS without registers for an operand tile [64][ROWS] (ROWS contiguous, rows ld_bytes
// apart).  One instruction fills 1 KiB = 1024/(2*ROWS) tile rows; lane l lands at byte 16*l of
// it and fetches the chunk whose swizzled slot that is.  Row k = RPI*I + kl with I = w + NW*i:
// k & 3 (or (k>>1)&1) does not depend on i, so one lane offset serves every pass.
template <int ROWS, int NW> struct DmaT {
    static constexpr int ROW_BYTES = 2 * ROWS, RPI = 1024 / ROW_BYTES;       // rows per instruction
    static constexpr int PER_WAVE = ROWS / (8 * NW);
    static_assert(ROWS % (8 * NW) == 0, "every wavefront issues whole instructions");
    static_assert(ROWS == 64 || ROWS == 128 || ROWS == 256, "unsupported tile edge");
    uint32_t voff;
    int wave;
    __device__ __forceinline__ void init(int64_t ld_bytes, int w)
    {
        const int lane = threadIdx.x & 63;
        wave = w;
        const int kl = (lane * 16) / ROW_BYTES;              // row within the instruction
        const int cpos = ((lane * 16) % ROW_BYTES) >> 4;     // 16-byte slot within the row
        const int k0 = RPI * wave + kl;
        voff = (uint32_t)kl * (uint32_t)ld_bytes + ((cpos ^ swz_t<ROWS>(k0)) << 4);
    }
    __device__ __forceinline__ void issue(const char *const (&base)[1], int64_t ld_bytes, char *lds, int i) const
    {
        const int I = wave + NW * i;
        dma16(base[0] + (int64_t)(RPI * I) * ld_bytes, voff, lds + I * 1024);
    }
};

// A slice of an operand on its way from HBM to LDS through registers.
//
// KMAJ:  HBM tile [ROWS][64], rows ld_bytes apart.  Thread t moves 16-byte chunks
//        t, t+256, ...: chunk q is row q/8, chunk q%8.  The rows may come from up to
//        NGRP row groups with separate base pointers.
// !KMAJ: HBM tile [64][ROWS] (ROWS contiguous).  Thread t owns reduction rows
//        8*(t/32)..+8 and columns NW*(t%32)..+NW, NW = ROWS/32, and turns them
//        into NW LDS rows of one 16-byte chunk each.
// RAGGED: chunks beyond `lim` valid elements of the contiguous dimension read as zero.
template <bool KMAJ, int ROWS, bool RAGGED, int NGRP = 1> struct Slice {
    static constexpr int NW = ROWS / 32;                       // !KMAJ: columns per thread
    static constexpr int NCH = KMAJ ? ROWS * 8 / kThreads : 1; // KMAJ: chunks per thread
    static constexpr int ND = KMAJ ? 4 * NCH : 4 * NW;         // dwords held
    static constexpr int NLOADS = KMAJ ? NCH : 8;
    static constexpr int NSTORES = KMAJ ? NCH : NW;
    static constexpr int NPERMS = KMAJ ? 0 : 4 * NW;
    static constexpr int GROUP_ROWS = ROWS / NGRP;
    static_assert(ROWS % 32 == 0 && (KMAJ ? NCH >= 1 : (NW == 2 || NW == 4 || NW == 8)), "unsupported tile edge");
    static_assert(!KMAJ || NGRP == 1 || (GROUP_ROWS % 32 == 0), "row groups must cover whole passes");
    uint32_t d[ND];

    template <class V> __device__ __forceinline__ static V ld(const char *p, const char *safe, bool ok)
    {
        if constexpr (RAGGED) {
            V v = *reinterpret_cast<const V *>(ok ? p : safe);   // `safe` is the (valid) start of the row
            V z = {};
            return ok ? v : z;
        } else {
            return *reinterpret_cast<const V *>(p);
        }
    }

    // base[g]: start of row group g (uniform).  lim = valid elements along the contiguous
    // dimension.  Addresses are a uniform 64-bit base plus one 32-bit lane offset, so that the
    // loads take the scalar-base form and no 64-bit lane addresses are kept in registers.
    __device__ __forceinline__ void load(const char *const (&base)[NGRP], int64_t ld_bytes, int lim)
    {
        if constexpr (KMAJ) {
            const int cc = threadIdx.x & 7;
            const uint32_t voff = (uint32_t)(threadIdx.x >> 3) * (uint32_t)ld_bytes + cc * 16;
            const bool ok = cc * 8 < lim;
#pragma unroll
            for (int q = 0; q < NCH; ++q) {
                const int g = (q * 32) / GROUP_ROWS;           // rows of pass q: 32q .. 32q+31
                const char *sbase = base[g] + (int64_t)(32 * q - g * GROUP_ROWS) * ld_bytes;
                const uint4 v = ld<uint4>(sbase + voff, sbase, ok);
                d[4 * q] = v.x; d[4 * q + 1] = v.y; d[4 * q + 2] = v.z; d[4 * q + 3] = v.w;
            }
        } else {
            const int ng = threadIdx.x & 31, kc = threadIdx.x >> 5;
            const uint32_t voff = (uint32_t)(kc * 8) * (uint32_t)ld_bytes + ng * (NW * 2);
            const bool ok = ng * NW < lim;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const char *sbase = base[0] + (int64_t)i * ld_bytes;
                if constexpr (NW == 8) {
                    const uint4 v = ld<uint4>(sbase + voff, sbase, ok);
                    d[4 * i] = v.x; d[4 * i + 1] = v.y; d[4 * i + 2] = v.z; d[4 * i + 3] = v.w;
                } else if constexpr (NW == 4) {
                    const uint2 v = ld<uint2>(sbase + voff, sbase, ok);
                    d[2 * i] = v.x; d[2 * i + 1] = v.y;
                } else {
                    d[i] = ld<uint32_t>(sbase + voff, sbase, ok);
                }
            }
        }
    }

    // Stores part PART of NPARTS equal parts of this slice (so that the stores can be
    // spread over several MFMA groups).
    template <int PART, int NPARTS> __device__ __forceinline__ void store(char *lds) const
    {
        constexpr int PER = NSTORES / NPARTS;
        static_assert(NSTORES % NPARTS == 0, "parts must divide the stores");
        if constexpr (KMAJ) {
#pragma unroll
            for (int q = PART * PER; q < (PART + 1) * PER; ++q) {
                const int c = threadIdx.x + q * kThreads;
                *reinterpret_cast<uint4 *>(lds + lds_off(c >> 3, c & 7)) =
                    make_uint4(d[4 * q], d[4 * q + 1], d[4 * q + 2], d[4 * q + 3]);
            }
        } else {
            // d[(NW/2)*i + w] holds columns 2w (low half) and 2w+1 (high half) of reduction row i.
            // LDS row n gets (row 0, row 1), (row 2, row 3), ... of column n as four dwords.
            const int ng = threadIdx.x & 31, kc = threadIdx.x >> 5;
            constexpr int DW_PER_ROW = NW / 2;
#pragma unroll
            for (int n = PART * PER; n < (PART + 1) * PER; ++n) {
                const uint32_t sel = (n & 1) ? 0x07060302u : 0x05040100u;
                uint32_t o[4];
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    o[j] = __builtin_amdgcn_perm(d[DW_PER_ROW * (2 * j + 1) + n / 2], d[DW_PER_ROW * (2 * j) + n / 2], sel);
                *reinterpret_cast<uint4 *>(lds + lds_off(ng * NW + n, kc)) = make_uint4(o[0], o[1], o[2], o[3]);
            }
        }
    }
};

// MFMA operand for the 32 rows (or columns) starting at `base32` of an LDS operand tile,
// reduction indices [kk*16, kk*16+16): lane l gets index base32 + l%32, reduction 8*(l/32)..+8.
// TR = false: tile [rows][64], one ds_read_b128.  TR = true: tile [64][ROWS] as in HBM, two
// transposing reads (ds_read_b64_tr_b16): within a group of 16 lanes, lane q loads 4 elements
// of row q/4 at columns 4*(q%4).. and receives column q of that 4 x 16 patch.
template <class T, bool TR, int ROWS>
__device__ __forceinline__ typename In<T>::vec read_frag(const char *lds, int base32, int kk)
{
    const int l = threadIdx.x & 63;
    if constexpr (!TR) {
        return *reinterpret_cast<const typename In<T>::vec *>(lds + lds_off(base32 + (l & 31), kk * 2 + (l >> 5)));
    } else {
        constexpr int ROW_BYTES = 2 * ROWS;
        const int k = kk * 16 + (l >> 5) * 8 + ((l & 15) >> 2);
        const int col = base32 + ((l >> 4) & 1) * 16 + (l & 3) * 4;
        const char *p = lds + k * ROW_BYTES + ((((col >> 3) ^ swz_t<ROWS>(k))) << 4) + ((col * 2) & 15);
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p + 4 * ROW_BYTES));
        const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        return __builtin_bit_cast(typename In<T>::vec, v);
    }
}

// Scheduling recipe for one MFMA group: each of the NM MFMAs is followed by its share of
// the LDS reads, global loads, VALU ops and LDS writes that were emitted with it.
constexpr int ceil_div(int a, int b) { return (a + b - 1) / b; }
template <int NM, int NDSR, int NVALU, int NDSW, int NVMEM>
__device__ __forceinline__ void interleave()
{
#pragma unroll
    for (int i = 0; i < NM; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                   // MFMA
        if constexpr (NDSR > 0) __builtin_amdgcn_sched_group_barrier(0x100, ceil_div(NDSR, NM), 0);   // DS read
        if constexpr (NVMEM > 0) __builtin_amdgcn_sched_group_barrier(0x020, ceil_div(NVMEM, NM), 0); // VMEM read
        if constexpr (NVALU > 0) __builtin_amdgcn_sched_group_barrier(0x002, ceil_div(NVALU, NM), 0); // VALU
        if constexpr (NDSW > 0) __builtin_amdgcn_sched_group_barrier(0x200, ceil_div(NDSW, NM), 0);   // DS write
    }
    __builtin_amdgcn_sched_barrier(0);
}

// s_waitcnt immediate (gfx9 encoding): wait until at most `vm` vector-memory operations
// are outstanding and all LDS/scalar operations have completed.
constexpr int waitcnt_vm_lgkm0(int vm) { return (vm & 15) | ((vm >> 4) << 14) | (7 << 4) | (0 << 8); }

// SPEC: the workgroup has NW more wavefronts (one more per SIMD) that do nothing but issue the
// direct loads, so that a load instruction held up by the memory pipeline never holds up MFMAs.
// (The body is a device function of the tile number, so that one launch can hold the workgroups
// of two operations; see bwd_fused_tile_kernel.)
template <int OP, class T, class OutT, int TM, int TN, int WM, int WN, bool RAGGED, bool SPEC, bool TAIL>
__device__ __forceinline__ void gemm_tile_body(const GemmParams &P, const int bid)
{
    constexpr int NW = WM * WN, NT = NW * 64 * (SPEC ? 2 : 1);   // computing wavefronts; threads
    static_assert(NW == 4 || (NW == 8 && !RAGGED), "4 wavefronts (8 only without the register path)");
    static_assert(!(SPEC && RAGGED), "loader wavefronts exist only where every operand is loaded directly");
    constexpr int WTM = TM / WM, WTN = TN / WN, MI = WTM / 32, NI = WTN / 32;
    static_assert(MI >= 1 && NI >= 1 && WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be 32-aligned");
    constexpr bool A_KMAJ = (OP != DW), B_KMAJ = (OP == DX);    // reduction index contiguous in HBM?
    // Operands go HBM -> LDS directly unless a ragged edge needs zero fill (the reduction tail
    // of DX, the N tail of W / dY in FWD / DW); those go through registers.
    constexpr bool A_DMA = !(RAGGED && OP == DX);
    constexpr bool B_DMA = !RAGGED;
    // A directly loaded operand whose reduction index is strided in HBM stays in that form in
    // LDS and is read with transposing reads.
    constexpr bool A_TR = A_DMA && !A_KMAJ, B_TR = B_DMA && !B_KMAJ;
    constexpr int A_BYTES = TM * TK * 2, B_BYTES = TN * TK * 2, STAGE_BYTES = A_BYTES + B_BYTES;
    constexpr int STAGES = stages_for(TM, TN);
    constexpr int AHEAD = STAGES - 1;          // a direct load issued in iteration s brings slice s + AHEAD
    constexpr int NGRP_MAX = 4;

    extern __shared__ __attribute__((aligned(16))) char smem[];

    GEMM_TICK(0);
    // a kernel handed a mask built for another problem writes nothing
    const MaskHeader *H = P.mv.hdr;
    if (H->magic != kMaskMagic || H->M != P.M || H->K != P.K || H->BM != P.BM || H->BK != P.BK) return;

    constexpr int esz = 2;
    const int lane = threadIdx.x & 63;
    const int wave_all = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const bool loader = SPEC && wave_all >= NW;          // uniform over the wavefront
    const int wave = loader ? wave_all - NW : wave_all;  // index among the wavefronts of the same role
    const int wm = wave / WN, wn = wave % WN;

    const char *a_tile = nullptr, *b_tile = nullptr;
    int64_t lda, ldb, ldc;                              // in bytes
    char *c_tile = nullptr;
    int c_lim = TN;                                     // valid output columns in this tile
    int nsteps = 0, sub_shift = 0;                      // reduction steps; log2(TK-slices per mask block)
    const int32_t *list = nullptr;                      // kept-block list walked by this tile
    int list_len = 0;
    // DX only: the tile's TN columns are DXG chunks of 64, each a (half) kept block of W / dX
    constexpr int DXG = (OP == DX) ? TN / 64 : 1;
    static_assert(DXG <= NGRP_MAX, "DX tile too wide");
    const char *bgrp[NGRP_MAX] = {nullptr, nullptr, nullptr, nullptr};
    char *cgrp[NGRP_MAX] = {nullptr, nullptr, nullptr, nullptr};
    int chunks_valid = 0;                               // 64-column chunks that hold real blocks
    // for the element-wise tail: global row of the tile's first row; global column of the tile
    // (FWD) or of each 64-column chunk (DX)
    int64_t out_row0 = 0;
    int out_col0[NGRP_MAX] = {0, 0, 0, 0};

    if constexpr (OP == FWD) {
        const int t = bid;
        const int rank = t / P.n_tiles, nt = t % P.n_tiles;
        const int i = uni(P.mv.row_order[rank]);
        const int rp = uni(P.mv.row_ptr[i]);
        list = P.mv.col_idx + rp;
        list_len = uni(P.mv.row_ptr[i + 1]) - rp;
        sub_shift = (P.BK == 128);
        nsteps = list_len << sub_shift;
        lda = P.K * esz; ldb = P.N * esz; ldc = P.N * (int64_t)sizeof(OutT);
        a_tile = P.A + (int64_t)i * P.BM * lda;
        b_tile = P.B + (int64_t)nt * TN * esz;
        c_tile = P.C + (int64_t)i * P.BM * ldc + (int64_t)nt * TN * sizeof(OutT);
        out_row0 = (int64_t)i * P.BM;
        out_col0[0] = nt * TN;
        { const int64_t left = P.N - (int64_t)nt * TN; c_lim = left < TN ? (int)left : TN; }
    } else if constexpr (OP == DW) {
        // bid = (rank of block column j in the schedule, N tile, part of the list)
        const int t = bid;
        const int per_col = P.n_tiles * P.splits;
        const int j = uni(P.mv.col_order[t / per_col]);
        const int nt = (t % per_col) / P.splits, part = t % P.splits;
        const int cp = uni(P.mv.col_ptr[j]);
        const int cnt = uni(P.mv.col_ptr[j + 1]) - cp;
        const int lo = (int)((int64_t)cnt * part / P.splits), hi = (int)((int64_t)cnt * (part + 1) / P.splits);
        list = P.mv.row_idx + cp + lo;
        list_len = hi - lo;
        sub_shift = (P.BM == 128);
        nsteps = list_len << sub_shift;
        lda = P.K * esz; ldb = P.N * esz; ldc = P.N * (int64_t)sizeof(OutT);
        a_tile = P.A + (int64_t)j * P.BK * esz;
        b_tile = P.B + (int64_t)nt * TN * esz;
        // with a split list, part `part` writes its own K x N plane of partial sums
        c_tile = P.C + (int64_t)part * P.K * ldc + (int64_t)j * P.BK * ldc + (int64_t)nt * TN * sizeof(OutT);
        { const int64_t left = P.N - (int64_t)nt * TN; c_lim = left < TN ? (int)left : TN; }
    } else {
        const int G_ = TN / P.BK;                     // kept blocks gathered into one tile
        lda = P.N * esz; ldb = P.N * esz; ldc = P.K * (int64_t)sizeof(OutT);
        const int cshift = (P.BK == 128);             // 64-column chunks per block, log2
        const int row_chunks = P.BK * (int)sizeof(OutT) / 16;
        auto zero_block = [&](int zi, int zj) __attribute__((always_inline)) {
            char *z = P.C + (int64_t)zi * P.BM * ldc + (int64_t)zj * P.BK * sizeof(OutT);
            for (int c = threadIdx.x; c < TM * row_chunks; c += NT)
                store_out(z + (c / row_chunks) * ldc + (c % row_chunks) * 16, make_uint4(0, 0, 0, 0));
        };
        int i, blocks_valid;                          // block row; kept blocks in this tile (<= 0: nothing to compute)
        int jg[NGRP_MAX] = {0, 0, 0, 0};
        // In both forms every index is fetched before the zero fill: a load that follows a store
        // cannot be proven unaliased and would lose its scalar form.
        if (G_ == 1) {
            // One kept block per tile.  Two duties per workgroup.  (1) Zero fill: block position
            // bid, if it is dropped.  (2) Compute: kept block e of the mask's locally ordered list
            // (groups of 8 block rows, column by column), where the hardware's round-robin placement
            // of workgroups on the 8 XCDs is undone: workgroup b runs on XCD b % 8 and takes
            // e = (b % 8) * ceil(nnz / 8) + b / 8.  Every XCD so gets the same number of tiles (its CUs
            // run one workgroup each, so a single extra tile on one XCD costs a whole round: 3 instead
            // of 2 at 4096^3 with half the blocks kept), and the ~32 tiles that run on it at one time
            // cover about 8 block rows x 8 block columns, so that each dY and W tile it fetches from
            // HBM serves several of them (measured at 4096^3, half kept, operands not in the Infinity
            // Cache: 78 us against 86-100 us in row-major order).
            const int b = bid;
            const int nnz = H->nnz;
            const int per_xcd = (nnz + 7) >> 3;
            const int e = (b & 7) * per_xcd + (b >> 3);
            const bool computes = (b >> 3) < per_xcd && e < nnz;
            const int ec = computes ? e : 0;          // the lists have room for at least one entry
            i = uni(P.mv.loc_row[ec]);
            jg[0] = uni(P.mv.loc_col[ec]);
#pragma unroll
            for (int g = 1; g < DXG; ++g) jg[g] = jg[0];
            const int total = P.MB * P.KB;
            const int zb = b < total ? b : total - 1;
            const int zi = zb / P.KB, zj = zb % P.KB;
            const uint64_t zword = P.mv.bits[(int64_t)zi * H->words_per_row + (zj >> 6)];
            if (b < total && !((zword >> (zj & 63)) & 1)) zero_block(zi, zj);
            blocks_valid = computes ? 1 : 0;
        } else {
            // bid = q * MB + i.  The workgroup computes the kept blocks of ranks
            // [q*G, q*G+G) of block row i as one TM x (G*BK) tile, and zero-fills the block
            // positions [q*G, q*G+G) of row i that are dropped.
            i = bid % P.MB;
            const int q = bid / P.MB;
            const int rp = uni(P.mv.row_ptr[i]);
            const int cnt = uni(P.mv.row_ptr[i + 1]) - rp;
            blocks_valid = cnt - q * G_ < G_ ? cnt - q * G_ : G_;
            if (blocks_valid > 0) {
#pragma unroll
                for (int g = 0; g < DXG; ++g) {
                    const int bb = g >> cshift;       // which of the gathered blocks (a missing one repeats the last)
                    jg[g] = uni(P.mv.col_idx[rp + q * G_ + (bb < blocks_valid ? bb : blocks_valid - 1)]);
                }
            }
            uint64_t keep_word[2];                    // the bits of positions [q*G_, q*G_ + G_) lie in at most two words
            const int pos0 = q * G_;
            {
                const uint64_t *row_bits = P.mv.bits + (int64_t)i * H->words_per_row;
                const int w0 = pos0 >> 6, w1 = (pos0 + G_ - 1) >> 6, wmax = (P.KB - 1) >> 6;
                keep_word[0] = row_bits[w0 < wmax ? w0 : wmax];
                keep_word[1] = row_bits[w1 < wmax ? w1 : wmax];
            }
            for (int g = 0; g < G_; ++g) {
                const int pos = pos0 + g;
                const uint64_t word = keep_word[(pos >> 6) != (pos0 >> 6)];
                if (pos < P.KB && !((word >> (pos & 63)) & 1)) zero_block(i, pos);
            }
        }
        chunks_valid = blocks_valid << cshift;
        if (blocks_valid <= 0) return;
#pragma unroll
        for (int g = 0; g < DXG; ++g) {
            const int64_t col0 = (int64_t)jg[g] * P.BK + (g & ((1 << cshift) - 1)) * 64;
            bgrp[g] = P.B + col0 * ldb;
            cgrp[g] = P.C + (int64_t)i * P.BM * ldc + col0 * sizeof(OutT);
            out_col0[g] = (int)col0;
        }
        out_row0 = (int64_t)i * P.BM;
        nsteps = (int)((P.N + TK - 1) / TK);
        a_tile = P.A + (int64_t)i * P.BM * lda;
    }

    f32x16 acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;

    GEMM_TICK(1);
    if (nsteps > 0) {
        using SliceA = Slice<A_KMAJ, TM, RAGGED && OP == DX>;
        using SliceB = Slice<B_KMAJ, TN, RAGGED, DXG>;
        SliceA ra;      // used only when !A_DMA
        SliceB rb;      // used only when !B_DMA

        // Kept-block indices: lane l holds entries 64*ch + l (idx_a) and 64*(ch+1) + l (idx_b)
        // of the list, so that positions up to 64 apart can be looked up.
        int idx_a = 0, idx_b = 0, idx_ch = 0;
        auto list_at = [&](int e) __attribute__((always_inline)) { return list[e < list_len ? e : list_len - 1]; };
        if constexpr (OP != DX) { idx_a = list_at(lane); idx_b = list_at(64 + lane); }
        // make the list position of step s available; runs outside the scheduled code
        auto refresh_for = [&](int s) __attribute__((always_inline)) {
            if constexpr (OP != DX) {
                const int sc = s < nsteps ? s : nsteps - 1;
                if (((sc >> sub_shift) >> 6) > idx_ch + 1) {
                    ++idx_ch;
                    idx_a = idx_b;
                    idx_b = list_at((idx_ch + 1) * 64 + lane);
                }
            }
        };
        auto block_at = [&](int pos) __attribute__((always_inline)) -> int {         // pos is uniform
            const int va = __builtin_amdgcn_readlane(idx_a, pos & 63);
            const int vb = __builtin_amdgcn_readlane(idx_b, pos & 63);
            return (pos >> 6) == idx_ch ? va : vb;
        };

        // Position of slice s along the reduction, in elements (clamped to the last slice: the
        // pipeline runs ahead of the loop and re-fetches the last slice rather than branch)
        auto offset_of = [&](int s) __attribute__((always_inline)) -> int64_t {
            const int sc = s < nsteps ? s : nsteps - 1;
            if constexpr (OP == FWD) {
                return (int64_t)block_at(sc >> sub_shift) * P.BK + (int64_t)(sc & ((1 << sub_shift) - 1)) * TK;
            } else if constexpr (OP == DW) {
                return (int64_t)block_at(sc >> sub_shift) * P.BM + (int64_t)(sc & ((1 << sub_shift) - 1)) * TK;
            } else {
                return (int64_t)sc * TK;
            }
        };
        // HBM addresses of the slice at reduction position `off`
        struct Src { const char *a[1]; const char *b[DXG]; int lim; };
        auto src_at = [&](int64_t off) __attribute__((always_inline)) -> Src {
            Src r;
            if constexpr (OP == FWD) {
                r.a[0] = a_tile + off * esz; r.b[0] = b_tile + off * ldb; r.lim = c_lim;
            } else if constexpr (OP == DW) {
                r.a[0] = a_tile + off * lda; r.b[0] = b_tile + off * ldb; r.lim = c_lim;
            } else {
                const int64_t left = P.N - off;
                r.lim = left < TK ? (int)left : TK;
                r.a[0] = a_tile + off * esz;
#pragma unroll
                for (int g = 0; g < DXG; ++g) r.b[g] = bgrp[g] + off * esz;
            }
            return r;
        };
        auto src_of = [&](int s) __attribute__((always_inline)) -> Src { return src_at(offset_of(s)); };
        auto a_lim = [&](const Src &x) __attribute__((always_inline)) { return OP == DX ? x.lim : (OP == FWD ? TK : TM); };

        // direct-load engines (lane offsets computed once)
        using DmaA = typename std::conditional<A_KMAJ, DmaK<TM, 1, NW>, DmaT<TM, NW>>::type;
        using DmaB = typename std::conditional<B_KMAJ, DmaK<TN, DXG, NW>, DmaT<TN, NW>>::type;
        DmaA da;
        DmaB db;
        if constexpr (A_DMA) da.init(lda, wave);
        if constexpr (B_DMA) db.init(ldb, wave);
        constexpr int NDMA_A = A_DMA ? TM / (8 * NW) : 0, NDMA_B = B_DMA ? TN / (8 * NW) : 0;   // per wavefront and slice
        constexpr int NDMA_ITER = NDMA_A + NDMA_B;
        // direct-load instruction j of a slice (A's first, then B's) into stage st
        auto dma_one = [&](const Src &x, char *st, int j) __attribute__((always_inline)) {
            if (j < NDMA_A) { if constexpr (A_DMA) da.issue(x.a, lda, st, j); }
            else { if constexpr (B_DMA) db.issue(x.b, ldb, st + A_BYTES, j - NDMA_A); }
        };
        auto dma_range = [&](const Src &x, char *st, int j0, int j1) __attribute__((always_inline)) {
#pragma unroll
            for (int j = j0; j < j1; ++j) dma_one(x, st, j);
        };

        auto stage_ptr = [&](int st) __attribute__((always_inline)) -> char * { return smem + st * STAGE_BYTES; };
        constexpr int NREG_ITER = (A_DMA ? 0 : SliceA::NLOADS) + (B_DMA ? 0 : SliceB::NLOADS);

        // ---- prologue.  Direct operands: slices 0 and 1 straight to stages 0 and 1.
        //      (with two stages only slice 0).  Register operands: slice 0 to stage 0, slice 1
        //      stays in registers. ----
        {
            const Src s0 = src_of(0);
            if (!SPEC || loader) dma_range(s0, stage_ptr(0), 0, NDMA_ITER);
            if constexpr (!A_DMA) { ra.load(s0.a, lda, a_lim(s0)); ra.template store<0, 1>(stage_ptr(0)); }
            if constexpr (!B_DMA) { rb.load(s0.b, ldb, s0.lim); rb.template store<0, 1>(stage_ptr(0) + A_BYTES); }
            const Src s1 = src_of(1);
            if constexpr (STAGES == 3) { if (!SPEC || loader) dma_range(s1, stage_ptr(1), 0, NDMA_ITER); }
            if constexpr (!A_DMA) ra.load(s1.a, lda, a_lim(s1));
            if constexpr (!B_DMA) rb.load(s1.b, ldb, s1.lim);
            __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(0));
            __builtin_amdgcn_s_barrier();
        }

        typename In<T>::vec fa[2][MI], fb[2][NI];
        auto read_frags = [&](int buf, const char *st, int kk) __attribute__((always_inline)) {
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) fa[buf][mi] = read_frag<T, A_TR, TM>(st, wm * WTM + mi * 32, kk);
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) fb[buf][ni] = read_frag<T, B_TR, TN>(st + A_BYTES, wn * WTN + ni * 32, kk);
        };
        auto mfmas = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NI; ++ni) acc[mi][ni] = In<T>::mfma(fb[buf][ni], fa[buf][mi], acc[mi][ni]);
        };
        constexpr int NM = MI * NI, NOPS = MI + NI;
        // operand reads requested per MFMA in the fine-grained loop (at least what fits the group)
        constexpr int RPM_MIN = ceil_div(NOPS, NM >= 4 ? NM - 2 : NM), RPM = 2 > RPM_MIN ? 2 : RPM_MIN;
        static_assert((NM >= 4 ? NM - 2 : NM) * RPM >= NOPS, "every operand of the next group must be requested within the group");
        constexpr int NFR = MI * (A_TR ? 2 : 1) + NI * (B_TR ? 2 : 1);              // LDS reads per operand set

        int st0 = 0, st1 = 1, st2 = 2;      // stages of slices s, s+1, s+2
        GEMM_TICK(2);
        if (!loader) read_frags(0, stage_ptr(0), 0);

        if (loader) {
            // A loader wavefront: per slice, all of this wavefront's direct loads of slice
            // s + AHEAD, then wait until its loads of slice s + 1 have landed and meet the others.
            if constexpr (SPEC) {
                int64_t nxt_off = offset_of(AHEAD);
                for (int s = 0; s < nsteps; ++s) {
                    char *nx2 = stage_ptr(STAGES == 3 ? st2 : st1);
                    const Src s2 = src_at(nxt_off);
                    refresh_for(s + AHEAD + 1);
                    dma_range(s2, nx2, 0, NDMA_ITER);
                    nxt_off = offset_of(s + 1 + AHEAD);
                    __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(STAGES == 3 ? NDMA_ITER : 0));
                    __builtin_amdgcn_s_barrier();
                    const int t0 = st0; st0 = st1; st1 = (STAGES == 3 ? st2 : t0); st2 = t0;
                }
            }
        } else if constexpr (A_DMA && B_DMA) {
            constexpr bool WITH_DMA = !SPEC;     // otherwise the loader wavefronts issue them
            // Every instruction has its place: MFMA c of a group is followed by its share of the
            // group's operand reads and of the slice's direct loads, and nothing moves across
            // the fence after it.  The direct loads of slice s+2 are spread over groups 0..2.
            // All indices are compile-time so that operands and accumulators stay in registers.
            int64_t nxt_off = WITH_DMA ? offset_of(AHEAD) : 0;
            for (int s = 0; s < nsteps; ++s) {
                const char *cur = stage_ptr(st0);
                const char *nx1 = stage_ptr(st1);
                char *nx2 = stage_ptr(STAGES == 3 ? st2 : st1);      // where this iteration's direct loads land
                const Src s2 = src_at(WITH_DMA ? nxt_off : 0);        // slice s + AHEAD
                if constexpr (WITH_DMA) refresh_for(s + AHEAD + 1);
                __builtin_amdgcn_sched_barrier(0);
                static_for<4>([&](auto gi) __attribute__((always_inline)) {
                    constexpr int g = decltype(gi)::value;
                    // In the last group the first NB MFMAs go out before the barrier (they need only
                    // operands already read), so that the matrix pipe has work while the wavefronts
                    // meet; the operand reads of slice s+1 follow the barrier.
                    constexpr int NB = (g == 3 && NM >= 4) ? 2 : 0;
                    static_for<NM>([&](auto ci) __attribute__((always_inline)) {
                        constexpr int c = decltype(ci)::value;
                        constexpr int mi = c / NI, ni = c % NI, cb = g & 1, nb = (g + 1) & 1;
                        if constexpr (g == 3 && c == NB) {
                            // slice s+1 must have landed everywhere: this wavefront's direct loads of it
                            // were issued one iteration ago (only this iteration's may stay in flight),
                            // and every wavefront must be done reading slice s before its stage is reused
                            __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(!WITH_DMA ? 63 : (STAGES == 3 ? NDMA_ITER : 0)));
                            __builtin_amdgcn_s_barrier();
                            __builtin_amdgcn_sched_barrier(0);
                        }
                        acc[mi][ni] = In<T>::mfma(fb[cb][ni], fa[cb][mi], acc[mi][ni]);
                        // operands for the next group (kk = g+1 of this slice, or kk = 0 of slice s+1) go to the
                        // other register set, so they are requested as early as the group allows, RPM per
                        // MFMA, in the order the next group's MFMAs (A index major) first use them:
                        // A0, B0 .. B(NI-1), A1 .. A(MI-1)
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
                        if constexpr (g < 3 && WITH_DMA) {
                            constexpr int gc = g * NM + c;
                            constexpr int j0 = gc * NDMA_ITER / (3 * NM), j1 = (gc + 1) * NDMA_ITER / (3 * NM);
                            static_for<j1 - j0>([&](auto ji) __attribute__((always_inline)) {
                                constexpr int j = j0 + decltype(ji)::value;
                                if constexpr (j < NDMA_A) da.issue(s2.a, lda, nx2, j);
                                else db.issue(s2.b, ldb, nx2 + A_BYTES, j - NDMA_A);
                            });
                        } else if constexpr (g == 3 && c == 0 && WITH_DMA) {
                            nxt_off = offset_of(s + 1 + AHEAD);   // list lookup for the next iteration
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    });
                });
                const int t0 = st0; st0 = st1; st1 = (STAGES == 3 ? st2 : t0); st2 = t0;
            }
        } else {
            constexpr int A_ST = A_DMA ? 0 : SliceA::NSTORES, A_PM = A_DMA ? 0 : SliceA::NPERMS;
            constexpr int B_ST = B_DMA ? 0 : SliceB::NSTORES, B_PM = B_DMA ? 0 : SliceB::NPERMS;
            for (int s = 0; s < nsteps; ++s) {
                // On entry: slice s complete in stage st0 and its kk=0 operands in flight to
                // fa[0]/fb[0]; direct slice s+1 in flight to st1; register slice s+1 in (ra, rb).
                const char *cur = stage_ptr(st0);
                char *nx1 = stage_ptr(st1), *nx2 = stage_ptr(STAGES == 3 ? st2 : st1);
                refresh_for(s + 2);
                const Src s2 = src_of(s + 2);            // register operands: slice s+2
                const Src sd = src_of(s + AHEAD);        // direct operand: slice s + AHEAD -> nx2
                __builtin_amdgcn_sched_barrier(0);
                // group 0: MFMAs kk=0 | operands kk=1; A: registers -> st1, or HBM -> st2; first half of B -> st1
                read_frags(1, cur, 1);
                if constexpr (A_DMA) dma_range(sd, nx2, 0, NDMA_A); else ra.template store<0, 1>(nx1);
                rb.template store<0, 2>(nx1 + A_BYTES);
                mfmas(0);
                interleave<NM, NFR, A_PM + B_PM / 2 + 2 * NDMA_ITER, A_ST + B_ST / 2, 0>();
                // group 1: MFMAs kk=1 | operands kk=2; second half of B
                read_frags(0, cur, 2);
                rb.template store<1, 2>(nx1 + A_BYTES);
                mfmas(1);
                interleave<NM, NFR, B_PM / 2, B_ST / 2, 0>();
                // group 2: MFMAs kk=2 | operands kk=3; register operands: global loads of slice s+2
                read_frags(1, cur, 3);
                if constexpr (!A_DMA) ra.load(s2.a, lda, a_lim(s2));
                rb.load(s2.b, ldb, s2.lim);
                mfmas(0);
                interleave<NM, NFR, 2 * NREG_ITER, 0, NREG_ITER>();
                __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0((STAGES == 3 ? NDMA_ITER : 0) + NREG_ITER));
                __builtin_amdgcn_s_barrier();
                __builtin_amdgcn_sched_barrier(0);
                // group 3: MFMAs kk=3 | kk=0 operands of slice s+1
                read_frags(0, nx1, 0);
                mfmas(1);
                interleave<NM, NFR, 0, 0, 0>();
                const int t0 = st0; st0 = st1; st1 = (STAGES == 3 ? st2 : t0); st2 = t0;
            }
        }
    }

    // epilogue: scale in fp32, round once, and store whole rows.  The MFMAs were issued with
    // the operands swapped (B's columns as the instruction's rows), so accumulator register r of
    // lane l is row l%32, column 8*(r/4) + 4*(l/32) + r%4 of its 32x32 patch: each register quad
    // is four consecutive columns.  A wavefront parks its WTM x WTN sub-tile in its own piece of
    // LDS (rows padded by one quad against bank conflicts) and writes it out 16 bytes per lane,
    // so that a store instruction covers full 128-byte lines instead of 32 scattered pieces.
    GEMM_TICK(3);
    {
        constexpr int ESZ = (int)sizeof(OutT);
        constexpr int ROWB = WTN * ESZ, RS = ROWB + 4 * ESZ, REGION = WTM * RS;
        static_assert(NW * REGION <= stages_for(TM, TN) * STAGE_BYTES, "epilogue staging must fit in the operand stages");
        // operand stages are dead: no direct load may still be landing, no wavefront still reading
        __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(0));
        __builtin_amdgcn_s_barrier();
        if (loader) return;
        char *reg = smem + wave * REGION;
        const float scale = P.scale;
        const Tail tl = make_tail(P);
        {
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int row = mi * 32 + (lane & 31), col = ni * 32 + q * 8 + (lane >> 5) * 4;
                        float v[4] = {acc[mi][ni][4 * q] * scale, acc[mi][ni][4 * q + 1] * scale,
                                      acc[mi][ni][4 * q + 2] * scale, acc[mi][ni][4 * q + 3] * scale};
                        if constexpr (TAIL && OP != DW) {
                            const int cl = wn * WTN + col;          // column within the tile
                            bool ok;
                            int64_t gcol;
                            if constexpr (OP == DX) {
                                const int g = cl >> 6;
                                ok = g < chunks_valid;
                                int c0 = out_col0[0];
#pragma unroll
                                for (int gg = 1; gg < DXG; ++gg) c0 = (g == gg) ? out_col0[gg] : c0;
                                gcol = c0 + (cl & 63);
                            } else {
                                ok = cl < c_lim;                    // c_lim is a multiple of 8
                                gcol = out_col0[0] + cl;
                            }
                            if (ok) tail4<T, true>(tl, v, gcol, (out_row0 + wm * WTM + row) * (ldc / ESZ) + gcol);
                        }
                        char *dst = reg + row * RS + col * ESZ;
                        if constexpr (ESZ == 4) {
                            *reinterpret_cast<float4 *>(dst) = make_float4(v[0], v[1], v[2], v[3]);
                        } else {
                            typedef __attribute__((__vector_size__(4 * sizeof(OutT)))) OutT out4;
                            const out4 o = {static_cast<OutT>(v[0]), static_cast<OutT>(v[1]), static_cast<OutT>(v[2]), static_cast<OutT>(v[3])};
                            *reinterpret_cast<out4 *>(dst) = o;
                        }
                    }
        }
        constexpr int CH = ROWB / 16, RPI = 64 / CH;         // 16-byte pieces per row; rows per store instruction
        static_assert(CH <= 64 && 64 % CH == 0 && WTM % RPI == 0, "sub-tile rows must tile a wavefront");
#pragma unroll
        for (int it = 0; it < WTM / RPI; ++it) {
            const int row = it * RPI + lane / CH, ch = lane % CH;
            const uint4 v = *reinterpret_cast<const uint4 *>(reg + row * RS + ch * 16);
            int col = wn * WTN + ch * (16 / ESZ);               // column within the tile
            char *cbase = c_tile;
            bool ok = col < c_lim;                             // c_lim is a multiple of 8
            if constexpr (OP == DX) {
                const int g = col >> 6;
                ok = g < chunks_valid;
                cbase = cgrp[0];
#pragma unroll
                for (int gg = 1; gg < DXG; ++gg) cbase = (g == gg) ? cgrp[gg] : cbase;
                col &= 63;
            }
            if (ok) store_out(cbase + (int64_t)(wm * WTM + row) * ldc + col * ESZ, v);
        }
        GEMM_TICK(4);
    }
}

template <int OP, class T, class OutT, int TM, int TN, int WM, int WN, bool RAGGED, bool SPEC, bool TAIL>
__global__ __launch_bounds__(WM * WN * 64 * (SPEC ? 2 : 1)) void gemm_kernel(GemmParams P)
{
    gemm_tile_body<OP, T, OutT, TM, TN, WM, WN, RAGGED, SPEC, TAIL>(P, (int)blockIdx.x);
}

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
    __device__ __forceinline__ void slice(const char *cur, const char *nx1)
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
                acc[mi][ni] = In<T>::mfma(fb[cb][ni], fa[cb][mi], acc[mi][ni]);
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
    // The tail's operands (bias values, and for 16-bit outputs the gate values, which lie where
    // the outputs go) are requested by tail_prefetch, called with the same dst before the tile's
    // last slice: their latency then hides behind that slice's MFMAs instead of adding to the
    // epilogue, which nothing overlaps.
    uint4 gate_r[MI * NJ][4];
    f32x4 bias_r[NJ][NIP * 4];
    template <class F> __device__ __forceinline__ void tail_prefetch(int64_t ldc, const Tail &tl, F &&dst)
    {
        const int lane = threadIdx.x & 63;
        const int whalf = lane >> 5, rrow = lane >> 3, rch = lane & 7;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int nj = 0; nj < NJ; ++nj) {
                int64_t gcol0 = 0;
                char *const out = dst(mi, nj, gcol0);
                if (!out) continue;                        // uniform
                if (mi == 0 && tl.bias) {
#pragma unroll
                    for (int i = 0; i < NIP * 4; ++i)
                        bias_r[nj][i] = *(const_f4)(uintptr_t)(tl.bias + gcol0 + (i >> 2) * 32 + 8 * (i & 3) + 4 * whalf);
                }
                if constexpr (ESZ == 2) {
                    if (tl.aux) {
#pragma unroll
                        for (int it = 0; it < 4; ++it)
                            gate_r[mi * NJ + nj][it] = *reinterpret_cast<const uint4 *>(tl.aux + (out - tl.c0) + (int64_t)(it * 8 + rrow) * ldc + rch * 16);
                    }
                }
            }
    }
    template <bool TAIL, class F> __device__ __forceinline__ void store(char *reg, float scale, int64_t ldc, const Tail &tl, F &&dst)
    {
        const int lane = threadIdx.x & 63;
        const int wrow = lane & 31, whalf = lane >> 5;
        const int rrow = lane >> 3, rch = lane & 7;
        const bool gate_rows = TAIL && ESZ == 2 && tl.aux != nullptr;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int nj = 0; nj < NJ; ++nj) {
                int64_t gcol0 = 0;
                char *const out = dst(mi, nj, gcol0);
                if (!out) continue;                        // uniform
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
                            act4(tl.act, v);
                            if constexpr (ESZ == 4) {
                                if (tl.aux) {
                                    // fp32 outputs: the gate matrix has 16-bit elements, read in the accumulator's layout
                                    using E = typename In<T>::out16;
                                    typedef __attribute__((__vector_size__(4 * sizeof(E)))) E e4;
                                    const int c = 8 * q + 4 * whalf;             // column within the piece
                                    const int64_t elem = (out - tl.c0) / ESZ + wrow * (ldc / ESZ) + c;
                                    const e4 x = *reinterpret_cast<const e4 *>(tl.aux + elem * (int64_t)sizeof(E));
#pragma unroll
                                    for (int e = 0; e < 4; ++e) v[e] = static_cast<float>(x[e]) > 0.f ? v[e] : 0.f;
                                }
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
#pragma unroll
                for (int it = 0; it < 4; ++it) {
                    const int row = it * 8 + rrow;
                    uint4 v;
                    if constexpr (ESZ == 4) {
                        v = *reinterpret_cast<const uint4 *>(reg + row * 128 + ((rch ^ (row & 7)) << 4));
                    } else {
                        const uint4 x = *reinterpret_cast<const uint4 *>(reg + row * 128 + ((rch ^ ((row & 15) >> 1)) << 4));
                        v = (row & 1) ? make_uint4(x.z, x.w, x.x, x.y) : x;
                        if constexpr (TAIL) {
                            if (gate_rows) v = gate16<T>(v, gate_r[mi * NJ + nj][it]);
                        }
                    }
                    store_out(out + (int64_t)row * ldc + rch * 16, v);
                }
            }
    }
};

// s_waitcnt immediate that waits only for vector-memory operations (at most `vm` outstanding).
constexpr int waitcnt_vm_only(int vm) { return (vm & 15) | ((vm >> 4) << 14) | (7 << 4) | (15 << 8); }

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
template <int OP, class T, class OutT, int TM, int TN, int WM, int WN, bool TAIL>
__device__ __forceinline__ void gemm_persistent_body(const GemmParams &P, const int G, const int w)
{
    static_assert(OP == FWD || OP == DW, "output-sparse dX is not handled here");
    constexpr int NW = WM * WN;
    static_assert(NW == 4, "one computing and one loading wavefront per SIMD");
    constexpr int WTM = TM / WM, WTN = TN / WN, MI = WTM / 32, NI = WTN / 32;
    constexpr bool A_KMAJ = (OP == FWD), A_TR = !A_KMAJ, B_TR = true;
    constexpr int A_BYTES = TM * TK * 2, B_BYTES = TN * TK * 2, STAGE_BYTES = A_BYTES + B_BYTES;
    constexpr int STAGES = 3, AHEAD = 2;
    constexpr int ESZ = (int)sizeof(OutT);
    constexpr int STAGING = 32 * 128;           // per computing wavefront: 32 rows of 128 bytes

    extern __shared__ __attribute__((aligned(16))) char smem[];
    char *const staging = smem + STAGES * STAGE_BYTES;

    const MaskHeader *H = P.mv.hdr;
    if (H->magic != kMaskMagic || H->M != P.M || H->K != P.K || H->BM != P.BM || H->BK != P.BK) return;

    const int lane = threadIdx.x & 63;
    const int wave_all = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const bool loader = wave_all >= NW;
    const int wave = loader ? wave_all - NW : wave_all;
    const int wm = wave / WN, wn = wave % WN;
    const int total = P.total_tiles;
    const int BLK = (OP == FWD) ? P.BK : P.BM;            // extent of a mask block along the reduction
    const int sub_shift = (BLK == 128), sub_mask = (1 << sub_shift) - 1;
    const int64_t lda = P.K * 2, ldb = P.N * 2, ldc = P.N * (int64_t)ESZ;
    const int32_t *const order = (OP == FWD) ? P.mv.row_order : P.mv.col_order;
    const int32_t *const ptr = (OP == FWD) ? P.mv.row_ptr : P.mv.col_ptr;
    const int32_t *const lists = (OP == FWD) ? P.mv.col_idx : P.mv.row_idx;
    const int per_line = P.n_tiles * P.splits;            // tiles per block row / column

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
        using DmaB = DmaT<TN, NW>;
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
        n1 = level1(0); level2(n1); level3(n1);
        n2 = level1(1); level2(n2);
        n3 = level1(2);
        int k = -1;                      // round of the tile being issued
        int s = 0, nsteps = 0;           // next slice of that tile; its number of slices
        int e_cur = 0, e_nxt = 0;        // list entries of slice s and of the block after it
        const char *a_tile = nullptr, *b_tile = nullptr;
        bool ended = false;

        // issues the next slice of the stream into stage `st`; false when the stream has ended
        auto issue_next = [&](int st) __attribute__((always_inline)) -> bool {
            while (s == nsteps) {
                if (ended) return false;
                ++k;
                cur = n1;
                if (cur.t >= total) { ended = true; return false; }
                n1 = n2; level3(n1);
                n2 = n3; level2(n2);
                n3 = level1(k + 3);
                s = 0;
                nsteps = cur.len << sub_shift;
                e_cur = cur.e0; e_nxt = cur.e1;
                const int line = cur.t % per_line;
                const int nt = line / P.splits;
                if constexpr (OP == FWD) a_tile = P.A + (int64_t)cur.ord * P.BM * lda;
                else a_tile = P.A + (int64_t)cur.ord * P.BK * 2;
                b_tile = P.B + (int64_t)nt * TN * 2;
            }
            const int64_t off = (int64_t)e_cur * BLK + (int64_t)(s & sub_mask) * TK;
            const char *const sa[1] = {a_tile + off * (OP == FWD ? 2 : lda)};
            const char *const sb[1] = {b_tile + off * ldb};
            char *stp = stage_ptr(st);
#pragma unroll
            for (int j = 0; j < NDMA_A; ++j) da.issue(sa, lda, stp, j);
#pragma unroll
            for (int j = 0; j < NDMA_B; ++j) db.issue(sb, ldb, stp + A_BYTES, j);
            ++s;
            if ((s & sub_mask) == 0) {
                e_cur = e_nxt;
                e_nxt = entry(cur, (s >> sub_shift) + 1);
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
    int ord0 = uni(c_order(0));
    int len0 = uni(c_len(0, c_count(ord0)));
    int ord1 = uni(c_order(1));
    int ord2_v = c_order(2);
    __builtin_amdgcn_s_waitcnt(waitcnt_vm_only(0));
    int ord2 = uni(ord2_v);

    Compute<T, OutT, A_TR, B_TR, TM, TN, WM, WN> cw;
    cw.wm = wm; cw.wn = wn;
    int st0 = 0, st1 = 1, st2 = 2;       // stages of the stream's slices g, g+1, g+2
    bool started = false;
    const float scale = P.scale;
    const Tail tl = make_tail(P);
    char *const reg = staging + wave * STAGING;

    for (int k = 0;; ++k) {
        const int t = tile_of(k);
        if (t >= total) break;
        const int ord = ord0, nsteps = len0 << sub_shift;
        GEMM_TICKW(k * 4);
        // requests for the tiles after this one; consumed after this tile's slices
        const int cnt1_v = c_count(ord1);
        const int ord3_v = c_order(k + 3);

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
            cw.slice(stage_ptr(st0), stage_ptr(st1));
            const int t0 = st0; st0 = st1; st1 = st2; st2 = t0;
            if (s == 0) GEMM_TICKW(k * 4 + 1);
        }
        // the look-ups have had the whole tile to arrive and no store is in flight: this wait is free
        __builtin_amdgcn_s_waitcnt(waitcnt_vm_only(0));
        len0 = uni(c_len(k + 1, cnt1_v));
        ord0 = ord1; ord1 = ord2; ord2 = uni(ord3_v);
        if constexpr (TAIL) cw.tail_prefetch(ldc, tl, dst);
        GEMM_TICKW(k * 4 + 2);
        cw.template store<TAIL>(reg, scale, ldc, tl, dst);
        GEMM_TICKW(k * 4 + 3);
    }
}

template <int OP, class T, class OutT, int TM, int TN, int WM, int WN, bool TAIL>
__global__ __launch_bounds__(WM * WN * 128) void gemm_persistent_kernel(GemmParams P)
{
    gemm_persistent_body<OP, T, OutT, TM, TN, WM, WN, TAIL>(P, gridDim.x, blockIdx.x);
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
template <class T, class OutT, int TM, int TN, int WM, int WN, bool TAIL>
__device__ __forceinline__ void gemm_persistent_dx_body(const GemmParams &P, const int G, const int w)
{
    constexpr int NW = WM * WN;
    static_assert(NW == 4 && TM == 128, "one computing and one loading wavefront per SIMD, 128-row tiles");
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
    if (H->magic != kMaskMagic || H->M != P.M || H->K != P.K || H->BM != P.BM || H->BK != P.BK) return;

    const int lane = threadIdx.x & 63;
    const int wave_all = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const bool loader = wave_all >= NW;
    const int wave = loader ? wave_all - NW : wave_all;
    const int wm = wave / WN, wn = wave % WN;
    const int GB = TN / P.BK;                          // kept blocks per group: 1, 2 or 4
    const int cshift = (P.BK == 128), cmask = (1 << cshift) - 1;   // 64-column chunks per block
    const int nnz = H->nnz;
    const int ngroups = (nnz + GB - 1) / GB;
    const int nsteps = (int)(P.N / TK);
    const int64_t lda = P.N * 2, ldb = P.N * 2, ldc = P.K * (int64_t)ESZ;
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
        DmaK<TN, DXG, NW> db;
        da.init(lda, wave);
        db.init(ldb, wave);
        constexpr int NDMA_A = TM / (8 * NW), NDMA_B = TN / (8 * NW), NDMA = NDMA_A + NDMA_B;
        typedef const __attribute__((address_space(4))) int32_t *const_i32;   // see gemm_persistent_kernel
        const const_i32 k_rows = (const_i32)(uintptr_t)rows, k_cols = (const_i32)(uintptr_t)cols;
        auto load_group = [&](int k) __attribute__((always_inline)) -> Group {
            Group g;
            g.u = group_of(k);
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
                const int row = sel4(cur.r, a);
                int nb = 1;
                while (a + nb < cur.n && sel4(cur.r, a + nb) == row) ++nb;
                a_tile = P.A + (int64_t)row * P.BM * lda;
#pragma unroll
                for (int g = 0; g < DXG; ++g) {
                    const int bb = g >> cshift;         // a missing block repeats the last one
                    const int col = sel4(cur.c, a + (bb < nb ? bb : nb - 1));
                    bgrp[g] = P.B + ((int64_t)col * P.BK + (g & cmask) * 64) * ldb;
                }
                a += nb;
                s = 0;
            }
            const int64_t off = (int64_t)s * TK * 2;
            const char *const sa[1] = {a_tile + off};
            const char *sb[DXG];
#pragma unroll
            for (int g = 0; g < DXG; ++g) sb[g] = bgrp[g] + off;
            char *stp = stage_ptr(st);
#pragma unroll
            for (int j = 0; j < NDMA_A; ++j) da.issue(sa, lda, stp, j);
#pragma unroll
            for (int j = 0; j < NDMA_B; ++j) db.issue(sb, ldb, stp + A_BYTES, j);
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
    Compute<T, OutT, false, false, TM, TN, WM, WN> cw;
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
    int tick_no = 0;        // timing builds only: tiles done by this workgroup
    for (int k = 0; gu >= 0; ++k) {
        nxt = c_load_group(k + 1);                      // in flight during this group's tiles
        int ngr[4] = {0, 0, 0, 0}, ngc[4] = {0, 0, 0, 0};
        int a = 0;
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
            GEMM_TICKW(tick_no * 4);
            for (int s = 0; s < nsteps; ++s) {
                cw.slice(stage_ptr(st0), stage_ptr(st1));
                const int t0 = st0; st0 = st1; st1 = st2; st2 = t0;
            }
            GEMM_TICKW(tick_no * 4 + 1);
            // the look-ups have had the whole tile to arrive and no store is in flight: this wait is free
            __builtin_amdgcn_s_waitcnt(waitcnt_vm_only(0));
#pragma unroll
            for (int b = 0; b < 4; ++b) { ngr[b] = uni(nxt.r[b]); ngc[b] = uni(nxt.c[b]); }
            if constexpr (TAIL) cw.tail_prefetch(ldc, tl, dst);
            cw.template store<TAIL>(reg, scale, ldc, tl, dst);
            GEMM_TICKW(tick_no * 4 + 2);
            GEMM_TICKW(tick_no * 4 + 3);
            ++tick_no;
            a += nb;
        }
#pragma unroll
        for (int b = 0; b < 4; ++b) { gr[b] = ngr[b]; gc[b] = ngc[b]; }
        gn = nxt.n; gu = nxt.u;
    }
}

template <class T, class OutT, int TM, int TN, int WM, int WN, bool TAIL>
__global__ __launch_bounds__(WM * WN * 128) void gemm_persistent_dx_kernel(GemmParams P)
{
    gemm_persistent_dx_body<T, OutT, TM, TN, WM, WN, TAIL>(P, gridDim.x, blockIdx.x);
}

// Both gradients of the layer in one launch (eq. 2 and eq. 3 share dY and the mask and do not
// depend on each other): workgroups [0, g_dx) are the persistent dX kernel, the rest the persistent
// dW kernel.  One workgroup fits a CU, so the dW workgroups start one by one on the CUs that the dX
// workgroups leave: no launch boundary (about 5 us of idle chip between dependent launches) and no
// idle tail between the two.  The dX workgroups come first, so dX workgroup w is workgroup w of
// the launch and runs on XCD w % 8, which its schedule assumes; the dW schedule assumes nothing.
template <class T, class OutDX, class OutDW, int TN_DX>
__global__ __launch_bounds__(512) void bwd_fused_kernel(GemmParams Pdx, GemmParams Pdw, int g_dx)
{
    if ((int)blockIdx.x < g_dx)
        gemm_persistent_dx_body<T, OutDX, 128, TN_DX, 2, 2, false>(Pdx, g_dx, (int)blockIdx.x);
    else
        gemm_persistent_body<DW, T, OutDW, 128, 256, 1, 4, false>(Pdw, (int)gridDim.x - g_dx, (int)blockIdx.x - g_dx);
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
        gemm_persistent_body<DW, T, OutDW, 128, 256, 1, 4, false>(Pdw, (int)gridDim.x - n_dx, (int)blockIdx.x - n_dx);
}

// WM x WN: wavefront grid of the kernel without ragged edges; WMR x WNR (4 wavefronts): with.
int cu_count();

// Kernels with the element-wise tail are separate instantiations, so that eq. (1)-(3) proper run
// exactly the code they would without it.
inline bool has_tail(const GemmParams &P) { return P.bias != nullptr || P.aux != nullptr || P.act != 0; }

template <bool TAIL, int OP, class T, class OutT, int TM, int TN, int WM, int WN, int WMR, int WNR>
int launch_t(const GemmParams &P, int grid, bool ragged, hipStream_t stream, bool persistent_ok);

template <int OP, class T, class OutT, int TM, int TN, int WM, int WN, int WMR = WM, int WNR = WN>
int launch(const GemmParams &P, int grid, bool ragged, hipStream_t stream, bool persistent_ok = true)
{
    if constexpr (OP != DW) {
        if (has_tail(P)) return launch_t<true, OP, T, OutT, TM, TN, WM, WN, WMR, WNR>(P, grid, ragged, stream, persistent_ok);
    }
    return launch_t<false, OP, T, OutT, TM, TN, WM, WN, WMR, WNR>(P, grid, ragged, stream, persistent_ok);
}

template <bool TAIL, int OP, class T, class OutT, int TM, int TN, int WM, int WN, int WMR, int WNR>
int launch_t(const GemmParams &P, int grid, bool ragged, hipStream_t stream, bool persistent_ok)
{
    constexpr int LDS_BYTES = stages_for(TM, TN) * (TM + TN) * TK * 2;
    constexpr bool SPEC = TM >= 128;     // loader wavefronts for the one-workgroup-per-CU tiles
    auto k_full = gemm_kernel<OP, T, OutT, TM, TN, WM, WN, false, SPEC, TAIL>;
    auto k_ragged = gemm_kernel<OP, T, OutT, TM, TN, WMR, WNR, true, false, TAIL>;
    static bool attr_set = false;   // per instantiation
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_full),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_ragged),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
        if (e != hipSuccess) return hip_status(e);
        attr_set = true;
    }
    if (grid <= 0) return SDROP_OK;
    if constexpr (OP != DX) {
        if (!ragged && persistent_ok) {
            // persistent form: three operand stages plus 4 KiB of output staging per computing wavefront
            constexpr int P_LDS = 3 * (TM + TN) * TK * 2 + WM * WN * 4096;
            auto k_pers = gemm_persistent_kernel<OP, T, OutT, TM, TN, WM, WN, TAIL>;
            static int pers_ok = -1;    // per instantiation: does the device grant that much LDS?
            if (pers_ok < 0) {
                hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_pers),
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, P_LDS);
                pers_ok = (e == hipSuccess);
                if (!pers_ok) (void)hipGetLastError();
            }
#ifdef SDROP_GEMM_TIMING
            const bool pers_off = getenv("SDROP_NO_PERSIST") != nullptr;
#else
            const bool pers_off = false;
#endif
            if (pers_ok && !pers_off) {
                GemmParams Q = P;
                Q.total_tiles = grid;
                const int ncu = cu_count();
                hipLaunchKernelGGL(k_pers, dim3(grid < ncu ? grid : ncu), dim3(WM * WN * 128), P_LDS, stream, Q);
                return hip_status(hipGetLastError());
            }
        }
    }
    if (ragged) hipLaunchKernelGGL(k_ragged, dim3(grid), dim3(WMR * WNR * 64), LDS_BYTES, stream, P);
    else hipLaunchKernelGGL(k_full, dim3(grid), dim3(WM * WN * 64 * (SPEC ? 2 : 1)), LDS_BYTES, stream, P);
    return hip_status(hipGetLastError());
}

// Persistent dX: one workgroup per CU (fewer when there are fewer block positions than CUs).
template <class T, class OutT, int TN, bool TAIL>
int launch_dx_persistent_t(const GemmParams &P, hipStream_t stream);

template <class T, class OutT, int TN>
int launch_dx_persistent(const GemmParams &P, hipStream_t stream)
{
    if (has_tail(P)) return launch_dx_persistent_t<T, OutT, TN, true>(P, stream);
    return launch_dx_persistent_t<T, OutT, TN, false>(P, stream);
}

template <class T, class OutT, int TN, bool TAIL>
int launch_dx_persistent_t(const GemmParams &P, hipStream_t stream)
{
    constexpr int P_LDS = 3 * (128 + TN) * TK * 2 + 4 * 4096;
    auto k = gemm_persistent_dx_kernel<T, OutT, 128, TN, 2, 2, TAIL>;
    static int ok = -1;     // per instantiation: does the device grant that much LDS?
    if (ok < 0) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, P_LDS);
        ok = (e == hipSuccess);
        if (!ok) (void)hipGetLastError();
    }
#ifdef SDROP_GEMM_TIMING
    if (getenv("SDROP_NO_PERSIST")) return -1;
#endif
    if (!ok) return -1;
    const int64_t positions = (int64_t)P.MB * P.KB;
    const int ncu = cu_count();
    hipLaunchKernelGGL(k, dim3((unsigned)(positions < ncu ? positions : ncu)), dim3(512), P_LDS, stream, P);
    return hip_status(hipGetLastError());
}

// out[e] = scale * sum_c part[c][e], rounded once (the second pass of a split DW)
template <class OutT>
__global__ __launch_bounds__(256) void reduce_parts_kernel(const float *part, OutT *out, int64_t n, int splits, float scale)
{
    const int64_t e = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (e >= n) return;
    float4 acc = *reinterpret_cast<const float4 *>(part + e);
    for (int c = 1; c < splits; ++c) {
        const float4 v = *reinterpret_cast<const float4 *>(part + (int64_t)c * n + e);
        acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
    out[e] = static_cast<OutT>(acc.x * scale); out[e + 1] = static_cast<OutT>(acc.y * scale);
    out[e + 2] = static_cast<OutT>(acc.z * scale); out[e + 3] = static_cast<OutT>(acc.w * scale);
}

// Parts the reduction of DW is cut into.  DW has only KB * ceil(N/256) output tiles; when
// that is fewer than the chip has CUs, each block column's kept-row list is cut into parts
// computed by different workgroups into fp32 planes that a second pass sums in a fixed
// order (deterministic, unlike atomics).  A pure function of the shape (not of p), so that
// the workspace size can be asked for without the mask.
//
// The number of parts minimises a small cost model, in units of one reduction slice: the launch
// runs ceil(tiles * parts / CUs) rounds of part-tiles, each costing its share of the list (taken
// at full length, M/64 slices) plus a fixed 10 for set-up and epilogue, and the summing pass reads
// parts * K * N floats (about 0.86e6 floats per slice time).  Measured against "always two rounds":
// 2048^3 with 128-blocks 37 -> 28 us, the 8192 x 1024 x 1024 layer 26 -> 23 us.  Only powers of
// two are tried (3 or 5 parts measured up to 1.5x slower than 2 or 4 on the same shapes).
int dw_splits(int64_t M, int64_t N, int BM, int BK, int64_t K)
{
    const int64_t tiles = (K / BK) * ((N + 255) / 256);
    const int64_t ncu = cu_count();
    if (tiles >= ncu) return 1;
#ifdef SDROP_GEMM_TIMING
    if (getenv("SDROP_DW_SPLITS")) return atoi(getenv("SDROP_DW_SPLITS"));
#endif
    int64_t max_parts = (M / BM) / 4;                      // keep at least ~4 row blocks per part
    if (max_parts > 16) max_parts = 16;
    const double len = (double)(M / 64), sum_cost = (double)K * (double)N / 0.86e6;
    int best = 1;
    double best_cost = 0.0;
    for (int64_t parts = 1; parts <= max_parts || parts == 1; parts *= 2) {   // powers of two: odd counts measured far worse
        const double rounds = (double)((tiles * parts + ncu - 1) / ncu);
        const double cost = rounds * (len / parts + 10.0) + (parts > 1 ? parts * sum_cost : 0.0);
        if (parts == 1 || cost < best_cost) { best = (int)parts; best_cost = cost; }
    }
    return best;
}

int cu_count()
{
    static int n = 0;
    if (n == 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
            n = v;
        else
            n = 256;
    }
    return n;
}

// groups of kept blocks per CU from which dX tiles of several blocks use the persistent kernel
int g_dx_persistent_groups_per_cu = 8;

// dX: width of the tiles, and whether the persistent kernel computes them.
// Every kept block costs the same, so the launch runs in ceil(tiles / CUs) rounds of
// equal tiles.  A 256-wide tile moves a quarter less data per flop than two 128-wide
// ones (a 128-wide tile was measured at 0.6 of the time of a wide one); take whichever shape is expected
// to finish first for the expected number of kept blocks, (1-p) MB KB.
// The persistent kernel deals out groups of TN/BK list entries and cuts a group where the block
// row changes inside it; with few groups per workgroup one such extra tile is a whole round, so it
// is used for single-block tiles (no cuts) and where a workgroup gets at least 8 groups.  Measured,
// persistent against per-tile: 1.8 groups per CU (4096^3, a tenth dropped) 134 against 103 us;
// 3 (16384 x 3072 x 768, 64-wide blocks, half dropped) 61 against 56; 5.6 (8192 x 8192 x 2048, 0.3
// dropped) 215 against 190; 9.6 (65536 x 4096 x 1024, 0.7 dropped) 235 against 270; 22 (the same,
// 0.3 dropped) 410 against 417.
int g_dx_tile_width = 0;    // 0: chosen per call; 128 or 256: forced (benchmarks and tests)
struct DxPlan { int TN; bool persistent; };
DxPlan dx_plan(const GemmParams &P)
{
    const double kept = (1.0 - P.p) * (double)P.MB * (double)P.KB;
    const int ncu = cu_count();
    auto rounds = [&](int tn) {
        const int g = tn / P.BK;
        // groups of g kept blocks per block row; a random row leaves (g-1)/2g of a group unfilled
        const double tiles = kept / g + (P.p > 0.0 ? P.MB * (g - 1) / (2.0 * g) : 0.0);
        return (double)((int64_t)((tiles + ncu - 1) / ncu));
    };
    DxPlan plan;
    plan.TN = (rounds(128) * 0.6 < rounds(256)) ? 128 : 256;
    if (g_dx_tile_width == 128 || g_dx_tile_width == 256) plan.TN = g_dx_tile_width;
    const int G_ = plan.TN / P.BK;
    plan.persistent = P.BM == 128 && P.N % TK == 0 && (G_ == 1 || kept / G_ >= (double)g_dx_persistent_groups_per_cu * ncu);
    return plan;
}

// Tile shapes: the tile edge that lies along the mask must equal the mask's block
// (Section 3.2); the N edge is free (Section 3.3) and is 256 wide.  DX gathers
// 256/BK kept blocks of one block row into a 256-wide tile.
template <int OP, class T, class OutT>
int dispatch_tile(GemmParams &P, hipStream_t stream)
{
    if constexpr (OP == FWD) {
        P.n_tiles = (int)((P.N + 255) / 256);
        const int grid = P.MB * P.n_tiles;
        const bool ragged = P.N % 256 != 0;
        if (P.BM == 128) return launch<FWD, T, OutT, 128, 256, 1, 4>(P, grid, ragged, stream);
        return launch<FWD, T, OutT, 64, 256, 1, 4>(P, grid, ragged, stream);
    } else if constexpr (OP == DW) {
        P.n_tiles = (int)((P.N + 255) / 256);
        const int grid = P.KB * P.n_tiles * P.splits;
        const bool ragged = P.N % 256 != 0;
        if (P.BK == 128) return launch<DW, T, OutT, 128, 256, 1, 4>(P, grid, ragged, stream);
        // 64-row tiles: the persistent kernel runs one workgroup per CU, whose epilogue nothing
        // overlaps; with short kept lists (a few slices per tile) three co-resident workgroups of the
        // per-tile kernel do better (8192 x 1024 x 1024, 64 x 64 blocks, half kept, 16 parts:
        // 26.5 against 29.5 us; 16384 x 3072 x 768, a tenth dropped, 4 parts: 121 against 101 us)
        const double slices = (1.0 - P.p) * P.MB / P.splits * (P.BM / 64);
        return launch<DW, T, OutT, 64, 256, 1, 4>(P, grid, ragged, stream, slices >= 16.0);
    } else {
        const DxPlan plan = dx_plan(P);
        const int TNsel = plan.TN, G_ = TNsel / P.BK;
        P.n_tiles = (P.KB + G_ - 1) / G_;
        // one kept block per tile: a workgroup per block position, rounded up to whole sets of 8 XCDs
        const int grid = G_ == 1 ? (P.MB * P.KB + 7) / 8 * 8 : P.MB * P.n_tiles;
        const bool ragged = P.N % TK != 0;
        if (plan.persistent) {
            const int rc = TNsel == 256 ? launch_dx_persistent<T, OutT, 256>(P, stream) : launch_dx_persistent<T, OutT, 128>(P, stream);
            if (rc != -1) return rc;      // -1: the device does not grant the LDS; use the per-tile kernels
        }
        if (TNsel == 256) {
            if (P.BM == 128) return launch<DX, T, OutT, 128, 256, 2, 2>(P, grid, ragged, stream);
            return launch<DX, T, OutT, 64, 256, 1, 4>(P, grid, ragged, stream);
        }
        if (P.BM == 128) return launch<DX, T, OutT, 128, 128, 2, 2>(P, grid, ragged, stream);
        return launch<DX, T, OutT, 64, 128, 1, 4>(P, grid, ragged, stream);
    }
}

// 32-bit tile numbers must do (no operand that fits the device's memory comes near this)
bool tile_count_ok(int64_t N, const sdrop_mask_layout_t &L)
{
    const int64_t n_tiles = (N + 255) / 256, lines = L.MB > L.KB ? L.MB : L.KB;
    return lines * n_tiles * 16 <= INT32_MAX;
}

GemmParams base_params(const void *a, const void *b, const void *mask, void *out,
                       int64_t M, int64_t K, int64_t N, int BM, int BK, double p, const sdrop_mask_layout_t &L)
{
    GemmParams P;
    P.A = static_cast<const char *>(a);
    P.B = static_cast<const char *>(b);
    P.C = static_cast<char *>(out);
    P.mv = make_view(mask, L);
    P.M = M; P.K = K; P.N = N; P.BM = BM; P.BK = BK;
    P.MB = (int32_t)L.MB; P.KB = (int32_t)L.KB;
    P.n_tiles = 0;
    P.splits = 1;
    P.total_tiles = 0;
    P.scale = (p < 1.0) ? (float)(1.0 / (1.0 - p)) : 0.0f;
    P.bias = nullptr; P.aux = nullptr; P.act = SDROP_ACT_NONE;
    P.p = p;
    return P;
}

// sums the fp32 planes of a split DW into the output (second pass)
int launch_reduce(const void *ws, void *out, int64_t n, int splits, float scale, int dtype, int out_dtype, hipStream_t st)
{
    const unsigned grid = (unsigned)((n / 4 + 255) / 256);
    const float *part = static_cast<const float *>(ws);
    if (out_dtype == SDROP_F32)
        hipLaunchKernelGGL(reduce_parts_kernel<float>, dim3(grid), dim3(256), 0, st, part, static_cast<float *>(out), n, splits, scale);
    else if (dtype == SDROP_F16)
        hipLaunchKernelGGL(reduce_parts_kernel<_Float16>, dim3(grid), dim3(256), 0, st, part, static_cast<_Float16 *>(out), n, splits, scale);
    else
        hipLaunchKernelGGL(reduce_parts_kernel<__bf16>, dim3(grid), dim3(256), 0, st, part, static_cast<__bf16 *>(out), n, splits, scale);
    return hip_status(hipGetLastError());
}

template <int OP>
int run(const void *a, const void *b, const void *mask, void *out,
        int64_t M, int64_t K, int64_t N, int BM, int BK, double p,
        int dtype, int out_dtype, void *ws, size_t ws_bytes, void *stream,
        const sdrop_epilogue_t *epi = nullptr)
{
    const int rc = check_gemm_args(a, b, mask, out, M, K, N, BM, BK, p, dtype, out_dtype);
    if (rc != SDROP_OK) return rc;
    if (epi) {
        if (epi->scale_mode != SDROP_SCALE_DROPOUT && epi->scale_mode != SDROP_SCALE_ONE) return SDROP_EINVAL;
        if (epi->act != SDROP_ACT_NONE && epi->act != SDROP_ACT_RELU && epi->act != SDROP_ACT_GELU_TANH) return SDROP_EINVAL;
        // the gradient of the weights takes a scale only
        if (OP == DW && (epi->act != SDROP_ACT_NONE || epi->bias || epi->relu_mask)) return SDROP_EINVAL;
        if ((reinterpret_cast<uintptr_t>(epi->bias) | reinterpret_cast<uintptr_t>(epi->relu_mask)) % 16) return SDROP_EALIGN;
    }
    const size_t ws_need = sdrop_workspace_bytes(OP, M, K, N, BM, BK, dtype, out_dtype);
    if (ws_bytes < ws_need || (ws_need && (!ws || reinterpret_cast<uintptr_t>(ws) % 16))) return SDROP_EWORKSPACE;
    sdrop_mask_layout_t L;
    sdrop_mask_layout(M, K, BM, BK, &L);
    if (!tile_count_ok(N, L)) return SDROP_ESHAPE;
    GemmParams P = base_params(a, b, mask, out, M, K, N, BM, BK, p, L);
    if (epi) {
        if (epi->scale_mode == SDROP_SCALE_ONE) P.scale = 1.0f;
        P.bias = epi->bias;
        P.aux = static_cast<const char *>(epi->relu_mask);
        P.act = epi->act;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    if constexpr (OP == DW) {
        P.splits = dw_splits(M, N, BM, BK, K);
        if (P.splits > 1) {
            // first pass: unscaled fp32 partial planes into the workspace; second pass: sum, scale, round
            const float scale = P.scale;
            P.C = static_cast<char *>(ws);
            P.scale = 1.0f;
            const int rc1 = (dtype == SDROP_F16) ? dispatch_tile<OP, F16, float>(P, st) : dispatch_tile<OP, BF16, float>(P, st);
            if (rc1 != SDROP_OK) return rc1;
            return launch_reduce(ws, out, K * N, P.splits, scale, dtype, out_dtype, st);
        }
    }
    if (dtype == SDROP_F16) {
        if (out_dtype == SDROP_F32) return dispatch_tile<OP, F16, float>(P, st);
        return dispatch_tile<OP, F16, _Float16>(P, st);
    }
    if (out_dtype == SDROP_F32) return dispatch_tile<OP, BF16, float>(P, st);
    return dispatch_tile<OP, BF16, __bf16>(P, st);
}

// both gradients in one launch where bwd_fused_kernel or bwd_fused_tile_kernel applies (128 x 128
// blocks, N a multiple of 256); anything else is the two calls in turn
int g_bwd_fused = 1;

template <class T, class OutDX, class OutDW, int TN_DX>
int launch_bwd_fused(const GemmParams &Pdx, const GemmParams &Pdw, hipStream_t stream)
{
    constexpr int LDS_DX = 3 * (128 + TN_DX) * TK * 2 + 4 * 4096, LDS_DW = 3 * (128 + 256) * TK * 2 + 4 * 4096;
    constexpr int P_LDS = LDS_DX > LDS_DW ? LDS_DX : LDS_DW;
    auto k = bwd_fused_kernel<T, OutDX, OutDW, TN_DX>;
    static int ok = -1;     // per instantiation: does the device grant that much LDS?
    if (ok < 0) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, P_LDS);
        ok = (e == hipSuccess);
        if (!ok) (void)hipGetLastError();
    }
    if (!ok) return -1;
    const int ncu = cu_count();
    const int64_t positions = (int64_t)Pdx.MB * Pdx.KB;
    const int g_dx = (int)(positions < ncu ? positions : ncu);
    const int g_dw = Pdw.total_tiles < ncu ? Pdw.total_tiles : ncu;
    hipLaunchKernelGGL(k, dim3((unsigned)(g_dx + g_dw)), dim3(512), P_LDS, stream, Pdx, Pdw, g_dx);
    return hip_status(hipGetLastError());
}

template <class T, class OutDX, class OutDW>
int launch_bwd_fused_tile(const GemmParams &Pdx, const GemmParams &Pdw, int n_dx, hipStream_t stream)
{
    constexpr int LDS_DX = 3 * (128 + 256) * TK * 2, LDS_DW = 3 * (128 + 256) * TK * 2 + 4 * 4096;
    constexpr int P_LDS = LDS_DX > LDS_DW ? LDS_DX : LDS_DW;
    auto k = bwd_fused_tile_kernel<T, OutDX, OutDW>;
    static int ok = -1;     // per instantiation: does the device grant that much LDS?
    if (ok < 0) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, P_LDS);
        ok = (e == hipSuccess);
        if (!ok) (void)hipGetLastError();
    }
    if (!ok) return -1;
    const int ncu = cu_count();
    const int g_dw = Pdw.total_tiles < ncu ? Pdw.total_tiles : ncu;
    hipLaunchKernelGGL(k, dim3((unsigned)(n_dx + g_dw)), dim3(512), P_LDS, stream, Pdx, Pdw, n_dx);
    return hip_status(hipGetLastError());
}

template <class T, class OutDX, class OutDW>
int launch_bwd_fused_tn(int TN, const GemmParams &Pdx, const GemmParams &Pdw, hipStream_t stream)
{
    if (TN == 256) return launch_bwd_fused<T, OutDX, OutDW, 256>(Pdx, Pdw, stream);
    return launch_bwd_fused<T, OutDX, OutDW, 128>(Pdx, Pdw, stream);
}

int run_bwd(const void *dy, const void *w, const void *x, const void *mask, void *dx, void *dw,
            int64_t M, int64_t K, int64_t N, int BM, int BK, double p,
            int dtype, int out_dtype, void *ws, size_t ws_bytes, void *stream)
{
    // every argument check of both calls before anything is enqueued
    int rc = check_gemm_args(dy, w, mask, dx, M, K, N, BM, BK, p, dtype, out_dtype);
    if (rc == SDROP_OK) rc = check_gemm_args(x, dy, mask, dw, M, K, N, BM, BK, p, dtype, out_dtype);
    if (rc != SDROP_OK) return rc;
    const size_t ws_need = sdrop_workspace_bytes(SDROP_OP_BWD_DW, M, K, N, BM, BK, dtype, out_dtype);
    if (ws_bytes < ws_need || (ws_need && (!ws || reinterpret_cast<uintptr_t>(ws) % 16))) return SDROP_EWORKSPACE;
    sdrop_mask_layout_t L;
    sdrop_mask_layout(M, K, BM, BK, &L);
    if (!tile_count_ok(N, L)) return SDROP_ESHAPE;
    hipStream_t st = static_cast<hipStream_t>(stream);

    GemmParams Pdx = base_params(dy, w, mask, dx, M, K, N, BM, BK, p, L);
    const DxPlan plan = dx_plan(Pdx);
    // dX as one workgroup per tile of two kept blocks (never with one block per tile: that form is persistent)
    const bool tile_form = !plan.persistent && plan.TN == 256;
    if (g_bwd_fused && BM == 128 && BK == 128 && N % 256 == 0 && (plan.persistent || tile_form)) {
        const int G_ = plan.TN / BK;
        Pdx.n_tiles = (Pdx.KB + G_ - 1) / G_;
        const int n_dx = Pdx.MB * Pdx.n_tiles;           // the per-tile launch's grid: (group of the row, block row)
        GemmParams Pdw = base_params(x, dy, mask, dw, M, K, N, BM, BK, p, L);
        Pdw.splits = dw_splits(M, N, BM, BK, K);
        Pdw.n_tiles = (int)(N / 256);
        Pdw.total_tiles = Pdw.KB * Pdw.n_tiles * Pdw.splits;
        const float scale = Pdw.scale;
        const bool split = Pdw.splits > 1;
        if (split) { Pdw.C = static_cast<char *>(ws); Pdw.scale = 1.0f; }
        const bool f16 = dtype == SDROP_F16, o32 = out_dtype == SDROP_F32;
        int rf;
        if (tile_form) {
            if (f16) {
                if (o32) rf = launch_bwd_fused_tile<F16, float, float>(Pdx, Pdw, n_dx, st);
                else if (split) rf = launch_bwd_fused_tile<F16, _Float16, float>(Pdx, Pdw, n_dx, st);
                else rf = launch_bwd_fused_tile<F16, _Float16, _Float16>(Pdx, Pdw, n_dx, st);
            } else {
                if (o32) rf = launch_bwd_fused_tile<BF16, float, float>(Pdx, Pdw, n_dx, st);
                else if (split) rf = launch_bwd_fused_tile<BF16, __bf16, float>(Pdx, Pdw, n_dx, st);
                else rf = launch_bwd_fused_tile<BF16, __bf16, __bf16>(Pdx, Pdw, n_dx, st);
            }
        } else if (f16) {
            if (o32) rf = launch_bwd_fused_tn<F16, float, float>(plan.TN, Pdx, Pdw, st);
            else if (split) rf = launch_bwd_fused_tn<F16, _Float16, float>(plan.TN, Pdx, Pdw, st);
            else rf = launch_bwd_fused_tn<F16, _Float16, _Float16>(plan.TN, Pdx, Pdw, st);
        } else {
            if (o32) rf = launch_bwd_fused_tn<BF16, float, float>(plan.TN, Pdx, Pdw, st);
            else if (split) rf = launch_bwd_fused_tn<BF16, __bf16, float>(plan.TN, Pdx, Pdw, st);
            else rf = launch_bwd_fused_tn<BF16, __bf16, __bf16>(plan.TN, Pdx, Pdw, st);
        }
        if (rf != -1) {     // -1: the device does not grant the LDS; fall through to the two calls
            if (rf != SDROP_OK || !split) return rf;
            return launch_reduce(ws, dw, K * N, Pdw.splits, scale, dtype, out_dtype, st);
        }
    }
    rc = run<DX>(dy, w, mask, dx, M, K, N, BM, BK, p, dtype, out_dtype, nullptr, 0, stream);
    if (rc != SDROP_OK) return rc;
    return run<DW>(x, dy, mask, dw, M, K, N, BM, BK, p, dtype, out_dtype, ws, ws_bytes, stream);
}

}  // namespace

int check_gemm_args(const void *a, const void *b, const void *mask, void *out,
                    int64_t M, int64_t K, int64_t N, int BM, int BK, double p,
                    int dtype, int out_dtype)
{
    if (!a || !b || !mask || !out) return SDROP_EINVAL;
    if (!(p >= 0.0 && p <= 1.0)) return SDROP_EINVAL;
    if (M <= 0 || K <= 0 || N <= 0 || !block_size_ok(BM) || !block_size_ok(BK)) return SDROP_ESHAPE;
    if (M % BM || K % BK || N % 8) return SDROP_ESHAPE;
    sdrop_mask_layout_t L;
    const int rc = sdrop_mask_layout(M, K, BM, BK, &L);
    if (rc != SDROP_OK) return rc;
    // lane offsets inside a slice are 32-bit: up to 64 rows of K or N 16-bit elements
    if (M > (int64_t(1) << 30) || K > (int64_t(1) << 24) || N > (int64_t(1) << 24)) return SDROP_ESHAPE;
    if (dtype != SDROP_F16 && dtype != SDROP_BF16) return SDROP_EDTYPE;
    if (out_dtype != dtype && out_dtype != SDROP_F32) return SDROP_EDTYPE;
    const uintptr_t bits = reinterpret_cast<uintptr_t>(a) | reinterpret_cast<uintptr_t>(b) |
                           reinterpret_cast<uintptr_t>(mask) | reinterpret_cast<uintptr_t>(out);
    if (bits % 16) return SDROP_EALIGN;
    return SDROP_OK;
}

}  // namespace sdrop

#ifdef SDROP_GEMM_TIMING
extern "C" int sdrop_debug_ticks(long long *host, int n)
{
    return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(sdrop::g_ticks), sizeof(long long) * n);
}
#endif

extern "C" {

int sdrop_set_tuning(int knob, int value)
{
    if (knob == SDROP_TUNE_DX_TILE_WIDTH && (value == 0 || value == 128 || value == 256)) {
        sdrop::g_dx_tile_width = value;
        return SDROP_OK;
    }
    if (knob == SDROP_TUNE_BWD_FUSED && (value == 0 || value == 1)) {
        sdrop::g_bwd_fused = value;
        return SDROP_OK;
    }
    if (knob == SDROP_TUNE_DX_PERSISTENT_GROUPS_PER_CU && value >= 0) {
        sdrop::g_dx_persistent_groups_per_cu = value;
        return SDROP_OK;
    }
    return SDROP_EINVAL;
}

size_t sdrop_workspace_bytes(int op, int64_t M, int64_t K, int64_t N, int BM, int BK,
                             int dtype, int out_dtype)
{
    (void)dtype; (void)out_dtype;
    if (op != SDROP_OP_BWD_DW) return 0;
    if (M <= 0 || K <= 0 || N <= 0 || !sdrop::block_size_ok(BM) || !sdrop::block_size_ok(BK) || M % BM || K % BK) return 0;
    const int splits = sdrop::dw_splits(M, N, BM, BK, K);
    return splits > 1 ? (size_t)splits * (size_t)K * (size_t)N * sizeof(float) : 0;
}

int sdrop_fwd(const void *X, const void *W, const void *mask, void *Y,
              int64_t M, int64_t K, int64_t N, int BM, int BK, double p,
              int dtype, int out_dtype, void *ws, size_t ws_bytes, void *stream)
{
    return sdrop::run<sdrop::FWD>(X, W, mask, Y, M, K, N, BM, BK, p, dtype, out_dtype, ws, ws_bytes, stream);
}

int sdrop_bwd_dx(const void *dY, const void *W, const void *mask, void *dX,
                 int64_t M, int64_t K, int64_t N, int BM, int BK, double p,
                 int dtype, int out_dtype, void *ws, size_t ws_bytes, void *stream)
{
    return sdrop::run<sdrop::DX>(dY, W, mask, dX, M, K, N, BM, BK, p, dtype, out_dtype, ws, ws_bytes, stream);
}

int sdrop_bwd_dw(const void *X, const void *dY, const void *mask, void *dW,
                 int64_t M, int64_t K, int64_t N, int BM, int BK, double p,
                 int dtype, int out_dtype, void *ws, size_t ws_bytes, void *stream)
{
    return sdrop::run<sdrop::DW>(X, dY, mask, dW, M, K, N, BM, BK, p, dtype, out_dtype, ws, ws_bytes, stream);
}

int sdrop_bwd(const void *dY, const void *W, const void *X, const void *mask, void *dX, void *dW,
              int64_t M, int64_t K, int64_t N, int BM, int BK, double p,
              int dtype, int out_dtype, void *ws, size_t ws_bytes, void *stream)
{
    return sdrop::run_bwd(dY, W, X, mask, dX, dW, M, K, N, BM, BK, p, dtype, out_dtype, ws, ws_bytes, stream);
}

int sdrop_fwd_ex(const void *X, const void *W, const void *mask, void *Y,
                 int64_t M, int64_t K, int64_t N, int BM, int BK, double p,
                 int dtype, int out_dtype, void *ws, size_t ws_bytes, void *stream,
                 const sdrop_epilogue_t *epi)
{
    return sdrop::run<sdrop::FWD>(X, W, mask, Y, M, K, N, BM, BK, p, dtype, out_dtype, ws, ws_bytes, stream, epi);
}

int sdrop_bwd_dx_ex(const void *dY, const void *W, const void *mask, void *dX,
                    int64_t M, int64_t K, int64_t N, int BM, int BK, double p,
                    int dtype, int out_dtype, void *ws, size_t ws_bytes, void *stream,
                    const sdrop_epilogue_t *epi)
{
    return sdrop::run<sdrop::DX>(dY, W, mask, dX, M, K, N, BM, BK, p, dtype, out_dtype, ws, ws_bytes, stream, epi);
}

int sdrop_bwd_dw_ex(const void *X, const void *dY, const void *mask, void *dW,
                    int64_t M, int64_t K, int64_t N, int BM, int BK, double p,
                    int dtype, int out_dtype, void *ws, size_t ws_bytes, void *stream,
                    const sdrop_epilogue_t *epi)
{
    return sdrop::run<sdrop::DW>(X, dY, mask, dW, M, K, N, BM, BK, p, dtype, out_dtype, ws, ws_bytes, stream, epi);
}

int sdrop_producer(const void *H, const void *W0, const float *bias, const void *mask, void *X,
                   int64_t M, int64_t N0, int64_t K, int BM, int BK, double p, int act,
                   int dtype, int out_dtype, void *stream)
{
    sdrop_epilogue_t epi;
    epi.scale_mode = SDROP_SCALE_ONE;
    epi.act = act;
    epi.bias = bias;
    epi.relu_mask = nullptr;
    return sdrop::run<sdrop::DX>(H, W0, mask, X, M, K, N0, BM, BK, p, dtype, out_dtype, nullptr, 0, stream, &epi);
}

}  // extern "C"
