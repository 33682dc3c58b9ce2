// Device-side building blocks of libsdrop's GEMM kernels (included by the GEMM translation units only): operand types and the MFMA
// wrapper, kernel parameters, the non-temporal output store, the element-wise tail, the LDS swizzle, the direct-load
// engines (HBM -> LDS), the register path for ragged edges, operand reads from LDS, scheduling helpers.
#ifndef SDROP_GEMM_DEVICE_COMMON_H
#define SDROP_GEMM_DEVICE_COMMON_H
#include "sdrop_internal.h"
#include <limits.h>
#include <stdlib.h>
#include <type_traits>
#include <utility>

namespace sdrop {

// What the translation units of the GEMMs share by name (everything else here is per translation unit).
struct F16 {};      // operand type tags
struct BF16 {};
enum Op { FWD = 0, DX = 1, DW = 2 };

struct GemmParams {
    const char *A;      // FWD: X   DX: dY  DW: X
    const char *B;      // FWD: W   DX: W   DW: dY
    char *C;            // FWD: Y   DX: dX  DW: dW
    MaskView mv;
    int64_t M, K, N;
    int64_t lda, ldb, ldc;   // bytes between consecutive rows of A, B and C (contiguous: columns * element size)
    int32_t BM, BK, MB, KB;
    int32_t n_tiles;    // FWD/DW: TN-wide tiles along N.  DX: groups of kept blocks per block row
    int32_t splits;     // DW: parts the kept-row list of a block column is cut into (1 = no split)
    int32_t total_tiles; // persistent kernels: tiles of the whole launch
    float scale;
    // optional element-wise tail of FWD and DX (see Tail below); all null / 0 for eq. (1)-(3) proper
    const float *bias;
    const char *aux;
    int32_t act;
    int32_t gate_mode;  // how aux gates the output (SDROP_GATE_*)
    char *C2;           // DX only: second output, the value before the activation (same shape, type and stride as C), or null
    double p;           // host only: dropout probability, for choosing tile shapes
    // the forward kernel that draws its own mask (SeededGrid): the generator's key (seed) and stream words, and the
    // keep threshold floor(p 2^32)
    uint32_t key0, key1, ctr2, ctr3;
    uint64_t threshold;
    double p_call;      // the dropout probability of the call (compared with the one a drawn mask records)
    int *status;        // the library's status word on this device, or null
    bool w_nk;          // host side: the weight is [N,K] and the kernel reads it so (see w_nk_native in the launch code)
    bool kept_given;    // host side: the caller stated the kept share itself (a mask of its own bits, whose structure is unknown)
};

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(_Float16)))) _Float16 f16x8;
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(8 * sizeof(short)))) short s16x8;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

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

// A value that is the same in every lane, told to the compiler (it then lives in a scalar register
// and everything derived from it is scalar arithmetic).
__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }




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
//         c = sqrt(2/pi), which is 0.5 v (1 + tanh(c (v + 0.044715 v^3)));
//         SDROP_ACT_GELU_ERF: 0.5 v (1 + erf(v / sqrt 2))
//   aux   matrix of the operands' type and the output's shape.  SDROP_GATE_RELU: where it is not > 0
//         the output is 0 (the backward of a ReLU, given the ReLU's output or input).
//         SDROP_GATE_GELU_TANH / SDROP_GATE_GELU_ERF: the output is multiplied by the derivative of
//         that GELU at aux (the backward of a GELU, given its input).
struct Tail {
    const float *bias;
    const char *aux;
    const char *c0;     // the output's origin
    int act;
    int gate_mode;
};
__device__ __forceinline__ Tail make_tail(const GemmParams &P)
{
    Tail t;
    t.bias = P.bias; t.aux = P.aux; t.c0 = P.C; t.act = P.act; t.gate_mode = P.gate_mode;
    return t;
}
// The tail that writes the second output of the producing layer: bias, no activation, no gate.
__device__ __forceinline__ Tail make_tail_preact(const GemmParams &P)
{
    Tail t;
    t.bias = P.bias; t.aux = nullptr; t.c0 = P.C2; t.act = SDROP_ACT_NONE; t.gate_mode = SDROP_GATE_RELU;
    return t;
}
// act4 / gate4 work on four consecutive columns of one output row (a register quad of the
// accumulator).  The persistent kernels gate their 16-bit outputs under a ReLU gate after rounding
// instead, 16 bytes at a time (gate16), which selects the same values.
// The bias does not change while the kernel runs: read through the constant address space, its
// loads may be moved and merged across the output stores.
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef const __attribute__((address_space(4))) f32x4 *const_f4;
// exp(-z^2/2) and erf(z / sqrt 2) together, the latter by the rational approximation 7.1.26 of
// Abramowitz and Stegun (Hastings): erf(x) = 1 - (a1 t + .. + a5 t^5) exp(-x^2), t = 1 / (1 + p x),
// x >= 0, odd in x; absolute error below 1.5e-7, far under the rounding of a 16-bit output and of
// the fp32 sums that feed it, at a third of the library routine's instructions.
__device__ __forceinline__ float erf_rsqrt2(float z, float &gauss)
{
    const float x = fabsf(z) * 0.7071067811865476f;
    const float t = __builtin_amdgcn_rcpf(1.f + 0.3275911f * x);
    gauss = __expf(-x * x);
    const float poly = t * (0.254829592f + t * (-0.284496736f + t * (1.421413741f + t * (-1.453152027f + t * 1.061405429f))));
    return copysignf(1.f - poly * gauss, z);
}
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
    } else if (act == SDROP_ACT_GELU_ERF) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float gauss;
            v[e] = 0.5f * v[e] * (1.f + erf_rsqrt2(v[e], gauss));
        }
    }
}
// v[e] gated by x[e] (see Tail)
__device__ __forceinline__ void gate4(int gate_mode, float (&v)[4], const float (&x)[4])
{
    if (gate_mode == SDROP_GATE_RELU) {
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = x[e] > 0.f ? v[e] : 0.f;
    } else if (gate_mode == SDROP_GATE_GELU_TANH) {
        // g = 0.5 x (1 + t), t = tanh(u), u = c (x + a x^3):  g' = 0.5 (1 + t) + 0.5 x (1 - t^2) c (1 + 3 a x^2)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float z = x[e];
            const float u = 0.7978845608028654f * (z + 0.044715f * z * z * z);
            const float t = 1.f - 2.f * __builtin_amdgcn_rcpf(1.f + __expf(2.f * u));
            v[e] *= 0.5f * (1.f + t) + 0.5f * z * (1.f - t * t) * 0.7978845608028654f * (1.f + 0.134145f * z * z);
        }
    } else {
        // g = x Phi(x):  g' = Phi(x) + x phi(x)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float z = x[e];
            float gauss;                                   // exp(-z^2 / 2), shared by both terms
            const float cdf = 0.5f * (1.f + erf_rsqrt2(z, gauss));
            v[e] *= cdf + z * 0.3989422804014327f * gauss;
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
    int wave, chunk_even;                                 // chunk_even: the 16-byte chunk this lane fetches in even passes
    __device__ __forceinline__ void init(int64_t ld_bytes, int w)
    {
        const int lane = threadIdx.x & 63;
        wave = w;
        const int r0 = 8 * wave + (lane >> 3);
        const uint32_t row_off = (uint32_t)r0 * (uint32_t)ld_bytes;
        chunk_even = (lane & 7) ^ swz(r0);
        voff_even = row_off + (chunk_even << 4);
        voff_odd = row_off + ((chunk_even ^ 4) << 4);
    }
    // pass i of this wavefront.  nch < 8: the slice is the ragged last one of the reduction and holds
    // only nch valid 16-byte chunks per row; lanes whose chunk lies beyond fetch nothing and clear
    // their 16 bytes of LDS instead (the caller waits for those LDS writes before it publishes the slice).
    __device__ __forceinline__ void issue(const char *const (&base)[NGRP], int64_t ld_bytes, char *lds, int i, int nch = 8) const
    {
        const int g = (PASS_ROWS * i) / GROUP_ROWS;       // uniform: pass i covers rows PASS_ROWS*i ..
        const char *sbase = base[g] + (int64_t)(PASS_ROWS * i - g * GROUP_ROWS) * ld_bytes;
        // bit 5 of the row (the only bit of a pass offset that swz() sees) picks the lane offset
        const bool odd = ((PASS_ROWS * i) & 32) != 0;
        char *const dst = lds + (wave + NW * i) * 1024;
        if (nch == 8) {
            dma16(sbase, odd ? voff_odd : voff_even, dst);
        } else {
            const int lane = threadIdx.x & 63;
            if ((odd ? chunk_even ^ 4 : chunk_even) < nch) dma16(sbase, odd ? voff_odd : voff_even, dst);
            else *reinterpret_cast<uint4 *>(dst + lane * 16) = make_uint4(0, 0, 0, 0);
        }
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
    int wave, chunk;                                         // chunk: the 16-byte chunk of the row this lane fetches
    __device__ __forceinline__ void init(int64_t ld_bytes, int w)
    {
        const int lane = threadIdx.x & 63;
        wave = w;
        const int kl = (lane * 16) / ROW_BYTES;              // row within the instruction
        const int cpos = ((lane * 16) % ROW_BYTES) >> 4;     // 16-byte slot within the row
        const int k0 = RPI * wave + kl;
        chunk = cpos ^ swz_t<ROWS>(k0);
        voff = (uint32_t)kl * (uint32_t)ld_bytes + (chunk << 4);
    }
    // nch < ROWS / 8: the tile hangs over the end of the rows (the last tile column of a ragged N)
    // and only its first nch >= 1 chunks per row exist: the other lanes fetch nothing, and their
    // LDS columns keep whatever they held (columns beyond N, which no one stores).
    __device__ __forceinline__ void issue(const char *const (&base)[1], int64_t ld_bytes, char *lds, int i, int nch = ROWS / 8) const
    {
        const int I = wave + NW * i;
        if (nch == ROWS / 8) dma16(base[0] + (int64_t)(RPI * I) * ld_bytes, voff, lds + I * 1024);
        else if (chunk < nch) dma16(base[0] + (int64_t)(RPI * I) * ld_bytes, voff, lds + I * 1024);
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

}  // namespace
}  // namespace sdrop
#endif
