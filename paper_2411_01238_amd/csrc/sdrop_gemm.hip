// The three block-sparse GEMMs of SparseDrop (arxiv 2411.01238, Section 3.1
// eq. (1)-(3), Section 3.2) as one MFMA main loop with three instantiations.
//
//   FWD  Y  = s (X . m') W        tile (block row i, N tile): walks the kept K-blocks of row i
//   DX   dX = s (dY W^T) . m'     tile = one kept block (i,j): reduction over all of N
//   DW   dW = s (X . m')^T dY     tile (block column j, N tile): walks the kept row blocks of column j
//
// Each workgroup owns one TM x TN output tile and steps through its reduction
// in slices of TK = 64.  A slice of each operand is staged in LDS exactly as it
// lies in HBM (16-byte global loads, 16-byte LDS stores), two LDS stages deep:
// the global loads of slice t+1 are issued before the MFMAs of slice t and land
// in the other stage afterwards, one barrier per slice.  The paper names the
// lack of this software pipelining as the reason its kernels lose to dense at
// zero sparsity (Section 5.1).
//
// The matrix-core instruction is v_mfma_f32_32x32x16_{f16,bf16}: lane l supplies
// row (l%32) of the left operand and column (l%32) of the right operand, each
// as 8 consecutive reduction indices starting at 8*(l/32).  An operand whose
// reduction index is contiguous in memory (X in FWD, dY and W in DX) is read
// from LDS with one 16-byte load per lane.  An operand whose reduction index is
// the strided one (W in FWD; X and dY in DW) is read with the transposing LDS
// load ds_read_b64_tr_b16, which hands each lane four reduction-consecutive
// values out of a row-major tile, so no transposed copy is ever made.
// LDS rows are padded (16 bytes for reduction-contiguous tiles, 64 bytes for
// the others) so that both kinds of read are free of bank conflicts.
#include "sdrop_internal.h"

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

constexpr int TK = 64;           // reduction slice staged per step
constexpr int kThreads = 256;    // 4 wavefronts per workgroup

enum Op { FWD = 0, DX = 1, DW = 2 };

struct GemmParams {
    const char *A;      // FWD: X   DX: dY  DW: X
    const char *B;      // FWD: W   DX: W   DW: dY
    char *C;            // FWD: Y   DX: dX  DW: dW
    MaskView mv;
    int64_t M, K, N;
    int32_t BM, BK, MB, KB;
    int32_t n_tiles_n;  // FWD/DW: number of TN-wide tiles along N
    float scale;
};

// LDS row strides in bytes.  kmajor: rows of TK reduction-contiguous elements.
constexpr int lds_stride(bool kmajor, int cols) { return cols * 2 + (kmajor ? 16 : 64); }

template <int OP, int TM, int TN> struct Geometry {
    static constexpr bool A_KMAJ = (OP != DW);
    static constexpr bool B_KMAJ = (OP == DX);
    // tile as it lies in memory: [rows][cols], cols contiguous
    static constexpr int A_ROWS = A_KMAJ ? TM : TK, A_COLS = A_KMAJ ? TK : TM;
    static constexpr int B_ROWS = B_KMAJ ? TN : TK, B_COLS = B_KMAJ ? TK : TN;
    static constexpr int SA = lds_stride(A_KMAJ, A_COLS), SB = lds_stride(B_KMAJ, B_COLS);
    static constexpr int A_BYTES = A_ROWS * SA, B_BYTES = B_ROWS * SB;
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr int LDS_BYTES = 2 * STAGE_BYTES;
    static constexpr int A_CHUNKS = A_ROWS * A_COLS / 8 / kThreads;   // 16-byte chunks per thread
    static constexpr int B_CHUNKS = B_ROWS * B_COLS / 8 / kThreads;
    static_assert(A_CHUNKS >= 1 && B_CHUNKS >= 1, "tile too small for 256 threads");
};

// One operand slice: global -> registers.
template <int ROWS, int COLS, int NCH>
__device__ __forceinline__ void load_slice(uint4 (&r)[NCH], const char *base, int64_t ld_bytes, int lim_cols)
{
    constexpr int CPR = COLS / 8;
#pragma unroll
    for (int q = 0; q < NCH; ++q) {
        const int c = threadIdx.x + q * kThreads;
        const int row = c / CPR, cc = c % CPR;
        if (cc * 8 < lim_cols)
            r[q] = *reinterpret_cast<const uint4 *>(base + row * ld_bytes + cc * 16);
        else
            r[q] = make_uint4(0, 0, 0, 0);
    }
}

// registers -> LDS, same [rows][cols] arrangement with padded rows.
template <int ROWS, int COLS, int NCH, int STRIDE>
__device__ __forceinline__ void store_slice(const uint4 (&r)[NCH], char *lds)
{
    constexpr int CPR = COLS / 8;
#pragma unroll
    for (int q = 0; q < NCH; ++q) {
        const int c = threadIdx.x + q * kThreads;
        const int row = c / CPR, cc = c % CPR;
        *reinterpret_cast<uint4 *>(lds + row * STRIDE + cc * 16) = r[q];
    }
}

// MFMA operand for 32 rows (or columns) starting at `base32` of the tile, reduction
// indices [kk*16, kk*16+16): lane l gets index base32 + l%32, reduction 8*(l/32)..+8.
template <class T, bool KMAJ, int STRIDE>
__device__ __forceinline__ typename In<T>::vec read_frag(const char *lds, int base32, int kk)
{
    const int l = threadIdx.x & 63;
    if constexpr (KMAJ) {
        const char *p = lds + (base32 + (l & 31)) * STRIDE + (kk * 2 + (l >> 5)) * 16;
        return *reinterpret_cast<const typename In<T>::vec *>(p);
    } else {
        // transposing read: within each group of 16 lanes, lane q loads 4 elements of
        // row q/4 at columns 4*(q%4).., and receives column (q) of the 4x16 patch
        const int row = kk * 16 + (l >> 5) * 8 + ((l & 15) >> 2);
        const int col = base32 + ((l >> 4) & 1) * 16 + (l & 3) * 4;
        const char *p = lds + row * STRIDE + col * 2;
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p + 4 * STRIDE));
        const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        return __builtin_bit_cast(typename In<T>::vec, v);
    }
}

template <class OutT> __device__ __forceinline__ void store_out(OutT *p, float v) { *p = static_cast<OutT>(v); }

template <int OP, class T, class OutT, int TM, int TN, int WM, int WN>
__global__ __launch_bounds__(kThreads) void gemm_kernel(GemmParams P)
{
    using G = Geometry<OP, TM, TN>;
    static_assert(WM * WN * 64 == kThreads, "4 wavefronts");
    constexpr int WTM = TM / WM, WTN = TN / WN, MI = WTM / 32, NI = WTN / 32;
    static_assert(MI >= 1 && NI >= 1 && WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be 32-aligned");

    extern __shared__ __attribute__((aligned(16))) char smem[];

    // a kernel handed a mask built for another problem writes nothing
    const MaskHeader *H = P.mv.hdr;
    if (H->magic != kMaskMagic || H->M != P.M || H->K != P.K || H->BM != P.BM || H->BK != P.BK) return;

    const int esz = 2;
    const char *a_tile = nullptr, *b_tile = nullptr;   // advanced per step
    int64_t lda, ldb, ldc;                              // in bytes
    char *c_tile;
    int c_lim;                                          // valid output columns in this tile
    int nsteps, sub;                                    // reduction steps; TK-slices per mask block
    const int32_t *list = nullptr;                      // kept-block list walked by this tile
    int a_lim = TK, b_lim = TK;

    if constexpr (OP == FWD) {
        const int t = blockIdx.x;
        const int i = P.mv.row_order[t / P.n_tiles_n], nt = t % P.n_tiles_n;
        const int rp = P.mv.row_ptr[i];
        list = P.mv.col_idx + rp;
        sub = P.BK / TK;
        nsteps = (P.mv.row_ptr[i + 1] - rp) * sub;
        lda = P.K * esz; ldb = P.N * esz; ldc = P.N * (int64_t)sizeof(OutT);
        a_tile = P.A + (int64_t)i * P.BM * lda;
        b_tile = P.B + (int64_t)nt * TN * esz;
        c_tile = P.C + (int64_t)i * P.BM * ldc + (int64_t)nt * TN * sizeof(OutT);
        { const int64_t left = P.N - (int64_t)nt * TN; c_lim = left < TN ? (int)left : TN; }
        b_lim = c_lim;
    } else if constexpr (OP == DW) {
        const int t = blockIdx.x;
        const int j = P.mv.col_order[t / P.n_tiles_n], nt = t % P.n_tiles_n;
        const int cp = P.mv.col_ptr[j];
        list = P.mv.row_idx + cp;
        sub = P.BM / TK;
        nsteps = (P.mv.col_ptr[j + 1] - cp) * sub;
        lda = P.K * esz; ldb = P.N * esz; ldc = P.N * (int64_t)sizeof(OutT);
        a_tile = P.A + (int64_t)j * P.BK * esz;
        b_tile = P.B + (int64_t)nt * TN * esz;
        c_tile = P.C + (int64_t)j * P.BK * ldc + (int64_t)nt * TN * sizeof(OutT);
        { const int64_t left = P.N - (int64_t)nt * TN; c_lim = left < TN ? (int)left : TN; }
        b_lim = c_lim;
        a_lim = TM;
    } else {
        // blockIdx.x = q * MB + i: rank-q kept block of row i is computed; block
        // position q of row i is zero-filled if it is a dropped one
        const int i = blockIdx.x % P.MB, q = blockIdx.x / P.MB;
        lda = P.N * esz; ldb = P.N * esz; ldc = P.K * (int64_t)sizeof(OutT);
        if (!((P.mv.bits[(int64_t)i * H->words_per_row + (q >> 6)] >> (q & 63)) & 1)) {
            char *z = P.C + (int64_t)i * P.BM * ldc + (int64_t)q * P.BK * sizeof(OutT);
            constexpr int row_chunks = TN * (int)sizeof(OutT) / 16;
            for (int c = threadIdx.x; c < TM * row_chunks; c += kThreads)
                *reinterpret_cast<uint4 *>(z + (c / row_chunks) * ldc + (c % row_chunks) * 16) = make_uint4(0, 0, 0, 0);
        }
        const int rp = P.mv.row_ptr[i];
        if (q >= P.mv.row_ptr[i + 1] - rp) return;
        const int j = P.mv.col_idx[rp + q];
        sub = 1;
        nsteps = (int)((P.N + TK - 1) / TK);
        a_tile = P.A + (int64_t)i * P.BM * lda;
        b_tile = P.B + (int64_t)j * P.BK * ldb;
        c_tile = P.C + (int64_t)i * P.BM * ldc + (int64_t)j * P.BK * sizeof(OutT);
        c_lim = TN;
    }

    // pointers to the slice of step s
    auto slice_ptrs = [&](int s, const char *&ap, const char *&bp, int &al, int &bl) {
        if constexpr (OP == FWD) {
            const int64_t k0 = (int64_t)list[s / sub] * P.BK + (int64_t)(s % sub) * TK;
            ap = a_tile + k0 * esz; bp = b_tile + k0 * ldb; al = TK; bl = b_lim;
        } else if constexpr (OP == DW) {
            const int64_t m0 = (int64_t)list[s / sub] * P.BM + (int64_t)(s % sub) * TK;
            ap = a_tile + m0 * lda; bp = b_tile + m0 * ldb; al = a_lim; bl = b_lim;
        } else {
            const int64_t n0 = (int64_t)s * TK;
            ap = a_tile + n0 * esz; bp = b_tile + n0 * esz;
            { const int64_t left = P.N - n0; al = bl = left < TK ? (int)left : TK; }
        }
    };

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int wm = wave / WN, wn = wave % WN;

    f32x16 acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;

    uint4 ra[G::A_CHUNKS], rb[G::B_CHUNKS];
    if (nsteps > 0) {
        const char *ap, *bp; int al, bl;
        slice_ptrs(0, ap, bp, al, bl);
        load_slice<G::A_ROWS, G::A_COLS, G::A_CHUNKS>(ra, ap, lda, al);
        load_slice<G::B_ROWS, G::B_COLS, G::B_CHUNKS>(rb, bp, ldb, bl);
        store_slice<G::A_ROWS, G::A_COLS, G::A_CHUNKS, G::SA>(ra, smem);
        store_slice<G::B_ROWS, G::B_COLS, G::B_CHUNKS, G::SB>(rb, smem + G::A_BYTES);
    }
    __syncthreads();

    for (int s = 0; s < nsteps; ++s) {
        const bool more = s + 1 < nsteps;
        if (more) {
            const char *ap, *bp; int al, bl;
            slice_ptrs(s + 1, ap, bp, al, bl);
            load_slice<G::A_ROWS, G::A_COLS, G::A_CHUNKS>(ra, ap, lda, al);
            load_slice<G::B_ROWS, G::B_COLS, G::B_CHUNKS>(rb, bp, ldb, bl);
        }
        const char *sa = smem + (s & 1) * G::STAGE_BYTES;
        const char *sb = sa + G::A_BYTES;
#pragma unroll
        for (int kk = 0; kk < TK / 16; ++kk) {
            typename In<T>::vec fa[MI], fb[NI];
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) fa[mi] = read_frag<T, G::A_KMAJ, G::SA>(sa, wm * WTM + mi * 32, kk);
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) fb[ni] = read_frag<T, G::B_KMAJ, G::SB>(sb, wn * WTN + ni * 32, kk);
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NI; ++ni) acc[mi][ni] = In<T>::mfma(fa[mi], fb[ni], acc[mi][ni]);
        }
        if (more) {
            char *da = smem + ((s + 1) & 1) * G::STAGE_BYTES;
            store_slice<G::A_ROWS, G::A_COLS, G::A_CHUNKS, G::SA>(ra, da);
            store_slice<G::B_ROWS, G::B_COLS, G::B_CHUNKS, G::SB>(rb, da + G::A_BYTES);
        }
        __syncthreads();
    }

    // epilogue: scale in fp32, round once, store.  Accumulator register r of lane l is
    // row 8*(r/4) + 4*(l/32) + r%4, column l%32 of its 32x32 patch.
    const float scale = P.scale;
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
            const int col = wn * WTN + ni * 32 + (lane & 31);
            if (col < c_lim) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = wm * WTM + mi * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
                    store_out(reinterpret_cast<OutT *>(c_tile + row * ldc) + col, acc[mi][ni][r] * scale);
                }
            }
        }
}

template <int OP, class T, class OutT, int TM, int TN, int WM, int WN>
int launch(const GemmParams &P, int grid, hipStream_t stream)
{
    using G = Geometry<OP, TM, TN>;
    auto kern = gemm_kernel<OP, T, OutT, TM, TN, WM, WN>;
    static bool attr_set = false;   // per instantiation
    if (!attr_set) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, G::LDS_BYTES);
        if (e != hipSuccess) return hip_status(e);
        attr_set = true;
    }
    if (grid <= 0) return SDROP_OK;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kThreads), G::LDS_BYTES, stream, P);
    return hip_status(hipGetLastError());
}

// Tile shapes: the tile edge that lies along the mask must equal the mask's block
// (Section 3.2); the N edge is free (Section 3.3) and is 256 where N allows.
template <int OP, class T, class OutT>
int dispatch_tile(GemmParams &P, hipStream_t stream)
{
    if constexpr (OP == FWD) {
        P.n_tiles_n = (int)((P.N + 255) / 256);
        const int grid = P.MB * P.n_tiles_n;
        if (P.BM == 128) return launch<FWD, T, OutT, 128, 256, 2, 2>(P, grid, stream);
        return launch<FWD, T, OutT, 64, 256, 1, 4>(P, grid, stream);
    } else if constexpr (OP == DW) {
        P.n_tiles_n = (int)((P.N + 255) / 256);
        const int grid = P.KB * P.n_tiles_n;
        if (P.BK == 128) return launch<DW, T, OutT, 128, 256, 2, 2>(P, grid, stream);
        return launch<DW, T, OutT, 64, 256, 1, 4>(P, grid, stream);
    } else {
        const int grid = P.MB * P.KB;
        if (P.BM == 128 && P.BK == 128) return launch<DX, T, OutT, 128, 128, 2, 2>(P, grid, stream);
        if (P.BM == 128 && P.BK == 64) return launch<DX, T, OutT, 128, 64, 2, 2>(P, grid, stream);
        if (P.BM == 64 && P.BK == 128) return launch<DX, T, OutT, 64, 128, 2, 2>(P, grid, stream);
        return launch<DX, T, OutT, 64, 64, 2, 2>(P, grid, stream);
    }
}

template <int OP>
int run(const void *a, const void *b, const void *mask, void *out,
        int64_t M, int64_t K, int64_t N, int BM, int BK, double p,
        int dtype, int out_dtype, void *ws, size_t ws_bytes, void *stream)
{
    const int rc = check_gemm_args(a, b, mask, out, M, K, N, BM, BK, p, dtype, out_dtype);
    if (rc != SDROP_OK) return rc;
    if (ws_bytes < sdrop_workspace_bytes(OP, M, K, N, BM, BK, dtype, out_dtype)) return SDROP_EWORKSPACE;
    (void)ws;
    sdrop_mask_layout_t L;
    sdrop_mask_layout(M, K, BM, BK, &L);
    GemmParams P;
    P.A = static_cast<const char *>(a);
    P.B = static_cast<const char *>(b);
    P.C = static_cast<char *>(out);
    P.mv = make_view(mask, L);
    P.M = M; P.K = K; P.N = N; P.BM = BM; P.BK = BK;
    P.MB = (int32_t)L.MB; P.KB = (int32_t)L.KB;
    P.n_tiles_n = 0;
    P.scale = (p < 1.0) ? (float)(1.0 / (1.0 - p)) : 0.0f;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (dtype == SDROP_F16) {
        if (out_dtype == SDROP_F32) return dispatch_tile<OP, F16, float>(P, st);
        return dispatch_tile<OP, F16, _Float16>(P, st);
    }
    if (out_dtype == SDROP_F32) return dispatch_tile<OP, BF16, float>(P, st);
    return dispatch_tile<OP, BF16, __bf16>(P, st);
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
    if (M > (int64_t(1) << 30) || K > (int64_t(1) << 30) || N > (int64_t(1) << 30)) return SDROP_ESHAPE;
    if (dtype != SDROP_F16 && dtype != SDROP_BF16) return SDROP_EDTYPE;
    if (out_dtype != dtype && out_dtype != SDROP_F32) return SDROP_EDTYPE;
    const uintptr_t bits = reinterpret_cast<uintptr_t>(a) | reinterpret_cast<uintptr_t>(b) |
                           reinterpret_cast<uintptr_t>(mask) | reinterpret_cast<uintptr_t>(out);
    if (bits % 16) return SDROP_EALIGN;
    return SDROP_OK;
}

}  // namespace sdrop

extern "C" {

size_t sdrop_workspace_bytes(int op, int64_t M, int64_t K, int64_t N, int BM, int BK,
                             int dtype, int out_dtype)
{
    (void)op; (void)M; (void)K; (void)N; (void)BM; (void)BK; (void)dtype; (void)out_dtype;
    return 0;
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

}  // extern "C"
