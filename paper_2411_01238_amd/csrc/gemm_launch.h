// Launch logic of the GEMM kernels for one operand type (included by the typed translation units only).
#ifndef SDROP_GEMM_LAUNCH_H
#define SDROP_GEMM_LAUNCH_H
#include "gemm_host.h"
#include "gemm_tile_kernel.h"
#include "gemm_persistent_kernels.h"

namespace sdrop {
namespace {

// WM x WN: wavefront grid of the kernel without ragged edges; WMR x WNR (4 wavefronts): with.


template <int TMODE, int OP, class T, class OutT, int TM, int TN, int WM, int WN, int WMR, int WNR>
int launch_t(const GemmParams &P, int grid, bool ragged, hipStream_t stream, bool persistent_ok);

template <int OP, class T, class OutT, int TM, int TN, int WM, int WN, int WMR = WM, int WNR = WN>
int launch(const GemmParams &P, int grid, bool ragged, hipStream_t stream, bool persistent_ok = true)
{
    // dW takes no tail, and dX with a tail runs on 128-wide tiles only (dx_plan)
    constexpr bool kHasTailForms = OP == FWD || (OP == DX && TN == 128);
    if constexpr (!kHasTailForms) {
        if (has_tail(P)) return SDROP_EINVAL;
    }
    if constexpr (kHasTailForms) {
        switch (tail_mode(P)) {
        case kTailNone: break;
#define SDROP_TAIL_CASE(m) case m: return launch_t<m, OP, T, OutT, TM, TN, WM, WN, WMR, WNR>(P, grid, ragged, stream, persistent_ok)
        SDROP_TAIL_CASE(kTailLight);
        SDROP_TAIL_CASE(kTailReluGate);
        SDROP_TAIL_CASE(kTailGeluErf);
        SDROP_TAIL_CASE(kTailGeluErfGate);
        default: SDROP_TAIL_CASE(kTailGeneric);
#undef SDROP_TAIL_CASE
        }
    }
    return launch_t<kTailNone, OP, T, OutT, TM, TN, WM, WN, WMR, WNR>(P, grid, ragged, stream, persistent_ok);
}

// TMODE picks the persistent kernel's form; the kernels that run one workgroup per tile have one form with a tail.
template <int TMODE, int OP, class T, class OutT, int TM, int TN, int WM, int WN, int WMR, int WNR>
int launch_t(const GemmParams &P, int grid, bool ragged, hipStream_t stream, bool persistent_ok)
{
    constexpr bool TAIL = TMODE != kTailNone;
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
        // the persistent form also has a variant for a ragged last tile column, without a tail
        if ((!ragged || !TAIL) && persistent_ok) {
            // persistent form: three operand stages plus 4 KiB of output staging per computing wavefront
            constexpr int P_LDS = 3 * (TM + TN) * TK * 2 + WM * WN * 4096;
            auto k_whole = gemm_persistent_kernel<OP, T, OutT, TM, TN, WM, WN, TMODE, false>;
            auto k_edge = gemm_persistent_kernel<OP, T, OutT, TM, TN, WM, WN, TMODE, !TAIL>;    // (the same kernel when there is a tail)
            static int pers_ok = -1;    // per instantiation: does the device grant that much LDS?
            if (pers_ok < 0) {
                hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_whole),
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, P_LDS);
                if (e == hipSuccess)
                    e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_edge),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, P_LDS);
                pers_ok = (e == hipSuccess);
                if (!pers_ok) (void)hipGetLastError();
            }
            auto k_pers = ragged ? k_edge : k_whole;
            if (pers_ok) {
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

// The forward kernel that draws its own mask and writes the mask object (block grids of at most 128 x 64; whole
// tiles or a ragged last tile column).  Returns -1 when the device does not grant the LDS.
template <class T, class OutT, int TM>
int launch_fwd_seeded(const GemmParams &P, hipStream_t stream)
{
    constexpr int P_LDS = 3 * (TM + 256) * TK * 2 + 4 * 4096;
    auto k_whole = fwd_seeded_kernel<T, OutT, TM, false>;
    auto k_edge = fwd_seeded_kernel<T, OutT, TM, true>;
    static int ok = -1;     // per instantiation: does the device grant that much LDS?
    if (ok < 0) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_whole), hipFuncAttributeMaxDynamicSharedMemorySize, P_LDS);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_edge), hipFuncAttributeMaxDynamicSharedMemorySize, P_LDS);
        ok = (e == hipSuccess);
        if (!ok) (void)hipGetLastError();
    }
    if (!ok) return -1;
    GemmParams Q = P;
    Q.n_tiles = (int)((P.N + 255) / 256);
    Q.splits = 1;
    Q.total_tiles = Q.MB * Q.n_tiles;
    const int ncu = cu_count();
    auto k = P.N % 256 != 0 ? k_edge : k_whole;
    hipLaunchKernelGGL(k, dim3((unsigned)(Q.total_tiles < ncu ? Q.total_tiles : ncu)), dim3(512), P_LDS, stream, Q);
    return hip_status(hipGetLastError());
}

// eq. (1) with the weight as [N,K], read in place (N a multiple of 256, no tail); SEEDED: the mask drawn in the same
// launch (block grids of at most 128 x 64).  Returns -1 when the device does not grant the LDS.
template <class T, class OutT, int TM, bool SEEDED = false>
int launch_fwd_nk(const GemmParams &P, hipStream_t stream)
{
    constexpr int P_LDS = 3 * (TM + 256) * TK * 2 + 4 * 4096;
    auto k = fwd_nk_kernel<T, OutT, TM, SEEDED>;
    static int ok = -1;     // per instantiation: does the device grant that much LDS?
    if (ok < 0) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, P_LDS);
        ok = (e == hipSuccess);
        if (!ok) (void)hipGetLastError();
    }
    if (!ok) return -1;
    GemmParams Q = P;
    Q.n_tiles = (int)(P.N / 256);
    Q.splits = 1;
    Q.total_tiles = Q.MB * Q.n_tiles;
    const int ncu = cu_count();
    hipLaunchKernelGGL(k, dim3((unsigned)(Q.total_tiles < ncu ? Q.total_tiles : ncu)), dim3(512), P_LDS, stream, Q);
    return hip_status(hipGetLastError());
}

// eq. (3) with the gradient written as [N,K] (tiles of TM = BK rows, N a multiple of 256; P.splits parts).
template <class T, class OutT, int TM>
int launch_dw_nk(const GemmParams &P, hipStream_t stream)
{
    constexpr int P_LDS = 3 * (TM + 256) * TK * 2 + 4 * 4096;
    auto k = dw_nk_kernel<T, OutT, TM>;
    static int ok = -1;     // per instantiation: does the device grant that much LDS?
    if (ok < 0) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, P_LDS);
        ok = (e == hipSuccess);
        if (!ok) (void)hipGetLastError();
    }
    if (!ok) return -1;
    GemmParams Q = P;
    Q.n_tiles = (int)(P.N / 256);
    Q.total_tiles = Q.KB * Q.n_tiles * Q.splits;
    const int ncu = cu_count();
    hipLaunchKernelGGL(k, dim3((unsigned)(Q.total_tiles < ncu ? Q.total_tiles : ncu)), dim3(512), P_LDS, stream, Q);
    return hip_status(hipGetLastError());
}

// Persistent dX: one workgroup per CU (fewer when there are fewer block positions than CUs).
template <class T, class OutT, int TN, int TAIL>
int launch_dx_persistent_t(const GemmParams &P, hipStream_t stream);

template <class T, class OutT, int TN>
int launch_dx_persistent(const GemmParams &P, hipStream_t stream)
{
    if constexpr (TN == 128) {
        switch (tail_mode(P)) {
        case kTailNone: break;
        case kTailLight: return launch_dx_persistent_t<T, OutT, TN, kTailLight>(P, stream);
        case kTailReluGate: return launch_dx_persistent_t<T, OutT, TN, kTailReluGate>(P, stream);
        case kTailGeluErf: return launch_dx_persistent_t<T, OutT, TN, kTailGeluErf>(P, stream);
        case kTailGeluErfGate: return launch_dx_persistent_t<T, OutT, TN, kTailGeluErfGate>(P, stream);
        default: return launch_dx_persistent_t<T, OutT, TN, kTailGeneric>(P, stream);
        }
    } else {
        if (has_tail(P)) return SDROP_EINVAL;       // dX with a tail runs on 128-wide tiles only (dx_plan)
    }
    return launch_dx_persistent_t<T, OutT, TN, kTailNone>(P, stream);
}

template <class T, class OutT, int TN, int TAIL>
int launch_dx_persistent_t(const GemmParams &P, hipStream_t stream)
{
    constexpr int P_LDS = 3 * (128 + TN) * TK * 2 + 4 * 4096;
    // two forms: N a multiple of the 64-wide slice, or with a ragged last slice
    auto k_whole = gemm_persistent_dx_kernel<T, OutT, 128, TN, 2, 2, TAIL, false>;
    auto k_ragged = gemm_persistent_dx_kernel<T, OutT, 128, TN, 2, 2, TAIL, true>;
    static int ok = -1;     // per instantiation: does the device grant that much LDS?
    if (ok < 0) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_whole), hipFuncAttributeMaxDynamicSharedMemorySize, P_LDS);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_ragged), hipFuncAttributeMaxDynamicSharedMemorySize, P_LDS);
        ok = (e == hipSuccess);
        if (!ok) (void)hipGetLastError();
    }
    auto k = P.N % TK == 0 ? k_whole : k_ragged;
    if (!ok) return -1;
    const int64_t positions = (int64_t)P.MB * P.KB;
    const int ncu = cu_count();
    hipLaunchKernelGGL(k, dim3((unsigned)(positions < ncu ? positions : ncu)), dim3(512), P_LDS, stream, P);
    return hip_status(hipGetLastError());
}

// Persistent dX over the mask's pair list (128 x 256 tiles of two kept blocks).
template <class T, class OutT>
int launch_dx_pairs(const GemmParams &P, hipStream_t stream)
{
    constexpr int P_LDS = 3 * (128 + 256) * TK * 2 + 4 * 4096;
    auto k = gemm_persistent_dx_kernel<T, OutT, 128, 256, 2, 2, kTailNone, false, true>;
    static int ok = -1;     // per instantiation: does the device grant that much LDS?
    if (ok < 0) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, P_LDS);
        ok = (e == hipSuccess);
        if (!ok) (void)hipGetLastError();
    }
    if (!ok) return -1;
    const int64_t positions = (int64_t)P.MB * P.KB;
    const int ncu = cu_count();
    hipLaunchKernelGGL(k, dim3((unsigned)(positions < ncu ? positions : ncu)), dim3(512), P_LDS, stream, P);
    return hip_status(hipGetLastError());
}

// Persistent dX with the weight as [N,K], read in place (128 x 128 blocks, one per tile; N a multiple of 64).
template <class T, class OutT>
int launch_dx_nk(const GemmParams &P, hipStream_t stream)
{
    constexpr int P_LDS = 3 * (128 + 128) * TK * 2 + 4 * 4096;
    auto k = gemm_persistent_dx_kernel<T, OutT, 128, 128, 2, 2, kTailNone, false, false, true>;
    static int ok = -1;     // per instantiation: does the device grant that much LDS?
    if (ok < 0) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, P_LDS);
        ok = (e == hipSuccess);
        if (!ok) (void)hipGetLastError();
    }
    if (!ok) return -1;
    const int64_t positions = (int64_t)P.MB * P.KB;
    const int ncu = cu_count();
    hipLaunchKernelGGL(k, dim3((unsigned)(positions < ncu ? positions : ncu)), dim3(512), P_LDS, stream, P);
    return hip_status(hipGetLastError());
}

// Tile shapes: the tile edge that lies along the mask must equal the mask's block
// (Section 3.2); the N edge is free (Section 3.3) and is 256 wide.  DX gathers
// 256/BK kept blocks of one block row into a 256-wide tile.
template <int OP, class T, class OutT>
int dispatch_tile(GemmParams &P, hipStream_t stream)
{
    if constexpr (OP != DX) {
        // N is not a multiple of the 256-wide tile: only the last tile column is ragged, but a launch is
        // one kernel, and the kernel with bounds checks is the slow one (4096^3 with N = 4104: fwd 158 us
        // against 66 us at N = 4096).  With at least a chip's worth of whole tiles the output columns are
        // cut in two, [0, N - N % 256) for the fast kernels and the rest for the checked one, which the
        // leading dimensions make a matter of pointers: operands and outputs keep their strides.
        const int64_t n_full = P.N / 256 * 256;
        // (Without a tail the persistent kernels take the ragged column themselves, where they apply.)
        const bool one_launch = !has_tail(P) && (OP == FWD || P.BK == 128 || dw64_persistent(P));
        if (!one_launch && P.N % 256 != 0 && n_full > 0 && (int64_t)(OP == FWD ? P.MB : P.KB * P.splits) * (n_full / 256) >= cu_count()) {
            GemmParams Q = P;
            Q.N = n_full;
            const int rc = dispatch_tile<OP, T, OutT>(Q, stream);
            if (rc != SDROP_OK) return rc;
            Q = P;
            Q.N = P.N - n_full;
            Q.B += n_full * 2;
            Q.C += n_full * (int64_t)sizeof(OutT);
            if (Q.bias) Q.bias += n_full;
            if (Q.aux) Q.aux += n_full * 2;
            return dispatch_tile<OP, T, OutT>(Q, stream);
        }
    }
    if constexpr (OP == FWD) {
        if (P.w_nk) {
            const int rc = P.BM == 128 ? launch_fwd_nk<T, OutT, 128>(P, stream) : launch_fwd_nk<T, OutT, 64>(P, stream);
            return rc == -1 ? SDROP_EHIP : rc;       // (the [K,N] persistent form needs the same LDS)
        }
        P.n_tiles = (int)((P.N + 255) / 256);
        const int grid = P.MB * P.n_tiles;
        const bool ragged = P.N % 256 != 0;
        if (P.BM == 128) return launch<FWD, T, OutT, 128, 256, 1, 4>(P, grid, ragged, stream);
        return launch<FWD, T, OutT, 64, 256, 1, 4>(P, grid, ragged, stream);
    } else if constexpr (OP == DW) {
        if (P.w_nk) {
            const int rc = P.BK == 128 ? launch_dw_nk<T, OutT, 128>(P, stream) : launch_dw_nk<T, OutT, 64>(P, stream);
            return rc == -1 ? SDROP_EHIP : rc;
        }
        P.n_tiles = (int)((P.N + 255) / 256);
        const int grid = P.KB * P.n_tiles * P.splits;
        const bool ragged = P.N % 256 != 0;
        if (P.BK == 128) return launch<DW, T, OutT, 128, 256, 1, 4>(P, grid, ragged, stream);
        // 64-row tiles: the persistent kernel runs one workgroup per CU, whose epilogue nothing
        // overlaps; with short kept lists (a few slices per tile) three co-resident workgroups of the
        // per-tile kernel do better (8192 x 1024 x 1024, 64 x 64 blocks, half kept, 16 parts:
        // 26.5 against 29.5 us; 16384 x 3072 x 768, a tenth dropped, 4 parts: 121 against 101 us)
        return launch<DW, T, OutT, 64, 256, 1, 4>(P, grid, ragged, stream, dw64_persistent(P));
    } else {
        if (P.w_nk) {
            const int rc = launch_dx_nk<T, OutT>(P, stream);
            return rc == -1 ? SDROP_EHIP : rc;
        }
        const DxPlan plan = dx_plan(P);
        const int TNsel = plan.TN, G_ = TNsel / P.BK;
        P.n_tiles = (P.KB + G_ - 1) / G_;
        // one kept block per tile: a workgroup per block position, rounded up to whole sets of 8 XCDs
        const int grid = G_ == 1 ? (P.MB * P.KB + 7) / 8 * 8 : P.MB * P.n_tiles;
        const bool ragged = P.N % TK != 0;
        if (plan.pairs) {
            const int rc = launch_dx_pairs<T, OutT>(P, stream);
            if (rc != -1) return rc;
            return SDROP_EHIP;            // (the plain 128 x 256 persistent form needs the same LDS)
        }
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

template <class T, class OutDX, class OutDW, int TN_DX, bool PAIRS = false, bool W_NK = false>
int launch_bwd_fused(const GemmParams &Pdx, const GemmParams &Pdw, hipStream_t stream)
{
    constexpr int LDS_DX = 3 * (128 + TN_DX) * TK * 2 + 4 * 4096, LDS_DW = 3 * (128 + 256) * TK * 2 + 4 * 4096;
    constexpr int P_LDS = LDS_DX > LDS_DW ? LDS_DX : LDS_DW;
    auto k = bwd_fused_kernel<T, OutDX, OutDW, TN_DX, PAIRS, W_NK>;
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
    if (TN == kTNPairs) return launch_bwd_fused<T, OutDX, OutDW, 256, true>(Pdx, Pdw, stream);
    if (TN == kTNNK) return launch_bwd_fused<T, OutDX, OutDW, 128, false, true>(Pdx, Pdw, stream);
    if (TN == 256) return launch_bwd_fused<T, OutDX, OutDW, 256>(Pdx, Pdw, stream);
    return launch_bwd_fused<T, OutDX, OutDW, 128>(Pdx, Pdw, stream);
}

template <class T, class OutDX, class OutDW, int TN_DX>
int launch_bwd_fused_tile64(const GemmParams &Pdx, const GemmParams &Pdw, int n_dx, int n_dw, hipStream_t stream)
{
    constexpr int P_LDS = stages_for(64, 256) * (64 + 256) * TK * 2;      // the larger of the two bodies' needs
    static_assert(stages_for(64, TN_DX) * (64 + TN_DX) * TK * 2 <= P_LDS, "dX's stages must fit");
    auto k = bwd_fused_tile64_kernel<T, OutDX, OutDW, TN_DX>;
    static int ok = -1;
    if (ok < 0) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, P_LDS);
        ok = (e == hipSuccess);
        if (!ok) (void)hipGetLastError();
    }
    if (!ok) return -1;
    hipLaunchKernelGGL(k, dim3((unsigned)(n_dx + n_dw)), dim3(256), P_LDS, stream, Pdx, Pdw, n_dx);
    return hip_status(hipGetLastError());
}

}  // namespace

template <class T> int dispatch_typed(int op, bool o32, GemmParams &P, hipStream_t stream)
{
    using O16 = typename In<T>::out16;
    if (op == FWD) return o32 ? dispatch_tile<FWD, T, float>(P, stream) : dispatch_tile<FWD, T, O16>(P, stream);
    if (op == DX) return o32 ? dispatch_tile<DX, T, float>(P, stream) : dispatch_tile<DX, T, O16>(P, stream);
    return o32 ? dispatch_tile<DW, T, float>(P, stream) : dispatch_tile<DW, T, O16>(P, stream);
}

template <class T> int fwd_seeded_typed(bool o32, const GemmParams &P, hipStream_t stream)
{
    using O16 = typename In<T>::out16;
    if (P.w_nk) {
        if (P.BM == 128) return o32 ? launch_fwd_nk<T, float, 128, true>(P, stream) : launch_fwd_nk<T, O16, 128, true>(P, stream);
        return o32 ? launch_fwd_nk<T, float, 64, true>(P, stream) : launch_fwd_nk<T, O16, 64, true>(P, stream);
    }
    if (P.BM == 128) return o32 ? launch_fwd_seeded<T, float, 128>(P, stream) : launch_fwd_seeded<T, O16, 128>(P, stream);
    return o32 ? launch_fwd_seeded<T, float, 64>(P, stream) : launch_fwd_seeded<T, O16, 64>(P, stream);
}

template <class T> int bwd_fused_typed(int form, int TN, bool o32, bool dw_f32, const GemmParams &Pdx, const GemmParams &Pdw,
                                       int n_dx, hipStream_t stream)
{
    using O16 = typename In<T>::out16;
    auto go = [&](auto odx, auto odw) -> int {
        using ODX = decltype(odx);
        using ODW = decltype(odw);
        if (form == kBwdPersistent) return launch_bwd_fused_tn<T, ODX, ODW>(TN, Pdx, Pdw, stream);
        if (form == kBwdTile128) return launch_bwd_fused_tile<T, ODX, ODW>(Pdx, Pdw, n_dx, stream);
        if (TN == 256) return launch_bwd_fused_tile64<T, ODX, ODW, 256>(Pdx, Pdw, n_dx, Pdw.total_tiles, stream);
        return launch_bwd_fused_tile64<T, ODX, ODW, 128>(Pdx, Pdw, n_dx, Pdw.total_tiles, stream);
    };
    if (o32) return go(float{}, float{});
    if (dw_f32) return go(O16{}, float{});
    return go(O16{}, O16{});
}

}  // namespace sdrop
#endif
