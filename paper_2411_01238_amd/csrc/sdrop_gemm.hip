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
#include "gemm_host.h"
#include <atomic>
#include <math.h>

namespace sdrop {

// ---- launch heuristics and knobs (shared with the typed translation units through gemm_host.h) ----
// out[e] = scale * sum_c part[c][e], rounded once (the second pass of a split DW)
template <class OutT>
__global__ __launch_bounds__(256) void reduce_parts_kernel(const float *part, OutT *out_base, int64_t n, int splits, float scale,
                                                           int64_t ncols, int64_t ld, const MaskHeader *H,
                                                           int64_t M, int64_t K, int BM, int BK, double p_call, int *status)
{
    // like the first pass, write nothing when the mask was built for another problem (the planes are then unwritten)
    if (!mask_header_ok(H, M, K, BM, BK, true, p_call, status)) return;
    // eight consecutive elements per thread (two 16-byte loads per plane in flight: with four, 80 MB of planes took
    // 18.6 us); n, ncols and ld are multiples of 8, so the eight lie in one output row and its stores are 16-byte aligned
    const int64_t e = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 8;
    if (e >= n) return;
    OutT *const out = out_base + (e / ncols) * (ld - ncols) + e;  // row e / ncols of an output with `ld` elements per row
    float4 a0 = *reinterpret_cast<const float4 *>(part + e), a1 = *reinterpret_cast<const float4 *>(part + e + 4);
    for (int c = 1; c < splits; ++c) {
        const float4 v0 = *reinterpret_cast<const float4 *>(part + (int64_t)c * n + e);
        const float4 v1 = *reinterpret_cast<const float4 *>(part + (int64_t)c * n + e + 4);
        a0.x += v0.x; a0.y += v0.y; a0.z += v0.z; a0.w += v0.w;
        a1.x += v1.x; a1.y += v1.y; a1.z += v1.z; a1.w += v1.w;
    }
    const float r[8] = {a0.x * scale, a0.y * scale, a0.z * scale, a0.w * scale, a1.x * scale, a1.y * scale, a1.z * scale, a1.w * scale};
    if constexpr (sizeof(OutT) == 4) {
        *reinterpret_cast<float4 *>(out) = make_float4(r[0], r[1], r[2], r[3]);
        *reinterpret_cast<float4 *>(out + 4) = make_float4(r[4], r[5], r[6], r[7]);
    } else {
        typedef __attribute__((__vector_size__(8 * sizeof(OutT)))) OutT out8;
        const out8 o = {static_cast<OutT>(r[0]), static_cast<OutT>(r[1]), static_cast<OutT>(r[2]), static_cast<OutT>(r[3]),
                        static_cast<OutT>(r[4]), static_cast<OutT>(r[5]), static_cast<OutT>(r[6]), static_cast<OutT>(r[7])};
        *reinterpret_cast<out8 *>(out) = o;
    }
}

// dst[c][r] = src[r][c] for a rows x cols matrix of 2- or 4-byte elements (rows of src ld_src elements apart, rows of dst
// ld_dst apart): 64 x 64 tiles through LDS, so that both the reads and the writes cover whole 128-byte (or longer) runs.
// Used where a weight comes, or its gradient goes, in the [N,K] layout (see run()).
template <class E>
__global__ __launch_bounds__(256) void transpose_kernel(const E *src, E *dst, int64_t rows, int64_t cols, int64_t ld_src, int64_t ld_dst)
{
    __shared__ E tile[64][65];
    const int64_t r0 = (int64_t)blockIdx.y * 64, c0 = (int64_t)blockIdx.x * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    for (int r = ty; r < 64; r += 4)
        if (r0 + r < rows && c0 + tx < cols) tile[r][tx] = src[(r0 + r) * ld_src + c0 + tx];
    __syncthreads();
    for (int c = ty; c < 64; c += 4)
        if (c0 + c < cols && r0 + tx < rows) dst[(c0 + c) * ld_dst + r0 + tx] = tile[tx][c];
}

int launch_transpose(const void *src, void *dst, int64_t rows, int64_t cols, int64_t ld_src, int64_t ld_dst, int esz, hipStream_t st)
{
    const dim3 grid((unsigned)((cols + 63) / 64), (unsigned)((rows + 63) / 64));
    if (esz == 4)
        hipLaunchKernelGGL(transpose_kernel<uint32_t>, grid, dim3(256), 0, st, static_cast<const uint32_t *>(src), static_cast<uint32_t *>(dst), rows, cols, ld_src, ld_dst);
    else
        hipLaunchKernelGGL(transpose_kernel<uint16_t>, grid, dim3(256), 0, st, static_cast<const uint16_t *>(src), static_cast<uint16_t *>(dst), rows, cols, ld_src, ld_dst);
    return hip_status(hipGetLastError());
}

int dw_splits(int64_t M, int64_t N, int BM, int BK, int64_t K);

// Workspace of one product: the fp32 planes of a split dW first, then (weight in the [N,K] layout) a K x N matrix: the
// transposed weight for FWD / DX (operand type), the gradient before its transposition for DW (output type).
size_t ws_planes_bytes(int op, int64_t M, int64_t K, int64_t N, int BM, int BK)
{
    if (op != SDROP_OP_BWD_DW) return 0;
    const int splits = dw_splits(M, N, BM, BK, K);
    return splits > 1 ? (size_t)splits * (size_t)K * (size_t)N * sizeof(float) : 0;
}
size_t ws_total_bytes(int op, int64_t M, int64_t K, int64_t N, int BM, int BK, int out_dtype, bool w_nk)
{
    size_t need = ws_planes_bytes(op, M, K, N, BM, BK);
    if (w_nk) need += (size_t)K * (size_t)N * (op == SDROP_OP_BWD_DW && out_dtype == SDROP_F32 ? 4 : 2);
    return need;
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
// The pair list (see build_units): every unit is a 128 x 256 tile of two kept blocks, from the same block row or
// the same block column, so no tile is cut and (almost) none is half empty: ceil(kept / 2) equal tiles, each
// about 1.6 single-block tiles long.  Needs 128 x 128 blocks, a grid the list exists for, whole slices, no tail,
// dY and W with the same row stride, and a drawn mask (a caller's own bits may pair badly: a diagonal has no pairs
// at all and every unit would cost a tile of two).  Taken in place of single-block tiles where those would fill the
// chip (at least 1.5 kept blocks per CU) and rows hold enough blocks to pair: always in sdrop_bwd's single launch,
// whose dW workgroups take the CUs that dX's last round leaves idle; on its own only where it is expected to finish
// first.  Measured at 4096^3 (dX alone /
// sdrop_bwd, pairs against what the plan took before): half dropped, 511 blocks, 63 against 68 us / 123 against 130;
// 0.7 dropped, 281 blocks, 49 against 47 / 89 against 87 (the chip is power bound, so single tiles on a chip that
// is not full run at a higher clock: the second round of 25 tiles costs far less than the first of 256); at 0.3
// dropped and below the plan takes 256-wide tiles of one block row, which the pair list equals (98 against 94 / 180
// against 180).
int g_dx_pairs = 0;         // 0: chosen per call; 1: wherever it applies; 2: never
DxPlan dx_plan(const GemmParams &P, bool fused)
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
    // With a tail the epilogue is the longer the wider the tile, nothing overlaps it, and a 64 x 128
    // sub-tile's accumulators leave the tail's operands no registers: 128-wide tiles (65536 x 4096 x
    // 1024, 128-wide blocks, half dropped: producer with bias and ReLU 528 against 377 us, ReLU-gated dX
    // 615 against 439, GELU forms 735 against 460-490; 32768 x 4096 x 512, 64-wide blocks: 213 against
    // 142, 227 against 163, 300-310 against 190-200; no difference where the per-tile kernels run).
    // (Whatever the knob says: the 256-wide kernels are not compiled with a tail.)
    if (has_tail(P)) plan.TN = 128;
    const int G_ = plan.TN / P.BK;
    plan.persistent = P.BM == 128 && (G_ == 1 || kept / G_ >= (double)g_dx_persistent_groups_per_cu * ncu);
    plan.pairs = false;
    const bool pairs_apply = units_apply(P.MB, P.KB, P.BM, P.BK) && P.N % TK == 0 && !has_tail(P) &&
                             P.lda == P.ldb && !P.kept_given && g_dx_tile_width == 0;
    if (pairs_apply && g_dx_pairs != 2) {
        // in place of single-block tiles that would fill the chip; on its own also only where the tiles of two are
        // expected to finish first (the kept count taken a standard deviation high: one tile more than the CUs can
        // hold at once is a whole extra round), or where there are rounds enough for that not to matter
        const double units_hi = kept / 2 + 2 + sqrt((double)P.MB * P.KB * P.p * (1.0 - P.p)) / 2;
        const double rounds_pairs = (double)((int64_t)((units_hi + ncu - 1) / ncu));
        const bool fills = plan.TN == 128 && plan.persistent && kept >= 1.5 * ncu && (1.0 - P.p) * P.KB >= 4.0;
        if (g_dx_pairs == 1 || (fills && (fused || rounds_pairs >= 4 || rounds_pairs < rounds(128) * 0.6))) {
            plan.pairs = true;
            plan.TN = 256;
            plan.persistent = true;
        }
    }
    return plan;
}

// Which calls read a weight given as [N,K] in place instead of through a transposed copy: eq. (1) on whole 256-wide
// tile columns (its persistent kernel loads W's rows the way eq. 2 loads its operands), and eq. (3) on whole tile
// columns where it runs its persistent kernel (which writes its tiles transposed), and eq. (2) with 128 x 128 blocks
// and whole slices (its persistent kernel on single-block tiles loads W's rows the way eq. 1 does).
bool w_nk_native(int op, int64_t N, int BM, int BK)
{
    if (op == FWD) return N % 256 == 0;
    if (op == DW) return N % 256 == 0;                    // (its persistent kernel's tiles, written transposed; see run)
    if (op == DX) return N % 64 == 0 && BM == 128 && BK == 128;     // (its persistent kernel, one kept block per tile)
    return false;
}

// dW with 64-row tiles: the persistent kernel from 16 expected slices per tile on (see dispatch_tile)
int g_dw64_persistent_slices = 16;
bool dw64_persistent(const GemmParams &P) { return (1.0 - P.p) * P.MB / P.splits * (P.BM / 64) >= (double)g_dw64_persistent_slices; }

namespace {

// 32-bit tile numbers must do (no operand that fits the device's memory comes near this)
bool tile_count_ok(int64_t N, const sdrop_mask_layout_t &L)
{
    const int64_t n_tiles = (N + 255) / 256, lines = L.MB > L.KB ? L.MB : L.KB;
    return lines * n_tiles * 16 <= INT32_MAX;
}

GemmParams base_params(int op, const void *a, const void *b, const void *mask, void *out,
                       int64_t M, int64_t K, int64_t N, int BM, int BK, double p, int out_dtype, const sdrop_mask_layout_t &L)
{
    GemmParams P;
    P.A = static_cast<const char *>(a);
    P.B = static_cast<const char *>(b);
    P.C = static_cast<char *>(out);
    P.mv = make_view(mask, L);
    P.M = M; P.K = K; P.N = N; P.BM = BM; P.BK = BK;
    {
        // contiguous operands: A is X[M,K] (FWD, DW) or dY[M,N] (DX); B is W[K,N] (FWD, DX) or dY[M,N] (DW);
        // C is Y[M,N], dX[M,K] or dW[K,N]
        const int64_t esz_out = out_dtype == SDROP_F32 ? 4 : 2;
        P.lda = (op == DX ? N : K) * 2;
        P.ldb = N * 2;
        P.ldc = (op == DX ? K : N) * esz_out;
    }
    P.MB = (int32_t)L.MB; P.KB = (int32_t)L.KB;
    P.n_tiles = 0;
    P.splits = 1;
    P.total_tiles = 0;
    P.scale = (p < 1.0) ? (float)(1.0 / (1.0 - p)) : 0.0f;
    P.bias = nullptr; P.aux = nullptr; P.act = SDROP_ACT_NONE;
    P.gate_mode = SDROP_GATE_RELU; P.C2 = nullptr;
    P.p = p;
    P.key0 = P.key1 = P.ctr2 = P.ctr3 = 0;
    P.threshold = 0;
    P.p_call = p;
    P.status = device_status_word();
    P.kept_given = false;
    P.w_nk = false;
    return P;
}

// sums the fp32 planes of a split DW into the output (second pass)
int launch_reduce(const void *ws, void *out, int64_t n, int splits, float scale, int dtype, int out_dtype, hipStream_t st,
                  int64_t ncols, int64_t ld, const GemmParams &P)
{
    const MaskHeader *H = P.mv.hdr;
    const int64_t M = P.M, K = P.K;
    const int BM = P.BM, BK = P.BK;
    const double p_call = P.p_call;
    int *const status = P.status;
    const unsigned grid = (unsigned)((n / 8 + 255) / 256);
    const float *part = static_cast<const float *>(ws);
    if (out_dtype == SDROP_F32)
        hipLaunchKernelGGL(reduce_parts_kernel<float>, dim3(grid), dim3(256), 0, st, part, static_cast<float *>(out), n, splits, scale, ncols, ld, H, M, K, BM, BK, p_call, status);
    else if (dtype == SDROP_F16)
        hipLaunchKernelGGL(reduce_parts_kernel<_Float16>, dim3(grid), dim3(256), 0, st, part, static_cast<_Float16 *>(out), n, splits, scale, ncols, ld, H, M, K, BM, BK, p_call, status);
    else
        hipLaunchKernelGGL(reduce_parts_kernel<__bf16>, dim3(grid), dim3(256), 0, st, part, static_cast<__bf16 *>(out), n, splits, scale, ncols, ld, H, M, K, BM, BK, p_call, status);
    return hip_status(hipGetLastError());
}

template <int OP>
int run(const void *a, const void *b, const void *mask, void *out,
        int64_t M, int64_t K, int64_t N, int BM, int BK, double p,
        int dtype, int out_dtype, void *ws, size_t ws_bytes, void *stream,
        const sdrop_epilogue_t *epi = nullptr, void *out2 = nullptr)
{
    const int rc = check_gemm_args(a, b, mask, out, M, K, N, BM, BK, p, dtype, out_dtype);
    if (rc != SDROP_OK) return rc;
    if (epi) {
        if (epi->scale_mode != SDROP_SCALE_DROPOUT && epi->scale_mode != SDROP_SCALE_ONE) return SDROP_EINVAL;
        if (epi->act < SDROP_ACT_NONE || epi->act > SDROP_ACT_GELU_ERF) return SDROP_EINVAL;
        if (epi->gate_mode < SDROP_GATE_RELU || epi->gate_mode > SDROP_GATE_GELU_ERF) return SDROP_EINVAL;
        if (epi->w_layout != SDROP_W_KN && epi->w_layout != SDROP_W_NK) return SDROP_EINVAL;
        if (!(epi->kept_fraction >= 0.0 && epi->kept_fraction <= 1.0)) return SDROP_EINVAL;
        // the gradient of the weights takes a scale only
        if (OP == DW && (epi->act != SDROP_ACT_NONE || epi->bias || epi->relu_mask)) return SDROP_EINVAL;
        if ((reinterpret_cast<uintptr_t>(epi->bias) | reinterpret_cast<uintptr_t>(epi->relu_mask)) % 16) return SDROP_EALIGN;
        // leading dimensions: 0 = contiguous; else at least the row length, rows 16-byte aligned, lane offsets 32-bit
        const bool nk = epi->w_layout == SDROP_W_NK;        // the weight (FWD, DX: second operand; DW: the output) as [N,K]
        const int64_t cols_a = OP == DX ? N : K, cols_b = (nk && OP != DW) ? K : N, cols_c = OP == DX ? K : (nk && OP == DW) ? K : N;
        const int64_t lds[3] = {epi->ld_a, epi->ld_b, epi->ld_out}, cols[3] = {cols_a, cols_b, cols_c};
        for (int i = 0; i < 3; ++i)
            if (lds[i] != 0 && (lds[i] < cols[i] || lds[i] % 8 || lds[i] > (int64_t(1) << 24))) return SDROP_ESHAPE;
    }
    if (out2 && reinterpret_cast<uintptr_t>(out2) % 16) return SDROP_EALIGN;
    const bool w_nk = epi && epi->w_layout == SDROP_W_NK;
    const size_t ws_planes = ws_planes_bytes(OP, M, K, N, BM, BK);
    const size_t ws_need = ws_total_bytes(OP, M, K, N, BM, BK, out_dtype, w_nk);
    if (ws_bytes < ws_need || (ws_need && (!ws || reinterpret_cast<uintptr_t>(ws) % 16))) return SDROP_EWORKSPACE;
    sdrop_mask_layout_t L;
    sdrop_mask_layout(M, K, BM, BK, &L);
    if (!tile_count_ok(N, L)) return SDROP_ESHAPE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    // A weight in the [N,K] layout: the kernels read W as [K,N] (eq. 1 walks its row blocks, eq. 2 its rows), so the
    // weight is transposed into the workspace first (one pass over K N elements; at 4096 x 4096 about 15 us beside a
    // product of 60), and eq. 3 writes its [K,N] result there and transposes it into the output afterwards.
    char *const ws_kn = static_cast<char *>(ws) + ws_planes;       // the K x N matrix behind the planes
    const int64_t esz_out = out_dtype == SDROP_F32 ? 4 : 2;
    void *final_out = out;
    int64_t final_ld = 0;
    // ... unless the call is one whose kernel has a form that reads (writes) the [N,K] array in place
    const bool has_tail_args = epi && (epi->act != SDROP_ACT_NONE || epi->bias || epi->relu_mask);
    bool nk_native = w_nk && !out2 && !has_tail_args && w_nk_native(OP, N, BM, BK);
    if (OP == DW && nk_native && BK == 64) {
        // 64-row tiles: only where the call takes the persistent kernel (see dw64_persistent)
        GemmParams Q = base_params(OP, a, b, mask, out, M, K, N, BM, BK, p, out_dtype, L);
        if (epi->kept_fraction > 0.0) Q.p = 1.0 - (epi->kept_fraction < 1.0 ? epi->kept_fraction : 1.0);
        Q.splits = dw_splits(M, N, BM, BK, K);
        nk_native = dw64_persistent(Q);
    }
    if (OP == DX && nk_native) {
        // eq. 2's in-place form computes one kept block per tile.  Where the [K,N] plan would take 256-wide tiles of
        // one block row (many tiles per CU: 65536 x 4096 x 1024, 431 us through the transposed copy against 450 in
        // place), the copy is the cheaper way; where it takes single blocks or the pair list (4096^3: 74 us in place
        // against 63 + 15), it is not.
        GemmParams Q = base_params(OP, a, b, mask, out, M, K, N, BM, BK, p, out_dtype, L);
        if (epi->kept_fraction > 0.0) { Q.p = 1.0 - (epi->kept_fraction < 1.0 ? epi->kept_fraction : 1.0); Q.kept_given = true; }
        const DxPlan plan = dx_plan(Q);
        if (plan.TN == 256 && !plan.pairs) nk_native = false;
    }
    if (w_nk && !nk_native) {
        if constexpr (OP == DW) {
            final_ld = epi->ld_out ? epi->ld_out : K;
            out = ws_kn;
        } else {
            const int rt = launch_transpose(b, ws_kn, N, K, epi->ld_b ? epi->ld_b : K, N, 2, st);
            if (rt != SDROP_OK) return rt;
            b = ws_kn;
        }
    }
    GemmParams P = base_params(OP, a, b, mask, out, M, K, N, BM, BK, p, out_dtype, L);
    if (epi) {
        if (epi->ld_a) P.lda = epi->ld_a * 2;
        if (epi->ld_b && !(w_nk && OP != DW)) P.ldb = epi->ld_b * 2;
        if (nk_native && OP != DW) { P.ldb = (epi->ld_b ? epi->ld_b : K) * 2; P.w_nk = true; }
        if (epi->ld_out && !(w_nk && OP == DW)) P.ldc = epi->ld_out * (out_dtype == SDROP_F32 ? 4 : 2);
        if (nk_native && OP == DW) { P.ldc = (epi->ld_out ? epi->ld_out : K) * (out_dtype == SDROP_F32 ? 4 : 2); P.w_nk = true; }
        if (epi->scale_mode == SDROP_SCALE_ONE) P.scale = 1.0f;
        // the kernel choice goes by the expected share of kept blocks: the caller's figure where given (a mask built
        // from the caller's own bits need not have the density 1 - p), else 1 - p
        if (epi->kept_fraction > 0.0) { P.p = 1.0 - (epi->kept_fraction < 1.0 ? epi->kept_fraction : 1.0); P.kept_given = true; }
        P.bias = epi->bias;
        P.aux = static_cast<const char *>(epi->relu_mask);
        P.act = epi->act;
        P.gate_mode = epi->gate_mode;
    }
    if (out2) P.C2 = static_cast<char *>(out2);
    if constexpr (OP == DW) {
        P.splits = dw_splits(M, N, BM, BK, K);
        if (P.splits > 1) {
            // first pass: unscaled fp32 partial planes into the workspace; second pass: sum, scale, round
            const float scale = P.scale;
            const int64_t ld_out = P.ldc / (out_dtype == SDROP_F32 ? 4 : 2);
            P.C = static_cast<char *>(ws);
            P.ldc = (nk_native ? K : N) * 4;            // the planes of partial sums are contiguous fp32, [K][N] or [N][K]
            P.scale = 1.0f;
            const int rc1 = (dtype == SDROP_F16) ? dispatch_typed<F16>(OP, true, P, st) : dispatch_typed<BF16>(OP, true, P, st);
            if (rc1 != SDROP_OK) return rc1;
            const int rc2 = launch_reduce(ws, out, K * N, P.splits, scale, dtype, out_dtype, st, nk_native ? K : N, ld_out, P);
            if (rc2 != SDROP_OK || !(w_nk && !nk_native)) return rc2;
            return launch_transpose(out, final_out, K, N, N, final_ld, (int)esz_out, st);
        }
    }
    const bool o32 = out_dtype == SDROP_F32;
    const int rcg = dtype == SDROP_F16 ? dispatch_typed<F16>(OP, o32, P, st) : dispatch_typed<BF16>(OP, o32, P, st);
    if (rcg != SDROP_OK || !(w_nk && !nk_native && OP == DW)) return rcg;
    return launch_transpose(out, final_out, K, N, N, final_ld, (int)esz_out, st);
}

// The mask and the forward product in one launch (fwd_seeded_kernel) where the block grid is small enough for every
// workgroup to draw it and keep it in registers: at most 128 block rows and 64 block columns (a workgroup draws 512
// blocks in 0.11 us, so the largest such grid costs it under 2 us).  Anything else is sdrop_mask followed by sdrop_fwd.
int g_fwd_seeded = 1;

bool fwd_seeded_applies(const sdrop_mask_layout_t &L)
{
    return g_fwd_seeded && L.MB <= 128 && L.KB <= 64;
}

// epi: null, or the weight layout and the leading dimensions of X, W and Y (nothing else of it may be set)
int run_fwd_seeded(const void *x, const void *w, void *mask, size_t mask_bytes, void *y,
                   int64_t M, int64_t K, int64_t N, int BM, int BK, double p, uint64_t seed, uint64_t rng_stream,
                   int dtype, int out_dtype, void *stream, const sdrop_epilogue_t *epi = nullptr, void *ws = nullptr, size_t ws_bytes = 0)
{
    // every argument check of both calls before anything is enqueued
    const int rc = check_gemm_args(x, w, mask, y, M, K, N, BM, BK, p, dtype, out_dtype);
    if (rc != SDROP_OK) return rc;
    sdrop_mask_layout_t L;
    sdrop_mask_layout(M, K, BM, BK, &L);
    if (mask_bytes < L.total_bytes) return SDROP_EWORKSPACE;
    if (!tile_count_ok(N, L)) return SDROP_ESHAPE;
    const bool w_nk = epi && epi->w_layout == SDROP_W_NK;
    if (epi) {
        if (epi->w_layout != SDROP_W_KN && epi->w_layout != SDROP_W_NK) return SDROP_EINVAL;
        if (epi->scale_mode != SDROP_SCALE_DROPOUT || epi->act != SDROP_ACT_NONE || epi->bias || epi->relu_mask ||
            epi->kept_fraction != 0.0) return SDROP_EINVAL;
        const int64_t lds[3] = {epi->ld_a, epi->ld_b, epi->ld_out}, cols[3] = {K, w_nk ? K : N, N};
        for (int i = 0; i < 3; ++i)
            if (lds[i] != 0 && (lds[i] < cols[i] || lds[i] % 8 || lds[i] > (int64_t(1) << 24))) return SDROP_ESHAPE;
        // the workspace of sdrop_fwd_ex with the same layout (used where the [N,K] weight goes through a transposed copy)
        const size_t need = ws_total_bytes(FWD, M, K, N, BM, BK, out_dtype, w_nk);
        if (ws_bytes < need || (need && (!ws || reinterpret_cast<uintptr_t>(ws) % 16))) return SDROP_EWORKSPACE;
    }
    if (fwd_seeded_applies(L) && (!w_nk || w_nk_native(FWD, N, BM, BK))) {
        GemmParams P = base_params(FWD, x, w, mask, y, M, K, N, BM, BK, p, out_dtype, L);
        if (epi) {
            if (epi->ld_a) P.lda = epi->ld_a * 2;
            if (epi->ld_b) P.ldb = epi->ld_b * 2;
            else if (w_nk) P.ldb = K * 2;
            if (epi->ld_out) P.ldc = epi->ld_out * (out_dtype == SDROP_F32 ? 4 : 2);
            P.w_nk = w_nk;
        }
        P.key0 = (uint32_t)seed; P.key1 = (uint32_t)(seed >> 32);
        P.ctr2 = (uint32_t)rng_stream; P.ctr3 = (uint32_t)(rng_stream >> 32);
        P.threshold = (uint64_t)floor(p * 4294967296.0);
        hipStream_t st = static_cast<hipStream_t>(stream);
        const bool o32 = out_dtype == SDROP_F32;
        const int rs = dtype == SDROP_F16 ? fwd_seeded_typed<F16>(o32, P, st) : fwd_seeded_typed<BF16>(o32, P, st);
        if (rs != -1) return rs;        // -1: the device does not grant the LDS; fall through to the two calls
    }
    const int rm = sdrop_mask(mask, mask_bytes, M, K, BM, BK, p, seed, rng_stream, stream);
    if (rm != SDROP_OK) return rm;
    return run<FWD>(x, w, mask, y, M, K, N, BM, BK, p, dtype, out_dtype, ws, ws_bytes, stream, epi);
}

// both gradients in one launch where bwd_fused_kernel or bwd_fused_tile_kernel applies (128 x 128
// blocks, N a multiple of 256); anything else is the two calls in turn
int g_bwd_fused = 1;

// ld: null (contiguous), or the leading dimensions of dY, W, X, dX, dW in elements (0 = contiguous)
// w_layout = SDROP_W_NK: W is given, and dW wanted, as [N,K] (ld[1], ld[4] then count rows of K elements): the two
// products are launched in turn, each in place where its kernel has a form for it (see run).
int run_bwd(const void *dy, const void *w, const void *x, const void *mask, void *dx, void *dw,
            int64_t M, int64_t K, int64_t N, int BM, int BK, double p,
            int dtype, int out_dtype, void *ws, size_t ws_bytes, void *stream, const int64_t *ld = nullptr,
            int w_layout = SDROP_W_KN)
{
    // every argument check of both calls before anything is enqueued
    int rc = check_gemm_args(dy, w, mask, dx, M, K, N, BM, BK, p, dtype, out_dtype);
    if (rc == SDROP_OK) rc = check_gemm_args(x, dy, mask, dw, M, K, N, BM, BK, p, dtype, out_dtype);
    if (rc != SDROP_OK) return rc;
    if (w_layout != SDROP_W_KN && w_layout != SDROP_W_NK) return SDROP_EINVAL;
    if (w_layout == SDROP_W_NK) {
        sdrop_epilogue_t e;
        e.scale_mode = SDROP_SCALE_DROPOUT; e.act = SDROP_ACT_NONE; e.bias = nullptr; e.relu_mask = nullptr;
        e.gate_mode = SDROP_GATE_RELU; e.w_layout = SDROP_W_NK; e.kept_fraction = 0.0;
        // the workspace of the larger of the two calls (eq. 3's: its planes and the transposed copy), checked first
        if (ld)
            for (int i = 0; i < 5; ++i) {
                const int64_t cols = (i == 0) ? N : K;     // dY has N columns; W[N,K], X, dX and dW[N,K] have K
                if (ld[i] != 0 && (ld[i] < cols || ld[i] % 8 || ld[i] > (int64_t(1) << 24))) return SDROP_ESHAPE;
            }
        const size_t need = ws_total_bytes(DW, M, K, N, BM, BK, out_dtype, true);
        if (ws_bytes < need || (need && (!ws || reinterpret_cast<uintptr_t>(ws) % 16))) return SDROP_EWORKSPACE;
        // One launch where both products have their in-place forms (128 x 128 blocks, whole tile columns, eq. 2 on
        // single-block tiles or where its [K,N] plan takes the pair list): the persistent bodies as in bwd_fused_kernel.
        if (g_bwd_fused && BM == 128 && BK == 128 && N % 256 == 0) {
            sdrop_mask_layout_t L;
            sdrop_mask_layout(M, K, BM, BK, &L);
            if (!tile_count_ok(N, L)) return SDROP_ESHAPE;
            GemmParams Pdx = base_params(DX, dy, w, mask, dx, M, K, N, BM, BK, p, out_dtype, L);
            GemmParams Pdw = base_params(DW, x, dy, mask, dw, M, K, N, BM, BK, p, out_dtype, L);
            const DxPlan plan = dx_plan(Pdx);
            if (plan.TN == 128 || plan.pairs) {
                const int64_t esz_out = out_dtype == SDROP_F32 ? 4 : 2;
                const int64_t l0 = ld && ld[0] ? ld[0] : N, l1 = ld && ld[1] ? ld[1] : K, l2 = ld && ld[2] ? ld[2] : K;
                const int64_t l3 = ld && ld[3] ? ld[3] : K, l4 = ld && ld[4] ? ld[4] : K;
                Pdx.lda = l0 * 2; Pdx.ldb = l1 * 2; Pdx.ldc = l3 * esz_out;
                Pdw.lda = l2 * 2; Pdw.ldb = l0 * 2; Pdw.ldc = l4 * esz_out;
                Pdx.w_nk = Pdw.w_nk = true;
                Pdw.splits = dw_splits(M, N, BM, BK, K);
                Pdw.n_tiles = (int)(N / 256);
                Pdw.total_tiles = Pdw.KB * Pdw.n_tiles * Pdw.splits;
                const float scale = Pdw.scale;
                const bool split = Pdw.splits > 1;
                if (split) { Pdw.C = static_cast<char *>(ws); Pdw.ldc = K * 4; Pdw.scale = 1.0f; }
                hipStream_t st = static_cast<hipStream_t>(stream);
                const bool o32 = out_dtype == SDROP_F32;
                const int rf = dtype == SDROP_F16 ? bwd_fused_typed<F16>(kBwdPersistent, kTNNK, o32, split, Pdx, Pdw, 0, st)
                                                  : bwd_fused_typed<BF16>(kBwdPersistent, kTNNK, o32, split, Pdx, Pdw, 0, st);
                if (rf != -1) {     // -1: the device does not grant the LDS; the two calls then
                    if (rf != SDROP_OK || !split) return rf;
                    return launch_reduce(ws, dw, K * N, Pdw.splits, scale, dtype, out_dtype, st, K, l4, Pdw);
                }
            }
        }
        e.ld_a = ld ? ld[0] : 0; e.ld_b = ld ? ld[1] : 0; e.ld_out = ld ? ld[3] : 0;
        rc = run<DX>(dy, w, mask, dx, M, K, N, BM, BK, p, dtype, out_dtype, ws, ws_bytes, stream, &e);
        if (rc != SDROP_OK) return rc;
        e.ld_a = ld ? ld[2] : 0; e.ld_b = ld ? ld[0] : 0; e.ld_out = ld ? ld[4] : 0;
        return run<DW>(x, dy, mask, dw, M, K, N, BM, BK, p, dtype, out_dtype, ws, ws_bytes, stream, &e);
    }
    int64_t lds[5] = {N, N, K, K, N};                    // dY[M,N], W[K,N], X[M,K], dX[M,K], dW[K,N]
    if (ld) {
        for (int i = 0; i < 5; ++i) {
            if (ld[i] != 0 && (ld[i] < lds[i] || ld[i] % 8 || ld[i] > (int64_t(1) << 24))) return SDROP_ESHAPE;
            if (ld[i]) lds[i] = ld[i];
        }
    }
    const size_t ws_need = sdrop_workspace_bytes(SDROP_OP_BWD_DW, M, K, N, BM, BK, dtype, out_dtype);
    if (ws_bytes < ws_need || (ws_need && (!ws || reinterpret_cast<uintptr_t>(ws) % 16))) return SDROP_EWORKSPACE;
    sdrop_mask_layout_t L;
    sdrop_mask_layout(M, K, BM, BK, &L);
    if (!tile_count_ok(N, L)) return SDROP_ESHAPE;
    hipStream_t st = static_cast<hipStream_t>(stream);

    GemmParams Pdx = base_params(DX, dy, w, mask, dx, M, K, N, BM, BK, p, out_dtype, L);
    GemmParams Pdw = base_params(DW, x, dy, mask, dw, M, K, N, BM, BK, p, out_dtype, L);
    {
        const int64_t esz_out = out_dtype == SDROP_F32 ? 4 : 2;
        Pdx.lda = lds[0] * 2; Pdx.ldb = lds[1] * 2; Pdx.ldc = lds[3] * esz_out;
        Pdw.lda = lds[2] * 2; Pdw.ldb = lds[0] * 2; Pdw.ldc = lds[4] * esz_out;
    }
    const DxPlan plan = dx_plan(Pdx, g_bwd_fused && N % 256 == 0 && BM == 128 && BK == 128);
    Pdw.splits = dw_splits(M, N, BM, BK, K);
    // Which single launch applies, if any (all need N to be a multiple of 256, so that neither product has a ragged edge):
    //   persistent dX + persistent dW                      128 x 128 blocks, dX on its persistent kernel
    //   dX a workgroup per tile of two blocks + persistent dW   128 x 128 blocks otherwise
    //   both a workgroup per tile                          64 x 64 blocks, dW with short kept lists
    int form = kBwdNone;
    if (g_bwd_fused && N % 256 == 0) {
        if (BM == 128 && BK == 128) form = plan.persistent ? kBwdPersistent : (plan.TN == 256 ? kBwdTile128 : kBwdNone);
        else if (BM == 64 && BK == 64 && !dw64_persistent(Pdw)) form = kBwdTile64;
    }
    if (form != kBwdNone) {
        const int G_ = plan.TN / BK;
        Pdx.n_tiles = (Pdx.KB + G_ - 1) / G_;
        const int n_dx = Pdx.MB * Pdx.n_tiles;           // the per-tile launch's grid: (group of the row, block row)
        Pdw.n_tiles = (int)(N / 256);
        Pdw.total_tiles = Pdw.KB * Pdw.n_tiles * Pdw.splits;
        const float scale = Pdw.scale;
        const bool split = Pdw.splits > 1;
        if (split) { Pdw.C = static_cast<char *>(ws); Pdw.ldc = N * 4; Pdw.scale = 1.0f; }
        const bool o32 = out_dtype == SDROP_F32;
        const int tn = plan.pairs ? kTNPairs : plan.TN;
        const int rf = dtype == SDROP_F16 ? bwd_fused_typed<F16>(form, tn, o32, split, Pdx, Pdw, n_dx, st)
                                          : bwd_fused_typed<BF16>(form, tn, o32, split, Pdx, Pdw, n_dx, st);
        if (rf != -1) {     // -1: the device does not grant the LDS; fall through to the two calls
            if (rf != SDROP_OK || !split) return rf;
            return launch_reduce(ws, dw, K * N, Pdw.splits, scale, dtype, out_dtype, st, N, lds[4], Pdw);
        }
    }
    sdrop_epilogue_t e;
    e.scale_mode = SDROP_SCALE_DROPOUT; e.act = SDROP_ACT_NONE; e.bias = nullptr; e.relu_mask = nullptr;
    e.gate_mode = SDROP_GATE_RELU; e.w_layout = SDROP_W_KN; e.kept_fraction = 0.0;
    e.ld_a = lds[0]; e.ld_b = lds[1]; e.ld_out = lds[3];
    rc = run<DX>(dy, w, mask, dx, M, K, N, BM, BK, p, dtype, out_dtype, nullptr, 0, stream, ld ? &e : nullptr);
    if (rc != SDROP_OK) return rc;
    e.ld_a = lds[2]; e.ld_b = lds[0]; e.ld_out = lds[4];
    return run<DW>(x, dy, mask, dw, M, K, N, BM, BK, p, dtype, out_dtype, ws, ws_bytes, stream, ld ? &e : nullptr);
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

// ---- device memory that belongs to the library: the planes of a split dW for sdrop_bwd_dw_static ----
// One copy per GPU, part of the code object's zero-initialised data, there from the moment the library
// is loaded on a device until the process ends.  In host code the array's name is only a handle: its
// device address is asked for once per device (with that device current) and kept.
constexpr size_t kStaticScratchBytes = SDROP_STATIC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
static std::atomic<void *> g_scratch_ptr[kMaxDevices];

// The status word: kernels that find a mask object that does not belong to their call record it here (one word per
// GPU, part of the code object like `scratch`; its device address is looked up once per device).
static __device__ int status_word;
static std::atomic<int *> g_status_ptr[kMaxDevices];

int *device_status_word()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    int *p = g_status_ptr[dev].load(std::memory_order_acquire);
    if (p) return p;
    void *v = nullptr;
    if (hipGetSymbolAddress(&v, HIP_SYMBOL(status_word)) != hipSuccess || !v) { (void)hipGetLastError(); return nullptr; }
    g_status_ptr[dev].store(static_cast<int *>(v), std::memory_order_release);
    return static_cast<int *>(v);
}

// The current device's copy of `scratch`, or null with the HIP error recorded.
void *static_scratch()
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess && (dev < 0 || dev >= kMaxDevices)) e = hipErrorInvalidDevice;
    if (e != hipSuccess) { hip_status(e); return nullptr; }
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (p) return p;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) { hip_status(e != hipSuccess ? e : hipErrorInvalidSymbol); return nullptr; }
    g_scratch_ptr[dev].store(p, std::memory_order_release);     // every thread that asks gets the same address
    return p;
}

}  // namespace sdrop


extern "C" {

int sdrop_status(int *flags_host, int clear, void *stream)
{
    if (!flags_host) return SDROP_EINVAL;
    int *const word = sdrop::device_status_word();
    if (!word) return SDROP_EHIP;
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t e = hipMemcpyAsync(flags_host, word, sizeof(int), hipMemcpyDeviceToHost, st);
    if (e == hipSuccess && clear) e = hipMemsetAsync(word, 0, sizeof(int), st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    return sdrop::hip_status(e);
}

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
    if (knob == SDROP_TUNE_FWD_SEEDED && (value == 0 || value == 1)) {
        sdrop::g_fwd_seeded = value;
        return SDROP_OK;
    }
    if (knob == SDROP_TUNE_DX_PAIRS && value >= 0 && value <= 2) {
        sdrop::g_dx_pairs = value;
        return SDROP_OK;
    }
    if (knob == SDROP_TUNE_DW64_PERSISTENT_SLICES && value >= 0) {
        sdrop::g_dw64_persistent_slices = value;
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
    return sdrop::ws_planes_bytes(op, M, K, N, BM, BK);
}

size_t sdrop_workspace_bytes_ex(int op, int64_t M, int64_t K, int64_t N, int BM, int BK,
                                int dtype, int out_dtype, const sdrop_epilogue_t *epi)
{
    (void)dtype;
    if (op != SDROP_OP_FWD && op != SDROP_OP_BWD_DX && op != SDROP_OP_BWD_DW) return 0;
    if (M <= 0 || K <= 0 || N <= 0 || !sdrop::block_size_ok(BM) || !sdrop::block_size_ok(BK) || M % BM || K % BK) return 0;
    return sdrop::ws_total_bytes(op, M, K, N, BM, BK, out_dtype, epi && epi->w_layout == SDROP_W_NK);
}

int sdrop_fwd(const void *X, const void *W, const void *mask, void *Y,
              int64_t M, int64_t K, int64_t N, int BM, int BK, double p,
              int dtype, int out_dtype, void *ws, size_t ws_bytes, void *stream)
{
    return sdrop::run<sdrop::FWD>(X, W, mask, Y, M, K, N, BM, BK, p, dtype, out_dtype, ws, ws_bytes, stream);
}

int sdrop_fwd_seeded(const void *X, const void *W, void *mask, size_t mask_bytes, void *Y,
                     int64_t M, int64_t K, int64_t N, int BM, int BK, double p, uint64_t seed, uint64_t rng_stream,
                     int dtype, int out_dtype, void *stream)
{
    return sdrop::run_fwd_seeded(X, W, mask, mask_bytes, Y, M, K, N, BM, BK, p, seed, rng_stream, dtype, out_dtype, stream);
}

int sdrop_fwd_seeded_ex(const void *X, const void *W, void *mask, size_t mask_bytes, void *Y,
                        int64_t M, int64_t K, int64_t N, int BM, int BK, double p, uint64_t seed, uint64_t rng_stream,
                        int dtype, int out_dtype, void *ws, size_t ws_bytes, void *stream, const sdrop_epilogue_t *epi)
{
    return sdrop::run_fwd_seeded(X, W, mask, mask_bytes, Y, M, K, N, BM, BK, p, seed, rng_stream, dtype, out_dtype, stream,
                                 epi, ws, ws_bytes);
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

int sdrop_bwd_dw_static(const void *X, const void *dY, const void *mask, void *dW,
                        int64_t M, int64_t K, int64_t N, int BM, int BK, double p,
                        int dtype, int out_dtype, void *stream)
{
    // argument errors first, as in sdrop_bwd_dw; then the size against the library's own memory
    const int rc = sdrop::check_gemm_args(X, dY, mask, dW, M, K, N, BM, BK, p, dtype, out_dtype);
    if (rc != SDROP_OK) return rc;
    const size_t need = sdrop_workspace_bytes(SDROP_OP_BWD_DW, M, K, N, BM, BK, dtype, out_dtype);
    if (need > sdrop::kStaticScratchBytes) return SDROP_EWORKSPACE;
    void *ws = nullptr;
    if (need) {
        ws = sdrop::static_scratch();
        if (!ws) return SDROP_EHIP;
    }
    return sdrop::run<sdrop::DW>(X, dY, mask, dW, M, K, N, BM, BK, p, dtype, out_dtype, ws, need, stream);
}

int sdrop_bwd(const void *dY, const void *W, const void *X, const void *mask, void *dX, void *dW,
              int64_t M, int64_t K, int64_t N, int BM, int BK, double p,
              int dtype, int out_dtype, void *ws, size_t ws_bytes, void *stream)
{
    return sdrop::run_bwd(dY, W, X, mask, dX, dW, M, K, N, BM, BK, p, dtype, out_dtype, ws, ws_bytes, stream);
}

int sdrop_bwd_ex(const void *dY, const void *W, const void *X, const void *mask, void *dX, void *dW,
                 int64_t M, int64_t K, int64_t N, int BM, int BK, double p,
                 int dtype, int out_dtype, void *ws, size_t ws_bytes, void *stream,
                 int64_t ld_dy, int64_t ld_w, int64_t ld_x, int64_t ld_dx, int64_t ld_dw, int w_layout)
{
    const int64_t ld[5] = {ld_dy, ld_w, ld_x, ld_dx, ld_dw};
    return sdrop::run_bwd(dY, W, X, mask, dX, dW, M, K, N, BM, BK, p, dtype, out_dtype, ws, ws_bytes, stream, ld, w_layout);
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

int sdrop_producer(const void *H, const void *W0, const float *bias, const void *mask, void *X, void *Z,
                   int64_t M, int64_t N0, int64_t K, int BM, int BK, double p, int act,
                   int dtype, int out_dtype, void *stream)
{
    sdrop_epilogue_t epi;
    epi.scale_mode = SDROP_SCALE_ONE;
    epi.act = act;
    epi.bias = bias;
    epi.relu_mask = nullptr;
    epi.ld_a = epi.ld_b = epi.ld_out = 0;
    epi.gate_mode = SDROP_GATE_RELU;
    epi.w_layout = SDROP_W_KN;
    epi.kept_fraction = 0.0;
    return sdrop::run<sdrop::DX>(H, W0, mask, X, M, K, N0, BM, BK, p, dtype, out_dtype, nullptr, 0, stream, &epi, Z);
}

int sdrop_producer_ex(const void *H, const void *W0, const float *bias, const void *mask, void *X, void *Z,
                      int64_t M, int64_t N0, int64_t K, int BM, int BK, double p, int act,
                      int dtype, int out_dtype, void *stream, int64_t ld_h, int64_t ld_w0, int64_t ld_out)
{
    sdrop_epilogue_t epi;
    epi.scale_mode = SDROP_SCALE_ONE;
    epi.act = act;
    epi.bias = bias;
    epi.relu_mask = nullptr;
    epi.ld_a = ld_h; epi.ld_b = ld_w0; epi.ld_out = ld_out;
    epi.gate_mode = SDROP_GATE_RELU;
    epi.w_layout = SDROP_W_KN;
    epi.kept_fraction = 0.0;
    return sdrop::run<sdrop::DX>(H, W0, mask, X, M, K, N0, BM, BK, p, dtype, out_dtype, nullptr, 0, stream, &epi, Z);
}

}  // extern "C"
