// The one-launch-per-tile form of the three block-sparse GEMMs (included by the typed GEMM translation units only; the design notes are
// at the top of that file).
#ifndef SDROP_GEMM_TILE_KERNEL_H
#define SDROP_GEMM_TILE_KERNEL_H
#include "gemm_device_common.h"

namespace sdrop {
namespace {

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

    // a kernel handed a mask built for another problem writes nothing
    const MaskHeader *H = P.mv.hdr;
    if (!mask_header_ok(H, P.M, P.K, P.BM, P.BK, true, P.p_call, P.status)) return;

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
        lda = P.lda; ldb = P.ldb; ldc = P.ldc;
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
        lda = P.lda; ldb = P.ldb; ldc = P.ldc;
        a_tile = P.A + (int64_t)j * P.BK * esz;
        b_tile = P.B + (int64_t)nt * TN * esz;
        // with a split list, part `part` writes its own K x N plane of partial sums
        c_tile = P.C + (int64_t)part * P.K * ldc + (int64_t)j * P.BK * ldc + (int64_t)nt * TN * sizeof(OutT);
        { const int64_t left = P.N - (int64_t)nt * TN; c_lim = left < TN ? (int)left : TN; }
    } else {
        const int G_ = TN / P.BK;                     // kept blocks gathered into one tile
        lda = P.lda; ldb = P.ldb; ldc = P.ldc;
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
        // Parks the sub-tile in LDS with tail tl applied and writes it out `delta` bytes from its place in C.
        // mode_c (a TailMode constant) says which tail this copy of the code is for: a copy holds one
        // activation's or one gate's arithmetic only, and the tail's operands are requested in batches
        // ahead of their arithmetic instead of one load, one wait per register quad.
        auto emit_mode = [&](auto mode_c, const Tail &tl, int64_t delta) __attribute__((always_inline)) {
            constexpr int MODE = decltype(mode_c)::value;
            constexpr bool TL = TAIL && OP != DW && MODE != kTailNone;
            // global column of register quad (ni, q) of this lane; false if it lies outside the output
            auto quad_col = [&](int ni, int q, int64_t &gcol) __attribute__((always_inline)) -> bool {
                const int cl = wn * WTN + ni * 32 + q * 8 + (lane >> 5) * 4;          // column within the tile
                if constexpr (OP == DX) {
                    const int g = cl >> 6;
                    int c0 = out_col0[0];
#pragma unroll
                    for (int gg = 1; gg < DXG; ++gg) c0 = (g == gg) ? out_col0[gg] : c0;
                    gcol = c0 + (cl & 63);
                    return g < chunks_valid;
                } else {
                    gcol = out_col0[0] + cl;
                    return cl < c_lim;                      // c_lim is a multiple of 8
                }
            };
            using E16 = typename In<T>::out16;
            typedef __attribute__((__vector_size__(4 * sizeof(E16)))) E16 e16x4;
            // Batch of the tail's operand requests: the register quads of NB 32-column blocks of one
            // 32-row block.  A wavefront with 128 accumulator registers takes one block at a time
            // (all four at once measured 182 -> 204 us on its ragged dX kernel), smaller ones all.
            constexpr int NB = MI * NI * 16 >= 128 ? 1 : NI;
            const bool has_bias = TL && tl.bias != nullptr;
            const bool gated = MODE == kTailReluGate || MODE == kTailGeluErfGate || (MODE == kTailGeneric && tl.aux != nullptr);
            const int gate_mode = MODE == kTailGeneric ? tl.gate_mode : MODE == kTailGeluErfGate ? SDROP_GATE_GELU_ERF : SDROP_GATE_RELU;
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int nb = 0; nb < NI; nb += NB) {
                const int row = mi * 32 + (lane & 31);
                f32x4 bias_v[NB * 4];
                e16x4 gate_v[NB * 4];
                if constexpr (TL) {
                    if (has_bias) {
#pragma unroll
                        for (int i = 0; i < NB * 4; ++i) {
                            int64_t gcol;
                            const bool ok = quad_col(nb + (i >> 2), i & 3, gcol);
                            bias_v[i] = ok ? *(const_f4)(uintptr_t)(tl.bias + gcol) : f32x4{0.f, 0.f, 0.f, 0.f};
                        }
                    }
                    if (gated) {
#pragma unroll
                        for (int i = 0; i < NB * 4; ++i) {
                            int64_t gcol;
                            const bool ok = quad_col(nb + (i >> 2), i & 3, gcol);
                            const int64_t elem = (out_row0 + wm * WTM + row) * (ldc / ESZ) + gcol;
                            gate_v[i] = ok ? *reinterpret_cast<const e16x4 *>(tl.aux + elem * (int64_t)sizeof(E16)) : e16x4{};
                        }
                    }
                }
#pragma unroll
                for (int ni = nb; ni < nb + NB; ++ni)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int col = ni * 32 + q * 8 + (lane >> 5) * 4;
                        float v[4] = {acc[mi][ni][4 * q] * scale, acc[mi][ni][4 * q + 1] * scale,
                                      acc[mi][ni][4 * q + 2] * scale, acc[mi][ni][4 * q + 3] * scale};
                        if constexpr (TL) {
                            // (lanes outside the output compute on zeros; their values are not stored)
                            if (has_bias) {
                                const f32x4 b = bias_v[(ni - nb) * 4 + q];
                                v[0] += b.x; v[1] += b.y; v[2] += b.z; v[3] += b.w;
                            }
                            if constexpr (MODE == kTailLight) {
                                if (tl.act == SDROP_ACT_RELU) act4(SDROP_ACT_RELU, v);
                            } else if constexpr (MODE == kTailGeluErf) {
                                act4(SDROP_ACT_GELU_ERF, v);
                            } else if constexpr (MODE == kTailGeneric) {
                                act4(tl.act, v);
                            }
                            if (gated) {
                                const e16x4 x = gate_v[(ni - nb) * 4 + q];
                                const float xf[4] = {static_cast<float>(x[0]), static_cast<float>(x[1]), static_cast<float>(x[2]), static_cast<float>(x[3])};
                                gate4(gate_mode, v, xf);
                            }
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
            if (ok) store_out(cbase + delta + (int64_t)(wm * WTM + row) * ldc + col * ESZ, v);
        }
        };
        // the tail's kind is branched on once (uniform), here at the end of the kernel
        auto emit = [&](const Tail &tl, int64_t delta) __attribute__((always_inline)) {
            if constexpr (!(TAIL && OP != DW)) {
                emit_mode(std::integral_constant<int, kTailNone>{}, tl, delta);
            } else if (tl.aux == nullptr) {
                if (tl.act == SDROP_ACT_NONE || tl.act == SDROP_ACT_RELU) emit_mode(std::integral_constant<int, kTailLight>{}, tl, delta);
                else if (tl.act == SDROP_ACT_GELU_ERF) emit_mode(std::integral_constant<int, kTailGeluErf>{}, tl, delta);
                else emit_mode(std::integral_constant<int, kTailGeneric>{}, tl, delta);
            } else if (tl.act == SDROP_ACT_NONE && tl.gate_mode == SDROP_GATE_RELU) {
                emit_mode(std::integral_constant<int, kTailReluGate>{}, tl, delta);
            } else if (tl.act == SDROP_ACT_NONE && tl.gate_mode == SDROP_GATE_GELU_ERF) {
                emit_mode(std::integral_constant<int, kTailGeluErfGate>{}, tl, delta);
            } else {
                emit_mode(std::integral_constant<int, kTailGeneric>{}, tl, delta);
            }
        };
        if constexpr (TAIL && OP == DX) {
            // the producing layer's value before the activation, to the second output
            if (P.C2) emit_mode(std::integral_constant<int, kTailLight>{}, make_tail_preact(P), P.C2 - P.C);
        }
        emit(make_tail(P), 0);
    }
}

template <int OP, class T, class OutT, int TM, int TN, int WM, int WN, bool RAGGED, bool SPEC, bool TAIL>
__global__ __launch_bounds__(WM * WN * 64 * (SPEC ? 2 : 1)) void gemm_kernel(GemmParams P)
{
    gemm_tile_body<OP, T, OutT, TM, TN, WM, WN, RAGGED, SPEC, TAIL>(P, (int)blockIdx.x);
}

}  // namespace
}  // namespace sdrop
#endif
