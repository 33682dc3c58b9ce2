// Block-mask draw and index-list compaction for SparseDrop (arxiv 2411.01238,
// Sections 3.2 and 3.4), plus the small host-side pieces of the C ABI that are
// not GEMMs (layout, error text).
//
// Two launches.  (1) The draw: one wavefront per 64 blocks of a block row (lane <-> block
// column), spread over the whole chip because ten Philox rounds per block are integer-multiply
// bound; the 64-lane ballot of the keep decisions IS the packed 64-bit mask word of
// Section 3.4.  (2) The lists: one 1024-thread workgroup turns the words into every index
// list.  The largest mask here has 16384 blocks, so this part is latency, not throughput,
// and a single workgroup needs no cross-workgroup scan: a wavefront owns a block row,
// popcount(word & lanes-below) is the position of a kept block inside its row's list, row
// totals become row_ptr by a workgroup prefix scan, and the column lists (what eq. 3 walks)
// are built the same way with lane <-> block row.
#include "sdrop_internal.h"
#include <math.h>

namespace sdrop {

static thread_local int g_last_hip_error = 0;

int hip_status(hipError_t e)
{
    if (e == hipSuccess) return SDROP_OK;
    g_last_hip_error = static_cast<int>(e);
    return SDROP_EHIP;
}

namespace {

constexpr int kMaskThreads = 1024;
constexpr int kMaskWaves = kMaskThreads / 64;
constexpr int kMaxBins = 4096;   // histogram bins of the descending-count sort

struct MaskParams {
    MaskHeader *hdr;
    uint64_t *bits;
    int32_t *row_ptr, *col_idx, *blk_row, *col_ptr, *row_idx, *row_order, *col_order, *loc_row, *loc_col, *units;
    const uint64_t *given_bits;      // non-null: take the bits from here instead of drawing
    int64_t M, K;
    int32_t BM, BK, MB, KB, wpr;
    int32_t split_m, split_k, KBL;   // block splitting: logical block = split_m x split_k blocks; logical columns
    uint32_t key0, key1, ctr2, ctr3; // seed and rng_stream split in 32-bit words
    uint64_t threshold;              // floor(p * 2^32)
    double p;                        // as given (recorded in the header)
    uint64_t seed, rng_stream;
};

// Number of the logical block that decides block (i, j): with block splitting (Section 3.3) the
// logical grid is (MB / split_m) x KBL and every logical entry is repeated split_m times along M
// and split_k times along K; without it this is i * KB + j.
__device__ __forceinline__ uint64_t logical_block(const MaskParams &P, int64_t i, int j)
{
    // without splitting: i * KB + j, below 2^26 (see sdrop_mask_layout), both factors below 2^24: one full-rate multiply
    // (the divisions below cost as much as half the generator's rounds)
    if (P.split_m == 1 && P.split_k == 1) return (uint64_t)(__umul24((uint32_t)i, (uint32_t)P.KB) + (uint32_t)j);
    // block rows and columns are below 2^31: 32-bit divisions (a 64-bit one costs several times as much)
    return (uint64_t)((uint32_t)i / (uint32_t)P.split_m) * (uint64_t)P.KBL + (uint64_t)((uint32_t)j / (uint32_t)P.split_k);
}

__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }
__device__ __forceinline__ int wave_id() { return threadIdx.x >> 6; }

__device__ __forceinline__ uint64_t lanes_below()
{
    return (uint64_t(1) << lane_id()) - 1;
}

// In-place inclusive prefix sum of a[0..n) by the whole workgroup.  `a` may be in
// LDS or in global memory written earlier by this same workgroup.
__device__ void block_inclusive_scan(int32_t *a, int n, int32_t *wave_tot /* LDS[kMaskWaves+1] */)
{
    int carry = 0;
    for (int base = 0; base < n; base += kMaskThreads) {
        const int idx = base + threadIdx.x;
        int v = (idx < n) ? a[idx] : 0;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int up = __shfl_up(v, d, 64);
            if (lane_id() >= d) v += up;
        }
        if (lane_id() == 63) wave_tot[wave_id()] = v;
        __syncthreads();
        int before = 0, total = 0;
        for (int w = 0; w < kMaskWaves; ++w) {
            const int t = wave_tot[w];
            if (w < wave_id()) before += t;
            total += t;
        }
        if (idx < n) a[idx] = v + before + carry;
        carry += total;
        __syncthreads();
    }
}

// order[] := indices 0..n-1 sorted by descending cnt(i) = ptr[i+1]-ptr[i] (counting
// sort; ties land in unspecified order).  max_cnt is the upper bound of cnt.
__device__ void descending_order(const int32_t *ptr, int n, int max_cnt, int32_t *order,
                                 int32_t *bins /* LDS[kMaxBins+1] */, int32_t *wave_tot,
                                 int32_t *largest /* LDS: receives the largest count */)
{
    if (threadIdx.x == 0) *largest = 0;
    const int nb = (max_cnt < kMaxBins ? max_cnt : kMaxBins) + 1;
    for (int b = threadIdx.x; b < nb; b += kMaskThreads) bins[b] = 0;
    __syncthreads();
    auto bin_of = [&](int cnt) {
        const int b = (max_cnt <= kMaxBins) ? cnt : int((int64_t)cnt * kMaxBins / max_cnt);
        return nb - 1 - b;             // bin 0 holds the largest counts
    };
    for (int i = threadIdx.x; i < n; i += kMaskThreads) {
        const int cnt = ptr[i + 1] - ptr[i];
        atomicAdd(&bins[bin_of(cnt)], 1);
        atomicMax(largest, cnt);
    }
    __syncthreads();
    block_inclusive_scan(bins, nb, wave_tot);
    // bins[b] is now the END of bin b; claim slots from the end backwards
    for (int i = threadIdx.x; i < n; i += kMaskThreads) {
        const int pos = atomicSub(&bins[bin_of(ptr[i + 1] - ptr[i])], 1) - 1;
        order[pos] = i;
    }
    __syncthreads();
}

// The kept blocks sorted by (i / 8, j, i % 8): a wavefront takes a group of 8 block rows, lane <->
// block column.  The group's blocks fill the same range of the list as in row-major order,
// [row_ptr[8g], row_ptr[8g + 8)); inside it a block's place is the number of kept blocks of the
// group in earlier columns (a prefix sum over the lanes) plus those above it in its own column.
// `bits` and `row_ptr` may be in LDS or in global memory written earlier by this workgroup.
// The groups are shared by wavefronts [wave0, wave0 + nw) of the workgroup; the others return at once.
// With several workgroups (wg of nwg) the groups are dealt out over the wavefronts of all of them.
__device__ void local_order(const uint64_t *bits, const int32_t *row_ptr, const MaskParams &P,
                            int wave0 = 0, int nw = kMaskWaves, int wg = 0, int nwg = 1)
{
    const int lane = lane_id();
    const int me = wave_id() - wave0;
    if (me < 0 || me >= nw) return;
    for (int i0 = (wg * nw + me) * 8; i0 < P.MB; i0 += nwg * nw * 8) {
        const int nr = P.MB - i0 < 8 ? P.MB - i0 : 8;
        int pos = row_ptr[i0];
        for (int w = 0; w < P.wpr; ++w) {
            int mine = 0, cnt = 0;                   // bit r: block (i0 + r, 64 w + lane) is kept
            for (int r = 0; r < nr; ++r) {
                const int bit = (int)((bits[(int64_t)(i0 + r) * P.wpr + w] >> lane) & 1);
                mine |= bit << r;
                cnt += bit;
            }
            int incl = cnt;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const int up = __shfl_up(incl, d, 64);
                if (lane >= d) incl += up;
            }
            int at = pos + incl - cnt;
            for (int r = 0; r < nr; ++r)
                if ((mine >> r) & 1) { P.loc_row[at] = i0 + r; P.loc_col[at] = w * 64 + lane; ++at; }
            pos += __shfl(incl, 63, 64);
        }
    }
}

// The draw: wavefront gid handles word gid of the packed mask (row gid / wpr, word gid % wpr).
__global__ __launch_bounds__(256) void mask_draw_kernel(MaskParams P)
{
    const int lane = lane_id();
    const int64_t gid = (int64_t)blockIdx.x * 4 + wave_id();
    if (gid >= (int64_t)P.MB * P.wpr) return;
    const int64_t i = gid / P.wpr;
    const int w = (int)(gid % P.wpr);
    const int j = w * 64 + lane;
    bool keep = false;
    if (j < P.KB) {
        const uint64_t b = logical_block(P, i, j);
        const uint32_t r = philox_word0((uint32_t)b, (uint32_t)(b >> 32), P.ctr2, P.ctr3, P.key0, P.key1);
        keep = (uint64_t)r >= P.threshold;
    }
    const uint64_t word = __ballot(keep);
    if (lane == 0) P.bits[gid] = word;
}

// Limits of the variant that keeps the bits and both pointer arrays in LDS between phases.
constexpr int kLdsWords = 2048;   // MB * words_per_row
constexpr int kLdsPtrs = 2048;    // MB, KB

// IN_LDS: bits, row_ptr and col_ptr live in LDS while the lists are built and are copied
// out once, so that no phase waits on a round trip to HBM.  Otherwise (large block grids)
// the same phases run on the global arrays.
template <bool IN_LDS>
__global__ __launch_bounds__(kMaskThreads) void mask_kernel(MaskParams P)
{
    __shared__ int32_t wave_tot[kMaskWaves + 1];
    __shared__ int32_t bins[kMaxBins + 1];
    __shared__ uint64_t s_bits[IN_LDS ? kLdsWords : 1];
    __shared__ int32_t s_row_ptr[IN_LDS ? kLdsPtrs + 1 : 1];
    __shared__ int32_t s_col_ptr[IN_LDS ? kLdsPtrs + 1 : 1];
    const int lane = lane_id(), wave = wave_id();
    uint64_t *const bits = IN_LDS ? s_bits : P.bits;
    int32_t *const row_ptr = IN_LDS ? s_row_ptr : P.row_ptr;
    int32_t *const col_ptr = IN_LDS ? s_col_ptr : P.col_ptr;

    // -- rows: fetch the packed words (drawn by mask_draw_kernel, or given by the caller with
    //    possibly dirty padding bits), count per row --
    const uint64_t *src_bits = P.given_bits ? P.given_bits : P.bits;
    for (int64_t g = threadIdx.x; g < (int64_t)P.MB * P.wpr; g += kMaskThreads) {
        const int w = (int)(g % P.wpr);
        const int valid = P.KB - w * 64;                 // columns covered by this word
        uint64_t word = src_bits[g];
        if (valid < 64) word &= (uint64_t(1) << valid) - 1;
        if (IN_LDS) bits[g] = word;
        if (IN_LDS || P.given_bits) P.bits[g] = word;
    }
    __syncthreads();
    for (int i = threadIdx.x; i < P.MB; i += kMaskThreads) {
        int cnt = 0;
        for (int w = 0; w < P.wpr; ++w) cnt += __popcll(bits[(int64_t)i * P.wpr + w]);
        row_ptr[i + 1] = cnt;
    }
    if (threadIdx.x == 0) row_ptr[0] = 0;
    __syncthreads();
    block_inclusive_scan(row_ptr + 1, P.MB, wave_tot);
    if (IN_LDS)
        for (int i = threadIdx.x; i <= P.MB; i += kMaskThreads) P.row_ptr[i] = row_ptr[i];

    // -- rows again: scatter kept columns to their slots --
    for (int i = wave; i < P.MB; i += kMaskWaves) {
        int pos = row_ptr[i];
        for (int w = 0; w < P.wpr; ++w) {
            const uint64_t word = bits[(int64_t)i * P.wpr + w];
            if ((word >> lane) & 1) {
                const int at = pos + __popcll(word & lanes_below());
                P.col_idx[at] = w * 64 + lane;
                P.blk_row[at] = i;
            }
            pos += __popcll(word);
        }
    }

    local_order(bits, row_ptr, P);

    // -- columns: lane <-> block row --
    for (int j = wave; j < P.KB; j += kMaskWaves) {
        int cnt = 0;
        for (int i0 = 0; i0 < P.MB; i0 += 64) {
            const int i = i0 + lane;
            const bool keep = (i < P.MB) && ((bits[(int64_t)i * P.wpr + (j >> 6)] >> (j & 63)) & 1);
            cnt += __popcll(__ballot(keep));
        }
        if (lane == 0) col_ptr[j + 1] = cnt;
    }
    if (threadIdx.x == 0) col_ptr[0] = 0;
    __syncthreads();
    block_inclusive_scan(col_ptr + 1, P.KB, wave_tot);
    if (IN_LDS)
        for (int j = threadIdx.x; j <= P.KB; j += kMaskThreads) P.col_ptr[j] = col_ptr[j];
    for (int j = wave; j < P.KB; j += kMaskWaves) {
        int pos = col_ptr[j];
        for (int i0 = 0; i0 < P.MB; i0 += 64) {
            const int i = i0 + lane;
            const bool keep = (i < P.MB) && ((bits[(int64_t)i * P.wpr + (j >> 6)] >> (j & 63)) & 1);
            const uint64_t word = __ballot(keep);
            if (keep) P.row_idx[pos + __popcll(word & lanes_below())] = i;
            pos += __popcll(word);
        }
    }

    // -- schedules: heavy rows / columns first --
    __shared__ int32_t s_first[2];
    descending_order(row_ptr, P.MB, P.KB, P.row_order, bins, wave_tot, &s_first[0]);
    descending_order(col_ptr, P.KB, P.MB, P.col_order, bins, wave_tot, &s_first[1]);

    if (threadIdx.x == 0) {
        MaskHeader h = {};
        h.M = P.M; h.K = P.K; h.BM = P.BM; h.BK = P.BK; h.MB = P.MB; h.KB = P.KB;
        h.words_per_row = P.wpr;
        h.nnz = row_ptr[P.MB];
        h.magic = kMaskMagic;
        h.max_row_cnt = s_first[0];
        h.max_col_cnt = s_first[1];
        if (!P.given_bits) { h.flags = kMaskDrawn; h.p = P.p; h.seed = P.seed; h.rng_stream = P.rng_stream; }
        *P.hdr = h;
    }
}

// ---- lists for small block grids (MB, KB <= 1024, at most 2048 mask words) ----
// Same result as mask_kernel, built for latency: three barriers instead of a dozen.  Scans run
// in one wavefront each (registers + shuffles), the schedules are rank sorts (rank = number of
// entries with a larger count, ties by index: deterministic), and for very small grids the
// draw itself is done here, which saves a launch.
constexpr int kSmallN = 1024;

// ptr[0..n] := exclusive prefix sums of cnt[0..n), by one wavefront (all 64 lanes call it).
__device__ __forceinline__ void wave_scan(const int32_t *cnt, int32_t *ptr, int n)
{
    const int lane = lane_id();
    const int per = (n + 63) / 64;
    const int lo = lane * per, hi = (lo + per < n) ? lo + per : n;
    int sum = 0;
    for (int i = lo; i < hi; ++i) sum += cnt[i];
    int incl = sum;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int up = __shfl_up(incl, d, 64);
        if (lane >= d) incl += up;
    }
    int run = incl - sum;
    for (int i = lo; i < hi; ++i) { ptr[i] = run; run += cnt[i]; }
    if (lane == 63) ptr[n] = incl;
}

// Launched as one workgroup or as several.  Several: every workgroup builds the same bits, counts and pointers in its
// own LDS (the draw is counter-based, so no workgroup needs another's result) and the lists, the part whose store
// count grows with the grid, are shared out wavefront by wavefront over all workgroups; workgroup 0 alone writes the
// bits, the pointer arrays, the schedules and the header.  For 512 x 32 blocks (57 k list entries, one CU's store
// rate was what the single workgroup spent its time on) mask_draw_kernel + this kernel took 5 + 31 us.
template <bool DRAW>
__global__ __launch_bounds__(kMaskThreads) void mask_small_kernel(MaskParams P)
{
    const bool first_wg = blockIdx.x == 0;
    __shared__ uint64_t s_bits[kLdsWords];
    __shared__ __attribute__((aligned(16))) int32_t s_rcnt[kSmallN], s_ccnt[kSmallN];
    __shared__ __attribute__((aligned(16))) int32_t s_rkey[kSmallN], s_ckey[kSmallN];   // sort keys, see phase 2
    __shared__ int32_t s_row_ptr[kSmallN + 1], s_col_ptr[kSmallN + 1];
    __shared__ int32_t s_max[2], s_nunits;
    const int lane = lane_id(), wave = wave_id();
    const int nwords = P.MB * P.wpr;

    // -- phase 0: the packed words into LDS (drawn here, drawn by mask_draw_kernel, or given) --
    for (int j = threadIdx.x; j < kSmallN; j += kMaskThreads) {
        if (j < P.KB) s_ccnt[j] = 0;
        else s_ckey[j] = -1;                 // keys past the end never outrank anything (the rank loops read quads)
        if (j >= P.MB) s_rkey[j] = -1;
    }
    if (threadIdx.x < 2) s_max[threadIdx.x] = 0;
    if constexpr (DRAW) {
        if (P.wpr == 1 && P.KB <= 32) {
            // narrow grids: a wavefront draws R = 64 / (KB rounded up to a power of two) block rows at
            // a time, so that no lane idles through the ten Philox rounds; the ballot holds R row words
            int kbp = 1;
            while (kbp < P.KB) kbp <<= 1;
            const int R = 64 / kbp, sub = lane / kbp, j = lane & (kbp - 1);
            for (int g = wave; g * R < P.MB; g += kMaskWaves) {
                const int i = g * R + sub;
                bool keep = false;
                if (i < P.MB && j < P.KB) {
                    const uint64_t b = logical_block(P, i, j);
                    const uint32_t r = philox_word0((uint32_t)b, (uint32_t)(b >> 32), P.ctr2, P.ctr3, P.key0, P.key1);
                    keep = (uint64_t)r >= P.threshold;
                }
                const uint64_t all = __ballot(keep);
                if (j == 0 && i < P.MB) {
                    const uint64_t word = (all >> (sub * kbp)) & ((uint64_t(1) << kbp) - 1);
                    s_bits[i] = word;
                    if (first_wg) P.bits[i] = word;
                }
            }
        } else
        for (int g = wave; g < nwords; g += kMaskWaves) {
            const int i = g / P.wpr, w = g % P.wpr, j = w * 64 + lane;
            bool keep = false;
            if (j < P.KB) {
                const uint64_t b = logical_block(P, i, j);
                const uint32_t r = philox_word0((uint32_t)b, (uint32_t)(b >> 32), P.ctr2, P.ctr3, P.key0, P.key1);
                keep = (uint64_t)r >= P.threshold;
            }
            const uint64_t word = __ballot(keep);
            if (lane == 0) { s_bits[g] = word; if (first_wg) P.bits[g] = word; }
        }
    } else {
        const uint64_t *src_bits = P.given_bits ? P.given_bits : P.bits;
        for (int g = threadIdx.x; g < nwords; g += kMaskThreads) {
            const int valid = P.KB - (g % P.wpr) * 64;       // columns covered by this word
            uint64_t word = src_bits[g];
            if (valid < 64) word &= (uint64_t(1) << valid) - 1;
            s_bits[g] = word;
            if (first_wg) P.bits[g] = word;
        }
    }
    __syncthreads();

    // -- phase 1: kept counts per block row and per block column --
    for (int i = threadIdx.x; i < P.MB; i += kMaskThreads) {
        int cnt = 0;
        for (int w = 0; w < P.wpr; ++w) cnt += __popcll(s_bits[i * P.wpr + w]);
        s_rcnt[i] = cnt;
        s_rkey[i] = cnt * kSmallN + (kSmallN - 1 - i);
    }
    // columns: lane <-> block column of a word; every wavefront sums its share of the rows, then one
    // atomic per lane and wavefront
    for (int w = 0; w < P.wpr; ++w) {
        int c = 0;
        for (int i = wave; i < P.MB; i += kMaskWaves) c += (int)((s_bits[i * P.wpr + w] >> lane) & 1);
        if (w * 64 + lane < P.KB && c) atomicAdd(&s_ccnt[w * 64 + lane], c);
    }
    __syncthreads();

    // -- phase 2: pointers (one wavefront each) and schedules.  rank = number of entries with a larger
    //    count, ties by index: with the key count * 1024 + (1023 - index) that is the number of larger
    //    keys, one compare and one add per entry.  Rows are ranked by the lower half of the workgroup
    //    and columns by the upper half at the same time; the keys are read four at a time --
    for (int j = threadIdx.x; j < P.KB; j += kMaskThreads) s_ckey[j] = s_ccnt[j] * kSmallN + (kSmallN - 1 - j);
    __syncthreads();
    if (wave == kMaskWaves - 1) wave_scan(s_rcnt, s_row_ptr, P.MB);
    if (wave == kMaskWaves - 2) wave_scan(s_ccnt, s_col_ptr, P.KB);
    auto rank_of = [](const int32_t *key, int n, int mine) {
        int rank = 0;
        const int4 *q = reinterpret_cast<const int4 *>(key);
#pragma unroll 4
        for (int o = 0; o < (n + 3) / 4; ++o) {
            const int4 v = q[o];
            rank += (v.x > mine) + (v.y > mine) + (v.z > mine) + (v.w > mine);
        }
        return rank;
    };
    // (with several workgroups the rows and columns to rank are dealt out over all of them: ranking is quadratic,
    // 512 rows took one workgroup 5 us)
    constexpr int kHalf = kMaskThreads / 2;
    const int rank_stride = (int)gridDim.x * kHalf;
    if (threadIdx.x < kHalf) {
        for (int i = (int)blockIdx.x * kHalf + threadIdx.x; i < P.MB; i += rank_stride) {
            const int rank = rank_of(s_rkey, P.MB, s_rkey[i]);
            P.row_order[rank] = i;
        }
    } else {
        for (int j = (int)blockIdx.x * kHalf + threadIdx.x - kHalf; j < P.KB; j += rank_stride) {
            const int rank = rank_of(s_ckey, P.KB, s_ckey[j]);
            P.col_order[rank] = j;
        }
    }
    // the largest counts, for the header (workgroup 0 writes it)
    // (a maximum per wavefront first: atomics of many lanes on one LDS word are served one by one)
    if (first_wg) {
        int mr = 0, mc = 0;
        for (int i = threadIdx.x; i < P.MB; i += kMaskThreads) mr = s_rcnt[i] > mr ? s_rcnt[i] : mr;
        for (int j = threadIdx.x; j < P.KB; j += kMaskThreads) mc = s_ccnt[j] > mc ? s_ccnt[j] : mc;
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) {
            const int orr = __shfl_xor(mr, d, 64), oc = __shfl_xor(mc, d, 64);
            mr = orr > mr ? orr : mr;
            mc = oc > mc ? oc : mc;
        }
        if (lane == 0) { atomicMax(&s_max[0], mr); atomicMax(&s_max[1], mc); }
    }
    __syncthreads();

    // -- phase 3: the lists --
    if (first_wg) {
        for (int i = threadIdx.x; i <= P.MB; i += kMaskThreads) P.row_ptr[i] = s_row_ptr[i];
        for (int j = threadIdx.x; j <= P.KB; j += kMaskThreads) P.col_ptr[j] = s_col_ptr[j];
    }
    // The three kinds of lists do not depend on each other.  One workgroup: with few groups of 8 block rows (a small
    // grid) the locally ordered list would keep only that many wavefronts busy, on top of their share of the other
    // lists: those groups then get wavefronts of their own, the last ones, and the row and column lists are shared
    // by the rest.  Several workgroups: every kind is dealt out over all wavefronts of the launch.
    const int nwg = (int)gridDim.x;
    const int ngroups = (P.MB + 7) / 8;
    const int nlo = (nwg == 1 && ngroups < kMaskWaves / 2) ? ngroups : 0;   // wavefronts that only build the locally ordered list
    // The pair list (grids of at most 128 x 64 blocks of 128 x 128: a block row is one word) is one wavefront's work,
    // the first workgroup's last; on a small grid that wavefront does nothing else.
    const bool pairs_here = first_wg && units_apply(P.MB, P.KB, P.BM, P.BK);
    const int npl = pairs_here && nlo > 0 ? 1 : 0;
    const int nls = kMaskWaves - nlo - npl;                        // wavefronts (per workgroup) that build the row and column lists
    if (first_wg && wave == kMaskWaves - 1) {
        int n = 0;
        if (pairs_here) n = build_units(lane < P.MB ? s_bits[lane] : 0, lane + 64 < P.MB ? s_bits[lane + 64] : 0, P.MB, P.units);
        if (lane == 0) s_nunits = n;
    }
    const int gw = (int)blockIdx.x * nls + wave, ngw = nwg * nls;  // this wavefront among those of the whole launch
    if (nlo > 0) local_order(s_bits, s_row_ptr, P, nls, nlo);
    for (int i = gw; i < P.MB && wave < nls; i += ngw) {
        int pos = s_row_ptr[i];
        for (int w = 0; w < P.wpr; ++w) {
            const uint64_t word = s_bits[i * P.wpr + w];
            if ((word >> lane) & 1) {
                const int at = pos + __popcll(word & lanes_below());
                P.col_idx[at] = w * 64 + lane;
                P.blk_row[at] = i;
            }
            pos += __popcll(word);
        }
    }
    if (nlo == 0) local_order(s_bits, s_row_ptr, P, 0, kMaskWaves, (int)blockIdx.x, nwg);
    for (int j = gw; j < P.KB && wave < nls; j += ngw) {
        int pos = s_col_ptr[j];
        for (int i0 = 0; i0 < P.MB; i0 += 64) {
            const int i = i0 + lane;
            const bool keep = (i < P.MB) && ((s_bits[i * P.wpr + (j >> 6)] >> (j & 63)) & 1);
            const uint64_t word = __ballot(keep);
            if (keep) P.row_idx[pos + __popcll(word & lanes_below())] = i;
            pos += __popcll(word);
        }
    }
    if (!first_wg) return;
    __syncthreads();                                   // s_nunits
    if (threadIdx.x == 0) {
        MaskHeader h = {};
        h.M = P.M; h.K = P.K; h.BM = P.BM; h.BK = P.BK; h.MB = P.MB; h.KB = P.KB;
        h.words_per_row = P.wpr;
        h.nnz = s_row_ptr[P.MB];
        h.magic = kMaskMagic;
        h.max_row_cnt = s_max[0];
        h.max_col_cnt = s_max[1];
        h.n_units = s_nunits;
        if (!P.given_bits) { h.flags = kMaskDrawn; h.p = P.p; h.seed = P.seed; h.rng_stream = P.rng_stream; }
        *P.hdr = h;
    }
}

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

int launch_mask(void *mask, size_t mask_bytes, int64_t M, int64_t K, int BM, int BK,
                double p, uint64_t seed, uint64_t rng_stream, const uint64_t *given_bits,
                void *stream, int split_m = 1, int split_k = 1)
{
    if (!mask) return SDROP_EINVAL;
    if (!(p >= 0.0 && p <= 1.0)) return SDROP_EINVAL;
    if (split_m < 1 || split_k < 1) return SDROP_EINVAL;
    sdrop_mask_layout_t L;
    const int rc = sdrop_mask_layout(M, K, BM, BK, &L);
    if (rc != SDROP_OK) return rc;
    if (reinterpret_cast<uintptr_t>(mask) % 16) return SDROP_EALIGN;
    if (given_bits && reinterpret_cast<uintptr_t>(given_bits) % 8) return SDROP_EALIGN;
    if (mask_bytes < L.total_bytes) return SDROP_EWORKSPACE;
    if (L.MB % split_m || L.KB % split_k) return SDROP_ESHAPE;

    char *b = static_cast<char *>(mask);
    MaskParams P;
    P.hdr = reinterpret_cast<MaskHeader *>(b);
    P.bits = reinterpret_cast<uint64_t *>(b + L.off_bits);
    P.row_ptr = reinterpret_cast<int32_t *>(b + L.off_row_ptr);
    P.col_idx = reinterpret_cast<int32_t *>(b + L.off_col_idx);
    P.blk_row = reinterpret_cast<int32_t *>(b + L.off_blk_row);
    P.col_ptr = reinterpret_cast<int32_t *>(b + L.off_col_ptr);
    P.row_idx = reinterpret_cast<int32_t *>(b + L.off_row_idx);
    P.row_order = reinterpret_cast<int32_t *>(b + L.off_row_order);
    P.col_order = reinterpret_cast<int32_t *>(b + L.off_col_order);
    P.loc_row = reinterpret_cast<int32_t *>(b + L.off_loc_row);
    P.loc_col = reinterpret_cast<int32_t *>(b + L.off_loc_col);
    P.units = reinterpret_cast<int32_t *>(b + L.off_units);
    P.given_bits = given_bits;
    P.M = M; P.K = K; P.BM = BM; P.BK = BK;
    P.MB = static_cast<int32_t>(L.MB); P.KB = static_cast<int32_t>(L.KB);
    P.wpr = static_cast<int32_t>(L.words_per_row);
    P.split_m = split_m; P.split_k = split_k; P.KBL = P.KB / split_k;
    P.key0 = static_cast<uint32_t>(seed); P.key1 = static_cast<uint32_t>(seed >> 32);
    P.ctr2 = static_cast<uint32_t>(rng_stream); P.ctr3 = static_cast<uint32_t>(rng_stream >> 32);
    P.threshold = static_cast<uint64_t>(floor(p * 4294967296.0));
    P.p = p; P.seed = seed; P.rng_stream = rng_stream;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int64_t words = L.MB * L.words_per_row;
    const bool small = L.MB <= kSmallN && L.KB <= kSmallN && words <= kLdsWords;
    // Small grids (and that is all five workloads') are drawn by the workgroups that build the lists: one launch.
    // The lists are shared out over several workgroups when there are many of them (about 32 list pieces, i.e. block
    // rows, block columns and groups of 8 block rows, per workgroup).
    const bool fused_draw = small && !given_bits;
    const int64_t pieces = L.MB + L.KB + (L.MB + 7) / 8;
    const unsigned n_wg = !small || words <= 64 ? 1u : (unsigned)(pieces / 32 < 1 ? 1 : pieces / 32 > 64 ? 64 : pieces / 32);
    if (!given_bits && !fused_draw) {
        hipLaunchKernelGGL(mask_draw_kernel, dim3((unsigned)((words + 3) / 4)), dim3(256), 0, st, P);
        const int rc2 = hip_status(hipGetLastError());
        if (rc2 != SDROP_OK) return rc2;
    }
    if (small) {
        if (fused_draw) hipLaunchKernelGGL(mask_small_kernel<true>, dim3(n_wg), dim3(kMaskThreads), 0, st, P);
        else hipLaunchKernelGGL(mask_small_kernel<false>, dim3(n_wg), dim3(kMaskThreads), 0, st, P);
        return hip_status(hipGetLastError());
    }
    const bool in_lds = L.MB * L.words_per_row <= kLdsWords && L.MB <= kLdsPtrs && L.KB <= kLdsPtrs;
    if (in_lds)
        hipLaunchKernelGGL(mask_kernel<true>, dim3(1), dim3(kMaskThreads), 0, st, P);
    else
        hipLaunchKernelGGL(mask_kernel<false>, dim3(1), dim3(kMaskThreads), 0, st, P);
    return hip_status(hipGetLastError());
}

}  // namespace
}  // namespace sdrop

extern "C" {

const char *sdrop_strerror(int code)
{
    switch (code) {
    case SDROP_OK: return "ok";
    case SDROP_EINVAL: return "invalid argument (null pointer, p outside [0,1], bad enum)";
    case SDROP_ESHAPE: return "bad shape (sizes must be positive, BM|M, BK|K, BM,BK in {64,128}, 8|N)";
    case SDROP_EDTYPE: return "unsupported dtype / out_dtype";
    case SDROP_EALIGN: return "pointer not 16-byte aligned";
    case SDROP_EWORKSPACE: return "mask buffer or workspace too small";
    case SDROP_EHIP: return "HIP runtime error (see sdrop_last_hip_error)";
    default: return "unknown sdrop error code";
    }
}

int sdrop_last_hip_error(void) { return sdrop::g_last_hip_error; }

int sdrop_mask_layout(int64_t M, int64_t K, int BM, int BK, sdrop_mask_layout_t *out)
{
    if (!out) return SDROP_EINVAL;
    if (M <= 0 || K <= 0 || !sdrop::block_size_ok(BM) || !sdrop::block_size_ok(BK)) return SDROP_ESHAPE;
    if (M % BM || K % BK) return SDROP_ESHAPE;
    const int64_t MB = M / BM, KB = K / BK;
    // the index lists are int32 and one workgroup builds them
    if (MB > (1 << 20) || KB > (1 << 20) || MB * KB > (int64_t(1) << 26)) return SDROP_ESHAPE;
    const int64_t wpr = (KB + 63) / 64;
    const size_t nblk = static_cast<size_t>(MB * KB);
    size_t off = sizeof(sdrop::MaskHeader);
    out->off_bits = off;      off = sdrop::align_up(off + sizeof(uint64_t) * MB * wpr, 256);
    out->off_row_ptr = off;   off = sdrop::align_up(off + 4 * (MB + 1), 256);
    out->off_col_idx = off;   off = sdrop::align_up(off + 4 * nblk, 256);
    out->off_blk_row = off;   off = sdrop::align_up(off + 4 * nblk, 256);
    out->off_col_ptr = off;   off = sdrop::align_up(off + 4 * (KB + 1), 256);
    out->off_row_idx = off;   off = sdrop::align_up(off + 4 * nblk, 256);
    out->off_row_order = off; off = sdrop::align_up(off + 4 * MB, 256);
    out->off_col_order = off; off = sdrop::align_up(off + 4 * KB, 256);
    out->off_loc_row = off;   off = sdrop::align_up(off + 4 * nblk, 256);
    out->off_loc_col = off;   off = sdrop::align_up(off + 4 * nblk, 256);
    out->off_units = off;     off = sdrop::align_up(off + 4 * nblk, 256);
    out->total_bytes = off;
    out->MB = MB; out->KB = KB; out->words_per_row = wpr;
    return SDROP_OK;
}

size_t sdrop_mask_bytes(int64_t M, int64_t K, int BM, int BK)
{
    sdrop_mask_layout_t L;
    return sdrop_mask_layout(M, K, BM, BK, &L) == SDROP_OK ? L.total_bytes : 0;
}

int sdrop_mask(void *mask, size_t mask_bytes, int64_t M, int64_t K, int BM, int BK,
               double p, uint64_t seed, uint64_t rng_stream, void *stream)
{
    return sdrop::launch_mask(mask, mask_bytes, M, K, BM, BK, p, seed, rng_stream, nullptr, stream);
}

int sdrop_mask_split(void *mask, size_t mask_bytes, int64_t M, int64_t K, int BM, int BK,
                     int split_m, int split_k, double p, uint64_t seed, uint64_t rng_stream, void *stream)
{
    return sdrop::launch_mask(mask, mask_bytes, M, K, BM, BK, p, seed, rng_stream, nullptr, stream, split_m, split_k);
}

int sdrop_mask_from_bits(void *mask, size_t mask_bytes, int64_t M, int64_t K, int BM, int BK,
                         const uint64_t *bits, void *stream)
{
    if (!bits) return SDROP_EINVAL;
    return sdrop::launch_mask(mask, mask_bytes, M, K, BM, BK, 0.0, 0, 0, bits, stream);
}

int sdrop_mask_bits(const void *mask, uint64_t *bits_host, size_t n_words, int64_t *nnz_host, void *stream)
{
    if (!mask || (!bits_host && !nnz_host)) return SDROP_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    // the header first (it says how many words there are), then the words: two copies, each waited for
    sdrop::MaskHeader h;
    hipError_t e = hipMemcpyAsync(&h, mask, sizeof(h), hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) return sdrop::hip_status(e);
    if (h.magic != sdrop::kMaskMagic || h.MB <= 0 || h.words_per_row <= 0) return SDROP_EINVAL;
    if (nnz_host) *nnz_host = h.nnz;
    if (bits_host) {
        const size_t words = (size_t)h.MB * (size_t)h.words_per_row;
        if (n_words < words) return SDROP_EWORKSPACE;
        e = hipMemcpyAsync(bits_host, static_cast<const char *>(mask) + sizeof(sdrop::MaskHeader), words * sizeof(uint64_t),
                           hipMemcpyDeviceToHost, st);
        if (e == hipSuccess) e = hipStreamSynchronize(st);
        if (e != hipSuccess) return sdrop::hip_status(e);
    }
    return SDROP_OK;
}

}  // extern "C"
