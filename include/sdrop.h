/*
 * sdrop.h -- C ABI of libsdrop: SparseDrop's block-structured dropout fused
 * into the following matrix multiply, as hand-written HIP kernels for gfx950.
 *
 * The operations are those of arxiv 2411.01238, Section 3.1 eq. (1)-(3), with
 * the block mask of Section 3.2:
 *
 *     m'  : one Bernoulli(1-p) keep flag per BM x BK block of X   (Section 3.2)
 *     Y   = s (X . m') W                                          (eq. 1)
 *     dX  = s (dY W^T) . m'                                       (eq. 2)
 *     dW  = s (X . m')^T dY                                       (eq. 3)
 *     s   = 1/(1-p)   (s = 0 when p = 1: everything is dropped)
 *
 * with X[M,K], W[K,N], Y[M,N], dY[M,N], dX[M,K], dW[K,N], no bias.
 *
 * Conventions shared by every entry point
 *   - All matrix and mask pointers are DEVICE pointers (HBM).  Matrices are dense
 *     row-major and contiguous (leading dimension = number of columns) and
 *     16-byte aligned.  The caller owns every buffer and the stream; the
 *     library allocates nothing, frees nothing and keeps no pointer after a
 *     call returns.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls only enqueue work on it and return; no call synchronises with the
 *     host or copies to the host.
 *   - Block sizes must divide the shape (Section 2.2, footnote): BM | M and
 *     BK | K, with BM, BK in {64, 128}.  N must be a multiple of 8.  M <= 2^30,
 *     K <= 2^24, N <= 2^24.
 *   - Inputs are fp16 or bf16 (SDROP_F16 / SDROP_BF16); products are
 *     accumulated in fp32 on the matrix cores; the scale s is applied to the
 *     fp32 accumulator; the result is rounded to nearest-even once, to
 *     `out_dtype` (the input type, or SDROP_F32 for unrounded fp32 output).
 *   - Outputs are completely overwritten.  Dropped blocks of dX are written as
 *     +0 by the library (Section 3.2 assumes a zero-initialised output; here no
 *     such precondition exists).  Dropped blocks of X are never read, so their
 *     contents (NaN included) cannot reach Y or dW.
 *   - Return value: SDROP_OK or an error code.  Argument errors are detected on
 *     the host before anything is enqueued and leave every buffer untouched.
 */
#ifndef SDROP_H
#define SDROP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    SDROP_OK = 0,
    SDROP_EINVAL = 1,      /* null pointer, p outside [0,1] or NaN, bad enum value */
    SDROP_ESHAPE = 2,      /* non-positive size, BM does not divide M, BK does not divide K,
                              unsupported block size, N not a multiple of 8 */
    SDROP_EDTYPE = 3,      /* unsupported dtype / out_dtype combination */
    SDROP_EALIGN = 4,      /* a pointer is not 16-byte aligned */
    SDROP_EWORKSPACE = 5,  /* mask buffer or workspace smaller than required */
    SDROP_EHIP = 6         /* the HIP runtime refused a launch; see sdrop_last_hip_error() */
};

enum { SDROP_F16 = 0, SDROP_BF16 = 1, SDROP_F32 = 2 /* out_dtype only */ };

enum { SDROP_OP_FWD = 0, SDROP_OP_BWD_DX = 1, SDROP_OP_BWD_DW = 2 };

/*
 * Host-side tuning knobs (process-wide; not thread-safe against concurrent GEMM calls).  They change
 * which kernel a call uses, never its result.
 *   SDROP_TUNE_DX_PERSISTENT_GROUPS_PER_CU  sdrop_bwd_dx with tiles of several kept blocks uses its
 *       persistent kernel when it expects at least this many tiles per CU (default 8; 0 = whenever
 *       the shape allows it)
 *   SDROP_TUNE_DX_TILE_WIDTH  columns of sdrop_bwd_dx's output tiles: 0 (default) chosen per call
 *       from the expected number of kept blocks, 128 or 256 forced
 *   SDROP_TUNE_BWD_FUSED  1 (default): sdrop_bwd computes both gradients in one launch where the
 *       shapes allow it; 0: always as the two separate launches
 *   SDROP_TUNE_FWD_SEEDED  1 (default): sdrop_fwd_seeded draws the mask inside the forward kernel where the
 *       block grid allows it; 0: always as sdrop_mask followed by sdrop_fwd
 *   SDROP_TUNE_DW64_PERSISTENT_SLICES  sdrop_bwd_dw with 64-row tiles (BK = 64) uses its persistent kernel
 *       when it expects at least this many reduction slices per tile (default 16; 0 = always)
 *   SDROP_TUNE_DX_PAIRS  sdrop_bwd_dx / sdrop_bwd with 128 x 128 blocks on grids of at most 128 x 64 blocks: tiles
 *       of two kept blocks from the mask's pair list; 0 (default) chosen per call, 1 wherever it applies, 2 never
 * Returns SDROP_EINVAL for an unknown knob or a value outside its range.
 */
enum { SDROP_TUNE_DX_PERSISTENT_GROUPS_PER_CU = 0, SDROP_TUNE_BWD_FUSED = 1, SDROP_TUNE_DX_TILE_WIDTH = 2,
       SDROP_TUNE_FWD_SEEDED = 3, SDROP_TUNE_DW64_PERSISTENT_SLICES = 4, SDROP_TUNE_DX_PAIRS = 5 };
int sdrop_set_tuning(int knob, int value);

/*
 * What the kernels have found wrong since the status word was last cleared.  Calls only enqueue work, so a condition
 * that only the device can see cannot come back as a return code: a kernel that is handed a mask object that does
 * not belong to its call (another shape or block size, not a mask object at all, or a mask drawn with a dropout
 * probability other than the call's p) writes nothing and sets SDROP_STATUS_MASK_MISMATCH in a status word that
 * lives in device memory (one per GPU).  sdrop_status copies that word to *flags_host, clears it if `clear` is
 * non-zero, and waits for `stream` (so work enqueued on it before the call has reported).  SDROP_EINVAL for a null
 * pointer.
 */
#define SDROP_STATUS_MASK_MISMATCH 1
int sdrop_status(int *flags_host, int clear, void *stream);

/* Text for an error code (static storage). */
const char *sdrop_strerror(int code);

/* The hipError_t (as int) of the last SDROP_EHIP on the calling thread, else 0. */
int sdrop_last_hip_error(void);

/*
 * Layout of a mask object in device memory.  A mask object is one caller-owned
 * buffer of `total_bytes`; all offsets are in bytes from its start.  With
 * MB = M/BM, KB = K/BK and nnz = number of kept blocks:
 *
 *   header   at 0 (256 bytes): int64 M, K; int32 BM, BK, MB, KB, words_per_row, nnz; ...; for a mask that was
 *            drawn also the p, seed and rng_stream it was drawn with (the kernels compare that p with the p of
 *            the call that uses the mask)
 *            (nnz is the int32 at byte offset SDROP_MASK_NNZ_OFFSET)
 *   bits     uint64[MB][words_per_row]: block (i,j) is bit j%64 of word j/64 of
 *            row i, 1 = kept, unused high bits zero (the 64-bit packing of Section 3.4)
 *   row_ptr  int32[MB+1], col_idx int32[nnz (room for MB*KB)]: kept block columns of
 *            each block row, ascending (what eq. 1 walks)
 *   blk_row  int32[nnz (room for MB*KB)]: block row of the t-th kept block in the same
 *            order as col_idx, i.e. (blk_row[t], col_idx[t]) lists the kept
 *            blocks row-major (what eq. 2 computes)
 *   col_ptr  int32[KB+1], row_idx int32[nnz (room for MB*KB)]: kept block rows of each
 *            block column, ascending (what eq. 3 walks)
 *   row_order int32[MB], col_order int32[KB]: block rows / columns sorted by
 *            descending kept count (ties in unspecified order); used to
 *            schedule heavy tiles first
 *   loc_row, loc_col  int32[nnz (room for MB*KB)] each: the kept blocks once more, as
 *            (loc_row[t], loc_col[t]), sorted by (i / 8, j, i % 8): groups of 8 block rows
 *            in order, inside a group column by column.  Blocks that are neighbours in
 *            this list share block rows AND block columns, which is the order eq. 2
 *            computes them in (tiles that run at the same time then share operand
 *            tiles in cache)
 *   units    int32[n_units (room for MB*KB)], for grids of at most 128 x 64 blocks of 128 x 128 (n_units, the
 *            int32 at byte offset SDROP_MASK_NUNITS_OFFSET of the header, is 0 for other grids): the kept blocks
 *            once more, as pairs that can share an output tile of eq. 2, and the few blocks left over.
 *            An entry is kind << 30 | x << 16 | y << 8 | z with kind 0: blocks (x, y) and (x, z) of one
 *            block row; kind 1: blocks (y, x) and (z, x) of one block column; kind 2: block (x, y) alone.
 *            Every kept block is in exactly one entry.
 */
typedef struct sdrop_mask_layout {
    size_t total_bytes;
    size_t off_bits, off_row_ptr, off_col_idx, off_blk_row;
    size_t off_col_ptr, off_row_idx, off_row_order, off_col_order;
    size_t off_loc_row, off_loc_col;
    size_t off_units;
    int64_t MB, KB, words_per_row;
} sdrop_mask_layout_t;

#define SDROP_MASK_NNZ_OFFSET 36
#define SDROP_MASK_NUNITS_OFFSET 80

/* Fills *out for a mask over X[M,K] in BM x BK blocks.  SDROP_ESHAPE on a bad shape. */
int sdrop_mask_layout(int64_t M, int64_t K, int BM, int BK, sdrop_mask_layout_t *out);

/* total_bytes of the layout above, or 0 on a bad shape. */
size_t sdrop_mask_bytes(int64_t M, int64_t K, int BM, int BK);

/*
 * Draws the block mask m' of Section 3.2 on the device and builds every index
 * list above from it in the same launch.
 *
 * The paper does not fix a generator.  This library uses Philox4x32-10 with
 * counter (b lo32, b hi32, rng_stream lo32, rng_stream hi32), where b = i*KB + j
 * is the block number, key (seed lo32, seed hi32), and keeps block (i,j) iff
 * output word 0 >= floor(p * 2^32).  The mask is a pure function of
 * (seed, rng_stream, MB, KB, p): the backward calls of a step reuse the object
 * written by the forward's call, or regenerate it.
 *
 *   mask        device buffer of at least sdrop_mask_bytes(...) bytes, 16-byte aligned
 *   p           dropout probability in [0,1]
 *   seed, rng_stream   generator key and stream (e.g. layer or step number)
 */
int sdrop_mask(void *mask, size_t mask_bytes, int64_t M, int64_t K, int BM, int BK,
               double p, uint64_t seed, uint64_t rng_stream, void *stream);

/*
 * Block splitting (Section 3.3): the mask object of a LOGICAL mask whose blocks are
 * (split_m * BM) x (split_k * BK), retiled to BM x BK blocks: one Bernoulli(1-p) draw per logical
 * block, numbered b = I * (KB / split_k) + J over the logical grid, repeated split_m times along M
 * and split_k times along K.  Objects made with different (BM, BK, split_m, split_k) but the same
 * products split_m * BM and split_k * BK, p, seed and rng_stream mask exactly the same elements, so
 * the forward pass and the two backward passes of one layer may each use the block size that
 * suits their GEMM.  split_m = split_k = 1 is sdrop_mask.  (The section's text and its figure
 * caption disagree on which factor goes with which axis; this follows the text's formula.)
 * SDROP_ESHAPE if split_m does not divide M/BM or split_k does not divide K/BK, SDROP_EINVAL if
 * a factor is < 1.
 */
int sdrop_mask_split(void *mask, size_t mask_bytes, int64_t M, int64_t K, int BM, int BK,
                     int split_m, int split_k, double p, uint64_t seed, uint64_t rng_stream,
                     void *stream);

/*
 * Same object, but the keep bits are given instead of drawn: `bits` is a device
 * array uint64[MB][words_per_row] in the packing described above (unused high
 * bits are ignored).  For callers that bring their own block mask, and for
 * tests that need a particular pattern (for example all blocks dropped).
 */
int sdrop_mask_from_bits(void *mask, size_t mask_bytes, int64_t M, int64_t K, int BM, int BK,
                         const uint64_t *bits, void *stream);

/*
 * Reads a mask object back: the packed keep bits of Section 3.4 (uint64[MB][words_per_row], as laid out
 * above) into HOST memory `bits_host` of `n_words` words, and the number of kept blocks into
 * `*nnz_host` (either may be NULL, not both).  This is the one entry point that synchronises: it waits
 * for `stream`, so the object as written by the work enqueued before the call is what is read.
 * SDROP_EINVAL if the buffer does not hold a mask object (nothing is written to the outputs);
 * SDROP_EWORKSPACE if n_words is less than MB * words_per_row of the object (nnz is still delivered).
 */
int sdrop_mask_bits(const void *mask, uint64_t *bits_host, size_t n_words, int64_t *nnz_host, void *stream);

/*
 * Bytes of device workspace an operation needs for these arguments (may be 0).  Only
 * sdrop_bwd_dw uses one: when K/BK * ceil(N/256) output tiles are too few to fill the chip,
 * the reduction over M is cut into `splits` parts that write fp32 planes [splits][K][N] to
 * the workspace, summed in a fixed order by a second pass.  A function of the shape and of
 * the device's CU count only.
 */
size_t sdrop_workspace_bytes(int op, int64_t M, int64_t K, int64_t N, int BM, int BK,
                             int dtype, int out_dtype);

/*
 * eq. (1): Y[M,N] = s (X . m') W.  For each block row only the kept K-blocks
 * are walked; dropped blocks of X and the matching row blocks of W are not read
 * (Section 3.2, structured dsd_matmul).
 *
 *   X[M,K], W[K,N]  inputs of type `dtype`;  Y[M,N] output of type `out_dtype`
 *   mask            object written by sdrop_mask / sdrop_mask_from_bits with the same
 *                   (M, K, BM, BK), in a buffer of at least sdrop_mask_bytes(M, K, BM, BK) bytes
 *                   for THIS call's shape (the kernels address the lists by the call's shape before
 *                   they have compared the header); a kernel that finds a different header writes
 *                   nothing
 *   p               the dropout probability the scale s is derived from; for a mask made by sdrop_mask /
 *                   sdrop_mask_split / sdrop_fwd_seeded it must be the p the mask was drawn with (a kernel
 *                   that finds another p in the object treats it like a mask of another problem: it writes
 *                   nothing, see sdrop_status); a mask built from the caller's bits goes with any p
 *   ws, ws_bytes    device workspace of at least sdrop_workspace_bytes(SDROP_OP_FWD, ...)
 *                   bytes (ws may be NULL when that is 0)
 */
int sdrop_fwd(const void *X, const void *W, const void *mask, void *Y,
              int64_t M, int64_t K, int64_t N, int BM, int BK, double p,
              int dtype, int out_dtype, void *ws, size_t ws_bytes, void *stream);

/*
 * The mask of a step and eq. (1) in one call: draws m' exactly as sdrop_mask(mask, ..., p, seed, rng_stream) does,
 * writes the same mask object to `mask` (for the backward calls of the step) and computes Y = s (X . m') W, all
 * bit-identical to sdrop_mask followed by sdrop_fwd.  The paper found mask generation to dominate small layers
 * (Section 3.4); here the mask kernel and the launch boundary behind it are what is left of that, and for block
 * grids of at most 128 rows x 64 columns this call removes both: one launch, in which every workgroup draws the grid itself (the generator is counter-based) and the
 * workgroups share the writing of the mask object.  Larger grids run the two launches in turn.
 *   mask, mask_bytes  device buffer of at least sdrop_mask_bytes(M, K, BM, BK) bytes: OUTPUT
 *   other arguments as for sdrop_mask and sdrop_fwd; no workspace is needed
 */
int sdrop_fwd_seeded(const void *X, const void *W, void *mask, size_t mask_bytes, void *Y,
                     int64_t M, int64_t K, int64_t N, int BM, int BK, double p, uint64_t seed, uint64_t rng_stream,
                     int dtype, int out_dtype, void *stream);

/*
 * eq. (2): dX[M,K] = s (dY W^T) . m'.  Only kept output blocks are computed
 * (Section 3.2, sdd_matmul); dropped blocks are filled with +0.
 *   dY[M,N], W[K,N] inputs;  dX[M,K] output.  Other arguments as for sdrop_fwd.
 */
int sdrop_bwd_dx(const void *dY, const void *W, const void *mask, void *dX,
                 int64_t M, int64_t K, int64_t N, int BM, int BK, double p,
                 int dtype, int out_dtype, void *ws, size_t ws_bytes, void *stream);

/*
 * eq. (3): dW[K,N] = s (X . m')^T dY.  For each block column of X only the kept
 * row blocks are walked (Section 3.3: a GEMM of size (K,N,M) whose reduction
 * runs over M in steps of the mask's row block).
 *   X[M,K], dY[M,N] inputs;  dW[K,N] output.  Other arguments as for sdrop_fwd.
 */
int sdrop_bwd_dw(const void *X, const void *dY, const void *mask, void *dW,
                 int64_t M, int64_t K, int64_t N, int BM, int BK, double p,
                 int dtype, int out_dtype, void *ws, size_t ws_bytes, void *stream);

/*
 * sdrop_bwd_dw for callers that cannot allocate device memory or pass a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, checks and
 * result (bit for bit) as sdrop_bwd_dw, without `ws`: the fp32 planes of a split reduction go to
 * SDROP_STATIC_SCRATCH_BYTES (128 MiB) of device memory that is part of the library's code object
 * (one copy per GPU, held from the library's load on that GPU to the end of the process).  The
 * call allocates and frees nothing.
 *   - SDROP_EWORKSPACE when sdrop_workspace_bytes(SDROP_OP_BWD_DW, ...) exceeds
 *     SDROP_STATIC_SCRATCH_BYTES (nothing is enqueued); all five workloads of the benchmark fit.
 *   - Every call on a GPU uses that GPU's one copy, which keeps the previous call's contents (a
 *     call overwrites all it reads, nothing needs clearing).  Two calls that overlap in time on
 *     one GPU (different streams, or threads) race on it: serialise them.
 */
#define SDROP_STATIC_SCRATCH_BYTES ((size_t)128 << 20)
int sdrop_bwd_dw_static(const void *X, const void *dY, const void *mask, void *dW,
                        int64_t M, int64_t K, int64_t N, int BM, int BK, double p,
                        int dtype, int out_dtype, void *stream);

/*
 * eq. (2) and eq. (3) in one call: both gradients of the layer, which share dY and the mask and
 * do not depend on each other.  Results are bit-identical to sdrop_bwd_dx followed by
 * sdrop_bwd_dw with the same arguments.  With 128 x 128 blocks (or 64 x 64 blocks and short
 * kept lists) and N a multiple of 256 one launch holds the workgroups of both products: those
 * of eq. (3) start on the CUs as those of eq. (2) leave them, with no launch boundary and no
 * idle tail in between; otherwise the two are launched in turn.
 *   dY[M,N], W[K,N], X[M,K] inputs;  dX[M,K], dW[K,N] outputs, both of type `out_dtype`
 *   ws, ws_bytes  as for sdrop_bwd_dw (sdrop_workspace_bytes(SDROP_OP_BWD_DW, ...))
 * All arguments are checked before anything is enqueued.
 */
int sdrop_bwd(const void *dY, const void *W, const void *X, const void *mask, void *dX, void *dW,
              int64_t M, int64_t K, int64_t N, int BM, int BK, double p,
              int dtype, int out_dtype, void *ws, size_t ws_bytes, void *stream);

/*
 * sdrop_bwd for row-strided matrices: the leading dimensions, in elements, of dY[M,N], W[K,N], X[M,K], dX[M,K] and
 * dW[K,N] (0 = contiguous; else at least the number of columns, a multiple of 8, at most 2^24, else SDROP_ESHAPE).
 * Same launches and results as sdrop_bwd on contiguous copies; nothing outside the column ranges is written.
 * w_layout = SDROP_W_NK: W is given and dW delivered as [N,K] (ld_w, ld_dw >= K): one launch where both products
 * read and write the arrays in place (128 x 128 blocks, N a multiple of 256, eq. 2 on single blocks), else
 * sdrop_bwd_dx_ex followed by sdrop_bwd_dw_ex with that layout; the same bits as those two calls, and the workspace
 * is that of sdrop_bwd_dw_ex with that layout (sdrop_workspace_bytes_ex(SDROP_OP_BWD_DW, ...)).
 */
int sdrop_bwd_ex(const void *dY, const void *W, const void *X, const void *mask, void *dX, void *dW,
                 int64_t M, int64_t K, int64_t N, int BM, int BK, double p,
                 int dtype, int out_dtype, void *ws, size_t ws_bytes, void *stream,
                 int64_t ld_dy, int64_t ld_w, int64_t ld_x, int64_t ld_dx, int64_t ld_dw, int w_layout);

/*
 * Sparse operators for the layers around the dropout (Section 4.3, closing remark: the layer
 * directly before the dropout can use sparse operators as well).  None of this is part of
 * eq. (1)-(3); it is what lets a block  H -> act(H W0^T + b0) -> SparseDrop -> . W  run without
 * ever computing, storing or reading a dropped block, forward and backward.
 *
 * An element-wise tail on the fp32 accumulator, before the single rounding:
 *
 *     out = [relu_mask > 0] act(scale * acc + bias[column])
 *
 *   scale_mode  SDROP_SCALE_DROPOUT: scale = 1/(1-p), as in eq. (1)-(3)
 *               SDROP_SCALE_ONE:     scale = 1 (a masked product that is not a dropout's output)
 *   act         SDROP_ACT_NONE, SDROP_ACT_RELU (max(v,0)), SDROP_ACT_GELU_TANH
 *               (0.5 v (1 + tanh(sqrt(2/pi) (v + 0.044715 v^3))), the "tanh" form of GELU),
 *               SDROP_ACT_GELU_ERF (0.5 v (1 + erf(v / sqrt 2)), the exact form)
 *               (erf is evaluated in fp32 by a rational approximation whose absolute error is
 *               below 1e-6, exp and tanh by the hardware's fast forms: far inside the rounding of
 *               a 16-bit output)
 *   bias        device, fp32[number of output columns], 16-byte aligned, or NULL
 *   relu_mask   device, a matrix of type `dtype` with the output's shape (and the output's
 *               leading dimension), 16-byte aligned, or NULL: where it is not > 0 the output is
 *               +-0 (the backward of a ReLU, given the ReLU's output).  Its dropped blocks are
 *               never read.
 *   gate_mode   what relu_mask does.  SDROP_GATE_RELU (0): as above.  SDROP_GATE_GELU_TANH /
 *               SDROP_GATE_GELU_ERF: the output is multiplied by the derivative of that GELU at
 *               relu_mask, which then holds the GELU's INPUT (the backward of a GELU; the second
 *               output of sdrop_producer is that input)
 *   kept_fraction   0, or the share of kept blocks the caller expects the mask to have, in (0,1].  Used only to choose
 *               tile shapes and kernel forms (never the result): the library plans by 1 - p, which a mask built by
 *               sdrop_mask_from_bits from the caller's own bits need not have.  Outside [0,1]: SDROP_EINVAL.
 *   ld_a, ld_b, ld_out   leading dimensions, in elements, of the first matrix argument, the
 *               second one and the output (row r starts r * ld elements after the pointer);
 *               0 = contiguous.  A leading dimension must be at least the number of columns, a
 *               multiple of 8 and at most 2^24, else SDROP_ESHAPE.  This is how a column range
 *               of a wider matrix (a slice of a fused QKV or gate/up projection, a padded buffer)
 *               is passed without a copy.  sdrop_bwd_dw_ex takes them too.
 *
 * sdrop_fwd_ex / sdrop_bwd_dx_ex / sdrop_bwd_dw_ex are sdrop_fwd / sdrop_bwd_dx / sdrop_bwd_dw
 * with such a tail (epi = NULL: exactly those).  sdrop_bwd_dw_ex takes scale_mode and the leading
 * dimensions only and returns SDROP_EINVAL for a bias, an activation or a relu_mask; bad enum values give SDROP_EINVAL, a misaligned bias
 * or relu_mask SDROP_EALIGN.  Dropped blocks of sdrop_bwd_dx_ex's output are +0 whatever the tail.
 */
enum { SDROP_SCALE_DROPOUT = 0, SDROP_SCALE_ONE = 1 };
enum { SDROP_ACT_NONE = 0, SDROP_ACT_RELU = 1, SDROP_ACT_GELU_TANH = 2, SDROP_ACT_GELU_ERF = 3 };
enum { SDROP_GATE_RELU = 0, SDROP_GATE_GELU_TANH = 1, SDROP_GATE_GELU_ERF = 2 };
/* Layout of the weight of eq. (1)-(3).  SDROP_W_KN: W[K,N] as Section 3.1 writes it.  SDROP_W_NK: Wt[N,K], one row
 * per output feature (the [out, in] layout of common frameworks): sdrop_fwd_ex and sdrop_bwd_dx_ex then take Wt as
 * their second operand (ld_b >= K), sdrop_bwd_dw_ex delivers the gradient as dWt[N,K] (ld_out >= K).  Without a tail
 * the array is read (written) in place where the product's kernel has a form for it: eq. 1 when N is a multiple of
 * 256; eq. 3 when N is a multiple of 256 (with BK = 64 only where its kept lists are long enough for the persistent
 * kernel); eq. 2 with 128 x 128 blocks when N is a multiple of 64 and the
 * call would compute single kept blocks or pairs.  Every other call transposes the weight into the workspace by a pass
 * of its own before the product (the gradient after it).  The results are the same bits either way, and
 * sdrop_workspace_bytes_ex gives the (larger) workspace that covers both. */
enum { SDROP_W_KN = 0, SDROP_W_NK = 1 };

typedef struct sdrop_epilogue {
    int32_t scale_mode;
    int32_t act;
    const float *bias;
    const void *relu_mask;
    int64_t ld_a, ld_b, ld_out;
    int32_t gate_mode;
    int32_t w_layout;
    double kept_fraction;
} sdrop_epilogue_t;

/* sdrop_workspace_bytes for an _ex call with this tail (epi may be NULL: then exactly sdrop_workspace_bytes). */
size_t sdrop_workspace_bytes_ex(int op, int64_t M, int64_t K, int64_t N, int BM, int BK,
                                int dtype, int out_dtype, const sdrop_epilogue_t *epi);

int sdrop_fwd_ex(const void *X, const void *W, const void *mask, void *Y,
                 int64_t M, int64_t K, int64_t N, int BM, int BK, double p,
                 int dtype, int out_dtype, void *ws, size_t ws_bytes, void *stream,
                 const sdrop_epilogue_t *epi);
int sdrop_bwd_dx_ex(const void *dY, const void *W, const void *mask, void *dX,
                    int64_t M, int64_t K, int64_t N, int BM, int BK, double p,
                    int dtype, int out_dtype, void *ws, size_t ws_bytes, void *stream,
                    const sdrop_epilogue_t *epi);
int sdrop_bwd_dw_ex(const void *X, const void *dY, const void *mask, void *dW,
                    int64_t M, int64_t K, int64_t N, int BM, int BK, double p,
                    int dtype, int out_dtype, void *ws, size_t ws_bytes, void *stream,
                    const sdrop_epilogue_t *epi);

/*
 * sdrop_fwd_seeded for row-strided matrices and for a weight given as [N,K]: of `epi` only w_layout, ld_a (X), ld_b (W)
 * and ld_out (Y) may be set (anything else: SDROP_EINVAL; epi = NULL: exactly sdrop_fwd_seeded).  ws, ws_bytes as for
 * sdrop_fwd_ex with the same epi (sdrop_workspace_bytes_ex(SDROP_OP_FWD, ...): nothing for [K,N] weights).  The mask
 * is drawn in the forward's launch on the same grids as in sdrop_fwd_seeded; an [N,K] weight is then read in place
 * when N is a multiple of 256, else the call is sdrop_mask followed by sdrop_fwd_ex.  Same bits as those two calls.
 */
int sdrop_fwd_seeded_ex(const void *X, const void *W, void *mask, size_t mask_bytes, void *Y,
                        int64_t M, int64_t K, int64_t N, int BM, int BK, double p, uint64_t seed, uint64_t rng_stream,
                        int dtype, int out_dtype, void *ws, size_t ws_bytes, void *stream,
                        const sdrop_epilogue_t *epi);


/*
 * The layer before the dropout as an output-sparse product: only the blocks of X that the
 * dropout keeps are computed; dropped blocks are written as +0.
 *
 *     X[M,K] = m' . act(H W0^T + b0)          Z[M,K] = m' . (H W0^T + b0)   (optional)
 *
 *   H[M,N0]   input of type `dtype`
 *   W0[K,N0]  the producing layer's weight, one ROW per output feature (the [out, in] layout)
 *   bias      device fp32[K] or NULL;  act as above;  mask over X[M,K] in BM x BK blocks
 *   Z         NULL, or a second output of X's shape and type that receives the value before the
 *             activation on the kept blocks (what the backward of a GELU needs); its dropped
 *             blocks are NOT written (nothing reads them)
 *   p         used only to choose tile shapes (the product is not scaled)
 * It is sdrop_bwd_dx_ex(H, W0, ...) with SDROP_SCALE_ONE: the same kernels.  Its backward uses
 * the other two (dZ = the gradient at the pre-activation, zero on dropped blocks):
 *     dH[M,N0]  = (dZ . m') W0      sdrop_fwd_ex(dZ, W0, mask, dH, M, K, N0, ..., SDROP_SCALE_ONE)
 *     dW0[K,N0] = (dZ . m')^T H     sdrop_bwd_dw_ex(dZ, H, mask, dW0, M, K, N0, ..., SDROP_SCALE_ONE)
 * and dZ itself comes from sdrop_bwd_dx_ex(dY, W, ...) with relu_mask = X for act = ReLU, or with
 * relu_mask = Z and the matching gate_mode for a GELU.
 */
int sdrop_producer(const void *H, const void *W0, const float *bias, const void *mask, void *X, void *Z,
                   int64_t M, int64_t N0, int64_t K, int BM, int BK, double p, int act,
                   int dtype, int out_dtype, void *stream);

/* sdrop_producer for row-strided matrices: leading dimensions of H[M,N0], W0[K,N0] and of X (and Z) [M,K], as above. */
int sdrop_producer_ex(const void *H, const void *W0, const float *bias, const void *mask, void *X, void *Z,
                      int64_t M, int64_t N0, int64_t K, int BM, int BK, double p, int act,
                      int dtype, int out_dtype, void *stream, int64_t ld_h, int64_t ld_w0, int64_t ld_out);

/*
 * Gradient of that layer's bias (the block of Section 4.3's closing remark, as above):
 *
 *     db[k] = sum over rows r of (dZ . m')[r, k]
 *
 * the column sums of dZ over the kept blocks; dropped blocks of dZ are not read.
 *
 *   dZ[M,K]   input of type `dtype` (fp16 / bf16), rows ld_dz elements apart (0 = K; else >= K, a
 *             multiple of 8)
 *   mask      the block mask over [M,K], as for the products
 *   db        device fp32[K], 16-byte aligned; every element is written (0 for a block column with
 *             no kept block)
 *   ws, ws_bytes  device workspace of at least sdrop_bias_grad_workspace_bytes(M, K, BM, BK) bytes
 *             (fp32 rows [parts][K] that a second launch adds in a fixed order: the result does not
 *             depend on scheduling); a function of the shape and of the device's CU count only
 * Sums are accumulated in fp32, in the kept list's order.  Errors as for the products; a mask
 * object built for another problem makes the kernels write nothing.
 */
size_t sdrop_bias_grad_workspace_bytes(int64_t M, int64_t K, int BM, int BK);
int sdrop_bias_grad(const void *dZ, const void *mask, float *db, int64_t M, int64_t K, int BM, int BK,
                    int dtype, int64_t ld_dz, void *ws, size_t ws_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SDROP_H */
