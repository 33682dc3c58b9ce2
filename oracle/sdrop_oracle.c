/*
 * sdrop_oracle.c -- slow, plain float64 CPU statement of what SparseDrop's
 * fused "block dropout + linear layer" computes.
 *
 * THIS IS TEST INFRASTRUCTURE.  It exists so that the HIP library can be
 * checked against something that is obviously the paper's definition.  Only
 * the tests, the smoke check and the benchmark's CPU-baseline leg may call it.
 * It shares no code, header, table or constant generator with the HIP path.
 *
 * What it follows (arxiv 2411.01238):
 *   - Section 3.1, eq. (1)-(3): Y = s (X.m) W,  dX = s (dY W^T).m,
 *     dW = s (X.m)^T dY, with s = 1/(1-p), X in R^{MxK}, W in R^{KxN},
 *     no bias.
 *   - Section 3.2: the mask is constant on Mblk x Kblk blocks of X, one
 *     Bernoulli(1-p) draw per block (1 = keep).
 *   - Section 2.2 footnote: block sizes divide the problem sizes.
 * Given the mask, the method reaches exactly (up to summation order) the
 * plain definition, so the oracle is the definition written out: an explicit
 * masked copy of X and dense triple loops.  Nothing is skipped, tiled, fused
 * or reordered.
 *
 * The paper does not say how the mask is drawn.  The convention of this
 * build (stated in the design notes as a reading, not a fact of the paper):
 *   Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11) with
 *     counter = (b lo32, b hi32, stream lo32, stream hi32), b = i*KB + j,
 *     key     = (seed lo32, seed hi32);
 *   r = output word 0;  T = floor(p * 2^32) as an integer in [0, 2^32];
 *   block (i,j) is kept  <=>  r >= T.
 *
 * Pins (tests/test_oracle_*.py): Philox known-answer vectors of the
 * generator's publication; counter/key placement through those same vectors;
 * p=0 against a library float64 matmul; hand-worked 2x2-block example;
 * central finite differences; adjoint identity; all-dropped gives zeros;
 * block linearity; Bernoulli rate concentration.  No function here is
 * "parity unpinned"; what no test can pin is the CHOICE of mask convention
 * itself, which is this build's and not the paper's.
 *
 * All matrices are dense row-major doubles.  16-bit inputs are widened to
 * double by the caller (exact).  Return value: 0 ok, -1 bad argument.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>

/* ---- Philox4x32-10 ------------------------------------------------------ */

/* One call of the generator: 10 rounds, key bumped between rounds. */
void sdo_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        if (round > 0) {
            k0 += 0x9E3779B9u;   /* golden ratio */
            k1 += 0xBB67AE85u;   /* sqrt(3) - 1 */
        }
        uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
        uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
        uint32_t n0 = hi1 ^ c1 ^ k0;
        uint32_t n1 = lo1;
        uint32_t n2 = hi0 ^ c3 ^ k1;
        uint32_t n3 = lo0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* The 32-bit uniform word that decides block number b. */
uint32_t sdo_block_word(uint64_t seed, uint64_t stream, uint64_t b)
{
    uint32_t ctr[4], key[2], out[4];
    ctr[0] = (uint32_t)(b & 0xFFFFFFFFu);
    ctr[1] = (uint32_t)(b >> 32);
    ctr[2] = (uint32_t)(stream & 0xFFFFFFFFu);
    ctr[3] = (uint32_t)(stream >> 32);
    key[0] = (uint32_t)(seed & 0xFFFFFFFFu);
    key[1] = (uint32_t)(seed >> 32);
    sdo_philox4x32_10(ctr, key, out);
    return out[0];
}

/* Drop threshold T = floor(p * 2^32); p must be in [0,1]. */
uint64_t sdo_threshold(double p)
{
    return (uint64_t)floor(p * 4294967296.0);
}

/*
 * Keep flags (1 = kept) for block rows [i0, i1) of an MB x KB block grid
 * (Section 3.2: one Bernoulli(1-p) per block).  keep has (i1-i0)*KB bytes.
 * The block number is always the global one, i*KB + j, so a row range
 * reproduces the matching slice of the whole mask.
 */
int sdo_mask_rows(int64_t i0, int64_t i1, int64_t KB, double p,
                  uint64_t seed, uint64_t stream, uint8_t *keep)
{
    if (!(p >= 0.0 && p <= 1.0) || i0 < 0 || i1 < i0 || KB <= 0 || !keep) return -1;
    uint64_t T = sdo_threshold(p);
    for (int64_t i = i0; i < i1; ++i)
        for (int64_t j = 0; j < KB; ++j) {
            uint64_t b = (uint64_t)i * (uint64_t)KB + (uint64_t)j;
            uint64_t r = sdo_block_word(seed, stream, b);
            keep[(i - i0) * KB + j] = (r >= T) ? 1 : 0;
        }
    return 0;
}

/*
 * Pack keep flags into 64-bit words, row by row: block j of row i is bit
 * (j mod 64) of word i*ceil(KB/64) + j/64; unused high bits are zero.
 * (Section 3.4 packs the mask bits as 64-bit integers; the bit order is this
 * build's reading.)
 */
int sdo_pack_bits(const uint8_t *keep, int64_t MB, int64_t KB, uint64_t *words)
{
    if (!keep || !words || MB <= 0 || KB <= 0) return -1;
    int64_t wpr = (KB + 63) / 64;
    for (int64_t w = 0; w < MB * wpr; ++w) words[w] = 0;
    for (int64_t i = 0; i < MB; ++i)
        for (int64_t j = 0; j < KB; ++j)
            if (keep[i * KB + j])
                words[i * wpr + j / 64] |= (uint64_t)1 << (j % 64);
    return 0;
}

/* ---- the three products -------------------------------------------------- */

static int shapes_ok(int64_t M, int64_t K, int64_t N, int64_t BM, int64_t BK, double p)
{
    if (M <= 0 || K <= 0 || N <= 0 || BM <= 0 || BK <= 0) return 0;
    if (M % BM || K % BK) return 0;               /* Section 2.2 footnote */
    if (!(p >= 0.0 && p <= 1.0)) return 0;
    return 1;
}

/* s = 1/(1-p); with p = 1 every block is dropped and s is taken as 0. */
static double scale_of(double p) { return (p < 1.0) ? 1.0 / (1.0 - p) : 0.0; }

/*
 * Xm = X (.) m' as an explicit M x K copy.  A dropped entry is exactly +0 and
 * is SELECTED, not multiplied, so a non-finite value in a dropped block does
 * not leak (Section 3.2: dropped blocks are not read at all).
 */
static double *masked_copy(const double *X, const uint8_t *keep,
                           int64_t M, int64_t K, int64_t BM, int64_t BK)
{
    int64_t KB = K / BK;
    double *Xm = (double *)malloc(sizeof(double) * (size_t)M * (size_t)K);
    if (!Xm) return NULL;
    #pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < M; ++r)
        for (int64_t c = 0; c < K; ++c)
            Xm[r * K + c] = keep[(r / BM) * KB + (c / BK)] ? X[r * K + c] : 0.0;
    return Xm;
}

/* eq. (1): Y[M,N] = s * (X (.) m') W */
int sdo_fwd(const double *X, const double *W, const uint8_t *keep,
            int64_t M, int64_t K, int64_t N, int64_t BM, int64_t BK, double p,
            double *Y)
{
    if (!X || !W || !keep || !Y || !shapes_ok(M, K, N, BM, BK, p)) return -1;
    double s = scale_of(p);
    double *Xm = masked_copy(X, keep, M, K, BM, BK);
    if (!Xm) return -1;
    #pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < M; ++r) {
        double *y = Y + r * N;
        for (int64_t c = 0; c < N; ++c) y[c] = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            double a = Xm[r * K + k];
            const double *w = W + k * N;
            for (int64_t c = 0; c < N; ++c) y[c] += a * w[c];
        }
        for (int64_t c = 0; c < N; ++c) y[c] *= s;
    }
    free(Xm);
    return 0;
}

/* eq. (2): dX[M,K] = s * (dY W^T) (.) m' ; dropped entries are exactly +0. */
int sdo_bwd_dx(const double *dY, const double *W, const uint8_t *keep,
               int64_t M, int64_t K, int64_t N, int64_t BM, int64_t BK, double p,
               double *dX)
{
    if (!dY || !W || !keep || !dX || !shapes_ok(M, K, N, BM, BK, p)) return -1;
    double s = scale_of(p);
    int64_t KB = K / BK;
    #pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < M; ++r) {
        for (int64_t k = 0; k < K; ++k) {
            const double *g = dY + r * N;
            const double *w = W + k * N;
            double acc = 0.0;
            for (int64_t c = 0; c < N; ++c) acc += g[c] * w[c];   /* (dY W^T)[r,k] */
            dX[r * K + k] = keep[(r / BM) * KB + (k / BK)] ? s * acc : 0.0;
        }
    }
    return 0;
}

/* eq. (3): dW[K,N] = s * (X (.) m')^T dY */
int sdo_bwd_dw(const double *X, const double *dY, const uint8_t *keep,
               int64_t M, int64_t K, int64_t N, int64_t BM, int64_t BK, double p,
               double *dW)
{
    if (!X || !dY || !keep || !dW || !shapes_ok(M, K, N, BM, BK, p)) return -1;
    double s = scale_of(p);
    double *Xm = masked_copy(X, keep, M, K, BM, BK);
    if (!Xm) return -1;
    #pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < K; ++k) {
        double *d = dW + k * N;
        for (int64_t c = 0; c < N; ++c) d[c] = 0.0;
        for (int64_t r = 0; r < M; ++r) {
            double a = Xm[r * K + k];                             /* (Xm^T)[k,r] */
            const double *g = dY + r * N;
            for (int64_t c = 0; c < N; ++c) d[c] += a * g[c];
        }
        for (int64_t c = 0; c < N; ++c) d[c] *= s;
    }
    free(Xm);
    return 0;
}

/* ---- single entries of the same three results ---------------------------- */
/*
 * For sizes where the whole product takes too long on a CPU, the same
 * definitions evaluated at n chosen (row, col) positions only.  Each entry is
 * the full inner product of eq. (1)/(2)/(3); nothing else changes.
 */
int sdo_fwd_at(const double *X, const double *W, const uint8_t *keep,
               int64_t M, int64_t K, int64_t N, int64_t BM, int64_t BK, double p,
               int64_t n, const int64_t *rows, const int64_t *cols, double *out)
{
    if (!X || !W || !keep || !out || !rows || !cols || n < 0 || !shapes_ok(M, K, N, BM, BK, p)) return -1;
    double s = scale_of(p);
    int64_t KB = K / BK;
    #pragma omp parallel for schedule(dynamic, 16)
    for (int64_t t = 0; t < n; ++t) {
        int64_t r = rows[t], c = cols[t];
        double acc = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            double a = keep[(r / BM) * KB + (k / BK)] ? X[r * K + k] : 0.0;
            acc += a * W[k * N + c];
        }
        out[t] = s * acc;
    }
    return 0;
}

int sdo_bwd_dx_at(const double *dY, const double *W, const uint8_t *keep,
                  int64_t M, int64_t K, int64_t N, int64_t BM, int64_t BK, double p,
                  int64_t n, const int64_t *rows, const int64_t *cols, double *out)
{
    if (!dY || !W || !keep || !out || !rows || !cols || n < 0 || !shapes_ok(M, K, N, BM, BK, p)) return -1;
    double s = scale_of(p);
    int64_t KB = K / BK;
    #pragma omp parallel for schedule(dynamic, 16)
    for (int64_t t = 0; t < n; ++t) {
        int64_t r = rows[t], k = cols[t];
        double acc = 0.0;
        for (int64_t c = 0; c < N; ++c) acc += dY[r * N + c] * W[k * N + c];
        out[t] = keep[(r / BM) * KB + (k / BK)] ? s * acc : 0.0;
    }
    return 0;
}

int sdo_bwd_dw_at(const double *X, const double *dY, const uint8_t *keep,
                  int64_t M, int64_t K, int64_t N, int64_t BM, int64_t BK, double p,
                  int64_t n, const int64_t *rows, const int64_t *cols, double *out)
{
    if (!X || !dY || !keep || !out || !rows || !cols || n < 0 || !shapes_ok(M, K, N, BM, BK, p)) return -1;
    double s = scale_of(p);
    int64_t KB = K / BK;
    #pragma omp parallel for schedule(dynamic, 4)
    for (int64_t t = 0; t < n; ++t) {
        int64_t k = rows[t], c = cols[t];
        double acc = 0.0;
        for (int64_t r = 0; r < M; ++r) {
            double a = keep[(r / BM) * KB + (k / BK)] ? X[r * K + k] : 0.0;
            acc += a * dY[r * N + c];
        }
        out[t] = s * acc;
    }
    return 0;
}

/* number of OpenMP threads the loops above will use (for the benchmark's report) */
#ifdef _OPENMP
#include <omp.h>
int sdo_threads(void) { return omp_get_max_threads(); }
#else
int sdo_threads(void) { return 1; }
#endif
