// Bias gradient of the layer before the dropout (arxiv 2411.01238, Section 4.3, closing remark:
// sparse operators for the layer directly before the dropout).  With Z = H W0^T + b0 and
// X = m' . act(Z), only the kept blocks of Z reach the output, so
//
//     db0[k] = sum over rows r of (dZ . m')[r, k]
//
// where dZ is what eq. (2) with the activation's gate in its tail has written.  Memory-bound: the
// kept blocks of dZ are read once (dropped blocks are never touched), nothing else moves.
//
// One workgroup sums, for one block column, every `parts`-th kept block of that column's list, in
// list order; the 256 threads cover R rows x BK columns per step with 16-byte loads, each thread
// keeping 8 column sums in registers; the R row groups are then added in a fixed order through LDS.
// With more than one part the workgroups write fp32 rows [parts][K] into the workspace and a second
// launch adds them in order: the result does not depend on scheduling (no atomics).
#include "sdrop_internal.h"

namespace sdrop {
namespace {

template <class T> struct Vec8 { typedef __attribute__((__vector_size__(8 * sizeof(T)))) T type; };

// (the sums carry no scale, so the mask's dropout probability is not compared)
__device__ __forceinline__ bool header_matches(const MaskHeader *H, int64_t M, int64_t K, int BM, int BK, int *status)
{
    return mask_header_ok(H, M, K, BM, BK, false, 0.0, status);
}

// out[part][k], k in block column kb: sum of dZ[r][k] over the rows r of the kept blocks number
// part, part + parts, ... of column kb's list.  ld: elements per row of dZ.
template <class T, int BK>
__global__ __launch_bounds__(256) void colsum_parts_kernel(const T *dz, int64_t ld, const MaskHeader *H, const int32_t *col_ptr,
                                                           const int32_t *row_idx, float *out, int parts,
                                                           int64_t M, int64_t K, int BM, int *status)
{
    // like the GEMMs: write nothing when the mask was built for another problem
    if (!header_matches(H, M, K, BM, BK, status)) return;
    constexpr int L = BK / 8;         // threads per row (8 elements = 16 bytes each)
    constexpr int R = 256 / L;        // rows per step; divides 64, so it divides BM
    __shared__ float red[R][BK];
    const int kb = blockIdx.x / parts, part = blockIdx.x % parts;
    const int lane = threadIdx.x % L, rg = threadIdx.x / L;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    const int end = col_ptr[kb + 1];
    for (int j = col_ptr[kb] + part; j < end; j += parts) {
        const T *src = dz + ((int64_t)row_idx[j] * BM + rg) * ld + (int64_t)kb * BK + lane * 8;
#pragma unroll 4
        for (int r = 0; r < BM; r += R, src += (int64_t)R * ld) {
            const typename Vec8<T>::type v = *reinterpret_cast<const typename Vec8<T>::type *>(src);
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[i] += static_cast<float>(v[i]);
        }
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) red[rg][lane * 8 + i] = acc[i];
    __syncthreads();
    if (threadIdx.x < BK) {
        float t = 0.f;
        for (int g = 0; g < R; ++g) t += red[g][threadIdx.x];
        out[(int64_t)part * K + (int64_t)kb * BK + threadIdx.x] = t;
    }
}

// db[k] = part[0][k] + part[1][k] + ... in that order
__global__ __launch_bounds__(256) void colsum_reduce_kernel(const float *part, float *db, int parts, const MaskHeader *H,
                                                            int64_t M, int64_t K, int BM, int BK, int *status)
{
    if (!header_matches(H, M, K, BM, BK, status)) return;
    const int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (k >= K) return;
    // eight loads in flight, added in order
    float t = 0.f;
    int c = 0;
    for (; c + 8 <= parts; c += 8) {
        float v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = part[(int64_t)(c + i) * K + k];
#pragma unroll
        for (int i = 0; i < 8; ++i) t += v[i];
    }
    for (; c < parts; ++c) t += part[(int64_t)c * K + k];
    db[k] = t;
}

// Parts per block column: about four workgroups per compute unit in all, at most one part per
// block row (a part with no kept block only writes zeros).  A function of the shape and of the
// device's CU count, so that the workspace can be sized without the mask.
int colsum_parts(int64_t M, int64_t K, int BM, int BK)
{
    const int64_t MB = M / BM, KB = K / BK;
    int64_t parts = (4 * (int64_t)cu_count() + KB - 1) / KB;
    if (parts > MB) parts = MB;
    if (parts > 64) parts = 64;
    return parts < 1 ? 1 : (int)parts;
}

template <class T>
void launch_parts(const void *dz, int64_t ld, const MaskView &V, float *out, int parts, int64_t M, int64_t K, int BM, int BK, hipStream_t st)
{
    const dim3 grid((unsigned)((K / BK) * parts)), block(256);
    const T *src = static_cast<const T *>(dz);
    if (BK == 64)
        hipLaunchKernelGGL((colsum_parts_kernel<T, 64>), grid, block, 0, st, src, ld, V.hdr, V.col_ptr, V.row_idx, out, parts, M, K, BM, device_status_word());
    else
        hipLaunchKernelGGL((colsum_parts_kernel<T, 128>), grid, block, 0, st, src, ld, V.hdr, V.col_ptr, V.row_idx, out, parts, M, K, BM, device_status_word());
}

int check_shape(int64_t M, int64_t K, int BM, int BK)
{
    if (M <= 0 || K <= 0 || !block_size_ok(BM) || !block_size_ok(BK) || M % BM || K % BK) return SDROP_ESHAPE;
    if (M > (int64_t(1) << 30) || K > (int64_t(1) << 24)) return SDROP_ESHAPE;
    return SDROP_OK;
}

}  // namespace
}  // namespace sdrop

using namespace sdrop;

extern "C" {

size_t sdrop_bias_grad_workspace_bytes(int64_t M, int64_t K, int BM, int BK)
{
    if (check_shape(M, K, BM, BK) != SDROP_OK) return 0;
    const int parts = colsum_parts(M, K, BM, BK);
    return parts > 1 ? (size_t)parts * (size_t)K * sizeof(float) : 0;
}

int sdrop_bias_grad(const void *dZ, const void *mask, float *db, int64_t M, int64_t K, int BM, int BK,
                    int dtype, int64_t ld_dz, void *ws, size_t ws_bytes, void *stream)
{
    if (!dZ || !mask || !db) return SDROP_EINVAL;
    const int rc = check_shape(M, K, BM, BK);
    if (rc != SDROP_OK) return rc;
    if (dtype != SDROP_F16 && dtype != SDROP_BF16) return SDROP_EDTYPE;
    if ((reinterpret_cast<uintptr_t>(dZ) | reinterpret_cast<uintptr_t>(mask) | reinterpret_cast<uintptr_t>(db)) % 16) return SDROP_EALIGN;
    if (ld_dz != 0 && (ld_dz < K || ld_dz % 8 || ld_dz > (int64_t(1) << 24))) return SDROP_ESHAPE;
    const size_t need = sdrop_bias_grad_workspace_bytes(M, K, BM, BK);
    if (ws_bytes < need || (need && (!ws || reinterpret_cast<uintptr_t>(ws) % 16))) return SDROP_EWORKSPACE;
    sdrop_mask_layout_t L;
    const int rl = sdrop_mask_layout(M, K, BM, BK, &L);
    if (rl != SDROP_OK) return rl;
    const MaskView V = make_view(mask, L);
    const int parts = colsum_parts(M, K, BM, BK);
    const int64_t ld = ld_dz ? ld_dz : K;
    hipStream_t st = static_cast<hipStream_t>(stream);
    float *first = parts > 1 ? static_cast<float *>(ws) : db;
    if (dtype == SDROP_F16) launch_parts<_Float16>(dZ, ld, V, first, parts, M, K, BM, BK, st);
    else launch_parts<__bf16>(dZ, ld, V, first, parts, M, K, BM, BK, st);
    int rs = hip_status(hipGetLastError());
    if (rs != SDROP_OK || parts == 1) return rs;
    hipLaunchKernelGGL(colsum_reduce_kernel, dim3((unsigned)((K + 255) / 256)), dim3(256), 0, st,
                       static_cast<const float *>(ws), db, parts, V.hdr, M, K, BM, BK, device_status_word());
    return hip_status(hipGetLastError());
}

}  // extern "C"
