// Stand-alone probe (not part of libsdrop): what shader clock does an MI355X hold while its matrix
// cores run, alone and with the operand traffic a GEMM main loop needs?
//
// One workgroup of 4 wavefronts per CU, all CUs.  Every iteration is shaped like one 128x256x64
// slice of the library's main loop for one wavefront: 32 v_mfma_f32_32x32x16_bf16, optionally the
// 24 16-byte-per-lane operand reads from LDS that feed them, optionally 12 direct HBM->LDS loads
// (global_load_lds_dwordx4, 1 KiB each) from a buffer that stays in the L2s / Infinity Cache.
// Wavefront 0 of each workgroup reads the shader clock counter (s_memtime) and the constant
// 100 MHz counter (s_memrealtime) before and after the loop; their ratio is the clock in MHz.
//
// Build and run:  hipcc --offload-arch=gfx950 -O3 probe_clock.hip -o probe_clock && ./probe_clock
#include <hip/hip_runtime.h>
#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <vector>

#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); exit(1); } } while (0)

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) const void gbl_void;

constexpr int kLds = 3 * 49152;      // three stages of 48 KiB, as in the library's 128x256 tile
constexpr int kWgBytes = 49152;      // bytes a workgroup fetches per iteration

template <bool MFMA, bool LDSR, bool DMA>
__global__ __launch_bounds__(256) void probe(const char *g, size_t g_bytes, int iters, long long *ticks, float *sink)
{
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    // operands with the bit patterns of N(0,1) bf16 data (so that the multipliers see real toggling)
    for (int i = t; i < kLds / 4; i += 256) {
        unsigned h = (unsigned)i * 2654435761u + blockIdx.x;
        h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
        const unsigned lo = 0x3c00u + (h & 0x83ffu), hi = 0x3c00u + ((h >> 16) & 0x83ffu);   // |x| in [0.0078, 2), random sign
        ((unsigned *)smem)[i] = lo | (hi << 16);
    }
    __syncthreads();
    f32x16 acc[8];
#pragma unroll
    for (int a = 0; a < 8; ++a)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[a][r] = 0.f;
    bf16x8 fa[4], fb[2];
#pragma unroll
    for (int i = 0; i < 4; ++i) fa[i] = *(const bf16x8 *)(smem + (i * 64 + lane) * 16);
#pragma unroll
    for (int i = 0; i < 2; ++i) fb[i] = *(const bf16x8 *)(smem + 8192 + (i * 64 + lane) * 16);
    const size_t span = g_bytes - kWgBytes;
    size_t off = ((size_t)blockIdx.x * 1048576u) % span;
    long long c0 = 0, w0 = 0;
    if (t == 0) { c0 = clock64(); w0 = wall_clock64(); }
    for (int it = 0; it < iters; ++it) {
        char *stage = smem + (it % 3) * 49152;
        if (DMA) {
            const char *src = g + off + wave * 12288 + lane * 16;
#pragma unroll
            for (int u = 0; u < 12; ++u)
                __builtin_amdgcn_global_load_lds((gbl_void *)(src + u * 1024), (lds_void *)(stage + wave * 12288 + u * 1024), 16, 0, 0);
            off += kWgBytes;
            if (off >= span) off -= span;
        }
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            if (LDSR) {
                // 6 operand reads per 8 MFMAs, conflict-free (consecutive lanes, consecutive 16-byte slots)
                const char *rd = smem + ((it + 1) % 3) * 49152 + kk * 6144;
#pragma unroll
                for (int i = 0; i < 4; ++i) fa[i] = *(const bf16x8 *)(rd + (i * 64 + lane) * 16);
#pragma unroll
                for (int i = 0; i < 2; ++i) fb[i] = *(const bf16x8 *)(rd + 4096 + (i * 64 + lane) * 16);
            }
            if (MFMA) {
#pragma unroll
                for (int a = 0; a < 8; ++a) acc[a] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[a & 1], fa[a >> 1], acc[a], 0, 0, 0);
            } else if (LDSR) {
#pragma unroll
                for (int i = 0; i < 4; ++i) asm volatile("" ::"v"(fa[i]));
#pragma unroll
                for (int i = 0; i < 2; ++i) asm volatile("" ::"v"(fb[i]));
            }
        }
        if (DMA) __builtin_amdgcn_s_waitcnt(0x0070 | (0xf << 8) | 12);     // vmcnt(12): one iteration's loads in flight
        __syncthreads();
    }
    if (t == 0) {
        ticks[blockIdx.x * 2] = clock64() - c0;
        ticks[blockIdx.x * 2 + 1] = wall_clock64() - w0;
    }
    float s = 0.f;
#pragma unroll
    for (int a = 0; a < 8; ++a) s += acc[a][lane & 15];
    if (s == 12345.678f) sink[0] = s;      // keeps the accumulators alive
}

template <bool MFMA, bool LDSR, bool DMA> void run(const char *name, const char *g, size_t g_bytes, long long *d_ticks, float *d_sink, int ncu)
{
    const int iters = 20000;
    auto k = probe<MFMA, LDSR, DMA>;
    CK(hipFuncSetAttribute((const void *)k, hipFuncAttributeMaxDynamicSharedMemorySize, kLds));
    for (int rep = 0; rep < 2; ++rep) {                 // the first launch warms clocks and caches
        hipLaunchKernelGGL(k, dim3(ncu), dim3(256), kLds, 0, g, g_bytes, rep == 0 ? 2000 : iters, d_ticks, d_sink);
        CK(hipDeviceSynchronize());
    }
    std::vector<long long> h(2 * ncu);
    CK(hipMemcpy(h.data(), d_ticks, sizeof(long long) * 2 * ncu, hipMemcpyDeviceToHost));
    std::vector<double> mhz(ncu), us(ncu);
    for (int i = 0; i < ncu; ++i) { us[i] = h[2 * i + 1] / 100.0; mhz[i] = h[2 * i] / us[i]; }
    std::sort(mhz.begin(), mhz.end());
    std::sort(us.begin(), us.end());
    const double t_us = us[ncu / 2];
    const double tflops = MFMA ? 32.0 * 32768.0 * 4 * ncu * iters / t_us / 1e6 : 0.0;
    printf("%-44s clock %6.0f MHz (min %4.0f max %4.0f)  %7.1f clocks/iteration  %7.3f us/iteration", name, mhz[ncu / 2], mhz.front(), mhz.back(),
           mhz[ncu / 2] * t_us / iters, t_us / iters);
    if (MFMA) printf("  %7.1f TFLOP/s", tflops);
    if (DMA) printf("  %5.2f TB/s into LDS", (double)kWgBytes * ncu * iters / t_us / 1e6);
    printf("\n");
    fflush(stdout);
}

int main()
{
    int ncu = 0;
    CK(hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, 0));
    const size_t g_bytes = (size_t)64 << 20;
    char *g;
    CK(hipMalloc(&g, g_bytes));
    CK(hipMemset(g, 0x3c, g_bytes));
    long long *d_ticks;
    CK(hipMalloc(&d_ticks, sizeof(long long) * 2 * ncu));
    float *d_sink;
    CK(hipMalloc(&d_sink, 4));
    printf("%d CUs, one workgroup of 4 wavefronts each; an iteration = 32 MFMA 32x32x16 bf16 per wavefront (1024 clocks of issue)\n", ncu);
    run<true, false, false>("MFMA only (operands fixed in registers)", g, g_bytes, d_ticks, d_sink, ncu);
    run<false, true, false>("LDS operand reads only", g, g_bytes, d_ticks, d_sink, ncu);
    run<false, false, true>("direct loads only (48 KiB per CU-iteration)", g, g_bytes, d_ticks, d_sink, ncu);
    run<true, true, false>("MFMA + LDS operand reads", g, g_bytes, d_ticks, d_sink, ncu);
    run<true, false, true>("MFMA + direct loads", g, g_bytes, d_ticks, d_sink, ncu);
    run<true, true, true>("MFMA + LDS operand reads + direct loads", g, g_bytes, d_ticks, d_sink, ncu);
    return 0;
}
