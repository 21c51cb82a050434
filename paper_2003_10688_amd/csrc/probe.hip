// Measured ceilings of the machine, for the roofline report: a plain device-to-device copy (what HBM delivers to the
// simplest possible kernel) and a register-resident MFMA loop (what the matrix cores deliver when nothing else is in
// the way).  Debug entry points; no layer arithmetic.
#include <algorithm>

#include "conv_common.h"

namespace sol {

// 16 bytes per lane and access, UN accesses in flight per lane, consecutive lanes on consecutive addresses
__global__ void __launch_bounds__(256) probe_copy_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, size_t n) {
    constexpr int UN = 4;
    const size_t stride = (size_t)gridDim.x * 256;
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    for (; i + (UN - 1) * stride < n; i += UN * stride) {
        uint4 v[UN];
#pragma unroll
        for (int u = 0; u < UN; u++) v[u] = src[i + u * stride];
#pragma unroll
        for (int u = 0; u < UN; u++) dst[i + u * stride] = v[u];
    }
    for (; i < n; i += stride) dst[i] = src[i];
}

// every wave: `iters` rounds of NACC independent v_mfma_f32_32x32x16_bf16 on operands that never leave registers
constexpr int PROBE_NACC = 4;
__global__ void __launch_bounds__(512) probe_mfma_kernel(float *sink, int iters) {
#if defined(__HIP_DEVICE_COMPILE__)
    f32x16_t acc[PROBE_NACC];
#pragma unroll
    for (int i = 0; i < PROBE_NACC; i++)
#pragma unroll
        for (int e = 0; e < 16; e++) acc[i][e] = 0.f;
    const uint4 a = make_uint4(0x3f803f80u + threadIdx.x, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u);   // bf16 values near 1
    const uint4 b = make_uint4(0x3c003c00u, 0x3c003c00u + threadIdx.x, 0x3c003c00u, 0x3c003c00u);   // ... near 2^-7
    for (int it = 0; it < iters; it++) {
#pragma unroll
        for (int i = 0; i < PROBE_NACC; i++) Mma<bf16_t>::run(acc[i], a, b);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < PROBE_NACC; i++)
#pragma unroll
        for (int e = 0; e < 16; e++) s += acc[i][e];
    if (s == 12345.678f) sink[0] = s;      // keeps the loop alive; practically never true
#endif
}

}  // namespace sol

using namespace sol;

extern "C" {

sol_status sol_debug_probe_copy(void *dst, const void *src, size_t bytes, void *stream) {
    SOL_REQUIRE(dst && src, SOL_ERR_NULL, "dst and src must not be NULL");
    SOL_REQUIRE(aligned16(dst) && aligned16(src) && bytes % 16 == 0, SOL_ERR_ALIGN, "16-byte aligned buffers and a multiple of 16 bytes");
    if (bytes == 0) return SOL_OK;
    const size_t n = bytes / 16;
    const int grid = (int)std::min<size_t>((n + 255) / 256, 256 * 16);
    hipLaunchKernelGGL(probe_copy_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream, static_cast<const uint4 *>(src),
                       static_cast<uint4 *>(dst), n);
    SOL_HIP(hipGetLastError());
    return SOL_OK;
}

sol_status sol_debug_probe_mfma(int iters, int workgroups, float *sink, double *flop, void *stream) {
    SOL_REQUIRE(sink && flop, SOL_ERR_NULL, "sink and flop must not be NULL");
    SOL_REQUIRE(iters > 0 && iters <= (1 << 24) && workgroups > 0 && workgroups <= (1 << 16), SOL_ERR_SHAPE, "iters %d / workgroups %d out of range", iters, workgroups);
    *flop = (double)workgroups * 8.0 * iters * PROBE_NACC * (2.0 * 32 * 32 * 16);
    hipLaunchKernelGGL(probe_mfma_kernel, dim3(workgroups), dim3(512), 0, (hipStream_t)stream, sink, iters);
    SOL_HIP(hipGetLastError());
    return SOL_OK;
}

}  // extern "C"
