// Measured ceilings for the benchmark report: what this very GPU sustains on nothing but bf16 MFMAs.
// (The copy ceiling is measured by the benchmark with a device-to-device copy of the framework it
// gets its buffers from.)  Not part of the method; exported so that bench.py can time it beside the
// published peak.
#include "pyr_internal.h"

namespace pyr {
namespace {

// Eight wavefronts per workgroup (two per SIMD), one workgroup per compute unit times four; every wavefront
// issues v_mfma_f32_32x32x16_bf16 back to back on four independent accumulators with constant operands.
__global__ __launch_bounds__(512, 2) void mfma_only_kernel(float* __restrict__ sink, int iters) {
    bf16x8 a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = (__bf16)(1.0f + 0.001f * (float)(threadIdx.x & 7));
        b[i] = (__bf16)0.5f;
    }
    f32x16 acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[j], 0, 0, 0);
    }
    float r = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j) r += acc[j][0];
    if (r == 12345.678f) sink[0] = r;                 // never true: keeps the loop alive without memory traffic
}

}  // namespace
}  // namespace pyr

extern "C" int pyr_diag_mfma_only(int32_t iters, float* sink_dev, void* stream, double* flops_out) {
    if (sink_dev == nullptr || flops_out == nullptr) return PYR_ERR_NULL;
    if (iters < 1) return PYR_ERR_SHAPE;
    pyr::DeviceInfo dev;
    if (pyr::device_info(&dev) != PYR_OK) return PYR_ERR_LAUNCH;
    const int grid = dev.compute_units * 4;
    hipLaunchKernelGGL(pyr::mfma_only_kernel, dim3(grid), dim3(512), 0, (hipStream_t)stream, sink_dev, iters);
    *flops_out = (double)grid * 8.0 * (double)iters * 16.0 * (2.0 * 32 * 32 * 16);
    return pyr::check_launch();
}
