// Measured ceilings for the benchmark report: what this very GPU sustains on nothing but bf16 MFMAs, and on
// nothing but reading HBM the way the score pass reads K.  (The copy ceiling is measured by the benchmark with a
// device-to-device copy of the framework it gets its buffers from.)  Not part of the method; exported so that
// bench.py can time them beside the published peaks.
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

// Nothing but LDS-direct loads, as the score pass issues them for K: two wavefronts per workgroup, three workgroups
// per compute unit (50 KB of LDS each), one 16 KB tile in flight per wavefront, requested again as soon as it has
// landed.  k_layout == 0: a wavefront reads consecutive 16 KB pieces; != 0: a tile is 64 rows of 256 bytes, 8 KB apart
// (one head of 64 tokens of a [T, 32, 128] bf16 K), the two wavefronts walk the 32 heads of the workgroup's 64 tokens.
constexpr int kStreamTile = 16384, kStreamTilesPerWave = 16, kStreamLds = 50 * 1024;

__global__ __launch_bounds__(128) void read_stream_kernel(const char* __restrict__ data, int k_layout, int* __restrict__ sink) {
    extern __shared__ __align__(1024) char stream_smem[];
    typedef __attribute__((address_space(3))) char* lptr_t;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lptr_t)stream_smem + wave * kStreamTile;
    const int ld_row = lane >> 4, ld_chunk = lane & 15;
    auto issue = [&](int t) {
        const char* base = k_layout ? data + (size_t)blockIdx.x * 64 * 8192 + (size_t)(wave + 2 * t) * 256
                                    : data + ((size_t)(blockIdx.x * 2 + wave) * kStreamTilesPerWave + t) * kStreamTile;
        const uint32_t stride = k_layout ? 8192 : 256;
        const uint64_t b64 = (uint64_t)(uintptr_t)base;                 // wave-uniform: into scalar registers
        const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)b64);
        const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(b64 >> 32));
        const char* b = (const char*)(uintptr_t)(((uint64_t)hi << 32) | lo);
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const uint32_t m0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)(lds0 + 1024 * i));
            const uint32_t voff = (uint32_t)(4 * i + ld_row) * stride + 16 * ld_chunk;
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(m0), "v"(voff), "s"(b) : "memory", "m0");
        }
    };
    issue(0);
    for (int t = 1; t < kStreamTilesPerWave; ++t) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        issue(t);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    if (data == nullptr) sink[0] = *(int*)stream_smem;                  // never true
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

extern "C" int pyr_diag_read_stream(const void* data_dev, size_t bytes, int32_t k_layout, int32_t* sink_dev, void* stream) {
    if (data_dev == nullptr || sink_dev == nullptr) return PYR_ERR_NULL;
    constexpr size_t kPerWorkgroup = (size_t)2 * pyr::kStreamTilesPerWave * pyr::kStreamTile;      // 512 KB
    if (bytes == 0 || bytes % kPerWorkgroup != 0 || bytes / kPerWorkgroup >= ((size_t)1 << 31)) return PYR_ERR_SHAPE;
    hipLaunchKernelGGL(pyr::read_stream_kernel, dim3((unsigned)(bytes / kPerWorkgroup)), dim3(128), pyr::kStreamLds,
                       (hipStream_t)stream, (const char*)data_dev, (int)k_layout, sink_dev);
    return pyr::check_launch();
}
