// Row gather: dst[j, :] = src[kept_idx[j], :]   (Algorithm 1, Gather(KV, index); the same
// kernel compacts the hidden rows that enter the next layer).
//
// Pure data movement, bound by HBM bandwidth: 2 * n_kept * row_bytes bytes move per source.
// One wavefront owns one output row; its 64 lanes move 16 bytes each per access, so a row is
// read and written in fully coalesced 1 KiB pieces, and up to kUnroll loads per lane are issued
// before the first store to keep enough bytes in flight per compute unit.  The grid has a
// wavefront per row (the stride loop only matters beyond 2^31 workgroups): workgroups start in
// index order, so the rows in flight at any moment are neighbours in memory, which HBM serves
// about a tenth faster than the far-apart rows a short grid with a stride loop has in flight
// (measured on an 8 KB-row copy of 1 GiB: 6.1-6.3 TB/s read + write against 5.5; two wavefronts
// per workgroup were the best of 1, 2, 4, 8, 16).
#include "pyr_internal.h"

namespace pyr {
namespace {

constexpr int kThreads = 128;
constexpr int kWavesPerBlock = kThreads / 64;
constexpr int kUnroll = 8;
constexpr int64_t kMaxBlocks = 0x7fffffff;      // gridDim.x limit; beyond it the kernels' stride loops take over

__global__ __launch_bounds__(kThreads) void gather_rows_kernel(
    const u32x4* __restrict__ src0, u32x4* __restrict__ dst0,
    const u32x4* __restrict__ src1, u32x4* __restrict__ dst1,
    const int32_t* __restrict__ kept_idx, int64_t n_rows, int32_t chunks_per_row) {
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const u32x4* __restrict__ src = blockIdx.y == 0 ? src0 : src1;
    u32x4* __restrict__ dst = blockIdx.y == 0 ? dst0 : dst1;
    const int64_t wave_stride = (int64_t)gridDim.x * kWavesPerBlock;
    for (int64_t j = (int64_t)blockIdx.x * kWavesPerBlock + wave; j < n_rows; j += wave_stride) {
        const int64_t from = (int64_t)kept_idx[j] * chunks_per_row;
        const int64_t to = j * chunks_per_row;
        for (int c0 = 0; c0 < chunks_per_row; c0 += 64 * kUnroll) {
            u32x4 buf[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int c = c0 + u * 64 + lane;
                if (c < chunks_per_row) buf[u] = __builtin_nontemporal_load(src + from + c);
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int c = c0 + u * 64 + lane;
                if (c < chunks_per_row) __builtin_nontemporal_store(buf[u], dst + to + c);
            }
        }
    }
}

// Several sources gathered with one index list in ONE launch (K, V, the hidden rows, the position ids): at small
// batch every launch costs about as much as the rows it moves (Appendix A.1 is about exactly this regime).
// blockIdx.y picks the source; the last y, if pos is given, gathers the 4-byte position ids.
struct GatherSources {
    const u32x4* src[3];
    u32x4* dst[3];
    int32_t chunks[3];                 // 16-byte chunks per row
    int32_t n;
    const int32_t* pos;
    int32_t* pos_out;
};

__global__ __launch_bounds__(kThreads) void gather_multi_kernel(GatherSources g, const int32_t* __restrict__ kept_idx,
                                                                int64_t n_rows) {
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int y = blockIdx.y;
    if (y >= g.n) {                    // position ids
        for (int64_t j = (int64_t)blockIdx.x * kThreads + threadIdx.x; j < n_rows; j += (int64_t)gridDim.x * kThreads)
            g.pos_out[j] = g.pos[kept_idx[j]];
        return;
    }
    const u32x4* __restrict__ src = y == 0 ? g.src[0] : y == 1 ? g.src[1] : g.src[2];
    u32x4* __restrict__ dst = y == 0 ? g.dst[0] : y == 1 ? g.dst[1] : g.dst[2];
    const int32_t chunks_per_row = y == 0 ? g.chunks[0] : y == 1 ? g.chunks[1] : g.chunks[2];
    const int64_t wave_stride = (int64_t)gridDim.x * kWavesPerBlock;
    for (int64_t j = (int64_t)blockIdx.x * kWavesPerBlock + wave; j < n_rows; j += wave_stride) {
        const int64_t from = (int64_t)kept_idx[j] * chunks_per_row;
        const int64_t to = j * chunks_per_row;
        for (int c0 = 0; c0 < chunks_per_row; c0 += 64 * kUnroll) {
            u32x4 buf[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int c = c0 + u * 64 + lane;
                if (c < chunks_per_row) buf[u] = __builtin_nontemporal_load(src + from + c);
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int c = c0 + u * 64 + lane;
                if (c < chunks_per_row) __builtin_nontemporal_store(buf[u], dst + to + c);
            }
        }
    }
}

// Position ids of the kept tokens (Appendix A.2: the survivors keep the position encodings
// they had; the ids are gathered with the same index as K and V): pos_out[j] = pos[kept_idx[j]].
__global__ __launch_bounds__(256) void gather_positions_kernel(const int32_t* __restrict__ pos,
                                                               const int32_t* __restrict__ kept_idx, int64_t n_kept,
                                                               int32_t* __restrict__ pos_out) {
    for (int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; j < n_kept; j += (int64_t)gridDim.x * blockDim.x)
        pos_out[j] = pos[kept_idx[j]];
}

}  // namespace

int launch_gather_positions(const int32_t* pos, const int32_t* kept_idx, int64_t n_kept, int32_t* pos_out,
                            hipStream_t stream) {
    if (n_kept == 0) return PYR_OK;
    int64_t blocks = (n_kept + 255) / 256;
    if (blocks > 256 * 8) blocks = 256 * 8;
    hipLaunchKernelGGL(gather_positions_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, pos, kept_idx, n_kept, pos_out);
    return check_launch();
}

int launch_gather_multi(int n, const void* const* srcs, void* const* dsts, const size_t* row_bytes, const int32_t* pos,
                        int32_t* pos_out, const int32_t* kept_idx, int64_t n_kept, hipStream_t stream) {
    if (n_kept == 0 || (n == 0 && pos == nullptr)) return PYR_OK;
    GatherSources g{};
    for (int i = 0; i < n; ++i) {
        g.src[i] = (const u32x4*)srcs[i];
        g.dst[i] = (u32x4*)dsts[i];
        g.chunks[i] = (int32_t)(row_bytes[i] / 16);
    }
    g.n = n;
    g.pos = pos;
    g.pos_out = pos_out;
    int64_t blocks = (n_kept + kWavesPerBlock - 1) / kWavesPerBlock;
    if (blocks > kMaxBlocks) blocks = kMaxBlocks;
    dim3 grid((unsigned)blocks, (unsigned)(n + (pos != nullptr ? 1 : 0)), 1);
    hipLaunchKernelGGL(gather_multi_kernel, grid, dim3(kThreads), 0, stream, g, kept_idx, n_kept);
    return check_launch();
}

int launch_gather(const void* src0, void* dst0, const void* src1, void* dst1, size_t row_bytes,
                  const int32_t* kept_idx, int64_t n_kept, hipStream_t stream) {
    if (n_kept == 0) return PYR_OK;
    const int32_t chunks = (int32_t)(row_bytes / 16);
    int64_t blocks = (n_kept + kWavesPerBlock - 1) / kWavesPerBlock;
    if (blocks > kMaxBlocks) blocks = kMaxBlocks;
    dim3 grid((unsigned)blocks, src1 != nullptr ? 2 : 1, 1);
    hipLaunchKernelGGL(gather_rows_kernel, grid, dim3(kThreads), 0, stream,
                       (const u32x4*)src0, (u32x4*)dst0, (const u32x4*)src1, (u32x4*)dst1,
                       kept_idx, n_kept, chunks);
    return check_launch();
}

}  // namespace pyr
