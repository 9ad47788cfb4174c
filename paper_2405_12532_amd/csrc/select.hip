// Stand-alone launch of the segmented top-k (Algorithm 1, TopP(A_e, p); see select_device.h):
// one workgroup of 1024 lanes per sequence.  Scores are staged in LDS when they fit (up to
// 36864 positions), otherwise every pass re-reads them from global memory (L2).
#include "select_device.h"

namespace pyr {
namespace {

constexpr int kThreads = 1024;
constexpr int kLdsKeys = 36864;            // 144 KiB of the 160 KiB LDS of a gfx950 compute unit

__global__ __launch_bounds__(kThreads) void select_topk_kernel(
    const float* __restrict__ scores, const int32_t* __restrict__ seq_offsets,
    const int32_t* __restrict__ keep_len, int32_t n_seqs, int32_t w, int32_t lds_cap,
    int32_t* __restrict__ kept_idx, int32_t* __restrict__ out_offsets) {
    extern __shared__ uint32_t lds_keys[];
    __shared__ SelectShared sh;
    select_sequence<kThreads>(blockIdx.x, scores, seq_offsets, keep_len, w, lds_keys, lds_cap, &sh, kept_idx, out_offsets);
}

}  // namespace

int launch_select(const float* scores, const int32_t* seq_offsets_dev, const int32_t* keep_len_dev,
                  int32_t n_seqs, int32_t max_seqlen, int32_t w, int32_t* kept_idx, int32_t* out_offsets_dev,
                  hipStream_t stream) {
    if (n_seqs == 0) return PYR_OK;
    int staged = max_seqlen < kLdsKeys ? max_seqlen : kLdsKeys;
    size_t lds_bytes = (size_t)staged * sizeof(uint32_t);
    static std::atomic<uint64_t> lds_set{0};          // the limit is raised once per device, to the most the kernel ever asks for
    if (ensure_dynamic_lds((const void*)select_topk_kernel, kLdsKeys * (int)sizeof(uint32_t), &lds_set) != PYR_OK)
        return PYR_ERR_LAUNCH;
    hipLaunchKernelGGL(select_topk_kernel, dim3(n_seqs), dim3(kThreads), lds_bytes, stream,
                       scores, seq_offsets_dev, keep_len_dev, n_seqs, w, (int32_t)staged, kept_idx, out_offsets_dev);
    return check_launch();
}

}  // namespace pyr
