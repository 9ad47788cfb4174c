// Internal declarations shared by the translation units of libpyr (not installed).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "../../include/pyr.h"

namespace pyr {

typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr float kLog2e = 1.4426950408889634f;

// Every launcher returns PYR_OK or PYR_ERR_LAUNCH; arguments are already validated.
int launch_gather(const void* src0, void* dst0, const void* src1, void* dst1, size_t row_bytes,
                  const int32_t* kept_idx, int64_t n_kept, hipStream_t stream);

// up to three row sources (row_bytes[i] a multiple of 16) and, if pos != nullptr, the position ids, in one launch
int launch_gather_multi(int n, const void* const* srcs, void* const* dsts, const size_t* row_bytes, const int32_t* pos,
                        int32_t* pos_out, const int32_t* kept_idx, int64_t n_kept, hipStream_t stream);

int launch_select(const float* scores, const int32_t* seq_offsets_dev, const int32_t* keep_len_dev,
                  int32_t n_seqs, int32_t max_seqlen, int32_t w, int32_t* kept_idx, int32_t* out_offsets_dev,
                  hipStream_t stream);

int launch_attention(const void* q, const void* k, const void* v, const int32_t* seq_offsets_dev,
                     const int32_t* seq_offsets_host, const pyr_shape& shape, int32_t uniform_len, float scale_log2,
                     void* out, float* lse, int32_t* item_map, int32_t* zero_ptr, int32_t zero_count,
                     hipStream_t stream);     // zero_ptr[0 .. zero_count) is cleared by the kernel (may be nullptr, 0)

// row_weights: device [w] or nullptr (uniform); min_seqlen: the shortest sequence (0 if not known)
int launch_score(const void* q, const void* k, const float* lse, const int32_t* seq_offsets_dev,
                 const pyr_shape& shape, int32_t min_seqlen, int32_t w, float scale_log2, const float* row_weights,
                 float* scores, hipStream_t stream);

// The score pass with its small-batch extra (see score.hip): the KV heads split over several workgroups per key
// block when the grid is small.  tail_ws: score_tail_bytes() bytes whose first score_tail_counters() int32 are zero
// at launch (the kernel leaves them zero).
size_t score_tail_bytes(const pyr_shape& shape);
int32_t score_tail_counters(const pyr_shape& shape);
int launch_score_groups(const void* q, const void* k, const float* lse, const int32_t* seq_offsets_dev,
                        const pyr_shape& shape, int32_t min_seqlen, int32_t w, float scale_log2,
                        const float* row_weights, float* scores, void* tail_ws, hipStream_t stream);

// Generation phase: the same scores from the window's own query buffer q_win [B, w, Hq, d]
// (right-aligned), three launches: per-block row statistics -> part, folded into lse_win
// [B, w, Hq], then the score pass.  part holds window_score_part_bytes() bytes.
size_t window_score_part_bytes(const pyr_shape& shape, int32_t w);
int launch_window_score(const void* q_win, const void* k, const int32_t* seq_offsets_dev, const pyr_shape& shape,
                        int32_t min_seqlen, int32_t w, float scale_log2, const float* row_weights, float* lse_win, void* part,
                        float* scores, hipStream_t stream);

int launch_gather_positions(const int32_t* pos, const int32_t* kept_idx, int64_t n_kept, int32_t* pos_out,
                            hipStream_t stream);

// Compute units and XCDs of the current device (cached per device); PYR_ERR_LAUNCH if the runtime
// cannot tell - the launchers do not guess.
struct DeviceInfo { int device, compute_units, xccs; };
int device_info(DeviceInfo* out);

// Raise a kernel's dynamic LDS limit to `bytes`, once per device (done_mask: one bit per device id).
int ensure_dynamic_lds(const void* kernel, int bytes, std::atomic<uint64_t>* done_mask);

inline int check_launch() { return hipGetLastError() == hipSuccess ? PYR_OK : PYR_ERR_LAUNCH; }

}  // namespace pyr
