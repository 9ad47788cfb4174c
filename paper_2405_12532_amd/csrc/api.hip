// C ABI of libpyr: argument checks on the host, then the launchers.  See include/pyr.h for
// the contract of every entry point (Algorithm 1 and Section 4.1 of the paper).
#include <math.h>

#include "pyr_internal.h"

// Device memory of pyr_prefill_layer_static: the workspace of one layer step, held by every GPU the
// library runs on until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress; kernels get the address that call returns (static_scratch()).
constexpr size_t kStaticScratchBytes = PYR_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

constexpr size_t kAlign = 256;
size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct BatchInfo {
    int32_t uniform_len;    // common length if all sequences have one (> 0), else 0
    int32_t max_len, min_len;
};

int check_shape(const pyr_shape* s) {
    if (s == nullptr) return PYR_ERR_NULL;
    if (s->n_seqs < 0 || s->total_tokens < 0 || s->max_seqlen < 0 || s->n_q_heads < 1 || s->n_kv_heads < 1)
        return PYR_ERR_SHAPE;
    if (s->max_seqlen > s->total_tokens) return PYR_ERR_SHAPE;
    if (s->head_dim != 64 && s->head_dim != 128) return PYR_ERR_UNSUPPORTED;
    if (s->n_q_heads % s->n_kv_heads != 0) return PYR_ERR_UNSUPPORTED;
    if (s->n_q_heads > 32767) return PYR_ERR_UNSUPPORTED;      // head numbers are packed into 16 bits, row strides into 24
    // the kernels index elements of q with 64-bit offsets, but row numbers stay 32-bit
    if ((int64_t)s->total_tokens * s->n_q_heads >= (int64_t)1 << 31) return PYR_ERR_UNSUPPORTED;
    return PYR_OK;
}

int check_offsets(const int32_t* off, int32_t n_seqs, int32_t total, int32_t max_len_claimed, BatchInfo* info) {
    if (off == nullptr) return PYR_ERR_NULL;
    if (off[0] != 0) return PYR_ERR_OFFSETS;
    int32_t max_len = 0, min_len = 0x7fffffff, first = n_seqs > 0 ? off[1] - off[0] : 0;
    bool uniform = n_seqs > 0;
    for (int32_t b = 0; b < n_seqs; ++b) {
        if (off[b + 1] < off[b]) return PYR_ERR_OFFSETS;
        const int32_t len = off[b + 1] - off[b];
        if (len > max_len) max_len = len;
        if (len < min_len) min_len = len;
        if (len != first) uniform = false;
    }
    if (off[n_seqs] != total) return PYR_ERR_OFFSETS;
    if (max_len_claimed >= 0 && max_len > max_len_claimed) return PYR_ERR_SHAPE;
    if (info != nullptr) {
        info->uniform_len = (uniform && first > 0) ? first : 0;
        info->max_len = max_len;
        info->min_len = n_seqs > 0 ? min_len : 0;
    }
    return PYR_OK;
}

int check_keep_len(const int32_t* keep, const int32_t* off, int32_t n_seqs, int32_t w, int64_t* total_kept) {
    if (keep == nullptr) return PYR_ERR_NULL;
    int64_t sum = 0;
    for (int32_t b = 0; b < n_seqs; ++b) {
        const int32_t len = off[b + 1] - off[b];
        const int32_t lo = w < len ? w : len;
        if (keep[b] < lo || keep[b] > len) return PYR_ERR_KEEP_LEN;
        sum += keep[b];
    }
    if (total_kept != nullptr) *total_kept = sum;
    return PYR_OK;
}

float scale_log2(float softmax_scale, int head_dim) {
    const float s = softmax_scale > 0.f ? softmax_scale : 1.0f / sqrtf((float)head_dim);
    return s * pyr::kLog2e;
}

bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

// Address of `scratch` on the current device, looked up once per device (every GPU has its own copy of
// the array at its own address); nullptr if the runtime cannot resolve it.
void* static_scratch() {
    constexpr int kMaxDevices = 64;
    static std::atomic<void*> ptrs[kMaxDevices];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    void* p = ptrs[dev].load(std::memory_order_acquire);
    if (p == nullptr) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return nullptr;
        ptrs[dev].store(p, std::memory_order_release);
    }
    return p;
}

}  // namespace

extern "C" {

const char* pyr_strerror(int status) {
    switch (status) {
        case PYR_OK: return "ok";
        case PYR_ERR_NULL: return "a required pointer is NULL";
        case PYR_ERR_SHAPE: return "negative or inconsistent sizes";
        case PYR_ERR_UNSUPPORTED: return "unsupported head_dim, head grouping, row size or alignment";
        case PYR_ERR_KEEP_LEN: return "keep_len outside [min(w, S), S]";
        case PYR_ERR_OFFSETS: return "seq_offsets not 0-based, not monotone or not ending at total_tokens";
        case PYR_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case PYR_ERR_LAUNCH: return "HIP launch failed";
        case PYR_ERR_TOO_LARGE: return "the step needs more workspace than the library's static buffer holds";
        default: return "unknown pyr status";
    }
}

int pyr_version(void) { return 200; }

int pyr_workspace_bytes(const pyr_shape* shape, int32_t w, size_t* bytes_out) {
    if (bytes_out == nullptr) return PYR_ERR_NULL;
    const int rc = check_shape(shape);
    if (rc != PYR_OK) return rc;
    if (w < 1) return PYR_ERR_SHAPE;
    *bytes_out = align_up((size_t)shape->total_tokens * shape->n_q_heads * sizeof(float)) +
                 align_up(((size_t)shape->n_seqs + 1) * sizeof(int32_t)) + align_up(pyr::score_tail_bytes(*shape));
    return PYR_OK;
}

int pyr_schedule_next(int32_t S, int32_t w, int32_t num, int32_t den, int32_t floor_len, int32_t* keep_len_out) {
    if (keep_len_out == nullptr) return PYR_ERR_NULL;
    if (S < 0 || w < 1 || den <= 0 || num < 0 || num > den || floor_len < 0) return PYR_ERR_SHAPE;
    int64_t k = ((int64_t)num * S + den / 2) / den;
    const int64_t recent = w < S ? w : S;
    if (k < floor_len) k = floor_len;
    if (k < recent) k = recent;
    if (k > S) k = S;
    *keep_len_out = (int32_t)k;
    return PYR_OK;
}

int pyr_schedule_plan(int32_t S, int32_t w, int32_t n_layers, const int32_t* num, int32_t den, const int32_t* floor_len,
                      int32_t context_relative, int32_t* len_out) {
    if (len_out == nullptr || (n_layers > 0 && (num == nullptr || floor_len == nullptr))) return PYR_ERR_NULL;
    if (S < 0 || w < 1 || den <= 0 || n_layers < 0) return PYR_ERR_SHAPE;
    len_out[0] = S;
    for (int32_t l = 0; l < n_layers; ++l) {
        if (num[l] < 0 || num[l] > den || floor_len[l] < 0) return PYR_ERR_SHAPE;
        const int64_t recent = w < S ? w : S;
        int64_t k = context_relative ? recent + ((int64_t)num[l] * (S - recent) + den / 2) / den
                                     : ((int64_t)num[l] * S + den / 2) / den;
        if (k < floor_len[l]) k = floor_len[l];
        if (k < recent) k = recent;
        if (k > S) k = S;
        S = (int32_t)k;
        len_out[l + 1] = S;
    }
    return PYR_OK;
}

int pyr_attention(const void* q, const void* k, const void* v,
                  const int32_t* seq_offsets_dev, const int32_t* seq_offsets_host,
                  const pyr_shape* shape, float softmax_scale,
                  void* out, float* lse, int32_t* tile_map, void* stream) {
    int rc = check_shape(shape);
    if (rc != PYR_OK) return rc;
    if (!q || !k || !v || !out || !seq_offsets_dev || !seq_offsets_host) return PYR_ERR_NULL;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out)) return PYR_ERR_UNSUPPORTED;
    BatchInfo info;
    rc = check_offsets(seq_offsets_host, shape->n_seqs, shape->total_tokens, shape->max_seqlen, &info);
    if (rc != PYR_OK) return rc;
    if (info.uniform_len == 0 && shape->total_tokens > 0 && tile_map == nullptr) return PYR_ERR_WORKSPACE;
    return pyr::launch_attention(q, k, v, seq_offsets_dev, seq_offsets_host, *shape, info.uniform_len,
                                 scale_log2(softmax_scale, shape->head_dim), out, lse, tile_map, nullptr, 0,
                                 (hipStream_t)stream);
}

int pyr_score_weighted(const void* q, const void* k, const float* lse,
                       const int32_t* seq_offsets_dev, const int32_t* seq_offsets_host,
                       const pyr_shape* shape, int32_t w, float softmax_scale,
                       const float* row_weights_dev, float* scores, void* stream) {
    int rc = check_shape(shape);
    if (rc != PYR_OK) return rc;
    if (w < 1) return PYR_ERR_SHAPE;
    if (!q || !k || !lse || !scores || !seq_offsets_dev || !seq_offsets_host) return PYR_ERR_NULL;
    if (!aligned16(q) || !aligned16(k)) return PYR_ERR_UNSUPPORTED;
    BatchInfo info;
    rc = check_offsets(seq_offsets_host, shape->n_seqs, shape->total_tokens, shape->max_seqlen, &info);
    if (rc != PYR_OK) return rc;
    pyr_shape s = *shape;
    s.max_seqlen = info.max_len;
    return pyr::launch_score(q, k, lse, seq_offsets_dev, s, info.min_len, w, scale_log2(softmax_scale, shape->head_dim),
                             row_weights_dev, scores, (hipStream_t)stream);
}

int pyr_score(const void* q, const void* k, const float* lse,
              const int32_t* seq_offsets_dev, const int32_t* seq_offsets_host,
              const pyr_shape* shape, int32_t w, float softmax_scale,
              float* scores, void* stream) {
    return pyr_score_weighted(q, k, lse, seq_offsets_dev, seq_offsets_host, shape, w, softmax_scale, nullptr, scores,
                              stream);
}

int pyr_select(const float* scores,
               const int32_t* seq_offsets_dev, const int32_t* seq_offsets_host,
               const int32_t* keep_len_dev, const int32_t* keep_len_host,
               int32_t n_seqs, int32_t w,
               int32_t* kept_idx, int32_t* out_offsets_dev, void* stream) {
    if (n_seqs < 0 || w < 1) return PYR_ERR_SHAPE;
    if (!scores || !seq_offsets_dev || !seq_offsets_host || !keep_len_dev || !keep_len_host || !kept_idx ||
        !out_offsets_dev)
        return PYR_ERR_NULL;
    BatchInfo info;
    int rc = check_offsets(seq_offsets_host, n_seqs, seq_offsets_host[n_seqs < 0 ? 0 : n_seqs], -1, &info);
    if (rc != PYR_OK) return rc;
    rc = check_keep_len(keep_len_host, seq_offsets_host, n_seqs, w, nullptr);
    if (rc != PYR_OK) return rc;
    return pyr::launch_select(scores, seq_offsets_dev, keep_len_dev, n_seqs, info.max_len, w, kept_idx,
                              out_offsets_dev, (hipStream_t)stream);
}

int pyr_compact2(const void* src0, void* dst0, const void* src1, void* dst1, size_t row_bytes,
                 const int32_t* kept_idx, int64_t n_kept, void* stream) {
    if (n_kept < 0) return PYR_ERR_SHAPE;
    if (n_kept == 0) return PYR_OK;
    if (!src0 || !dst0 || !src1 || !dst1 || !kept_idx) return PYR_ERR_NULL;
    if (row_bytes == 0 || row_bytes % 16 != 0 || row_bytes / 16 > 0x7fffffff) return PYR_ERR_UNSUPPORTED;
    if (!aligned16(src0) || !aligned16(dst0) || !aligned16(src1) || !aligned16(dst1)) return PYR_ERR_UNSUPPORTED;
    return pyr::launch_gather(src0, dst0, src1, dst1, row_bytes, kept_idx, n_kept, (hipStream_t)stream);
}

int pyr_compact(const void* src, size_t row_bytes, const int32_t* kept_idx, int64_t n_kept,
                void* dst, void* stream) {
    if (n_kept < 0) return PYR_ERR_SHAPE;
    if (n_kept == 0) return PYR_OK;
    if (!src || !dst || !kept_idx) return PYR_ERR_NULL;
    if (row_bytes == 0 || row_bytes % 16 != 0 || row_bytes / 16 > 0x7fffffff) return PYR_ERR_UNSUPPORTED;
    if (!aligned16(src) || !aligned16(dst)) return PYR_ERR_UNSUPPORTED;
    return pyr::launch_gather(src, dst, nullptr, nullptr, row_bytes, kept_idx, n_kept, (hipStream_t)stream);
}

int pyr_gather_positions(const int32_t* pos, const int32_t* kept_idx, int64_t n_kept, int32_t* pos_out, void* stream) {
    if (n_kept < 0) return PYR_ERR_SHAPE;
    if (n_kept == 0) return PYR_OK;
    if (!pos || !kept_idx || !pos_out) return PYR_ERR_NULL;
    return pyr::launch_gather_positions(pos, kept_idx, n_kept, pos_out, (hipStream_t)stream);
}

int pyr_prefill_layer(const void* q, const void* k, const void* v,
                      const int32_t* seq_offsets_dev, const int32_t* seq_offsets_host,
                      const pyr_shape* shape, int32_t w, float softmax_scale,
                      const int32_t* keep_len_dev, const int32_t* keep_len_host,
                      void* out, float* scores, int32_t* kept_idx, int32_t* out_offsets_dev,
                      void* k_out, void* v_out,
                      void* workspace, size_t workspace_bytes, void* stream) {
    return pyr_prefill_layer_ex(q, k, v, seq_offsets_dev, seq_offsets_host, shape, w, softmax_scale, keep_len_dev,
                                keep_len_host, nullptr, nullptr, out, scores, kept_idx, out_offsets_dev, k_out, v_out,
                                nullptr, workspace, workspace_bytes, stream);
}

int pyr_prefill_layer_ex(const void* q, const void* k, const void* v,
                      const int32_t* seq_offsets_dev, const int32_t* seq_offsets_host,
                      const pyr_shape* shape, int32_t w, float softmax_scale,
                      const int32_t* keep_len_dev, const int32_t* keep_len_host,
                      const float* row_weights_dev, const int32_t* pos,
                      void* out, float* scores, int32_t* kept_idx, int32_t* out_offsets_dev,
                      void* k_out, void* v_out, int32_t* pos_out,
                      void* workspace, size_t workspace_bytes, void* stream) {
    return pyr_prefill_layer_fused(q, k, v, seq_offsets_dev, seq_offsets_host, shape, w, softmax_scale, keep_len_dev,
                                   keep_len_host, row_weights_dev, nullptr, 0, pos, out, scores, kept_idx, out_offsets_dev,
                                   k_out, v_out, nullptr, pos_out, workspace, workspace_bytes, stream);
}

int pyr_prefill_layer_fused(const void* q, const void* k, const void* v,
                      const int32_t* seq_offsets_dev, const int32_t* seq_offsets_host,
                      const pyr_shape* shape, int32_t w, float softmax_scale,
                      const int32_t* keep_len_dev, const int32_t* keep_len_host,
                      const float* row_weights_dev, const void* hidden, size_t hidden_row_bytes, const int32_t* pos,
                      void* out, float* scores, int32_t* kept_idx, int32_t* out_offsets_dev,
                      void* k_out, void* v_out, void* hidden_out, int32_t* pos_out,
                      void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_shape(shape);
    if (rc != PYR_OK) return rc;
    if (w < 1) return PYR_ERR_SHAPE;
    if (!q || !k || !v || !out || !scores || !kept_idx || !out_offsets_dev || !seq_offsets_dev ||
        !seq_offsets_host || !keep_len_dev || !keep_len_host)
        return PYR_ERR_NULL;
    if ((k_out == nullptr) != (v_out == nullptr) || (pos == nullptr) != (pos_out == nullptr) ||
        (hidden == nullptr) != (hidden_out == nullptr))
        return PYR_ERR_NULL;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) || !aligned16(k_out) || !aligned16(v_out) ||
        !aligned16(hidden) || !aligned16(hidden_out))
        return PYR_ERR_UNSUPPORTED;
    if (hidden != nullptr && (hidden_row_bytes == 0 || hidden_row_bytes % 16 != 0 || hidden_row_bytes / 16 > 0x7fffffff))
        return PYR_ERR_UNSUPPORTED;
    BatchInfo info;
    rc = check_offsets(seq_offsets_host, shape->n_seqs, shape->total_tokens, shape->max_seqlen, &info);
    if (rc != PYR_OK) return rc;
    int64_t total_kept = 0;
    rc = check_keep_len(keep_len_host, seq_offsets_host, shape->n_seqs, w, &total_kept);
    if (rc != PYR_OK) return rc;
    size_t need = 0;
    rc = pyr_workspace_bytes(shape, w, &need);
    if (rc != PYR_OK) return rc;
    if (workspace == nullptr || ((uintptr_t)workspace % kAlign) != 0 || workspace_bytes < need) return PYR_ERR_WORKSPACE;

    // workspace: row statistics | tile map | the score pass's counters and partial sums
    float* lse = (float*)workspace;
    char* at = (char*)workspace + align_up((size_t)shape->total_tokens * shape->n_q_heads * sizeof(float));
    int32_t* tile_map = (int32_t*)at;
    at += align_up(((size_t)shape->n_seqs + 1) * sizeof(int32_t));
    void* tail_ws = at;
    hipStream_t st = (hipStream_t)stream;
    const float c = scale_log2(softmax_scale, shape->head_dim);
    pyr_shape s = *shape;
    s.max_seqlen = info.max_len;

    // four launches (five for a ragged batch: the tile map): attention, which also clears the counters of the
    // next one; the score pass; the selection; one gather for everything
    rc = pyr::launch_attention(q, k, v, seq_offsets_dev, seq_offsets_host, s, info.uniform_len, c, out, lse, tile_map,
                               (int32_t*)tail_ws, pyr::score_tail_counters(s), st);
    if (rc != PYR_OK) return rc;
    rc = pyr::launch_score_groups(q, k, lse, seq_offsets_dev, s, info.min_len, w, c, row_weights_dev, scores, tail_ws, st);
    if (rc != PYR_OK) return rc;
    rc = pyr::launch_select(scores, seq_offsets_dev, keep_len_dev, s.n_seqs, info.max_len, w, kept_idx, out_offsets_dev, st);
    if (rc != PYR_OK) return rc;
    if (total_kept > 0) {
        const void* srcs[3];
        void* dsts[3];
        size_t rows[3];
        int n = 0;
        if (k_out != nullptr) {
            const size_t kv_row = (size_t)shape->n_kv_heads * shape->head_dim * 2;
            srcs[n] = k; dsts[n] = k_out; rows[n++] = kv_row;
            srcs[n] = v; dsts[n] = v_out; rows[n++] = kv_row;
        }
        if (hidden != nullptr) { srcs[n] = hidden; dsts[n] = hidden_out; rows[n++] = hidden_row_bytes; }
        rc = pyr::launch_gather_multi(n, srcs, dsts, rows, pos, pos_out, kept_idx, total_kept, st);
    }
    return rc;
}

int pyr_prefill_layer_static(const void* q, const void* k, const void* v,
                             const int32_t* seq_offsets_dev, const int32_t* seq_offsets_host,
                             const pyr_shape* shape, int32_t w, float softmax_scale,
                             const int32_t* keep_len_dev, const int32_t* keep_len_host,
                             void* out, float* scores, int32_t* kept_idx, int32_t* out_offsets_dev,
                             void* k_out, void* v_out, void* stream) {
    size_t need = 0;
    const int rc = pyr_workspace_bytes(shape, w, &need);
    if (rc != PYR_OK) return rc;
    if (need > kStaticScratchBytes) return PYR_ERR_TOO_LARGE;
    void* ws = static_scratch();
    if (ws == nullptr) return PYR_ERR_LAUNCH;
    // Nothing in the workspace has to start at zero: the row statistics and the tile map are written in full
    // by the step's first kernels before anything reads them, so the last call's contents do not matter.
    return pyr_prefill_layer_ex(q, k, v, seq_offsets_dev, seq_offsets_host, shape, w, softmax_scale, keep_len_dev,
                                keep_len_host, nullptr, nullptr, out, scores, kept_idx, out_offsets_dev, k_out, v_out,
                                nullptr, ws, kStaticScratchBytes, stream);
}

int pyr_decode_workspace_bytes(const pyr_shape* shape, int32_t w, size_t* bytes_out) {
    if (bytes_out == nullptr) return PYR_ERR_NULL;
    const int rc = check_shape(shape);
    if (rc != PYR_OK) return rc;
    if (w < 1) return PYR_ERR_SHAPE;
    *bytes_out = align_up((size_t)shape->n_seqs * w * shape->n_q_heads * sizeof(float)) +
                 align_up(pyr::window_score_part_bytes(*shape, w));
    return PYR_OK;
}

int pyr_decode_update(const void* q_win, const void* k, const void* v,
                      const int32_t* seq_offsets_dev, const int32_t* seq_offsets_host,
                      const pyr_shape* shape, int32_t w, float softmax_scale,
                      const int32_t* keep_len_dev, const int32_t* keep_len_host,
                      const float* row_weights_dev, const int32_t* pos,
                      float* scores, int32_t* kept_idx, int32_t* out_offsets_dev,
                      void* k_out, void* v_out, int32_t* pos_out,
                      void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_shape(shape);
    if (rc != PYR_OK) return rc;
    if (w < 1) return PYR_ERR_SHAPE;
    if (!q_win || !k || !v || !scores || !kept_idx || !out_offsets_dev || !seq_offsets_dev || !seq_offsets_host ||
        !keep_len_dev || !keep_len_host)
        return PYR_ERR_NULL;
    if ((k_out == nullptr) != (v_out == nullptr) || (pos == nullptr) != (pos_out == nullptr)) return PYR_ERR_NULL;
    if (!aligned16(q_win) || !aligned16(k) || !aligned16(v) || !aligned16(k_out) || !aligned16(v_out))
        return PYR_ERR_UNSUPPORTED;
    BatchInfo info;
    rc = check_offsets(seq_offsets_host, shape->n_seqs, shape->total_tokens, shape->max_seqlen, &info);
    if (rc != PYR_OK) return rc;
    int64_t total_kept = 0;
    rc = check_keep_len(keep_len_host, seq_offsets_host, shape->n_seqs, w, &total_kept);
    if (rc != PYR_OK) return rc;
    size_t need = 0;
    rc = pyr_decode_workspace_bytes(shape, w, &need);
    if (rc != PYR_OK) return rc;
    if (workspace == nullptr || ((uintptr_t)workspace % kAlign) != 0 || workspace_bytes < need) return PYR_ERR_WORKSPACE;

    float* lse_win = (float*)workspace;
    void* part = (char*)workspace + align_up((size_t)shape->n_seqs * w * shape->n_q_heads * sizeof(float));
    hipStream_t st = (hipStream_t)stream;
    pyr_shape s = *shape;
    s.max_seqlen = info.max_len;
    rc = pyr::launch_window_score(q_win, k, seq_offsets_dev, s, info.min_len, w, scale_log2(softmax_scale, shape->head_dim),
                                  row_weights_dev, lse_win, part, scores, st);
    if (rc != PYR_OK) return rc;
    rc = pyr::launch_select(scores, seq_offsets_dev, keep_len_dev, s.n_seqs, info.max_len, w, kept_idx,
                            out_offsets_dev, st);
    if (rc != PYR_OK) return rc;
    if (total_kept > 0) {                             // K, V and the position ids in one launch
        const size_t row_bytes = (size_t)shape->n_kv_heads * shape->head_dim * 2;
        const void* srcs[2] = {k, v};
        void* dsts[2] = {k_out, v_out};
        const size_t rows[2] = {row_bytes, row_bytes};
        rc = pyr::launch_gather_multi(k_out != nullptr ? 2 : 0, srcs, dsts, rows, pos, pos_out, kept_idx, total_kept, st);
    }
    return rc;
}

}  // extern "C"
