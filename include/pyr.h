/*
 * pyr.h - C ABI of the MI355X (gfx950) prefill layer step of PyramidInfer
 * (arXiv 2405.12532, Algorithm 1 "One forward pass in PyramidInfer" and the
 * prefill paragraph of Section 4.1).
 *
 * One layer step, for every sequence of a packed batch:
 *   attention weights  ->  ensemble weights of the recent window  ->  TopP
 *   ->  Gather of K, V (and of the hidden rows that feed the next layer).
 *
 * Conventions that hold for every function below
 *   - returns PYR_OK (0) or a negative pyr_status; never throws;
 *   - arguments are checked on the host before anything is launched; a
 *     failed check launches nothing;
 *   - "dev" pointers are device (HBM) addresses, "host" pointers are ordinary
 *     host memory read during the call only; all buffers are caller-owned;
 *   - work is enqueued on `stream` (a hipStream_t passed as void*, NULL is the
 *     default stream); nothing synchronises the stream or the device and
 *     nothing allocates or frees device memory;
 *   - packed layouts, row-major, token-major, bfloat16 unless said otherwise:
 *       q, out : [T, Hq, d]      k, v : [T, Hkv, d]      hidden : [T, D]
 *     sequence b owns rows seq_offsets[b] .. seq_offsets[b+1]-1 (S_b rows);
 *     query head h reads key/value head h / (Hq / Hkv);
 *   - supported: d in {64, 128}, Hq % Hkv == 0, w >= 1, T < 2^31.
 */
#ifndef PYR_H
#define PYR_H

#include <stddef.h>
#include <stdint.h>

#if defined(__GNUC__)
#define PYR_API __attribute__((visibility("default")))
#else
#define PYR_API
#endif

#ifdef __cplusplus
extern "C" {
#endif

typedef enum pyr_status {
    PYR_OK = 0,
    PYR_ERR_NULL = -1,        /* a required pointer is NULL                               */
    PYR_ERR_SHAPE = -2,       /* negative / inconsistent sizes                            */
    PYR_ERR_UNSUPPORTED = -3, /* head_dim, head grouping or row size outside the set     */
    PYR_ERR_KEEP_LEN = -4,    /* keep_len[b] outside [min(w, S_b), S_b]                   */
    PYR_ERR_OFFSETS = -5,     /* seq_offsets not 0-based, not monotone, or != T at end    */
    PYR_ERR_WORKSPACE = -6,   /* workspace NULL, misaligned (256 B) or too small          */
    PYR_ERR_LAUNCH = -7,      /* the HIP runtime refused a launch (see hipGetLastError)   */
    PYR_ERR_TOO_LARGE = -8    /* needs more than PYR_STATIC_SCRATCH_BYTES of workspace     */
} pyr_status;

/* Size of the library's own workspace buffer (see pyr_prefill_layer_static). */
#define PYR_STATIC_SCRATCH_BYTES ((size_t)40 << 20)

typedef struct pyr_shape {
    int32_t n_seqs;       /* B                                   */
    int32_t total_tokens; /* T = sum of S_b                      */
    int32_t max_seqlen;   /* max S_b                             */
    int32_t n_q_heads;    /* Hq                                  */
    int32_t n_kv_heads;   /* Hkv                                 */
    int32_t head_dim;     /* d                                   */
} pyr_shape;

/* Text for a status code (static storage, never NULL). */
PYR_API const char* pyr_strerror(int status);

/* Library version, major*10000 + minor*100 + patch. */
PYR_API int pyr_version(void);

/*
 * Host only.  Bytes of device workspace pyr_prefill_layer needs for this
 * shape and window (row statistics of the softmax for the score pass, the
 * tile map of ragged batches, arrival counters and partial sums of the score
 * pass).  Align the buffer to 256 bytes.
 */
PYR_API int pyr_workspace_bytes(const pyr_shape* shape, int32_t w, size_t* bytes_out);

/*
 * Host only.  Retention count for the next layer (Algorithm 1: the ratio p is
 * reduced layer by layer, and a layer whose length is at or below the minimum
 * PvC length N_l is left alone):
 *   k = max(floor((num*S + den/2)/den), floor_len, min(w, S)), capped at S.
 * Errors: PYR_ERR_NULL, PYR_ERR_SHAPE (S < 0, w < 1, den <= 0, num < 0, num > den).
 */
PYR_API int pyr_schedule_next(int32_t S, int32_t w, int32_t num, int32_t den, int32_t floor_len,
                      int32_t* keep_len_out);

/*
 * Host only.  Lengths of one sequence through n_layers layers, each with its own ratio
 * num[l]/den and minimum PvC length floor_len[l] (Algorithm 1: input N = {N_0, ...} and a p
 * that decays from layer to layer - the caller chooses the sequence p_l, e.g. geometric or
 * one of the patterns of the decay ablation in Section 5):
 *   context_relative == 0:  k = floor((num[l]*S + den/2)/den)                 (as pyr_schedule_next)
 *   context_relative != 0:  k = L' + floor((num[l]*(S-L') + den/2)/den), L' = min(w,S)
 *                           (Algorithm 1 ranks the columns :-L only: p as a fraction of the context)
 * then k = max(k, floor_len[l], L') capped at S, and S <- k.
 *   len_out            host int32 [n_layers+1], written: len_out[0] = S, len_out[l+1] after layer l
 * Errors: PYR_ERR_NULL, PYR_ERR_SHAPE (as pyr_schedule_next, per layer; len_out is then partly written).
 */
PYR_API int pyr_schedule_plan(int32_t S, int32_t w, int32_t n_layers, const int32_t* num, int32_t den,
                      const int32_t* floor_len, int32_t context_relative, int32_t* len_out);

/*
 * Step 1 - attention weights applied to V (Algorithm 1, "compute attention
 * weights of KV"): causal softmax attention inside each sequence,
 *   out[i,h,:] = sum_{j<=i} softmax_j(scale * q[i,h,:].k[j,h/g,:]) v[j,h/g,:].
 * bf16 MFMA products, fp32 accumulation and fp32 online softmax.
 *   q, k, v            dev, in
 *   seq_offsets_dev    dev int32 [B+1];  seq_offsets_host  host copy of the same
 *   softmax_scale      <= 0 selects 1/sqrt(d)
 *   out                dev bf16 [T,Hq,d], written
 *   lse                dev fp32 [T,Hq], written: log2 of the softmax denominator of
 *                      every row, in the scaled base-2 domain,
 *                      lse[i,h] = log2(sum_j 2^(scale*log2(e)*s_ij)); may be NULL
 *   tile_map           dev int32 [B+1] scratch, written (prefix sums of query
 *                      tiles per sequence); part of the workspace
 */
PYR_API int pyr_attention(const void* q, const void* k, const void* v,
                  const int32_t* seq_offsets_dev, const int32_t* seq_offsets_host,
                  const pyr_shape* shape, float softmax_scale,
                  void* out, float* lse, int32_t* tile_map, void* stream);

/*
 * Step 2 - ensemble attention weights (Algorithm 1, A_e = weighted_avg(A[-L:, :-L]);
 * Section 3.2.1): for every key position t of every sequence
 *   scores[t] = 1/(Hq*L') * sum_h sum_{i=S-L'}^{S-1} A_h[i,t],   L' = min(w, S),
 * uniform weights, all S columns written (the last L' too), fixed summation
 * order (bit-reproducible).  Needs `lse` from pyr_attention.
 *   scores             dev fp32 [T], written
 */
PYR_API int pyr_score(const void* q, const void* k, const float* lse,
              const int32_t* seq_offsets_dev, const int32_t* seq_offsets_host,
              const pyr_shape* shape, int32_t w, float softmax_scale,
              float* scores, void* stream);

/*
 * Step 2 with averaging weights (Section 4.1, prefill phase: the ensemble is a weighted
 * average that may favour the more recent rows; the paper prints no weights, so they are
 * an argument):
 *   scores[t] = 1/Hq * sum_h sum_i omega_i A_h[i,t] / sum_i omega_i.
 *   row_weights_dev    dev fp32 [w], one weight per row of a full recent window in
 *                      position order (row_weights_dev[w-1]: the last token); a sequence
 *                      shorter than w uses the last S_b of them.  NULL = uniform, the
 *                      same as pyr_score.  The values are not checked (they live on the
 *                      device): they must be finite and >= 0, with a positive sum over
 *                      the rows in use, else the scores are undefined (NaN or inf).
 */
PYR_API int pyr_score_weighted(const void* q, const void* k, const float* lse,
                       const int32_t* seq_offsets_dev, const int32_t* seq_offsets_host,
                       const pyr_shape* shape, int32_t w, float softmax_scale,
                       const float* row_weights_dev, float* scores, void* stream);

/*
 * Step 3 - TopP (Algorithm 1, TopP(A_e, p) with a count: Section 3.1.1 calls p
 * a retention ratio): per sequence the keep_len[b]-L' context positions
 * (0 .. S_b-L'-1) with the largest score, ties to the lower position, plus the
 * last L' positions; ascending.  Exact on the fp32 values given.
 *   scores             dev fp32 [T], in, all values >= 0 and not NaN
 *   keep_len_dev       dev int32 [B];  keep_len_host  host copy, min(w,S_b) <= k_b <= S_b
 *   kept_idx           dev int32 [sum k_b], written: global packed row numbers
 *   out_offsets_dev    dev int32 [B+1], written: prefix sums of keep_len
 * A sequence of length 0 (keep_len 0) contributes nothing; with n_seqs == 0 nothing is launched
 * and nothing is written, out_offsets_dev[0] included.
 */
PYR_API int pyr_select(const float* scores,
               const int32_t* seq_offsets_dev, const int32_t* seq_offsets_host,
               const int32_t* keep_len_dev, const int32_t* keep_len_host,
               int32_t n_seqs, int32_t w,
               int32_t* kept_idx, int32_t* out_offsets_dev, void* stream);

/*
 * Steps 4/5 - Gather (Algorithm 1, PvC <- Gather(KV, index); Figure 2(c): the
 * next layer only computes the kept tokens): dst[j,:] = src[kept_idx[j],:]
 * for j < n_kept, byte-exact.
 *   src, dst           dev, rows of row_bytes bytes (a multiple of 16, both
 *                      16-byte aligned), dst must not overlap src
 *   kept_idx           dev int32 [n_kept], every value a valid row of src
 *   n_kept == 0 is a no-op.
 */
PYR_API int pyr_compact(const void* src, size_t row_bytes, const int32_t* kept_idx, int64_t n_kept,
                void* dst, void* stream);

/* Same as two pyr_compact calls with one index list, in a single launch (K and V). */
PYR_API int pyr_compact2(const void* src0, void* dst0, const void* src1, void* dst1, size_t row_bytes,
                 const int32_t* kept_idx, int64_t n_kept, void* stream);

/*
 * Position ids of the kept tokens (Appendix A.2, the "gather" strategy of Table 5: the
 * survivors keep the position encodings they had instead of being renumbered):
 *   pos_out[j] = pos[kept_idx[j]]  for j < n_kept.
 *   pos                dev int32, indexed by packed row; pos_out dev int32 [n_kept], written
 *   kept_idx           dev int32 [n_kept], every value a valid row of pos
 * Carried through every layer, pos_out names each row's place in the original prompt.
 * n_kept == 0 is a no-op.
 */
PYR_API int pyr_gather_positions(const int32_t* pos, const int32_t* kept_idx, int64_t n_kept,
                         int32_t* pos_out, void* stream);

/*
 * The whole layer step (Algorithm 1, body of the loop, prefill phase): what
 * pyr_attention -> pyr_score -> pyr_select -> pyr_compact2 compute, on one stream
 * (see pyr_prefill_layer_fused for how the launches are merged).
 *   scores             dev fp32 [T], written (required: the selection reads it)
 *   k_out, v_out       dev bf16 [sum k_b, Hkv, d]; both NULL skips the gather
 *   workspace          dev, >= pyr_workspace_bytes(), 256-byte aligned
 */
PYR_API int pyr_prefill_layer(const void* q, const void* k, const void* v,
                      const int32_t* seq_offsets_dev, const int32_t* seq_offsets_host,
                      const pyr_shape* shape, int32_t w, float softmax_scale,
                      const int32_t* keep_len_dev, const int32_t* keep_len_host,
                      void* out, float* scores, int32_t* kept_idx, int32_t* out_offsets_dev,
                      void* k_out, void* v_out,
                      void* workspace, size_t workspace_bytes, void* stream);

/*
 * pyr_prefill_layer for callers that cannot hand over a workspace they allocated: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments without
 * `workspace`; the workspace is a buffer inside the library's device image instead
 * (PYR_STATIC_SCRATCH_BYTES = 40 MiB per GPU the library runs on, held until the process ends;
 * enough for every shape with pyr_workspace_bytes() <= 40 MiB, i.e. T*Hq <= about 10.4 M rows x heads:
 * 64 x 2048 tokens x 32 heads uses 16 MiB, 4 x 32768 x 64 heads 32 MiB).  The call allocates
 * and frees nothing; the first call on a device looks the buffer's address up.
 *   - a larger step returns PYR_ERR_TOO_LARGE and launches nothing;
 *   - all calls on one GPU share the buffer: calls that overlap in time on one GPU (different
 *     streams or threads) race; serialise them or use pyr_prefill_layer with separate workspaces;
 *   - results are identical to pyr_prefill_layer's.
 */
PYR_API int pyr_prefill_layer_static(const void* q, const void* k, const void* v,
                      const int32_t* seq_offsets_dev, const int32_t* seq_offsets_host,
                      const pyr_shape* shape, int32_t w, float softmax_scale,
                      const int32_t* keep_len_dev, const int32_t* keep_len_host,
                      void* out, float* scores, int32_t* kept_idx, int32_t* out_offsets_dev,
                      void* k_out, void* v_out, void* stream);

/*
 * The same with the two optional extras: averaging weights for step 2 (see
 * pyr_score_weighted; NULL = uniform) and position ids gathered alongside K and V
 * (see pyr_gather_positions; pos and pos_out both NULL skips it).
 */
PYR_API int pyr_prefill_layer_ex(const void* q, const void* k, const void* v,
                      const int32_t* seq_offsets_dev, const int32_t* seq_offsets_host,
                      const pyr_shape* shape, int32_t w, float softmax_scale,
                      const int32_t* keep_len_dev, const int32_t* keep_len_host,
                      const float* row_weights_dev, const int32_t* pos,
                      void* out, float* scores, int32_t* kept_idx, int32_t* out_offsets_dev,
                      void* k_out, void* v_out, int32_t* pos_out,
                      void* workspace, size_t workspace_bytes, void* stream);

/*
 * The whole layer step in as few launches as it takes (Appendix A.1 and the Limitations section: at small
 * batch the cost of selecting the PvC eats the gain - there every launch counts): attention; the score pass,
 * in which, when the batch is too small to fill the chip with one workgroup per 64 keys, the KV heads are
 * split over several workgroups whose partial sums the last of them adds in a fixed order; the selection;
 * ONE gather for K, V, the hidden rows and the position ids.
 * pyr_prefill_layer and pyr_prefill_layer_ex are this call without the hidden rows.
 *   hidden             dev, rows of hidden_row_bytes bytes (a multiple of 16) indexed by packed row; hidden_out
 *                      dev [sum k_b rows], written; both NULL skips them
 *   everything else as in pyr_prefill_layer_ex; results are those of the separate calls (scores may differ in
 *   the last bit when the heads are split: the partial sums are rounded once more).
 */
PYR_API int pyr_prefill_layer_fused(const void* q, const void* k, const void* v,
                      const int32_t* seq_offsets_dev, const int32_t* seq_offsets_host,
                      const pyr_shape* shape, int32_t w, float softmax_scale,
                      const int32_t* keep_len_dev, const int32_t* keep_len_host,
                      const float* row_weights_dev, const void* hidden, size_t hidden_row_bytes, const int32_t* pos,
                      void* out, float* scores, int32_t* kept_idx, int32_t* out_offsets_dev,
                      void* k_out, void* v_out, void* hidden_out, int32_t* pos_out,
                      void* workspace, size_t workspace_bytes, void* stream);

/*
 * Generation-phase update of one layer's compressed cache (Algorithm 1 with a non-empty
 * cache, KV = cat(PvC_past, KV); Section 4.1, generation phase: the recent window slides
 * over the generated tokens and the PvC is selected again with the prefill phase's
 * operation; with a constant keep_len the cache stays at a fixed size for any input length).
 *   k, v               dev bf16 [T,Hkv,d]: the packed caches with the new tokens' rows
 *                      already appended - per sequence its kept context rows, then its
 *                      recent rows, S_b rows in all (seq_offsets as elsewhere)
 *   q_win              dev bf16 [B,w,Hq,d]: the queries of the recent rows, right-aligned:
 *                      q_win[b,w-1] belongs to the newest token (cache row S_b-1); a
 *                      sequence with S_b < w uses the last S_b slots, the others are not read
 *   row_weights_dev    as in pyr_score_weighted, NULL = uniform;  pos / pos_out as in
 *                      pyr_prefill_layer_ex, both NULL skips them
 *   scores             dev fp32 [T], written: window row i (cache row S_b-L'+i) sees the
 *                      cache rows 0 .. S_b-L'+i; otherwise as pyr_score
 *   kept_idx, out_offsets_dev, k_out, v_out: as in pyr_prefill_layer (out of place: k_out
 *                      must not overlap k)
 *   workspace          dev, >= pyr_decode_workspace_bytes(), 256-byte aligned
 * Five launches on the stream: per-key-block softmax statistics of the window rows, their
 * fold into row denominators, the score pass, the selection, one gather for K, V and position ids.  The attention
 * output of the new token itself is not computed here.
 */
PYR_API int pyr_decode_workspace_bytes(const pyr_shape* shape, int32_t w, size_t* bytes_out);
PYR_API int pyr_decode_update(const void* q_win, const void* k, const void* v,
                      const int32_t* seq_offsets_dev, const int32_t* seq_offsets_host,
                      const pyr_shape* shape, int32_t w, float softmax_scale,
                      const int32_t* keep_len_dev, const int32_t* keep_len_host,
                      const float* row_weights_dev, const int32_t* pos,
                      float* scores, int32_t* kept_idx, int32_t* out_offsets_dev,
                      void* k_out, void* v_out, int32_t* pos_out,
                      void* workspace, size_t workspace_bytes, void* stream);

/*
 * Diagnostic for the benchmark report, not part of the method: a launch of nothing but bf16 MFMAs
 * (v_mfma_f32_32x32x16_bf16 back to back, two wavefronts per SIMD, every compute unit), so that the
 * rate this very GPU sustains can be printed beside the published peak.
 *   iters              loop trips per wavefront (16 MFMAs each)
 *   sink_dev           dev, one float (never written in practice)
 *   flops_out          host, written: floating-point operations of the launch
 */
PYR_API int pyr_diag_mfma_only(int32_t iters, float* sink_dev, void* stream, double* flops_out);

/*
 * Diagnostic for the benchmark report, not part of the method: a launch that only reads `bytes` of device
 * memory with the LDS-direct loads the score pass uses for K (16 KB tiles, one in flight per wavefront, six
 * wavefronts per compute unit) and discards them, so that the read rate this very GPU sustains can be printed
 * beside the published HBM peak.
 *   data_dev           dev, `bytes` readable bytes, 16-byte aligned
 *   bytes              a positive multiple of 524288, below 2^50
 *   k_layout           0: consecutive tiles; != 0: tiles of 64 rows x 256 bytes, rows 8192 bytes apart (one head of
 *                      64 tokens of a [T, 32, 128] bf16 K)
 *   sink_dev           dev, one int32 (never written in practice)
 * Errors: PYR_ERR_NULL, PYR_ERR_SHAPE (bytes), PYR_ERR_LAUNCH.
 */
PYR_API int pyr_diag_read_stream(const void* data_dev, size_t bytes, int32_t k_layout, int32_t* sink_dev, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* PYR_H */
