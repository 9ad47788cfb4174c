// Ensemble attention weights of the recent window (Algorithm 1,
// A_e = weighted_avg(A[-L:, :-L], dim=-2); Section 3.2.1), uniform weights, mean over heads:
//   scores[t] = 1/(Hq*L') * sum_h sum_{i=S-L'}^{S-1} A_h[i, t],   L' = min(w, S).
//
// The weights of the last L' rows are rebuilt from the logits and the row denominators the
// attention kernel saved (log2 domain), so the S x S matrix is never stored:
//   A_h[i,t] = 2^(c * q_i.k_t - lse_h[i]).
// One wavefront owns 64 consecutive key positions of one sequence and walks over every
// head and every 32-row block of the window; with S^T = K Q^T in the MFMA accumulator a
// lane holds 16 keys of one window row, adds its probabilities into 2x16 per-lane sums and
// only at the very end the 32 lanes of each half are added up through LDS in a fixed order.
// No atomics: the result is bit-reproducible.  All S columns are written, the window's own
// columns too (so each sequence's scores sum to one).
#include "pyr_internal.h"

namespace pyr {
namespace {

constexpr int kWavesPerBlock = 4;
constexpr int kKeysPerWave = 64;

template <int D>
__global__ __launch_bounds__(kWavesPerBlock * 64) void score_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const float* __restrict__ lse,
    const int32_t* __restrict__ seq_offsets, int32_t n_q_heads, int32_t n_kv_heads, int32_t w, int32_t blocks_per_seq,
    float c, float* __restrict__ scores) {
    constexpr int kKSteps = D / 16;
    __shared__ float red[kWavesPerBlock][64][17];    // +1 column: conflict-free column sums

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int li = lane & 31, gl = lane >> 5;
    const int b = blockIdx.x / blocks_per_seq;
    const int row0 = seq_offsets[b];
    const int S = seq_offsets[b + 1] - row0;
    const int key_base = ((blockIdx.x % blocks_per_seq) * kWavesPerBlock + wave) * kKeysPerWave;
    const bool active = key_base < S;                 // wave-uniform
    const int L = min(w, S);
    const int first_row = S - L;                      // local position of the first window row
    const int n_row_blocks = (L + 31) / 32;
    const int group = n_q_heads / n_kv_heads;

    float acc[2][16];
#pragma unroll
    for (int sk = 0; sk < 2; ++sk)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[sk][r] = 0.f;

    for (int kvh = 0; active && kvh < n_kv_heads; ++kvh) {
        bf16x8 kf[2][kKSteps];
#pragma unroll
        for (int sk = 0; sk < 2; ++sk) {
            const int key = min(key_base + 32 * sk + li, S - 1);
            const uint16_t* src = k + ((size_t)(row0 + key) * n_kv_heads + kvh) * D + 8 * gl;
#pragma unroll
            for (int ks = 0; ks < kKSteps; ++ks) kf[sk][ks] = *(const bf16x8*)(src + 16 * ks);
        }
        for (int gi = 0; gi < group; ++gi) {
            const int h = kvh * group + gi;
            for (int rb = 0; rb < n_row_blocks; ++rb) {
                const int qpos = first_row + 32 * rb + li;          // this lane's window row
                const int qrow = min(qpos, S - 1);
                if (first_row + 32 * rb + 31 < key_base) continue;  // whole row block precedes the keys
                const uint16_t* qsrc = q + ((size_t)(row0 + qrow) * n_q_heads + h) * D + 8 * gl;
                const float lse_row = lse[(size_t)(row0 + qrow) * n_q_heads + h];
                bf16x8 qf[kKSteps];
#pragma unroll
                for (int ks = 0; ks < kKSteps; ++ks) qf[ks] = *(const bf16x8*)(qsrc + 16 * ks);
#pragma unroll
                for (int sk = 0; sk < 2; ++sk) {
                    f32x16 s;
#pragma unroll
                    for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
                    for (int ks = 0; ks < kKSteps; ++ks)
                        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[sk][ks], qf[ks], s, 0, 0, 0);
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int key = key_base + 32 * sk + 8 * (r >> 2) + 4 * gl + (r & 3);
                        const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], c, -lse_row));
                        const bool visible = key <= qpos && qpos < S;   // causal, and the row exists
                        acc[sk][r] += visible ? p : 0.f;
                    }
                }
            }
        }
    }

    // ---- add the 32 window-row lanes of each half, fixed order
    const float norm = 1.0f / ((float)n_q_heads * (float)L);
#pragma unroll
    for (int sk = 0; sk < 2; ++sk) {
#pragma unroll
        for (int r = 0; r < 16; ++r) red[wave][lane][r] = acc[sk][r];
        __syncthreads();
        if (active && lane < 32) {
            // key offset `lane` inside the sub-tile lives in half (lane>>2)&1, register 4*(lane>>3)+(lane&3)
            const int half = (lane >> 2) & 1, r = 4 * (lane >> 3) + (lane & 3);
            float sum = 0.f;
            for (int j = 0; j < 32; ++j) sum += red[wave][32 * half + j][r];
            const int key = key_base + 32 * sk + lane;
            if (key < S) scores[row0 + key] = sum * norm;
        }
        __syncthreads();
    }
}

}  // namespace

int launch_score(const void* q, const void* k, const float* lse, const int32_t* seq_offsets_dev,
                 const pyr_shape& s, int32_t w, float scale_log2, float* scores, hipStream_t stream) {
    if (s.n_seqs == 0 || s.max_seqlen == 0) return PYR_OK;
    const int keys_per_block = kWavesPerBlock * kKeysPerWave;
    const int32_t blocks_per_seq = (s.max_seqlen + keys_per_block - 1) / keys_per_block;
    dim3 grid((unsigned)((int64_t)blocks_per_seq * s.n_seqs), 1, 1);
    if (s.head_dim == 128)
        hipLaunchKernelGGL(score_kernel<128>, grid, dim3(kWavesPerBlock * 64), 0, stream, (const uint16_t*)q,
                           (const uint16_t*)k, lse, seq_offsets_dev, s.n_q_heads, s.n_kv_heads, w, blocks_per_seq,
                           scale_log2, scores);
    else
        hipLaunchKernelGGL(score_kernel<64>, grid, dim3(kWavesPerBlock * 64), 0, stream, (const uint16_t*)q,
                           (const uint16_t*)k, lse, seq_offsets_dev, s.n_q_heads, s.n_kv_heads, w, blocks_per_seq,
                           scale_log2, scores);
    return check_launch();
}

}  // namespace pyr
