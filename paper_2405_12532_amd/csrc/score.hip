// Ensemble attention weights of the recent window (Algorithm 1,
// A_e = weighted_avg(A[-L:, :-L], dim=-2); Section 3.2.1), uniform weights, mean over heads:
//   scores[t] = 1/(Hq*L') * sum_h sum_{i=S-L'}^{S-1} A_h[i, t],   L' = min(w, S),
// or, with averaging weights omega (Section 4.1: more recent rows may weigh more; one weight
// per row of a full window, a shorter sequence uses the last L' of them),
//   scores[t] = 1/Hq * sum_h sum_i omega_i A_h[i, t] / sum_i omega_i.
//
// The weights of the last L' rows are rebuilt from the logits and the row denominators the
// attention kernel saved (log2 domain), so the S x S matrix is never stored:
//   A_h[i,t] = 2^(c * q_i.k_t - lse_h[i]);  a weight enters as  - log2(omega_i)  next to lse_h[i].
// One workgroup owns 64 consecutive key positions of one sequence; its two wavefronts share
// out the KV heads (so a small batch still fills the chip) and each walks over its heads and,
// per head, over "steps": one query head x one 32-row block of the window.  With
// S^T = K Q^T in the MFMA accumulator a lane holds 16 keys of one window row, adds its
// probabilities into 2x16 per-lane sums, and only at the very end the 32 lanes of each half
// and the two wavefronts are added up through LDS in a fixed order.  No atomics: the result
// is bit-reproducible.  All S columns are written, the window's own columns too (so each
// sequence's scores sum to one).
//
// Every byte of K (once, from HBM) and of the window's Q rows (once per 64 keys, from L2)
// passes the CU's vector L1, and loads into registers get through it at roughly a quarter of
// the rate of loads that write LDS directly - with them this kernel ran at the pace of that
// L1, not of HBM.  So all operands take the direct path: a wavefront keeps a private 64 x d K
// tile, a 32 x d Q tile and 32 row denominators in LDS, fills them with global_load_lds
// (fully coalesced: 16 lanes per 256-byte row, 16-byte chunks XOR-swizzled against bank
// conflicts), copies the fragments into registers and at once requests the next tile into
// the same LDS space, which then arrives while the MFMAs and exponentials of this one run.
//
// The same walk serves the generation-phase update of the cache (Algorithm 1 with a non-empty
// cache; Section 4.1): there the queries of the recent rows come in a buffer of their own
// ([B, w, Hq, d], right-aligned) and no attention pass has left row denominators behind, so a
// first pass (kStats) writes, per 64-key workgroup, every window row's maximum and sum of
// exponentials, a small kernel folds them into denominators, and the score pass runs as above.
//
// Small batches.  With one workgroup per 64 keys a single 2048-token prompt gives 32 workgroups to 256
// compute units, and the step then spends a third of its time here (Appendix A.1 of the paper: the
// selection overhead eats the gain at small batch).  The launcher may therefore split the KV heads over
// gridDim.y workgroups per key block; each writes its partial sums, and the workgroup that arrives last at
// the block's counter adds them up in head-group order (so the result does not depend on who was last).
// (Letting the workgroup that completes a sequence's scores run the top-k selection as well was built and
// measured: it replaces a launch that costs as much as the selection it carries, and was slower at every
// shape - 27.8 against 26.5 us per step at one 256-token prompt, 40.0 against 39.5 ms over the 32-layer
// pyramid at batch 64 - so the selection stays a kernel of its own.)  The counters live in the caller's
// workspace, start at zero and are put back to zero by their last arrival.
#include "pyr_internal.h"

namespace pyr {
namespace {

constexpr int kWavesPerBlock = 2;    // wavefronts sharing out a workgroup's KV heads
enum Mode { kScores = 0, kScoresWeighted = 1, kStats = 2 };
constexpr int kKeysPerBlock = 64;

typedef __attribute__((address_space(3))) char* lptr_t;

constexpr int kMaxHeadGroups = 16;

// What the last-arriving workgroup of a key block does when the KV heads are split over gridDim.y workgroups
// (all pointers device; counters == nullptr: no split).
struct ScoreTail {
    int32_t* counters;            // [n_seqs * blocks_per_seq] one per key block; zero at launch
    float* part_sums;             // [gridDim.y, total_tokens] partial scores
    int32_t total_tokens;
};

// 64 lanes x 16 bytes (or x 4 bytes) from base + voff[lane] to LDS at lds_addr + 16 (4) * lane.
// Assembly because the wavefront orders these loads itself with s_waitcnt vmcnt(N); they
// retire in the order issued.
__device__ __forceinline__ void lds_dma(const char* base_, uint32_t voff, uint32_t lds_addr, bool dword) {
    const uint32_t m0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)lds_addr);
    const uint64_t b64 = (uint64_t)(uintptr_t)base_;         // wave-uniform by construction: keep it in scalar registers
    const uint32_t b_lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)b64);          // (the builtin returns a signed int:
    const uint32_t b_hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(b64 >> 32));  //  widen it unsigned)
    const char* base = (const char*)(uintptr_t)(((uint64_t)b_hi << 32) | (uint64_t)b_lo);
    if (dword)
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2" ::"s"(m0), "v"(voff), "s"(base) : "memory", "m0");
    else
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(m0), "v"(voff), "s"(base) : "memory", "m0");
}

template <int N>
__device__ __forceinline__ void wait_loads() {      // until at most N of this wavefront's loads are outstanding
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
__device__ __forceinline__ void wait_lds() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

// q_window == 0: q and lse are indexed by packed row like k ([T, Hq, d], [T, Hq]);
// q_window != 0: by (sequence, window slot): [B, w, Hq, d], [B, w, Hq], the last row in slot w-1.
// kStats writes part[((key block * B + b) * Hq + h) * w + slot] = (max, sum of 2^(x - max)) over the
// block's visible keys, x = c * q.k, and touches neither lse nor scores.
template <int D, int kMode>
__global__ __launch_bounds__(kWavesPerBlock * 64, 2) void score_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const float* __restrict__ lse,
    const int32_t* __restrict__ seq_offsets, int32_t n_seqs, int32_t n_q_heads, int32_t n_kv_heads, int32_t w,
    int32_t blocks_per_seq, int32_t chunk_blocks, int32_t xcds, int32_t head_step, int32_t q_window, float c,
    const float* __restrict__ row_weights, float* __restrict__ scores, float2* __restrict__ part, ScoreTail tail) {
    constexpr bool kWeighted = kMode == kScoresWeighted;
    constexpr int kKSteps = D / 16;
    constexpr int kChunks = D / 8;                  // 16-byte chunks per row
    constexpr int kRowBytes = D * 2;
    constexpr int kRowsPerLoad = 64 / kChunks;      // rows one load instruction covers
    constexpr int kKBytes = 64 * kRowBytes, kQBytes = 32 * kRowBytes, kLseBytes = 256;
    constexpr int kNK = kKBytes / 1024, kNQ = kQBytes / 1024;       // load instructions per K tile, per Q tile
    constexpr int kStepLoads = kNQ + (kMode == kStats ? 0 : kWeighted ? 2 : 1);   // ... per step: Q tile, denominators, weights
    constexpr int kRedBytes = kWavesPerBlock * 2 * 64 * 17 * 4;     // +1 column: conflict-free column sums
    constexpr int kSmemBytes = kWavesPerBlock * (kKBytes + kQBytes + 2 * kLseBytes);
    static_assert(kSmemBytes >= kRedBytes, "the final reduction reuses the tiles' space");
    __shared__ __align__(1024) char smem[kSmemBytes];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int li = lane & 31, gl = lane >> 5;
    // Workgroup -> (sequence, key block).  Consecutive workgroup ids go to consecutive XCDs; a chunk of
    // chunk_blocks key blocks of one sequence stays on one XCD, so that the window's Q rows, which every key
    // block of the sequence re-reads, are found in that XCD's L2.
    const int wg_slot = (int)blockIdx.x / xcds;
    const int chunk = (wg_slot / chunk_blocks) * xcds + (int)blockIdx.x % xcds;
    const int chunks_per_seq = (blocks_per_seq + chunk_blocks - 1) / chunk_blocks;
    const int b = chunk / chunks_per_seq;
    const int key_block = (chunk % chunks_per_seq) * chunk_blocks + wg_slot % chunk_blocks;
    if (b >= n_seqs || key_block >= blocks_per_seq) return;      // (uniform over the workgroup, like the next one)
    const int row0 = seq_offsets[b];
    const int S = seq_offsets[b + 1] - row0;
    const int key_base = key_block * kKeysPerBlock;
    if (key_base >= S) return;
    const int L = min(w, S);
    const int first_row = S - L;                      // local position of the first window row
    const int q_row_base = q_window ? b * w + (w - L) : row0 + first_row;   // row of q / lse holding the first window row
    const int n_row_blocks = (L + 31) / 32;
    const int group = n_q_heads / n_kv_heads;
    const int n_steps = group * n_row_blocks;         // per KV head
    // this workgroup's share of the KV heads (all of them unless the launcher split them over gridDim.y), halved
    // between the two wavefronts
    const int wg_heads = n_kv_heads / (int)gridDim.y, wg_first = (int)blockIdx.y * wg_heads;
    // Each wavefront takes half of the workgroup's heads, and, where the launcher asks for it (head_step != 0), every
    // key block starts its walk at another head: workgroups that run side by side then read different 256-byte
    // columns of their token rows, which spreads them over the memory channels when the rows are a power of two
    // apart (a read-only stream over 8 KB rows: 5.5 -> 5.9 TB/s with steps of 7; 1 and 8 are worse than none).
    const int head_rot = (key_block * head_step) % wg_heads;
    auto head_at = [&](int i) { const int r = i + head_rot; return wg_first + (r >= wg_heads ? r - wg_heads : r); };   // i < wg_heads

    float acc[2][16];
#pragma unroll
    for (int sk = 0; sk < 2; ++sk)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[sk][r] = 0.f;

    // sum of the weights in use (fixed order: every lane strides over them, then a butterfly).
    // These are the only ordinary loads of the kernel and they are complete before the first
    // LDS-direct load is issued: the wait counts below assume nothing else is in flight.
    float weight_sum = (float)L;
    if (kWeighted) {
        float part = 0.f;
        for (int j = lane; j < L; j += 64) part += row_weights[w - L + j];
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) part += __shfl_xor(part, m, 64);
        asm volatile("s_waitcnt vmcnt(0)" : "+v"(part) : : "memory");
        weight_sum = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, part)));   // uniform: a scalar register
    }

    // ---- this wavefront's LDS: K tile, Q tile (1 KB aligned), then the row denominators
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lptr_t)smem;
    const uint32_t kt = lds0 + wave * (kKBytes + kQBytes), qt = kt + kKBytes;
    const uint32_t lt = lds0 + kWavesPerBlock * (kKBytes + kQBytes) + wave * 2 * kLseBytes;   // denominators, then weights
    const uint32_t wt = lt + kLseBytes;

    // ---- load side: lane -> (row inside an instruction's row group, physical chunk).  The LDS
    // slot of a lane is fixed by the instruction, so the swizzle picks the global chunk.
    const int ld_row = lane / kChunks, ld_chunk = lane % kChunks;
    const uint32_t k_row_bytes = (uint32_t)n_kv_heads * kRowBytes, q_row_bytes = (uint32_t)n_q_heads * kRowBytes;
    const int last_key = S - 1 - key_base;            // rows past the end of the sequence re-read its last row
    // (the offsets are recomputed at every use - a few VALU operations per load; kept live they
    //  would push the kernel past the registers of two wavefronts per SIMD)
    auto issue_k = [&](int kvh) {
        const char* base = (const char*)(k + ((size_t)(row0 + key_base) * n_kv_heads + kvh) * D);
        int lim = last_key;
        asm volatile("" : "+v"(lim));
#pragma unroll
        for (int i = 0; i < kNK; ++i) {
            const int row = kRowsPerLoad * i + ld_row;
            // (24-bit multiply: full rate, where the 32-bit one takes four times as long; rows and strides are far below 2^24)
            lds_dma(base, __umul24((uint32_t)min(row, lim), k_row_bytes) + 16 * (ld_chunk ^ (row & (kChunks - 1))), kt + 1024 * i,
                    false);
        }
    };
    auto issue_q = [&](int kvh, int st) {             // kStepLoads instructions
        const int h = kvh * group + st / n_row_blocks, rb = st % n_row_blocks;
        const int rb_row0 = first_row + 32 * rb;
        int last_row = L - 1 - 32 * rb;
        asm volatile("" : "+v"(last_row));
        const char* base = (const char*)(q + ((size_t)(q_row_base + 32 * rb) * n_q_heads + h) * D);
#pragma unroll
        for (int i = 0; i < kNQ; ++i) {
            const int row = kRowsPerLoad * i + ld_row;
            lds_dma(base, __umul24((uint32_t)min(row, last_row), q_row_bytes) + 16 * (ld_chunk ^ (row & (kChunks - 1))),
                    qt + 1024 * i, false);
        }
        if (kMode != kStats)
            lds_dma((const char*)(lse + (size_t)(q_row_base + 32 * rb) * n_q_heads + h),
                    __umul24((uint32_t)min(li, last_row), (uint32_t)n_q_heads * 4), lt, true);
        if (kWeighted) lds_dma((const char*)(row_weights + (w - L) + 32 * rb), (uint32_t)min(li, last_row) * 4, wt, true);
    };

    // ---- fragment side: operand row li, logical chunk 2*ks + gl
    auto frag = [&](uint32_t tile, int row, int ks) {
        const uint32_t a = tile + row * kRowBytes + (((2 * ks + gl) ^ (row & (kChunks - 1))) << 4);
        return *(const bf16x8 __attribute__((address_space(3)))*)(uintptr_t)a;
    };

    const int hi_begin = wave * wg_heads / kWavesPerBlock, hi_end = (wave + 1) * wg_heads / kWavesPerBlock;
    if (hi_begin < hi_end) {
        issue_k(head_at(hi_begin));
        issue_q(head_at(hi_begin), 0);
    }
    // Outstanding loads at the top of a head: its K tile (oldest), then its first step's rows.
    for (int hi = hi_begin; hi < hi_end; ++hi) {
        const bool has_next = hi + 1 < hi_end;
        const int kvh = head_at(hi), kvh_next = has_next ? head_at(hi + 1) : kvh;
        wait_loads<kStepLoads>();                     // the K tile has landed
        bf16x8 kf[2][kKSteps];
#pragma unroll
        for (int sk = 0; sk < 2; ++sk)
#pragma unroll
            for (int ks = 0; ks < kKSteps; ++ks) kf[sk][ks] = frag(kt, 32 * sk + li, ks);
        wait_lds();                                   // fragments are in registers: the tile's space is free
        if (has_next) issue_k(kvh_next);
        for (int st = 0; st < n_steps; ++st) {
            // the step's rows are older than the next K tile only in the head's first step
            if (st == 0 && has_next) wait_loads<kNK>(); else wait_loads<0>();
            bf16x8 qf[kKSteps];
#pragma unroll
            for (int ks = 0; ks < kKSteps; ++ks) qf[ks] = frag(qt, li, ks);
            float lse_row = 0.f;
            if (kMode != kStats) lse_row = *(const float __attribute__((address_space(3)))*)(uintptr_t)(lt + 4 * li);
            if (kWeighted)      // omega * 2^x = 2^(x + log2 omega); a zero weight gives 2^-inf = 0
                lse_row -= __builtin_amdgcn_logf(*(const float __attribute__((address_space(3)))*)(uintptr_t)(wt + 4 * li));
            wait_lds();
            if (st + 1 < n_steps) issue_q(kvh, st + 1);
            else if (has_next) issue_q(kvh_next, 0);

            const int rb = st % n_row_blocks;
            const int qpos = first_row + 32 * rb + li;              // this lane's window row
            if (first_row + 32 * rb + 31 < key_base) continue;      // whole row block precedes the keys
            // masks are only needed where the keys reach into the window or the row block is ragged
            const bool plain = key_base + 63 <= first_row + 32 * rb && first_row + 32 * rb + 31 < S;   // uniform
            if (kMode == kStats) {
                // this row's maximum and sum of exponentials over the 32 keys the lane holds, then
                // over the 32 the other half-wavefront holds
                f32x16 x[2];
                float mx = -INFINITY;
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
                        const bool visible = plain || (key <= qpos && qpos < S);
                        x[sk][r] = visible ? s[r] * c : -INFINITY;
                        mx = fmaxf(mx, x[sk][r]);
                    }
                }
                float sum = 0.f;
                if (mx > -INFINITY) {
#pragma unroll
                    for (int sk = 0; sk < 2; ++sk)
#pragma unroll
                        for (int r = 0; r < 16; ++r) sum += __builtin_amdgcn_exp2f(x[sk][r] - mx);
                }
                const float mo = __shfl_xor(mx, 32, 64), so = __shfl_xor(sum, 32, 64);
                const float m_all = fmaxf(mx, mo);
                if (gl == 0 && m_all > -INFINITY && 32 * rb + li < L) {
                    const float total = (mx > -INFINITY ? sum * __builtin_amdgcn_exp2f(mx - m_all) : 0.f) +
                                        (mo > -INFINITY ? so * __builtin_amdgcn_exp2f(mo - m_all) : 0.f);
                    const int h = kvh * group + st / n_row_blocks, slot = (w - L) + 32 * rb + li;
                    part[(((size_t)key_block * n_seqs + b) * n_q_heads + h) * w + slot] = make_float2(m_all, total);   // 32 rows: 256 consecutive bytes
                }
                continue;
            }
#pragma unroll
            for (int sk = 0; sk < 2; ++sk) {
                f32x16 s;
#pragma unroll
                for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
                for (int ks = 0; ks < kKSteps; ++ks)
                    s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[sk][ks], qf[ks], s, 0, 0, 0);
                if (plain) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[sk][r] += __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], c, -lse_row));
                } else {
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
    // every load issued above has been waited for: nothing is in flight towards LDS here
    if (kMode == kStats) return;

    // ---- add the 32 window-row lanes of each half and the two head groups, fixed order
    const float norm = 1.0f / ((float)n_q_heads * weight_sum);
    float (*red)[2][64][17] = (float (*)[2][64][17])smem;
    __syncthreads();                                  // both wavefronts are done with their tiles
#pragma unroll
    for (int sk = 0; sk < 2; ++sk)
#pragma unroll
        for (int r = 0; r < 16; ++r) red[wave][sk][lane][r] = acc[sk][r];
    __syncthreads();
    if (lane < 32) {
        const int sk = wave;                          // wavefront 0 sums the first 32 keys, wavefront 1 the rest
        // key offset `lane` inside the sub-tile lives in half (lane>>2)&1, register 4*(lane>>3)+(lane&3)
        const int half = (lane >> 2) & 1, r = 4 * (lane >> 3) + (lane & 3);
        float sum = 0.f;
        for (int v = 0; v < kWavesPerBlock; ++v)
            for (int j = 0; j < 32; ++j) sum += red[v][sk][32 * half + j][r];
        const int key = key_base + 32 * sk + lane;
        float* dst = gridDim.y > 1 ? tail.part_sums + (size_t)blockIdx.y * tail.total_tokens : scores;
        if (key < S) dst[row0 + key] = sum * norm;
    }
    if (gridDim.y == 1) return;

    // ---- the last of this key block's head groups to arrive adds up the partial sums, in head-group order.
    // (Uniform over the workgroup from here on.)
    int* flag = (int*)smem;                           // (past the reduction's reads: behind a barrier)
    __syncthreads();
    if (threadIdx.x == 0) {
        __threadfence();                              // this workgroup's partial sums are visible before its count is
        int* cnt = tail.counters + b * blocks_per_seq + key_block;
        const int old = atomicAdd(cnt, 1);
        *flag = old == (int)gridDim.y - 1;
        if (*flag) *cnt = 0;                          // back to zero for the next launch
    }
    __syncthreads();
    if (*flag == 0) return;
    __threadfence();                                  // the other head groups' partial sums are visible now
    const int key = key_base + (int)threadIdx.x;
    if (threadIdx.x < 64 && key < S) {
        float sum = 0.f;
        for (int hg = 0; hg < (int)gridDim.y; ++hg) sum += tail.part_sums[(size_t)hg * tail.total_tokens + row0 + key];
        scores[row0 + key] = sum;
    }
}

// Row denominators of the window rows from the per-block statistics: for every (sequence,
// window slot, head) fold (max, sum) over the key blocks the row can see, in block order:
//   lse = M + log2(sum_kb sum_kb * 2^(m_kb - M)),  M = max_kb m_kb.
__global__ __launch_bounds__(256) void fold_stats_kernel(const float2* __restrict__ part,
                                                         const int32_t* __restrict__ seq_offsets, int32_t n_seqs,
                                                         int32_t n_q_heads, int32_t w, float* __restrict__ lse_win) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;        // (b, h, slot), slot fastest, as in part
    if (idx >= (int64_t)n_seqs * w * n_q_heads) return;
    const int slot = (int)(idx % w), h = (int)((idx / w) % n_q_heads), b = (int)(idx / ((int64_t)n_q_heads * w));
    float* dst = lse_win + ((size_t)b * w + slot) * n_q_heads + h;
    const int S = seq_offsets[b + 1] - seq_offsets[b];
    const int L = min(w, S), i = slot - (w - L);
    if (i < 0) {                                      // slot not in use (sequence shorter than the window)
        *dst = 0.f;
        return;
    }
    const int n_blocks = (S - L + i) / kKeysPerBlock + 1;        // key blocks row S-L+i can see
    const size_t stride = (size_t)n_seqs * w * n_q_heads;
    float m_run = -INFINITY, s_run = 0.f;
    for (int kb = 0; kb < n_blocks; ++kb) {
        const float2 p = part[kb * stride + idx];
        if (p.x > m_run) {
            s_run = s_run * __builtin_amdgcn_exp2f(m_run - p.x) + p.y;      // (2^-inf = 0 the first time)
            m_run = p.x;
        } else {
            s_run += p.y * __builtin_amdgcn_exp2f(p.x - m_run);
        }
    }
    *dst = m_run + __builtin_amdgcn_logf(s_run);
}

}  // namespace

namespace {
template <int kMode>
int launch_walk(const void* q, const void* k, const float* lse, const int32_t* seq_offsets_dev, const pyr_shape& s,
                int32_t min_seqlen, int32_t w, int32_t q_window, float scale_log2, const float* row_weights, float* scores,
                float2* part, hipStream_t stream,
                const ScoreTail& tail = ScoreTail{nullptr, nullptr, 0}, int head_groups = 1) {
    const int32_t blocks_per_seq = (s.max_seqlen + kKeysPerBlock - 1) / kKeysPerBlock;
    DeviceInfo dev;
    if (device_info(&dev) != PYR_OK) return PYR_ERR_LAUNCH;
    // A whole sequence per XCD where that spreads the work evenly by construction (equal lengths, a multiple of the XCD
    // count); otherwise the plain order, key block after key block over the XCDs: with ragged lengths the sequences
    // of one XCD can be much longer than another's (measured: 32 sequences of 512...8192 tokens, 0.35 -> 0.51 ms).
    const int32_t xcds = dev.xccs;
    const int32_t chunk_blocks = min_seqlen == s.max_seqlen && s.n_seqs % xcds == 0 ? blocks_per_seq : 1;
    // (rows of 10 KB - 40 heads - are spread well as they are, and lose 4 % to the rotation: neighbouring key blocks then
    //  no longer share the window's Q rows of one head in L2)
    const size_t k_row_bytes = (size_t)s.n_kv_heads * s.head_dim * 2;
    const int32_t head_step = (k_row_bytes & (k_row_bytes - 1)) == 0 ? 7 : 0;
    const int64_t chunks = (int64_t)s.n_seqs * ((blocks_per_seq + chunk_blocks - 1) / chunk_blocks);
    const int64_t n_blocks = (chunks + xcds - 1) / xcds * xcds * chunk_blocks;
    if (n_blocks >= (int64_t)1 << 31) return PYR_ERR_UNSUPPORTED;
    dim3 grid((unsigned)n_blocks, (unsigned)head_groups, 1), block(kWavesPerBlock * 64);
    if (s.head_dim == 128)
        hipLaunchKernelGGL((score_kernel<128, kMode>), grid, block, 0, stream, (const uint16_t*)q, (const uint16_t*)k, lse,
                           seq_offsets_dev, s.n_seqs, s.n_q_heads, s.n_kv_heads, w, blocks_per_seq, chunk_blocks, xcds, head_step,
                           q_window, scale_log2, row_weights, scores, part, tail);
    else
        hipLaunchKernelGGL((score_kernel<64, kMode>), grid, block, 0, stream, (const uint16_t*)q, (const uint16_t*)k, lse,
                           seq_offsets_dev, s.n_seqs, s.n_q_heads, s.n_kv_heads, w, blocks_per_seq, chunk_blocks, xcds, head_step,
                           q_window, scale_log2, row_weights, scores, part, tail);
    return check_launch();
}
}  // namespace

int launch_score(const void* q, const void* k, const float* lse, const int32_t* seq_offsets_dev,
                 const pyr_shape& s, int32_t min_seqlen, int32_t w, float scale_log2, const float* row_weights,
                 float* scores, hipStream_t stream) {
    if (s.n_seqs == 0 || s.max_seqlen == 0) return PYR_OK;
    return row_weights ? launch_walk<kScoresWeighted>(q, k, lse, seq_offsets_dev, s, min_seqlen, w, 0, scale_log2, row_weights, scores,
                                                      nullptr, stream)
                       : launch_walk<kScores>(q, k, lse, seq_offsets_dev, s, min_seqlen, w, 0, scale_log2, nullptr, scores, nullptr,
                                              stream);
}

// Head groups for a grid of n_blocks key blocks: enough workgroups for two per compute unit, every group at least
// two KV heads (one per wavefront) where there are two, an even split.
static int pick_head_groups(int64_t n_blocks, int n_kv_heads, int compute_units) {
    int g = 1;
    while (g < kMaxHeadGroups && n_blocks * g < 2 * (int64_t)compute_units && n_kv_heads % (2 * g) == 0 &&
           n_kv_heads / (2 * g) >= 2)
        g *= 2;
    return g;
}

size_t score_tail_bytes(const pyr_shape& s) {
    const size_t blocks_per_seq = ((size_t)s.max_seqlen + kKeysPerBlock - 1) / kKeysPerBlock;
    const size_t counters = ((size_t)s.n_seqs * blocks_per_seq * sizeof(int32_t) + 255) / 256 * 256;
    // partial sums are only ever used by grids of fewer than 2 x 256 key blocks
    const size_t parts = (size_t)s.n_seqs * blocks_per_seq < 1024 ? (size_t)kMaxHeadGroups * s.total_tokens * sizeof(float) : 0;
    return counters + (parts + 255) / 256 * 256;
}

int32_t score_tail_counters(const pyr_shape& s) {
    const int32_t blocks_per_seq = (s.max_seqlen + kKeysPerBlock - 1) / kKeysPerBlock;
    return s.n_seqs * blocks_per_seq;
}

int launch_score_groups(const void* q, const void* k, const float* lse, const int32_t* seq_offsets_dev,
                        const pyr_shape& s, int32_t min_seqlen, int32_t w, float scale_log2, const float* row_weights,
                        float* scores, void* tail_ws, hipStream_t stream) {
    if (s.n_seqs == 0 || s.max_seqlen == 0) return PYR_OK;
    DeviceInfo dev;
    if (device_info(&dev) != PYR_OK) return PYR_ERR_LAUNCH;
    const int64_t blocks_per_seq = (s.max_seqlen + kKeysPerBlock - 1) / kKeysPerBlock;
    const int64_t n_blocks = blocks_per_seq * s.n_seqs;
    const int g = n_blocks < 1024 ? pick_head_groups(n_blocks, s.n_kv_heads, dev.compute_units) : 1;
    if (g == 1) return launch_score(q, k, lse, seq_offsets_dev, s, min_seqlen, w, scale_log2, row_weights, scores, stream);
    const size_t counter_bytes = ((size_t)s.n_seqs * blocks_per_seq * sizeof(int32_t) + 255) / 256 * 256;
    ScoreTail tail{(int32_t*)tail_ws, (float*)((char*)tail_ws + counter_bytes), s.total_tokens};
    return row_weights ? launch_walk<kScoresWeighted>(q, k, lse, seq_offsets_dev, s, min_seqlen, w, 0, scale_log2, row_weights, scores,
                                                      nullptr, stream, tail, g)
                       : launch_walk<kScores>(q, k, lse, seq_offsets_dev, s, min_seqlen, w, 0, scale_log2, nullptr, scores, nullptr,
                                              stream, tail, g);
}

size_t window_score_part_bytes(const pyr_shape& s, int32_t w) {
    const size_t blocks_per_seq = ((size_t)s.max_seqlen + kKeysPerBlock - 1) / kKeysPerBlock;
    return blocks_per_seq * (size_t)s.n_seqs * (size_t)w * (size_t)s.n_q_heads * sizeof(float2);
}

int launch_window_score(const void* q_win, const void* k, const int32_t* seq_offsets_dev, const pyr_shape& s,
                        int32_t min_seqlen, int32_t w, float scale_log2, const float* row_weights, float* lse_win, void* part, float* scores,
                        hipStream_t stream) {
    if (s.n_seqs == 0 || s.max_seqlen == 0) return PYR_OK;
    int rc = launch_walk<kStats>(q_win, k, nullptr, seq_offsets_dev, s, min_seqlen, w, 1, scale_log2, nullptr, nullptr, (float2*)part,
                                 stream);
    if (rc != PYR_OK) return rc;
    const int64_t n = (int64_t)s.n_seqs * w * s.n_q_heads;
    if ((n + 255) / 256 >= (int64_t)1 << 31) return PYR_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(fold_stats_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, (const float2*)part,
                       seq_offsets_dev, s.n_seqs, s.n_q_heads, w, lse_win);
    if (check_launch() != PYR_OK) return PYR_ERR_LAUNCH;
    return row_weights ? launch_walk<kScoresWeighted>(q_win, k, lse_win, seq_offsets_dev, s, min_seqlen, w, 1, scale_log2, row_weights,
                                                      scores, nullptr, stream)
                       : launch_walk<kScores>(q_win, k, lse_win, seq_offsets_dev, s, min_seqlen, w, 1, scale_log2, nullptr, scores,
                                              nullptr, stream);
}

}  // namespace pyr
