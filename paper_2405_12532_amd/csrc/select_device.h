// Device code of the segmented top-k (Algorithm 1, TopP(A_e, p) with the retention ratio turned
// into a count, followed by the recent window that is always kept), written for a workgroup of
// any multiple of 64 lanes; the selection kernel (select.hip) runs it with 1024 lanes per sequence.
//
// The paper names the sort inside TopP as the one extra cost of the method that matters
// (Appendix A.1).  Nothing is sorted here: the workgroup finds the value of the need-th largest
// context score with a most-significant-digit-first radix select on the fp32 bit patterns
// (4 passes of 8 bits, histogram in LDS), then emits the survivors with wavefront ballots and
// prefix counts, which yields ascending positions for free.  Ties at the threshold go to the
// lower positions.
#pragma once

#include "pyr_internal.h"

namespace pyr {

// LDS the selection needs besides the staged keys
struct SelectShared {
    uint32_t hist[256];
    int wave_cnt[2 * 16];
    int bcast[2];
    int red[16];
};

// Monotone map float -> uint32 (larger float, larger key); -0 is folded onto +0 so that
// equal floats always get equal keys.
__device__ __forceinline__ uint32_t ordered_key(float x) {
    uint32_t b = __float_as_uint(x);
    if (b == 0x80000000u) b = 0u;
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

__device__ __forceinline__ uint64_t lanemask_lt() {
    const int lane = threadIdx.x & 63;
    return lane == 0 ? 0ull : (~0ull >> (64 - lane));
}

template <bool kStaged>
__device__ __forceinline__ uint32_t get_key(const uint32_t* lds_keys, const float* __restrict__ g, int i) {
    if (kStaged) return lds_keys[i];
    return ordered_key(g[i]);
}

// The body after the keys are reachable through get_key<kStaged>; kT lanes (a multiple of 64, at most 1024).
template <bool kStaged, int kT>
__device__ void select_body(const uint32_t* lds_keys, const float* __restrict__ sc, int C, int need,
                            int32_t row0, int32_t* __restrict__ out, SelectShared* sh) {
    constexpr int kW = kT / 64;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c_round = (C + kT - 1) / kT * kT;
    uint32_t* hist = sh->hist;

    // ---- radix select: threshold key `prefix` and the number of ties still to admit
    uint32_t prefix = 0, mask = 0;
    int remaining = need;
    for (int shift = 24; shift >= 0; shift -= 8) {
        for (int i = tid; i < 256; i += kT) hist[i] = 0;
        __syncthreads();
        for (int i = tid; i < c_round; i += kT) {
            const bool valid = i < C;
            const uint32_t key = valid ? get_key<kStaged>(lds_keys, sc, i) : 0u;
            bool match = valid && ((key & mask) == prefix);
            const uint32_t digit = (key >> shift) & 255u;
            // Scores of one sequence share their leading bits, so most lanes of a wavefront
            // hit the same bin: peel the two most common digits with ballots first.
            uint64_t active = __ballot(match);
#pragma unroll 1
            for (int round = 0; round < 2 && active != 0; ++round) {
                const int leader = __ffsll((unsigned long long)active) - 1;
                const uint32_t dl = __builtin_amdgcn_readlane(digit, leader);
                const uint64_t same = __ballot(match && digit == dl);
                if (lane == leader) atomicAdd(&hist[dl], (uint32_t)__popcll(same));
                match = match && digit != dl;
                active &= ~same;
            }
            if (match) atomicAdd(&hist[digit], 1u);
        }
        __syncthreads();
        if (wave == 0) {
            // lane l owns bins 255-4l .. 252-4l (descending order of value)
            const int top = 255 - 4 * lane;
            const uint32_t h0 = hist[top], h1 = hist[top - 1], h2 = hist[top - 2], h3 = hist[top - 3];
            const int mine = (int)(h0 + h1 + h2 + h3);
            int incl = mine;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const int up = __shfl_up(incl, d);
                if (lane >= d) incl += up;
            }
            const int excl = incl - mine;
            if (excl < remaining && remaining <= incl) {
                int run = excl, sel = top - 3;
                const uint32_t hh[4] = {h0, h1, h2, h3};
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    if (run + (int)hh[b] >= remaining) { sel = top - b; break; }
                    run += (int)hh[b];
                }
                sh->bcast[0] = sel;
                sh->bcast[1] = remaining - run;
            }
        }
        __syncthreads();
        prefix |= (uint32_t)sh->bcast[0] << shift;
        mask |= 255u << shift;
        remaining = sh->bcast[1];
        // (the next pass starts with a barrier after clearing hist, which also orders these reads)
    }
    const uint32_t tau = prefix;
    const int ties = remaining;                 // >= 1 ties at tau are admitted, lowest positions first

    // ---- ordered emission: wavefront `wave` owns positions [wave*seg, (wave+1)*seg)
    const int seg = (C + kW * 64 - 1) / (kW * 64) * 64;
    const int lo = wave * seg;
    const int hi = min(C, lo + seg);
    int n_gt = 0, n_eq = 0;
    for (int i0 = lo; i0 < hi; i0 += 64) {
        const int i = i0 + lane;
        const uint32_t key = i < hi ? get_key<kStaged>(lds_keys, sc, i) : 0u;
        n_gt += __popcll(__ballot(i < hi && key > tau));
        n_eq += __popcll(__ballot(i < hi && key == tau));
    }
    if (lane == 0) { sh->wave_cnt[2 * wave] = n_gt; sh->wave_cnt[2 * wave + 1] = n_eq; }
    __syncthreads();
    int gt_before = 0, eq_before = 0;
    for (int u = 0; u < wave; ++u) { gt_before += sh->wave_cnt[2 * u]; eq_before += sh->wave_cnt[2 * u + 1]; }
    int kept_cnt = gt_before + min(eq_before, ties);
    const uint64_t lt = lanemask_lt();
    for (int i0 = lo; i0 < hi; i0 += 64) {
        const int i = i0 + lane;
        const uint32_t key = i < hi ? get_key<kStaged>(lds_keys, sc, i) : 0u;
        const bool gt = i < hi && key > tau;
        const bool eq = i < hi && key == tau;
        const uint64_t eq_mask = __ballot(eq);
        const int eq_rank = eq_before + __popcll(eq_mask & lt);
        const bool keep = gt || (eq && eq_rank < ties);
        const uint64_t keep_mask = __ballot(keep);
        if (keep) out[kept_cnt + __popcll(keep_mask & lt)] = row0 + i;
        kept_cnt += __popcll(keep_mask);
        eq_before += __popcll(eq_mask);
    }
}

// The selection of sequence b by the calling workgroup (all kT lanes take part; uniform control
// flow).  lds_keys: room for lds_cap keys; scores of longer contexts are re-read from memory in
// every pass.  Also writes out_offsets[b + 1] (and out_offsets[0] for b == 0).
template <int kT>
__device__ void select_sequence(int b, const float* __restrict__ scores, const int32_t* __restrict__ seq_offsets,
                                const int32_t* __restrict__ keep_len, int32_t w, uint32_t* lds_keys, int32_t lds_cap,
                                SelectShared* sh, int32_t* __restrict__ kept_idx, int32_t* __restrict__ out_offsets) {
    constexpr int kW = kT / 64;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    // packed position of this sequence's output: sum of the keep counts before it
    int part = 0;
    for (int u = tid; u < b; u += kT) part += keep_len[u];
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) part += __shfl_xor(part, d);
    if (lane == 0) sh->red[wave] = part;
    __syncthreads();
    int out_base = 0;
#pragma unroll
    for (int u = 0; u < kW; ++u) out_base += sh->red[u];

    const int32_t row0 = seq_offsets[b];
    const int S = seq_offsets[b + 1] - row0;
    const int L = min(w, S);
    const int k = min(max(keep_len[b], L), S);
    const int C = S - L;                        // context positions, the candidates
    const int need = k - L;                     // how many of them survive
    if (tid == 0) {
        out_offsets[b + 1] = out_base + k;
        if (b == 0) out_offsets[0] = 0;
    }
    int32_t* __restrict__ out = kept_idx + out_base;

    // the recent window is always kept (A_e ranks the columns before it only)
    for (int i = tid; i < L; i += kT) out[need + i] = row0 + C + i;
    if (need == 0) return;
    if (need == C) {                            // nothing to evict: identity
        for (int i = tid; i < C; i += kT) out[i] = row0 + i;
        return;
    }
    const float* __restrict__ sc = scores + row0;
    if (C <= lds_cap) {
        for (int i = tid; i < C; i += kT) lds_keys[i] = ordered_key(sc[i]);
        __syncthreads();
        select_body<true, kT>(lds_keys, sc, C, need, row0, out, sh);
    } else {
        select_body<false, kT>(lds_keys, sc, C, need, row0, out, sh);
    }
}

}  // namespace pyr
