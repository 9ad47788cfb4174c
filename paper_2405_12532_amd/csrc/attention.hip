// Causal softmax attention over packed, ragged sequences (Algorithm 1, "compute attention
// weights of KV", applied to V), flash style: the S x S weight matrix never exists.
//
// Work split.  The unit of work is a SEGMENT: kAttnBlockRows (128) consecutive query
// positions of one (sequence, query head); each of the 4 wavefronts of a workgroup owns 32 of
// them.  Segments are paired into ITEMS - query tile j of a sequence together with tile
// n-1-j - so every item of a sequence sweeps the same number of causal key tiles.  Workgroups
// are persistent: two per compute unit, each walking items with a fixed stride, and the first
// K/V tile and the query fragments of the next segment are requested while the last tile of
// the current one is still being computed, so a compute unit never drains between segments.
// Two workgroups per compute unit put two free-running wavefronts on each SIMD: one feeds the
// matrix pipe while the other does softmax arithmetic.
//
// Keys/values stream through LDS in tiles of 64 positions, double buffered, one tile ahead
// of the arithmetic and written by the load unit itself (global_load ... lds), so they never
// pass through registers.
//
// MFMA mapping (v_mfma_f32_32x32x16_bf16, 64-lane wavefronts).  The kernel computes the
// TRANSPOSED logits  S^T = K Q^T  (keys x queries): in the accumulator layout a lane then
// holds 16 keys of ONE query column, so the softmax row statistics are per-lane scalars (one
// exchange with lane^32 completes them) and rescaling the output is a per-lane multiply.
// The output is accumulated transposed too,  O^T += V^T P^T,  whose B operand P^T is exactly
// what the lane already holds once the K rows of a 32-key sub-tile are fed in the order
// "bits 2 and 3 of the row number swapped".  V sits in LDS row-major like K; its A-operand
// fragments (8 keys of one head-dim column per lane) come out of LDS already transposed
// through ds_read_b64_tr_b16, so no transposition pass and no 2-byte LDS traffic exists.
//
// Numerics: bf16 products, fp32 accumulation, fp32 online softmax in base 2 with the scale
// folded into one FMA per logit; probabilities are rounded to bf16 for the PV product while
// the softmax denominator is summed from the unrounded fp32 values.  The reference of the
// exponent is NOT the running row maximum: it is set from the true maxima on the first tile
// and afterwards only when some row's partial sum shows that it outgrew the reference by
// more than 2^16 (probabilities stay exact in fp32 and as precise in bf16 as at any other
// magnitude).  The common tile therefore takes no row maximum, no cross-lane exchange and no
// rescale of the output: one FMA, one exponential, one add and half a convert per logit.
#include <type_traits>

#include "pyr_internal.h"

namespace pyr {
namespace {

constexpr int kBN = 64;                    // key positions per LDS tile
constexpr int kNW = 4;                     // wavefronts per workgroup
constexpr int kBM = kNW * 32;              // query positions per segment
static_assert(kBM == kAttnBlockRows, "the host counts items with this segment height");

// LDS image of one K or V tile: 64 rows of D bf16, NO padding (the direct global->LDS loads
// fill 1 KiB of consecutive LDS per wavefront instruction).  Bank conflicts are avoided by an
// XOR swizzle of the 16-byte chunk index inside a row instead:
//   K: chunk ^ (row & 15)        -> the 16 rows a b128 fragment read touches hit 16 bank groups
//   V: chunk ^ ((row & 3) << 2)  -> the 4 rows x 64 B a transposing read touches tile the banks
// (for D = 64 two rows share a 256-byte bank line: row is replaced by row / 2 and the masks
// shrink to 7 and 1).
template <int D>
struct Tile {
    static constexpr int kChunks = D / 8;                       // 16-byte chunks per row
    static constexpr int kRowBytes = D * 2;
    static constexpr int kMatBytes = kBN * kRowBytes;           // one K or V tile
    static constexpr int kStageBytes = 2 * kMatBytes;           // K then V
    static constexpr size_t kLdsBytes = 2 * (size_t)kStageBytes;
};

typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) char* lptr_t;

// v_permlane32_swap(x, x): result 0 holds lanes 0..31 of x in both halves, result 1 holds
// lanes 32..63 of x in both halves; combining the two gives "own op other half" in every lane.
__device__ __forceinline__ float max_with_other_half(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum_with_other_half(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Transposing LDS read (ds_read_b64_tr_b16).  Inside every group of 16 lanes, lane j receives
// element (j & 3) of the 8-byte words addressed by lanes (j >> 2), 4 + (j >> 2), 8 + (j >> 2)
// and 12 + (j >> 2), in this order.
__device__ __forceinline__ s16x4 lds_read_tr(const char* p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)p);
}

// 16 bytes per lane from global memory straight into LDS: lane l's data lands at
// lds + 16*l (lds wave-uniform), its source is base (wave-uniform) + voff (per lane).
// Written in assembly on purpose: the compiler makes every later LDS read wait for ALL
// outstanding loads of this kind (it cannot tell the two LDS stages apart), which would
// serialise the prefetch of the next tile with the arithmetic on the current one.  The
// kernel orders these loads itself: s_waitcnt vmcnt(0) and a barrier before a stage is read.
__device__ __forceinline__ void lds_dma16(const char* base, uint32_t voff, char* lds) {
    const uint32_t m0 = (uint32_t)(uintptr_t)(lptr_t)lds;
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(m0), "v"(voff), "s"(base) : "memory", "m0");
}

__device__ __forceinline__ int items_of(int seq_len) {       // paired query tiles of one (sequence, head)
    return ((seq_len + kBM - 1) / kBM + 1) / 2;
}

// prefix sums of the number of items per (sequence, head) (ragged batches only)
__global__ __launch_bounds__(1024) void item_map_kernel(const int32_t* __restrict__ seq_offsets, int32_t n_seqs,
                                                        int32_t* __restrict__ item_map) {
    __shared__ int part[1024];
    const int tid = threadIdx.x;
    const int chunk = (n_seqs + 1023) / 1024;
    const int lo = min(tid * chunk, n_seqs), hi = min(lo + chunk, n_seqs);
    int sum = 0;
    for (int b = lo; b < hi; ++b) sum += items_of(seq_offsets[b + 1] - seq_offsets[b]);
    part[tid] = sum;
    __syncthreads();
    for (int d = 1; d < 1024; d <<= 1) {
        const int add = tid >= d ? part[tid - d] : 0;
        __syncthreads();
        part[tid] += add;
        __syncthreads();
    }
    int run = part[tid] - sum;
    for (int b = lo; b < hi; ++b) {
        item_map[b] = run;
        run += items_of(seq_offsets[b + 1] - seq_offsets[b]);
    }
    if (tid == 1023) item_map[n_seqs] = part[1023];
}

struct Segment {                // all fields wave-uniform
    int row0;                   // first packed row of the sequence
    int S;                      // its length
    int h, kvh;                 // query head, key/value head
    int q_base;                 // first query position of the segment
};

template <int D>
__global__ __launch_bounds__(kNW * 64, 2) void attention_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const int32_t* __restrict__ seq_offsets, const int32_t* __restrict__ item_map,
    int32_t n_seqs, int32_t n_q_heads, int32_t n_kv_heads, int32_t uniform_len, int32_t xcds,
    long long items_per_xcd, float c, uint16_t* __restrict__ out, float* __restrict__ lse) {
    using T = Tile<D>;
    constexpr int kKSteps = D / 16;               // MFMA k-steps over the head dimension
    constexpr int kDTiles = D / 32;               // 32-row tiles of O^T
    constexpr int kRowsPerInstr = 1024 / T::kRowBytes;          // rows one 64-lane x 16 B LDS-direct load fills
    constexpr int kInstrPerMat = kBN / kRowsPerInstr;
    constexpr int kInstrPerWave = kInstrPerMat / kNW;
    static_assert(kInstrPerMat % kNW == 0, "tile rows must split evenly over the wavefronts");
    constexpr int kLine = 256 / T::kRowBytes;                   // rows per 256-byte bank line (1 or 2)

    extern __shared__ __attribute__((aligned(16))) char smem[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 31;                     // row (A operand) / column (B, C) inside a 32-wide tile
    const int gl = lane >> 5;                     // which half of the k-slots / accumulator rows
    const int group = n_q_heads / n_kv_heads;

    // ---- item -> segments.  Consecutive workgroup ids sit on different XCDs (round robin), so
    // the id is split into (xcd, slot); the items of one XCD are ordered sequence, KV head,
    // tile pair, query head of the group: workgroups that run at the same time on an XCD read
    // the same K/V rows through its L2.
    const int xcd = blockIdx.x % xcds;
    const long long slot_stride = gridDim.x / xcds;
    const long long per_item = (long long)(n_kv_heads / xcds) * group;
    long long item = blockIdx.x / xcds;           // index inside this XCD's list
    int phase = 0;                                // 0: the late (long) tile of the pair, 1: the early one
    int it_pair = 0, it_nq = 0;                   // decoded item (uniform)
    Segment seg;

    // decode `item`/`phase` into sg; returns false when the list is exhausted
    auto decode = [&](Segment& sg) -> bool {
        if (item >= items_per_xcd) return false;
        if (phase == 0) {
            long long before;
            int b, n_items;
            if (uniform_len > 0) {
                n_items = items_of(uniform_len);
                b = (int)(item / (per_item * n_items));
                before = (long long)b * n_items;
            } else {
                int lo = 0, hi = n_seqs;
                while (hi - lo > 1) {
                    const int mid = (lo + hi) >> 1;
                    if (per_item * item_map[mid] <= item) lo = mid; else hi = mid;
                }
                b = lo;
                before = item_map[lo];
                n_items = item_map[lo + 1] - item_map[lo];
            }
            const long long rem = item - per_item * before;
            const int kv_local = (int)(rem / ((long long)n_items * group));
            const int rem2 = (int)(rem % ((long long)n_items * group));
            it_pair = rem2 / group;
            sg.kvh = kv_local * xcds + xcd;
            sg.h = sg.kvh * group + rem2 % group;
            sg.row0 = uniform_len > 0 ? b * uniform_len : seq_offsets[b];
            sg.S = uniform_len > 0 ? uniform_len : seq_offsets[b + 1] - sg.row0;
            it_nq = (sg.S + kBM - 1) / kBM;
            sg.q_base = (it_nq - 1 - it_pair) * kBM;
        } else {
            sg.q_base = it_pair * kBM;            // same sequence and head, the early tile
        }
        return true;
    };
    // step to the next segment of the list
    auto advance = [&]() {
        if (phase == 0 && it_nq - 1 - it_pair != it_pair) {
            phase = 1;
        } else {
            phase = 0;
            item += slot_stride;
        }
    };

    // ---- per-lane constants of the data movement
    // K/V tiles: instruction i of this wavefront fills LDS rows (wave*kInstrPerWave + i)*kRowsPerInstr ..
    // with lane l writing physical chunk l % kChunks of row l / kChunks; the lane therefore
    // fetches the logical chunk that the swizzle stores there.
    const uint32_t tok_bytes = (uint32_t)n_kv_heads * D * 2;
    const int l_row = lane / T::kChunks, l_chunk = lane % T::kChunks;
    uint32_t k_goff[kInstrPerWave], v_goff[kInstrPerWave];
#pragma unroll
    for (int i = 0; i < kInstrPerWave; ++i) {
        const int r = (wave * kInstrPerWave + i) * kRowsPerInstr + l_row;
        k_goff[i] = (uint32_t)r * tok_bytes + ((l_chunk ^ ((r / kLine) & (T::kChunks - 1))) << 4);
        v_goff[i] = (uint32_t)r * tok_bytes + ((l_chunk ^ (((r / kLine) & (T::kChunks / 4 - 1)) << 2)) << 4);
    }
    auto load_tile = [&](const Segment& sg, int t, int stage) {
        char* lds_k = smem + stage * T::kStageBytes + (wave * kInstrPerWave) * 1024;
        char* lds_v = lds_k + T::kMatBytes;
        const size_t first = ((size_t)(sg.row0 + t * kBN) * n_kv_heads + sg.kvh) * D * 2;
        const char* kt = (const char*)k + first;
        const char* vt = (const char*)v + first;
        const bool partial = (t + 1) * kBN > sg.S;   // last tile of a ragged sequence: rows past the end re-read row S-1
#pragma unroll
        for (int i = 0; i < kInstrPerWave; ++i) {
            uint32_t kg = k_goff[i], vg = v_goff[i];
            if (partial) {
                const int r = (wave * kInstrPerWave + i) * kRowsPerInstr + l_row;
                const uint32_t back = (uint32_t)max(t * kBN + r - (sg.S - 1), 0) * tok_bytes;
                kg -= back;
                vg -= back;
            }
            lds_dma16(kt, kg, lds_k + i * 1024);
            lds_dma16(vt, vg, lds_v + i * 1024);
        }
    };

    // query fragments: B operand of S^T = K Q^T, in registers for the whole segment
    bf16x8 qf[kKSteps];
    auto load_q = [&](const Segment& sg) {
        const int row = min(sg.q_base + 32 * wave + li, sg.S - 1);
        const uint16_t* src = q + ((size_t)(sg.row0 + row) * n_q_heads + sg.h) * D + 8 * gl;
#pragma unroll
        for (int ks = 0; ks < kKSteps; ++ks) qf[ks] = *(const bf16x8*)(src + 16 * ks);
    };

    // K row fed as A-operand row li of a 32-key sub-tile: bits 2 and 3 swapped (see header)
    const int krow = (li & ~12) | ((li & 4) << 1) | ((li & 8) >> 1);
    // Byte offset of this lane's K fragment inside a 32-row half: row krow, logical chunk
    // 2*ks + gl, physical chunk (2*ks + gl) ^ swz.  XOR is bitwise, so the offset for k-step ks
    // is k_lane ^ (ks << 5): one per-lane constant instead of one register per k-step.
    const int k_lane = krow * T::kRowBytes + ((gl ^ ((krow / kLine) & (T::kChunks - 1))) << 4);
    // V fragments come through the transposing read: this lane supplies the 8-byte word at key
    // 8*gl + ((lane & 15) >> 2) (+4 for the second read) of the 16-key step, head-dim columns
    // 32*dt + 16*((lane >> 4) & 1) + 4*(lane & 3) ..+3, i.e. half (lane & 1) of logical chunk
    // 4*dt + 2*((lane >> 4) & 1) + ((lane & 3) >> 1); the swizzle only touches chunk bits 2..3,
    // so the offset for tile dt is v_lane ^ (dt << 6).
    const int vrow = 8 * gl + ((lane & 15) >> 2);
    const int v_lane = vrow * T::kRowBytes +
                       (((((vrow / kLine) & (T::kChunks / 4 - 1)) << 2) + 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1)) << 4) +
                       8 * (lane & 1);

    // ---- state of the segment being computed
    f32x16 oacc[kDTiles];
    float m_run, l_run;
    int qlo, qrow;                                // first query position of the wavefront / of this lane
    auto reset_state = [&](const Segment& sg) {
#pragma unroll
        for (int dt = 0; dt < kDTiles; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[dt][r] = 0.f;
        m_run = -INFINITY;
        l_run = 0.f;
        qlo = sg.q_base + 32 * wave;
        qrow = qlo + li;
    };

    // One 64-key tile.  The two 32-key halves are two independent instruction streams that
    // are overlapped inside the wavefront: while the matrix pipe runs QK^T of the second half
    // the vector pipe exponentiates the first, and while it runs P V of the first half the
    // vector pipe exponentiates the second.  The tile is written as two pieces, tile_front
    // (up to the last use of the query fragments) and tile_back, so that the last tile of a
    // segment can request the next segment's query fragments in between.
    f32x16 s0, s1;
    bf16x8 pf[4];
    bf16x8 vf[kDTiles][2];
    int kl, vl;
    const char *Ks, *Vs;
    int key0, S;
    auto tile_begin = [&](const Segment& sg, int t, int stage) {
        Ks = smem + stage * T::kStageBytes;
        Vs = Ks + T::kMatBytes;
        key0 = t * kBN;
        S = sg.S;
        kl = k_lane;                                     // opaque per tile, see load_tile
        vl = v_lane;
        asm volatile("" : "+v"(kl), "+v"(vl));
    };

        auto k_frag = [&](int half, int ks) { return *(const bf16x8*)(Ks + 32 * half * T::kRowBytes + (kl ^ (ks << 5))); };
        auto v_frag = [&](int dt, int ks) {
            const char* p = Vs + 16 * ks * T::kRowBytes + (vl ^ (dt << 6));
            const s16x4 lo = lds_read_tr(p);
            const s16x4 hi = lds_read_tr(p + 4 * T::kRowBytes);
            return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
        };
        // causal / end-of-sequence mask of one half (diagonal tiles only; wave-uniform test)
        auto mask_half = [&](f32x16& sv, int half) {
            const int kbase = key0 + 32 * half;
            if ((kbase + 31 > qlo) || (kbase + 32 > S)) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = kbase + 16 * (r >> 3) + 8 * gl + (r & 7);
                    if (key > qrow || key >= S) sv[r] = -INFINITY;
                }
            }
        };
        // p = 2^(c s - c m) for one half against the CURRENT reference m: fp32 row sum of this
        // lane's 16 keys, bf16 fragments for the PV product.  No row maximum is taken: a
        // reference that has become too small shows up as a huge (or infinite, or NaN) sum.
        auto half_exp = [&](const f32x16& sv, bf16x8& p0, bf16x8& p1) -> float {
            const float mc = m_run * c;
            float lsum = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float a = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[e], c, -mc));
                const float b2 = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[8 + e], c, -mc));
                lsum += a + b2;
                p0[e] = (__bf16)a;
                p1[e] = (__bf16)b2;
            }
            return lsum;
        };
        // Rare path: some row of the wavefront outgrew the reference by more than 2^16 (always
        // the case on the first tile, where the reference is -inf).  Take the true row maxima,
        // move the reference, rescale what has been accumulated, redo the half.
        auto renew_half = [&](const f32x16& sv, bf16x8& p0, bf16x8& p1, float lsum) -> float {
            if (__ballot(!(lsum <= 65536.0f)) != 0) {
                float mx = sv[0];
#pragma unroll
                for (int r = 1; r < 16; r += 2) {
                    const float nxt = r + 1 < 16 ? sv[r + 1] : sv[r];
                    mx = fmaxf(fmaxf(mx, sv[r]), nxt);              // v_max3_f32
                }
                mx = max_with_other_half(mx);
                const float m_new = fmaxf(m_run, mx);
                const float alpha = m_new == m_run ? 1.0f : __builtin_amdgcn_exp2f((m_run - m_new) * c);
                l_run *= alpha;
#pragma unroll
                for (int dt = 0; dt < kDTiles; ++dt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) oacc[dt][r] *= alpha;
                m_run = m_new;
                lsum = half_exp(sv, p0, p1);
            }
            return lsum;
        };
        // Order wanted inside an overlapped region: one MFMA, then a share of the vector work
        // (a wavefront issues in order, so vector instructions placed behind a dependent MFMA
        // would wait for it), then a share of the LDS fragment reads of the next region.
        auto interleave = [&]() {
#pragma unroll
            for (int i = 0; i < kKSteps; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                    // MFMA
                __builtin_amdgcn_sched_group_barrier(0x402, 56 / kKSteps, 0);         // VALU + transcendental
                __builtin_amdgcn_sched_group_barrier(0x100, 2 * kDTiles * 2 / kKSteps, 0);   // DS reads
            }
        };

    auto tile_front = [&]() {
        // ---- R0: S0^T = K0 Q^T (keys 0..31 of the tile)
        {
            bf16x8 kf[kKSteps];
#pragma unroll
            for (int i = 0; i < kKSteps; ++i) kf[i] = k_frag(0, i);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int r = 0; r < 16; ++r) s0[r] = 0.f;
#pragma unroll
            for (int i = 0; i < kKSteps; ++i) s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[i], qf[i], s0, 0, 0, 0);
        }
        bf16x8 kf1[kKSteps];
#pragma unroll
        for (int i = 0; i < kKSteps; ++i) kf1[i] = k_frag(1, i);
        __builtin_amdgcn_sched_barrier(0);
        mask_half(s0, 0);
        __builtin_amdgcn_sched_barrier(0);

        // ---- R1: S1^T = K1 Q^T on the matrix pipe  ||  exponentials of the first half
#pragma unroll
        for (int r = 0; r < 16; ++r) s1[r] = 0.f;
#pragma unroll
        for (int i = 0; i < kKSteps; ++i) s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf1[i], qf[i], s1, 0, 0, 0);
        float ls = half_exp(s0, pf[0], pf[1]);
#pragma unroll
        for (int dt = 0; dt < kDTiles; ++dt)
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) vf[dt][ks] = v_frag(dt, ks);
        // keep the exponentials in this region (the optimiser would sink them to their first use)
        asm volatile("" : "+v"(pf[0]), "+v"(pf[1]), "+v"(ls));
        interleave();
        __builtin_amdgcn_sched_barrier(0);
        l_run += renew_half(s0, pf[0], pf[1], ls);
        mask_half(s1, 1);
        __builtin_amdgcn_sched_barrier(0);
    };
    auto tile_back = [&]() {
        // ---- R2: O^T += V0^T P0^T on the matrix pipe  ||  exponentials of the second half
#pragma unroll
        for (int dt = 0; dt < kDTiles; ++dt)
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
                oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[dt][ks], pf[ks], oacc[dt], 0, 0, 0);
        float ls = half_exp(s1, pf[2], pf[3]);
#pragma unroll
        for (int dt = 0; dt < kDTiles; ++dt)
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) vf[dt][ks] = v_frag(dt, 2 + ks);
        asm volatile("" : "+v"(pf[2]), "+v"(pf[3]), "+v"(ls));
        interleave();
        __builtin_amdgcn_sched_barrier(0);
        l_run += renew_half(s1, pf[2], pf[3], ls);
        __builtin_amdgcn_sched_barrier(0);

        // ---- R3: O^T += V1^T P1^T
#pragma unroll
        for (int dt = 0; dt < kDTiles; ++dt)
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
                oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[dt][ks], pf[2 + ks], oacc[dt], 0, 0, 0);
    };

    // normalise, round to bf16, store; log2 of the denominator for the score pass
    auto epilogue = [&](const Segment& sg) {
        const float ltot = sum_with_other_half(l_run);
        const float inv = 1.0f / ltot;
        if (qrow < sg.S) {
            uint16_t* dst = out + ((size_t)(sg.row0 + qrow) * n_q_heads + sg.h) * D + 4 * gl;
#pragma unroll
            for (int dt = 0; dt < kDTiles; ++dt)
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    bf16x4 o4;
#pragma unroll
                    for (int e = 0; e < 4; ++e) o4[e] = (__bf16)(oacc[dt][4 * a + e] * inv);
                    *(bf16x4*)(dst + 32 * dt + 8 * a) = o4;
                }
            if (lse != nullptr && gl == 0)
                lse[(size_t)(sg.row0 + qrow) * n_q_heads + sg.h] = m_run * c + __builtin_amdgcn_logf(ltot);
        }
    };

    // ---- the walk over this workgroup's segments
    if (!decode(seg)) return;
    int g = 0;                                    // tiles issued so far: LDS stage = g & 1
    load_q(seg);
    load_tile(seg, 0, 0);
    while (true) {
        // The query fragments must have landed before the sweep starts: a register load still
        // pending at the head of the tile loop would make every iteration wait for ALL
        // outstanding loads, the tile prefetch included.
#pragma unroll
        for (int ks = 0; ks < kKSteps; ++ks) asm volatile("" : "+v"(qf[ks]));
        reset_state(seg);
        const int n_kv_tiles = (min(seg.S, seg.q_base + kBM) + kBN - 1) / kBN;
        for (int t = 0; t + 1 < n_kv_tiles; ++t, ++g) {
            __builtin_amdgcn_s_waitcnt(0x0f70);   // vmcnt(0): this wavefront's share of tile t is in LDS
            __syncthreads();                      // everyone's share is; everyone left the other stage
            load_tile(seg, t + 1, (g + 1) & 1);
            // the wavefront takes part while some key of the tile is visible to its last row
            if (t * kBN <= qlo + 31) {
                tile_begin(seg, t, g & 1);
                tile_front();
                tile_back();
            }
        }
        // last tile of the segment: the other stage and the query registers go to the next
        // segment (when the list is exhausted the same fragments are simply fetched again)
        const int t_last = n_kv_tiles - 1;
        __builtin_amdgcn_s_waitcnt(0x0f70);
        __syncthreads();
        advance();
        Segment nxt = seg;
        const bool have_next = decode(nxt);
        if (have_next) load_tile(nxt, 0, (g + 1) & 1);
        const bool takes_part = t_last * kBN <= qlo + 31;
        if (takes_part) {
            tile_begin(seg, t_last, g & 1);
            tile_front();
        }
        load_q(nxt);
        if (takes_part) tile_back();
        ++g;
        epilogue(seg);
        if (!have_next) break;
        seg = nxt;
    }
}

int device_slots() {
    static int slots = 0;            // workgroups the device holds at 2 per compute unit
    if (slots == 0) {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
            cus = 256;
        slots = 2 * cus;
    }
    return slots;
}

template <int D>
int launch_attention_d(const void* q, const void* k, const void* v, const int32_t* seq_offsets_dev,
                       const pyr_shape& s, int32_t uniform_len, int64_t total_items, float c,
                       void* out, float* lse, int32_t* item_map, hipStream_t stream) {
    auto kern = attention_kernel<D>;
    static bool attr_done = false;   // benign race: the attribute call is idempotent
    if (!attr_done) {
        if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)Tile<D>::kLdsBytes) != hipSuccess)
            return PYR_ERR_LAUNCH;
        attr_done = true;
    }
    if (total_items == 0) return PYR_OK;
    if (uniform_len == 0) {
        hipLaunchKernelGGL(item_map_kernel, dim3(1), dim3(1024), 0, stream, seq_offsets_dev, s.n_seqs, item_map);
        if (check_launch() != PYR_OK) return PYR_ERR_LAUNCH;
    }
    const int xcds = (s.n_kv_heads % 8 == 0) ? 8 : 1;
    const long long items_per_xcd = (long long)total_items * s.n_q_heads / xcds;
    long long per_xcd_slots = device_slots() / xcds;
    if (per_xcd_slots > items_per_xcd) per_xcd_slots = items_per_xcd;
    const unsigned grid = (unsigned)(per_xcd_slots * xcds);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kNW * 64), Tile<D>::kLdsBytes, stream,
                       (const uint16_t*)q, (const uint16_t*)k, (const uint16_t*)v, seq_offsets_dev,
                       (const int32_t*)item_map, s.n_seqs, s.n_q_heads, s.n_kv_heads, uniform_len, xcds,
                       items_per_xcd, c, (uint16_t*)out, lse);
    return check_launch();
}

}  // namespace

int launch_attention(const void* q, const void* k, const void* v, const int32_t* seq_offsets_dev,
                     const pyr_shape& shape, int32_t uniform_len, int64_t total_items, float scale_log2,
                     void* out, float* lse, int32_t* item_map, hipStream_t stream) {
    if (shape.head_dim == 128)
        return launch_attention_d<128>(q, k, v, seq_offsets_dev, shape, uniform_len, total_items, scale_log2,
                                       out, lse, item_map, stream);
    return launch_attention_d<64>(q, k, v, seq_offsets_dev, shape, uniform_len, total_items, scale_log2,
                                  out, lse, item_map, stream);
}

}  // namespace pyr
