// Causal softmax attention over packed, ragged sequences (Algorithm 1, "compute attention
// weights of KV", applied to V), flash style: the S x S weight matrix never exists.
//
// Work split.  The unit of work is a SEGMENT: kAttnBlockRows (256) consecutive query
// positions of one (sequence, query head); each of the 8 wavefronts of a workgroup owns 32 of
// them.  Segments are paired into ITEMS - query tile j of a sequence together with tile
// n-1-j - so every item of a sequence sweeps the same number of causal key tiles.  Workgroups
// are persistent, one per compute unit (two wavefronts per SIMD), each walking items with a
// fixed stride.  The 32-row blocks are dealt to the wavefronts so that the two wavefronts of a
// SIMD own blocks b and 7-b: every SIMD gets the same amount of causal work per segment.
//
// Keys/values stream through LDS in tiles of 64 positions in rings of four tiles each,
// written by the load unit itself (global_load ... lds), so they never pass through
// registers.  The tiles of all segments of a workgroup form ONE stream: the loads run ahead
// of the arithmetic across segment boundaries, so the compute unit never drains between
// segments.  The query rows take the same road (a small private LDS area per wavefront, in
// two halves) because loads into registers cost the vector memory path four times as much
// and, issued by eight wavefronts at once, used to hold up the K/V stream at every change of
// segment; for the same reason the output is stored 16 bytes per lane after a quad exchange
// between the two halves of the wavefront.
//
// MFMA mapping (v_mfma_f32_32x32x16_bf16, 64-lane wavefronts).  The kernel computes the
// TRANSPOSED logits  S^T = K Q^T  (keys x queries): in the accumulator layout a lane then
// holds 16 keys of ONE query column, so the softmax row statistics are per-lane scalars (one
// exchange with lane^32 completes them) and rescaling the output is a per-lane multiply.
// The output is accumulated transposed too,  O^T += V^T P^T,  whose B operand P^T is exactly
// what the lane already holds once the K rows of a 32-key sub-tile are fed in the order
// "bits 2 and 3 of the row number swapped".  V sits in LDS row-major like K; its A-operand
// fragments (8 keys of one head-dim column per lane) come out of LDS already transposed
// through ds_read_b64_tr_b16.
//
// Software pipeline inside a wavefront.  A 64-key tile is two 32-key halves; per half there
// is one group of MFMAs for the logits (QK) and one for the output (PV), and the
// exponentials of a half are cut in two chunks (E..a, E..b).  In the steady state every
// group of MFMAs is issued interleaved, instruction by instruction, with one chunk of
// exponentials of ANOTHER half and with the LDS reads of the next group's fragments:
//     QK0(t+1) | E1a(t)      PV0(t) | E1b(t)      QK1(t+1) | E0a(t+1)      PV1(t) | E0b(t+1)
// A matrix instruction keeps the matrix pipe busy for 32 cycles but occupies the issue port
// for about 10; the vector work of one slice (one FMA, one exponential, one add, half a
// convert per logit pair) fits in the remainder; the second wavefront of the SIMD, kept half a
// step apart, covers the rest (barriers, waits, cursor arithmetic).  The sum and the bf16
// pack of an exponential are issued one slice after it, so no slice waits on a transcendental.
// Scheduling barriers after every slice pin this order.
//
// Numerics: bf16 products, fp32 accumulation, fp32 online softmax in base 2 with the scale
// folded into one FMA per logit; probabilities are rounded to bf16 for the PV product while
// the softmax denominator is summed from the unrounded fp32 values.  The reference of the
// exponent is NOT the running row maximum: it is set from the true maxima of the first 32
// keys and afterwards only moved when some row's partial sum shows that it outgrew the
// reference by more than 2^16 (probabilities stay exact in fp32 and as precise in bf16 as at
// any other magnitude).  The common tile therefore takes no row maximum, no cross-lane
// exchange and no rescale of the output.
#include <type_traits>

#include "pyr_internal.h"

namespace pyr {
namespace {

constexpr int kBN = 64;                    // key positions per LDS tile
constexpr int kRing = 4;                   // LDS tiles per ring (one ring for K, one for V)

// LDS image of one K or V tile: 64 rows of D bf16, NO padding (the direct global->LDS loads
// fill 1 KiB of consecutive LDS per wavefront instruction).  Bank conflicts are avoided by an
// XOR swizzle of the 16-byte chunk index inside a row instead:
//   K: chunk ^ (row & 15)        -> the 16 rows a b128 fragment read touches hit 16 bank groups
//   V: chunk ^ ((row & 3) << 2)  -> the 4 rows x 64 B a transposing read touches tile the banks
// (for D = 64 two rows share a 256-byte bank line: row is replaced by row / 2 and the masks
// shrink to 7 and 1).
template <int D, int kNW>
struct Tile {
    static constexpr int kChunks = D / 8;                       // 16-byte chunks per row
    static constexpr int kRowBytes = D * 2;
    static constexpr int kMatBytes = kBN * kRowBytes;           // one K or V tile
    static constexpr int kQStageBytes = 32 * kRowBytes / 2;     // half of a wavefront's 32 query rows
    static constexpr size_t kLdsBytes = 2 * (size_t)kRing * kMatBytes + (size_t)kNW * kQStageBytes;
};

typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
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
__device__ __forceinline__ s16x4 lds_read_tr(int lds_addr) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(uintptr_t)lds_addr);
}

// 16 bytes per lane from global memory straight into LDS: lane l's data lands at
// lds + 16*l (lds wave-uniform), its source is base (wave-uniform) + voff (per lane).
// Written in assembly on purpose: the compiler would make every later LDS read wait for ALL
// outstanding loads of this kind (it cannot tell the ring slots apart).  The kernel orders
// these loads itself: s_waitcnt vmcnt(0) and a barrier before a slot is read.
__device__ __forceinline__ void lds_dma16(const char* base_, uint32_t voff, uint32_t lds_addr) {
    const uint32_t m0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)lds_addr);
    const uint64_t b64 = (uint64_t)(uintptr_t)base_;         // wave-uniform by construction: keep it in scalar registers
    const uint32_t b_lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)b64);          // (the builtin returns a signed int:
    const uint32_t b_hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(b64 >> 32));  //  widen it unsigned)
    const char* base = (const char*)(uintptr_t)(((uint64_t)b_hi << 32) | (uint64_t)b_lo);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(m0), "v"(voff), "s"(base) : "memory", "m0");
}

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {      // v_cvt_pk_bf16_f32
    bf16x2 v;
    v[0] = (__bf16)a;
    v[1] = (__bf16)b;
    return __builtin_bit_cast(uint32_t, v);
}

__host__ __device__ __forceinline__ int items_of(int seq_len, int block_rows) {       // paired query tiles of one (sequence, head)
    return ((seq_len + block_rows - 1) / block_rows + 1) / 2;
}

// prefix sums of the number of items per (sequence, head) (ragged batches only)
__global__ __launch_bounds__(1024) void item_map_kernel(const int32_t* __restrict__ seq_offsets, int32_t n_seqs,
                                                        int32_t block_rows, int32_t* __restrict__ item_map) {
    __shared__ int part[1024];
    const int tid = threadIdx.x;
    const int chunk = (n_seqs + 1023) / 1024;
    const int lo = min(tid * chunk, n_seqs), hi = min(lo + chunk, n_seqs);
    int sum = 0;
    for (int b = lo; b < hi; ++b) sum += items_of(seq_offsets[b + 1] - seq_offsets[b], block_rows);
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
        run += items_of(seq_offsets[b + 1] - seq_offsets[b], block_rows);
    }
    if (tid == 1023) item_map[n_seqs] = part[1023];
}

struct Segment {                // all fields wave-uniform
    int row0;                   // first packed row of the sequence
    int S;                      // its length
    int h, kvh;                 // query head, key/value head
    int q_base;                 // first query position of the segment
    int n_tiles;                // key tiles the workgroup sweeps for it
};

// A position in the workgroup's list of segments (and, for the load cursors, in the stream
// of key tiles).  All fields wave-uniform.
struct Walker {
    int j;                      // index inside this workgroup's list of items
    int phase;                  // 0: the late (long) tile of the pair, 1: the early one
    int pair, nq;               // decoded item: pair index, query tiles of the sequence
    int t;                      // key tile inside the segment (load cursors only)
    Segment seg;
};

template <int D, int kNW>
__global__ __launch_bounds__(kNW * 64, 2) void attention_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const int32_t* __restrict__ seq_offsets, const int32_t* __restrict__ item_map,
    int32_t n_seqs, int32_t n_q_heads, int32_t n_kv_heads, int32_t uniform_len, int32_t xcds,
    int32_t items_per_xcd, int32_t first_wave_slots, float c, uint16_t* __restrict__ out, float* __restrict__ lse,
    int32_t* __restrict__ zero_ptr, int32_t zero_count) {
    using T = Tile<D, kNW>;
    constexpr int kBM = kNW * 32;                 // query positions per segment
    constexpr int NS = D / 16;                    // MFMAs per group = k-steps of QK^T = V fragments of a half
    constexpr int kDTiles = D / 32;               // 32-row tiles of O^T
    constexpr int EPS = 8 / NS;                   // logits of a chunk handled per slice (1 or 2)
    constexpr int kLook = NS - 2;                 // slices between the LDS read of a fragment and its MFMA
    constexpr int kRowsPerInstr = 1024 / T::kRowBytes;          // rows one 64-lane x 16 B LDS-direct load fills
    constexpr int kInstrPerMat = kBN / kRowsPerInstr;
    constexpr int kInstrPerWave = kInstrPerMat / kNW;
    static_assert(kInstrPerMat % kNW == 0 && kInstrPerWave >= 1, "tile rows must split evenly over the wavefronts");
    constexpr int kLine = 256 / T::kRowBytes;                   // rows per 256-byte bank line (1 or 2)

    extern __shared__ __attribute__((aligned(16))) char smem[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // A service to the kernels that follow on the stream: their arrival counters start at zero.
    if (blockIdx.x == 0)
        for (int i = tid; i < zero_count; i += kNW * 64) zero_ptr[i] = 0;
    // 32-row block of this wavefront.  Eight wavefronts: SIMD s owns blocks s and 7-s.  Four: one wavefront per
    // SIMD, and the second workgroup of a compute unit (slot >= first_wave_slots) deals the blocks the other
    // way round, so that the two wavefronts sharing a SIMD again own blocks s and 3-s.
    const int rb = kNW == 8 ? (wave < 4 ? wave : 11 - wave)
                            : ((int)(blockIdx.x / xcds) >= first_wave_slots ? kNW - 1 - wave : wave);
    const int li = lane & 31;                     // row (A operand) / column (B, C) inside a 32-wide tile
    const int gl = lane >> 5;                     // which half of the k-slots / accumulator rows
    const int group = n_q_heads / n_kv_heads;

    // ---- item -> segments.  Consecutive workgroup ids sit on different XCDs (round robin), so
    // the id is split into (xcd, slot); the items of one XCD are ordered sequence, KV head,
    // tile pair, query head of the group: workgroups that run at the same time on an XCD read
    // the same K/V rows through its L2.
    const int xcd = blockIdx.x % xcds;
    const int slot_stride = gridDim.x / xcds;
    const int per_item = (n_kv_heads / xcds) * group;    // (the host checked that the item count fits 31 bits)

    // This workgroup takes the items first, first + stride, ... of its XCD's list.  Turning an item number
    // into (sequence, heads, tile pair) costs integer divisions (or a search through the ragged batch's
    // prefix sums), far too slow for the scalar unit at a change of segment; so the lanes do it, 64 items at
    // a time: lane l of every wavefront holds item tbl_base + l of the workgroup's list, decoded, in four
    // registers, and a walker fetches an entry with four v_readlane.
    const int first_item = blockIdx.x / xcds;
    const int n_mine = (items_per_xcd - first_item + slot_stride - 1) / slot_stride;
    int tbl_base = 0;
    int t_row0 = 0, t_len = 0, t_heads = 0, t_pair = 0;       // per lane: first row, length, h | kvh << 16, pair | tiles << 16
    auto fill_table = [&](int base) __attribute__((always_inline)) {
        tbl_base = base;
        const int jj = base + lane;
        if (jj < n_mine) {
            const int item = first_item + jj * slot_stride;
            int before, b, n_items;
            if (uniform_len > 0) {
                n_items = items_of(uniform_len, kBM);
                b = item / (per_item * n_items);
                before = b * n_items;
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
            const int rem = item - per_item * before;
            const int kv_local = rem / (n_items * group);
            const int rem2 = rem % (n_items * group);
            const int kvh = kv_local * xcds + xcd;
            t_row0 = uniform_len > 0 ? b * uniform_len : seq_offsets[b];
            t_len = uniform_len > 0 ? uniform_len : seq_offsets[b + 1] - t_row0;
            t_heads = (kvh * group + rem2 % group) | (kvh << 16);
            t_pair = (rem2 / group) | (((t_len + kBM - 1) / kBM) << 16);
        }
        // The entries may come out of global loads (ragged batches).  Use them once here: the compiler then waits
        // for those loads now, not at every later fetch - where its wait would also cover the key/value tiles in
        // flight and the output rows just stored, a full memory latency at every change of segment.
        asm volatile("" : "+v"(t_row0), "+v"(t_len), "+v"(t_heads), "+v"(t_pair));
    };
    // decode w.j / w.phase into w.seg; false when the list is exhausted.  (The table is moved along once per
    // segment, in the main loop, far enough ahead of every walker: kTableMargin.)
    constexpr int kTableMargin = 16;              // items a walker may advance during one segment, generously
    auto decode = [&](Walker& w) __attribute__((always_inline)) -> bool {
        if (w.j >= n_mine) return false;
        Segment& sg = w.seg;
        if (w.phase == 0) {
            const int rel = w.j - tbl_base;
            sg.row0 = __builtin_amdgcn_readlane(t_row0, rel);
            sg.S = __builtin_amdgcn_readlane(t_len, rel);
            const int hk = __builtin_amdgcn_readlane(t_heads, rel), pn = __builtin_amdgcn_readlane(t_pair, rel);
            sg.h = hk & 0xffff;
            sg.kvh = (int)((unsigned)hk >> 16);
            w.pair = pn & 0xffff;
            w.nq = (int)((unsigned)pn >> 16);
            sg.q_base = (w.nq - 1 - w.pair) * kBM;
        } else {
            sg.q_base = w.pair * kBM;             // same sequence and head, the early tile
        }
        sg.n_tiles = (min(sg.S, sg.q_base + kBM) + kBN - 1) / kBN;
        return true;
    };
    // step to the next segment of the list; false (w unchanged) when there is none
    auto next_segment = [&](Walker& w) __attribute__((always_inline)) -> bool {
        Walker n = w;
        if (n.phase == 0 && n.nq - 1 - n.pair != n.pair) {
            n.phase = 1;
        } else {
            n.phase = 0;
            n.j += 1;
        }
        if (!decode(n)) return false;
        n.t = 0;
        w = n;
        return true;
    };
    // ---- per-lane constants of the data movement
    // K/V tiles: instruction i of this wavefront fills LDS rows (wave*kInstrPerWave + i)*kRowsPerInstr ..
    // with lane l writing physical chunk l % kChunks of row l / kChunks; the lane therefore
    // fetches the logical chunk that the swizzle stores there.
    const uint32_t tok_bytes = (uint32_t)n_kv_heads * D * 2;
    const uint32_t lds_base = (uint32_t)(uintptr_t)(lptr_t)smem;
    const int l_row = lane / T::kChunks, l_chunk = lane % T::kChunks;
    uint32_t k_goff[kInstrPerWave], v_goff[kInstrPerWave];
#pragma unroll
    for (int i = 0; i < kInstrPerWave; ++i) {
        const int r = (wave * kInstrPerWave + i) * kRowsPerInstr + l_row;
        k_goff[i] = (uint32_t)r * tok_bytes + ((l_chunk ^ ((r / kLine) & (T::kChunks - 1))) << 4);
        v_goff[i] = (uint32_t)r * tok_bytes + ((l_chunk ^ (((r / kLine) & (T::kChunks / 4 - 1)) << 2)) << 4);
    }
    struct LoadPos { size_t off; int t, S; };     // a tile of the stream, as far as the loads care: byte offset of its
                                                  // first row and head in k and v, tile number, sequence length
    auto pos_of = [&](const Walker& w) __attribute__((always_inline)) -> LoadPos {
        return LoadPos{((size_t)(w.seg.row0 + w.t * kBN) * n_kv_heads + w.seg.kvh) * D * 2, w.t, w.seg.S};
    };
    // instruction i of this wavefront's share of the K (which == 0) or V tile at position p, into ring slot `slot`
    // A tile may reach past the end of a ragged sequence: its rows past the end re-read row S-1.
    // The per-lane source offsets in force for the K tile and the V tile being requested are
    // kept in registers (k_eff, v_eff) and only touched when a ragged tile comes or goes.
    auto ragged = [&](const LoadPos& p) __attribute__((always_inline)) { return (p.t + 1) * kBN > p.S; };
    uint32_t k_eff[kInstrPerWave], v_eff[kInstrPerWave];
    bool k_rag = false, v_rag = false;
    auto set_k_eff = [&](const LoadPos& p) __attribute__((always_inline)) {
        k_rag = ragged(p);
#pragma unroll
        for (int i = 0; i < kInstrPerWave; ++i) {
            const int r = (wave * kInstrPerWave + i) * kRowsPerInstr + l_row;
            const uint32_t back = k_rag ? (uint32_t)max(p.t * kBN + r - (p.S - 1), 0) * tok_bytes : 0u;
            k_eff[i] = k_goff[i] - back;
        }
    };
    // instruction i of this wavefront's share of the K (which == 0) or V tile at position p, into ring slot `slot`
    auto load_piece = [&](const LoadPos& p, int which, int slot, int i) __attribute__((always_inline)) {
        const uint32_t lds = lds_base + (which * kRing + slot) * T::kMatBytes + (wave * kInstrPerWave + i) * 1024;
        lds_dma16((const char*)(which == 0 ? k : v) + p.off, which == 0 ? k_eff[i] : v_eff[i], lds);
    };

    // K row fed as A-operand row li of a 32-key sub-tile: bits 2 and 3 swapped (see header)
    const int krow = (li & ~12) | ((li & 4) << 1) | ((li & 8) >> 1);
    // Byte offset of this lane's K fragment inside a 32-row half: row krow, logical chunk
    // 2*ks + gl, physical chunk (2*ks + gl) ^ swz, i.e. k_lane ^ (ks << 5).
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
    // LDS addresses of the fragments.  The ring slot is part of the register: kaddr points into the
    // K slot of stream position "kpos", vaddr into the V slot of position "vpos"; both are moved on
    // by one slot once per stream position (bump_k, bump_v).  The half and the 16-key step are
    // immediates.
    int kaddr[NS], vaddr[kDTiles];
    const int lds0 = (int)(uintptr_t)(lptr_t)smem;
#pragma unroll
    for (int i = 0; i < NS; ++i) kaddr[i] = lds0 + (k_lane ^ (i << 5));
#pragma unroll
    for (int dt = 0; dt < kDTiles; ++dt)
        vaddr[dt] = lds0 + (2 * kRing - 1) * T::kMatBytes + (v_lane ^ (dt << 6));     // V ring behind the K ring; last slot
    int kslot = 0, vslot = kRing - 1;             // wave-uniform
    auto bump_k = [&]() __attribute__((always_inline)) {
        const int delta = kslot == kRing - 1 ? -(kRing - 1) * T::kMatBytes : T::kMatBytes;
        kslot = kslot == kRing - 1 ? 0 : kslot + 1;
#pragma unroll
        for (int i = 0; i < NS; ++i) kaddr[i] += delta;
    };
    auto bump_v = [&]() __attribute__((always_inline)) {
        const int delta = vslot == kRing - 1 ? -(kRing - 1) * T::kMatBytes : T::kMatBytes;
        vslot = vslot == kRing - 1 ? 0 : vslot + 1;
#pragma unroll
        for (int dt = 0; dt < kDTiles; ++dt) vaddr[dt] += delta;
    };

    auto k_frag = [&](int half, int i) __attribute__((always_inline)) {
        return *(const bf16x8 __attribute__((address_space(3)))*)(uintptr_t)(kaddr[i] + 32 * half * T::kRowBytes);
    };
    // V fragment i of half `half`: 16-key step 2*half + i / kDTiles, head-dim tile i % kDTiles
    auto v_frag = [&](int half, int i) __attribute__((always_inline)) {
        const int p = vaddr[i % kDTiles] + 16 * (2 * half + i / kDTiles) * T::kRowBytes;
        const s16x4 lo = lds_read_tr(p);
        const s16x4 hi = lds_read_tr(p + 4 * T::kRowBytes);
        return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };

    // ---- registers of the wavefront
    bf16x8 qf[NS];                                // query fragments: B operand of S^T = K Q^T
    bf16x8 F[NS];                                 // A-operand fragments (K or V) of the group in flight and, from
                                                  // slot 0 up, of the group after it: fragment j always sits in F[j]
    f32x16 oacc[kDTiles];                         // O^T
    f32x16 s0, s1;                                // logits of the two halves
    u32x4 p0[2], p1[2];                           // probabilities of the two halves, bf16, two 16-key steps each
    float m_run, nmc, l_run;                      // exponent reference, -c * reference, row denominators (this lane's keys)
    float ls0, ls1;                               // partial denominators of the half in flight

    // segment being computed, as seen by this wavefront
    Segment cs;
    int qlo = 0, qrow = 0;                        // first query position of the wavefront / of this lane
    int H = 0;                                    // 32-key halves this wavefront needs (the last one holds the diagonal)
    int n_my = 0;                                 // key tiles this wavefront takes part in
    auto enter_segment = [&](const Segment& sg) __attribute__((always_inline)) {
        cs = sg;
        qlo = sg.q_base + 32 * rb;
        qrow = qlo + li;
        H = qlo / 32 + 1;
        n_my = qlo < sg.S ? (H + 1) / 2 : 0;
    };
    // ---- the workgroup's stream of key tiles
    Walker nx;                                    // walks the list of segments one ahead of the arithmetic
    fill_table(0);
    nx.j = 0;
    nx.phase = 0;
    nx.pair = nx.nq = nx.t = 0;
    if (!decode(nx)) return;
    Walker lc = nx;                               // load cursor: the K tile kRing stream positions ahead
    LoadPos kp = pos_of(lc);                      // its tile,
    LoadPos vp = kp;                              // and the tile before it: V runs one position behind K
    set_k_eff(kp);
#pragma unroll
    for (int i = 0; i < kInstrPerWave; ++i) v_eff[i] = v_goff[i];
    enter_segment(nx.seg);                        // cs: the segment being computed; nx: the one after it
    bool has_next = next_segment(nx);
    int lslot = 0;                                // ring slot the next K tile is loaded into (V: the slot before it)
    int q_age = 0;                                // stream positions requested since the next segment's first query half was

    // The loads of one stream position: 2 * kInstrPerWave instructions per wavefront, K first.
    auto request_piece = [&](int idx) __attribute__((always_inline)) {
        if (idx < kInstrPerWave) load_piece(kp, 0, lslot, idx);
        else load_piece(vp, 1, lslot == 0 ? kRing - 1 : lslot - 1, idx - kInstrPerWave);
    };
    auto request_end = [&]() __attribute__((always_inline)) {
        vp = kp;
        if (lc.t + 1 < lc.seg.n_tiles) {          // next tile of the same segment
            ++lc.t;
            ++kp.t;
            kp.off += (size_t)kBN * tok_bytes;
        } else {                                  // first tile of the next segment (past the end: the same tile again)
            next_segment(lc);
            kp = pos_of(lc);
        }
        lslot = lslot == kRing - 1 ? 0 : lslot + 1;
        ++q_age;
        if (k_rag || v_rag || ragged(kp)) {       // rare: the V offsets take over what the K tile had, K gets its own
#pragma unroll
            for (int i = 0; i < kInstrPerWave; ++i) v_eff[i] = v_goff[i] - (k_goff[i] - k_eff[i]);
            v_rag = k_rag;
            set_k_eff(kp);
        }
    };
    auto request = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int idx = 0; idx < 2 * kInstrPerWave; ++idx) request_piece(idx);
        request_end();
    };
    // The synchronisation of stream position g, run by every wavefront once, anywhere between its
    // last read of K(g+1) and its first read of K(g+2): afterwards K(g+2) and V(g+1) are in LDS and
    // the slots of K(g) and V(g-1) may be overwritten (by K(g+4) and V(g+3): `request`).  Only the
    // loads of the youngest position may still be in flight after the wait.
    // (No wait for this wavefront's LDS reads: the slots written next were last read a whole
    // stream position ago, and every fragment read then has been consumed by an MFMA since.)
    // Half of the wavefronts (one of the two on every SIMD) synchronise two groups earlier in
    // their steady-state step than the other half, which keeps the two wavefronts of a SIMD half
    // a step apart: while one is between groups (checks, cursor arithmetic, the barrier itself)
    // the other one feeds the matrix pipe.
    const bool early_sync = kNW == 8 && wave >= kNW / 2;

    // ---- query fragments.  Loads into registers pass the vector memory path at a quarter of the
    // rate of loads that write LDS, and eight of them per wavefront at every change of segment held
    // up the K/V loads of the whole workgroup.  The 32 query rows of a wavefront therefore come
    // through a private LDS area of half their size, in two halves of the head dimension:
    //   half 0 of the NEXT segment is requested as soon as a segment starts (the area is free then),
    //   copied into registers once the current segment's last QK^T has been issued (q_turn), and
    //   half 1 is requested into the same area at that moment and copied when the next segment starts.
    // Rows are fetched 16 bytes per lane, 8 (4) lanes per 128-byte (64-byte) half row, chunks
    // XOR-swizzled by row like the K tile.
    constexpr int kQChunks = D / 16;                            // 16-byte chunks per half row
    constexpr int kQRowsPerInstr = 64 / kQChunks;
    constexpr int kQInstr = 32 / kQRowsPerInstr;                // load instructions per half
    const uint32_t qstage = lds_base + 2 * kRing * T::kMatBytes + wave * T::kQStageBytes;
    const int qs_row = lane / kQChunks, qs_chunk = lane % kQChunks;
    auto q_request = [&](const Segment& sg, int half) __attribute__((always_inline)) {
        const int first = min(sg.q_base + 32 * rb, sg.S - 1);   // rows past the end re-read the last row
        const char* base = (const char*)(q + ((size_t)(sg.row0 + first) * n_q_heads + sg.h) * D);
#pragma unroll
        for (int i = 0; i < kQInstr; ++i) {
            const int row = kQRowsPerInstr * i + qs_row;
            const uint32_t voff = (uint32_t)min(row, sg.S - 1 - first) * ((uint32_t)n_q_heads * D * 2) +
                                  (((qs_chunk ^ (row & (kQChunks - 1))) + half * kQChunks) << 4);
            lds_dma16(base, voff, qstage + 1024 * i);
        }
    };
    auto q_copy = [&](int half) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < NS / 2; ++j) {
            const int a = (int)qstage + ((li * kQChunks + ((2 * j + gl) ^ (li & (kQChunks - 1)))) << 4);
            qf[half * (NS / 2) + j] = *(const bf16x8 __attribute__((address_space(3)))*)(uintptr_t)a;
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");      // in registers: the area may be overwritten
    };
    // Once the current segment's last QK^T has been issued (the fragments are dead): half 0 into registers,
    // request half 1 into the same area.
    auto q_turn = [&]() __attribute__((always_inline)) {
        // Half 0 was requested when the current segment started.  Once a whole stream position has been requested
        // after it, the wait of the synchronisation just passed has covered it; only in a very short segment it
        // may still be among the youngest loads.
        if (q_age == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        q_copy(0);
        q_request(nx.seg, 1);
    };
    // at the start of a segment: half 1 has landed (a whole stream position was requested after it)
    auto wait_q = [&]() __attribute__((always_inline)) {
        asm volatile("s_waitcnt vmcnt(%0)" :: "n"(2 * kInstrPerWave) : "memory");
        q_copy(1);
        if (has_next) q_request(nx.seg, 0);
        q_age = 0;
    };
    auto sync = [&](bool with_q) __attribute__((always_inline)) {
        asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" :: "n"(2 * kInstrPerWave) : "memory");
        if (with_q && has_next) q_turn();
    };

    // ---- slices.  Everything below is written in the order it should be issued; a scheduling
    // barrier after every slice keeps it.
    // exponentials of logits sv[base + EPS*i ..] into fragment pf (element EPS*i ..)
    float pend = 0.f;                             // even element waiting for its partner (EPS == 1)
    float last_e = 0.f;                           // the exponential of the slice before (EPS == 1)
    auto e_use = [&](int j, u32x4& pf, float& lsum) __attribute__((always_inline)) {
        lsum += last_e;
        asm volatile("" : "+v"(lsum));
        if (j & 1) {
            pf[j >> 1] = pack_bf16(pend, last_e);
            asm volatile("" : "+v"(pf[j >> 1]));
        } else {
            pend = last_e;
        }
    };
    auto e_slice = [&](const f32x16& sv, int base, int i, u32x4& pf, float& lsum) __attribute__((always_inline)) {
        if (EPS == 2) {
            float a = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[base + 2 * i], c, nmc));
            float b = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[base + 2 * i + 1], c, nmc));
            lsum += a;
            lsum += b;
            pf[i] = pack_bf16(a, b);
            asm volatile("" : "+v"(pf[i]), "+v"(lsum));   // computed HERE: the optimiser would sink it to its first use
        } else {
            // The sum and the bf16 pack of an exponential are issued one slice after it: used
            // straight away, every exponential costs a wait state.
            float a = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[base + i], c, nmc));
            asm volatile("" : "+v"(a));                   // computed HERE: the optimiser would sink it to its first use
            if (i > 0) e_use(i - 1, pf, lsum);
            last_e = a;
            if (i == NS - 1) e_use(i, pf, lsum);
        }
    };
    auto fence = [&]() __attribute__((always_inline)) { __builtin_amdgcn_sched_barrier(0); };

    // What a group does besides its MFMAs.
    struct Chunk {                                // a chunk of exponentials: logits se[base ..+7] -> pe, lsum
        bool on;
        const f32x16* se;
        int base;
        u32x4* pe;
        float* lsum;
    };
    struct Frags {                                // a set of NS fragments in LDS: kind 0 none, 1 K (at kpos), 2 V (at vpos)
        int kind, half;
    };
    auto frag = [&](const Frags& f, int j) __attribute__((always_inline)) -> bf16x8 {
        return f.kind == 1 ? k_frag(f.half, j) : v_frag(f.half, j);
    };
    // fragments 0 .. kLook-1 of a group that no previous group fetched
    auto prime = [&](const Frags& f) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < kLook; ++j) F[j] = frag(f, j);
    };
    // the load of slice i: fragment i + kLook of the own set, or of the next group's set
    auto slice_load = [&](const Frags& own, const Frags& next, int i) __attribute__((always_inline)) {
        const int j = i + kLook;
        if (j < NS) {
            if (own.kind != 0) F[j] = frag(own, j);
        } else {
            if (next.kind != 0) F[j - NS] = frag(next, j - NS);
        }
    };
    // QK group: sd = K_half Q^T
    auto qk_group = [&](f32x16& sd, const Chunk& e, const Frags& own, const Frags& next) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < NS; ++i) {
            if (i == 0) {
                f32x16 z;
#pragma unroll
                for (int r = 0; r < 16; ++r) z[r] = 0.f;
                sd = __builtin_amdgcn_mfma_f32_32x32x16_bf16(F[0], qf[0], z, 0, 0, 0);
            } else {
                sd = __builtin_amdgcn_mfma_f32_32x32x16_bf16(F[i], qf[i], sd, 0, 0, 0);
            }
            if (e.on) e_slice(*e.se, e.base, i, *e.pe, *e.lsum);
            slice_load(own, next, i);
            fence();
        }
    };
    // PV group: O^T += V_half^T P_half^T (fragment i: 16-key step i / kDTiles, head-dim tile i % kDTiles)
    // With `loads` every other slice also requests one piece of the stream position being loaded.
    auto pv_group = [&](const u32x4 (&pp)[2], const Chunk& e, const Frags& own, const Frags& next, bool loads)
                        __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < NS; ++i) {
            oacc[i % kDTiles] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                F[i], __builtin_bit_cast(bf16x8, pp[i / kDTiles]), oacc[i % kDTiles], 0, 0, 0);
            if (e.on) e_slice(*e.se, e.base, i, *e.pe, *e.lsum);
            slice_load(own, next, i);
            if (loads) {
                if (NS == 2 * kInstrPerWave) request_piece(i);       // one piece per slice
                else if (i & 1) request_piece(i >> 1);               // one every other slice
            }
            fence();
        }
    };
    static_assert(NS / 2 == 2 * kInstrPerWave || NS == 2 * kInstrPerWave, "the slices of one group cover a stream position");
    // a chunk of exponentials alone
    auto e_group = [&](const f32x16& se, int ebase, u32x4& pe, float& lsum) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < NS; ++i) e_slice(se, ebase, i, pe, lsum);
    };
    const Chunk no_e = {false, &s0, 0, &p0[0], &ls0};
    const Frags no_f = {0, 0};
    const Frags fk0 = {1, 0}, fk1 = {1, 1}, fv0 = {2, 0}, fv1 = {2, 1};

    // causal mask of half number hh (0, 1, 2, ... along the keys) of this wavefront: nothing
    // below the diagonal half H-1, the triangle inside it, everything beyond it
    const int diag = li - 8 * gl;                 // register r of a diagonal half is masked if 16*(r>>3) + (r&7) > diag
    auto mask_half = [&](f32x16& sv, int hh) __attribute__((always_inline)) {
        if (hh >= H - 1) {
            int thr = hh > H - 1 ? -1 : diag;
            asm volatile("" : "+v"(thr));         // (opaque: 16 lane masks hoisted out of the loops would cost 32 scalar registers)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (16 * (r >> 3) + (r & 7) > thr) sv[r] = -INFINITY;
        }
    };
    // Rare path: some row of the wavefront outgrew the reference by more than 2^16.  Take the
    // true row maxima of the half, move the reference, rescale what has been accumulated, redo
    // the half.
    auto settle_half = [&](const f32x16& sv, u32x4 (&pp)[2], float lsum) __attribute__((always_inline)) {
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
            nmc = -m_new * c;
            lsum = 0.f;
            e_group(sv, 0, pp[0], lsum);
            e_group(sv, 8, pp[1], lsum);
        }
        l_run += lsum;
    };

    // First steps of a segment, run while the previous segment's last tile is the current
    // stream position (kpos = tile 0 of the new segment):
    //   QK0(0), reference from its true maxima, QK1(0) | E0a(0), E0b(0).
    auto pre_iteration = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int dt = 0; dt < kDTiles; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[dt][r] = 0.f;
        l_run = 0.f;
        prime(fk0);
        qk_group(s0, no_e, fk0, fk1);
        mask_half(s0, 0);
        float mx = s0[0];
#pragma unroll
        for (int r = 1; r < 16; r += 2) {
            const float nxt = r + 1 < 16 ? s0[r + 1] : s0[r];
            mx = fmaxf(fmaxf(mx, s0[r]), nxt);
        }
        m_run = max_with_other_half(mx);          // key 0 is visible to every row: finite
        nmc = -m_run * c;
        ls0 = 0.f;
        fence();
        const Chunk e0a = {true, &s0, 0, &p0[0], &ls0};
        qk_group(s1, e0a, fk1, no_f);
        e_group(s0, 8, p0[1], ls0);
        l_run += ls0;
        mask_half(s1, 1);
        fence();
    };

    // One stream position in the steady state: tile t (probabilities, PV; vpos) and tile t+1
    // (logits; kpos on entry).  Leaves kpos at tile t+2 with its first fragments in F.
    auto steady = [&](int t) __attribute__((always_inline)) {
        const Chunk e1a = {true, &s1, 0, &p1[0], &ls1}, e1b = {true, &s1, 8, &p1[1], &ls1};
        const Chunk e0a = {true, &s0, 0, &p0[0], &ls0}, e0b = {true, &s0, 8, &p0[1], &ls0};
        ls1 = 0.f;
        bump_v();
        qk_group(s0, e1a, fk0, fv0);              // QK0(t+1) | E1a(t)
        if (early_sync) sync(false);
        pv_group(p0, e1b, fv0, fk1, false);       // PV0(t)   | E1b(t)
        settle_half(s1, p1, ls1);
        mask_half(s0, 2 * t + 2);
        fence();
        ls0 = 0.f;
        qk_group(s1, e0a, fk1, fv1);              // QK1(t+1) | E0a(t+1)
        if (!early_sync) sync(t + 2 == n_my);     // (the query fragments are dead from here on if this was the last QK)
        bump_k();
        fence();
        pv_group(p1, e0b, fv1, fk0, true);        // PV1(t)   | E0b(t+1) | loads of the next stream position
        request_end();
        settle_half(s0, p0, ls0);
        mask_half(s1, 2 * t + 3);
        fence();
    };
    // The wavefront's last tile of the segment: no further logits.
    auto last = [&]() __attribute__((always_inline)) {
        const Chunk e1b = {true, &s1, 8, &p1[1], &ls1};
        ls1 = 0.f;
        prime(fv0);
        e_group(s1, 0, p1[0], ls1);
        fence();
        pv_group(p0, e1b, fv0, fv1, false);       // PV0(t) | E1b(t)
        settle_half(s1, p1, ls1);
        fence();
        pv_group(p1, no_e, fv1, no_f, false);     // PV1(t)
    };

    // normalise, round to bf16, store; log2 of the denominator for the score pass
    auto epilogue = [&]() __attribute__((always_inline)) {
        const float ltot = sum_with_other_half(l_run);
        const float inv = 1.0f / ltot;
        // A lane holds 4 consecutive head-dim values of its row per accumulator quad (those of the
        // other half-wavefront's lane follow them).  Stores cost the vector memory path one slot
        // per lane whatever their width, so two quads are traded with the partner lane first: every
        // lane then owns 8 consecutive values and stores 16 bytes.
        u32x4 o16[kDTiles][2];
#pragma unroll
        for (int dt = 0; dt < kDTiles; ++dt)
#pragma unroll
            for (int ap = 0; ap < 2; ++ap) {
                uint32_t lo[2], hi[2];              // quads a = 2*ap and a = 2*ap + 1, two packed pairs each
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    lo[e] = pack_bf16(oacc[dt][8 * ap + 2 * e] * inv, oacc[dt][8 * ap + 2 * e + 1] * inv);
                    hi[e] = pack_bf16(oacc[dt][8 * ap + 4 + 2 * e] * inv, oacc[dt][8 * ap + 4 + 2 * e + 1] * inv);
                    // afterwards lanes 0..31 hold their own quad 2*ap and the partner's, lanes 32..63 the
                    // partner's quad 2*ap + 1 and their own
                    auto r = __builtin_amdgcn_permlane32_swap(lo[e], hi[e], false, false);
                    o16[dt][ap][e] = r[0];
                    o16[dt][ap][2 + e] = r[1];
                }
            }
        if (qrow < cs.S) {
            uint16_t* dst = out + ((size_t)(cs.row0 + qrow) * n_q_heads + cs.h) * D + 8 * gl;
#pragma unroll
            for (int dt = 0; dt < kDTiles; ++dt)
#pragma unroll
                for (int ap = 0; ap < 2; ++ap) *(u32x4*)(dst + 32 * dt + 16 * ap) = o16[dt][ap];
            if (lse != nullptr && gl == 0)
                lse[(size_t)(cs.row0 + qrow) * n_q_heads + cs.h] = m_run * c + __builtin_amdgcn_logf(ltot);
        }
    };

    // ---- the walk
    q_request(cs, 0);                             // the first segment's queries: both halves one after the other
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    q_copy(0);
    q_request(cs, 1);
    // K(0), K(1), V(0) first, then two more positions; wait for the first three
#pragma unroll
    for (int i = 0; i < kInstrPerWave; ++i) load_piece(kp, 0, 0, i);
    request_end();
    request();
    request();
    request();
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" :: "n"(4 * kInstrPerWave) : "memory");

    while (true) {
        // kpos is tile 0 of the segment cs; the stream position is the one before it
        wait_q();
        if (n_my > 0) pre_iteration();
        bump_k();
        if (n_my > 1) prime(fk0);
        const int n_wg = cs.n_tiles;
        int t = 0;
#pragma unroll 1
        for (; t + 1 < n_my; ++t) steady(t);
#pragma unroll 1
        for (; t < n_wg; ++t) {
            bump_v();
            sync(early_sync ? t == max(n_my - 1, 0) : n_my < 2 && t == 0);     // (with the next segment's queries once the fragments are dead)
            request();
            if (t + 1 == n_my) {
                last();
                epilogue();
            }
            if (t + 1 < n_wg) bump_k();           // (the last position's move happens after the next segment's first steps)
        }
        if (!has_next) break;
        enter_segment(nx.seg);
        // keep the item table ahead of both walkers (they are never more than a few items apart)
        if (max(nx.j, lc.j) + kTableMargin >= tbl_base + 64 && tbl_base + 64 < n_mine) fill_table(min(nx.j, lc.j));
        has_next = next_segment(nx);
    }
    __builtin_amdgcn_s_waitcnt(0x0f70);           // no load may still be writing LDS when the workgroup ends
}

template <int D, int kNW>
int launch_attention_d(const void* q, const void* k, const void* v, const int32_t* seq_offsets_dev,
                       const int32_t* seq_offsets_host, const pyr_shape& s, int32_t uniform_len, float c,
                       void* out, float* lse, int32_t* item_map, int32_t* zero_ptr, int32_t zero_count,
                       hipStream_t stream) {
    auto kern = attention_kernel<D, kNW>;
    using T = Tile<D, kNW>;
    constexpr int kBM = kNW * 32;
    static std::atomic<uint64_t> lds_set{0};
    if (ensure_dynamic_lds((const void*)kern, (int)T::kLdsBytes, &lds_set) != PYR_OK) return PYR_ERR_LAUNCH;
    long long total_items = 0;                       // work items per query head
    for (int32_t b = 0; b < s.n_seqs; ++b) total_items += items_of(seq_offsets_host[b + 1] - seq_offsets_host[b], kBM);
    if (total_items == 0) return PYR_OK;
    if (total_items * s.n_q_heads >= (1ll << 31)) return PYR_ERR_UNSUPPORTED;
    DeviceInfo dev;
    if (device_info(&dev) != PYR_OK) return PYR_ERR_LAUNCH;
    if (uniform_len == 0) {
        hipLaunchKernelGGL(item_map_kernel, dim3(1), dim3(1024), 0, stream, seq_offsets_dev, s.n_seqs, (int32_t)kBM, item_map);
        if (check_launch() != PYR_OK) return PYR_ERR_LAUNCH;
    }
    // Workgroup ids go round robin over the XCDs; the items are split by KV head so that one XCD's L2 serves
    // one head's K/V rows.  That needs the KV heads to divide evenly; otherwise one list for the whole device.
    const int xcds = (s.n_kv_heads % dev.xccs == 0 && dev.compute_units % dev.xccs == 0) ? dev.xccs : 1;
    const int32_t items_per_xcd = (int32_t)(total_items * s.n_q_heads / xcds);
    const int wgs_per_cu = (int)(160 * 1024 / T::kLdsBytes) >= 2 ? 2 : 1;    // persistent workgroups, as many as the LDS holds
    const int32_t first_wave_slots = dev.compute_units / xcds;
    long long per_xcd_slots = (long long)first_wave_slots * wgs_per_cu;
    if (per_xcd_slots > items_per_xcd) per_xcd_slots = items_per_xcd;
    const unsigned grid = (unsigned)(per_xcd_slots * xcds);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kNW * 64), T::kLdsBytes, stream,
                       (const uint16_t*)q, (const uint16_t*)k, (const uint16_t*)v, seq_offsets_dev,
                       (const int32_t*)item_map, s.n_seqs, s.n_q_heads, s.n_kv_heads, uniform_len, xcds,
                       items_per_xcd, first_wave_slots, c, (uint16_t*)out, lse, zero_ptr, zero_count);
    return check_launch();
}

}  // namespace

int launch_attention(const void* q, const void* k, const void* v, const int32_t* seq_offsets_dev,
                     const int32_t* seq_offsets_host, const pyr_shape& shape, int32_t uniform_len, float scale_log2,
                     void* out, float* lse, int32_t* item_map, int32_t* zero_ptr, int32_t zero_count,
                     hipStream_t stream) {
    // Segments of 256 query rows (eight wavefronts) make the most of every K/V tile brought into LDS; when they
    // leave compute units without work (small batches), segments of 128 rows (four wavefronts) double the number
    // of work items.
    DeviceInfo dev;
    if (device_info(&dev) != PYR_OK) return PYR_ERR_LAUNCH;
    long long items256 = 0;
    for (int32_t b = 0; b < shape.n_seqs; ++b) items256 += items_of(seq_offsets_host[b + 1] - seq_offsets_host[b], 256);
    const bool small = items256 * shape.n_q_heads < dev.compute_units;
    if (shape.head_dim == 128)
        return small ? launch_attention_d<128, 4>(q, k, v, seq_offsets_dev, seq_offsets_host, shape, uniform_len, scale_log2,
                                                  out, lse, item_map, zero_ptr, zero_count, stream)
                     : launch_attention_d<128, 8>(q, k, v, seq_offsets_dev, seq_offsets_host, shape, uniform_len, scale_log2,
                                                  out, lse, item_map, zero_ptr, zero_count, stream);
    return small ? launch_attention_d<64, 4>(q, k, v, seq_offsets_dev, seq_offsets_host, shape, uniform_len, scale_log2,
                                             out, lse, item_map, zero_ptr, zero_count, stream)
                 : launch_attention_d<64, 8>(q, k, v, seq_offsets_dev, seq_offsets_host, shape, uniform_len, scale_log2,
                                             out, lse, item_map, zero_ptr, zero_count, stream);
}

}  // namespace pyr
