// Streaming vote kernel of the BRACE aggregation (device code, gfx950).
//
// What is computed (Sec. 3, Phases I-IV; Eq. (1)): for every coordinate k of a
// ring chunk, S[k] = sum over the n clients of sign(g_i[k]), and the result is
// +1 if S[k] > lambda, else -1, written at k's place in the global update.
//
// Shape of the work: a pure stream.  The n x d fp32 matrix is read exactly once
// (4*n bytes per coordinate) and a few bytes per coordinate are written, so the
// bound is HBM bandwidth.  There is no reuse, no contraction and no cross-lane
// traffic in the main loop: each lane owns V consecutive coordinates per load
// slot and keeps two small integer counters per coordinate (#positive,
// #negative) in registers while it walks down the n client rows.
//
// Launch layout.  The range [lo, hi) of a call is split in
//   body  [lo_a, hi_a): whole "wave slots" of 64*V coordinates, aligned from
//         coordinate 0, read with V-dword loads and no bounds checks;
//   edges [lo, lo_a) and [hi_a, hi): one thread per coordinate with dword
//         loads, run by the FIRST blocks of the same grid so that they overlap
//         with the body instead of trailing it.
// A wave owns COLS adjacent slots, i.e. a contiguous run of 64*V*COLS floats
// in every row; the row pointer is wave-uniform so row stepping is scalar
// arithmetic and each load is "scalar base + lane offset".
//
// Writes.  Interleaving even 1 % of writes with the read stream costs far more
// than 1 % of the time (the DRAM keeps turning the bus around and the writes
// land on scattered pages), so for large ranges the body only emits one bit per
// coordinate and a second, write-only kernel expands the bits to +-1.0f.

#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace brace_dev {

#ifndef BRACE_BLOCK
#define BRACE_BLOCK 256
#endif
constexpr int kBlock = BRACE_BLOCK;         // threads per block (waves of 64)
constexpr int kWaves = kBlock / 64;
constexpr int kXcds = 8;                    // MI355X: 8 XCDs, blocks are dealt round-robin
constexpr int kGroup = 1024;                // coordinates whose 32 bit-words fill one 128 B line

template <int V> struct Vec;
template <> struct Vec<1> { typedef float type; };
template <> struct Vec<2> { typedef float type __attribute__((ext_vector_type(2))); };
template <> struct Vec<4> { typedef float type __attribute__((ext_vector_type(4))); };

template <int V> struct IVec;
template <> struct IVec<1> { typedef short type; };
template <> struct IVec<2> { typedef short type __attribute__((ext_vector_type(2))); };
template <> struct IVec<4> { typedef short type __attribute__((ext_vector_type(4))); };

template <int V>
__device__ __forceinline__ float elem(const typename Vec<V>::type& v, int e)
{
    if constexpr (V == 1) return v; else return v[e];
}

template <int V, bool NT>
__device__ __forceinline__ typename Vec<V>::type load_vec(const float* p)
{
    typedef typename Vec<V>::type T;
    if constexpr (NT)
        return __builtin_nontemporal_load(reinterpret_cast<const T*>(p));
    else
        return *reinterpret_cast<const T*>(p);
}

template <bool NT, typename T>
__device__ __forceinline__ void store_vec(T* p, const T& v)
{
    if constexpr (NT)
        __builtin_nontemporal_store(v, p);
    else
        *p = v;
}

// Scalars of one launch.  Pointers are separate kernel parameters so that the compiler
// knows they are global memory and keeps wave-uniform address arithmetic in SGPRs.
struct VoteArgs {
    int64_t ld;             // row i at updates + i*ld
    int32_t n;
    int32_t thresh;         // result is +1 iff S >= thresh  (thresh = floor(lambda) + 1)
    int32_t zero_sign;
    int32_t swizzle;        // XCD-aware block -> tile map
    int64_t lo, hi;         // coordinates of this call
    int64_t lo_a, hi_a;     // aligned body
    int64_t d;              // full dimension (bit padding past d is zeroed)
    int64_t edge_blocks;    // blocks [0, edge_blocks) run the edges, the rest the body
    int64_t body_blocks;    // blocks that run the body
    int64_t tiles;          // tiles in the body; body block b takes tiles b, b + body_blocks, ...
    int32_t split;          // 1: the body emits bit-words only (a second kernel writes the floats)
    int32_t reserved;
};

typedef void (*vote_kernel_t)(const float*, float*, uint32_t*, int16_t*, const VoteArgs);

// Where the bit-word of coordinates [32j, 32j+32) lives when the floats' own buffer is used
// as scratch: the 32 words of a 1024-coordinate group sit in the first 128 bytes of the
// 4 KiB that the group expands to, so the expansion of a group only overwrites its own words.
__device__ __forceinline__ int64_t scratch_word(int64_t k)
{
    return (k & ~(int64_t)(kGroup - 1)) + ((k & (kGroup - 1)) >> 5);
}

// Sign-sum from the two counters (Phase I + II); the consensus map (Phase III) is
// "sum >= thresh".
__device__ __forceinline__ int sign_sum(int pos, int neg, int n, int zero_sign)
{
    return pos - neg + zero_sign * (n - pos - neg);
}

// One wave: COLS adjacent slots starting at wave-uniform coordinate k0.
// PIPE: the next batch of RU rows is requested before the current one is consumed, so the
// wave never drains its outstanding loads between batches.
// out == nullptr: no floats are written here; bit-words go to `bits` (linear layout) when
// given, else to `scratch` (the floats' buffer, scratch_word layout) when given.
template <int V, int COLS, int RU, bool NT, bool PIPE>
__device__ __forceinline__ void vote_slots(const float* __restrict__ updates,
                                           float* __restrict__ out, uint32_t* __restrict__ bits,
                                           uint32_t* __restrict__ scratch,
                                           int16_t* __restrict__ sums, int64_t ld, int n,
                                           int thresh, int zero_sign, int64_t k0, int lane)
{
    typedef typename Vec<V>::type VT;
    int pos[COLS][V], neg[COLS][V];
#pragma unroll
    for (int c = 0; c < COLS; ++c)
#pragma unroll
        for (int e = 0; e < V; ++e) { pos[c][e] = 0; neg[c][e] = 0; }

    const float* row = updates + k0;            // wave-uniform
    const uint32_t loff = (uint32_t)lane * V;   // per lane, in elements

    auto load_batch = [&](VT (&x)[RU][COLS]) {
#pragma unroll
        for (int r = 0; r < RU; ++r)
#pragma unroll
            for (int c = 0; c < COLS; ++c)
                x[r][c] = load_vec<V, NT>(row + (int64_t)r * ld + loff + c * (64 * V));
        row += (int64_t)RU * ld;
        // keep every load of the batch in flight before the first compare waits on one
        __builtin_amdgcn_sched_barrier(0);
    };
    auto count = [&](const VT (&x)[RU][COLS]) {
#pragma unroll
        for (int r = 0; r < RU; ++r)
#pragma unroll
            for (int c = 0; c < COLS; ++c)
#pragma unroll
                for (int e = 0; e < V; ++e) {
                    const float v = elem<V>(x[r][c], e);
                    pos[c][e] += (v > 0.0f) ? 1 : 0;
                    neg[c][e] += (v < 0.0f) ? 1 : 0;
                }
    };

    int i = 0;
    if constexpr (PIPE) {
        if (n >= RU) {
            VT xa[RU][COLS], xb[RU][COLS];
            load_batch(xa);
            i = RU;                             // rows [0, i) are requested
            while (i + 2 * RU <= n) {
                load_batch(xb);
                count(xa);
                load_batch(xa);
                count(xb);
                i += 2 * RU;
            }
            if (i + RU <= n) {
                load_batch(xb);
                i += RU;
                count(xa);
                count(xb);
            } else {
                count(xa);
            }
        }
    } else {
        for (; i + RU <= n; i += RU) {
            VT x[RU][COLS];
            load_batch(x);
            count(x);
        }
    }
    for (; i < n; ++i) {
        VT x[COLS];
#pragma unroll
        for (int c = 0; c < COLS; ++c)
            x[c] = load_vec<V, NT>(row + loff + c * (64 * V));
#pragma unroll
        for (int c = 0; c < COLS; ++c)
#pragma unroll
            for (int e = 0; e < V; ++e) {
                const float v = elem<V>(x[c], e);
                pos[c][e] += (v > 0.0f) ? 1 : 0;
                neg[c][e] += (v < 0.0f) ? 1 : 0;
            }
        row += ld;
    }

#pragma unroll
    for (int c = 0; c < COLS; ++c) {
        const int64_t k = k0 + c * (64 * V) + loff;
        int s[V];
        uint32_t mybits = 0;
#pragma unroll
        for (int e = 0; e < V; ++e) {
            s[e] = sign_sum(pos[c][e], neg[c][e], n, zero_sign);
            mybits |= (s[e] >= thresh ? 1u : 0u) << e;
        }
        if (out) {
            VT o;
#pragma unroll
            for (int e = 0; e < V; ++e) {
                const float v = (s[e] >= thresh) ? 1.0f : -1.0f;
                if constexpr (V == 1) o = v; else o[e] = v;
            }
            store_vec<NT>(reinterpret_cast<VT*>(out + k), o);
        }
        if (sums) {
            typedef typename IVec<V>::type ST;
            ST sv;
#pragma unroll
            for (int e = 0; e < V; ++e) {
                if constexpr (V == 1) sv = (short)s[e]; else sv[e] = (short)s[e];
            }
            store_vec<NT>(reinterpret_cast<ST*>(sums + k), sv);
        }
        if (bits || scratch) {
            // 32/V lanes share one 32-bit word; OR them together, the first lane stores.
            constexpr int L = 32 / V;
            uint32_t w = mybits << (V * (lane & (L - 1)));
#pragma unroll
            for (int m = 1; m < L; m <<= 1)
                w |= (uint32_t)__shfl_xor((int)w, m, 64);
            if ((lane & (L - 1)) == 0) {
                if (bits)
                    bits[k >> 5] = w;
                else
                    scratch[scratch_word(k)] = w;
            }
        }
    }
}

// Edge coordinates: one thread each, dword loads, bits merged atomically because a
// 32-bit word can be shared with a neighbouring chunk's call.
__device__ __forceinline__ void vote_edges(const float* __restrict__ updates,
                                           float* __restrict__ out, uint32_t* __restrict__ bits,
                                           int16_t* __restrict__ sums, const VoteArgs& a, int64_t e)
{
    const int64_t head = a.lo_a - a.lo;
    const int64_t k = (e < head) ? a.lo + e : a.hi_a + (e - head);
    int64_t hi_ext = a.hi;
    if (bits && a.hi == a.d)
        hi_ext = (a.d + 31) & ~(int64_t)31;      // zero the padding bits of the last word
    if (k >= hi_ext)
        return;
    if (k >= a.hi) {
        atomicAnd(&bits[k >> 5], ~(1u << (k & 31)));
        return;
    }
    const float* p = updates + k;
    int pos = 0, neg = 0;
    int i = 0;
    for (; i + 8 <= a.n; i += 8) {
        float v[8];
#pragma unroll
        for (int r = 0; r < 8; ++r)
            v[r] = p[(int64_t)r * a.ld];
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            pos += (v[r] > 0.0f) ? 1 : 0;
            neg += (v[r] < 0.0f) ? 1 : 0;
        }
        p += 8 * a.ld;
    }
    for (; i < a.n; ++i) {
        const float v = *p;
        pos += (v > 0.0f) ? 1 : 0;
        neg += (v < 0.0f) ? 1 : 0;
        p += a.ld;
    }
    const int s = sign_sum(pos, neg, a.n, a.zero_sign);
    const bool up = s >= a.thresh;
    if (out)
        out[k] = up ? 1.0f : -1.0f;
    if (sums)
        sums[k] = (int16_t)s;
    if (bits) {
        if (up)
            atomicOr(&bits[k >> 5], 1u << (k & 31));
        else
            atomicAnd(&bits[k >> 5], ~(1u << (k & 31)));
    }
}

template <int V, int COLS, int RU, bool NT, bool PIPE>
__global__ void __launch_bounds__(kBlock)
brace_vote_kernel(const float* __restrict__ updates, float* __restrict__ out,
                  uint32_t* __restrict__ bits, int16_t* __restrict__ sums, const VoteArgs a)
{
    if ((int64_t)blockIdx.x < a.edge_blocks) {
        vote_edges(updates, out, bits, sums, a, (int64_t)blockIdx.x * kBlock + threadIdx.x);
        return;
    }
    const int64_t b = (int64_t)blockIdx.x - a.edge_blocks;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    constexpr int64_t kSlot = 64 * V;
    const int64_t slots = (a.hi_a - a.lo_a) / kSlot;
    float* body_out = a.split ? nullptr : out;
    uint32_t* scratch = (a.split && !bits) ? reinterpret_cast<uint32_t*>(out) : nullptr;
    // With body_blocks == tiles every block runs one tile.  With fewer (resident) blocks a
    // block walks tiles b, b + body_blocks, ...
    for (int64_t t = b; t < a.tiles; t += a.body_blocks) {
        // Blocks are dealt to the 8 XCDs round-robin.  With the swizzle, XCD x works on the
        // x-th eighth of the tiles, so neighbouring tiles (which share boundary cache lines
        // when rows are not line-aligned) meet in the same L2.
        int64_t tile = t;
        if (a.swizzle) {
            const int64_t per = a.tiles / kXcds;       // tiles is a multiple of 8 here
            tile = (t % kXcds) * per + t / kXcds;
        }
        const int64_t s0 = (tile * kWaves + wave) * COLS;
        if (s0 >= slots)
            continue;
        const int64_t k0 = a.lo_a + s0 * kSlot;
        if (s0 + COLS <= slots) {
            vote_slots<V, COLS, RU, NT, PIPE>(updates, body_out, bits, scratch, sums, a.ld, a.n,
                                              a.thresh, a.zero_sign, k0, lane);
        } else {
            for (int64_t s = s0; s < slots; ++s)   // fewer than COLS slots left at the very end
                vote_slots<V, 1, RU, NT, PIPE>(updates, body_out, bits, scratch, sums, a.ld, a.n,
                                               a.thresh, a.zero_sign, a.lo_a + s * kSlot, lane);
        }
    }
}

template <int V, int COLS, int RU>
vote_kernel_t pick_nt(int nt, int pipe)
{
    if (pipe)
        return nt ? brace_vote_kernel<V, COLS, RU, true, true>
                  : brace_vote_kernel<V, COLS, RU, false, true>;
    return nt ? brace_vote_kernel<V, COLS, RU, true, false>
              : brace_vote_kernel<V, COLS, RU, false, false>;
}

template <int V, int COLS>
vote_kernel_t pick_ru(int ru, int nt, int pipe)
{
    switch (ru) {
    case 2: return pick_nt<V, COLS, 2>(nt, pipe);
    case 8: return pick_nt<V, COLS, 8>(nt, pipe);
    default: return pick_nt<V, COLS, 4>(nt, pipe);
    }
}

template <int V>
vote_kernel_t pick_cols(int cols, int ru, int nt, int pipe)
{
    switch (cols) {
    case 1: return pick_ru<V, 1>(ru, nt, pipe);
    case 2: return pick_ru<V, 2>(ru, nt, pipe);
    case 4: return pick_ru<V, 4>(ru, nt, pipe);
    default: return pick_ru<V, 8>(ru, nt, pipe);
    }
}

}  // namespace brace_dev

// One translation unit per load width instantiates its share of the kernels.
brace_dev::vote_kernel_t brace_vote_pick_v1(int cols, int ru, int nt, int pipe);
brace_dev::vote_kernel_t brace_vote_pick_v2(int cols, int ru, int nt, int pipe);
brace_dev::vote_kernel_t brace_vote_pick_v4(int cols, int ru, int nt, int pipe);
