// Streaming column-reduction skeleton for gfx950: one pass over an n x d fp32 matrix that
// folds the n client rows of every coordinate into a small per-coordinate state held in
// registers, then hands the state to an epilogue.  The BRACE vote (Sec. 3, Phases I-IV) and
// the plain ring-all-reduce sum it replaces (Sec. 2.2) are two "ops" plugged into it.
//
// Shape of the work: a pure stream.  The matrix is read exactly once (4*n bytes per
// coordinate) and a few bytes per coordinate are written, so the bound is HBM bandwidth.
// There is no reuse, no contraction and no cross-lane traffic in the main loop.
//
// Launch layout.  The range [lo, hi) of a call is split in
//   body  [lo_a, hi_a): whole "wave slots" of 64*V coordinates, aligned from coordinate 0,
//         read with V-dword loads and no bounds checks;
//   edges [lo, lo_a) and [hi_a, hi) (+ whatever padding the op asks for): one thread per
//         coordinate with dword loads, run by the FIRST blocks of the same grid so that
//         they overlap with the body instead of trailing it.
// A wave owns COLS adjacent slots, i.e. a contiguous run of 64*V*COLS floats in every row;
// the row pointer is wave-uniform so row stepping is scalar arithmetic and each load is
// "scalar base + lane offset".  Rows are requested in batches of RU rows x COLS loads; with
// PIPE the next batch is requested before the current one is consumed, so a wave never
// drains its outstanding loads between batches.
//
// Short ranges (a single ring chunk, small models) do not have enough columns to fill 256
// compute units with one wave per slot.  In row-split mode the 4 waves of a block share the
// same slots, each folds a quarter of the client rows, and the partial states meet in LDS.
//
// An op provides
//   struct State;                                  per-coordinate accumulator
//   static void init(State&);
//   static void add(State&, float);                fold one client's value
//   static void merge(State&, const State&);       combine two partial states (row split)
//   template <int V, bool NT> void store_body(int64_t k, const State (&)[V], int lane, int n) const;
//                                                  lane's V consecutive coordinates from k
//   void store_edge(int64_t k, const State&, int n) const;     one coordinate
//   void pad_edge(int64_t k) const;                coordinate in [hi, hi_ext): op-specific padding
// and, for the staged variant (one float per coordinate, written in large bursts):
//   template <int V> Vec<V>::type stage_prefetch(int64_t k) const;
//                                                  what the op wants to have read before the
//                                                  rows of a tile (old values it updates)
//   float stage_value(const State&, int n, float old) const;
//                                                  the float a coordinate ends up as
//   void flush4(int64_t k, f32x4 v) const;         consume 4 consecutive coordinates from k

#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace brace_dev {

#ifndef BRACE_BLOCK
#define BRACE_BLOCK 256
#endif
constexpr int kBlock = BRACE_BLOCK;         // threads per block (waves of 64)
constexpr int kWaves = kBlock / 64;

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

template <int V>
__device__ __forceinline__ void set_elem(typename Vec<V>::type& v, int e, float x)
{
    if constexpr (V == 1) v = x; else v[e] = x;
}

// Row loads only promise 4-byte alignment: with a pitch that is not a multiple of 4 elements
// every client row has its own 16-byte phase, and gfx950 global loads of 2 or 4 dwords do not
// need more than dword alignment.  Aligned rows get the same instruction.
template <int V, bool NT>
__device__ __forceinline__ typename Vec<V>::type load_vec(const float* p)
{
    typedef typename Vec<V>::type T;
    typedef T TU __attribute__((aligned(4)));
    if constexpr (NT)
        return __builtin_nontemporal_load(reinterpret_cast<const TU*>(p));
    else
        return *reinterpret_cast<const TU*>(p);
}

template <bool NT, typename T>
__device__ __forceinline__ void store_vec(T* p, const T& v)
{
    if constexpr (NT)
        __builtin_nontemporal_store(v, p);
    else
        *p = v;
}

typedef float f32x4 __attribute__((ext_vector_type(4)));

// Scalars of one launch that do not depend on the op.
struct StreamArgs {
    int64_t ld;             // row i at updates + i*ld
    int32_t n;
    int32_t reserved;
    int64_t lo, hi;         // coordinates of this call
    int64_t lo_a, hi_a;     // aligned body
    int64_t hi_ext;         // edges run up to here; [hi, hi_ext) is op-specific padding
    int64_t edge_blocks;    // blocks [0, edge_blocks) run the edges, the rest the body
};

// One wave folds rows [0, n) starting at `updates` (already offset to its first row) into the
// states of COLS adjacent slots starting at wave-uniform coordinate k0, in row order.
template <class Op, int V, int COLS, int RU, bool NT, bool PIPE>
__device__ __forceinline__ void stream_fold(const float* __restrict__ updates, int64_t ld, int n,
                                            int64_t k0, int lane,
                                            typename Op::State (&st)[COLS][V])
{
    typedef typename Vec<V>::type VT;
    const float* row = updates + k0;            // wave-uniform
    const uint32_t loff = (uint32_t)lane * V;   // per lane, in elements

    auto load_batch = [&](VT (&x)[RU][COLS]) {
#pragma unroll
        for (int r = 0; r < RU; ++r)
#pragma unroll
            for (int c = 0; c < COLS; ++c)
                x[r][c] = load_vec<V, NT>(row + (int64_t)r * ld + loff + c * (64 * V));
        row += (int64_t)RU * ld;
        // keep every load of the batch in flight before the first use waits on one
        __builtin_amdgcn_sched_barrier(0);
    };
    auto fold = [&](const VT (&x)[RU][COLS]) {
#pragma unroll
        for (int r = 0; r < RU; ++r)
#pragma unroll
            for (int c = 0; c < COLS; ++c)
#pragma unroll
                for (int e = 0; e < V; ++e)
                    Op::add(st[c][e], elem<V>(x[r][c], e));
    };

    int i = 0;
    if constexpr (PIPE) {
        if (n >= RU) {
            VT xa[RU][COLS], xb[RU][COLS];
            load_batch(xa);
            i = RU;                             // rows [0, i) are requested
            while (i + 2 * RU <= n) {
                load_batch(xb);
                fold(xa);
                load_batch(xa);
                fold(xb);
                i += 2 * RU;
            }
            if (i + RU <= n) {
                load_batch(xb);
                i += RU;
                fold(xa);
                fold(xb);
            } else {
                fold(xa);
            }
        }
    } else {
        for (; i + RU <= n; i += RU) {
            VT x[RU][COLS];
            load_batch(x);
            fold(x);
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
            for (int e = 0; e < V; ++e)
                Op::add(st[c][e], elem<V>(x[c], e));
        row += ld;
    }
}

// The same from freshly initialised states.
template <class Op, int V, int COLS, int RU, bool NT, bool PIPE>
__device__ __forceinline__ void stream_accumulate(const float* __restrict__ updates, int64_t ld,
                                                  int n, int64_t k0, int lane,
                                                  typename Op::State (&st)[COLS][V])
{
#pragma unroll
    for (int c = 0; c < COLS; ++c)
#pragma unroll
        for (int e = 0; e < V; ++e)
            Op::init(st[c][e]);
    stream_fold<Op, V, COLS, RU, NT, PIPE>(updates, ld, n, k0, lane, st);
}

// COLS slots from k0: the whole column reduction and its epilogue.  In row-split mode the
// block's waves each take a contiguous share of the rows; partial states of waves 1.. are
// parked in LDS (`lds`, (kWaves-1) x COLS*V x 64 states) and wave 0 merges and stores.
template <class Op, int V, int COLS, int RU, bool NT, bool PIPE, bool RS>
__device__ __forceinline__ void stream_slots(const float* __restrict__ updates, int64_t ld, int n,
                                             int64_t k0, int lane, int wave, const Op& op)
{
    typedef typename Op::State State;
    State st[COLS][V];
    if constexpr (!RS) {
        stream_accumulate<Op, V, COLS, RU, NT, PIPE>(updates, ld, n, k0, lane, st);
    } else {
        extern __shared__ unsigned char lds_raw[];
        State* lds = reinterpret_cast<State*>(lds_raw);
        const int r0 = (int)(((int64_t)n * wave) / kWaves);
        const int r1 = (int)(((int64_t)n * (wave + 1)) / kWaves);
        stream_accumulate<Op, V, COLS, RU, NT, PIPE>(updates + (int64_t)r0 * ld, ld, r1 - r0, k0,
                                                     lane, st);
        if (wave > 0) {
#pragma unroll
            for (int c = 0; c < COLS; ++c)
#pragma unroll
                for (int e = 0; e < V; ++e)
                    lds[((wave - 1) * (COLS * V) + c * V + e) * 64 + lane] = st[c][e];
        }
        __syncthreads();
        if (wave == 0) {
            for (int w = 0; w < kWaves - 1; ++w)
#pragma unroll
                for (int c = 0; c < COLS; ++c)
#pragma unroll
                    for (int e = 0; e < V; ++e)
                        Op::merge(st[c][e], lds[(w * (COLS * V) + c * V + e) * 64 + lane]);
        }
        __syncthreads();                        // LDS is reused by the next slot of a ragged tile
        if (wave > 0)
            return;
    }
#pragma unroll
    for (int c = 0; c < COLS; ++c)
        op.template store_body<V, NT>(k0 + c * (64 * V) + (int64_t)lane * V, st[c], lane, n);
}

// Edge coordinates: one thread each, dword loads, 8 rows in flight.
template <class Op>
__device__ __forceinline__ void stream_edges(const float* __restrict__ updates,
                                             const StreamArgs& a, int64_t e, const Op& op)
{
    const int64_t head = a.lo_a - a.lo;
    const int64_t k = (e < head) ? a.lo + e : a.hi_a + (e - head);
    if (k >= a.hi_ext)
        return;
    if (k >= a.hi) {
        op.pad_edge(k);
        return;
    }
    typename Op::State st;
    Op::init(st);
    const float* p = updates + k;
    int i = 0;
    for (; i + 8 <= a.n; i += 8) {
        float v[8];
#pragma unroll
        for (int r = 0; r < 8; ++r)
            v[r] = p[(int64_t)r * a.ld];
#pragma unroll
        for (int r = 0; r < 8; ++r)
            Op::add(st, v[r]);
        p += 8 * a.ld;
    }
    for (; i < a.n; ++i) {
        Op::add(st, *p);
        p += a.ld;
    }
    op.store_edge(k, st, a.n);
}

template <class Op, int V, int COLS, int RU, bool NT, bool PIPE, bool RS>
__global__ void __launch_bounds__(kBlock)
stream_kernel(const float* __restrict__ updates, const StreamArgs a, const Op op)
{
    if ((int64_t)blockIdx.x < a.edge_blocks) {
        stream_edges<Op>(updates, a, (int64_t)blockIdx.x * kBlock + threadIdx.x, op);
        return;
    }
    const int64_t b = (int64_t)blockIdx.x - a.edge_blocks;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    constexpr int64_t kSlot = 64 * V;
    const int64_t slots = (a.hi_a - a.lo_a) / kSlot;
    // One tile per block.  (Measured and dropped: an XCD-aware block -> tile map and resident
    // blocks walking several tiles; neither moved the time by more than noise.)
    const int64_t tile = b;
    // Row split: all waves of the block share the tile's COLS slots (block-uniform flow).
    const int64_t s0 = RS ? tile * COLS : (tile * kWaves + wave) * COLS;
    if (s0 >= slots)
        return;
    if (s0 + COLS <= slots) {
        stream_slots<Op, V, COLS, RU, NT, PIPE, RS>(updates, a.ld, a.n, a.lo_a + s0 * kSlot, lane,
                                                    wave, op);
    } else {
        for (int64_t s = s0; s < slots; ++s)       // fewer than COLS slots left at the very end
            stream_slots<Op, V, 1, RU, NT, PIPE, RS>(updates, a.ld, a.n, a.lo_a + s * kSlot, lane,
                                                     wave, op);
    }
}

// Staged variant for ops whose result is one float per coordinate with no compact form
// (plain sum / mean, in-place model update).  Stores issued from inside the read stream cost
// far more than their share of the bytes; the smaller and more scattered they are, the worse.
// Here a block runs `stage_tiles` adjacent tiles one after the other, parks their results in
// LDS, and then writes them as ONE contiguous burst (128 KiB at the default shape) with
// full-line non-temporal stores.  Measured on the n = 100, d = 25 M sum: 1.456 ms against
// 1.50-1.52 ms with per-wave stores, on a box where the read-only floor is 1.43 ms.
template <class Op, int V, int COLS, int RU, bool PIPE>
__global__ void __launch_bounds__(kBlock)
stream_staged_kernel(const float* __restrict__ updates, const StreamArgs a, const Op op,
                     const int stage_tiles)
{
    if ((int64_t)blockIdx.x < a.edge_blocks) {
        stream_edges<Op>(updates, a, (int64_t)blockIdx.x * kBlock + threadIdx.x, op);
        return;
    }
    extern __shared__ unsigned char lds_raw[];
    float* stage = reinterpret_cast<float*>(lds_raw);
    typedef typename Op::State State;
    const int64_t b = (int64_t)blockIdx.x - a.edge_blocks;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    constexpr int64_t kSlot = 64 * V;
    constexpr int64_t kTileSlots = (int64_t)kWaves * COLS;
    const int64_t slots = (a.hi_a - a.lo_a) / kSlot;
    const int64_t slot0 = b * stage_tiles * kTileSlots;         // first slot of this block's group
    for (int t = 0; t < stage_tiles; ++t) {
        const int64_t s0 = slot0 + (t * kTileSlots + (int64_t)wave * COLS);
        if (s0 >= slots)
            break;                                              // wave-uniform; the barrier is below
        if (s0 + COLS <= slots) {
            State st[COLS][V];
            typename Vec<V>::type old[COLS];
#pragma unroll
            for (int c = 0; c < COLS; ++c)
                old[c] = op.template stage_prefetch<V>(a.lo_a + (s0 + c) * kSlot + lane * V);
            stream_accumulate<Op, V, COLS, RU, true, PIPE>(updates, a.ld, a.n, a.lo_a + s0 * kSlot,
                                                           lane, st);
#pragma unroll
            for (int c = 0; c < COLS; ++c)
#pragma unroll
                for (int e = 0; e < V; ++e)
                    stage[(s0 - slot0 + c) * kSlot + lane * V + e] =
                        op.stage_value(st[c][e], a.n, elem<V>(old[c], e));
        } else {
            for (int64_t s = s0; s < slots; ++s) {              // ragged end of the range
                State st[1][V];
                const typename Vec<V>::type old =
                    op.template stage_prefetch<V>(a.lo_a + s * kSlot + lane * V);
                stream_accumulate<Op, V, 1, RU, true, PIPE>(updates, a.ld, a.n, a.lo_a + s * kSlot,
                                                            lane, st);
#pragma unroll
                for (int e = 0; e < V; ++e)
                    stage[(s - slot0) * kSlot + lane * V + e] =
                        op.stage_value(st[0][e], a.n, elem<V>(old, e));
            }
        }
    }
    __syncthreads();
    const int64_t base = a.lo_a + slot0 * kSlot;
    int64_t valid = (int64_t)stage_tiles * kTileSlots * kSlot;
    if (valid > a.hi_a - base)
        valid = a.hi_a - base;                                  // a multiple of kSlot, hence of 4
    for (int64_t i = (int64_t)threadIdx.x * 4; i < valid; i += kBlock * 4)
        op.flush4(base + i, *reinterpret_cast<const f32x4*>(stage + i));
}

template <class Op>
using stream_staged_kernel_t = void (*)(const float*, const StreamArgs, const Op, int);

constexpr int kStageColsWide = 8;           // the staged variant exists for the two large-range
constexpr int kStageColsNarrow = 4;         // shapes: 8 loads per row, and 4 for few clients
constexpr int kStageUnroll = 2;
constexpr size_t kStageBytes = 128 * 1024;  // burst per block; the LDS of a compute unit is 160 KiB

template <class Op, int V>
stream_staged_kernel_t<Op> pick_staged(int cols, int pipe)
{
    if (cols == kStageColsNarrow)
        return pipe ? stream_staged_kernel<Op, V, kStageColsNarrow, kStageUnroll, true>
                    : stream_staged_kernel<Op, V, kStageColsNarrow, kStageUnroll, false>;
    return pipe ? stream_staged_kernel<Op, V, kStageColsWide, kStageUnroll, true>
                : stream_staged_kernel<Op, V, kStageColsWide, kStageUnroll, false>;
}

// Kernel lookup by launch tuning; instantiates the whole table for one (Op, V).  Row-split
// kernels exist for 1 and 2 loads per row (short ranges never want more), non-temporal only.
template <class Op>
using stream_kernel_t = void (*)(const float*, const StreamArgs, const Op);

constexpr int kRowsplitMaxCols = 2;

template <class Op, int V, int COLS, int RU>
stream_kernel_t<Op> pick_nt(int nt, int pipe, int rs)
{
    if constexpr (COLS <= kRowsplitMaxCols) {
        if (rs)
            return pipe ? stream_kernel<Op, V, COLS, RU, true, true, true>
                        : stream_kernel<Op, V, COLS, RU, true, false, true>;
    }
    if (pipe)
        return nt ? stream_kernel<Op, V, COLS, RU, true, true, false>
                  : stream_kernel<Op, V, COLS, RU, false, true, false>;
    return nt ? stream_kernel<Op, V, COLS, RU, true, false, false>
              : stream_kernel<Op, V, COLS, RU, false, false, false>;
}

template <class Op, int V, int COLS>
stream_kernel_t<Op> pick_ru(int ru, int nt, int pipe, int rs)
{
    switch (ru) {
    case 2: return pick_nt<Op, V, COLS, 2>(nt, pipe, rs);
    case 8: return pick_nt<Op, V, COLS, 8>(nt, pipe, rs);
    default: return pick_nt<Op, V, COLS, 4>(nt, pipe, rs);
    }
}

// `cols` must already be <= kRowsplitMaxCols when rs is set.
template <class Op, int V>
stream_kernel_t<Op> pick_cols(int cols, int ru, int nt, int pipe, int rs)
{
    switch (cols) {
    case 1: return pick_ru<Op, V, 1>(ru, nt, pipe, rs);
    case 2: return pick_ru<Op, V, 2>(ru, nt, pipe, rs);
    case 4: return pick_ru<Op, V, 4>(ru, nt, pipe, rs);
    default: return pick_ru<Op, V, 8>(ru, nt, pipe, rs);
    }
}

// ---------------------------------------------------------------------------------------
// Ring-order variant for the plain sum (Sec. 2.2, Share-Reduce).  In the ring, chunk c
// starts as client c's own sub-vector and every following client adds its own to what it
// received, so coordinate k of chunk c is ((g_c + g_{c+1}) + ...) + g_{c-1} (indices mod n)
// in the clients' precision, one fp32 rounding per step.  The start row therefore depends on
// the chunk a coordinate falls in.  The launch layout is that of the kernels above (aligned
// body of wave slots, edges one coordinate per thread, optionally results parked in LDS and
// written as one burst per block); a wave looks up the chunk of its run of slots, folds rows
// c .. n-1 and then 0 .. c-1, and falls back to one slot at a time, and inside a slot that a
// chunk boundary cuts to one coordinate at a time, where the run spans two chunks.
// ---------------------------------------------------------------------------------------
struct RingArgs {
    int64_t q, r;           // chunk c is [c*q + min(c, r), + q + (c < r)): the first r hold q + 1
    int32_t mean;           // 1: divide the sum by n once, in fp32 (Mean rule of Sec. 2.1)
    int32_t reserved;
};

struct RingSumOp {
    struct State { float acc; };
    // -0.0f is the exact identity of fp32 addition (0.0f would turn a sum of -0.0f into +0.0f)
    __device__ static __forceinline__ void init(State& s) { s.acc = -0.0f; }
    __device__ static __forceinline__ void add(State& s, float v) { s.acc += v; }
};

__device__ __forceinline__ int ring_chunk_of(int64_t k, const RingArgs& g)
{
    const int64_t head = g.r * (g.q + 1);       // coordinates held by the longer chunks
    return (int)(k < head ? k / (g.q + 1) : g.r + (k - head) / g.q);   // k >= head implies q >= 1
}

__device__ __forceinline__ float ring_result(float acc, int n, const RingArgs& g)
{
    return g.mean ? __fdiv_rn(acc, (float)n) : acc;
}

// One coordinate, rows in the ring order of its chunk.
__device__ __forceinline__ float ring_one(const float* __restrict__ updates, int64_t ld, int n,
                                          int64_t k, const RingArgs& g)
{
    const int c = ring_chunk_of(k, g);
    float acc = updates[(int64_t)c * ld + k];
    for (int i = c + 1; i < n; ++i)
        acc += updates[(int64_t)i * ld + k];
    for (int i = 0; i < c; ++i)
        acc += updates[(int64_t)i * ld + k];
    return ring_result(acc, n, g);
}

// One wave folds all n rows in the ring order of chunk c (rows c, c+1, ..., n-1, 0, ..., c-1)
// for COLS adjacent slots from wave-uniform coordinate k0: the double-buffered batches of
// stream_fold, with the row of a batch entry looked up by its position in that sequence, so
// that the wrap from row n-1 to row 0 does not drain the loads in flight.
template <int V, int COLS, int RU>
__device__ __forceinline__ void ring_fold(const float* __restrict__ updates, int64_t ld, int n,
                                          int c, int64_t k0, int lane,
                                          RingSumOp::State (&st)[COLS][V])
{
    typedef typename Vec<V>::type VT;
    const float* col = updates + k0;            // wave-uniform
    const uint32_t loff = (uint32_t)lane * V;
    int j = 0;                                  // position in the sequence of the next row to request
    auto row_of = [&](int pos) {
        const int r = c + pos;
        return col + (int64_t)(r >= n ? r - n : r) * ld;
    };
    auto load_batch = [&](VT (&x)[RU][COLS]) {
#pragma unroll
        for (int r = 0; r < RU; ++r) {
            const float* row = row_of(j + r);
#pragma unroll
            for (int s = 0; s < COLS; ++s)
                x[r][s] = load_vec<V, true>(row + loff + s * (64 * V));
        }
        j += RU;
        __builtin_amdgcn_sched_barrier(0);
    };
    auto fold = [&](const VT (&x)[RU][COLS]) {
#pragma unroll
        for (int r = 0; r < RU; ++r)
#pragma unroll
            for (int s = 0; s < COLS; ++s)
#pragma unroll
                for (int e = 0; e < V; ++e)
                    RingSumOp::add(st[s][e], elem<V>(x[r][s], e));
    };
    if (n >= RU) {
        VT xa[RU][COLS], xb[RU][COLS];
        load_batch(xa);
        while (j + 2 * RU <= n) {
            load_batch(xb);
            fold(xa);
            load_batch(xa);
            fold(xb);
        }
        if (j + RU <= n) {
            load_batch(xb);
            fold(xa);
            fold(xb);
        } else {
            fold(xa);
        }
    }
    for (; j < n; ++j) {                        // the last n mod RU rows
        const float* row = row_of(j);
        VT x[COLS];
#pragma unroll
        for (int s = 0; s < COLS; ++s)
            x[s] = load_vec<V, true>(row + loff + s * (64 * V));
#pragma unroll
        for (int s = 0; s < COLS; ++s)
#pragma unroll
            for (int e = 0; e < V; ++e)
                RingSumOp::add(st[s][e], elem<V>(x[s], e));
    }
}

// COLS slots from wave-uniform coordinate k0; emit(slot, values) receives the lane's V results
// of slot `slot` (0 .. COLS-1) of the run.
template <int V, int COLS, int RU, class Emit>
__device__ __forceinline__ void ring_slots(const float* __restrict__ updates, int64_t ld, int n,
                                           const RingArgs& g, int64_t k0, int lane, Emit emit)
{
    constexpr int64_t kSlot = 64 * V;
    const int c_first = ring_chunk_of(k0, g);                               // wave-uniform
    const int c_last = ring_chunk_of(k0 + COLS * kSlot - 1, g);
    if (c_first == c_last) {
        RingSumOp::State st[COLS][V];
#pragma unroll
        for (int s = 0; s < COLS; ++s)
#pragma unroll
            for (int e = 0; e < V; ++e)
                RingSumOp::init(st[s][e]);
        ring_fold<V, COLS, RU>(updates, ld, n, c_first, k0, lane, st);
#pragma unroll
        for (int s = 0; s < COLS; ++s) {
            float v[V];
#pragma unroll
            for (int e = 0; e < V; ++e)
                v[e] = ring_result(st[s][e].acc, n, g);
            emit(s, v);
        }
        return;
    }
    if constexpr (COLS > 1) {
        for (int s = 0; s < COLS; ++s)              // a chunk boundary inside the run: slot by slot
            ring_slots<V, 1, RU>(updates, ld, n, g, k0 + s * kSlot, lane,
                                 [&](int, const float (&v)[V]) { emit(s, v); });
    } else {
        float v[V];                                 // a chunk boundary inside the slot
#pragma unroll
        for (int e = 0; e < V; ++e)
            v[e] = ring_one(updates, ld, n, k0 + (int64_t)lane * V + e, g);
        emit(0, v);
    }
}

template <int V, int COLS, int RU, bool STAGED>
__global__ void __launch_bounds__(kBlock)
ring_sum_kernel(const float* __restrict__ updates, const StreamArgs a, const RingArgs g,
                float* __restrict__ out, const int stage_tiles)
{
    typedef typename Vec<V>::type VT;
    if ((int64_t)blockIdx.x < a.edge_blocks) {
        const int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x;
        const int64_t head = a.lo_a - a.lo;
        const int64_t k = (e < head) ? a.lo + e : a.hi_a + (e - head);
        if (k < a.hi)
            out[k] = ring_one(updates, a.ld, a.n, k, g);
        return;
    }
    const int64_t b = (int64_t)blockIdx.x - a.edge_blocks;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    constexpr int64_t kSlot = 64 * V;
    const int64_t slots = (a.hi_a - a.lo_a) / kSlot;
    if constexpr (!STAGED) {
        const int64_t s0 = (b * kWaves + wave) * COLS;
        if (s0 >= slots)
            return;
        const int64_t k0 = a.lo_a + s0 * kSlot;
        auto store = [&](int64_t kbase) {
            return [=](int s, const float (&v)[V]) {
                VT o;
#pragma unroll
                for (int e = 0; e < V; ++e)
                    set_elem<V>(o, e, v[e]);
                store_vec<true>(reinterpret_cast<VT*>(out + kbase + s * kSlot + (int64_t)lane * V), o);
            };
        };
        if (s0 + COLS <= slots) {
            ring_slots<V, COLS, RU>(updates, a.ld, a.n, g, k0, lane, store(k0));
        } else {
            for (int64_t s = s0; s < slots; ++s)       // fewer than COLS slots left at the very end
                ring_slots<V, 1, RU>(updates, a.ld, a.n, g, a.lo_a + s * kSlot, lane,
                                     store(a.lo_a + s * kSlot));
        }
    } else {
        extern __shared__ unsigned char lds_raw[];
        float* stage = reinterpret_cast<float*>(lds_raw);
        constexpr int64_t kTileSlots = (int64_t)kWaves * COLS;
        const int64_t slot0 = b * stage_tiles * kTileSlots;         // first slot of this block's group
        auto park = [&](int64_t sbase) {
            return [=](int s, const float (&v)[V]) {
#pragma unroll
                for (int e = 0; e < V; ++e)
                    stage[(sbase - slot0 + s) * kSlot + lane * V + e] = v[e];
            };
        };
        for (int t = 0; t < stage_tiles; ++t) {
            const int64_t s0 = slot0 + (t * kTileSlots + (int64_t)wave * COLS);
            if (s0 >= slots)
                break;                                              // wave-uniform; the barrier is below
            if (s0 + COLS <= slots) {
                ring_slots<V, COLS, RU>(updates, a.ld, a.n, g, a.lo_a + s0 * kSlot, lane, park(s0));
            } else {
                for (int64_t s = s0; s < slots; ++s)
                    ring_slots<V, 1, RU>(updates, a.ld, a.n, g, a.lo_a + s * kSlot, lane, park(s));
            }
        }
        __syncthreads();
        const int64_t base = a.lo_a + slot0 * kSlot;
        int64_t valid = (int64_t)stage_tiles * kTileSlots * kSlot;
        if (valid > a.hi_a - base)
            valid = a.hi_a - base;                                  // a multiple of kSlot, hence of 4
        for (int64_t i = (int64_t)threadIdx.x * 4; i < valid; i += kBlock * 4)
            __builtin_nontemporal_store(*reinterpret_cast<const f32x4*>(stage + i),
                                        reinterpret_cast<f32x4*>(out + base + i));
    }
}

using ring_sum_kernel_t = void (*)(const float*, const StreamArgs, const RingArgs, float*, int);

// Tile shapes of the ring-order kernel: the two large-range shapes (also staged) and one load
// per row for short ranges.
template <int V>
ring_sum_kernel_t pick_ring(int cols, bool staged)
{
    if (cols >= kStageColsWide)
        return staged ? ring_sum_kernel<V, kStageColsWide, kStageUnroll, true>
                      : ring_sum_kernel<V, kStageColsWide, kStageUnroll, false>;
    if (cols >= kStageColsNarrow)
        return staged ? ring_sum_kernel<V, kStageColsNarrow, kStageUnroll, true>
                      : ring_sum_kernel<V, kStageColsNarrow, kStageUnroll, false>;
    return ring_sum_kernel<V, 1, 4, false>;
}

}  // namespace brace_dev
