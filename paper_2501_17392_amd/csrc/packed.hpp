// Quantise-once form of BRACE for gfx950.
//
// Sec. 3 Phase I (the sign quantisation) kept as data: every client's update becomes two
// bit planes, "x > 0" and "x < 0" (two planes because +-0 and NaN abstain), 2 bits per
// coordinate instead of 32.  Phases II-IV then run on the planes: the per-coordinate counts
// of the n clients are kept bit-sliced (one register per counter bit, 32 coordinates per
// register), so folding one client's word costs a handful of logic ops for 32 coordinates,
// and the consensus map of Eq. (1) is evaluated on the slices as well.
//
// Layout of the packed matrix: row i (client i) at signs + i*ld_words; word pair j of a row
// is (positive bits, negative bits) of coordinates 32j .. 32j+31, bit b <-> coordinate 32j+b.
// Rows hold an even number of pairs (16-byte granularity); padding bits are zero.

#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "ops.hpp"

namespace brace_dev {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kQuantSpan = 4096;            // coordinates per wave task: 64 loads of 64 lanes

// Phase I for one span: a wave turns 4096 consecutive coordinates of one client (from src,
// coordinate k0 of a row of d) into 128 word pairs.  A dword load per lane covers 64
// coordinates, and the two compares of that load already are the two 64-bit plane masks (one
// bit per lane, held in scalar registers); the masks of load r are written into lane r of
// the result, so every lane ends with 16 bytes: (pos, neg) of coordinates k0 + 64 r .. + 31
// and (pos, neg) of the next 32.
__device__ __forceinline__ u32x4 quantize_span(const float* __restrict__ src, int64_t k0, int64_t d,
                                               int lane)
{
    const bool full = k0 + kQuantSpan <= d;
    uint32_t o0 = 0, o1 = 0, o2 = 0, o3 = 0;
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        float x[16];
        if (full) {
#pragma unroll
            for (int u = 0; u < 16; ++u)
                x[u] = __builtin_nontemporal_load(src + (16 * b + u) * 64 + lane);
        } else {
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const int64_t k = k0 + (16 * b + u) * 64 + lane;
                x[u] = (k < d) ? src[(16 * b + u) * 64 + lane] : 0.0f;
            }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const unsigned long long mp = __ballot(x[u] > 0.0f);
            const unsigned long long mn = __ballot(x[u] < 0.0f);
            if (lane == 16 * b + u) {
                o0 = (uint32_t)mp;
                o1 = (uint32_t)mn;
                o2 = (uint32_t)(mp >> 32);
                o3 = (uint32_t)(mn >> 32);
            }
        }
    }
    u32x4 o;
    o[0] = o0;
    o[1] = o1;
    o[2] = o2;
    o[3] = o3;
    return o;
}

// Phase I for whole rows, one span per wave, one 1 KiB store per span.
__global__ void __launch_bounds__(kBlock)
brace_quantize_kernel(const float* __restrict__ updates, int64_t ld, int64_t d,
                      uint32_t* __restrict__ signs, int64_t ld_words, int64_t spans_per_row,
                      int64_t tasks)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int64_t task = (int64_t)blockIdx.x * kWaves + wave;
    if (task >= tasks)
        return;
    const int64_t row = task / spans_per_row;
    const int64_t k0 = (task % spans_per_row) * kQuantSpan;
    const u32x4 o = quantize_span(updates + row * ld + k0, k0, d, lane);
    const int64_t pair = k0 / 32 + 2 * lane;            // first of this lane's two word pairs
    const int64_t pairs = (d + 31) / 32 + (((d + 31) / 32) & 1);   // per row, padded to even
    if (pair < pairs) {
        // streaming store: 11 % faster than a plain store at n = 100, d = 25 M
        __builtin_nontemporal_store(o, reinterpret_cast<u32x4*>(signs + row * ld_words + 2 * pair));
    }
}

constexpr int kQuantBlock = 1024;           // 16 waves: enough loads in flight with one block per CU
constexpr int kQuantWaves = kQuantBlock / 64;
constexpr int kQuantGroup = 128;            // spans per block: 128 KiB of planes, one burst
constexpr int kQuantWideGroup = 144;        // KiB per burst of the 4-dword form (a multiple of 16)
constexpr size_t kQuantWideBytes = (size_t)kQuantWideGroup * 1024;

// The same for long rows, with the stores gathered: a block owns 128 adjacent spans of one
// row; its 16 waves take them 16 at a time and park the planes in LDS, and the block then
// writes its 128 KiB as one contiguous burst.  Measured at n = 100, d = 25 M on one device:
// 1.85 ms with a store per span, 1.72 ms with the bursts, 1.40 ms for the reads alone.
__global__ void __launch_bounds__(kQuantBlock)
brace_quantize_staged_kernel(const float* __restrict__ updates, int64_t ld, int64_t d,
                             uint32_t* __restrict__ signs, int64_t ld_words, int64_t groups_per_row)
{
    extern __shared__ unsigned char lds_raw[];
    u32x4* stage = reinterpret_cast<u32x4*>(lds_raw);           // kQuantGroup x 64 entries
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int64_t row = (int64_t)blockIdx.x / groups_per_row;
    const int64_t span0 = ((int64_t)blockIdx.x % groups_per_row) * kQuantGroup;
    const int64_t spans = (d + kQuantSpan - 1) / kQuantSpan;    // per row
    const float* rowp = updates + row * ld;
    for (int it = 0; it < kQuantGroup / kQuantWaves; ++it) {
        const int local = it * kQuantWaves + wave;
        const int64_t span = span0 + local;
        if (span >= spans)
            break;                                              // wave-uniform; barrier is below
        const int64_t k0 = span * kQuantSpan;
        // lane's two word pairs: coordinates k0 + 64 * lane ..
        stage[local * 64 + lane] = quantize_span(rowp + k0, k0, d, lane);
    }
    __syncthreads();
    // Entry e of the group = word pairs 2e, 2e+1 counted from the group's first pair.
    const int64_t pairs = (d + 31) / 32 + (((d + 31) / 32) & 1);   // per row, padded to even
    const int64_t pair0 = span0 * (kQuantSpan / 32);
    u32x4* dst = reinterpret_cast<u32x4*>(signs + row * ld_words + 2 * pair0);
    int64_t entries = (pairs - pair0) / 2;
    if (entries > (int64_t)kQuantGroup * 64)
        entries = (int64_t)kQuantGroup * 64;
    for (int64_t e = threadIdx.x; e < entries; e += kQuantBlock)
        __builtin_nontemporal_store(stage[e], dst + e);
}

// Long, 16-byte aligned rows: the burst kernel with 4-dword loads.  A lane's load covers 4
// consecutive coordinates, its two compares per value give a nibble per plane, and three
// butterfly steps over 8 neighbouring lanes assemble the 32-bit words; the lane that leads each
// group of 8 writes the word (pair) straight into its final place in the block's LDS stage, so
// the burst at the end is a plain copy.  Half the vector instructions of the ballot form
// (7.5 against 16 lane operations per value) and 16 KiB in flight per wave.  Measured at n = 100, d = 25 M (both planes): 1.69 ms
// with bursts of 144 KiB, 1.72 ms with 128 KiB, against 1.77 ms for the ballot form with
// 128 KiB bursts and 1.40 ms for the reads alone.
// TWO: both planes (x > 0, x < 0), else the one-bit vote (up_if_not_negative as in vote_span).
// `group` spans per block (a multiple of kQuantWaves); LDS: group KiB (TWO) or group/2 KiB.
template <bool TWO>
__global__ void __launch_bounds__(kQuantBlock)
brace_quantize_wide_kernel(const float* __restrict__ updates, int64_t ld, int64_t d,
                           uint32_t* __restrict__ planes, int64_t ld_words, int64_t row_words,
                           int64_t groups_per_row, int group, int up_if_not_negative)
{
    extern __shared__ unsigned char lds_raw[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int64_t row = (int64_t)blockIdx.x / groups_per_row;
    const int64_t span0 = ((int64_t)blockIdx.x % groups_per_row) * group;
    const int64_t spans = (d + kQuantSpan - 1) / kQuantSpan;    // per row
    const float* rowp = updates + row * ld;
    const f32x4 pad = up_if_not_negative && !TWO ? (f32x4)(-1.0f) : (f32x4)(0.0f);   // votes -1 / abstains
    for (int it = 0; it < group / kQuantWaves; ++it) {
        const int local = it * kQuantWaves + wave;
        const int64_t span = span0 + local;
        if (span >= spans)
            break;                                              // wave-uniform; barrier is below
        const int64_t k0 = span * kQuantSpan;
        const f32x4* src = reinterpret_cast<const f32x4*>(rowp + k0);
        f32x4 x[16];
        if (k0 + kQuantSpan <= d) {
#pragma unroll
            for (int j = 0; j < 16; ++j)
                x[j] = __builtin_nontemporal_load(src + 64 * j + lane);
        } else {
#pragma unroll
            for (int j = 0; j < 16; ++j)                        // d is a multiple of 4 on this path
                x[j] = (k0 + 256 * j + 4 * lane < d) ? src[64 * j + lane] : pad;
        }
        __builtin_amdgcn_sched_barrier(0);
        const int shift = 4 * (lane & 7);
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            uint32_t p, m = 0;
            if (TWO || !up_if_not_negative)
                p = (x[j][0] > 0.f ? 1u : 0u) | (x[j][1] > 0.f ? 2u : 0u) | (x[j][2] > 0.f ? 4u : 0u) |
                    (x[j][3] > 0.f ? 8u : 0u);
            else
                p = (!(x[j][0] < 0.f) ? 1u : 0u) | (!(x[j][1] < 0.f) ? 2u : 0u) |
                    (!(x[j][2] < 0.f) ? 4u : 0u) | (!(x[j][3] < 0.f) ? 8u : 0u);
            p <<= shift;
            p |= (uint32_t)__shfl_xor((int)p, 1, 64);
            p |= (uint32_t)__shfl_xor((int)p, 2, 64);
            p |= (uint32_t)__shfl_xor((int)p, 4, 64);
            if (TWO) {
                m = (x[j][0] < 0.f ? 1u : 0u) | (x[j][1] < 0.f ? 2u : 0u) | (x[j][2] < 0.f ? 4u : 0u) |
                    (x[j][3] < 0.f ? 8u : 0u);
                m <<= shift;
                m |= (uint32_t)__shfl_xor((int)m, 1, 64);
                m |= (uint32_t)__shfl_xor((int)m, 2, 64);
                m |= (uint32_t)__shfl_xor((int)m, 4, 64);
            }
            if ((lane & 7) == 0) {                              // word 8 j + lane / 8 of the span
                const int word = local * 128 + 8 * j + (lane >> 3);
                if (TWO) {
                    u32x2 pr;
                    pr[0] = p;
                    pr[1] = m;
                    reinterpret_cast<u32x2*>(lds_raw)[word] = pr;
                } else {
                    reinterpret_cast<uint32_t*>(lds_raw)[word] = p;
                }
            }
        }
    }
    __syncthreads();
    // The stage now holds the rows' words from word0 on, in row order: copy what the row has.
    const int64_t word0 = span0 * (TWO ? 256 : 128);
    const u32x4* st4 = reinterpret_cast<const u32x4*>(lds_raw);
    u32x4* dst = reinterpret_cast<u32x4*>(planes + row * ld_words + word0);
    int64_t entries = (row_words - word0) / 4;                  // row_words is a multiple of 4
    const int64_t cap = (int64_t)group * (TWO ? 64 : 32);
    if (entries > cap)
        entries = cap;
    for (int64_t e = threadIdx.x; e < entries; e += kQuantBlock)
        __builtin_nontemporal_store(st4[e], dst + e);
}

// (h, l) <- a + b + c on 32 independent 1-bit lanes per component (carry-save adder):
// parity and majority, each one three-input bit operation on gfx950 (truth tables 0x96, 0xE8;
// both are symmetric in their inputs).
__device__ __forceinline__ void csa(u32x4& h, u32x4& l, const u32x4 a, const u32x4 b, const u32x4 c)
{
    u32x4 maj, par;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        par[e] = __builtin_amdgcn_bitop3_b32(a[e], b[e], c[e], 0x96);
        maj[e] = __builtin_amdgcn_bitop3_b32(a[e], b[e], c[e], 0xE8);
    }
    l = par;
    h = maj;
}

// Pins a wave-uniform pointer to scalar registers, so that loads through it take the
// "scalar base + 32-bit lane offset" form and need no per-lane 64-bit address registers.
template <class T>
__device__ __forceinline__ const T* scalar_ptr(const T* q)
{
    const uint64_t v = reinterpret_cast<uint64_t>(q);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return reinterpret_cast<const T*>(((uint64_t)hi << 32) | lo);
}

// Share-Reduce on packed rows, common to both packed forms: folds the n client rows of one
// 16-byte column per lane into bit-sliced counters, cnt[b] = bit b of the four running counts
// (one count per 32-bit component, 32 coordinates each).  Eight clients are folded at a time
// through a carry-save tree (ones -> twos -> fours -> eights), and only the "eights" word
// ripples into the higher counter bits.  `p` is the wave's first column in row 0 (wave-uniform:
// row stepping stays in scalar registers, every load is scalar base + lane offset); lanes
// with !ok lie past the end of the row and read nothing.  (Measured and dropped: requesting
// the next rows before folding the current ones, 16 rows per batch, two columns per lane.)
template <int B>
__device__ __forceinline__ void fold_packed_rows(const u32x4* __restrict__ p, int64_t ld4, int n,
                                                 uint32_t lane, bool ok, u32x4 (&cnt)[B])
{
#pragma unroll
    for (int b = 0; b < B; ++b)
        cnt[b] = (u32x4)(0u);
    int i = 0;
    for (; i + 8 <= n; i += 8) {
        u32x4 a[8];
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const u32x4* src = scalar_ptr(p + (int64_t)r * ld4) + lane;
            a[r] = ok ? __builtin_nontemporal_load(src) : (u32x4)(0u);
        }
        __builtin_amdgcn_sched_barrier(0);
        u32x4 twos_a, twos_b, fours_a, fours_b, eights;
        csa(twos_a, cnt[0], cnt[0], a[0], a[1]);
        csa(twos_b, cnt[0], cnt[0], a[2], a[3]);
        csa(fours_a, cnt[1], cnt[1], twos_a, twos_b);
        csa(twos_a, cnt[0], cnt[0], a[4], a[5]);
        csa(twos_b, cnt[0], cnt[0], a[6], a[7]);
        csa(fours_b, cnt[1], cnt[1], twos_a, twos_b);
        csa(eights, cnt[2], cnt[2], fours_a, fours_b);
        u32x4 carry = eights;
#pragma unroll
        for (int b = 3; b < B; ++b) {
            const u32x4 t = cnt[b] & carry;
            cnt[b] ^= carry;
            carry = t;
        }
        p += 8 * ld4;
    }
    for (; i < n; ++i) {
        u32x4 carry = ok ? scalar_ptr(p)[lane] : (u32x4)(0u);
#pragma unroll
        for (int b = 0; b < B; ++b) {
            const u32x4 t = cnt[b] & carry;
            cnt[b] ^= carry;
            carry = t;
        }
        p += ld4;
    }
}

// Bit set <=> X - Y - c >= 0, evaluated on the slices: x[b], y[b] are bit b of X and Y (32
// coordinates per word, X, Y < 2^B), c is wave-uniform with |c| < 2^(B+1).
template <int B>
__device__ __forceinline__ uint32_t sliced_not_below(const uint32_t (&x)[B], const uint32_t (&y)[B], int c)
{
    uint32_t diff[B];
    uint32_t borrow = 0;
#pragma unroll
    for (int b = 0; b < B; ++b) {
        const uint32_t u = x[b] ^ y[b];
        diff[b] = u ^ borrow;
        borrow = (~x[b] & y[b]) | (~u & borrow);
    }
    const uint32_t sign = borrow;               // all higher bits of X - Y
    uint32_t borrow2 = 0, top = 0;
#pragma unroll
    for (int b = 0; b < B + 2; ++b) {
        const uint32_t xv = (b < B) ? diff[b] : sign;
        const uint32_t yv = ((c >> b) & 1) ? ~0u : 0u;
        const uint32_t u = xv ^ yv;
        top = u ^ borrow2;
        borrow2 = (~xv & yv) | (~u & borrow2);
    }
    return ~top;
}

// Where the result word of coordinates [k, k + 32) goes: the linear bit array, or parked in
// the float output's own memory (see scratch_word).  Padding bits past d stay zero.
__device__ __forceinline__ void put_result_word(uint32_t* __restrict__ dst, int parked, int64_t k,
                                                int64_t d, uint32_t result)
{
    if (k >= d)
        return;
    if (d - k < 32)
        result &= (1u << (d - k)) - 1u;
    if (parked)
        dst[scratch_word(k)] = result;
    else
        dst[k >> 5] = result;
}

// Phases II-IV on the two planes.  A wave owns `seq` adjacent groups of 64 columns (1 KiB of
// every row each) and takes them one after the other; a lane owns one 16-byte column of the
// current group, i.e. two adjacent word pairs (64 coordinates): component 0/1 =
// positive/negative plane of the first pair, 2/3 of the second.  Walking two or three
// neighbouring groups per wave instead of one group per wave with three times the waves
// measured 4-5 % faster (n = 100, d = 25 M: 97 against 102 us; a linear read of the same
// bytes takes 89 us), groups spread across the row measured slower.
// The decision S >= thresh is taken on the slices as X - Y - c >= 0 with X = pos & mask_p,
// Y = neg & mask_n and the constant c chosen by the host for the zero_sign in force.
template <int B>
__global__ void __launch_bounds__(kBlock)
brace_vote_packed_kernel(const u32x4* __restrict__ signs, int64_t ld4, int n, int64_t cols4, int seq,
                         uint32_t mask_p, uint32_t mask_n, int c, uint32_t* __restrict__ dst,
                         int parked, int64_t d)
{
    const uint32_t lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int64_t first = ((int64_t)blockIdx.x * kWaves + wave) * seq;       // group index
    for (int q = 0; q < seq; ++q) {
        const int64_t col0 = (first + q) * 64;
        if (col0 >= cols4)
            return;                                                          // wave-uniform
        const int64_t col = col0 + lane;
        u32x4 cnt[B];
        fold_packed_rows<B>(signs + col0, ld4, n, lane, col < cols4, cnt);
        if (col >= cols4)
            continue;
        // Eq. (1) on the slices, for each of the lane's two word pairs.
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            uint32_t x[B], y[B];
#pragma unroll
            for (int b = 0; b < B; ++b) {
                x[b] = cnt[b][2 * h] & mask_p;
                y[b] = cnt[b][2 * h + 1] & mask_n;
            }
            put_result_word(dst, parked, (2 * col + h) * 32, d, sliced_not_below<B>(x, y, c));
        }
    }
}

// ---------------------------------------------------------------------------------------
// One-bit form: when every coordinate votes (zero_sign = +1 or -1) a client's quantised
// update is one bit per dimension, bit = 1 <=> the vote is +1, which is the wire format the
// cost analysis of Sec. 3 counts.  Row i at votes + i*ld_words, bit b of word j <->
// coordinate 32j + b, rows padded with zero bits to a multiple of 4 words.
// ---------------------------------------------------------------------------------------
// One span (4096 coordinates) of one client: the ballot of load r is the 64-bit mask of
// coordinates k0 + 64 r .. + 63 and ends in lane r, 8 bytes per lane, 512 bytes per span.
// up_if_not_negative: zero_sign = +1 (only x < 0 votes -1); else zero_sign = -1 (only x > 0
// votes +1).  Coordinates past d read as a -1 vote, i.e. a zero padding bit.
__device__ __forceinline__ u32x2 vote_span(const float* __restrict__ src, int64_t k0, int64_t d,
                                           int lane, bool up_if_not_negative)
{
    const bool full = k0 + kQuantSpan <= d;
    const float pad = up_if_not_negative ? -1.0f : 0.0f;
    uint32_t o0 = 0, o1 = 0;
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        float x[16];
        if (full) {
#pragma unroll
            for (int u = 0; u < 16; ++u)
                x[u] = __builtin_nontemporal_load(src + (16 * b + u) * 64 + lane);
        } else {
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const int64_t k = k0 + (16 * b + u) * 64 + lane;
                x[u] = (k < d) ? src[(16 * b + u) * 64 + lane] : pad;
            }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const unsigned long long m =
                up_if_not_negative ? __ballot(!(x[u] < 0.0f)) : __ballot(x[u] > 0.0f);
            if (lane == 16 * b + u) {
                o0 = (uint32_t)m;
                o1 = (uint32_t)(m >> 32);
            }
        }
    }
    u32x2 o;
    o[0] = o0;
    o[1] = o1;
    return o;
}

// One span per wave, one 512-byte store per span.
__global__ void __launch_bounds__(kBlock)
brace_quantize_1bit_kernel(const float* __restrict__ updates, int64_t ld, int64_t d,
                           uint32_t* __restrict__ votes, int64_t ld_words, int64_t row_words,
                           int64_t spans_per_row, int64_t tasks, int up_if_not_negative)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int64_t task = (int64_t)blockIdx.x * kWaves + wave;
    if (task >= tasks)
        return;
    const int64_t row = task / spans_per_row;
    const int64_t k0 = (task % spans_per_row) * kQuantSpan;
    const u32x2 o = vote_span(updates + row * ld + k0, k0, d, lane, up_if_not_negative != 0);
    const int64_t word = k0 / 32 + 2 * lane;            // first of this lane's two words
    if (word < row_words)                               // row_words is even
        __builtin_nontemporal_store(o, reinterpret_cast<u32x2*>(votes + row * ld_words + word));
}

constexpr int kVoteGroup = 256;             // spans per block of the burst variant: 128 KiB of votes

// Long rows: a block owns 256 adjacent spans of one row, parks their votes in LDS and writes
// one contiguous burst of 128 KiB.
__global__ void __launch_bounds__(kQuantBlock)
brace_quantize_1bit_staged_kernel(const float* __restrict__ updates, int64_t ld, int64_t d,
                                  uint32_t* __restrict__ votes, int64_t ld_words, int64_t row_words,
                                  int64_t groups_per_row, int up_if_not_negative)
{
    extern __shared__ unsigned char lds_raw[];
    u32x2* stage = reinterpret_cast<u32x2*>(lds_raw);           // kVoteGroup x 64 entries
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int64_t row = (int64_t)blockIdx.x / groups_per_row;
    const int64_t span0 = ((int64_t)blockIdx.x % groups_per_row) * kVoteGroup;
    const int64_t spans = (d + kQuantSpan - 1) / kQuantSpan;    // per row
    const float* rowp = updates + row * ld;
    for (int it = 0; it < kVoteGroup / kQuantWaves; ++it) {
        const int local = it * kQuantWaves + wave;
        const int64_t span = span0 + local;
        if (span >= spans)
            break;                                              // wave-uniform; barrier is below
        const int64_t k0 = span * kQuantSpan;
        stage[local * 64 + lane] = vote_span(rowp + k0, k0, d, lane, up_if_not_negative != 0);
    }
    __syncthreads();
    // Entry e of the group = words 4e .. 4e+3 counted from the group's first word.
    const int64_t word0 = span0 * (kQuantSpan / 32);
    const u32x4* st4 = reinterpret_cast<const u32x4*>(lds_raw);
    u32x4* dst = reinterpret_cast<u32x4*>(votes + row * ld_words + word0);
    int64_t entries = (row_words - word0) / 4;                  // row_words is a multiple of 4
    if (entries > (int64_t)kVoteGroup * 32)
        entries = (int64_t)kVoteGroup * 32;
    for (int64_t e = threadIdx.x; e < entries; e += kQuantBlock)
        __builtin_nontemporal_store(st4[e], dst + e);
}

// Phases II-IV on one-bit votes.  As above with 4 adjacent words (128 coordinates) per lane;
// cnt[b] is bit b of the running count P of +1 votes.  S = 2P - n, so S >= thresh <=>
// P - q >= 0 with q = ceil((n + thresh) / 2) from the host.
template <int B>
__global__ void __launch_bounds__(kBlock)
brace_vote_1bit_kernel(const u32x4* __restrict__ votes, int64_t ld4, int n, int64_t cols4, int seq,
                       int q_min, uint32_t* __restrict__ dst, int parked, int64_t d)
{
    const uint32_t lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int64_t first = ((int64_t)blockIdx.x * kWaves + wave) * seq;
    for (int q = 0; q < seq; ++q) {
        const int64_t col0 = (first + q) * 64;
        if (col0 >= cols4)
            return;                                                          // wave-uniform
        const int64_t col = col0 + lane;
        u32x4 cnt[B];
        fold_packed_rows<B>(votes + col0, ld4, n, lane, col < cols4, cnt);
        if (col >= cols4)
            continue;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            uint32_t x[B], y[B];
#pragma unroll
            for (int b = 0; b < B; ++b) {
                x[b] = cnt[b][e];
                y[b] = 0u;
            }
            put_result_word(dst, parked, (4 * col + e) * 32, d, sliced_not_below<B>(x, y, q_min));
        }
    }
}

}  // namespace brace_dev
