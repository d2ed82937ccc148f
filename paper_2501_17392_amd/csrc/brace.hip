// BRACE robust chunk aggregation for MI355X (gfx950): kernels and C ABI.
//
// What is computed (Sec. 3, Phases I-IV; Eq. (1)): for every coordinate k of a
// ring chunk, S[k] = sum over the n clients of sign(g_i[k]), and the result is
// +1 if S[k] > lambda, else -1, written at k's place in the global update.
//
// Shape of the work: a pure stream.  The n x d fp32 matrix is read exactly once
// (4*n bytes per coordinate) and 4 bytes per coordinate are written, so the
// bound is HBM bandwidth.  There is no reuse, no contraction, no cross-lane
// traffic in the main loop: each lane owns V consecutive coordinates per load
// slot and keeps two small integer counters per coordinate (#positive,
// #negative) in registers while it walks down the n client rows.
//
// Launch layout.  The range [lo, hi) of a call is split in
//   body  [lo_a, hi_a): whole "wave slots" of 64*V coordinates, aligned to
//         64*V coordinates from coordinate 0, handled with V-dword loads and
//         no bounds checks;
//   edges [lo, lo_a) and [hi_a, hi): at most 2*(64*V-1) coordinates, one
//         thread per coordinate with dword loads, run by extra blocks at the
//         end of the same grid.
// A wave owns COLS adjacent slots, i.e. a contiguous run of 64*V*COLS floats
// in every row; the row pointer is wave-uniform so row stepping is scalar
// arithmetic and each load is "scalar base + lane offset".

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <cstring>

#include "brace.h"

namespace {

constexpr int kBlock = 256;                 // 4 waves of 64
constexpr int kWaves = kBlock / 64;
constexpr int kXcds = 8;                    // MI355X: 8 XCDs, blocks are dealt round-robin

thread_local char g_err[256] = "";

int fail(int code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

brace_tuning_t default_tuning()
{
    brace_tuning_t t;
    t.struct_size = sizeof(brace_tuning_t);
    t.vec = 0;
    t.cols = 2;
    t.unroll = 8;
    t.nontemporal = 1;
    t.xcd_swizzle = 0;
    return t;
}

brace_tuning_t g_tuning = default_tuning();

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
    int64_t body_blocks;    // blocks that run the body; the rest run the edges
};

// Sign-sum from the two counters (Phase I + II); the consensus map (Phase III) is
// "sum >= thresh".
__device__ __forceinline__ int sign_sum(int pos, int neg, int n, int zero_sign)
{
    return pos - neg + zero_sign * (n - pos - neg);
}

// One wave: COLS adjacent slots starting at wave-uniform coordinate k0.
template <int V, int COLS, int RU, bool NT>
__device__ __forceinline__ void vote_slots(const float* __restrict__ updates,
                                           float* __restrict__ out, uint32_t* __restrict__ bits,
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

    int i = 0;
    for (; i + RU <= n; i += RU) {
        VT x[RU][COLS];
#pragma unroll
        for (int r = 0; r < RU; ++r)
#pragma unroll
            for (int c = 0; c < COLS; ++c)
                x[r][c] = load_vec<V, NT>(row + (int64_t)r * ld + loff + c * (64 * V));
        // keep all RU*COLS loads in flight before the first compare waits on one
        __builtin_amdgcn_sched_barrier(0);
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
        row += (int64_t)RU * ld;
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
            *reinterpret_cast<VT*>(out + k) = o;
        }
        if (sums) {
            typename IVec<V>::type sv;
#pragma unroll
            for (int e = 0; e < V; ++e) {
                if constexpr (V == 1) sv = (short)s[e]; else sv[e] = (short)s[e];
            }
            *reinterpret_cast<typename IVec<V>::type*>(sums + k) = sv;
        }
        if (bits) {
            // 32/V lanes share one 32-bit word; OR them together, the first lane stores.
            constexpr int L = 32 / V;
            uint32_t w = mybits << (V * (lane & (L - 1)));
#pragma unroll
            for (int m = 1; m < L; m <<= 1)
                w |= (uint32_t)__shfl_xor((int)w, m, 64);
            if ((lane & (L - 1)) == 0)
                bits[k >> 5] = w;
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
    for (int i = 0; i < a.n; ++i) {
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

template <int V, int COLS, int RU, bool NT>
__global__ void __launch_bounds__(kBlock)
brace_vote_kernel(const float* __restrict__ updates, float* __restrict__ out,
                  uint32_t* __restrict__ bits, int16_t* __restrict__ sums, const VoteArgs a)
{
    const int64_t b = blockIdx.x;
    if (b >= a.body_blocks) {
        vote_edges(updates, out, bits, sums, a, (b - a.body_blocks) * kBlock + threadIdx.x);
        return;
    }
    // Blocks are dealt to the 8 XCDs round-robin.  With the swizzle, XCD x works on the
    // x-th eighth of the tiles, so neighbouring tiles (which share boundary cache lines
    // when rows are not line-aligned) meet in the same L2.
    int64_t tile = b;
    if (a.swizzle) {
        const int64_t per = a.body_blocks / kXcds;     // body_blocks is a multiple of 8 here
        tile = (b % kXcds) * per + b / kXcds;
    }
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    constexpr int64_t kSlot = 64 * V;
    const int64_t slots = (a.hi_a - a.lo_a) / kSlot;
    const int64_t s0 = (tile * kWaves + wave) * COLS;
    if (s0 >= slots)
        return;
    const int64_t k0 = a.lo_a + s0 * kSlot;
    if (s0 + COLS <= slots) {
        vote_slots<V, COLS, RU, NT>(updates, out, bits, sums, a.ld, a.n, a.thresh, a.zero_sign,
                                    k0, lane);
    } else {
        for (int64_t s = s0; s < slots; ++s)       // fewer than COLS slots left at the very end
            vote_slots<V, 1, RU, NT>(updates, out, bits, sums, a.ld, a.n, a.thresh, a.zero_sign,
                                     a.lo_a + s * kSlot, lane);
    }
}

typedef void (*vote_kernel_t)(const float*, float*, uint32_t*, int16_t*, const VoteArgs);

template <int V, int COLS, int RU>
vote_kernel_t pick_nt(int nt)
{
    return nt ? brace_vote_kernel<V, COLS, RU, true> : brace_vote_kernel<V, COLS, RU, false>;
}

template <int V, int COLS>
vote_kernel_t pick_ru(int ru, int nt)
{
    switch (ru) {
    case 2: return pick_nt<V, COLS, 2>(nt);
    case 4: return pick_nt<V, COLS, 4>(nt);
    case 16: return pick_nt<V, COLS, 16>(nt);
    default: return pick_nt<V, COLS, 8>(nt);
    }
}

template <int V>
vote_kernel_t pick_cols(int cols, int ru, int nt)
{
    switch (cols) {
    case 1: return pick_ru<V, 1>(ru, nt);
    case 4: return pick_ru<V, 4>(ru, nt);
    default: return pick_ru<V, 2>(ru, nt);
    }
}

vote_kernel_t pick_kernel(int v, int cols, int ru, int nt)
{
    switch (v) {
    case 4: return pick_cols<4>(cols, ru, nt);
    case 2: return pick_cols<2>(cols, ru, nt);
    default: return pick_cols<1>(cols, ru, nt);
    }
}

bool aligned_to(const void* p, uintptr_t bytes)
{
    return (reinterpret_cast<uintptr_t>(p) & (bytes - 1)) == 0;
}

int validate(const float* updates, int64_t n, int64_t d, int64_t f, const brace_params_t* p,
             const float* out, int64_t* ld_out, int* thresh_out)
{
    if (!p)
        return fail(BRACE_EINVAL, "params is NULL");
    if (p->struct_size != sizeof(brace_params_t))
        return fail(BRACE_EINVAL, "params->struct_size is %u, expected %zu", p->struct_size,
                    sizeof(brace_params_t));
    if (n < 1)
        return fail(BRACE_EINVAL, "n must be >= 1 (got %lld)", (long long)n);
    if (n > BRACE_MAX_CLIENTS)
        return fail(BRACE_ERANGE, "n = %lld exceeds BRACE_MAX_CLIENTS", (long long)n);
    if (d < 0)
        return fail(BRACE_EINVAL, "d must be >= 0 (got %lld)", (long long)d);
    if (f < 0 || f > n)
        return fail(BRACE_EINVAL, "f must be in [0, n] (got %lld)", (long long)f);
    if (!std::isfinite(p->lambda))
        return fail(BRACE_EINVAL, "lambda must be finite");
    if (p->zero_sign < -1 || p->zero_sign > 1)
        return fail(BRACE_EINVAL, "zero_sign must be -1, 0 or +1");
    if (p->reserved0 != 0)
        return fail(BRACE_EINVAL, "reserved0 must be 0");
    if (p->ld != 0 && p->ld < d)
        return fail(BRACE_EINVAL, "ld = %lld is smaller than d = %lld", (long long)p->ld,
                    (long long)d);
    *ld_out = p->ld ? p->ld : d;
    *thresh_out = 0;
    if (d == 0)
        return BRACE_OK;       // nothing is read or written, so empty buffers may be NULL
    if (!updates)
        return fail(BRACE_EINVAL, "updates_dev is NULL");
    if (!out && !p->out_bits_dev && !p->sums_dev)
        return fail(BRACE_EINVAL, "no output: out_dev, out_bits_dev and sums_dev are all NULL");
    if (!aligned_to(updates, 4) || (out && !aligned_to(out, 4)))
        return fail(BRACE_EINVAL, "updates_dev and out_dev must be 4-byte aligned");
    if (p->out_bits_dev && !aligned_to(p->out_bits_dev, 4))
        return fail(BRACE_EINVAL, "out_bits_dev must be 4-byte aligned");
    if (p->sums_dev && !aligned_to(p->sums_dev, 2))
        return fail(BRACE_EINVAL, "sums_dev must be 2-byte aligned");
    const int64_t ld = p->ld ? p->ld : d;
    if (out && d > 0) {
        const float* in_end = updates + (n - 1) * ld + d;
        if (out < in_end && updates < out + d)
            return fail(BRACE_EINVAL, "out_dev overlaps updates_dev");
    }
    *ld_out = ld;
    const double fl = std::floor((double)p->lambda);
    int t;
    if (fl >= (double)n)
        t = (int)n + 1;            // never reached: all -1
    else if (fl < -(double)n - 1.0)
        t = -(int)n;               // always reached: all +1
    else
        t = (int)fl + 1;
    *thresh_out = t;
    return BRACE_OK;
}

int launch_range(const float* updates, int64_t n, int64_t d, int64_t ld, int thresh,
                 const brace_params_t* p, float* out, int64_t lo, int64_t hi, hipStream_t stream)
{
    if (hi <= lo)
        return BRACE_OK;
    const brace_tuning_t t = g_tuning;

    // Widest load every row, every slot and every vector store can use.
    int v = 4;
    while (v > 1) {
        const uintptr_t bytes = 4u * v;
        const bool ok = aligned_to(updates, bytes) && (ld % v == 0 || n == 1) &&
                        (!out || aligned_to(out, bytes)) &&
                        (!p->sums_dev || aligned_to(p->sums_dev, 2u * v));
        if (ok)
            break;
        v >>= 1;
    }
    if (t.vec == 1 || t.vec == 2 || t.vec == 4)
        v = v < t.vec ? v : t.vec;
    const int cols = (t.cols == 1 || t.cols == 4) ? t.cols : 2;

    VoteArgs a;
    a.ld = ld;
    a.n = (int32_t)n;
    a.thresh = thresh;
    a.zero_sign = p->zero_sign;
    a.swizzle = t.xcd_swizzle ? 1 : 0;
    a.lo = lo;
    a.hi = hi;
    a.d = d;
    uint32_t* bits = static_cast<uint32_t*>(p->out_bits_dev);

    const int64_t slot = 64 * (int64_t)v;
    int64_t lo_a = (lo + slot - 1) / slot * slot;
    int64_t hi_a = hi / slot * slot;
    if (lo_a >= hi_a)
        lo_a = hi_a = lo;          // no body: everything is "tail" edge
    a.lo_a = lo_a;
    a.hi_a = hi_a;

    const int64_t slots = (hi_a - lo_a) / slot;
    const int64_t per_block = (int64_t)kWaves * cols;
    int64_t body_blocks = (slots + per_block - 1) / per_block;
    if (a.swizzle)                 // the swizzled map needs a multiple of 8 tiles' worth of ids
        body_blocks = (body_blocks + kXcds - 1) / kXcds * kXcds;
    a.body_blocks = body_blocks;

    int64_t edge = (lo_a - lo) + (hi - hi_a);
    if (bits && hi == d)
        edge += ((d + 31) & ~(int64_t)31) - d;
    const int64_t edge_blocks = (edge + kBlock - 1) / kBlock;
    const int64_t grid = body_blocks + edge_blocks;
    if (grid <= 0)
        return BRACE_OK;
    if (grid > 0x7fffffffLL)
        return fail(BRACE_ERANGE, "range needs %lld blocks, more than one launch can hold",
                    (long long)grid);

    vote_kernel_t k = pick_kernel(v, cols, t.unroll, t.nontemporal);
    hipLaunchKernelGGL(k, dim3((unsigned)grid), dim3(kBlock), 0, stream, updates, out, bits, p->sums_dev, a);
    const hipError_t err = hipGetLastError();
    if (err != hipSuccess)
        return fail(BRACE_EHIP, "kernel launch failed: %s", hipGetErrorString(err));
    return BRACE_OK;
}

}  // namespace

extern "C" {

void brace_params_init(brace_params_t* params)
{
    if (!params)
        return;
    std::memset(params, 0, sizeof(*params));
    params->struct_size = sizeof(brace_params_t);
    params->lambda = 5.0f;
}

int brace_chunk_range(int64_t n, int64_t d, int64_t chunk, int64_t* lo, int64_t* hi)
{
    if (!lo || !hi)
        return fail(BRACE_EINVAL, "lo/hi is NULL");
    if (n < 1 || d < 0)
        return fail(BRACE_EINVAL, "need n >= 1 and d >= 0");
    if (chunk < 0 || chunk >= n)
        return fail(BRACE_ERANGE, "chunk %lld outside [0, %lld)", (long long)chunk, (long long)n);
    const int64_t q = d / n, r = d % n;
    const int64_t start = chunk * q + (chunk < r ? chunk : r);
    *lo = start;
    *hi = start + q + (chunk < r ? 1 : 0);
    return BRACE_OK;
}

int brace_chunk_owner(int64_t n, int64_t chunk, int64_t* owner_client)
{
    if (!owner_client)
        return fail(BRACE_EINVAL, "owner_client is NULL");
    if (n < 1)
        return fail(BRACE_EINVAL, "need n >= 1");
    if (chunk < 0 || chunk >= n)
        return fail(BRACE_ERANGE, "chunk %lld outside [0, %lld)", (long long)chunk, (long long)n);
    *owner_client = (chunk + n - 1) % n;
    return BRACE_OK;
}

int brace_aggregate(const float* updates_dev, int64_t n, int64_t d, int64_t f,
                    const brace_params_t* params, float* out_dev, void* hip_stream)
{
    int64_t ld;
    int thresh;
    const int rc = validate(updates_dev, n, d, f, params, out_dev, &ld, &thresh);
    if (rc != BRACE_OK)
        return rc;
    // Eq. (1) is per coordinate, so the n chunk aggregations are one pass over [0, d):
    // chunk c's result lands at [lo_c, hi_c) and the chunks tile [0, d).
    return launch_range(updates_dev, n, d, ld, thresh, params, out_dev, 0, d,
                        static_cast<hipStream_t>(hip_stream));
}

int brace_aggregate_chunk(const float* updates_dev, int64_t n, int64_t d, int64_t f,
                          int64_t chunk, const brace_params_t* params, float* out_dev,
                          void* hip_stream)
{
    int64_t ld;
    int thresh;
    int rc = validate(updates_dev, n, d, f, params, out_dev, &ld, &thresh);
    if (rc != BRACE_OK)
        return rc;
    int64_t lo, hi;
    rc = brace_chunk_range(n, d, chunk, &lo, &hi);
    if (rc != BRACE_OK)
        return rc;
    return launch_range(updates_dev, n, d, ld, thresh, params, out_dev, lo, hi,
                        static_cast<hipStream_t>(hip_stream));
}

const char* brace_last_error(void)
{
    return g_err;
}

int brace_set_tuning(const brace_tuning_t* tuning)
{
    if (!tuning) {
        g_tuning = default_tuning();
        return BRACE_OK;
    }
    if (tuning->struct_size != sizeof(brace_tuning_t))
        return fail(BRACE_EINVAL, "tuning->struct_size is %u, expected %zu", tuning->struct_size,
                    sizeof(brace_tuning_t));
    const int v = tuning->vec, c = tuning->cols, u = tuning->unroll;
    if (!(v == 0 || v == 1 || v == 2 || v == 4) || !(c == 1 || c == 2 || c == 4) ||
        !(u == 2 || u == 4 || u == 8 || u == 16))
        return fail(BRACE_EINVAL, "tuning: vec in {0,1,2,4}, cols in {1,2,4}, unroll in {2,4,8,16}");
    g_tuning = *tuning;
    return BRACE_OK;
}

int brace_get_tuning(brace_tuning_t* tuning)
{
    if (!tuning)
        return fail(BRACE_EINVAL, "tuning is NULL");
    *tuning = g_tuning;
    return BRACE_OK;
}

}  // extern "C"
