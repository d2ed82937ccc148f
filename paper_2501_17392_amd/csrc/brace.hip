// BRACE robust chunk aggregation for MI355X (gfx950): C ABI, host logic, and the small
// kernels (bit expansion, measurement aids).  The streaming skeleton lives in
// stream_kernel.hpp, the vote and sum operations in ops.hpp; they are instantiated per
// load width in vote_v{1,2,4}.hip and sum_v{1,2,4}.hip.

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <atomic>
#include <cstring>
#include <mutex>

#include "brace.h"
#include "brace_tuning.h"
#include "ops.hpp"
#include "packed.hpp"

namespace {

using namespace brace_dev;

// Writing the floats from a second kernel pays once the matrix range is well past the
// 256 MiB memory-side cache: below that, stores from inside the read stream cost nothing
// measurable and the second launch is pure overhead (n = 8, d = 8 M, 256 MB: 52 us in one
// kernel, 58 us split; n = 32, d = 4 M, 512 MB: 85 against 87 us); above it the split wins
// (n = 100, d = 2 M, 800 MB: 119 against 122 us; n = 100, d = 25 M: 1.44 against 1.51 ms).
constexpr int64_t kSplitMinBytes = (int64_t)512 << 20;
// With few clients the floats are a large share of the traffic and the second kernel has
// to write all of them on its own; LDS-staged bursts from the first kernel are cheaper
// (n = 8, d = 100 M: 582 us staged, 618 us split; equal at n = 16, split ahead from n = 24).
constexpr int64_t kStageBelowClients = 16;
constexpr int64_t kNarrowBelowClients = 48;

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
    t.cols = 0;
    t.unroll = 0;
    t.nontemporal = 1;
    t.pipeline = 1;
    t.split_writes = 0;
    t.rowsplit = 0;
    t.stage_writes = 0;
    return t;
}

constexpr int kMaxDevices = 64;            // per-device caches; devices beyond are queried every call

// Compute units of the current device (0 if it cannot be queried); cached per device.
int compute_units()
{
    static std::atomic<int> cached[kMaxDevices];   // zero-initialised: 0 = not known yet
    int dev = 0, cu = 0;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return 0;
    }
    if (dev >= 0 && dev < kMaxDevices) {
        const int known = cached[dev].load(std::memory_order_relaxed);
        if (known > 0)
            return known;
    }
    if (hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) {
        (void)hipGetLastError();
        return 0;
    }
    if (dev >= 0 && dev < kMaxDevices)
        cached[dev].store(cu, std::memory_order_relaxed);
    return cu;
}

brace_tuning_t g_tuning = default_tuning();
std::mutex g_tuning_guard;

brace_tuning_t current_tuning()
{
    const std::lock_guard<std::mutex> lock(g_tuning_guard);
    return g_tuning;
}

void store_tuning(const brace_tuning_t& t)
{
    const std::lock_guard<std::mutex> lock(g_tuning_guard);
    g_tuning = t;
}

// Second phase of a split call: one wave turns the 32 bit-words of a 1024-coordinate group
// into 1024 floats.  `words` is the linear bit array, or null when the words were parked in
// the first 128 bytes of the group's own 4 KiB of `out`; the wave reads all its words with
// one load before its first store, so overwriting them is safe.  The last group may be cut
// short at coordinate `hi`.
__global__ void __launch_bounds__(kBlock)
brace_expand_kernel(float* out, const uint32_t* words, int64_t lo_s, int64_t groups, int64_t hi)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int64_t g = (int64_t)blockIdx.x * kWaves + wave;
    if (g >= groups)
        return;
    const int64_t k0 = lo_s + g * kGroup;
    const int64_t valid = hi - k0 < kGroup ? hi - k0 : kGroup;      // wave-uniform
    const uint32_t* src = words ? words + (k0 >> 5) : reinterpret_cast<const uint32_t*>(out) + k0;
    const uint32_t w = ((lane & 31) < (valid + 31) / 32) ? src[lane & 31] : 0u;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t ww = (uint32_t)__shfl((int)w, 8 * j + (lane >> 3), 64);
        const uint32_t nib = ww >> (4 * (lane & 7));
        f32x4 o;
        o[0] = (nib & 1u) ? 1.0f : -1.0f;
        o[1] = (nib & 2u) ? 1.0f : -1.0f;
        o[2] = (nib & 4u) ? 1.0f : -1.0f;
        o[3] = (nib & 8u) ? 1.0f : -1.0f;
        const int64_t r = 256 * j + 4 * lane;                       // offset inside the group
        if (r + 4 <= valid) {
            __builtin_nontemporal_store(o, reinterpret_cast<f32x4*>(out + k0 + r));
        } else {
            for (int e = 0; e < 4; ++e)
                if (r + e < valid)
                    out[k0 + r + e] = o[e];
        }
    }
}

// Same walk over the bit-words, applied to the model instead: w <- w - eta * (+-1).
__global__ void __launch_bounds__(kBlock)
brace_apply_kernel(float* __restrict__ w, const uint32_t* __restrict__ words, float eta,
                   int64_t lo_s, int64_t groups)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int64_t g = (int64_t)blockIdx.x * kWaves + wave;
    if (g >= groups)
        return;
    const int64_t k0 = lo_s + g * kGroup;
    const uint32_t word = words[(k0 >> 5) + (lane & 31)];
    f32x4 v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
        v[j] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(w + k0 + 256 * j + 4 * lane));
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t ww = (uint32_t)__shfl((int)word, 8 * j + (lane >> 3), 64);
        const uint32_t nib = ww >> (4 * (lane & 7));
        v[j][0] -= (nib & 1u) ? eta : -eta;
        v[j][1] -= (nib & 2u) ? eta : -eta;
        v[j][2] -= (nib & 4u) ? eta : -eta;
        v[j][3] -= (nib & 8u) ? eta : -eta;
        __builtin_nontemporal_store(v[j], reinterpret_cast<f32x4*>(w + k0 + 256 * j + 4 * lane));
    }
}

// Coordinates outside whole, aligned groups: one thread each.  out and w may each be null.
__global__ void __launch_bounds__(kBlock)
brace_bits_tail_kernel(float* out, float* w, const uint32_t* __restrict__ words, float eta,
                       int64_t lo, int64_t hi)
{
    const int64_t k = lo + (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (k >= hi)
        return;
    const bool up = (words[k >> 5] >> (k & 31)) & 1u;
    if (out)
        out[k] = up ? 1.0f : -1.0f;
    if (w)
        w[k] = w[k] - (up ? eta : -eta);
}

// Packed vote for the coordinates of a range that lie outside whole 1024-coordinate groups:
// one thread per coordinate reads its bit of every client's two planes and applies Eq. (1)
// to the integer sum.  Bits are merged atomically (a word can be shared with a neighbouring
// chunk's call); [hi, hi_ext) are padding bits of the last word, cleared.
__global__ void __launch_bounds__(kBlock)
brace_packed_edge_kernel(const uint32_t* __restrict__ signs, int64_t ld_words, int n, int thresh,
                         int zero_sign, float* out, uint32_t* bits, int64_t lo, int64_t lo_a,
                         int64_t hi_a, int64_t hi, int64_t hi_ext)
{
    const int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    const int64_t head = lo_a - lo;
    const int64_t k = (e < head) ? lo + e : hi_a + (e - head);
    if (k >= hi_ext)
        return;
    const uint32_t bit = 1u << (k & 31);
    if (k >= hi) {
        atomicAnd(&bits[k >> 5], ~bit);
        return;
    }
    const uint32_t* pair = signs + 2 * (k >> 5);
    int pos = 0, neg = 0;
    for (int i = 0; i < n; ++i) {
        pos += (pair[0] & bit) ? 1 : 0;
        neg += (pair[1] & bit) ? 1 : 0;
        pair += ld_words;
    }
    const bool up = pos - neg + zero_sign * (n - pos - neg) >= thresh;
    if (out)
        out[k] = up ? 1.0f : -1.0f;
    if (bits) {
        if (up)
            atomicOr(&bits[k >> 5], bit);
        else
            atomicAnd(&bits[k >> 5], ~bit);
    }
}

// Sec. 3 Phase III on partial sign-sums: S[k] = sum_j parts[j][k] over the g partial sums an
// owner has received, then Eq. (1).  One thread per 8 consecutive coordinates: a 16-byte load
// per part, two 16-byte float stores and one byte of packed bits.
typedef short i16x8 __attribute__((ext_vector_type(8)));

__global__ void __launch_bounds__(kBlock)
brace_consensus_kernel(const int16_t* __restrict__ parts, int64_t ld, int g, int64_t octets,
                       int thresh, float* __restrict__ out, uint8_t* __restrict__ bits)
{
    const int64_t o = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (o >= octets)
        return;
    const int16_t* p = parts + 8 * o;
    int s[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    int j = 0;
    for (; j + 4 <= g; j += 4) {
        i16x8 v[4];
#pragma unroll
        for (int r = 0; r < 4; ++r)
            v[r] = __builtin_nontemporal_load(reinterpret_cast<const i16x8*>(p + (int64_t)r * ld));
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int e = 0; e < 8; ++e)
                s[e] += v[r][e];
        p += 4 * ld;
    }
    for (; j < g; ++j) {
        const i16x8 v = *reinterpret_cast<const i16x8*>(p);
#pragma unroll
        for (int e = 0; e < 8; ++e)
            s[e] += v[e];
        p += ld;
    }
    uint32_t byte = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e)
        byte |= (s[e] >= thresh ? 1u : 0u) << e;
    if (out) {
        f32x4 a, b;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            a[e] = (byte >> e) & 1u ? 1.0f : -1.0f;
            b[e] = (byte >> (e + 4)) & 1u ? 1.0f : -1.0f;
        }
        __builtin_nontemporal_store(a, reinterpret_cast<f32x4*>(out + 8 * o));
        __builtin_nontemporal_store(b, reinterpret_cast<f32x4*>(out + 8 * o + 4));
    }
    if (bits)
        bits[o] = (uint8_t)byte;
}

// The same one coordinate per thread for [lo, d): rows that are not 16-byte aligned, and the
// last d mod 8 coordinates.  Every bit is set or cleared atomically (threads share words).
__global__ void __launch_bounds__(kBlock)
brace_consensus_tail_kernel(const int16_t* __restrict__ parts, int64_t ld, int g, int64_t lo,
                            int64_t d, int thresh, float* __restrict__ out, uint32_t* bits)
{
    const int64_t k = lo + (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (k >= d)
        return;
    int s = 0;
    const int16_t* p = parts + k;
    for (int j = 0; j < g; ++j) {
        s += *p;
        p += ld;
    }
    const bool up = s >= thresh;
    if (out)
        out[k] = up ? 1.0f : -1.0f;
    if (bits) {
        const uint32_t bit = 1u << (k & 31);
        if (up)
            atomicOr(&bits[k >> 5], bit);
        else
            atomicAnd(&bits[k >> 5], ~bit);
    }
}

// Clears the padding bits [d, roundup32(d)) of the last word (d is not a multiple of 32).
__global__ void brace_clear_pad_kernel(uint32_t* bits, int64_t d)
{
    if (threadIdx.x == 0 && blockIdx.x == 0)
        atomicAnd(&bits[d >> 5], (1u << (d & 31)) - 1u);
}

// The same for one-bit votes: S = 2P - n with P the number of set bits among the n clients.
__global__ void __launch_bounds__(kBlock)
brace_1bit_edge_kernel(const uint32_t* __restrict__ votes, int64_t ld_words, int n, int thresh,
                       float* out, uint32_t* bits, int64_t lo, int64_t lo_a, int64_t hi_a,
                       int64_t hi, int64_t hi_ext)
{
    const int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    const int64_t head = lo_a - lo;
    const int64_t k = (e < head) ? lo + e : hi_a + (e - head);
    if (k >= hi_ext)
        return;
    const uint32_t bit = 1u << (k & 31);
    if (k >= hi) {
        atomicAnd(&bits[k >> 5], ~bit);
        return;
    }
    const uint32_t* word = votes + (k >> 5);
    int up_votes = 0;
    for (int i = 0; i < n; ++i) {
        up_votes += (*word & bit) ? 1 : 0;
        word += ld_words;
    }
    const bool up = 2 * up_votes - n >= thresh;
    if (out)
        out[k] = up ? 1.0f : -1.0f;
    if (bits) {
        if (up)
            atomicOr(&bits[k >> 5], bit);
        else
            atomicAnd(&bits[k >> 5], ~bit);
    }
}

// ---------------------------------------------------------------------------------------
// Measurement aids: a plain streaming read and a plain copy of a buffer of known size.
// They calibrate what the HBM counters report per byte and give the bandwidth a trivially
// linear access pattern reaches on the same device, next to which the vote kernel is judged.
// ---------------------------------------------------------------------------------------
template <bool NT>
__global__ void __launch_bounds__(kBlock)
probe_read_kernel(const f32x4* __restrict__ src, int64_t nvec, int64_t per_block, float* sink)
{
    const int64_t begin = (int64_t)blockIdx.x * per_block;
    int64_t end = begin + per_block;
    if (end > nvec)
        end = nvec;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    int64_t i = begin + threadIdx.x;
    for (; i + 7 * kBlock < end; i += 8 * kBlock) {
        f32x4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            v[u] = NT ? __builtin_nontemporal_load(src + i + u * kBlock) : src[i + u * kBlock];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            acc += v[u];
    }
    for (; i < end; i += kBlock)
        acc += NT ? __builtin_nontemporal_load(src + i) : src[i];
    const float t = acc[0] + acc[1] + acc[2] + acc[3];
    if (t == 123456789.0f)           // practically never: keeps the loads alive
        sink[0] = t;
}

__global__ void __launch_bounds__(kBlock)
probe_copy_kernel(f32x4* __restrict__ dst, const f32x4* __restrict__ src, int64_t nvec,
                  int64_t per_block)
{
    const int64_t begin = (int64_t)blockIdx.x * per_block;
    int64_t end = begin + per_block;
    if (end > nvec)
        end = nvec;
    int64_t i = begin + threadIdx.x;
    for (; i + 3 * kBlock < end; i += 4 * kBlock) {
        f32x4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
            v[u] = __builtin_nontemporal_load(src + i + u * kBlock);
#pragma unroll
        for (int u = 0; u < 4; ++u)
            __builtin_nontemporal_store(v[u], dst + i + u * kBlock);
    }
    for (; i < end; i += kBlock)
        dst[i] = src[i];
}

bool aligned_to(const void* p, uintptr_t bytes)
{
    return (reinterpret_cast<uintptr_t>(p) & (bytes - 1)) == 0;
}

// Sizes are caller-supplied 64-bit numbers: a matrix of `rows` rows with pitch `pitch` must
// stay far inside the address space (2^47 bytes), so that no byte count computed from it
// can overflow.  Returns BRACE_OK or fails with BRACE_ERANGE.
int check_extent(int64_t rows, int64_t pitch, int64_t elem_bytes)
{
    const int64_t limit = ((int64_t)1 << 47) / elem_bytes;
    if (pitch > limit || rows > limit / (pitch > 0 ? pitch : 1))
        return fail(BRACE_ERANGE, "a matrix of %lld rows with pitch %lld does not fit the address space",
                    (long long)rows, (long long)pitch);
    return BRACE_OK;
}

// Eq. (1) on an integer sign-sum S with |S| <= limit:  S > lambda  <=>  S >= floor(lambda) + 1.
// The threshold saturates one step outside the range S can take: limit + 1 is never reached
// (all -1), -limit always is (all +1).  Every entry point that applies Eq. (1) takes its
// threshold from here.
int threshold_from_lambda(int64_t limit, float lambda)
{
    const double t = std::floor((double)lambda) + 1.0;
    if (t > (double)limit)
        return (int)limit + 1;
    if (t < -(double)limit)
        return -(int)limit;
    return (int)t;
}

// The buffers of one call, as byte intervals.  Two of them may not overlap unless both are
// only read; an overlap is reported with both names.
struct Span {
    const void* ptr;
    int64_t bytes;
    const char* name;
    bool written;
};

int check_disjoint(const Span* spans, int count)
{
    for (int i = 0; i < count; ++i) {
        if (!spans[i].ptr || spans[i].bytes <= 0)
            continue;
        const uintptr_t a0 = reinterpret_cast<uintptr_t>(spans[i].ptr);
        const uintptr_t a1 = a0 + (uintptr_t)spans[i].bytes;
        for (int j = i + 1; j < count; ++j) {
            if (!spans[j].ptr || spans[j].bytes <= 0 || !(spans[i].written || spans[j].written))
                continue;
            const uintptr_t b0 = reinterpret_cast<uintptr_t>(spans[j].ptr);
            const uintptr_t b1 = b0 + (uintptr_t)spans[j].bytes;
            if (a0 < b1 && b0 < a1)
                return fail(BRACE_EINVAL, "%s overlaps %s", spans[j].name, spans[i].name);
        }
    }
    return BRACE_OK;
}

// Checks of the consensus parameters shared by every entry point that takes brace_params_t.
int check_params(const brace_params_t* p, int64_t n, int64_t d, int64_t f)
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
    if (p->rule != 0 && p->rule != 1)
        return fail(BRACE_EINVAL, "rule must be 0 (Eq. (1)) or 1 (majority sign)");
    if (p->rule == 1 && p->out_bits_dev)
        return fail(BRACE_EINVAL, "the majority rule is three-valued and has no 1-bit form");
    return BRACE_OK;
}

int validate(const float* updates, int64_t n, int64_t d, int64_t f, const brace_params_t* p,
             const float* out, int64_t* ld_out, int* thresh_out)
{
    const int rc = check_params(p, n, d, f);
    if (rc != BRACE_OK)
        return rc;
    if (p->ld != 0 && p->ld < d)
        return fail(BRACE_EINVAL, "ld = %lld is smaller than d = %lld", (long long)p->ld,
                    (long long)d);
    const int64_t ld = p->ld ? p->ld : d;
    *ld_out = ld;
    *thresh_out = 0;
    if (check_extent(n, ld, 4) != BRACE_OK)
        return BRACE_ERANGE;
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
    // `out` is the float vector the call writes: out_dev, or w_dev of the fused update.
    const Span spans[] = {
        {updates, ((n - 1) * ld + d) * 4, "updates_dev", false},
        {out, d * 4, "out_dev", true},
        {p->out_bits_dev, ((d + 31) / 32) * 4, "out_bits_dev", true},
        {p->sums_dev, d * 2, "sums_dev", true},
    };
    if (check_disjoint(spans, 4) != BRACE_OK)
        return BRACE_EINVAL;
    // sign(S): +1 iff S >= 1, 0 at S == 0 (set by the kernel)
    *thresh_out = p->rule == 1 ? 1 : threshold_from_lambda(n, p->lambda);
    return BRACE_OK;
}

// Access width (in dwords) for one launch.  Vector stores need natural alignment: 4-byte
// outputs at out4, 2-byte outputs at out2.  Loads of the matrix only need dword alignment
// (see load_vec); measured on cfg 1 / cfg 2: rows that are 8-byte aligned run best with
// aligned 2-dword loads (6.96 vs 6.5 TB/s with misaligned 4-dword loads), rows that are only
// 4-byte aligned run best with misaligned 4-dword loads (14.2 vs 17.6 us with dword loads).
// `cap` (tuning) can only narrow the result.
int pick_width(const float* updates, int64_t n, int64_t ld, const void* out4, const void* out2,
               int cap)
{
    int rows = 4;                   // widest load that is aligned in every row
    while (rows > 1 && !(aligned_to(updates, 4u * rows) && (ld % rows == 0 || n == 1)))
        rows >>= 1;
    int v = rows == 1 ? 4 : rows;
    while (v > 1) {
        if ((!out4 || aligned_to(out4, 4u * v)) && (!out2 || aligned_to(out2, 2u * v)))
            break;
        v >>= 1;
    }
    if (cap == 1 || cap == 2 || cap == 4)
        v = v < cap ? v : cap;
    return v;
}

// Large ranges run about 1 % (n = 100) to 8 % (n = 200) faster with 2-dword than with 4-dword
// loads even where the rows would allow the wider ones: half the registers per wave, twice the
// waves per compute unit and tiles of half the size, which fill the last round of blocks
// better (n = 100, d = 25 M: 1.418 against 1.431 ms; n = 64, d = 100 M: 3.663 against 3.688 ms;
// n = 50, d = 11.2 M with rows on whole lines: 0.316 against 0.340 ms).  Not so where the
// floats written are a large share of the traffic (n = 8, d = 100 M: 0.68 against 0.57 ms), for
// ranges that fit the memory-side cache or a single ring chunk (n = 100, d = 500 k: 0.033
// against 0.030 ms), or when sign-sums leave through per-lane stores.  `few` is the client
// count below which the call's float traffic outweighs the gain.
int narrow_if_large(int v, const brace_tuning_t& t, int64_t n, int64_t coords, int64_t few,
                    bool per_lane_sums)
{
    if (v == 4 && t.vec == 0 && !per_lane_sums && n >= few && 4 * n * coords >= kSplitMinBytes)
        return 2;
    return v;
}

// Tile shape of one launch: loads per lane per row, rows per batch, row split.
struct Shape {
    int cols, unroll, rowsplit;
};

// Explicit tuning values win; zeros mean "choose from the size of the range".  Large ranges
// want long contiguous runs per wave (8 loads per row, 2 rows per batch, double-buffered:
// 32 KiB in flight per wave at 4-dword loads).  Shorter ranges shrink the tile until there are
// about 2 waves per SIMD (measured on single ring chunks of cfg 2-4: one load per row with 4
// rows per batch beats wider tiles and beats splitting rows); only when there are fewer
// waves than compute units do the waves of a block split the client rows.
Shape choose_shape(const brace_tuning_t& t, int64_t slots, int64_t n)
{
    const int64_t cus = compute_units() > 0 ? compute_units() : 256;
    const int64_t target = 8 * cus;                // 4 SIMDs per CU x 2 waves
    Shape s;
    s.cols = t.cols;
    if (s.cols == 0) {
        // With few client rows a wave is short-lived and its start-up and epilogue weigh more
        // than long contiguous runs gain: 4 loads per row below 48 clients (n = 4: 239 us
        // against 384 us with 8; n = 8: 488 / 537; n = 32: 561 / 572; n = 64: 3.76 / 3.75 ms).
        s.cols = n < kNarrowBelowClients ? 4 : 8;
        while (s.cols > 1 && slots / s.cols < target)
            s.cols >>= 1;
    }
    if (t.rowsplit == 0)
        s.rowsplit = (n >= 2 * kWaves && slots / s.cols < cus) ? 1 : 0;
    else
        s.rowsplit = t.rowsplit == 2 ? 1 : 0;
    if (s.rowsplit && s.cols > kRowsplitMaxCols)
        s.cols = kRowsplitMaxCols;
    s.unroll = t.unroll;
    if (s.unroll == 0) {
        s.unroll = s.cols >= 4 ? 2 : 4;             // 4 loads x 4 rows double-buffered runs out of registers
        const int64_t rows = s.rowsplit ? n / kWaves : n;
        while (s.unroll > 2 && 2 * s.unroll > rows)
            s.unroll >>= 1;
    }
    return s;
}

// Geometry of one launch over [lo, hi): body aligned to `unit` coordinates (a multiple of the
// wave slot 64*v), edges first, optional padding [hi, hi_ext) for the op.  Returns the grid.
int64_t plan_range(StreamArgs& a, Shape& shape, const brace_tuning_t& t, int64_t n, int64_t ld,
                   int v, int64_t unit, int64_t lo, int64_t hi, int64_t hi_ext)
{
    a.ld = ld;
    a.n = (int32_t)n;
    a.reserved = 0;
    a.lo = lo;
    a.hi = hi;
    a.hi_ext = hi_ext;
    int64_t lo_a = (lo + unit - 1) / unit * unit;
    int64_t hi_a = hi / unit * unit;
    if (lo_a >= hi_a)
        lo_a = hi_a = lo;          // no body: everything is "tail" edge
    a.lo_a = lo_a;
    a.hi_a = hi_a;

    const int64_t slots = (hi_a - lo_a) / (64 * (int64_t)v);
    shape = choose_shape(t, slots, n);
    const int64_t per_block = (shape.rowsplit ? 1 : (int64_t)kWaves) * shape.cols;
    const int64_t body_blocks = (slots + per_block - 1) / per_block;
    const int64_t edge = (lo_a - lo) + (hi_ext - hi_a);
    a.edge_blocks = (edge + kBlock - 1) / kBlock;
    return body_blocks + a.edge_blocks;
}

// Before anything is enqueued: every buffer must be device memory and the bytes the kernels
// will touch must lie inside the allocation that holds the pointer.  A wrong shape is then
// an error code on the host instead of a memory fault on the device.  Can be switched off
// (brace_set_pointer_checks) by callers that cannot afford the two runtime queries per buffer.
std::atomic<bool> g_pointer_checks{true};

int check_device_range(const void* ptr, int64_t bytes, const char* name)
{
    if (!g_pointer_checks || !ptr || bytes <= 0)
        return BRACE_OK;
    hipPointerAttribute_t attr;
    hipError_t err = hipPointerGetAttributes(&attr, ptr);
    if (err != hipSuccess) {
        (void)hipGetLastError();                   // do not leave the error for the next launch check
        return fail(BRACE_EINVAL, "%s is not a device pointer known to the HIP runtime (%s)", name,
                    hipGetErrorString(err));
    }
    if (attr.type != hipMemoryTypeDevice && attr.type != hipMemoryTypeManaged &&
        attr.type != hipMemoryTypeUnified)
        return fail(BRACE_EINVAL, "%s is not device memory", name);
    hipDeviceptr_t base = nullptr;
    size_t size = 0;
    err = hipMemGetAddressRange(&base, &size, const_cast<void*>(ptr));
    if (err != hipSuccess) {
        (void)hipGetLastError();
        return fail(BRACE_EINVAL, "%s: cannot query its allocation (%s)", name, hipGetErrorString(err));
    }
    const uintptr_t p = reinterpret_cast<uintptr_t>(ptr);
    const uintptr_t b = reinterpret_cast<uintptr_t>(base);
    if (p < b || (uint64_t)bytes > (uint64_t)size || p - b > size - (uint64_t)bytes)
        return fail(BRACE_EINVAL, "%s: the call needs %lld bytes from this pointer but its allocation "
                                  "ends after %lld", name, (long long)bytes,
                    (long long)(size - (size_t)(p - b)));
    return BRACE_OK;
}

// The buffers of a vote / sum / update call over the FULL vectors (chunk calls address them too).
int check_buffers(const float* updates, int64_t n, int64_t d, int64_t ld, const float* out,
                  const void* bits, const void* sums, const float* w)
{
    int rc = check_device_range(updates, ((n - 1) * ld + d) * 4, "updates_dev");
    if (rc == BRACE_OK)
        rc = check_device_range(out, d * 4, "out_dev");
    if (rc == BRACE_OK)
        rc = check_device_range(bits, ((d + 31) / 32) * 4, "out_bits_dev");
    if (rc == BRACE_OK)
        rc = check_device_range(sums, d * 2, "sums_dev");
    if (rc == BRACE_OK)
        rc = check_device_range(w, d * 4, "w_dev");
    return rc;
}

// Staged (burst-write) launch: legal when the op writes one float per coordinate to 16-byte
// aligned arrays with 2- or 4-dword accesses; chosen for ranges large enough to get the
// widest tile anyway.  Returns the tiles per block (0 = use the ordinary kernel).
int stage_tiles_for(const brace_tuning_t& t, const Shape& sh, int v, int64_t slots, int64_t n,
                    const void* out, const void* w, const void* sums = nullptr)
{
    if (t.stage_writes == 1 || (v != 2 && v != 4) || sh.rowsplit)
        return 0;
    if (sums && !aligned_to(sums, 8))
        return 0;
    // A range that fits the memory-side cache gains nothing from bursts (n = 8, d = 8 M:
    // 44.6 us with stores per wave, 47.8 us staged).
    if (t.stage_writes != 2 && 4 * n * slots * 64 * v < kSplitMinBytes)
        return 0;
    if ((out && !aligned_to(out, 16)) || (w && !aligned_to(w, 16)))
        return 0;
    // The large-range shapes: 8 loads per row, or 4 where that is the choice for few clients
    // (and not a tile shrunk because the range is short).
    const bool stage_shape = sh.cols == kStageColsWide ||
                             (sh.cols == kStageColsNarrow && n < kNarrowBelowClients);
    if (t.stage_writes != 2 && (t.cols != 0 || t.unroll != 0 || !stage_shape))
        return 0;                  // explicit tile tuning, or a short range: ordinary kernel
    const int scols = sh.cols == kStageColsNarrow ? kStageColsNarrow : kStageColsWide;
    // The LDS burst limits a compute unit to one block, so the blocks run in rounds of one
    // per unit and a last, part-filled round costs as much as a full one.  Among the burst
    // sizes that fit, take the largest whose rounds are (nearly) as full as the best one.
    const size_t tile_bytes = (size_t)kWaves * scols * 64 * v * 4;
    const int max_tiles = (int)(kStageBytes / tile_bytes);
    const int64_t cus = compute_units() > 0 ? compute_units() : 256;
    const int64_t tiles = (slots + kWaves * scols - 1) / (kWaves * scols);
    int best = 0;
    double best_fill = 0.0;
    for (int k = 2; k <= max_tiles; ++k) {
        const int64_t blocks = (tiles + k - 1) / k;
        if (blocks < cus)
            break;
        const double fill = (double)blocks / (double)((blocks + cus - 1) / cus * cus);
        if (fill >= 0.95 * best_fill) {
            best = k;
            if (fill > best_fill)
                best_fill = fill;
        }
    }
    if (t.stage_writes == 2 && best == 0 && slots > 0)
        best = max_tiles;          // forced: correctness tests on inputs of any size
    return best;
}

// Opt a kernel in to more than the default 64 KiB of dynamic LDS (once per kernel and device).
int allow_stage_lds(const void* kernel, size_t bytes = kStageBytes)
{
    struct Seen { const void* kernel; int dev; };
    static Seen done[64] = {};
    static std::mutex guard;                   // entry points may be called from several threads
    const std::lock_guard<std::mutex> lock(guard);
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return fail(BRACE_EHIP, "no current device");
    }
    for (const Seen& s : done)
        if (s.kernel == kernel && s.dev == dev)
            return BRACE_OK;
    const hipError_t err = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                               (int)bytes);
    if (err != hipSuccess) {
        (void)hipGetLastError();
        return fail(BRACE_EHIP, "cannot reserve %zu bytes of LDS: %s", bytes, hipGetErrorString(err));
    }
    for (Seen& s : done)
        if (!s.kernel) {           // a full table only means the attribute is set again next time
            s.kernel = kernel;
            s.dev = dev;
            break;
        }
    return BRACE_OK;
}

int check_launch(const char* what)
{
    const hipError_t err = hipGetLastError();
    if (err != hipSuccess)
        return fail(BRACE_EHIP, "%s launch failed: %s", what, hipGetErrorString(err));
    return BRACE_OK;
}

// Library-owned workspace of brace_aggregate_update_noalloc: the bit-words that pass the vote
// from the streaming kernel to the kernel that updates the model, for callers that cannot
// hand over a bit array.  One copy per device, held until the process ends.  In host code the
// array's name is only a handle: the device address is looked up once per device and every
// launch takes that address as an argument.
constexpr int64_t kScratchWords = BRACE_NOALLOC_MAX_D / 32;             // 16 MiB
static __device__ __align__(256) uint32_t scratch[kScratchWords];

std::atomic<uint32_t*> g_scratch_addr[kMaxDevices];                     // null = not looked up yet

int scratch_of_current_device(uint32_t** addr)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return fail(BRACE_EHIP, "no current device");
    }
    if (dev < 0 || dev >= kMaxDevices)
        return fail(BRACE_ERANGE, "device %d is beyond the %d devices the library keeps a "
                                  "workspace address for", dev, kMaxDevices);
    uint32_t* known = g_scratch_addr[dev].load(std::memory_order_acquire);
    if (!known) {
        void* found = nullptr;
        const hipError_t err = hipGetSymbolAddress(&found, HIP_SYMBOL(scratch));
        if (err != hipSuccess || !found) {
            (void)hipGetLastError();
            return fail(BRACE_EHIP, "cannot find the workspace on device %d: %s", dev,
                        hipGetErrorString(err));
        }
        known = static_cast<uint32_t*>(found);
        g_scratch_addr[dev].store(known, std::memory_order_release);   // same value from any thread
    }
    *addr = known;
    return BRACE_OK;
}

// `ws_bits` (optional) is a workspace of at least ceil(d/32) words that may carry the vote of
// the fused update from the streaming kernel to the kernel that applies it when the caller
// gave no bit array; its contents after the call are unspecified.
int launch_vote(const float* updates, int64_t n, int64_t d, int64_t ld, int thresh,
                const brace_params_t* p, float* out, float* w, float eta, int64_t lo, int64_t hi,
                hipStream_t stream, uint32_t* ws_bits = nullptr)
{
    if (hi <= lo)
        return BRACE_OK;
    int rc = check_buffers(updates, n, d, ld, out, p->out_bits_dev, p->sums_dev, w);
    if (rc != BRACE_OK)
        return rc;
    const brace_tuning_t t = current_tuning();
    int v = pick_width(updates, n, ld, out, p->sums_dev, t.vec);
    if (w)
        v = pick_width(updates, n, ld, w, nullptr, v);
    uint32_t* bits = static_cast<uint32_t*>(p->out_bits_dev);
    // the in-place update without a bit-word carrier reads and writes the model in the stream
    v = narrow_if_large(v, t, n, hi - lo, (w && !bits && !ws_bits) ? kNarrowBelowClients : kStageBelowClients,
                        p->sums_dev != nullptr);

    // Split the writes off the read stream?  Needs float output, 16-byte aligned, and whole
    // 1024-coordinate groups; worth it only for large ranges unless forced.
    const int64_t lo_s = (lo + kGroup - 1) / kGroup * kGroup;
    const int64_t hi_s = hi / kGroup * kGroup;
    const int64_t groups = hi_s > lo_s ? (hi_s - lo_s) / kGroup : 0;
    // The fused model update can only be split off when the caller gave a bit array: the
    // model itself holds live data and cannot park the bit-words.
    bool split = (out || w) && (!out || aligned_to(out, 16)) &&
                 (!w || ((bits || ws_bits) && aligned_to(w, 16))) && groups > 0 && t.split_writes != 1;
    if (split && t.split_writes != 2)
        split = 4 * n * (hi - lo) >= kSplitMinBytes;
    if (p->rule == 1)
        split = false;             // three values do not fit the bit-words
    if (split && t.split_writes == 0 && t.stage_writes == 0 && n < kStageBelowClients && !bits &&
        !ws_bits && !p->sums_dev) {
        // Few clients: prefer bursts from this kernel if the range qualifies for them.
        StreamArgs a0;
        Shape sh0;
        (void)plan_range(a0, sh0, t, n, ld, v, 64 * (int64_t)v, lo, hi, hi);
        const int64_t slots0 = (a0.hi_a - a0.lo_a) / (64 * (int64_t)v);
        if (stage_tiles_for(t, sh0, v, slots0, n, out, w) > 0)
            split = false;
    }

    // Where the body's bit-words go: the caller's array (also the packed output), the
    // workspace of a split update without one, else (float output) they are parked in `out`.
    uint32_t* const body_bits = (split && w && !bits) ? ws_bits : bits;
    VoteOp op;
    op.out = out;
    op.bits = body_bits;
    op.sums = p->sums_dev;
    op.w = w;
    op.eta = eta;
    op.thresh = thresh;
    op.zero_sign = p->zero_sign;
    op.split = split ? 1 : 0;
    op.tie_zero = p->rule == 1 ? 1 : 0;
    op.stage_sums = 0;

    int64_t hi_ext = hi;
    if (bits && hi == d)
        hi_ext = (d + 31) & ~(int64_t)31;          // the last word's padding bits are zeroed
    StreamArgs a;
    Shape sh;
    const int64_t grid = plan_range(a, sh, t, n, ld, v, split ? kGroup : 64 * (int64_t)v, lo, hi,
                                    hi_ext);
    if (grid <= 0)
        return BRACE_OK;
    if (grid > 0x7fffffffLL)
        return fail(BRACE_ERANGE, "range needs %lld blocks, more than one launch can hold",
                    (long long)grid);

    const int64_t slots = (a.hi_a - a.lo_a) / (64 * (int64_t)v);
    const bool plain_floats = !split && !body_bits && !p->sums_dev && (out || w);
    const bool stage_ok = plain_floats;
    // Sign-sums alone (the partial sums a device contributes to Share-Reduce) are staged the
    // same way (n = 12, d = 100 M: 852 us with stores per wave, 727 us for the reads alone).
    const bool sums_only = p->sums_dev && !out && !w && !bits;
    int stage = 0;
    if (stage_ok)
        stage = stage_tiles_for(t, sh, v, slots, n, out, w);
    else if (sums_only)
        stage = stage_tiles_for(t, sh, v, slots, n, nullptr, nullptr, p->sums_dev);
    op.stage_sums = (stage > 0 && sums_only) ? 1 : 0;
    if (stage > 0) {
        const int scols = sh.cols == kStageColsNarrow ? kStageColsNarrow : kStageColsWide;
        const int64_t per_block = (int64_t)stage * kWaves * scols;
        const int64_t sgrid = (slots + per_block - 1) / per_block + a.edge_blocks;
        stream_staged_kernel_t<VoteOp> ks = brace_vote_pick_staged(v, scols, t.pipeline);
        rc = allow_stage_lds(reinterpret_cast<const void*>(ks));
        if (rc != BRACE_OK)
            return rc;
        hipLaunchKernelGGL(ks, dim3((unsigned)sgrid), dim3(kBlock), kStageBytes, stream, updates, a,
                           op, stage);
        return check_launch("staged vote kernel");
    }
    stream_kernel_t<VoteOp> k;
    switch (v) {
    case 4: k = brace_vote_pick_v4(sh.cols, sh.unroll, t.nontemporal, t.pipeline,
                                    sh.rowsplit); break;
    case 2: k = brace_vote_pick_v2(sh.cols, sh.unroll, t.nontemporal, t.pipeline,
                                    sh.rowsplit); break;
    default: k = brace_vote_pick_v1(sh.cols, sh.unroll, t.nontemporal, t.pipeline,
                                    sh.rowsplit); break;
    }
    const size_t lds = sh.rowsplit ? sizeof(VoteOp::State) * (kWaves - 1) * sh.cols * v * 64 : 0;
    hipLaunchKernelGGL(k, dim3((unsigned)grid), dim3(kBlock), lds, stream, updates, a, op);
    rc = check_launch("vote kernel");
    if (rc != BRACE_OK)
        return rc;
    if (split) {
        const int64_t egrid = (groups + kWaves - 1) / kWaves;
        if (out) {
            hipLaunchKernelGGL(brace_expand_kernel, dim3((unsigned)egrid), dim3(kBlock), 0, stream,
                               out, static_cast<const uint32_t*>(bits), a.lo_a, groups, a.hi_a);
            rc = check_launch("expand kernel");
            if (rc != BRACE_OK)
                return rc;
        }
        if (w) {
            hipLaunchKernelGGL(brace_apply_kernel, dim3((unsigned)egrid), dim3(kBlock), 0, stream,
                               w, static_cast<const uint32_t*>(body_bits), eta, a.lo_a, groups);
            rc = check_launch("apply kernel");
        }
    }
    return rc;
}

int launch_sum(const float* updates, int64_t n, int64_t d, int64_t ld, double scale, float* out,
               int64_t lo, int64_t hi, hipStream_t stream)
{
    if (hi <= lo)
        return BRACE_OK;
    const int rc = check_buffers(updates, n, d, ld, out, nullptr, nullptr, nullptr);
    if (rc != BRACE_OK)
        return rc;
    const brace_tuning_t t = current_tuning();
    const int v = narrow_if_large(pick_width(updates, n, ld, out, nullptr, t.vec), t, n, hi - lo,
                                  kStageBelowClients, false);
    SumOp op;
    op.out = out;
    op.scale = scale;
    StreamArgs a;
    Shape sh;
    const int64_t grid = plan_range(a, sh, t, n, ld, v, 64 * (int64_t)v, lo, hi, hi);
    if (grid <= 0)
        return BRACE_OK;
    if (grid > 0x7fffffffLL)
        return fail(BRACE_ERANGE, "range needs %lld blocks, more than one launch can hold",
                    (long long)grid);
    const int64_t slots = (a.hi_a - a.lo_a) / (64 * (int64_t)v);
    const int stage = stage_tiles_for(t, sh, v, slots, n, out, nullptr);
    if (stage > 0) {
        const int scols = sh.cols == kStageColsNarrow ? kStageColsNarrow : kStageColsWide;
        const int64_t per_block = (int64_t)stage * kWaves * scols;
        const int64_t sgrid = (slots + per_block - 1) / per_block + a.edge_blocks;
        stream_staged_kernel_t<SumOp> ks = brace_sum_pick_staged(v, scols, t.pipeline);
        const int rcs = allow_stage_lds(reinterpret_cast<const void*>(ks));
        if (rcs != BRACE_OK)
            return rcs;
        hipLaunchKernelGGL(ks, dim3((unsigned)sgrid), dim3(kBlock), kStageBytes, stream, updates, a,
                           op, stage);
        return check_launch("staged sum kernel");
    }
    stream_kernel_t<SumOp> k;
    switch (v) {
    case 4: k = brace_sum_pick_v4(sh.cols, sh.unroll, t.nontemporal, t.pipeline,
                                    sh.rowsplit); break;
    case 2: k = brace_sum_pick_v2(sh.cols, sh.unroll, t.nontemporal, t.pipeline,
                                    sh.rowsplit); break;
    default: k = brace_sum_pick_v1(sh.cols, sh.unroll, t.nontemporal, t.pipeline,
                                    sh.rowsplit); break;
    }
    const size_t lds = sh.rowsplit ? sizeof(SumOp::State) * (kWaves - 1) * sh.cols * v * 64 : 0;
    hipLaunchKernelGGL(k, dim3((unsigned)grid), dim3(kBlock), lds, stream, updates, a, op);
    return check_launch("sum kernel");
}

// The ring-order fp32 sum over the coordinate range [lo, hi): same launch planning as the
// fp64 sum (tile shape from the size of the range, bursts for large ranges); the kernel finds
// the chunk, hence the start row, of every run of slots by itself.
int launch_ring_sum(const float* updates, int64_t n, int64_t d, int64_t ld, int mean, float* out,
                    int64_t lo, int64_t hi, hipStream_t stream)
{
    if (hi <= lo)
        return BRACE_OK;
    const int rc = check_buffers(updates, n, d, ld, out, nullptr, nullptr, nullptr);
    if (rc != BRACE_OK)
        return rc;
    const brace_tuning_t t = current_tuning();
    const int v = narrow_if_large(pick_width(updates, n, ld, out, nullptr, t.vec), t, n, hi - lo,
                                  kStageBelowClients, false);
    RingArgs g;
    g.q = d / n;
    g.r = d % n;
    g.mean = mean;
    g.reserved = 0;
    StreamArgs a;
    Shape sh;
    (void)plan_range(a, sh, t, n, ld, v, 64 * (int64_t)v, lo, hi, hi);
    // the ring kernel exists for 8, 4 and 1 loads per row and never splits the rows of a block
    int cols = sh.cols >= kStageColsWide ? kStageColsWide
             : sh.cols >= kStageColsNarrow ? kStageColsNarrow : 1;
    sh.cols = cols;
    sh.rowsplit = 0;
    const int64_t slots = (a.hi_a - a.lo_a) / (64 * (int64_t)v);
    const int stage = stage_tiles_for(t, sh, v, slots, n, out, nullptr);
    if (stage > 0)                 // the burst kernels exist for the two large-range shapes only
        cols = sh.cols == kStageColsNarrow ? kStageColsNarrow : kStageColsWide;
    const int64_t per_block = (int64_t)kWaves * cols * (stage > 0 ? stage : 1);
    const int64_t grid = (slots + per_block - 1) / per_block + a.edge_blocks;
    if (grid <= 0)
        return BRACE_OK;
    if (grid > 0x7fffffffLL)
        return fail(BRACE_ERANGE, "range needs %lld blocks, more than one launch can hold",
                    (long long)grid);
    ring_sum_kernel_t k = brace_ring_pick(v, cols, stage > 0);
    size_t lds = 0;
    if (stage > 0) {
        const int rcs = allow_stage_lds(reinterpret_cast<const void*>(k));
        if (rcs != BRACE_OK)
            return rcs;
        lds = kStageBytes;
    }
    hipLaunchKernelGGL(k, dim3((unsigned)grid), dim3(kBlock), lds, stream, updates, a, g, out, stage);
    return check_launch("ring-order sum kernel");
}

int validate_rar(const float* updates, int64_t n, int64_t d, const brace_rar_params_t* p,
                 const float* out, int64_t* ld_out, double* scale_out)
{
    if (!p)
        return fail(BRACE_EINVAL, "params is NULL");
    if (p->struct_size != sizeof(brace_rar_params_t))
        return fail(BRACE_EINVAL, "params->struct_size is %u, expected %zu", p->struct_size,
                    sizeof(brace_rar_params_t));
    if (n < 1)
        return fail(BRACE_EINVAL, "n must be >= 1 (got %lld)", (long long)n);
    if (n > BRACE_MAX_CLIENTS)
        return fail(BRACE_ERANGE, "n = %lld exceeds BRACE_MAX_CLIENTS", (long long)n);
    if (d < 0)
        return fail(BRACE_EINVAL, "d must be >= 0 (got %lld)", (long long)d);
    if (p->mean != 0 && p->mean != 1)
        return fail(BRACE_EINVAL, "mean must be 0 (sum) or 1 (mean)");
    if ((p->order != 0 && p->order != 1) || p->reserved != 0)
        return fail(BRACE_EINVAL, "order must be 0 (fp64, index order) or 1 (fp32, ring order) "
                                  "and reserved 0");
    if (p->ld != 0 && p->ld < d)
        return fail(BRACE_EINVAL, "ld = %lld is smaller than d = %lld", (long long)p->ld,
                    (long long)d);
    const int64_t ld = p->ld ? p->ld : d;
    *ld_out = ld;
    *scale_out = p->mean ? 1.0 / (double)n : 1.0;
    if (check_extent(n, ld, 4) != BRACE_OK)
        return BRACE_ERANGE;
    if (d == 0)
        return BRACE_OK;
    if (!updates || !out)
        return fail(BRACE_EINVAL, "updates_dev or out_dev is NULL");
    if (!aligned_to(updates, 4) || !aligned_to(out, 4))
        return fail(BRACE_EINVAL, "updates_dev and out_dev must be 4-byte aligned");
    const Span spans[] = {{updates, ((n - 1) * ld + d) * 4, "updates_dev", false},
                          {out, d * 4, "out_dev", true}};
    return check_disjoint(spans, 2);
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

// The run of ring chunks [chunk_begin, chunk_end) as one coordinate range (consecutive chunks
// are contiguous); an empty run gives lo = hi.
static int chunk_run_range(int64_t n, int64_t d, int64_t chunk_begin, int64_t chunk_end, int64_t* lo,
                    int64_t* hi)
{
    if (n < 1 || d < 0)
        return fail(BRACE_EINVAL, "need n >= 1 and d >= 0");
    if (chunk_begin < 0 || chunk_end > n || chunk_begin > chunk_end)
        return fail(BRACE_ERANGE, "chunk range [%lld, %lld) outside [0, %lld]",
                    (long long)chunk_begin, (long long)chunk_end, (long long)n);
    *lo = *hi = 0;
    if (chunk_begin == chunk_end)
        return BRACE_OK;
    int64_t unused;
    int rc = brace_chunk_range(n, d, chunk_begin, lo, &unused);
    if (rc == BRACE_OK)
        rc = brace_chunk_range(n, d, chunk_end - 1, &unused, hi);
    return rc;
}

int brace_threshold(int64_t n, float lambda, int32_t* threshold)
{
    if (!threshold)
        return fail(BRACE_EINVAL, "threshold is NULL");
    if (n < 1 || !std::isfinite(lambda))
        return fail(BRACE_EINVAL, "need n >= 1 and a finite lambda");
    if (n > ((int64_t)1 << 30))
        return fail(BRACE_ERANGE, "n = %lld is beyond the range of a 32-bit threshold", (long long)n);
    *threshold = threshold_from_lambda(n, lambda);
    return BRACE_OK;
}

int brace_comm_cost(int32_t scheme, int64_t m, int64_t n, int64_t d, double* bits_per_client)
{
    if (!bits_per_client)
        return fail(BRACE_EINVAL, "bits_per_client is NULL");
    if (m < 1 || m > 64 || n < 1 || d < 0)
        return fail(BRACE_EINVAL, "need 1 <= m <= 64, n >= 1 and d >= 0");
    const long double M = (long double)m, N = (long double)n, D = (long double)d;
    switch (scheme) {
    case BRACE_COST_SERVER_CLIENT: *bits_per_client = (double)(M * N * D); break;
    case BRACE_COST_RING_ALL_REDUCE: *bits_per_client = (double)(2.0L * M * D * (N - 1.0L) / N); break;
    case BRACE_COST_BRACE: *bits_per_client = (double)(D * (N - 1.0L) * (M + 1.0L) / N); break;
    default: return fail(BRACE_EINVAL, "unknown scheme %d", (int)scheme);
    }
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
    return launch_vote(updates_dev, n, d, ld, thresh, params, out_dev, nullptr, 0.0f, 0, d,
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
    return launch_vote(updates_dev, n, d, ld, thresh, params, out_dev, nullptr, 0.0f, lo, hi,
                       static_cast<hipStream_t>(hip_stream));
}

int brace_aggregate_chunks(const float* updates_dev, int64_t n, int64_t d, int64_t f,
                           int64_t chunk_begin, int64_t chunk_end, const brace_params_t* params,
                           float* out_dev, void* hip_stream)
{
    int64_t ld;
    int thresh;
    int rc = validate(updates_dev, n, d, f, params, out_dev, &ld, &thresh);
    if (rc != BRACE_OK)
        return rc;
    int64_t lo, hi;
    rc = chunk_run_range(n, d, chunk_begin, chunk_end, &lo, &hi);
    if (rc != BRACE_OK)
        return rc;
    return launch_vote(updates_dev, n, d, ld, thresh, params, out_dev, nullptr, 0.0f, lo, hi,
                       static_cast<hipStream_t>(hip_stream));
}

// Shared by the fused-update entry points: the vote's validation plus the model buffer.
static int validate_update(const float* updates, int64_t n, int64_t d, int64_t f,
                           const brace_params_t* p, float eta, const float* w, int64_t* ld,
                           int* thresh)
{
    // `w` stands in for the float output in the shared checks (non-NULL, aligned, no overlap).
    const int rc = validate(updates, n, d, f, p, w, ld, thresh);
    if (rc != BRACE_OK)
        return rc;
    if (!std::isfinite(eta))
        return fail(BRACE_EINVAL, "eta must be finite");
    if (d > 0 && !w)
        return fail(BRACE_EINVAL, "w_dev is NULL");
    return BRACE_OK;
}

int brace_aggregate_update(const float* updates_dev, int64_t n, int64_t d, int64_t f,
                           const brace_params_t* params, float eta, float* w_dev, void* hip_stream)
{
    int64_t ld;
    int thresh;
    const int rc = validate_update(updates_dev, n, d, f, params, eta, w_dev, &ld, &thresh);
    if (rc != BRACE_OK)
        return rc;
    return launch_vote(updates_dev, n, d, ld, thresh, params, nullptr, w_dev, eta, 0, d,
                       static_cast<hipStream_t>(hip_stream));
}

int brace_aggregate_update_chunk(const float* updates_dev, int64_t n, int64_t d, int64_t f,
                                 int64_t chunk, const brace_params_t* params, float eta,
                                 float* w_dev, void* hip_stream)
{
    int64_t ld;
    int thresh;
    int rc = validate_update(updates_dev, n, d, f, params, eta, w_dev, &ld, &thresh);
    if (rc != BRACE_OK)
        return rc;
    int64_t lo, hi;
    rc = brace_chunk_range(n, d, chunk, &lo, &hi);
    if (rc != BRACE_OK)
        return rc;
    return launch_vote(updates_dev, n, d, ld, thresh, params, nullptr, w_dev, eta, lo, hi,
                       static_cast<hipStream_t>(hip_stream));
}

int brace_aggregate_update_noalloc(const float* updates_dev, int64_t n, int64_t d, int64_t f,
                                   const brace_params_t* params, float eta, float* w_dev,
                                   void* hip_stream)
{
    // The size limit first: it does not depend on any other argument.
    if (d > BRACE_NOALLOC_MAX_D)
        return fail(BRACE_ERANGE, "d = %lld exceeds BRACE_NOALLOC_MAX_D = %lld, the size of the "
                                  "library's workspace", (long long)d, (long long)BRACE_NOALLOC_MAX_D);
    int64_t ld;
    int thresh;
    int rc = validate_update(updates_dev, n, d, f, params, eta, w_dev, &ld, &thresh);
    if (rc != BRACE_OK)
        return rc;
    if (params->out_bits_dev)
        return fail(BRACE_EINVAL, "this entry point takes no bit array (its bit-words live in the "
                                  "library's own workspace); use brace_aggregate_update");
    if (d == 0)
        return BRACE_OK;
    uint32_t* ws = nullptr;
    rc = scratch_of_current_device(&ws);
    if (rc != BRACE_OK)
        return rc;
    // Nothing in the workspace has to start at zero: the streaming kernel writes every word
    // that the applying kernel reads, earlier on the same stream.
    return launch_vote(updates_dev, n, d, ld, thresh, params, nullptr, w_dev, eta, 0, d,
                       static_cast<hipStream_t>(hip_stream), ws);
}

// Receive side of Share-Only: a client holding the packed result materialises it.
static int launch_from_bits(const uint32_t* bits, int64_t d, float* out, float* w, float eta,
                            hipStream_t stream)
{
    if (d == 0)
        return BRACE_OK;
    int rc = check_device_range(bits, ((d + 31) / 32) * 4, "bits_dev");
    if (rc == BRACE_OK)
        rc = check_device_range(out, d * 4, "out_dev");
    if (rc == BRACE_OK)
        rc = check_device_range(w, d * 4, "w_dev");
    if (rc != BRACE_OK)
        return rc;
    float* target = out ? out : w;
    const int64_t groups = aligned_to(target, 16) ? d / kGroup : 0;
    if (groups > 0) {
        const int64_t egrid = (groups + kWaves - 1) / kWaves;
        if (egrid > 0x7fffffffLL)
            return fail(BRACE_ERANGE, "vector too long for one launch");
        if (out)
            hipLaunchKernelGGL(brace_expand_kernel, dim3((unsigned)egrid), dim3(kBlock), 0, stream,
                               out, bits, (int64_t)0, groups, groups * kGroup);
        else
            hipLaunchKernelGGL(brace_apply_kernel, dim3((unsigned)egrid), dim3(kBlock), 0, stream,
                               w, bits, eta, (int64_t)0, groups);
        rc = check_launch("bits kernel");
        if (rc != BRACE_OK)
            return rc;
    }
    const int64_t lo = groups * kGroup;
    if (lo < d) {
        const int64_t tgrid = (d - lo + kBlock - 1) / kBlock;
        if (tgrid > 0x7fffffffLL)
            return fail(BRACE_ERANGE, "vector too long for one launch");
        hipLaunchKernelGGL(brace_bits_tail_kernel, dim3((unsigned)tgrid), dim3(kBlock), 0, stream,
                           out, out ? nullptr : w, bits, eta, lo, d);
        rc = check_launch("bits tail kernel");
    }
    return rc;
}

int brace_expand_bits(const void* bits_dev, int64_t d, float* out_dev, void* hip_stream)
{
    if (d < 0)
        return fail(BRACE_EINVAL, "d must be >= 0");
    if (check_extent(1, d, 4) != BRACE_OK)
        return BRACE_ERANGE;
    if (d > 0 && (!bits_dev || !out_dev || !aligned_to(bits_dev, 4) || !aligned_to(out_dev, 4)))
        return fail(BRACE_EINVAL, "bits_dev and out_dev must be non-NULL and 4-byte aligned");
    return launch_from_bits(static_cast<const uint32_t*>(bits_dev), d, out_dev, nullptr, 0.0f,
                            static_cast<hipStream_t>(hip_stream));
}

int brace_apply_bits(const void* bits_dev, int64_t d, float eta, float* w_dev, void* hip_stream)
{
    if (d < 0)
        return fail(BRACE_EINVAL, "d must be >= 0");
    if (check_extent(1, d, 4) != BRACE_OK)
        return BRACE_ERANGE;
    if (!std::isfinite(eta))
        return fail(BRACE_EINVAL, "eta must be finite");
    if (d > 0 && (!bits_dev || !w_dev || !aligned_to(bits_dev, 4) || !aligned_to(w_dev, 4)))
        return fail(BRACE_EINVAL, "bits_dev and w_dev must be non-NULL and 4-byte aligned");
    return launch_from_bits(static_cast<const uint32_t*>(bits_dev), d, nullptr, w_dev, eta,
                            static_cast<hipStream_t>(hip_stream));
}

// ---------------------------------------------------------------------------------------
// Quantise-once route.  The two packed forms differ in a few constants only:
//   two planes (pos, neg): 2 bits per coordinate, a 16-byte lane load covers 64 coordinates;
//   one bit (vote is +1):  1 bit per coordinate,  a 16-byte lane load covers 128.
// ---------------------------------------------------------------------------------------
}  // extern "C"

namespace {

struct PlaneForm {
    bool two_planes;
    const char* matrix;         // name of the packed matrix argument in messages
    int64_t (*row_words)(int64_t);
    int coords_per_load;        // coordinates in one u32x4 of a row
};

int64_t roundup_words(int64_t w, int64_t to)
{
    return w / to * to + (w % to ? to : 0);     // no overflow for any w the callers pass
}

const PlaneForm kTwoPlanes = {true, "signs_dev", brace_packed_row_words, 64};
const PlaneForm kOneBit = {false, "votes_dev", brace_1bit_row_words, 128};

// Shape checks of a packed matrix of n rows for vectors of d coordinates; resolves ld_words.
int check_plane_shape(const PlaneForm& form, int64_t n, int64_t d, int64_t* ld_words)
{
    if (d > ((int64_t)1 << 45))
        return fail(BRACE_ERANGE, "d = %lld does not fit the address space", (long long)d);
    const int64_t row_words = form.row_words(d);
    if (*ld_words == 0)
        *ld_words = row_words;
    if (*ld_words < row_words || (*ld_words & 3))
        return fail(BRACE_EINVAL, "ld_words must be a multiple of 4 and at least the %lld words "
                                  "of a row", (long long)row_words);
    return check_extent(n, *ld_words, 4);
}

// Phase I as data, both forms: validation, the choice between a store per span and 128 KiB
// bursts, and the launch.
int quantize_to_planes(const PlaneForm& form, const float* updates_dev, int64_t n, int64_t d,
                       int64_t ld, int up_if_not_negative, uint32_t* planes_dev, int64_t ld_words,
                       hipStream_t stream)
{
    if (n < 1 || d < 0)
        return fail(BRACE_EINVAL, "need n >= 1 and d >= 0");
    if (n > BRACE_MAX_CLIENTS)
        return fail(BRACE_ERANGE, "n = %lld exceeds BRACE_MAX_CLIENTS", (long long)n);
    if (ld == 0)
        ld = d;
    if (ld < d)
        return fail(BRACE_EINVAL, "ld = %lld is smaller than d = %lld", (long long)ld, (long long)d);
    if (check_extent(n, ld, 4) != BRACE_OK)
        return BRACE_ERANGE;
    int rc = check_plane_shape(form, n, d, &ld_words);
    if (rc != BRACE_OK)
        return rc;
    if (d == 0)
        return BRACE_OK;
    if (!updates_dev || !planes_dev || !aligned_to(updates_dev, 4) || !aligned_to(planes_dev, 16))
        return fail(BRACE_EINVAL, "updates_dev (4-byte aligned) and %s (16-byte aligned) must be "
                                  "non-NULL", form.matrix);
    const int64_t row_words = form.row_words(d);
    const int64_t in_bytes = ((n - 1) * ld + d) * 4;
    const int64_t out_bytes = ((n - 1) * ld_words + row_words) * 4;
    const Span spans[] = {{updates_dev, in_bytes, "updates_dev", false},
                          {planes_dev, out_bytes, form.matrix, true}};
    if (check_disjoint(spans, 2) != BRACE_OK)
        return BRACE_EINVAL;
    rc = check_device_range(updates_dev, in_bytes, "updates_dev");
    if (rc == BRACE_OK)
        rc = check_device_range(planes_dev, out_bytes, form.matrix);
    if (rc != BRACE_OK)
        return rc;

    const int64_t spans_row = (d + kQuantSpan - 1) / kQuantSpan;
    const brace_tuning_t t = current_tuning();
    const int64_t cus = compute_units() > 0 ? compute_units() : 256;
    // The burst kernels run one block per compute unit at a time (about 2 MiB of input each),
    // so their blocks come in rounds and a thinly filled last round costs as much as a full one.
    // Measured: ahead by 2-5 % with well filled rounds (n = 64, d = 8 M: 4.0 rounds; n = 8,
    // d = 100 M: 5.97; n = 100, d = 25 M: 18.75), behind with ragged ones (n = 50, d = 11 M:
    // 4.3 rounds, 0.447 against 0.408 ms; n = 100, d = 8 M: 6.25 rounds, 601 against 572 us).
    auto round_fill = [&](int64_t spans_per_burst, int64_t* blocks_out) {
        const int64_t blocks = (spans_row + spans_per_burst - 1) / spans_per_burst * n;
        *blocks_out = blocks;
        return (double)blocks / (double)((blocks + cus - 1) / cus * cus);
    };
    auto bursts_pay = [&](int64_t spans_per_burst, int64_t blocks, double fill) {
        return t.stage_writes == 2 || (t.stage_writes == 0 && spans_row >= spans_per_burst &&
                                       blocks >= 4 * cus && fill >= 0.9);
    };
    // Rows of whole 16-byte vectors take the 4-dword form, with bursts of 144 KiB unless the
    // rounds of 128 KiB bursts are clearly fuller.
    const bool wide_ok = aligned_to(updates_dev, 16) && ld % 4 == 0 && d % 4 == 0;
    if (wide_ok) {
        const int kib = form.two_planes ? 1 : 2;                // spans per KiB of burst
        int64_t blocks_a, blocks_b;
        const double fill_a = round_fill(kQuantWideGroup * kib, &blocks_a);
        const double fill_b = round_fill(kQuantGroup * kib, &blocks_b);
        const bool take_a = fill_a + 0.03 >= fill_b;
        const int64_t group = (take_a ? kQuantWideGroup : kQuantGroup) * kib;
        const int64_t blocks = take_a ? blocks_a : blocks_b;
        if (bursts_pay(group, blocks, take_a ? fill_a : fill_b)) {
            if (blocks > 0x7fffffffLL)
                return fail(BRACE_ERANGE, "matrix too large for one launch");
            const size_t lds = (size_t)group / kib * 1024;
            const void* k = form.two_planes
                                ? reinterpret_cast<const void*>(brace_quantize_wide_kernel<true>)
                                : reinterpret_cast<const void*>(brace_quantize_wide_kernel<false>);
            rc = allow_stage_lds(k, kQuantWideBytes);
            if (rc != BRACE_OK)
                return rc;
            const int64_t groups = (spans_row + group - 1) / group;
            if (form.two_planes)
                hipLaunchKernelGGL(brace_quantize_wide_kernel<true>, dim3((unsigned)blocks),
                                   dim3(kQuantBlock), lds, stream, updates_dev, ld, d, planes_dev,
                                   ld_words, row_words, groups, (int)group, 0);
            else
                hipLaunchKernelGGL(brace_quantize_wide_kernel<false>, dim3((unsigned)blocks),
                                   dim3(kQuantBlock), lds, stream, updates_dev, ld, d, planes_dev,
                                   ld_words, row_words, groups, (int)group, up_if_not_negative);
            return check_launch("wide quantize kernel");
        }
    }
    const int spans_per_burst = form.two_planes ? kQuantGroup : kVoteGroup;   // 128 KiB either way
    const int64_t groups = (spans_row + spans_per_burst - 1) / spans_per_burst;    // per row
    int64_t blocks;
    const double fill = round_fill(spans_per_burst, &blocks);
    const bool staged = bursts_pay(spans_per_burst, blocks, fill);
    if (staged) {
        if (blocks > 0x7fffffffLL)
            return fail(BRACE_ERANGE, "matrix too large for one launch");
        constexpr size_t lds2 = (size_t)kQuantGroup * 64 * sizeof(u32x4);
        constexpr size_t lds1 = (size_t)kVoteGroup * 64 * sizeof(u32x2);
        static_assert(lds2 <= kStageBytes && lds1 <= kStageBytes,
                      "the staged planes exceed the LDS opted in to");
        if (form.two_planes) {
            rc = allow_stage_lds(reinterpret_cast<const void*>(brace_quantize_staged_kernel));
            if (rc != BRACE_OK)
                return rc;
            hipLaunchKernelGGL(brace_quantize_staged_kernel, dim3((unsigned)blocks),
                               dim3(kQuantBlock), lds2, stream, updates_dev, ld, d, planes_dev,
                               ld_words, groups);
        } else {
            rc = allow_stage_lds(reinterpret_cast<const void*>(brace_quantize_1bit_staged_kernel));
            if (rc != BRACE_OK)
                return rc;
            hipLaunchKernelGGL(brace_quantize_1bit_staged_kernel, dim3((unsigned)blocks),
                               dim3(kQuantBlock), lds1, stream, updates_dev, ld, d, planes_dev,
                               ld_words, row_words, groups, up_if_not_negative);
        }
        return check_launch("staged quantize kernel");
    }
    const int64_t tasks = spans_row * n;
    const int64_t grid = (tasks + kWaves - 1) / kWaves;
    if (grid > 0x7fffffffLL)
        return fail(BRACE_ERANGE, "matrix too large for one launch");
    if (form.two_planes)
        hipLaunchKernelGGL(brace_quantize_kernel, dim3((unsigned)grid), dim3(kBlock), 0, stream,
                           updates_dev, ld, d, planes_dev, ld_words, spans_row, tasks);
    else
        hipLaunchKernelGGL(brace_quantize_1bit_kernel, dim3((unsigned)grid), dim3(kBlock), 0,
                           stream, updates_dev, ld, d, planes_dev, ld_words, row_words, spans_row,
                           tasks, up_if_not_negative);
    return check_launch("quantize kernel");
}

// Phases II-IV on packed rows over the coordinate range [lo, hi) (the whole vector, one ring
// chunk, or a run of chunks), both forms.
int vote_on_planes(const PlaneForm& form, const uint32_t* planes_dev, int64_t n, int64_t d,
                   int64_t ld_words, int64_t f, const brace_params_t* params, float* out_dev,
                   int64_t lo, int64_t hi, hipStream_t stream)
{
    int rc = check_params(params, n, d, f);
    if (rc != BRACE_OK)
        return rc;
    if (params->rule != 0 || params->sums_dev)
        return fail(BRACE_EINVAL, "the vote on packed signs implements rule 0 and produces no "
                                  "sign-sums");
    rc = check_plane_shape(form, n, d, &ld_words);
    if (rc != BRACE_OK)
        return rc;
    if (d == 0 || hi <= lo)
        return BRACE_OK;
    uint32_t* bits = static_cast<uint32_t*>(params->out_bits_dev);
    if (!planes_dev || !aligned_to(planes_dev, 16))
        return fail(BRACE_EINVAL, "%s must be non-NULL and 16-byte aligned", form.matrix);
    if (!out_dev && !bits)
        return fail(BRACE_EINVAL, "no output: out_dev and out_bits_dev are both NULL");
    if (out_dev && !aligned_to(out_dev, 16))
        return fail(BRACE_EINVAL, "out_dev must be 16-byte aligned for the vote on packed signs");
    if (bits && !aligned_to(bits, 4))
        return fail(BRACE_EINVAL, "out_bits_dev must be 4-byte aligned");
    const int64_t plane_bytes = ((n - 1) * ld_words + form.row_words(d)) * 4;
    const Span spans[] = {{planes_dev, plane_bytes, form.matrix, false},
                          {out_dev, d * 4, "out_dev", true},
                          {bits, ((d + 31) / 32) * 4, "out_bits_dev", true}};
    if (check_disjoint(spans, 3) != BRACE_OK)
        return BRACE_EINVAL;

    const int ni = (int)n;
    const int thresh = threshold_from_lambda(n, params->lambda);
    // S >= thresh as X - Y - c >= 0 on the count slices:
    //   two planes, zero_sign  0: S = P - N    X = P, Y = N, c = thresh
    //   two planes, zero_sign +1: S = n - 2N   N <= floor((n - thresh) / 2)   X = 0, Y = N, c = -M
    //   zero_sign -1, or one bit: S = 2P - n   P >= ceil((n + thresh) / 2)    X = P, Y = 0, c = Q
    // (n + thresh is in [0, 2n + 1]).
    uint32_t mask_p = ~0u, mask_n = ~0u;
    int c = thresh;
    if (form.two_planes && params->zero_sign == 1) {
        mask_p = 0u;
        const int num = ni - thresh;
        c = -(num >= 0 ? num / 2 : -1);
    } else if (!form.two_planes || params->zero_sign == -1) {
        mask_n = 0u;
        c = (ni + thresh + 1) / 2;
    }

    rc = check_device_range(planes_dev, plane_bytes, form.matrix);
    if (rc == BRACE_OK)
        rc = check_device_range(out_dev, d * 4, "out_dev");
    if (rc == BRACE_OK)
        rc = check_device_range(bits, ((d + 31) / 32) * 4, "out_bits_dev");
    if (rc != BRACE_OK)
        return rc;

    // Whole vector: the slice kernel covers everything, ragged end included.  A sub-range is
    // split like the float path: whole 1024-coordinate groups go through the slice kernel on
    // offset pointers, the coordinates before and after them are voted one per thread.
    const bool whole = lo == 0 && hi == d;
    int64_t lo_a = whole ? 0 : (lo + kGroup - 1) / kGroup * kGroup;
    int64_t hi_a = whole ? d : hi / kGroup * kGroup;
    if (lo_a >= hi_a)
        lo_a = hi_a = lo;          // no body: the whole range is edge
    if (hi_a > lo_a) {
        const int64_t d_body = hi_a - lo_a;
        const int64_t cols4 = whole ? form.row_words(d) / 4 : d_body / form.coords_per_load;
        // A wave walks `seq` neighbouring 64-column groups one after the other: up to 3, so
        // that about 7 waves remain for every compute unit (6,104 groups: 3 per wave, 97 us
        // against 102 us with 1 and 100 us with 4; 3,052 groups: 2 per wave, 49.7 us against
        // 51.2 us with 1 and 54.4 us with 3).
        const int64_t groups64 = (cols4 + 63) / 64;
        const int64_t cus = compute_units() > 0 ? compute_units() : 256;
        const int64_t fit = (2 * groups64 + 7 * cus) / (14 * cus);      // groups / (7 cus), rounded
        const int seq = fit >= 3 ? 3 : fit >= 1 ? (int)fit : 1;
        const int64_t grid = (groups64 + (int64_t)kWaves * seq - 1) / ((int64_t)kWaves * seq);
        if (grid > 0x7fffffffLL)
            return fail(BRACE_ERANGE, "vector too long for one launch");
        // Bit-words go to the caller's bit array when there is one, else they are parked in out_dev.
        uint32_t* dst = bits ? bits + lo_a / 32 : reinterpret_cast<uint32_t*>(out_dev + lo_a);
        const int parked = bits ? 0 : 1;
        const u32x4* rows = reinterpret_cast<const u32x4*>(planes_dev) + lo_a / form.coords_per_load;
        const int64_t ld4 = ld_words / 4;
        const bool wide = n > 255;             // 8 counter bits hold up to 255 clients
        if (form.two_planes) {
            if (!wide)
                hipLaunchKernelGGL(brace_vote_packed_kernel<8>, dim3((unsigned)grid), dim3(kBlock), 0,
                                   stream, rows, ld4, ni, cols4, seq, mask_p, mask_n, c, dst, parked,
                                   d_body);
            else
                hipLaunchKernelGGL(brace_vote_packed_kernel<16>, dim3((unsigned)grid), dim3(kBlock), 0,
                                   stream, rows, ld4, ni, cols4, seq, mask_p, mask_n, c, dst, parked,
                                   d_body);
        } else {
            if (!wide)
                hipLaunchKernelGGL(brace_vote_1bit_kernel<8>, dim3((unsigned)grid), dim3(kBlock), 0,
                                   stream, rows, ld4, ni, cols4, seq, c, dst, parked, d_body);
            else
                hipLaunchKernelGGL(brace_vote_1bit_kernel<16>, dim3((unsigned)grid), dim3(kBlock), 0,
                                   stream, rows, ld4, ni, cols4, seq, c, dst, parked, d_body);
        }
        rc = check_launch("packed vote kernel");
        if (rc != BRACE_OK)
            return rc;
        if (out_dev) {
            const int64_t groups = (d_body + kGroup - 1) / kGroup;
            const int64_t egrid = (groups + kWaves - 1) / kWaves;
            hipLaunchKernelGGL(brace_expand_kernel, dim3((unsigned)egrid), dim3(kBlock), 0, stream,
                               out_dev, static_cast<const uint32_t*>(bits), lo_a, groups, hi_a);
            rc = check_launch("expand kernel");
            if (rc != BRACE_OK)
                return rc;
        }
    }
    if (whole)
        return BRACE_OK;
    int64_t hi_ext = hi;
    if (bits && hi == d)
        hi_ext = (d + 31) & ~(int64_t)31;          // the last word's padding bits are zeroed
    const int64_t edge = (lo_a - lo) + (hi_ext - hi_a);
    if (edge > 0) {
        const int64_t tgrid = (edge + kBlock - 1) / kBlock;
        if (form.two_planes)
            hipLaunchKernelGGL(brace_packed_edge_kernel, dim3((unsigned)tgrid), dim3(kBlock), 0,
                               stream, planes_dev, ld_words, ni, thresh, params->zero_sign, out_dev,
                               bits, lo, lo_a, hi_a, hi, hi_ext);
        else
            hipLaunchKernelGGL(brace_1bit_edge_kernel, dim3((unsigned)tgrid), dim3(kBlock), 0,
                               stream, planes_dev, ld_words, ni, thresh, out_dev, bits, lo, lo_a,
                               hi_a, hi, hi_ext);
        rc = check_launch("packed edge kernel");
    }
    return rc;
}

}  // namespace

extern "C" {

int64_t brace_packed_row_words(int64_t d)
{
    if (d < 0)
        return 0;
    int64_t w = d / 32 + (d % 32 != 0);        // no overflow for any d
    w += w & 1;
    return 2 * w;
}

int64_t brace_packed_row_pitch(int64_t d)
{
    return roundup_words(brace_packed_row_words(d), 32);
}

int64_t brace_1bit_row_words(int64_t d)
{
    if (d < 0)
        return 0;
    return roundup_words(d / 32 + (d % 32 != 0), 4);
}

int64_t brace_1bit_row_pitch(int64_t d)
{
    return roundup_words(brace_1bit_row_words(d), 32);
}

int brace_quantize(const float* updates_dev, int64_t n, int64_t d, int64_t ld,
                   uint32_t* signs_dev, int64_t ld_words, void* hip_stream)
{
    return quantize_to_planes(kTwoPlanes, updates_dev, n, d, ld, 0, signs_dev, ld_words,
                              static_cast<hipStream_t>(hip_stream));
}

int brace_quantize_1bit(const float* updates_dev, int64_t n, int64_t d, int64_t ld, int32_t zero_sign,
                        uint32_t* votes_dev, int64_t ld_words, void* hip_stream)
{
    if (zero_sign != 1 && zero_sign != -1)
        return fail(BRACE_EINVAL, "the one-bit form needs zero_sign = +1 or -1 (a zero that abstains "
                                  "needs the two-plane form)");
    return quantize_to_planes(kOneBit, updates_dev, n, d, ld, zero_sign == 1 ? 1 : 0, votes_dev,
                              ld_words, static_cast<hipStream_t>(hip_stream));
}

int brace_vote_packed(const uint32_t* signs_dev, int64_t n, int64_t d, int64_t ld_words, int64_t f,
                      const brace_params_t* params, float* out_dev, void* hip_stream)
{
    return vote_on_planes(kTwoPlanes, signs_dev, n, d, ld_words, f, params, out_dev, 0,
                          d < 0 ? 0 : d, static_cast<hipStream_t>(hip_stream));
}

int brace_vote_packed_chunks(const uint32_t* signs_dev, int64_t n, int64_t d, int64_t ld_words,
                             int64_t f, int64_t chunk_begin, int64_t chunk_end,
                             const brace_params_t* params, float* out_dev, void* hip_stream)
{
    int64_t lo, hi;
    const int rc = chunk_run_range(n, d, chunk_begin, chunk_end, &lo, &hi);
    if (rc != BRACE_OK)
        return rc;
    return vote_on_planes(kTwoPlanes, signs_dev, n, d, ld_words, f, params, out_dev, lo, hi,
                          static_cast<hipStream_t>(hip_stream));
}

int brace_vote_packed_chunk(const uint32_t* signs_dev, int64_t n, int64_t d, int64_t ld_words,
                            int64_t f, int64_t chunk, const brace_params_t* params, float* out_dev,
                            void* hip_stream)
{
    if (n >= 1 && (chunk < 0 || chunk >= n))
        return fail(BRACE_ERANGE, "chunk %lld outside [0, %lld)", (long long)chunk, (long long)n);
    return brace_vote_packed_chunks(signs_dev, n, d, ld_words, f, chunk, chunk + 1, params, out_dev,
                                    hip_stream);
}

int brace_vote_1bit(const uint32_t* votes_dev, int64_t n, int64_t d, int64_t ld_words, int64_t f,
                    const brace_params_t* params, float* out_dev, void* hip_stream)
{
    return vote_on_planes(kOneBit, votes_dev, n, d, ld_words, f, params, out_dev, 0, d < 0 ? 0 : d,
                          static_cast<hipStream_t>(hip_stream));
}

int brace_vote_1bit_chunks(const uint32_t* votes_dev, int64_t n, int64_t d, int64_t ld_words,
                           int64_t f, int64_t chunk_begin, int64_t chunk_end,
                           const brace_params_t* params, float* out_dev, void* hip_stream)
{
    int64_t lo, hi;
    const int rc = chunk_run_range(n, d, chunk_begin, chunk_end, &lo, &hi);
    if (rc != BRACE_OK)
        return rc;
    return vote_on_planes(kOneBit, votes_dev, n, d, ld_words, f, params, out_dev, lo, hi,
                          static_cast<hipStream_t>(hip_stream));
}

int brace_consensus_sums(const int16_t* parts_dev, int64_t g, int64_t d, int64_t ld,
                         const brace_params_t* params, float* out_dev, void* hip_stream)
{
    if (g < 1)
        return fail(BRACE_EINVAL, "need g >= 1 and d >= 0");
    if (g > BRACE_MAX_CLIENTS)
        return fail(BRACE_ERANGE, "g = %lld exceeds BRACE_MAX_CLIENTS", (long long)g);
    {
        const int prc = check_params(params, g, d, 0);      // g stands in for the row count
        if (prc != BRACE_OK)
            return prc;
    }
    if (params->rule != 0 || params->sums_dev)
        return fail(BRACE_EINVAL, "the consensus of partial sums implements rule 0 and produces "
                                  "no sign-sums");
    if (ld == 0)
        ld = d;
    if (ld < d)
        return fail(BRACE_EINVAL, "ld = %lld is smaller than d = %lld", (long long)ld, (long long)d);
    if (check_extent(g, ld, 4) != BRACE_OK)
        return BRACE_ERANGE;
    if (d == 0)
        return BRACE_OK;
    uint32_t* bits = static_cast<uint32_t*>(params->out_bits_dev);
    if (!parts_dev || !aligned_to(parts_dev, 2))
        return fail(BRACE_EINVAL, "parts_dev must be non-NULL and 2-byte aligned");
    if (!out_dev && !bits)
        return fail(BRACE_EINVAL, "no output: out_dev and out_bits_dev are both NULL");
    if ((out_dev && !aligned_to(out_dev, 4)) || (bits && !aligned_to(bits, 4)))
        return fail(BRACE_EINVAL, "out_dev and out_bits_dev must be 4-byte aligned");
    {
        const Span spans[] = {{parts_dev, ((g - 1) * ld + d) * 2, "parts_dev", false},
                              {out_dev, d * 4, "out_dev", true},
                              {bits, ((d + 31) / 32) * 4, "out_bits_dev", true}};
        if (check_disjoint(spans, 3) != BRACE_OK)
            return BRACE_EINVAL;
    }
    int rc = check_device_range(parts_dev, ((g - 1) * ld + d) * 2, "parts_dev");
    if (rc == BRACE_OK)
        rc = check_device_range(out_dev, d * 4, "out_dev");
    if (rc == BRACE_OK)
        rc = check_device_range(bits, ((d + 31) / 32) * 4, "out_bits_dev");
    if (rc != BRACE_OK)
        return rc;

    // |S| <= g * 32767 < 2^30, so thresholds beyond that range saturate.
    const int thresh = threshold_from_lambda((int64_t)1 << 30, params->lambda);

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const bool wide = aligned_to(parts_dev, 16) && (ld % 8 == 0 || g == 1) &&
                      (!out_dev || aligned_to(out_dev, 16));
    const int64_t octets = wide ? d / 8 : 0;
    if (octets > 0) {
        const int64_t grid = (octets + kBlock - 1) / kBlock;
        if (grid > 0x7fffffffLL)
            return fail(BRACE_ERANGE, "vector too long for one launch");
        hipLaunchKernelGGL(brace_consensus_kernel, dim3((unsigned)grid), dim3(kBlock), 0, stream,
                           parts_dev, ld, (int)g, octets, thresh, out_dev,
                           reinterpret_cast<uint8_t*>(bits));
        rc = check_launch("consensus kernel");
        if (rc != BRACE_OK)
            return rc;
    }
    const int64_t lo = octets * 8;
    if (lo < d) {
        const int64_t tgrid = (d - lo + kBlock - 1) / kBlock;
        if (tgrid > 0x7fffffffLL)
            return fail(BRACE_ERANGE, "vector too long for one launch");
        hipLaunchKernelGGL(brace_consensus_tail_kernel, dim3((unsigned)tgrid), dim3(kBlock), 0, stream,
                           parts_dev, ld, (int)g, lo, d, thresh, out_dev, bits);
        rc = check_launch("consensus tail kernel");
        if (rc != BRACE_OK)
            return rc;
    }
    if (bits && (d & 31)) {
        hipLaunchKernelGGL(brace_clear_pad_kernel, dim3(1), dim3(64), 0, stream, bits, d);
        rc = check_launch("pad kernel");
    }
    return rc;
}

void brace_rar_params_init(brace_rar_params_t* params)
{
    if (!params)
        return;
    std::memset(params, 0, sizeof(*params));
    params->struct_size = sizeof(brace_rar_params_t);
}

int brace_rar_aggregate(const float* updates_dev, int64_t n, int64_t d,
                        const brace_rar_params_t* params, float* out_dev, void* hip_stream)
{
    int64_t ld;
    double scale;
    const int rc = validate_rar(updates_dev, n, d, params, out_dev, &ld, &scale);
    if (rc != BRACE_OK)
        return rc;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (params->order == 1)
        return launch_ring_sum(updates_dev, n, d, ld, params->mean, out_dev, 0, d, stream);
    return launch_sum(updates_dev, n, d, ld, scale, out_dev, 0, d, stream);
}

int brace_rar_aggregate_chunk(const float* updates_dev, int64_t n, int64_t d, int64_t chunk,
                              const brace_rar_params_t* params, float* out_dev, void* hip_stream)
{
    int64_t ld;
    double scale;
    int rc = validate_rar(updates_dev, n, d, params, out_dev, &ld, &scale);
    if (rc != BRACE_OK)
        return rc;
    int64_t lo, hi;
    rc = brace_chunk_range(n, d, chunk, &lo, &hi);
    if (rc != BRACE_OK)
        return rc;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (params->order == 1)
        return launch_ring_sum(updates_dev, n, d, ld, params->mean, out_dev, lo, hi, stream);
    return launch_sum(updates_dev, n, d, ld, scale, out_dev, lo, hi, stream);
}

const char* brace_last_error(void)
{
    return g_err;
}

int brace_set_tuning(const brace_tuning_t* tuning)
{
    if (!tuning) {
        store_tuning(default_tuning());
        return BRACE_OK;
    }
    if (tuning->struct_size != sizeof(brace_tuning_t))
        return fail(BRACE_EINVAL, "tuning->struct_size is %u, expected %zu", tuning->struct_size,
                    sizeof(brace_tuning_t));
    const int v = tuning->vec, c = tuning->cols, u = tuning->unroll;
    if (!(v == 0 || v == 1 || v == 2 || v == 4) ||
        !(c == 0 || c == 1 || c == 2 || c == 4 || c == 8) ||
        !(u == 0 || u == 2 || u == 4 || u == 8) || tuning->split_writes < 0 || tuning->split_writes > 2 || tuning->rowsplit < 0 ||
        tuning->rowsplit > 2 || tuning->stage_writes < 0 || tuning->stage_writes > 2)
        return fail(BRACE_EINVAL, "tuning: vec in {0,1,2,4}, cols in {0,1,2,4,8}, unroll in {0,2,4,8}, "
                    "split_writes, rowsplit and stage_writes in {0,1,2}");
    store_tuning(*tuning);
    return BRACE_OK;
}

int brace_get_tuning(brace_tuning_t* tuning)
{
    if (!tuning)
        return fail(BRACE_EINVAL, "tuning is NULL");
    *tuning = current_tuning();
    return BRACE_OK;
}

int brace_init_device(void)
{
    // Everything a first call would do on the host besides launching: the device query, the
    // loading of each translation unit's code object (triggered by asking for a kernel's
    // attributes) and the LDS opt-in of every burst-writing kernel.
    (void)compute_units();
    const void* one_per_unit[] = {
        reinterpret_cast<const void*>(brace_vote_pick_v1(1, 2, 1, 0, 0)),
        reinterpret_cast<const void*>(brace_vote_pick_v2(1, 2, 1, 0, 0)),
        reinterpret_cast<const void*>(brace_vote_pick_v4(1, 2, 1, 0, 0)),
        reinterpret_cast<const void*>(brace_sum_pick_v1(1, 2, 1, 0, 0)),
        reinterpret_cast<const void*>(brace_sum_pick_v2(1, 2, 1, 0, 0)),
        reinterpret_cast<const void*>(brace_sum_pick_v4(1, 2, 1, 0, 0)),
        reinterpret_cast<const void*>(brace_expand_kernel),
    };
    for (const void* k : one_per_unit) {
        hipFuncAttributes fa;
        const hipError_t err = hipFuncGetAttributes(&fa, k);
        if (err != hipSuccess) {
            (void)hipGetLastError();
            return fail(BRACE_EHIP, "cannot load a kernel: %s", hipGetErrorString(err));
        }
    }
    for (int v = 2; v <= 4; v += 2)
        for (int cols = kStageColsNarrow; cols <= kStageColsWide; cols += kStageColsWide - kStageColsNarrow)
            for (int pipe = 0; pipe <= 1; ++pipe) {
                int rc = allow_stage_lds(
                    reinterpret_cast<const void*>(brace_vote_pick_staged(v, cols, pipe)));
                if (rc == BRACE_OK)
                    rc = allow_stage_lds(
                        reinterpret_cast<const void*>(brace_sum_pick_staged(v, cols, pipe)));
                if (rc == BRACE_OK)
                    rc = allow_stage_lds(reinterpret_cast<const void*>(brace_ring_pick(v, cols, 1)));
                if (rc != BRACE_OK)
                    return rc;
            }
    int rc = allow_stage_lds(reinterpret_cast<const void*>(brace_quantize_staged_kernel));
    if (rc == BRACE_OK)
        rc = allow_stage_lds(reinterpret_cast<const void*>(brace_quantize_1bit_staged_kernel));
    if (rc == BRACE_OK)
        rc = allow_stage_lds(reinterpret_cast<const void*>(brace_quantize_wide_kernel<true>),
                             kQuantWideBytes);
    if (rc == BRACE_OK)
        rc = allow_stage_lds(reinterpret_cast<const void*>(brace_quantize_wide_kernel<false>),
                             kQuantWideBytes);
    if (rc != BRACE_OK)
        return rc;
    uint32_t* ws = nullptr;
    return scratch_of_current_device(&ws);
}

int brace_set_pointer_checks(int32_t enabled)
{
    g_pointer_checks = enabled != 0;
    return BRACE_OK;
}

int brace_probe_read(const void* src_dev, int64_t nbytes, int32_t nontemporal, void* sink_dev,
                     void* hip_stream)
{
    if (!src_dev || !sink_dev || nbytes < 0 || (nbytes & 15) || !aligned_to(src_dev, 16) ||
        !aligned_to(sink_dev, 4))
        return fail(BRACE_EINVAL, "probe_read: need 16-byte aligned src, nbytes %% 16 == 0, a sink");
    const int64_t nvec = nbytes / 16;
    if (nvec == 0)
        return BRACE_OK;
    const int64_t per_block = 8 * kBlock * 4;                 // 128 KiB per block
    const int64_t grid = (nvec + per_block - 1) / per_block;
    if (grid > 0x7fffffffLL)
        return fail(BRACE_ERANGE, "probe_read: buffer too large for one launch");
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (nontemporal)
        hipLaunchKernelGGL(probe_read_kernel<true>, dim3((unsigned)grid), dim3(kBlock), 0, st,
                           static_cast<const f32x4*>(src_dev), nvec, per_block,
                           static_cast<float*>(sink_dev));
    else
        hipLaunchKernelGGL(probe_read_kernel<false>, dim3((unsigned)grid), dim3(kBlock), 0, st,
                           static_cast<const f32x4*>(src_dev), nvec, per_block,
                           static_cast<float*>(sink_dev));
    const hipError_t err = hipGetLastError();
    if (err != hipSuccess)
        return fail(BRACE_EHIP, "probe_read launch failed: %s", hipGetErrorString(err));
    return BRACE_OK;
}

int brace_probe_copy(void* dst_dev, const void* src_dev, int64_t nbytes, void* hip_stream)
{
    if (!src_dev || !dst_dev || nbytes < 0 || (nbytes & 15) || !aligned_to(src_dev, 16) ||
        !aligned_to(dst_dev, 16))
        return fail(BRACE_EINVAL, "probe_copy: need 16-byte aligned buffers, nbytes %% 16 == 0");
    const int64_t nvec = nbytes / 16;
    if (nvec == 0)
        return BRACE_OK;
    const int64_t per_block = 4 * kBlock * 4;                 // 64 KiB per block
    const int64_t grid = (nvec + per_block - 1) / per_block;
    if (grid > 0x7fffffffLL)
        return fail(BRACE_ERANGE, "probe_copy: buffer too large for one launch");
    hipLaunchKernelGGL(probe_copy_kernel, dim3((unsigned)grid), dim3(kBlock), 0,
                       static_cast<hipStream_t>(hip_stream), static_cast<f32x4*>(dst_dev),
                       static_cast<const f32x4*>(src_dev), nvec, per_block);
    const hipError_t err = hipGetLastError();
    if (err != hipSuccess)
        return fail(BRACE_EHIP, "probe_copy launch failed: %s", hipGetErrorString(err));
    return BRACE_OK;
}

}  // extern "C"
