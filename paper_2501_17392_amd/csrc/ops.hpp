// The per-coordinate operations plugged into the streaming skeleton.
//
//   VoteOp  BRACE: sign quantisation (Sec. 3 Phase I), sign-sum over the clients
//           (Phase II), consensus map of Eq. (1) (Phase III), result placed at the
//           coordinate's position in the global update (Phase IV).
//   SumOp   the operation BRACE replaces: the plain ring-all-reduce sum of Sec. 2.2, or the
//           Mean rule of Sec. 2.1 when scaled by 1/n.

#pragma once

#include "stream_kernel.hpp"

namespace brace_dev {

constexpr int kGroup = 1024;                // coordinates whose 32 bit-words fill one 128 B line

// Where the bit-word of coordinates [32j, 32j+32) lives when the floats' own buffer is used
// as scratch: the 32 words of a 1024-coordinate group sit in the first 128 bytes of the
// 4 KiB that the group expands to, so the expansion of a group only overwrites its own words.
__device__ __forceinline__ int64_t scratch_word(int64_t k)
{
    return (k & ~(int64_t)(kGroup - 1)) + ((k & (kGroup - 1)) >> 5);
}

struct VoteOp {
    float* out;             // d floats, may be null
    uint32_t* bits;         // packed result, may be null
    int16_t* sums;          // sign-sums, may be null
    float* w;               // model parameters updated in place, may be null
    float eta;              // learning rate of the fused update w <- w - eta * result
    int32_t thresh;         // result is +1 iff S >= thresh  (thresh = floor(lambda) + 1)
    int32_t zero_sign;      // vote of +-0 and NaN
    int32_t split;          // 1: the body emits bit-words only (a second kernel writes the floats)
    int32_t tie_zero;       // 1: majority rule, S == 0 gives 0 (thresh is 1 then)
    int32_t stage_sums;     // 1: the staged kernel delivers the sign-sums (and nothing else)

    // Two counters per coordinate: clients voting +1 and clients voting -1.
    struct State { int pos, neg; };

    __device__ static __forceinline__ void init(State& s) { s.pos = 0; s.neg = 0; }

    // Phase I + II: compares (not a sign-bit test) so that -0.0 and NaN land in neither count.
    __device__ static __forceinline__ void add(State& s, float v)
    {
        s.pos += (v > 0.0f) ? 1 : 0;
        s.neg += (v < 0.0f) ? 1 : 0;
    }

    __device__ static __forceinline__ void merge(State& s, const State& o)
    {
        s.pos += o.pos;
        s.neg += o.neg;
    }

    // Phase III: Eq. (1), or the three-valued majority sign.
    __device__ __forceinline__ float decide(int s) const
    {
        const float v = (s >= thresh) ? 1.0f : -1.0f;
        return (tie_zero && s == 0) ? 0.0f : v;
    }

    __device__ __forceinline__ int sign_sum(const State& s, int n) const
    {
        return s.pos - s.neg + zero_sign * (n - s.pos - s.neg);
    }

    template <int V, bool NT>
    __device__ __forceinline__ void store_body(int64_t k, const State (&st)[V], int lane, int n) const
    {
        typedef typename Vec<V>::type VT;
        int s[V];
        uint32_t mybits = 0;
#pragma unroll
        for (int e = 0; e < V; ++e) {
            s[e] = sign_sum(st[e], n);
            mybits |= (s[e] >= thresh ? 1u : 0u) << e;             // Phase III, Eq. (1)
        }
        if (out && !split) {
            VT o;
#pragma unroll
            for (int e = 0; e < V; ++e)
                set_elem<V>(o, e, decide(s[e]));
            store_vec<NT>(reinterpret_cast<VT*>(out + k), o);
        }
        if (w && !split) {
            // Fused consumer of the result (Sec. 2.1; App. A update rule): every coordinate
            // moves by exactly eta, against the sign of the vote.
            VT wv = load_vec<V, NT>(w + k);
#pragma unroll
            for (int e = 0; e < V; ++e)
                set_elem<V>(wv, e, elem<V>(wv, e) - eta * decide(s[e]));
            store_vec<NT>(reinterpret_cast<VT*>(w + k), wv);
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
        if (bits || split) {
            // 32/V lanes share one 32-bit word; OR them together, the first lane stores.
            constexpr int L = 32 / V;
            uint32_t word = mybits << (V * (lane & (L - 1)));
#pragma unroll
            for (int m = 1; m < L; m <<= 1)
                word |= (uint32_t)__shfl_xor((int)word, m, 64);
            if ((lane & (L - 1)) == 0) {
                if (bits)
                    bits[k >> 5] = word;
                else
                    reinterpret_cast<uint32_t*>(out)[scratch_word(k)] = word;
            }
        }
    }

    // Bits are merged atomically: a 32-bit word can be shared with a neighbouring chunk's call.
    __device__ __forceinline__ void store_edge(int64_t k, const State& st, int n) const
    {
        const int s = sign_sum(st, n);
        const bool up = s >= thresh;
        if (out)
            out[k] = decide(s);
        if (w)
            w[k] = w[k] - eta * decide(s);
        if (sums)
            sums[k] = (int16_t)s;
        if (bits) {
            if (up)
                atomicOr(&bits[k >> 5], 1u << (k & 31));
            else
                atomicAnd(&bits[k >> 5], ~(1u << (k & 31)));
        }
    }

    // Padding bits of the last 32-bit word are zero.
    __device__ __forceinline__ void pad_edge(int64_t k) const
    {
        if (bits)
            atomicAnd(&bits[k >> 5], ~(1u << (k & 31)));
    }

    // Staged variant: the float result, the in-place model update, or (stage_sums) the
    // sign-sums alone -- the partial sums of Share-Reduce, exact in a float up to 2^24.
    // For the update the old parameters of a tile are requested before its rows, so that
    // they arrive under the row stream and the burst at the end is write-only.
    template <int V>
    __device__ __forceinline__ typename Vec<V>::type stage_prefetch(int64_t k) const
    {
        typename Vec<V>::type zero = {};
        return w ? load_vec<V, true>(w + k) : zero;
    }

    __device__ __forceinline__ float stage_value(const State& st, int n, float old) const
    {
        const int s = sign_sum(st, n);
        if (stage_sums)
            return (float)s;
        return w ? old - eta * decide(s) : decide(s);
    }

    __device__ __forceinline__ void flush4(int64_t k, f32x4 v) const
    {
        if (stage_sums) {
            typename IVec<4>::type s4;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                s4[e] = (short)v[e];
            __builtin_nontemporal_store(s4, reinterpret_cast<typename IVec<4>::type*>(sums + k));
            return;
        }
        __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(w ? w + k : out + k));
    }
};

struct SumOp {
    float* out;             // d floats
    double scale;           // 1 for the ring-all-reduce sum, 1/n for the Mean rule

    // fp64 accumulator: the fp32 result is then the correctly rounded sum up to one double
    // rounding, whatever the cancellation between benign and Byzantine rows.
    struct State { double acc; };

    __device__ static __forceinline__ void init(State& s) { s.acc = 0.0; }
    __device__ static __forceinline__ void add(State& s, float v) { s.acc += (double)v; }
    __device__ static __forceinline__ void merge(State& s, const State& o) { s.acc += o.acc; }

    template <int V, bool NT>
    __device__ __forceinline__ void store_body(int64_t k, const State (&st)[V], int, int) const
    {
        typedef typename Vec<V>::type VT;
        VT o;
#pragma unroll
        for (int e = 0; e < V; ++e)
            set_elem<V>(o, e, (float)(st[e].acc * scale));
        store_vec<NT>(reinterpret_cast<VT*>(out + k), o);
    }

    __device__ __forceinline__ void store_edge(int64_t k, const State& st, int) const
    {
        out[k] = (float)(st.acc * scale);
    }

    __device__ __forceinline__ void pad_edge(int64_t) const {}

    template <int V>
    __device__ __forceinline__ typename Vec<V>::type stage_prefetch(int64_t) const
    {
        typename Vec<V>::type zero = {};
        return zero;
    }

    __device__ __forceinline__ float stage_value(const State& st, int, float) const
    {
        return (float)(st.acc * scale);
    }

    __device__ __forceinline__ void flush4(int64_t k, f32x4 v) const
    {
        __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(out + k));
    }
};

}  // namespace brace_dev

// One translation unit per (op, load width) instantiates its share of the kernels.
brace_dev::stream_staged_kernel_t<brace_dev::VoteOp> brace_vote_pick_staged(int v, int cols, int pipe);
brace_dev::stream_staged_kernel_t<brace_dev::SumOp> brace_sum_pick_staged(int v, int cols, int pipe);
brace_dev::ring_sum_kernel_t brace_ring_pick(int v, int cols, int staged);
brace_dev::stream_kernel_t<brace_dev::VoteOp> brace_vote_pick_v1(int cols, int ru, int nt, int pipe,
                                                                 int rs);
brace_dev::stream_kernel_t<brace_dev::VoteOp> brace_vote_pick_v2(int cols, int ru, int nt, int pipe,
                                                                 int rs);
brace_dev::stream_kernel_t<brace_dev::VoteOp> brace_vote_pick_v4(int cols, int ru, int nt, int pipe,
                                                                 int rs);
brace_dev::stream_kernel_t<brace_dev::SumOp> brace_sum_pick_v1(int cols, int ru, int nt, int pipe,
                                                                 int rs);
brace_dev::stream_kernel_t<brace_dev::SumOp> brace_sum_pick_v2(int cols, int ru, int nt, int pipe,
                                                                 int rs);
brace_dev::stream_kernel_t<brace_dev::SumOp> brace_sum_pick_v4(int cols, int ru, int nt, int pipe,
                                                                 int rs);
