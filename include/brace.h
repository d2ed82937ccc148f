/*
 * brace.h -- C ABI of the MI355X (gfx950) BRACE robust chunk aggregation library.
 *
 * BRACE (Byzantine-robust ring-all-reduce) replaces the summation inside
 * ring-all-reduce by a per-coordinate vote: every client quantises its update
 * to its element-wise sign (Sec. 3, Phase I), the ring adds the signs chunk by
 * chunk (Phase II, Share-Reduce), the owner of each chunk maps the sign-sum S
 * to +1 if S > lambda and to -1 otherwise (Phase III, Eq. (1); App. A writes
 * the same map as 2*I(S > lambda) - 1), and the +-1 chunks are circulated until
 * every client holds the same full vector (Phase IV, Share-Only).
 *
 * Here all n clients' flattened updates are resident on one GPU.  The ring is
 * chunk ownership and indexing: the gradient is split in n about equally long
 * sub-vectors (Sec. 2.2), each chunk is aggregated across the n clients'
 * copies, and the aggregated chunks are written back ("gathered") at their
 * place in the global update.
 *
 * Conventions
 *   - Pointers named *_dev are DEVICE pointers; the caller owns every buffer.
 *     The library allocates nothing and the calls declared here keep no state
 *     besides the last error text (thread-local).  Launch tuning, the switch of the
 *     host-side pointer checks and the measurement aids are process-wide and live in
 *     brace_tuning.h; no caller of the method needs them.
 *   - Buffers of one call must not overlap each other, with one exception noted at
 *     brace_aggregate; a call that sees an overlap returns BRACE_EINVAL.
 *   - Before a call enqueues anything, every buffer is checked on the host: it must be
 *     device memory known to the HIP runtime and the bytes the call will touch (from the
 *     sizes given) must lie inside the allocation that holds the pointer; otherwise the
 *     call returns BRACE_EINVAL and launches nothing.
 *   - Calls validate on the host, enqueue on `hip_stream` (a hipStream_t passed
 *     as void*; NULL is the default stream) and return without synchronising.
 *     BRACE_OK therefore means "validated and enqueued".
 *   - Errors are return codes; nothing is thrown across this boundary.
 *     brace_last_error() gives a short text for the last failure on this thread.
 *   - Coordinates, chunks and clients are 0-indexed.
 */
#ifndef BRACE_H
#define BRACE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum brace_status {
    BRACE_OK = 0,
    BRACE_EINVAL = 1,   /* NULL/invalid argument, bad struct_size, bad alignment        */
    BRACE_ERANGE = 2,   /* chunk outside [0, n), n above BRACE_MAX_CLIENTS             */
    BRACE_EHIP = 3      /* a HIP runtime call failed (text in brace_last_error)         */
} brace_status_t;

#define BRACE_MAX_CLIENTS 32767   /* sign-sums are delivered as int16 */

/*
 * Parameters of the consensus map (Sec. 3 Phase III, Eq. (1)) and optional outputs.
 * Fill with brace_params_init() and then change what you need.
 */
typedef struct brace_params {
    uint32_t struct_size;  /* sizeof(brace_params_t); checked                                    */
    float    lambda;       /* threshold of Eq. (1); any finite real.  Sec. 5.1 uses 5.            */
    int32_t  zero_sign;    /* vote cast by +0, -0 and NaN: 0 (default), +1 or -1.  The paper does  */
                           /* not define sign(0); infinities and denormals keep their sign.       */
    int32_t  rule;         /* 0: Eq. (1).  1: plain majority sign(S) with ties S = 0 -> 0, i.e.    */
                           /* signSGD run over the same four phases (Sec. 5.2); lambda is then     */
                           /* ignored, the result is in {-1, 0, +1} and has no 1-bit form          */
                           /* (out_bits_dev must be NULL).  Majority with ties -> -1 is rule 0     */
                           /* with lambda = 0.                                                     */
    int64_t  ld;           /* row pitch of updates_dev in elements; 0 means ld = d.  Any pitch >= d */
                           /* works; a multiple of 32 (rows on whole 128-byte lines) avoids re-     */
                           /* fetching the lines that rows of another phase cut (about 3 %).        */
    void*    out_bits_dev; /* optional 1-bit-per-dimension result (the Share-Only wire format of   */
                           /* Sec. 3): bit j of byte b is coordinate 8b+j, 1 <=> +1.  Must be      */
                           /* 4-byte aligned and hold 4*ceil(d/32) bytes; bits past d are zeroed.  */
    int16_t* sums_dev;     /* optional sign-sums S[k] (end state of Share-Reduce), d entries       */
} brace_params_t;

/* struct_size, lambda = 5, zero_sign = 0, ld = 0, no optional outputs. */
void brace_params_init(brace_params_t* params);

/*
 * Communication volume of one aggregation, the quantity the paper compares (Sec. 2.1,
 * Sec. 2.2, Sec. 3 and Table 1), for gradients of d dimensions at m bits each over n clients:
 *   BRACE_COST_SERVER_CLIENT    m*n*d            what the server of a server-client round receives
 *   BRACE_COST_RING_ALL_REDUCE  2*m*d*(n-1)/n    what one client sends in plain ring-all-reduce
 *   BRACE_COST_BRACE            d*(n-1)*(m+1)/n  what one client sends in BRACE: m-bit partial
 *                                                sums in Share-Reduce, 1 bit in Share-Only
 * Pure host arithmetic.  EINVAL unless 1 <= m <= 64, n >= 1, d >= 0 and the scheme is known.
 */
enum { BRACE_COST_SERVER_CLIENT = 0, BRACE_COST_RING_ALL_REDUCE = 1, BRACE_COST_BRACE = 2 };
int brace_comm_cost(int32_t scheme, int64_t m, int64_t n, int64_t d, double* bits_per_client);

/*
 * Aggregate the whole update: Eq. (1) on every coordinate of every ring chunk,
 * gathered into out_dev[0 .. d).
 *
 *   updates_dev  n rows of d fp32 values, row i (client i) at updates_dev + i*ld; read once.
 *   n            number of clients, 1 .. BRACE_MAX_CLIENTS
 *   d            dimension, >= 0; d < n is allowed (some chunks are empty).  d = 0 is a no-op
 *                that touches no buffer (pointers may then be NULL).
 *   f            number of Byzantine clients the caller assumes, 0 <= f <= n.  Validated only:
 *                Eq. (1) does not depend on it.
 *   out_dev      d fp32 values, each exactly +1.0f or -1.0f.  May be NULL when out_bits_dev or
 *                sums_dev is given.
 * updates_dev, out_dev, out_bits_dev and sums_dev must be pairwise disjoint (checked on the
 * extents the call addresses: (n-1)*ld + d floats, d floats, 4*ceil(d/32) bytes, d int16).
 */
int brace_aggregate(const float* updates_dev, int64_t n, int64_t d, int64_t f,
                    const brace_params_t* params, float* out_dev, void* hip_stream);

/*
 * Aggregate one ring chunk c in [0, n): writes out_dev[lo_c .. hi_c) only (and the matching
 * part of the optional outputs).  out_dev, out_bits_dev and sums_dev still address the FULL
 * length-d vectors, so calling this for every chunk reproduces brace_aggregate byte for byte.
 * Calls for different chunks may run concurrently on different streams (bits that share a
 * 32-bit word with a neighbouring chunk are merged atomically).
 */
int brace_aggregate_chunk(const float* updates_dev, int64_t n, int64_t d, int64_t f,
                          int64_t chunk, const brace_params_t* params, float* out_dev,
                          void* hip_stream);

/*
 * A run of consecutive ring chunks [chunk_begin, chunk_end) in one launch -- the share of one
 * device when the coordinate axis is split over several.  Same contract as the single-chunk
 * form; an empty run is a no-op.
 */
int brace_aggregate_chunks(const float* updates_dev, int64_t n, int64_t d, int64_t f,
                           int64_t chunk_begin, int64_t chunk_end, const brace_params_t* params,
                           float* out_dev, void* hip_stream);

/*
 * Chunk partition (Sec. 2.2: n sub-vectors of about equal size).  Contiguous, ascending;
 * with q = d div n, r = d mod n the first r chunks have q+1 coordinates, the rest q.
 * Host arithmetic only.  [lo, hi) is half-open.
 */
int brace_chunk_range(int64_t n, int64_t d, int64_t chunk, int64_t* lo, int64_t* hi);

/*
 * Client that holds the fully reduced chunk after Share-Reduce in the simulated ring
 * (client i sends to client i+1; the three-client example of Sec. 2.2 puts the second
 * sub-vector on Client 1): owner = (chunk - 1) mod n.  Host arithmetic only.
 */
int brace_chunk_owner(int64_t n, int64_t chunk, int64_t* owner_client);

/*
 * Eq. (1) on integers.  A sign-sum S over n clients is an integer in [-n, n], so S > lambda
 * <=> S >= T with T = floor(lambda) + 1, saturated one step outside that range: T = n + 1 when
 * no sum can exceed lambda (all -1), T = -n when every sum does (all +1).  This is the
 * threshold every entry point applies; a caller that holds sign-sums can apply it itself.
 * Host arithmetic only.  EINVAL for n < 1, a non-finite lambda or a NULL result.
 */
int brace_threshold(int64_t n, float lambda, int32_t* threshold);

/*
 * Vote fused with its consumer, the model update of Sec. 2.1 / App. A:
 *     w[k] <- w[k] - eta * GAR(g_1..g_n)[k]        i.e. every coordinate moves by exactly eta.
 * w_dev holds d fp32 model parameters, updated in place (one fp32 rounding per coordinate); it
 * must not overlap updates_dev.  out_bits_dev / sums_dev of params are still produced when
 * given; when out_bits_dev is given and the range is large, the update itself runs as a
 * second kernel that reads the bits, which keeps the model's read-modify-write traffic off
 * the streaming read.  The _chunk form touches w_dev[lo_c .. hi_c) only.
 */
int brace_aggregate_update(const float* updates_dev, int64_t n, int64_t d, int64_t f,
                           const brace_params_t* params, float eta, float* w_dev, void* hip_stream);
int brace_aggregate_update_chunk(const float* updates_dev, int64_t n, int64_t d, int64_t f,
                                 int64_t chunk, const brace_params_t* params, float eta,
                                 float* w_dev, void* hip_stream);

/*
 * brace_aggregate_update for callers that can neither allocate device memory nor hand over a
 * bit array: code under HIP graph capture, tight serving loops, harnesses that forbid
 * allocation.  Same result as brace_aggregate_update, bit for bit.  The bit-words that pass the
 * vote from the streaming kernel to the kernel that updates w_dev (what out_bits_dev carries in
 * brace_aggregate_update) live in a 16 MiB array inside the library's device code, one copy
 * per device, held until the process ends; the call allocates nothing and frees nothing.
 *   - d must not exceed BRACE_NOALLOC_MAX_D (BRACE_ERANGE otherwise, nothing launched).
 *   - params->out_bits_dev must be NULL (BRACE_EINVAL); sums_dev is honoured as usual.
 *   - Every call on a device uses that device's one array: two calls that overlap in time on
 *     the same device (different streams or threads) race and give wrong updates.  Calls on
 *     one stream, or ordered by events, are safe.  Nothing in it needs clearing between calls.
 *   - The array's address is looked up on the first call on a device (or by
 *     brace_init_device); do that before a graph capture.
 */
#define BRACE_NOALLOC_MAX_D ((int64_t)1 << 27)
int brace_aggregate_update_noalloc(const float* updates_dev, int64_t n, int64_t d, int64_t f,
                                   const brace_params_t* params, float eta, float* w_dev,
                                   void* hip_stream);

/*
 * Receive side of the Share-Only phase (Sec. 3 Phase IV): a client that holds the packed
 * 1-bit result (layout of out_bits_dev, 4*ceil(d/32) bytes) materialises it as d floats of
 * +-1.0f, or applies it to its model copy as w <- w - eta * (+-1).
 */
int brace_expand_bits(const void* bits_dev, int64_t d, float* out_dev, void* hip_stream);
int brace_apply_bits(const void* bits_dev, int64_t d, float eta, float* w_dev, void* hip_stream);

/*
 * Quantise-once form.  brace_quantize is Sec. 3 Phase I kept as data: each client's update
 * becomes two bit planes ("x > 0", "x < 0"; +-0 and NaN set neither), 2 bits per coordinate.
 * brace_vote_packed runs Phases II-IV on those planes and gives the same result as
 * brace_aggregate on the floats, reading 1/16 of the bytes.
 *
 * Layout: client i's row at signs_dev + i*ld_words (uint32 words); word pair j of a row is
 * (positive bits, negative bits) of coordinates 32j .. 32j+31, bit b <-> coordinate 32j+b.
 * A row has brace_packed_row_words(d) = 2 * roundup(ceil(d/32), 2) words of data; padding
 * bits are zero.  ld_words is the row pitch in words: 0 means brace_packed_row_words(d)
 * (dense rows); otherwise a multiple of 4 that is at least that.  The recommended pitch is
 * brace_packed_row_pitch(d), the row words rounded up to a multiple of 32: every row then
 * starts on a 128-byte line and no line is shared by two rows, which removes the lines that
 * dense rows make the kernels touch twice; words between the row's data and the pitch are
 * never read or written.
 * signs_dev must be 16-byte aligned and must not overlap updates_dev.  brace_vote_packed honours lambda, zero_sign and
 * out_bits_dev of params (params->ld is ignored, sums_dev must be NULL); out_dev must be
 * 16-byte aligned and may be NULL when out_bits_dev is given.
 *
 * The _chunk / _chunks forms vote one ring chunk c, or the run [chunk_begin, chunk_end), of
 * the Sec. 2.2 partition (brace_chunk_range) and write only out_dev[lo .. hi) and the bits of
 * those coordinates (merged atomically into words shared with a neighbouring chunk; the caller
 * clears the bit array once).  out_dev / out_bits_dev are still the full-length vectors.  This is
 * what one device of a sharded run executes on the planes it received for its chunks.
 */
int64_t brace_packed_row_words(int64_t d);
int64_t brace_packed_row_pitch(int64_t d);
int brace_quantize(const float* updates_dev, int64_t n, int64_t d, int64_t ld,
                   uint32_t* signs_dev, int64_t ld_words, void* hip_stream);
int brace_vote_packed(const uint32_t* signs_dev, int64_t n, int64_t d, int64_t ld_words, int64_t f,
                      const brace_params_t* params, float* out_dev, void* hip_stream);
int brace_vote_packed_chunk(const uint32_t* signs_dev, int64_t n, int64_t d, int64_t ld_words,
                            int64_t f, int64_t chunk, const brace_params_t* params, float* out_dev,
                            void* hip_stream);
int brace_vote_packed_chunks(const uint32_t* signs_dev, int64_t n, int64_t d, int64_t ld_words,
                             int64_t f, int64_t chunk_begin, int64_t chunk_end,
                             const brace_params_t* params, float* out_dev, void* hip_stream);

/*
 * One-bit form of the quantise-once route, for rules in which every coordinate votes
 * (zero_sign = +1 or -1): then a client's quantised update is exactly one bit per dimension,
 * the format whose volume the cost analysis of Sec. 3 counts.  brace_quantize_1bit writes
 * bit = 1 where the client's vote is +1 (zero_sign = +1: everything but x < 0; zero_sign = -1:
 * only x > 0); it returns BRACE_EINVAL for zero_sign = 0, where a zero abstains and the
 * two-plane form above is needed.  brace_vote_1bit runs Phases II-IV on those bits: with P
 * votes of +1 among n the sign-sum is 2P - n, then Eq. (1); the result equals brace_aggregate
 * on the floats with the same zero_sign.  It honours lambda and out_bits_dev of params
 * (zero_sign and ld are not used, rule must be 0, sums_dev NULL).
 *
 * Layout: client i's row at votes_dev + i*ld_words (uint32 words), bit b of word j <->
 * coordinate 32j + b, brace_1bit_row_words(d) = roundup(ceil(d/32), 4) words per row, padding
 * bits zero; ld_words = 0 means exactly that, otherwise a multiple of 4 at least that;
 * recommended: brace_1bit_row_pitch(d), the row words rounded up to a multiple of 32 (rows
 * start on 128-byte lines).
 * votes_dev and out_dev 16-byte aligned; votes_dev must not overlap updates_dev.
 */
int64_t brace_1bit_row_words(int64_t d);
int64_t brace_1bit_row_pitch(int64_t d);
int brace_quantize_1bit(const float* updates_dev, int64_t n, int64_t d, int64_t ld, int32_t zero_sign,
                        uint32_t* votes_dev, int64_t ld_words, void* hip_stream);
int brace_vote_1bit(const uint32_t* votes_dev, int64_t n, int64_t d, int64_t ld_words, int64_t f,
                    const brace_params_t* params, float* out_dev, void* hip_stream);
/* The run of ring chunks [chunk_begin, chunk_end) only, as brace_vote_packed_chunks. */
int brace_vote_1bit_chunks(const uint32_t* votes_dev, int64_t n, int64_t d, int64_t ld_words,
                           int64_t f, int64_t chunk_begin, int64_t chunk_end,
                           const brace_params_t* params, float* out_dev, void* hip_stream);

/*
 * Sec. 3 Phase III on its own, for an owner that holds partial sign-sums: in Share-Reduce
 * (Phase II) what travels are partial sums of signs (m bits per dimension in the cost
 * analysis of Sec. 3).  parts_dev[j][k], j in [0, g), are g such partial sums as int16 (row
 * pitch ld elements, 0 = d), e.g. one per device; S[k] = sum_j parts[j][k] and Eq. (1) gives
 * out_dev[k] = S[k] > lambda ? +1 : -1 and / or the packed bits (params->out_bits_dev, padding
 * bits zero).  zero_sign of params is not used (the signs are already summed); rule must be 0
 * and sums_dev NULL.  |S| must stay below 2^30 (g <= BRACE_MAX_CLIENTS guarantees it).
 * 16-byte aligned parts_dev / out_dev with ld a multiple of 8 take the wide path.
 */
int brace_consensus_sums(const int16_t* parts_dev, int64_t g, int64_t d, int64_t ld,
                         const brace_params_t* params, float* out_dev, void* hip_stream);

/*
 * The operation BRACE replaces: plain ring-all-reduce aggregation (Sec. 2.2), out[k] =
 * sum_i updates[i][k], or the Mean rule of Sec. 2.1 (sum / n) with mean = 1.  Same streaming
 * shape and chunking as brace_aggregate.
 *
 * order = 0 (default): accumulation in fp64 over the clients in index order, rounded to fp32
 * once, so the result matches the exact sum within one fp32 rounding whatever the
 * cancellation between rows.
 * order = 1: what a ring of fp32 clients delivers (Sec. 2.2 Share-Reduce: every receiver adds
 * its own sub-vector to the one it received): ring chunk c is accumulated in fp32 in the
 * order c, c+1, ..., n-1, 0, ..., c-1, one rounding per addition, so the bits depend on the
 * chunk a coordinate falls in (brace_chunk_range); the mean divides by n once, in fp32.
 * Bit-identical to that ring; NOT within 1e-5 of the exact sum where large rows cancel.
 */
typedef struct brace_rar_params {
    uint32_t struct_size;  /* sizeof(brace_rar_params_t); checked                              */
    int32_t  mean;         /* 0: sum (Sec. 2.2), 1: mean (Sec. 2.1)                             */
    int64_t  ld;           /* row pitch in elements; 0 means ld = d                              */
    int32_t  order;        /* 0: fp64, index order; 1: fp32, ring order of the chunk            */
    int32_t  reserved;     /* must be 0                                                          */
} brace_rar_params_t;

/* struct_size, sum, dense rows, order 0. */
void brace_rar_params_init(brace_rar_params_t* params);

int brace_rar_aggregate(const float* updates_dev, int64_t n, int64_t d,
                        const brace_rar_params_t* params, float* out_dev, void* hip_stream);
int brace_rar_aggregate_chunk(const float* updates_dev, int64_t n, int64_t d, int64_t chunk,
                              const brace_rar_params_t* params, float* out_dev, void* hip_stream);

/*
 * Optional: does, for the current device, the host-side set-up that the first call of some
 * entry points would otherwise do (a device query; loading the kernels; opting the
 * burst-writing kernels in to 128 KiB of LDS; the address of the workspace of
 * brace_aggregate_update_noalloc).  Callers that capture calls into a HIP graph call it once per device
 * before the capture, so that the captured calls only launch kernels.  Launches nothing.
 */
int brace_init_device(void);

/* Text of the last error on the calling thread ("" if none).  Static storage; do not free. */
const char* brace_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* BRACE_H */
