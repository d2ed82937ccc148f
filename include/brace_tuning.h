/*
 * brace_tuning.h -- launch tuning, diagnostics and measurement aids of libbrace.
 *
 * Nothing here is part of the aggregation method and no caller of brace.h needs it: these
 * calls exist for benchmarks, autotuning and tests.  Unlike the calls of brace.h they set
 * process-wide state (guarded: they may be called from any thread).  Every tuning
 * combination produces bit-identical results.
 */
#ifndef BRACE_TUNING_H
#define BRACE_TUNING_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Switch of the host-side buffer checks of brace.h (is it device memory, does the call stay
 * inside its allocation).  On by default (two runtime queries per buffer; measured 0.3 us of a
 * 4.3 us call); process-wide switch for callers that cannot afford them.
 */
int brace_set_pointer_checks(int32_t enabled);

/*
 * Launch tuning for the streaming kernel (process-wide: a call reads the setting in force when
 * it is made).
 */
typedef struct brace_tuning {
    uint32_t struct_size;  /* sizeof(brace_tuning_t)                                             */
    int32_t  vec;          /* widest load in dwords: 1, 2, 4 (narrowed to what alignment allows);  */
                           /* 0 = auto: what alignment allows, 2 instead of 4 for large ranges     */
    int32_t  cols;         /* loads per lane per row: 1, 2, 4 or 8; 0 = from the size of the range */
    int32_t  unroll;       /* rows per batch of loads: 2, 4 or 8; 0 = from the size of the range  */
    int32_t  nontemporal;  /* 1: streaming (non-temporal) loads                                   */
    int32_t  pipeline;     /* 1: request the next batch of rows before consuming the current one  */
    int32_t  split_writes; /* fp32 output written by a second, write-only kernel from the bits:   */
                           /* 0 = for large ranges (default), 1 = never, 2 = whenever possible    */
    int32_t  rowsplit;     /* the 4 waves of a block share their columns and split the client     */
                           /* rows (partial results meet in LDS): 0 = for short ranges (default), */
                           /* 1 = never, 2 = always                                               */
    int32_t  stage_writes; /* results with no compact form (sum / mean, in-place update, the bit   */
                           /* planes of brace_quantize) are parked in LDS and written as one      */
                           /* 128 KiB burst per block:                                            */
                           /* 0 = for large ranges (default), 1 = never, 2 = whenever possible    */
} brace_tuning_t;

int brace_set_tuning(const brace_tuning_t* tuning);   /* NULL restores the defaults */
int brace_get_tuning(brace_tuning_t* tuning);

/*
 * Measurement aids (not part of the method): a streaming read and a plain copy of a buffer
 * of known size, used to calibrate the HBM byte counters and to report the bandwidth a
 * trivially linear access pattern reaches on the same device.  Buffers are device memory,
 * 16-byte aligned, nbytes a multiple of 16.  sink_dev is 4 bytes that are (practically)
 * never written.  Enqueued on hip_stream; no synchronisation.
 */
int brace_probe_read(const void* src_dev, int64_t nbytes, int32_t nontemporal, void* sink_dev,
                     void* hip_stream);
int brace_probe_copy(void* dst_dev, const void* src_dev, int64_t nbytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* BRACE_TUNING_H */
