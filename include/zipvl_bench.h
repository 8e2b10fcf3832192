/*
 * zipvl_bench.h - measurement aids of libzipvl.so.  Nothing here is part of the method or of the
 * product boundary (that is zipvl.h): per-kernel timing with HIP events, and two probe kernels that
 * show what the GPU sustains, for the benchmark's roofline figures.
 */
#ifndef ZIPVL_BENCH_H
#define ZIPVL_BENCH_H

#include "zipvl.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Per-kernel timing for benchmarks (not part of the method).  While enabled,
 * every kernel launch of the calling process is bracketed by two HIP events on
 * its own stream (up to 8192 launches are kept; later ones are not timed).
 * zipvl_timing_read waits for the recorded events and returns the summed
 * duration and launch count of one kernel, then keeps accumulating;
 * zipvl_timing_enable(1) clears the records, zipvl_timing_enable(0) stops.
 */
#define ZIPVL_K_SCORE_ROWSTATS  0
#define ZIPVL_K_SCORE_COLSUM    1
#define ZIPVL_K_SELECT          2
#define ZIPVL_K_COMPACT_KV      3
#define ZIPVL_K_KV_APPEND       4
#define ZIPVL_K_ZERO_FILL       5
#define ZIPVL_K_PACK_KV         6
#define ZIPVL_K_FLASH_KEPT      7
#define ZIPVL_K_DECODE_PARTIAL  8
#define ZIPVL_K_DECODE_COMBINE  9
#define ZIPVL_K_SCORE_ROWFINAL 10
#define ZIPVL_K_SHARE_SCORES   11
#define ZIPVL_K_TOKEN_SLOTS    12
#define ZIPVL_K_QUANTIZE_ROWS  13
#define ZIPVL_K_DECODE_Q_PARTIAL 14
#define ZIPVL_K_ALLROWS_LSE    15
#define ZIPVL_K_ALLROWS_COLSUM 16
#define ZIPVL_K_PROBE_MFMA     17
#define ZIPVL_K_PROBE_READ     18
#define ZIPVL_K_DECODE_STEP    19
#define ZIPVL_K_SELECT_HIST    20
#define ZIPVL_K_COUNT          21
int zipvl_timing_enable(int on);
int zipvl_timing_read(int kernel_id, double* total_ms, int* launches);

/*
 * What the GPU sustains (measurement aids for the benchmark's roofline, not part of the method).
 * zipvl_probe_mfma: `workgroups` x 4 waves each issue iters x 8 independent 32x32x16 bf16 MFMAs
 * (32768 flop each) and nothing else; out [device]: workgroups * 256 floats (a checksum that keeps the
 * work alive).  zipvl_probe_stream_read: reads `bytes` (multiple of 16) of src once with 16-byte loads;
 * out [device]: workgroups * 256 uint32.  Time them with zipvl_timing_enable / zipvl_timing_read.
 */
int zipvl_probe_mfma(int iters, int workgroups, float* out, void* stream);
int zipvl_probe_stream_read(const void* src, size_t bytes, int workgroups, uint32_t* out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* ZIPVL_BENCH_H */
