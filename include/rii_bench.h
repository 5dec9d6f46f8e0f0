/*
 * rii_bench.h -- measurement aids of the library declared in rii.h.  Nothing here is needed to
 * search; a benchmark uses these calls to time one kernel of an online call in isolation, to read
 * the tallies the scan kernels keep while it does so, and to measure the LDS look-up ceiling the
 * batched scan is bound by.  Same conventions as rii.h (status codes, host / device pointers).
 */
#ifndef RII_BENCH_H
#define RII_BENCH_H

#include "rii.h"

#ifdef __cplusplus
extern "C" {
#endif

/* While two hipEvent_t (passed as void*) are set, every rii_adc_scan_linear call (and the
 * linear-scan branch of rii_query) records `start_event` right before and `stop_event` right
 * after the kernel that streams the code array (Alg. 1, the loop over s), on the call's stream.
 * Pass NULL, NULL to switch it off.  The caller owns the events. */
int rii_index_set_scan_events(rii_index_t* index, void* start_event, void* stop_event);

#define RII_SCAN_COUNTERS 8
/* While the scan events are set, the kernels of Alg. 1 over the whole database keep tallies.
 * This call returns them (counters_out[RII_SCAN_COUNTERS], host) as accumulated since the last
 * call and resets them.  Synchronous (waits for the device).
 *   [0] batched scan: slices (64 rows x one group of four queries, i.e. 64 x M table look-ups) scored
 *   [1] batched scan: slices abandoned after M/2 look-ups at the latest
 *   [3] batched scan, M = 32: those of [1] that were abandoned after M/4 look-ups already
 *   [4] batched scan, M = 32: slices abandoned after 3M/4 look-ups
 *   one-query scan of an M = 32 array (two planes of 16 bytes per row; the first plane is always
 *   streamed, N x 16 bytes per pass):
 *   [2] 128-byte memory lines of the second plane it fetched (a row's second half is asked for
 *       only when its first 16 look-ups leave it within the bound)
 *   [5] .. [7] unused (zero). */
int rii_index_read_scan_counters(rii_index_t* index, uint64_t* counters_out);

/* Launch shape rii_adc_scan_linear uses for a batch of Q queries on this index (so that a
 * benchmark can name the kernel it timed): *queries_per_block = 4, 2 or 1 queries sharing one
 * pass over the codes (Alg. 1 run for several queries at once; results are per query);
 * *row_chunks = blocks that share one query group's rows.  Host call, no GPU work. */
int rii_scan_linear_plan(const rii_index_t* index, int Q, int topk, int* queries_per_block, int64_t* row_chunks);

/* LDS look-up ceiling of the scan kernels' inner loop, for the roofline of the batched scan
 * (Sec. 3: a distance is M table look-ups; with several queries per pass these, not the code
 * stream, bound the kernel).  Runs `blocks` blocks of `threads` threads; every lane performs
 * iters * 32 dependent-free look-ups (one byte-permute, one LDS read of `width` bytes at a
 * conflict-free pseudo-random address in a 64 KB table, one add per component) and nothing
 * else; no global memory traffic inside the loop.
 *   width 4 or 8 (ds_read_b32 / ds_read_b64 with 32-bit adds per component) or 64 (ds_read_b64
 *   with one 64-bit integer add per look-up); threads a multiple of 64 up to 1024; lds_bytes >=
 *   65536 sizes the block's LDS allocation (and thereby blocks per CU); sink device uint32 [1]
 *   (written only to keep the loop alive).  The caller times the call with events on `stream`.
 * Look-ups performed = blocks * threads * 32 * iters. */
int rii_bench_lds_lookups(int width, int blocks, int threads, int iters, int lds_bytes, uint32_t* sink, void* stream);

/* rii_adc_scan_linear with the half-precision table variant of the batched kernel (Sec. 3 leaves the
 * precision of the distance table open; the library's batched kernel filters with a 15-bit integer
 * table, this variant with fp16 entries and packed fp16 sums; both re-score the rows that pass in
 * fp32, so the results are the same -- what differs is the time).  Same arguments as
 * rii_adc_scan_linear; RII_ERR_UNSUPPORTED when the batch would not take the four-queries-per-block
 * kernel (see rii_scan_linear_plan). */
int rii_bench_scan_linear_half(rii_index_t* index, const float* lut, int Q, int topk, int32_t* ids, float* dist,
                               void* stream);

/* The LDS pipe's own read ceiling, beside the look-up ceiling above: the same launch shape, but
 * every lane only reads -- `width` = 4, 8 or 16 bytes (ds_read_b32 / _b64 / _b128) at conflict-free
 * addresses, 16 / 8 / 4 reads in flight per wave, one exclusive-or per returned dword, no address
 * arithmetic.  Reads performed = blocks * threads * iters * (16, 8 or 4 for width 4, 8, 16). */
int rii_bench_lds_reads(int width, int blocks, int threads, int iters, int lds_bytes, uint32_t* sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* RII_BENCH_H */
