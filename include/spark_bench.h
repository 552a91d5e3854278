/*
 * spark_bench.h -- measurement aids that ship in the same library as the SparK hot path
 * (include/spark.h) but are no part of the method.  bench.py and the profiler runs use them;
 * nothing in the method's entry points calls them.
 */
#ifndef SPARK_BENCH_H
#define SPARK_BENCH_H

#include "spark.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Reads `bytes` (a multiple of 16) from the device buffer `src` once, with 16-byte non-temporal
 * loads from n_blocks blocks of 256 threads, and discards them.  Its time is the streaming-read
 * ceiling the decode kernel is compared with, and its known size calibrates the HBM byte counters
 * of a profiler run.  `sink` is 4 writable device bytes.  Enqueued on `hip_stream`; no
 * synchronisation.  SPARK_ERR_INVALID_ARG for NULL / misaligned pointers, bytes < 16 or n_blocks < 1.
 */
spark_status spark_probe_read(const void *src, size_t bytes, void *sink, int32_t n_blocks,
                              void *hip_stream);

/*
 * Per-block timeline of the decode kernel.  After this call every decode launch of the process whose grid
 * fits (64 bytes per block) lets thread 0 of each block file eight 64-bit words into `device_buffer`:
 *   0 wall clock (100 MHz) at entry          1 at the start of streaming      2 at its end (wavefront 0)
 *   3 when its partial state is stored       4 at exit (after the merge, if it merged)
 *   5 tiles it streamed                      6 XCC id << 32 | HW_ID           7 1 if it merged a pair
 * (in the balanced cut of a ragged batch the wavefronts of a block work on their own: the words are wavefront
 * 0's, and word 5 is 1 << 32 | its tiles).
 * The caller owns the buffer, clears it, reads it back after synchronising, and calls again with NULL to
 * switch the aid off (the buffer must stay valid until then).  Process-wide and not thread safe; the
 * method's results do not depend on it.  SPARK_ERR_INVALID_ARG for a misaligned buffer or bytes < 64.
 */
spark_status spark_decode_timeline(void *device_buffer, size_t bytes);

#ifdef __cplusplus
}
#endif
#endif /* SPARK_BENCH_H */
