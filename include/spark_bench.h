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

#ifdef __cplusplus
}
#endif
#endif /* SPARK_BENCH_H */
