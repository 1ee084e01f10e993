/* Measurement aid of libnuq.so: per-launch kernel times for benchmarks.
 *
 * Not part of the method and not needed by a caller of include/nuq.h: bench.py uses it to bracket the
 * main kernel of each entry point with HIP events on the stream the kernel is launched on.  The
 * capture is process-global state: one capture at a time, not thread-safe.
 */
#ifndef NUQ_BENCH_H
#define NUQ_BENCH_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Entry-point ids reported by nuq_timing_collect. */
enum { NUQ_T_NORMS = 1, NUQ_T_QUANTIZE = 2, NUQ_T_ENCODE = 3, NUQ_T_QUANTIZE_ENCODE = 4, NUQ_T_DECODE = 5 };

/* After nuq_timing_begin(n), each of the next n launches of a main kernel (the per-bucket kernel
 * of nuq_bucket_norms / nuq_quantize / nuq_encode / nuq_quantize_encode, the tile kernel of
 * nuq_decode_accumulate) is bracketed by a pair of HIP events recorded on its stream.  The small
 * offset-scan and gather kernels of the encoders are outside the brackets.  n <= 4096.
 * Not thread-safe; meant for benchmarks. */
int nuq_timing_begin(uint32_t max_launches);

/* Waits for the bracketed launches, writes up to `cap` durations (milliseconds) and entry-point
 * ids to the HOST arrays ms[] and entry[], the number written to *count, and ends the capture. */
int nuq_timing_collect(float *ms, int32_t *entry, uint32_t cap, uint32_t *count);

#ifdef __cplusplus
}
#endif
#endif /* NUQ_BENCH_H */
