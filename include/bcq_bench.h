/*
 * bcq_bench.h -- reference kernels for the benchmark.  They are not part of the
 * AnyBCQ method: they measure what the same GPU reaches on plain bandwidth-bound
 * work, so that a product's time can be set against an achievable figure and not
 * only against the data-sheet peak (the paper's Table 2 sets its kernel against a
 * half-precision product in the same way).
 * All pointers are DEVICE pointers; `stream` is a hipStream_t passed as void*;
 * work is enqueued, nothing is allocated or synchronised.  Return 0, or the
 * negative bcq_status values of bcq.h (-1 NULL, -3 shape, -4 alignment, -5 HIP).
 */
#ifndef BCQ_BENCH_H
#define BCQ_BENCH_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Streaming read of `bytes` bytes (a multiple of 16, 16-byte aligned) with 128-bit
 * non-temporal loads and no stores to speak of: `sink` (64 words) is written only
 * if a workgroup's XOR of everything it read equals one particular constant.
 */
int bcq_bench_stream_read(const void *src, int64_t bytes, uint32_t *sink, void *stream);

/*
 * y[r] = sum_j w[r][j] * x[j] for binary16 w [m][n] (row-major), x [n], y [m];
 * one wavefront per row, fp32 accumulation, n a multiple of 8, w and x 16-byte aligned.
 */
int bcq_bench_fp16_gemv(const uint16_t *w, const uint16_t *x, uint16_t *y, int64_t m, int64_t n, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* BCQ_BENCH_H */
