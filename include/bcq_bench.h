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
 * Test and benchmark knobs.  They live here and not in bcq.h because no product call needs them; their state is
 * PER HOST THREAD (thread-local): a thread that forces a variant or a shape changes its own later calls only, and
 * bcq_last_kernel reports the calling thread's own most recent launch.
 */

/* Kernel variants for bcq_select_kernel. */
typedef enum {
    BCQ_KERNEL_AUTO = 0,        /* pick by shape and batch */
    BCQ_KERNEL_SIGN_SELECT = 1, /* generic per-bit add/subtract kernel, any legal shape */
    BCQ_KERNEL_PLANE_MFMA = 2,  /* bit-planes fed to the FP4 matrix pipe, small batches */
    BCQ_KERNEL_DEQUANT_MFMA = 3,/* dequantise to fp16 tiles in LDS + fp16 MFMA, large batches */
    BCQ_KERNEL_PLANE_F16 = 4,   /* +-1 planes as fp16 MFMA operands, group sums scaled in fp32 by each request's own scales; groups >= 128 */
    BCQ_KERNEL_LUT = 5          /* table look-ups: 16 signed sums per four activations in LDS, a nibble of a plane word picks one; any legal shape */
} bcq_kernel;

/*
 * Force one kernel variant for the calling thread's later product calls (BCQ_KERNEL_AUTO restores the default
 * choice).  A forced variant that cannot handle a problem makes the call return BCQ_ERR_VARIANT (-6).
 * Returns 0, or -6 for an unknown id.
 */
int bcq_select_kernel(int variant);

/* The variant the calling thread has forced (BCQ_KERNEL_AUTO if none). */
int bcq_selected_kernel(void);

/*
 * Force the workgroup shape of the large-batch kernel for the calling thread's later calls (the library otherwise
 * picks it from m and the batch): `request_tiles` tiles of 64 requests and `row_blocks` blocks of 16 rows per
 * workgroup, one of (1,4) (1,2) (1,1) (2,4) (2,2) (4,4), or (0,4) (0,2) (0,1) for a single tile of 16 requests and
 * (32,4) (32,2) (32,1) for one of 32, (0,8) and (32,8) for those tiles with one row block whose columns are split
 * over eight teams of waves instead of four, (4,8) and (2,8) for 256 and 128 requests with eight row blocks, (4,40)
 * for 256 requests and four row blocks served by two teams of waves that share the activation tiles; per-request
 * precision uses the row blocks and whether the tile has 32 requests only, beyond 64 requests the whole shape if it
 * has 64 requests or more.  (0, 0) restores the automatic choice.  Returns 0, or -6 for any other pair.
 */
int bcq_select_dequant_shape(int request_tiles, int row_blocks);

/* Name of the variant the calling thread's most recent successful launch used ("" before any): "sign_select",
 * "lut", "plane_mfma" ("plane_mfma_rows" where that family ran in its row-streaming form: tall matrices with two to eight
 * requests, or with one request at one or two planes), "dequant_mfma", "plane_f16", "quantize". */
const char *bcq_last_kernel(void);

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

/*
 * Instruction-issue probe: ONE workgroup of `waves` wavefronts (1 .. 16; beyond four they share SIMDs) runs `iters`
 * times four matrix instructions, each followed by `valu` (0, 4, 8 or 16) independent fp32 vector FMAs.  kind 0:
 * v_mfma_f32_16x16x32_f16, 1: v_mfma_f32_32x32x16_f16, 2: v_mfma_f32_16x16x128_f8f6f4 (E5M2 x FP4 operands).
 * ticks[2w] receives the shader-clock ticks and ticks[2w + 1] the 100 MHz ticks that wave w's loop took (ticks: room
 * for 32 values); sink: room for 1024 floats, written with values that mean nothing.  Returns -3 for other arguments.
 */
int bcq_bench_issue_probe(int kind, int valu, int waves, int iters, uint64_t *ticks, float *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* BCQ_BENCH_H */
