/*
 * bcq.h -- C ABI of the MI355X (gfx950) AnyBCQ inference library.
 *
 * The library computes the multi-precision binary-coded-quantisation product
 *
 *     y[b][r] = sum_{i < p_b} sum_j alpha^{(p_b)}_i[r][j / group] * B_i[r][j] * x[b][j]
 *
 * where B_i in {-1,+1} are bit-planes shared by all precisions, each precision p
 * owns a group-wise scale set alpha^{(p)}, and request b runs at precision p_b
 * using only the first p_b planes (paper sections 2.2, 3.1 and 3.3).
 *
 * Conventions common to every entry point
 *   - All data pointers are DEVICE pointers unless a parameter says "host".
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Work is enqueued on it; no entry point synchronises or allocates.
 *   - The caller owns every buffer and must keep it alive until the enqueued
 *     work has finished.  The library keeps no reference after that.
 *   - Functions return BCQ_OK or a negative bcq_status; they never throw, never
 *     terminate the process and enqueue nothing when they return an error.
 *   - bcq_half is the raw 16-bit pattern of an IEEE binary16 value.
 *
 * Storage format (section 3.3, bit-plane storage; Fig. 1 caption: 0 means -1)
 *   planes  uint32 [n_planes][m][n/32], plane-major then row-major.  Input
 *           column j of row r in plane i is bit (j & 31) of word
 *           planes[(i*m + r)*(n/32) + (j >> 5)]; bit 1 = +1, bit 0 = -1.
 *           Plane 0 is the first (coarsest) plane; precision p reads planes
 *           0..p-1 and never touches the others.
 *   scales  bcq_half [p][m][n/group] for the set of precision p: one scale per
 *           (plane, output row, `group` consecutive input columns).
 *   x       bcq_half [batch][n], y  bcq_half [batch][m], both row-major.
 *
 * Shape rules: m >= 1, n >= group, group % 32 == 0, n % group == 0,
 * 1 <= p <= p_max <= BCQ_MAX_PLANES, batch >= 0 (0 is a no-op).
 * planes, scales and x must be 16-byte aligned, y 2-byte aligned.
 * Accumulation is in fp32; the result is rounded once to binary16.
 */
#ifndef BCQ_H
#define BCQ_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef uint16_t bcq_half;

#define BCQ_MAX_PLANES 8
#define BCQ_MAX_MULTI 4   /* matrices per bcq_gemv_multi call */

typedef enum {
    BCQ_OK = 0,
    BCQ_ERR_NULL = -1,       /* a required pointer is NULL */
    BCQ_ERR_BAD_P = -2,      /* precision / plane count out of range */
    BCQ_ERR_BAD_SHAPE = -3,  /* m, n, batch or group violate the shape rules */
    BCQ_ERR_ALIGN = -4,      /* a pointer is not aligned as required */
    BCQ_ERR_HIP = -5,        /* the HIP runtime reported an error at launch */
    BCQ_ERR_VARIANT = -6     /* a forced kernel variant cannot run this problem */
} bcq_status;

/* Static, NUL-terminated description of a status code.  Host call. */
const char *bcq_strerror(int status);

/*
 * bcq_pack -- bit-plane storage (section 3.3): turn +-1 codes into planes.
 *   codes   int8  [n_planes][m][n]; a value > 0 is the code +1, anything else -1
 *   planes  uint32 [n_planes][m][n/32], written in the storage format above
 * n % 32 == 0, 1 <= n_planes <= BCQ_MAX_PLANES.  Integer work, bit-exact.
 */
int bcq_pack(const int8_t *codes, uint32_t *planes, int n_planes,
             int64_t m, int64_t n, void *stream);

/* bcq_unpack -- inverse of bcq_pack: bit 1 -> +1, bit 0 -> -1 (int8). */
int bcq_unpack(const uint32_t *planes, int8_t *codes, int n_planes,
               int64_t m, int64_t n, void *stream);

/*
 * bcq_gemv -- the AnyBCQ kernel of section 3.3 at one precision for the whole
 * batch: for every plane i < p form B_i x by adding/subtracting activations,
 * multiply by alpha_i, accumulate, and return after plane p.
 *   planes    uint32 [>= p][m][n/32]; only planes 0..p-1 are read
 *   scales_p  bcq_half [p][m][n/group], the scale set OF PRECISION p
 *   x         bcq_half [batch][n]
 *   y         bcq_half [batch][m] (written)
 */
int bcq_gemv(const uint32_t *planes, const bcq_half *scales_p, int p,
             const bcq_half *x, bcq_half *y,
             int64_t m, int64_t n, int batch, int group, void *stream);

/*
 * bcq_gemm_mixed -- per-request precision (sections 1 and 3.3): request b uses
 * planes 0..p_req[b]-1 with the scale set of precision p_req[b]; the planes
 * are stored once to p_max and read once up to max_b p_req[b].
 *   planes       uint32 [p_max][m][n/32]
 *   scales_by_p  HOST array of p_max+1 device pointers; entry q is the set of
 *                precision q ([q][m][n/group]); entry 0 is ignored; an entry
 *                may be NULL if no request uses that precision (a request that
 *                does name it is then computed as all-zero output)
 *   p_req        DEVICE int32 [batch]; values are clamped to [1, p_max]
 *   x, y         as for bcq_gemv
 */
int bcq_gemm_mixed(const uint32_t *planes, const bcq_half *const *scales_by_p,
                   const int32_t *p_req, int p_max,
                   const bcq_half *x, bcq_half *y,
                   int64_t m, int64_t n, int batch, int group, void *stream);

/*
 * Asymmetric BCQ (section 4.1, implementation details: the models are quantised
 * under the asymmetric scheme): every (row, group) also carries an offset z, so
 * W_p[r][j] = z^{(p)}[r][j/group] + sum_{i<p} alpha^{(p)}_i[r][j/group] B_i[r][j]
 * and y gains sum_g z^{(p)}[r][g] * sum_{j in g} x[b][j].  Each precision has its
 * own offsets, as it has its own scales.
 *
 * bcq_gemv_offset: as bcq_gemv, plus
 *   offsets_p  bcq_half [m][n/group] (device), the offsets OF PRECISION p;
 *              NULL gives exactly bcq_gemv
 * bcq_gemm_mixed_offset: as bcq_gemm_mixed, plus
 *   offsets_by_p  HOST array of p_max+1 device pointers; entry q is the offset
 *                 set of precision q ([m][n/group]) or NULL for none; entry 0
 *                 is ignored; the array itself may be NULL (no offsets at all)
 * Offset sets must be 16-byte aligned.  Errors as for the symmetric calls.
 */
int bcq_gemv_offset(const uint32_t *planes, const bcq_half *scales_p, const bcq_half *offsets_p, int p,
                    const bcq_half *x, bcq_half *y,
                    int64_t m, int64_t n, int batch, int group, void *stream);

int bcq_gemm_mixed_offset(const uint32_t *planes, const bcq_half *const *scales_by_p,
                          const bcq_half *const *offsets_by_p,
                          const int32_t *p_req, int p_max,
                          const bcq_half *x, bcq_half *y,
                          int64_t m, int64_t n, int batch, int group, void *stream);

/*
 * bcq_gemv_multi -- several weight matrices applied to the SAME activations at
 * the same precision in one call (the q/k/v and the gate/up projections of a
 * decoder layer; section 4.4 measures whole decoding steps made of such layers).
 * Equivalent to `count` calls of bcq_gemv, but as a single kernel launch
 * where one kernel family serves the matrices taken together.  The kernel
 * form and workgroup shape, and with them the order of the fp32 sums, are
 * chosen for the sum of the rows: results agree with separate calls within
 * the accuracy both are held to, and bit for bit wherever the same form
 * serves both (with one request always; with up to 8 unless the matrices
 * are tall enough only together for the row-streaming form).
 *   count      1 .. BCQ_MAX_MULTI
 *   planes     HOST array of `count` device pointers, matrix k: [>= p][m[k]][n/32]
 *   scales_p   HOST array of `count` device pointers, matrix k: [p][m[k]][n/group]
 *   m          HOST array of `count` row counts
 *   y          HOST array of `count` device pointers, matrix k: [batch][m[k]] (written)
 *   x          bcq_half [batch][n], shared
 * Errors as for bcq_gemv (the first offending matrix decides).
 */
int bcq_gemv_multi(int count, const uint32_t *const *planes, const bcq_half *const *scales_p, const int64_t *m,
                   bcq_half *const *y, int p, const bcq_half *x,
                   int64_t n, int batch, int group, void *stream);

/*
 * bcq_quantize -- the offline quantiser: Algorithm 1 of section 3.2 ("AnyBCQ
 * initialization and progressive precision expansion") built from the blocks
 * of section 2.2 (greedy initialisation; scales by least squares; codes
 * reassigned to the nearest of the 2^p levels), applied group-wise (section
 * 4.1).  Every (row, group) of `w` is quantised on its own:
 *   base precision p_low : greedy start, then `cycles` rounds of LS and BS;
 *   p = p_low+1..p_high  : planes 0..p-2 stay frozen; `cycles` rounds of
 *                          residual -> sign (the new plane p-1) -> LS over all
 *                          p scales, starting from [alpha^(p-1), 0].
 * The scale set of precision p is what the scales are when its rounds end.
 * With `offsets_by_p` the asymmetric scheme of section 4.1 is fitted: the
 * offset is one more least-squares unknown (all-ones basis vector).
 * Definitions that decide codes: sign(0) = +1; the residual that re-signs the
 * new plane excludes that plane (section 2.2's residual after p-1 planes; the
 * listing's own form, which takes the new plane's term out as well, is
 * available through bcq_quantize_form);
 * nearest-level ties go to the first level when enumerated with plane 0 as the
 * most significant bit of the index; a plane that is linearly dependent on the
 * planes before it gets scale 0.  Arithmetic is IEEE double (sums of binary16
 * weights are exact in it), results are rounded once to binary16.
 *   w             bcq_half [m][n], 16-byte aligned (finite values)
 *   p_low, p_high 1 <= p_low <= p_high <= 4
 *   cycles        T of Algorithm 1, >= 0; >= 1 if p_high > p_low
 *   planes        uint32 [p_high][m][n/32] (written), storage format above
 *   scales_by_p   HOST array of p_high+1 device pointers; entry p in
 *                 p_low..p_high: bcq_half [p][m][n/group] (written); other
 *                 entries are ignored
 *   offsets_by_p  NULL (symmetric), or HOST array of p_high+1 device pointers;
 *                 entry p in p_low..p_high: bcq_half [m][n/group] (written)
 *   group         32, 64, 128 or 256
 * Errors: BCQ_ERR_NULL, BCQ_ERR_BAD_P (precisions or cycles out of range),
 * BCQ_ERR_BAD_SHAPE, BCQ_ERR_ALIGN, BCQ_ERR_HIP.
 */
int bcq_quantize(const bcq_half *w, int p_low, int p_high, int cycles, uint32_t *planes, bcq_half *const *scales_by_p,
                 bcq_half *const *offsets_by_p, int64_t m, int64_t n, int group, void *stream);

/*
 * bcq_quantize_form -- bcq_quantize with the residual of the expansion cycles
 * chosen by the caller.  Algorithm 1 (section 3.2) prints the cycle as
 * "R <- W - Dequant({alpha_i^p, B_i} for i = 1..p); B_p <- sign(R); LS": read
 * literally, the new plane's own term alpha_p B_p is subtracted too from the
 * second cycle on (in the first both are zero).  Section 2.2 defines the
 * residual that a new plane takes the sign of as the one after the planes
 * before it, and the literal form does not settle (a code whose residual is
 * smaller than the new scale flips every cycle; on Gaussian weights its 3-bit
 * error is about 2.5 times that of the other form), so bcq_quantize uses
 *   BCQ_RESIDUAL_FROZEN_PLANES  R = W - sum_{i<p} alpha_i B_i  (planes 1..p-1)
 * and this call also offers
 *   BCQ_RESIDUAL_LISTING        R = W - sum_{i<=p} alpha_i B_i (all p planes).
 * Both agree after one cycle.  Any other value: BCQ_ERR_VARIANT.  All other
 * arguments, results and errors as for bcq_quantize.
 */
enum { BCQ_RESIDUAL_FROZEN_PLANES = 0, BCQ_RESIDUAL_LISTING = 1 };
int bcq_quantize_form(const bcq_half *w, int p_low, int p_high, int cycles, int residual_form, uint32_t *planes,
                      bcq_half *const *scales_by_p, bcq_half *const *offsets_by_p, int64_t m, int64_t n, int group,
                      void *stream);

#ifdef __cplusplus
}
#endif
#endif /* BCQ_H */
