/*
 * CPU oracle for the AnyBCQ inference product.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain definition the GPU library is checked against.
 * It shares no code, header, table or helper with the HIP path and must never
 * be linked into it.  Only tests, the smoke check and the benchmark's
 * cpu_baseline leg may call it.
 *
 * What it computes (paper section 2.2, "Binary-coded Quantization": a weight
 * matrix is a sum of binary {-1,+1} planes times real scales; section 1 /
 * Fig. 1(b): p-bit inference uses the scale set that belongs to precision p
 * together with the FIRST p planes; section 3.1 / Fig. 2: a stored 0 means
 * -alpha_i, a stored 1 means +alpha_i, and the value is the running sum over
 * the active planes):
 *
 *   B_i[r][j]   = +1 if bit (j & 31) of planes[i][r][j >> 5] is set, else -1
 *   W_p[r][j]   = sum_{i<p} alpha^{(p)}_i[r][j / group] * B_i[r][j]
 *   y[b][r]     = sum_j W_p[r][j] * x[b][j]
 *   abs[b][r]   = sum_j |W_p[r][j] * x[b][j]|      (used by the tolerance)
 *
 * Asymmetric variant (section 4.1, implementation details: the models are
 * quantised under the asymmetric BCQ scheme, i.e. every (row, group) also
 * carries an offset): with an offset set z^{(p)} for precision p,
 *   W_p[r][j]   = z^{(p)}[r][j / group] + sum_{i<p} alpha^{(p)}_i[r][j / group] * B_i[r][j]
 * and y, abs as above.
 *
 * All arithmetic is IEEE double.  Scales and activations arrive as the raw
 * 16 bits of IEEE binary16 values and are widened exactly.  Nothing is
 * blocked, fused or reordered: one row of W_p is materialised, then dotted
 * with each activation vector from column 0 upwards.  Rows are independent, so
 * the only concession to speed is an OpenMP "parallel for" over rows.
 *
 * Group-wise scales: one scale per (plane, output row, `group` consecutive
 * input columns) (experimental settings, g = 128).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Exact widening of an IEEE binary16 bit pattern to double. */
static double half_bits_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int expo = (h >> 10) & 0x1f;
    int frac = h & 0x3ff;
    double v;
    if (expo == 0) {
        v = ldexp((double)frac, -24);            /* zero and subnormals */
    } else if (expo == 31) {
        v = frac ? NAN : INFINITY;
    } else {
        v = ldexp((double)(frac | 0x400), expo - 25);
    }
    return sign ? -v : v;
}

/* Number of threads the parallel loops below will use. */
int bcq_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void bcq_oracle_set_num_threads(int t)
{
#ifdef _OPENMP
    if (t > 0) omp_set_num_threads(t);
#else
    (void)t;
#endif
}

/*
 * Packing (bit-plane storage, section 3.3: an M x K matrix with p_H bits is
 * kept as p_H separate binary planes so that only the first p are fetched).
 * codes: int8 [n_planes][m][n], a value > 0 is the code +1 (bit 1), anything
 * else is -1 (bit 0).  planes: uint32 [n_planes][m][n/32]; column j lives in
 * word j>>5 at bit j&31.  n must be a multiple of 32.  Returns 0, or -1 on a
 * bad shape.
 */
int bcq_oracle_pack(const int8_t *codes, uint32_t *planes,
                    int n_planes, int64_t m, int64_t n)
{
    if (n_planes < 0 || m < 0 || n < 0 || (n % 32) != 0) return -1;
    int64_t words = n / 32;
    for (int i = 0; i < n_planes; ++i)
        for (int64_t r = 0; r < m; ++r)
            for (int64_t w = 0; w < words; ++w) {
                uint32_t acc = 0;
                for (int b = 0; b < 32; ++b) {
                    int8_t c = codes[((int64_t)i * m + r) * n + w * 32 + b];
                    if (c > 0) acc |= (uint32_t)1 << b;
                }
                planes[((int64_t)i * m + r) * words + w] = acc;
            }
    return 0;
}

/* Inverse of bcq_oracle_pack: bit 1 -> +1, bit 0 -> -1. */
int bcq_oracle_unpack(const uint32_t *planes, int8_t *codes,
                      int n_planes, int64_t m, int64_t n)
{
    if (n_planes < 0 || m < 0 || n < 0 || (n % 32) != 0) return -1;
    int64_t words = n / 32;
    for (int i = 0; i < n_planes; ++i)
        for (int64_t r = 0; r < m; ++r)
            for (int64_t j = 0; j < n; ++j) {
                uint32_t w = planes[((int64_t)i * m + r) * words + (j >> 5)];
                codes[((int64_t)i * m + r) * n + j] = ((w >> (j & 31)) & 1) ? 1 : -1;
            }
    return 0;
}

/*
 * One row of the dequantised matrix W_p (section 2.2 with the precision-p
 * scale set): out[j] = sum_{i<p} alpha_i[r][j/group] * B_i[r][j], j = 0..n-1,
 * plus offsets[r][j/group] when an offset set is given (asymmetric scheme).
 * planes: [>=p][m][n/32]; scales: binary16 bits, [p][m][n/group];
 * offsets: binary16 bits [m][n/group], or NULL.
 */
static void dequant_row(const uint32_t *planes, const uint16_t *scales,
                        const uint16_t *offsets, int p,
                        int64_t m, int64_t n, int64_t group, int64_t r,
                        double *out)
{
    int64_t words = n / 32, ngroups = n / group;
    for (int64_t j = 0; j < n; ++j) {
        double w = 0.0;
        for (int i = 0; i < p; ++i) {
            uint32_t word = planes[((int64_t)i * m + r) * words + (j >> 5)];
            double sign = ((word >> (j & 31)) & 1) ? 1.0 : -1.0;
            double alpha = half_bits_to_double(
                scales[((int64_t)i * m + r) * ngroups + j / group]);
            w += alpha * sign;
        }
        if (offsets) w += half_bits_to_double(offsets[r * ngroups + j / group]);
        out[j] = w;
    }
}

/* Materialise W_p (double [m][n]) -- for tests on small shapes. */
int bcq_oracle_dequant_offset(const uint32_t *planes, const uint16_t *scales,
                              const uint16_t *offsets, int p,
                              int64_t m, int64_t n, int64_t group, double *w_out)
{
    if (p < 1 || m < 0 || n < 0 || group < 1 || (n % 32) || (n % group)) return -1;
    for (int64_t r = 0; r < m; ++r)
        dequant_row(planes, scales, offsets, p, m, n, group, r, w_out + r * n);
    return 0;
}

int bcq_oracle_dequant(const uint32_t *planes, const uint16_t *scales, int p,
                       int64_t m, int64_t n, int64_t group, double *w_out)
{
    return bcq_oracle_dequant_offset(planes, scales, NULL, p, m, n, group, w_out);
}

/*
 * Per-request product.  Request b uses precision p_req[b], i.e. planes
 * 0..p_req[b]-1 and the scale set scales_by_p[p_req[b]] (section 3.3:
 * precision is selected per request at run time; section 1: each precision has
 * its own scale set while the planes are shared).
 *
 * planes      uint32 [p_max][m][n/32]
 * scales_by_p p_max+1 pointers; entry q is binary16 bits [q][m][n/group] or
 *             NULL when no request uses precision q
 * offsets_by_p NULL, or p_max+1 pointers; entry q is binary16 bits
 *             [m][n/group], the offsets of precision q, or NULL for none
 * p_req       int32 [batch], each in [1, p_max]
 * x           binary16 bits [batch][n]
 * y, abs_out  double [batch][m]; abs_out may be NULL
 * Returns 0, or -1 on a bad argument.
 */
int bcq_oracle_gemm_mixed_offset(const uint32_t *planes,
                                 const uint16_t *const *scales_by_p,
                                 const uint16_t *const *offsets_by_p,
                                 const int32_t *p_req, int p_max,
                                 const uint16_t *x, double *y, double *abs_out,
                                 int64_t m, int64_t n, int64_t batch, int64_t group)
{
    if (p_max < 1 || m < 0 || n < 0 || batch < 0 || group < 1 ||
        (n % 32) || (n % group))
        return -1;
    for (int64_t b = 0; b < batch; ++b) {
        if (p_req[b] < 1 || p_req[b] > p_max || !scales_by_p[p_req[b]]) return -1;
    }
    int failed = 0;
#pragma omp parallel
    {
        double *wrow = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
        if (!wrow) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(static)
        for (int64_t r = 0; r < m; ++r) {
            if (!wrow) continue;
            for (int q = 1; q <= p_max; ++q) {
                int used = 0;
                for (int64_t b = 0; b < batch; ++b) used |= (p_req[b] == q);
                if (!used) continue;
                dequant_row(planes, scales_by_p[q], offsets_by_p ? offsets_by_p[q] : NULL, q, m, n, group, r, wrow);
                for (int64_t b = 0; b < batch; ++b) {
                    if (p_req[b] != q) continue;
                    double acc = 0.0, aacc = 0.0;
                    for (int64_t j = 0; j < n; ++j) {
                        double t = wrow[j] * half_bits_to_double(x[b * n + j]);
                        acc += t;
                        aacc += fabs(t);
                    }
                    y[b * m + r] = acc;
                    if (abs_out) abs_out[b * m + r] = aacc;
                }
            }
        }
        free(wrow);
    }
    return failed ? -1 : 0;
}

/* Symmetric scheme: the same without offsets. */
int bcq_oracle_gemm_mixed(const uint32_t *planes,
                          const uint16_t *const *scales_by_p,
                          const int32_t *p_req, int p_max,
                          const uint16_t *x, double *y, double *abs_out,
                          int64_t m, int64_t n, int64_t batch, int64_t group)
{
    return bcq_oracle_gemm_mixed_offset(planes, scales_by_p, NULL, p_req, p_max,
                                        x, y, abs_out, m, n, batch, group);
}

/*
 * Uniform precision: every request uses precision p with scale set `scales`
 * ([p][m][n/group]) and, when `offsets` is not NULL, the offset set `offsets`
 * ([m][n/group]).  Same definition as above with p_req[b] = p for all b.
 */
int bcq_oracle_gemv_offset(const uint32_t *planes, const uint16_t *scales,
                           const uint16_t *offsets, int p,
                           const uint16_t *x, double *y, double *abs_out,
                           int64_t m, int64_t n, int64_t batch, int64_t group)
{
    if (p < 1 || p > 64 || batch < 0) return -1;
    const uint16_t *sets[65];
    const uint16_t *offs[65];
    memset(sets, 0, sizeof(sets));
    memset(offs, 0, sizeof(offs));
    sets[p] = scales;
    offs[p] = offsets;
    int32_t *preq = (int32_t *)malloc(sizeof(int32_t) * (size_t)(batch > 0 ? batch : 1));
    if (!preq) return -1;
    for (int64_t b = 0; b < batch; ++b) preq[b] = p;
    int rc = bcq_oracle_gemm_mixed_offset(planes, sets, offs, preq, p, x, y, abs_out,
                                          m, n, batch, group);
    free(preq);
    return rc;
}

int bcq_oracle_gemv(const uint32_t *planes, const uint16_t *scales, int p,
                    const uint16_t *x, double *y, double *abs_out,
                    int64_t m, int64_t n, int64_t batch, int64_t group)
{
    return bcq_oracle_gemv_offset(planes, scales, NULL, p, x, y, abs_out, m, n, batch, group);
}
