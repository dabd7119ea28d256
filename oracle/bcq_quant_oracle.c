/*
 * CPU oracle for the AnyBCQ quantiser.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow statement of Algorithm 1 ("AnyBCQ initialization and progressive
 * precision expansion", section 3.2) with the building blocks of section 2.2
 * ("Binary-coded Quantization": greedy initialisation, least-squares scales,
 * code reassignment by search over the levels).  It shares no code, header,
 * table or helper with the HIP path and must never be linked into it.  Only
 * tests, the smoke check and the benchmark's cpu_baseline leg may call it.
 *
 * The weights are quantised group-wise (section 4.1: groups of g = 128
 * consecutive input columns of an output row); every (row, group) is an
 * independent problem over a vector w of g numbers:
 *
 *   base precision p_L
 *     greedy (section 2.2):  r_0 = w;  b_i = sign(r_{i-1}),
 *                            a_i = <r_{i-1}, b_i> / g,  r_i = r_{i-1} - a_i b_i
 *     T cycles:              a   <- LS(B, w)   = argmin_a |w - sum_i a_i b_i|^2
 *                            B   <- BS(a, w)   : every w_j takes the codes of
 *                                   the nearest of the 2^p levels sum_i +-a_i
 *   precision p = p_L+1 .. p_H  (planes 1..p-1 stay frozen)
 *     a^(p) <- [a^(p-1), 0],  b_p <- 0
 *     T cycles:              R   <- w - sum_{i<p} a_i b_i
 *                            b_p <- sign(R)
 *                            a   <- LS([b_1..b_p], w)
 *   The scale set of precision p is what a holds when its T cycles end.
 *
 * Readings taken where the paper leaves a choice:
 *   - sign(0) = +1.
 *   - Residual of the expansion step: the listing subtracts Dequant over all p
 *     planes, which from the second cycle on includes the new plane itself;
 *     section 2.2 defines the residual that initialises plane p as the one
 *     after p-1 planes, and the text of section 3.2 speaks of "the residual
 *     weights with the optimised scaling factors".  The default follows that
 *     (the new plane does not enter its own residual); `literal_residual`
 *     selects the listing's form so that tests can compare the two.
 *   - BS ties: the 2^p levels are enumerated with plane 1 as the most
 *     significant bit of the code index (bit set = +1), and the first strict
 *     minimum of |w_j - level| wins.
 *   - LS with linearly dependent planes: the normal equations are eliminated
 *     in plane order without pivoting; a plane whose pivot is not above 1e-9
 *     (an independent plane has a pivot of at least g^-(k-1)) gets scale 0.
 *   - Asymmetric scheme (section 4.1 names it; Algorithm 1 does not show it):
 *     the offset z is one more least-squares unknown whose basis vector is the
 *     all-ones vector, placed after the planes; greedy starts from
 *     z = mean(w), r_0 = w - z; levels and residuals include z.
 *
 * All arithmetic is IEEE double, sums run over the group from its first
 * column upwards, nothing is blocked or reordered, and the file is compiled
 * without floating-point contraction.  Weights arrive as the raw 16 bits of
 * IEEE binary16 values and are widened exactly.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define QMAX_P 4
#define QMAX_K (QMAX_P + 1)     /* planes + offset */

static double half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int expo = (h >> 10) & 0x1f;
    int frac = h & 0x3ff;
    double v;
    if (expo == 0) {
        v = ldexp((double)frac, -24);
    } else if (expo == 31) {
        v = frac ? NAN : INFINITY;
    } else {
        v = ldexp((double)(frac | 0x400), expo - 25);
    }
    return sign ? -v : v;
}

static double sign1(double v) { return v >= 0.0 ? 1.0 : -1.0; }

/*
 * Least squares over the columns basis[0..k-1] (each of length g):
 * minimise |w - sum_c coef[c] basis[c]|^2 through the normal equations
 * (section 2.2: a = (B^T B)^-1 B^T w), solved by Gaussian elimination in
 * column order without pivoting.
 */
static void least_squares(const double *const *basis, int k, const double *w, int64_t g, double *coef)
{
    double A[QMAX_K][QMAX_K], rhs[QMAX_K];
    int dead[QMAX_K];
    for (int a = 0; a < k; ++a) {
        for (int b = 0; b < k; ++b) {
            double s = 0.0;
            for (int64_t j = 0; j < g; ++j) s += basis[a][j] * basis[b][j];
            A[a][b] = s;
        }
        double s = 0.0;
        for (int64_t j = 0; j < g; ++j) s += basis[a][j] * w[j];
        rhs[a] = s;
    }
    for (int c = 0; c < k; ++c) {
        dead[c] = !(A[c][c] > 1e-9);
        if (dead[c]) continue;
        for (int r = c + 1; r < k; ++r) {
            double f = A[r][c] / A[c][c];
            for (int d = c; d < k; ++d) A[r][d] = A[r][d] - f * A[c][d];
            rhs[r] = rhs[r] - f * rhs[c];
        }
    }
    for (int c = k - 1; c >= 0; --c) {
        if (dead[c]) {
            coef[c] = 0.0;
            continue;
        }
        double s = rhs[c];
        for (int d = c + 1; d < k; ++d)
            if (!dead[d]) s = s - A[c][d] * coef[d];
        coef[c] = s / A[c][c];
    }
}

/* value of the level that the codes b[0..p-1][j] select: ((a_0 b_0 + a_1 b_1) + ...) + z */
static double level_of(const double *const *b, int p, const double *a, double z, int with_offset, int64_t j)
{
    double v = 0.0;
    for (int i = 0; i < p; ++i) v = (i == 0) ? a[0] * b[0][j] : v + a[i] * b[i][j];
    return with_offset ? v + z : v;
}

/*
 * One group.  w[g] in; b[i][j] (i < p_high) in {-1,+1} out; alpha_out[p - p_low][i] and
 * z_out[p - p_low] receive the scale set / offset of every precision p_low..p_high.
 */
static void quantize_group(const double *w, int64_t g, int p_low, int p_high, int T, int with_offset,
                           int literal_residual, double **b, double alpha_out[][QMAX_P], double *z_out)
{
    double a[QMAX_P] = {0.0, 0.0, 0.0, 0.0};
    double z = 0.0;
    double *r = (double *)malloc(sizeof(double) * (size_t)g);
    double *ones = (double *)malloc(sizeof(double) * (size_t)g);
    for (int64_t j = 0; j < g; ++j) ones[j] = 1.0;

    /* greedy initialisation at the base precision */
    if (with_offset) {
        double s = 0.0;
        for (int64_t j = 0; j < g; ++j) s += w[j];
        z = s / (double)g;
    }
    for (int64_t j = 0; j < g; ++j) r[j] = with_offset ? w[j] - z : w[j];
    for (int i = 0; i < p_low; ++i) {
        double s = 0.0;
        for (int64_t j = 0; j < g; ++j) {
            b[i][j] = sign1(r[j]);
            s += r[j] * b[i][j];
        }
        a[i] = s / (double)g;
        for (int64_t j = 0; j < g; ++j) r[j] = r[j] - a[i] * b[i][j];
    }

    for (int p = p_low; p <= p_high; ++p) {
        const double *basis[QMAX_K];
        for (int i = 0; i < p; ++i) basis[i] = b[i];
        basis[p] = ones;
        const int k = p + (with_offset ? 1 : 0);
        double coef[QMAX_K];
        if (p == p_low) {
            for (int t = 0; t < T; ++t) {
                least_squares(basis, k, w, g, coef);
                for (int i = 0; i < p; ++i) a[i] = coef[i];
                if (with_offset) z = coef[p];
                /* reassign the codes: nearest of the 2^p levels */
                double lev[1 << QMAX_P];
                for (int c = 0; c < (1 << p); ++c) {
                    double v = 0.0;
                    for (int i = 0; i < p; ++i) {
                        double term = ((c >> (p - 1 - i)) & 1) ? a[i] : -a[i];
                        v = (i == 0) ? term : v + term;
                    }
                    lev[c] = with_offset ? v + z : v;
                }
                for (int64_t j = 0; j < g; ++j) {
                    int best = 0;
                    double dbest = fabs(w[j] - lev[0]);
                    for (int c = 1; c < (1 << p); ++c) {
                        double d = fabs(w[j] - lev[c]);
                        if (d < dbest) {
                            dbest = d;
                            best = c;
                        }
                    }
                    for (int i = 0; i < p; ++i) b[i][j] = ((best >> (p - 1 - i)) & 1) ? 1.0 : -1.0;
                }
            }
        } else {
            a[p - 1] = 0.0;
            for (int64_t j = 0; j < g; ++j) b[p - 1][j] = 0.0;
            for (int t = 0; t < T; ++t) {
                for (int64_t j = 0; j < g; ++j) {
                    double deq = level_of((const double *const *)b, literal_residual ? p : p - 1, a, z, with_offset, j);
                    r[j] = w[j] - deq;
                }
                for (int64_t j = 0; j < g; ++j) b[p - 1][j] = sign1(r[j]);
                least_squares(basis, k, w, g, coef);
                for (int i = 0; i < p; ++i) a[i] = coef[i];
                if (with_offset) z = coef[p];
            }
        }
        for (int i = 0; i < QMAX_P; ++i) alpha_out[p - p_low][i] = (i < p) ? a[i] : 0.0;
        z_out[p - p_low] = z;
    }
    free(r);
    free(ones);
}

/*
 * W: binary16 bit patterns [m][n].  codes: int8 [p_high][m][n] in {-1,+1}.
 * scales: double, the sets of p = p_low..p_high one after another, set p laid out [p][m][n/group].
 * offsets: double [p_high-p_low+1][m][n/group], written only if with_offset.
 * Returns 0, or -1 on a bad argument.
 */
int bcq_oracle_quantize(const uint16_t *W, int64_t m, int64_t n, int64_t group, int p_low, int p_high, int T,
                        int with_offset, int literal_residual, int8_t *codes, double *scales, double *offsets)
{
    if (!W || !codes || !scales || (with_offset && !offsets)) return -1;
    if (m < 1 || n < 1 || group < 1 || n % group != 0) return -1;
    if (p_low < 1 || p_high < p_low || p_high > QMAX_P || T < 0 || (T < 1 && p_high > p_low)) return -1;
    const int64_t ngroups = n / group;
    int64_t set_base[QMAX_P + 1];
    {
        int64_t at = 0;
        for (int p = p_low; p <= p_high; ++p) {
            set_base[p] = at;
            at += (int64_t)p * m * ngroups;
        }
    }
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < m; ++r) {
        double *w = (double *)malloc(sizeof(double) * (size_t)group);
        double *bbuf = (double *)malloc(sizeof(double) * (size_t)group * QMAX_P);
        double *b[QMAX_P];
        for (int i = 0; i < QMAX_P; ++i) b[i] = bbuf + (int64_t)i * group;
        for (int64_t G = 0; G < ngroups; ++G) {
            for (int64_t j = 0; j < group; ++j) w[j] = half_to_double(W[r * n + G * group + j]);
            double alpha[QMAX_P][QMAX_P], z[QMAX_P];
            quantize_group(w, group, p_low, p_high, T, with_offset, literal_residual, b, alpha, z);
            for (int i = 0; i < p_high; ++i)
                for (int64_t j = 0; j < group; ++j)
                    codes[((int64_t)i * m + r) * n + G * group + j] = (int8_t)(b[i][j] > 0.0 ? 1 : -1);
            for (int p = p_low; p <= p_high; ++p) {
                for (int i = 0; i < p; ++i) scales[set_base[p] + ((int64_t)i * m + r) * ngroups + G] = alpha[p - p_low][i];
                if (with_offset) offsets[((int64_t)(p - p_low) * m + r) * ngroups + G] = z[p - p_low];
            }
        }
        free(w);
        free(bbuf);
    }
    return 0;
}
