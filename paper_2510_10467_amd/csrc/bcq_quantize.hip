// Offline quantiser: Algorithm 1 (section 3.2, "AnyBCQ initialization and progressive precision
// expansion") with the building blocks of section 2.2 (greedy initialisation, least-squares scales,
// reassignment of the codes to the nearest level), group-wise (section 4.1: g = 128).
//
// Every (row, group) is an independent problem over g weights, so the work is spread as
//   one lane  = one 32-column word of one group: its 32 weights live in registers as doubles, its codes
//               are the bits of one uint32 per plane, exactly the word the packed format stores;
//   g/32 adjacent lanes = one group; they meet only in sums (lane-exchange adds).
// Why doubles: the weights are binary16 values, so every sum of +-w over a group is EXACT in double
// (multiples of 2^-24 below 2^24) and so are the integer Gram entries <b_i, b_k> = g - 2 popcount(b_i ^ b_k).
// What is left of the arithmetic - the elimination of a k x k system, the level values, one subtraction
// per residual - is a fixed sequence of scalar operations with no freedom of order, so codes come out the
// same on any machine that follows IEEE double without contraction.  Nothing here is bound by memory:
// a weight is read once and costs some thousand operations.
//
// Choices where the algorithm leaves room (they decide codes, so they are part of the definition):
//   sign(0) = +1;  the residual that re-signs the new plane p is taken after the p-1 frozen planes under
//   the current scales (section 2.2's residual);  code reassignment enumerates the 2^p levels with the first
//   plane as the most significant bit of the index and keeps the first strict minimum of |w - level|;  the
//   normal equations are eliminated in plane order without pivoting, and a plane whose pivot is not above
//   1e-9 (it depends on the planes before it) gets scale 0;  in the asymmetric scheme the offset is one
//   more unknown with the all-ones basis vector, placed last, greedy starting from the group mean.
#include <hip/hip_runtime.h>

#include "bcq_internal.hpp"

#pragma clang fp contract(off)

namespace bcq {
namespace {

constexpr int kMaxP = 4;

struct QuantParams {
    const _Float16 *w;                   // [m][n] = [total_words][32]
    uint32_t *planes;                    // [p_high][total_words]
    _Float16 *scales[kMaxP + 1];         // [p]: [p][total_groups]
    _Float16 *offsets[kMaxP + 1];        // [p]: [total_groups]
    uint64_t total_words;                // m * n / 32
    uint64_t total_groups;               // m * n / group
    int p_low, p_high, cycles;
};

typedef _Float16 half8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ double flip(double v, uint32_t sign_mask)   // sign_mask: 0 or 0x80000000
{
    return __builtin_bit_cast(double, __builtin_bit_cast(uint64_t, v) ^ ((uint64_t)sign_mask << 32));
}

// 0x80000000 where column j of the word is -1 (bit clear); nw is the complemented word
__device__ __forceinline__ uint32_t minus_mask(uint32_t nw, int j) { return (nw << (31 - j)) & 0x80000000u; }

template <int LANES>
__device__ __forceinline__ double group_sum(double v)
{
#pragma unroll
    for (int mask = 1; mask < LANES; mask <<= 1) v += __shfl_xor(v, mask, 64);
    return v;
}

template <int LANES>
__device__ __forceinline__ int group_sum(int v)
{
#pragma unroll
    for (int mask = 1; mask < LANES; mask <<= 1) v += __shfl_xor(v, mask, 64);
    return v;
}

// Correctly rounded double -> binary16: through a float rounded to odd (truncate, then set the last bit
// if anything was lost), which a second rounding to the 11-bit format cannot get wrong.
__device__ __forceinline__ _Float16 to_half(double d)
{
    float f = (float)d;
    const double back = (double)f;
    if (back != d) {
        uint32_t u = __builtin_bit_cast(uint32_t, f);
        if (__builtin_fabs(back) > __builtin_fabs(d)) u -= 1;     // step towards zero
        f = __builtin_bit_cast(float, u | 1u);
    }
    return (_Float16)f;
}

// Least squares through the normal equations, eliminated in order without pivoting.
// A is the full symmetric Gram matrix on entry.
template <int K>
__device__ __forceinline__ void solve(double (&A)[K][K], double (&rhs)[K], double (&coef)[K])
{
    bool dead[K];
#pragma unroll
    for (int c = 0; c < K; ++c) {
        dead[c] = !(A[c][c] > 1e-9);
        if (!dead[c]) {
#pragma unroll
            for (int r = c + 1; r < K; ++r) {
                const double f = A[r][c] / A[c][c];
#pragma unroll
                for (int d = c + 1; d < K; ++d) A[r][d] = A[r][d] - f * A[c][d];
                rhs[r] = rhs[r] - f * rhs[c];
            }
        }
    }
#pragma unroll
    for (int c = K - 1; c >= 0; --c) {
        if (dead[c]) {
            coef[c] = 0.0;
        } else {
            double s = rhs[c];
#pragma unroll
            for (int d = c + 1; d < K; ++d)
                if (!dead[d]) s = s - A[c][d] * coef[d];
            coef[c] = s / A[c][c];
        }
    }
}

// State of one lane: its 32 weights, its word of every plane, and the group's current scales / offset
// (the same in all lanes of a group).
struct Lane {
    double w[32];
    uint32_t word[kMaxP];
    double alpha[kMaxP];
    double z;
};

// Gram matrix and right-hand side of planes 0..P-1 (and the ones vector when OFFSET), then the solve.
// rhs_w[i] = <w, b_i> over the group (exact), sum_w = <w, 1>.
template <int P, int LANES, bool OFFSET>
__device__ __forceinline__ void least_squares(Lane &s, const double (&rhs_w)[kMaxP], double sum_w)
{
    constexpr int K = P + (OFFSET ? 1 : 0);
    constexpr double g = 32.0 * LANES;
    double A[K][K], rhs[K], coef[K];
#pragma unroll
    for (int i = 0; i < P; ++i) {
        A[i][i] = g;
        rhs[i] = rhs_w[i];
#pragma unroll
        for (int k = i + 1; k < P; ++k) {
            const int differ = group_sum<LANES>((int)__builtin_popcount(s.word[i] ^ s.word[k]));
            A[i][k] = A[k][i] = g - 2.0 * (double)differ;
        }
        if constexpr (OFFSET) {
            const int plus = group_sum<LANES>((int)__builtin_popcount(s.word[i]));
            A[i][P] = A[P][i] = 2.0 * (double)plus - g;
        }
    }
    if constexpr (OFFSET) {
        A[P][P] = g;
        rhs[P] = sum_w;
    }
    solve<K>(A, rhs, coef);
#pragma unroll
    for (int i = 0; i < P; ++i) s.alpha[i] = coef[i];
    if constexpr (OFFSET) s.z = coef[P];
}

// <w, b_i> over the group for plane i
template <int LANES>
__device__ __forceinline__ double signed_sum(const Lane &s, int i)
{
    const uint32_t nw = ~s.word[i];
    double acc = 0.0;
#pragma unroll
    for (int j = 0; j < 32; ++j) acc += flip(s.w[j], minus_mask(nw, j));
    return group_sum<LANES>(acc);
}

// Greedy plane I: b_I = sign(r_{I-1}), a_I = <r_{I-1}, b_I> / g, with r_{I-1} = ((w - z) - a_0 b_0) - ...
template <int I, int LANES, bool OFFSET>
__device__ __forceinline__ void greedy_plane(Lane &s)
{
    uint32_t nw[kMaxP];
#pragma unroll
    for (int i = 0; i < kMaxP; ++i) nw[i] = ~s.word[i];
    double acc = 0.0;
    uint32_t bits = 0;
#pragma unroll
    for (int j = 0; j < 32; ++j) {
        double r = OFFSET ? s.w[j] - s.z : s.w[j];
#pragma unroll
        for (int i = 0; i < I; ++i) r = r - flip(s.alpha[i], minus_mask(nw[i], j));
        const bool plus = r >= 0.0;
        bits |= plus ? (1u << j) : 0u;
        acc += plus ? r : -r;
    }
    s.word[I] = bits;
    s.alpha[I] = group_sum<LANES>(acc) / (32.0 * LANES);
}

// T cycles at the base precision P: LS, then every weight takes the codes of its nearest level.
template <int P, int LANES, bool OFFSET>
__device__ __forceinline__ void base_stage(Lane &s, int cycles, double sum_w)
{
    for (int t = 0; t < cycles; ++t) {
        double rhs_w[kMaxP] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
        for (int i = 0; i < P; ++i) rhs_w[i] = signed_sum<LANES>(s, i);
        least_squares<P, LANES, OFFSET>(s, rhs_w, sum_w);
        double lev[1 << P];
#pragma unroll
        for (int c = 0; c < (1 << P); ++c) {
            double v = ((c >> (P - 1)) & 1) ? s.alpha[0] : -s.alpha[0];
#pragma unroll
            for (int i = 1; i < P; ++i) v = v + (((c >> (P - 1 - i)) & 1) ? s.alpha[i] : -s.alpha[i]);
            lev[c] = OFFSET ? v + s.z : v;
        }
        uint32_t word[P];
#pragma unroll
        for (int i = 0; i < P; ++i) word[i] = 0;
#pragma unroll
        for (int j = 0; j < 32; ++j) {
            int best = 0;
            double dbest = __builtin_fabs(s.w[j] - lev[0]);
#pragma unroll
            for (int c = 1; c < (1 << P); ++c) {
                const double d = __builtin_fabs(s.w[j] - lev[c]);
                const bool better = d < dbest;
                dbest = better ? d : dbest;
                best = better ? c : best;
            }
#pragma unroll
            for (int i = 0; i < P; ++i) word[i] |= (uint32_t)((best >> (P - 1 - i)) & 1) << j;
        }
#pragma unroll
        for (int i = 0; i < P; ++i) s.word[i] = word[i];
    }
}

// The same for P = 2, the base precision of the paper's experiments, as a tournament: the nearer of
// levels 0/1, the nearer of levels 2/3, then the nearer of the two winners, the lower index winning ties
// at every node (which is the first strict minimum of the enumeration).  The signed sums <w, b_i> that
// the next cycle's LS needs are gathered while the codes are chosen.
template <int LANES, bool OFFSET>
__device__ __forceinline__ void base_stage_two(Lane &s, int cycles, double sum_w)
{
    double rhs_w[kMaxP] = {0.0, 0.0, 0.0, 0.0};
    rhs_w[0] = signed_sum<LANES>(s, 0);
    rhs_w[1] = signed_sum<LANES>(s, 1);
    for (int t = 0; t < cycles; ++t) {
        least_squares<2, LANES, OFFSET>(s, rhs_w, sum_w);
        double lev[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const double v = ((c & 2) ? s.alpha[0] : -s.alpha[0]) + ((c & 1) ? s.alpha[1] : -s.alpha[1]);
            lev[c] = OFFSET ? v + s.z : v;
        }
        uint32_t word0 = 0, word1 = 0;
        double acc0[2] = {0.0, 0.0}, acc1[2] = {0.0, 0.0};
#pragma unroll
        for (int j = 0; j < 32; ++j) {
            const double wj = s.w[j];
            const double d0 = __builtin_fabs(wj - lev[0]), d1 = __builtin_fabs(wj - lev[1]);
            const double d2 = __builtin_fabs(wj - lev[2]), d3 = __builtin_fabs(wj - lev[3]);
            const bool c01 = d1 < d0, c23 = d3 < d2;
            const double m01 = __builtin_fmin(d0, d1), m23 = __builtin_fmin(d2, d3);
            const bool top = m23 < m01;                 // plane 0: +1 for levels 2, 3
            const bool low = top ? c23 : c01;           // plane 1
            word0 |= top ? (1u << j) : 0u;
            word1 |= low ? (1u << j) : 0u;
            acc0[j & 1] += top ? wj : -wj;
            acc1[j & 1] += low ? wj : -wj;
        }
        s.word[0] = word0;
        s.word[1] = word1;
        rhs_w[0] = group_sum<LANES>(acc0[0] + acc0[1]);
        rhs_w[1] = group_sum<LANES>(acc1[0] + acc1[1]);
    }
}

// Expansion to precision P: planes 0..P-2 frozen; T cycles of residual -> sign -> LS.
// The frozen codes of a column select one of 2^(P-1) levels; each cycle the lanes of a group write those
// levels into the group's LDS table (`table`, 8 doubles) and every column reads its own back.  The table
// is private to lanes of one wave, whose LDS accesses complete in program order.
// LISTING: the residual as Algorithm 1 prints it, R = W - Dequant over all P planes: the new plane's own term
// alpha_P b_P (zero in the first cycle, where both start as zero) is taken out too, in the order
// ((a_1 b_1 + ... + a_{P-1} b_{P-1}) + a_P b_P) + z.
template <int P, int LANES, bool OFFSET, bool LISTING>
__device__ __forceinline__ void expand_stage(Lane &s, int cycles, double sum_w, double *table, int lane_in_group)
{
    constexpr int NL = 1 << (P - 1);
    double rhs_w[kMaxP] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int i = 0; i < P - 1; ++i) rhs_w[i] = signed_sum<LANES>(s, i);     // frozen planes: once
    // byte (j & 3) of pick[j >> 2]: eight times the level index of column j (plane 0 = most significant bit)
    uint32_t pick[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        uint32_t v = 0;
#pragma unroll
        for (int i = 0; i < P - 1; ++i) {
            // bits 4k..4k+3 of the word spread to bit (3 + P-2-i) of bytes 0..3
            const uint32_t nib = (s.word[i] >> (4 * k)) & 0xfu;
            const uint32_t spread = (nib & 1u) | ((nib & 2u) << 7) | ((nib & 4u) << 14) | ((nib & 8u) << 21);
            v |= spread << (3 + (P - 2 - i));
        }
        pick[k] = v;
    }
    s.alpha[P - 1] = 0.0;
    for (int t = 0; t < cycles; ++t) {
        for (int c = lane_in_group; c < NL; c += LANES) {
            double v = ((c >> (P - 2)) & 1) ? s.alpha[0] : -s.alpha[0];
#pragma unroll
            for (int i = 1; i < P - 1; ++i) v = v + (((c >> (P - 2 - i)) & 1) ? s.alpha[i] : -s.alpha[i]);
            table[c] = (OFFSET && !LISTING) ? v + s.z : v;
        }
        const uint32_t own = s.word[P - 1];              // the new plane's codes of the previous cycle
        const double own_scale = s.alpha[P - 1];
        __builtin_amdgcn_wave_barrier();
        double acc[2] = {0.0, 0.0};
        uint32_t minus = 0;                              // sign bits of the residuals, column 31 first
#pragma unroll
        for (int j = 31; j >= 0; --j) {
            const uint32_t off = (pick[j >> 2] >> (8 * (j & 3))) & 0xffu;
            double lev = *reinterpret_cast<const double *>(reinterpret_cast<const char *>(table) + off);
            if constexpr (LISTING) {
                const double own_term = t == 0 ? 0.0 : flip(own_scale, ((own >> j) & 1u) ? 0u : 0x80000000u);
                lev = lev + own_term;
                if constexpr (OFFSET) lev = lev + s.z;
            }
            const double r = s.w[j] - lev;               // never -0: the weights hold no -0
            const uint32_t rhi = (uint32_t)(__builtin_bit_cast(uint64_t, r) >> 32);
            minus = __builtin_amdgcn_alignbit(minus, rhi, 31);
            acc[j & 1] += flip(s.w[j], rhi & 0x80000000u);
        }
        __builtin_amdgcn_wave_barrier();
        s.word[P - 1] = ~minus;
        rhs_w[P - 1] = group_sum<LANES>(acc[0] + acc[1]);
        least_squares<P, LANES, OFFSET>(s, rhs_w, sum_w);
    }
}

template <int LANES, bool OFFSET>
__device__ __forceinline__ void store_set(const QuantParams &a, const Lane &s, int p, uint64_t gid, bool writer)
{
    if (!writer) return;
    _Float16 *set = a.scales[p];
#pragma unroll
    for (int i = 0; i < kMaxP; ++i)
        if (i < p) set[(uint64_t)i * a.total_groups + gid] = to_half(s.alpha[i]);
    if constexpr (OFFSET) a.offsets[p][gid] = to_half(s.z);
}

template <int LANES, bool OFFSET, bool LISTING>
__global__ __launch_bounds__(256) void quantize_kernel(QuantParams a)
{
    __shared__ double tables[(256 / LANES) * 8];
    double *table = tables + (threadIdx.x / LANES) * 8;
    const int lane_in_group = threadIdx.x % LANES;
    const uint64_t gw = (uint64_t)blockIdx.x * 256 + threadIdx.x;      // this lane's word
    const bool valid = gw < a.total_words;                              // whole groups are valid or not
    const uint64_t src = valid ? gw : a.total_words - 1;
    Lane s;
    {
        const half8 *wp = reinterpret_cast<const half8 *>(a.w + src * 32);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const half8 v = wp[k];
#pragma unroll
            for (int e = 0; e < 8; ++e) s.w[8 * k + e] = (double)v[e] + 0.0;      // -0 becomes +0
        }
    }
#pragma unroll
    for (int i = 0; i < kMaxP; ++i) {
        s.word[i] = 0;
        s.alpha[i] = 0.0;
    }
    s.z = 0.0;
    double sum_w = 0.0;
#pragma unroll
    for (int j = 0; j < 32; ++j) sum_w += s.w[j];
    sum_w = group_sum<LANES>(sum_w);
    if constexpr (OFFSET) s.z = sum_w / (32.0 * LANES);

    const int p_low = a.p_low;
    greedy_plane<0, LANES, OFFSET>(s);
    if (p_low > 1) greedy_plane<1, LANES, OFFSET>(s);
    if (p_low > 2) greedy_plane<2, LANES, OFFSET>(s);
    if (p_low > 3) greedy_plane<3, LANES, OFFSET>(s);
    switch (p_low) {
    case 1: base_stage<1, LANES, OFFSET>(s, a.cycles, sum_w); break;
    case 2: base_stage_two<LANES, OFFSET>(s, a.cycles, sum_w); break;
    case 3: base_stage<3, LANES, OFFSET>(s, a.cycles, sum_w); break;
    default: base_stage<4, LANES, OFFSET>(s, a.cycles, sum_w); break;
    }
    const uint64_t gid = gw / LANES;
    const bool writer = valid && (threadIdx.x % LANES) == 0;
    store_set<LANES, OFFSET>(a, s, p_low, gid, writer);
    for (int p = p_low + 1; p <= a.p_high; ++p) {
        switch (p) {
        case 2: expand_stage<2, LANES, OFFSET, LISTING>(s, a.cycles, sum_w, table, lane_in_group); break;
        case 3: expand_stage<3, LANES, OFFSET, LISTING>(s, a.cycles, sum_w, table, lane_in_group); break;
        default: expand_stage<4, LANES, OFFSET, LISTING>(s, a.cycles, sum_w, table, lane_in_group); break;
        }
        store_set<LANES, OFFSET>(a, s, p, gid, writer);
    }
    if (valid) {
#pragma unroll
        for (int i = 0; i < kMaxP; ++i)
            if (i < a.p_high) a.planes[(uint64_t)i * a.total_words + gw] = s.word[i];
    }
}

template <int LANES>
hipError_t launch_lanes(const QuantParams &pr, bool offset, bool listing, hipStream_t stream)
{
    const unsigned blocks = (unsigned)((pr.total_words + 255) / 256);
    if (listing) {
        if (offset) hipLaunchKernelGGL((quantize_kernel<LANES, true, true>), dim3(blocks), dim3(256), 0, stream, pr);
        else hipLaunchKernelGGL((quantize_kernel<LANES, false, true>), dim3(blocks), dim3(256), 0, stream, pr);
    } else {
        if (offset) hipLaunchKernelGGL((quantize_kernel<LANES, true, false>), dim3(blocks), dim3(256), 0, stream, pr);
        else hipLaunchKernelGGL((quantize_kernel<LANES, false, false>), dim3(blocks), dim3(256), 0, stream, pr);
    }
    return hipGetLastError();
}

}  // namespace

bool quantize_supports(int64_t m, int64_t n, int group)
{
    const bool group_ok = group == 32 || group == 64 || group == 128 || group == 256;
    // one thread per 32-column word, 256 per workgroup, at most 2^31 - 1 workgroups
    return group_ok && m >= 1 && n >= group && n % group == 0 && ((m * n) / 32 + 255) / 256 < (int64_t(1) << 31);
}

hipError_t quantize_launch(const _Float16 *w, int p_low, int p_high, int cycles, uint32_t *planes, _Float16 *const *scales_by_p,
                           _Float16 *const *offsets_by_p, int64_t m, int64_t n, int group, bool listing_residual, hipStream_t stream)
{
    QuantParams pr{};
    pr.w = w;
    pr.planes = planes;
    for (int p = p_low; p <= p_high; ++p) {
        pr.scales[p] = scales_by_p[p];
        pr.offsets[p] = offsets_by_p ? offsets_by_p[p] : nullptr;
    }
    pr.total_words = (uint64_t)(m * n / 32);
    pr.total_groups = (uint64_t)(m * n / group);
    pr.p_low = p_low;
    pr.p_high = p_high;
    pr.cycles = cycles;
    const bool offset = offsets_by_p != nullptr;
    switch (group) {
    case 32: return launch_lanes<1>(pr, offset, listing_residual, stream);
    case 64: return launch_lanes<2>(pr, offset, listing_residual, stream);
    case 128: return launch_lanes<4>(pr, offset, listing_residual, stream);
    default: return launch_lanes<8>(pr, offset, listing_residual, stream);
    }
}

}  // namespace bcq
