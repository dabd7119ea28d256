// Small-batch kernel: bit-planes go straight into the CDNA4 FP4 matrix pipe.
//
// Section 3.3 forms B_i x per plane by adding and subtracting activations and
// keeps the regime memory-bound.  On gfx950 the vector ALU cannot add/subtract
// fast enough to keep up with 8 TB/s of one-bit weights, so the sign-accumulate
// of one whole scale group (16 rows x 128 columns x 1 plane = 2048 weight bits)
// is issued as ONE v_mfma_f32_16x16x128_f8f6f4:
//
//   * weight operand (MFMA "B", 16 columns = 16 weight rows): every weight bit
//     becomes an FP4 (E2M1) code 0x2 | sign, i.e. exactly +-1.  Four AND/OR
//     (three of them after a shift) turn a 32-bit plane word into the lane's four
//     operand registers.  Which bit lands in which K slot is a fixed
//     permutation, mirrored on the activation side.
//   * activation operand (MFMA "A", 16 rows): binary16 activations are split
//     EXACTLY into four E5M2 terms (E5M2 is the top byte of binary16, so
//     x = t0 + t1 + t2 + t3 with t_k = top byte of the running remainder).  Row
//     4*b + k of the operand holds term k of request b, so one instruction
//     serves up to four requests.  The split is done once per workgroup and
//     parked in LDS in operand-register order.
//   * result: lane (row r, request b) receives the four term sums of its own
//     row, adds them, multiplies by alpha_i[r][group] of ITS request's
//     precision, and accumulates in fp32.  Requests at different precisions
//     share the plane sweep; a lane simply stops accumulating at p_b.
//
// Work split: a workgroup owns RB blocks of 16 rows and the whole K range;
// wave (rb, ks) handles K slice ks (1024 columns) of row block rb, issues all
// of its plane and scale loads up front (128-bit, 128 contiguous bytes per row
// and plane), and the KS partial sums are combined through LDS in a fixed
// order, so results are deterministic and no global scratch is needed.
#include <hip/hip_runtime.h>

#include "bcq_internal.hpp"

namespace bcq {
namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef unsigned v2u __attribute__((ext_vector_type(2)));
typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kSliceCols = 1024;            // columns per wave and chunk: 8 groups of 128
constexpr int kSliceGroups = 8;
constexpr int kMaxBatchTile = 4;            // requests per MFMA (4 E5M2 terms each = 16 operand rows)
constexpr int kMaxP = 4;                    // planes this kernel keeps in registers

// Byte offset inside the LDS activation image.
//   g: group within the chunk, h: operand register half (0: regs 0-3, 1: regs 4-7),
//   qa: lane quarter, row: 4*request + term, nrows = 4 * requests in the tile.
__device__ __forceinline__ int image_offset(int g, int h, int qa, int row, int nrows)
{
    return ((((g * 2 + h) * 4 + qa) * nrows) + row) * 16;
}

// 4x4 transpose of one dword per register across the four lane quarters
// (lanes l, l+16, l+32, l+48): afterwards register t of quarter q holds what
// register q of quarter t held.
__device__ __forceinline__ void quarter_transpose(uint32_t &v0, uint32_t &v1, uint32_t &v2, uint32_t &v3)
{
    v2u s;
    s = __builtin_amdgcn_permlane32_swap(v0, v2, false, false); v0 = s[0]; v2 = s[1];
    s = __builtin_amdgcn_permlane32_swap(v1, v3, false, false); v1 = s[0]; v3 = s[1];
    s = __builtin_amdgcn_permlane16_swap(v0, v1, false, false); v0 = s[0]; v1 = s[1];
    s = __builtin_amdgcn_permlane16_swap(v2, v3, false, false); v2 = s[0]; v3 = s[1];
}

// Sweep of one wave over its K slices for PH planes; returns this lane's partial sum.
//   p_mine   precision of the request this lane reports on (0: none)
//   sptr     scale set of that precision (any valid set when p_mine == 0)
template <int PH>
__device__ __forceinline__ float sweep(const GemmArgs &a, unsigned char *lds, int KS, int nchunk, int ks, int q, int lane,
                                       int tid, int nthreads, int b0, int nb, int64_t row, int p_mine,
                                       const _Float16 *sptr)
{
    const int nrows = 4 * nb;
    const int words = (int)(a.n >> 5);
    const int ngroups = (int)(a.n >> 7);
    const int nslices = (int)(a.n / kSliceCols);
    const int chunk_cols = KS * kSliceCols;
    const int image_bytes = KS * kSliceGroups * 128 * nrows;      // followed by 16 zero bytes, then the staging area
    const int stage_off = image_bytes + 16;
    const int arow = lane & 15;

    if (tid < 4) reinterpret_cast<uint32_t *>(lds + image_bytes)[tid] = 0u;

    float acc = 0.f;
    for (int chunk = 0; chunk < nchunk; ++chunk) {
        const int slice = chunk * KS + ks;                         // global K slice of this wave
        const bool slice_ok = slice < nslices;
        const int slice_c = slice_ok ? slice : nslices - 1;
        const int p_eff = slice_ok ? p_mine : 0;

        // ---- 1. issue every plane and scale load of this wave, unconditionally -------------
        u32x4 wlo[PH], whi[PH];
        u32x4 sc[PH];
#pragma unroll
        for (int i = 0; i < PH; ++i) {
            const u32x4 *wp = reinterpret_cast<const u32x4 *>(
                a.planes + ((int64_t)i * a.m + row) * words + slice_c * (kSliceCols / 32) + q * 8);
            wlo[i] = __builtin_nontemporal_load(wp);                // group 2q of the slice
            whi[i] = __builtin_nontemporal_load(wp + 1);            // group 2q + 1
            const int ii = min(i, max(p_mine, 1) - 1);             // stay inside the lane's own scale set
            sc[i] = *reinterpret_cast<const u32x4 *>(sptr + ((int64_t)ii * a.m + row) * ngroups + slice_c * kSliceGroups);
        }

        // ---- 2. workgroup builds the activation image of this chunk ------------------------
        if (chunk > 0) __syncthreads();                            // previous image and staging no longer read
        {
            // 2a. stage the chunk's activations in LDS, 16 bytes per thread and trip, coalesced
            const int64_t col0 = (int64_t)chunk * chunk_cols;
            const int per_req = chunk_cols / 8;                     // 16-byte units per request
            const int total = nb * per_req;
            u32x4 *stage = reinterpret_cast<u32x4 *>(lds + stage_off);
            for (int base = 0; base < total; base += 2 * nthreads) {
                u32x4 xv[2];
                int idx[2];
#pragma unroll
                for (int k2 = 0; k2 < 2; ++k2) {                    // both loads in flight before any use
                    idx[k2] = base + k2 * nthreads + tid;
                    const int ic = min(idx[k2], total - 1);
                    const int b = ic / per_req;
                    const int64_t col = col0 + (int64_t)(ic - b * per_req) * 8;
                    xv[k2] = *reinterpret_cast<const u32x4 *>(a.x + (int64_t)(b0 + b) * a.n + min(col, a.n - 8));
                    if (col >= a.n) xv[k2] = u32x4{0, 0, 0, 0};     // ragged last chunk: columns past n are zero
                }
#pragma unroll
                for (int k2 = 0; k2 < 2; ++k2)
                    if (idx[k2] < total) stage[idx[k2]] = xv[k2];
            }
            __syncthreads();
            // 2b. one task = four columns (stride 4) of one request -> one dword in each of the four term rows
            const unsigned short *xs = reinterpret_cast<const unsigned short *>(lds + stage_off);
            const int ntask = nb * KS * 256;
            for (int task = tid; task < ntask; task += nthreads) {
                const int dw = task & 3, qa = (task >> 2) & 3, h = (task >> 4) & 1;
                const int rest = task >> 5;
                const int b = rest % nb, g = rest / nb;
                // operand byte 8z + tt of lane quarter qa pairs with column 64h + 32(qa>>1) + 4tt + 3 - (2(qa&1) + z)
                const int z = dw >> 1;
                const int cl0 = 64 * h + 32 * (qa >> 1) + 16 * (dw & 1) + 3 - (2 * (qa & 1) + z);
                const unsigned short *src = xs + b * chunk_cols + g * 128 + cl0;
                const uint32_t v01 = (uint32_t)src[0] | ((uint32_t)src[4] << 16);
                const uint32_t v23 = (uint32_t)src[8] | ((uint32_t)src[12] << 16);
                // exact split into four E5M2 terms: top bytes of the running binary16 remainders
                h2 r01 = __builtin_bit_cast(h2, v01), r23 = __builtin_bit_cast(h2, v23);
                uint32_t *dst = reinterpret_cast<uint32_t *>(lds + image_offset(g, h, qa, 4 * b, nrows) + 4 * dw);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t t01 = __builtin_bit_cast(uint32_t, r01) & 0xFF00FF00u;
                    const uint32_t t23 = __builtin_bit_cast(uint32_t, r23) & 0xFF00FF00u;
                    r01 = r01 - __builtin_bit_cast(h2, t01);
                    r23 = r23 - __builtin_bit_cast(h2, t23);
                    dst[4 * j] = __builtin_amdgcn_perm(t23, t01, 0x07050301u);   // bytes: col0, col0+4, col0+8, col0+12
                }
            }
        }
        __syncthreads();

        // scales of planes this lane must not use (beyond its precision, or a slice past the end) become zero
#pragma unroll
        for (int i = 0; i < PH; ++i)
            if (!(i < p_eff)) sc[i] = u32x4{0, 0, 0, 0};

        // ---- 3. per group: expand plane words, one MFMA per (group, plane), scale, accumulate
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            // after the transpose, register t of quarter q is dword q of group 2t + j of the slice
            uint32_t wt[PH][4];
#pragma unroll
            for (int i = 0; i < PH; ++i) {
                const u32x4 src = j ? whi[i] : wlo[i];
                wt[i][0] = src.x; wt[i][1] = src.y; wt[i][2] = src.z; wt[i][3] = src.w;
                quarter_transpose(wt[i][0], wt[i][1], wt[i][2], wt[i][3]);
            }
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int gl = 2 * t + j;                           // group inside the slice
                const int gc = ks * kSliceGroups + gl;
                // lanes whose operand row is unused read the 16 zero bytes behind the image
                const int o_lo = arow < nrows ? image_offset(gc, 0, q, arow, nrows) : image_bytes;
                const int o_hi = arow < nrows ? image_offset(gc, 1, q, arow, nrows) : image_bytes;
                const u32x4 lo = *reinterpret_cast<const u32x4 *>(lds + o_lo);
                const u32x4 hi = *reinterpret_cast<const u32x4 *>(lds + o_hi);
                const v8i xa = {(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
#pragma unroll
                for (int i = 0; i < PH; ++i) {
                    const uint32_t w = wt[i][t];
                    v8i wb = {0, 0, 0, 0, 0, 0, 0, 0};
                    wb[0] = (int)((w & 0x88888888u) | 0x22222222u);
                    wb[1] = (int)(((w << 1) & 0x88888888u) | 0x22222222u);
                    wb[2] = (int)(((w << 2) & 0x88888888u) | 0x22222222u);
                    wb[3] = (int)(((w << 3) & 0x88888888u) | 0x22222222u);
                    v4f d = {0.f, 0.f, 0.f, 0.f};
                    // A: E5M2 activation terms (cbsz = 1), B: FP4 signs (blgp = 4), no block scaling
                    d = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(xa, wb, d, 1, 4, 0, 0, 0, 0);
                    const uint32_t sw = sc[i][gl >> 1];
                    const float alpha = (float)__builtin_bit_cast(_Float16, (unsigned short)((gl & 1) ? (sw >> 16) : (sw & 0xffffu)));
                    const float s = (d[0] + d[1]) + (d[2] + d[3]);
                    // the FP4 sign bit is set for weight bit 1 (= +1), so the instruction returns -(B_i x)
                    acc = fmaf(-alpha, s, acc);
                }
            }
        }
    }
    return acc;
}

template <int P, bool MIXED>
__global__ __launch_bounds__(1024) void plane_mfma_kernel(GemmArgs a, int KS, int RB, int nchunk)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

    const int tid = threadIdx.x;
    const int nthreads = blockDim.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int ks = wave % KS;                 // K slice of this wave inside a chunk
    const int rb = wave / KS;                 // row block of this wave inside the workgroup
    const int q = lane >> 4;                  // lane quarter: K sub-block on the weight side, request on the output side
    const int b0 = blockIdx.y * kMaxBatchTile;
    const int nb = min(kMaxBatchTile, a.batch - b0);

    int64_t row = ((int64_t)blockIdx.x * RB + rb) * 16 + (lane & 15);
    const bool row_ok = row < a.m;
    if (!row_ok) row = a.m - 1;               // keep loads in bounds; the result is discarded

    float acc = 0.f;
    if constexpr (!MIXED) {
        acc = sweep<P>(a, lds, KS, nchunk, ks, q, lane, tid, nthreads, b0, nb, row, P, a.scales[P]);
    } else {
        // precision of the request this lane reports on, and the deepest plane any request of the tile needs
        int p_mine = 0, p_hi = 0;
        for (int b = 0; b < nb; ++b) {
            const int pb = request_precision(a, b0 + b);
            p_hi = max(p_hi, pb);
            if (b == q) p_mine = pb;
        }
        const _Float16 *sptr = a.scales[p_mine > 0 ? p_mine : p_hi];
        // one straight-line sweep per possible depth: only planes 0 .. p_hi-1 are fetched
        switch (p_hi) {
        case 1: acc = sweep<1>(a, lds, KS, nchunk, ks, q, lane, tid, nthreads, b0, nb, row, p_mine, sptr); break;
        case 2: if constexpr (P >= 2) acc = sweep<2>(a, lds, KS, nchunk, ks, q, lane, tid, nthreads, b0, nb, row, p_mine, sptr); break;
        case 3: if constexpr (P >= 3) acc = sweep<3>(a, lds, KS, nchunk, ks, q, lane, tid, nthreads, b0, nb, row, p_mine, sptr); break;
        case 4: if constexpr (P >= 4) acc = sweep<4>(a, lds, KS, nchunk, ks, q, lane, tid, nthreads, b0, nb, row, p_mine, sptr); break;
        default: break;                                            // no request has a scale set: zeros
        }
    }

    // ---- combine the KS partial sums of each row block in a fixed order, store binary16 -----
    __syncthreads();
    float *red = reinterpret_cast<float *>(lds);
    red[wave * 64 + lane] = acc;
    __syncthreads();
    if (ks == 0) {
        float v = 0.f;
        for (int k = 0; k < KS; ++k) v += red[(rb * KS + k) * 64 + lane];
        if (row_ok && q < nb) a.y[(int64_t)(b0 + q) * a.m + row] = (_Float16)v;
    }
}

struct Plan {
    int KS, RB, nchunk;
    size_t lds_bytes;
};

constexpr size_t kLdsBudget = 128 * 1024;     // of the 160 KiB per CU

Plan make_plan(const GemmArgs &a)
{
    const int nslices = (int)(a.n / kSliceCols);
    const int nb = a.batch < kMaxBatchTile ? a.batch : kMaxBatchTile;
    // per slice and request: 4 KiB of operand image + 2 KiB of staged activations
    int ks_cap = (int)(kLdsBudget / (6144 * (size_t)nb));
    if (ks_cap > 16) ks_cap = 16;
    int KS = 1;
    for (int d = 1; d <= ks_cap && d <= nslices; ++d)
        if (nslices % d == 0) KS = d;
    if (KS < ks_cap / 2 && nslices > ks_cap) KS = ks_cap;   // awkward factorisation: ragged last chunk instead
    Plan pl;
    pl.KS = KS;
    pl.nchunk = (nslices + KS - 1) / KS;
    pl.RB = 1;
    while (pl.RB * 2 * KS <= 16) pl.RB *= 2;                 // up to 16 waves share one activation image
    const int64_t row_blocks = (a.m + 15) / 16;
    while (pl.RB > 1 && (row_blocks + pl.RB - 1) / pl.RB < 256) pl.RB /= 2;   // but keep one workgroup per CU
    size_t image = (size_t)KS * kSliceGroups * 512 * nb + 16 + (size_t)KS * kSliceCols * 2 * nb;
    size_t red = (size_t)KS * pl.RB * 64 * sizeof(float);
    pl.lds_bytes = image > red ? image : red;
    return pl;
}

template <typename K>
hipError_t launch_one(K kernel, const GemmArgs &a, const Plan &pl, dim3 grid, dim3 block, hipStream_t stream)
{
    if (pl.lds_bytes > 64 * 1024) {
        // opt in to more than 64 KiB of dynamic LDS (a per-function attribute, cheap to repeat)
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)pl.lds_bytes);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kernel, grid, block, pl.lds_bytes, stream, a, pl.KS, pl.RB, pl.nchunk);
    return hipGetLastError();
}

}  // namespace

bool plane_mfma_supports(const GemmArgs &a)
{
    return a.group == 128 && (a.n % kSliceCols) == 0 && a.p_max <= kMaxP &&
           (a.batch + kMaxBatchTile - 1) / kMaxBatchTile <= 65535;
}

hipError_t plane_mfma_launch(const GemmArgs &a, hipStream_t stream)
{
    const Plan pl = make_plan(a);
    const int64_t row_blocks = (a.m + 15) / 16;
    dim3 grid((unsigned)((row_blocks + pl.RB - 1) / pl.RB), (unsigned)((a.batch + kMaxBatchTile - 1) / kMaxBatchTile));
    dim3 block(64 * pl.KS * pl.RB);
    const bool mixed = a.uniform_p == 0;
#define BCQ_LAUNCH(PP, MM) return launch_one(plane_mfma_kernel<PP, MM>, a, pl, grid, block, stream)
    switch (a.p_max) {
    case 1: if (mixed) BCQ_LAUNCH(1, true); else BCQ_LAUNCH(1, false);
    case 2: if (mixed) BCQ_LAUNCH(2, true); else BCQ_LAUNCH(2, false);
    case 3: if (mixed) BCQ_LAUNCH(3, true); else BCQ_LAUNCH(3, false);
    default: if (mixed) BCQ_LAUNCH(4, true); else BCQ_LAUNCH(4, false);
    }
#undef BCQ_LAUNCH
}

}  // namespace bcq
