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

template <int P>
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
    const int nrows = 4 * nb;
    const int words = (int)(a.n >> 5);
    const int ngroups = (int)(a.n >> 7);

    int64_t row = ((int64_t)blockIdx.x * RB + rb) * 16 + (lane & 15);
    const bool row_ok = row < a.m;
    if (!row_ok) row = a.m - 1;               // keep loads in bounds; the result is discarded

    // precision of the request this lane reports on, and the deepest plane any request of the tile needs
    int p_mine = 0, p_hi = 0;
    for (int b = 0; b < nb; ++b) {
        int pb = request_precision(a, b0 + b);
        p_hi = max(p_hi, pb);
        if (b == q) p_mine = pb;
    }
    const _Float16 *scale_set = a.scales[p_mine];

    float acc = 0.f;
    for (int chunk = 0; chunk < nchunk; ++chunk) {
        const int slice = chunk * KS + ks;                         // global K slice index of this wave
        const int nslices = (int)(a.n / kSliceCols);
        const bool slice_ok = slice < nslices;
        const int slice_c = slice_ok ? slice : nslices - 1;

        // ---- 1. issue this wave's plane and scale loads ------------------------------------
        u32x4 wlo[P], whi[P];
        uint4 sc[P];
#pragma unroll
        for (int i = 0; i < P; ++i) {
            wlo[i] = u32x4{0, 0, 0, 0};
            whi[i] = u32x4{0, 0, 0, 0};
            sc[i] = make_uint4(0, 0, 0, 0);
            if (i < p_hi) {
                const u32x4 *wp = reinterpret_cast<const u32x4 *>(
                    a.planes + ((int64_t)i * a.m + row) * words + slice_c * (kSliceCols / 32) + q * 8);
                wlo[i] = __builtin_nontemporal_load(wp);            // group 2q of the slice
                whi[i] = __builtin_nontemporal_load(wp + 1);        // group 2q + 1
            }
            if (i < p_mine)
                sc[i] = *reinterpret_cast<const uint4 *>(
                    scale_set + ((int64_t)i * a.m + row) * ngroups + slice_c * kSliceGroups);
        }

        // ---- 2. workgroup builds the activation image of this chunk ------------------------
        if (chunk > 0) __syncthreads();                            // previous image no longer read
        {
            const int chunk_cols = KS * kSliceCols;
            const int64_t col0 = (int64_t)chunk * chunk_cols;
            const int pairs = chunk_cols / 2;
            for (int idx = tid; idx < nb * pairs; idx += nthreads) {
                const int b = idx / pairs;
                const int c = (idx - b * pairs) * 2;                // even column inside the chunk
                uint32_t v = 0;
                if (col0 + c < a.n)
                    v = *reinterpret_cast<const uint32_t *>(a.x + (int64_t)(b0 + b) * a.n + col0 + c);
                // exact split of both halves into four E5M2 terms (top bytes of the running remainders)
                uint32_t t[4];
                h2 r = __builtin_bit_cast(h2, v);
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    t[k] = __builtin_bit_cast(uint32_t, r) & 0xFF00FF00u;
                    r = r - __builtin_bit_cast(h2, t[k]);
                }
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    const int cl = (c + e) & 127;                   // column inside its group
                    const int g = (c + e) >> 7;
                    const int h = cl >> 6, u = (cl >> 5) & 1, tt = (cl >> 2) & 7;
                    const int inv = (~cl) & 3;                      // 3 - (cl & 3) = shift that exposes this bit
                    const int qa = 2 * u + (inv >> 1);
                    const int off = image_offset(g, h, qa, 4 * b, nrows) + 8 * (inv & 1) + tt;
#pragma unroll
                    for (int k = 0; k < 4; ++k) lds[off + 16 * k] = (unsigned char)(t[k] >> (e ? 24 : 8));
                }
            }
        }
        __syncthreads();

        // ---- 3. per group: expand plane words, one MFMA per (group, plane), scale, accumulate
        const int arow = lane & 15;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            // after the transpose, register t of quarter q is dword q of group 2t + j of the slice
            uint32_t wt[P][4];
#pragma unroll
            for (int i = 0; i < P; ++i) {
                const u32x4 src = j ? whi[i] : wlo[i];
                wt[i][0] = src.x; wt[i][1] = src.y; wt[i][2] = src.z; wt[i][3] = src.w;
                quarter_transpose(wt[i][0], wt[i][1], wt[i][2], wt[i][3]);
            }
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int gl = 2 * t + j;                           // group inside the slice
                v8i xa = {0, 0, 0, 0, 0, 0, 0, 0};
                if (arow < nrows) {
                    const int gc = ks * kSliceGroups + gl;
                    const uint4 lo = *reinterpret_cast<const uint4 *>(lds + image_offset(gc, 0, q, arow, nrows));
                    const uint4 hi = *reinterpret_cast<const uint4 *>(lds + image_offset(gc, 1, q, arow, nrows));
                    xa[0] = lo.x; xa[1] = lo.y; xa[2] = lo.z; xa[3] = lo.w;
                    xa[4] = hi.x; xa[5] = hi.y; xa[6] = hi.z; xa[7] = hi.w;
                }
#pragma unroll
                for (int i = 0; i < P; ++i) {
                    if (i < p_hi) {
                        const uint32_t w = wt[i][t];
                        v8i wb = {0, 0, 0, 0, 0, 0, 0, 0};
                        wb[0] = (int)((w & 0x88888888u) | 0x22222222u);
                        wb[1] = (int)(((w << 1) & 0x88888888u) | 0x22222222u);
                        wb[2] = (int)(((w << 2) & 0x88888888u) | 0x22222222u);
                        wb[3] = (int)(((w << 3) & 0x88888888u) | 0x22222222u);
                        v4f d = {0.f, 0.f, 0.f, 0.f};
                        // A: E5M2 activation terms (cbsz = 1), B: FP4 signs (blgp = 4), no block scaling
                        d = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(xa, wb, d, 1, 4, 0, 0, 0, 0);
                        const uint32_t sw = (gl >> 1) == 0 ? sc[i].x : (gl >> 1) == 1 ? sc[i].y : (gl >> 1) == 2 ? sc[i].z : sc[i].w;
                        const float alpha = (float)__builtin_bit_cast(_Float16, (unsigned short)((gl & 1) ? (sw >> 16) : (sw & 0xffffu)));
                        const float s = (d[0] + d[1]) + (d[2] + d[3]);
                        // the FP4 sign bit is set for weight bit 1 (= +1), so the instruction returns -(B_i x)
                        if (slice_ok) acc = fmaf(-alpha, s, acc);
                    }
                }
            }
        }
    }

    // ---- 4. combine the KS partial sums of each row block in a fixed order, store binary16 --
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

Plan make_plan(const GemmArgs &a)
{
    const int nslices = (int)(a.n / kSliceCols);
    const int nb = a.batch < kMaxBatchTile ? a.batch : kMaxBatchTile;
    const int ks_cap = 16 / nb;                       // activation image <= 64 KiB per chunk
    int KS = 1;
    for (int d = 1; d <= ks_cap && d <= nslices; ++d)
        if (nslices % d == 0) KS = d;
    if (KS < ks_cap / 2 && nslices > ks_cap) KS = ks_cap;   // awkward factorisation: ragged last chunk instead
    Plan pl;
    pl.KS = KS;
    pl.nchunk = (nslices + KS - 1) / KS;
    pl.RB = KS >= 8 ? 1 : 8 / KS;
    const int64_t row_blocks = (a.m + 15) / 16;
    while (pl.RB > 1 && row_blocks / pl.RB < 512) pl.RB /= 2;     // keep enough workgroups to fill 256 CUs
    size_t image = (size_t)KS * kSliceGroups * 512 * nb;
    size_t red = (size_t)KS * pl.RB * 64 * sizeof(float);
    pl.lds_bytes = image > red ? image : red;
    return pl;
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
    switch (a.p_max) {
    case 1: hipLaunchKernelGGL(plane_mfma_kernel<1>, grid, block, pl.lds_bytes, stream, a, pl.KS, pl.RB, pl.nchunk); break;
    case 2: hipLaunchKernelGGL(plane_mfma_kernel<2>, grid, block, pl.lds_bytes, stream, a, pl.KS, pl.RB, pl.nchunk); break;
    case 3: hipLaunchKernelGGL(plane_mfma_kernel<3>, grid, block, pl.lds_bytes, stream, a, pl.KS, pl.RB, pl.nchunk); break;
    default: hipLaunchKernelGGL(plane_mfma_kernel<4>, grid, block, pl.lds_bytes, stream, a, pl.KS, pl.RB, pl.nchunk); break;
    }
    return hipGetLastError();
}

}  // namespace bcq
