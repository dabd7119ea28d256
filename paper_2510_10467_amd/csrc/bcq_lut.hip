// Table-lookup kernel: the formulation section 3.3 names for the product (LUT-based GEMM: the partial sums of
// short runs of activations are kept in a table and looked up with the weight bits instead of being added and
// subtracted bit by bit).  Runs of four activations: a table entry is one of the 16 signed sums of four
// consecutive activations, a nibble of a plane word picks it, and eight look-ups give B_i x over a 32-column word;
// the word sum is multiplied by the group's scale and accumulated in fp32, plane by plane.
//
// It accepts every legal shape, group size (multiples of 32), precision (to 8 planes), batch and per-request
// precision, with or without offsets, and is the fallback for the problems the matrix-pipe kernels do not take.
//
// Work split: a workgroup of four waves owns 16 rows (four per wave; 8 or 4 on short matrices) and walks the columns
// in stretches of TT tiles of 2048 columns (one 32-column word per lane and tile): two tiles with one request, one
// tile with up to four requests.  Per stretch it asks for everything it needs from memory at once (the activations
// behind the tables, its rows' plane words and scales), builds the tables in LDS (32 KiB per request and tile) and
// then looks up.  Tables are laid out [nibble][entry][lane]: the 64 look-ups of an instruction fall into 64
// consecutive words whatever the weight bits are.
#include <hip/hip_runtime.h>

#include "bcq_internal.hpp"

namespace bcq {
namespace {

constexpr int kLutWaves = 4;                                // several workgroups share a compute unit and hide each other's waits
constexpr int kLutTileCols = 2048;                         // columns per table tile: one plane word per lane
constexpr int kLutTileBytes = 8 * 16 * 64 * 4;             // [nibble of the word][entry][lane] fp32: 32 KiB

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// PU: planes the loops are unrolled for (4 or 8; planes beyond the deepest precision present are skipped)
// RPW: rows per wave (4, 2 or 1: 16, 8 or 4 rows per workgroup, so that short matrices still fill the chip)
// TT: tiles per stretch; NR: requests per workgroup (TT * NR tables of 32 KiB)
// UNI: one precision for all requests (their scales are fetched with the plane words)
template <int PU, int RPW, int TT, int NR, bool UNI>
__global__ __launch_bounds__(64 * kLutWaves) void lut_kernel(GemmArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    constexpr int kRows = kLutWaves * RPW;
    constexpr int kRequestBytes = TT * kLutTileBytes;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int b0 = blockIdx.y * NR;
    const int64_t words = a.n / 32;
    const int words_per_group = a.group / 32;
    const int64_t ngroups = a.n / a.group;
    const int64_t last_row = a.m - 1;

    int pb[NR];
    int p_hi = 0;
#pragma unroll
    for (int t = 0; t < NR; ++t) {
        // (every lane asks for the same request: the precision is the same in all of them, so it may live in a scalar register)
        pb[t] = __builtin_amdgcn_readfirstlane((b0 + t < a.batch) ? request_precision(a, b0 + t) : 0);
        p_hi = pb[t] > p_hi ? pb[t] : p_hi;
    }
    constexpr bool uniform = UNI;
    const _Float16 *const uniform_set = a.scales[uniform ? a.uniform_p : 0];
    // rows of this wave; rows past the end repeat the last row (their sums are never stored).  Word and scale indices
    // inside one plane fit 32 bits (checked on the host): a load is a scalar base per plane plus a lane offset.
    uint32_t row_word0[RPW], row_scale0[RPW];
#pragma unroll
    for (int k = 0; k < RPW; ++k) {
        const int64_t r = (int64_t)blockIdx.x * kRows + wave * RPW + k;
        const int64_t rr = r < last_row ? r : last_row;
        row_word0[k] = (uint32_t)(rr * words);
        row_scale0[k] = (uint32_t)(rr * ngroups);
    }
    const int64_t plane_words = a.m * words, plane_scales = a.m * ngroups;
    float acc[RPW][NR];
#pragma unroll
    for (int k = 0; k < RPW; ++k)
#pragma unroll
        for (int t = 0; t < NR; ++t) acc[k][t] = 0.f;

    // table building: a thread takes two runs of four columns (c0 and c0 + 1) of a tile with all 16 entries of each;
    // run c belongs to word c >> 3 (the lane that will look it up) and nibble c & 7.  The 64 threads of a wave take
    // the same pair of nibbles of 64 different words, so that their stores fall into 64 consecutive LDS words.
    const int c0 = (lane << 3) + 2 * wave;
    unsigned char *build_at = lds + ((c0 & 7) * 16 * 64 + (c0 >> 3)) * 4;
    const unsigned char *lane_tables = lds + lane * 4;

    const int ntiles = (int)((a.n + kLutTileCols - 1) / kLutTileCols);
    for (int tile0 = 0; tile0 < ntiles; tile0 += TT) {
        // ---- everything this stretch needs from memory is asked for first
        f16x8 xh[TT][NR];
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
            const int64_t col = (int64_t)(tile0 + tt) * kLutTileCols + 4 * c0;
#pragma unroll
            for (int t = 0; t < NR; ++t) {
                // n is a multiple of 32: eight columns from a multiple of eight lie inside the row or past its end (then zeros)
                const _Float16 z = (_Float16)0.f;
                xh[tt][t] = f16x8{z, z, z, z, z, z, z, z};
                if (pb[t] != 0 && col < a.n) xh[tt][t] = *reinterpret_cast<const f16x8 *>(a.x + (int64_t)(b0 + t) * a.n + col);
            }
        }
        bool w_ok[TT];
        uint32_t g[TT];
        uint32_t w[TT][PU][RPW];
        _Float16 alpha_u[TT][PU][RPW];
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
            const int64_t w_idx = (int64_t)(tile0 + tt) * (kLutTileCols / 32) + lane;
            w_ok[tt] = w_idx < words;
            const uint32_t w_at = w_ok[tt] ? (uint32_t)w_idx : 0u;     // lanes past the end of the row read word 0 and weigh it with zero
            g[tt] = w_at / (uint32_t)words_per_group;
#pragma unroll
            for (int i = 0; i < PU; ++i) {
                // (planes beyond the deepest precision present repeat its last plane: a load without a branch around it
                // stays up here, ahead of the table building, and those words are never looked up)
                const int ii = i < p_hi ? i : (p_hi > 0 ? p_hi - 1 : 0);
                const uint32_t *plane = a.planes + (int64_t)ii * plane_words;
                const _Float16 *scale_plane = uniform_set + (int64_t)ii * plane_scales;
#pragma unroll
                for (int k = 0; k < RPW; ++k) {
                    w[tt][i][k] = plane[row_word0[k] + w_at];
                    alpha_u[tt][i][k] = (_Float16)0.f;
                    if constexpr (uniform) alpha_u[tt][i][k] = scale_plane[row_scale0[k] + g[tt]];
                }
            }
        }

        __builtin_amdgcn_sched_barrier(0);                  // (the loads stay ahead of everything below)
        if (tile0 > 0) __syncthreads();                     // the previous stretch's tables are no longer read
#pragma unroll
        for (int tt = 0; tt < TT; ++tt)
#pragma unroll
            for (int t = 0; t < NR; ++t) {
                if (pb[t] == 0) continue;                   // (the same in every thread of the workgroup)
#pragma unroll
                for (int cc = 0; cc < 2; ++cc) {
                    const float x0 = (float)xh[tt][t][4 * cc], x1 = (float)xh[tt][t][4 * cc + 1];
                    const float x2 = (float)xh[tt][t][4 * cc + 2], x3 = (float)xh[tt][t][4 * cc + 3];
                    // entry e = sum over k of (bit k of e ? +x_k : -x_k)
                    float e[16];
                    e[0] = -x3 - x0 - x1 - x2;
                    e[1] = e[0] + 2.f * x0;
                    e[2] = e[0] + 2.f * x1;
                    e[3] = e[2] + 2.f * x0;
                    e[4] = e[0] + 2.f * x2;
                    e[5] = e[4] + 2.f * x0;
                    e[6] = e[4] + 2.f * x1;
                    e[7] = e[6] + 2.f * x0;
#pragma unroll
                    for (int q = 0; q < 8; ++q) e[8 + q] = e[q] + 2.f * x3;
                    float *dst = reinterpret_cast<float *>(build_at + t * kRequestBytes + tt * kLutTileBytes + cc * (16 * 64 * 4));
#pragma unroll
                    for (int q = 0; q < 16; ++q) dst[q * 64] = e[q];
                }
            }
        __syncthreads();

#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
            if (tile0 + tt >= ntiles) continue;
            // asymmetric scheme: the offset of the group times the sum of the word's activations, which is the
            // last entry (all bits set) of each of its eight tables
#pragma unroll
            for (int t = 0; t < NR; ++t) {
                if (pb[t] == 0) continue;
                const _Float16 *zp = a.offsets[pb[t]];
                if (zp == nullptr) continue;
                float xs = 0.f;
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    xs += *reinterpret_cast<const float *>(lane_tables + t * kRequestBytes + tt * kLutTileBytes + (j * 16 + 15) * 256);
                if (!w_ok[tt]) xs = 0.f;
#pragma unroll
                for (int k = 0; k < RPW; ++k) acc[k][t] = fmaf((float)zp[row_scale0[k] + g[tt]], xs, acc[k][t]);
            }
#pragma unroll
            for (int i = 0; i < PU; ++i) {
                if (!(i < p_hi)) continue;
#pragma unroll
                for (int k = 0; k < RPW; ++k) {
                    // byte offsets of the eight entries this word picks: entry (j, nibble) of this lane at (16 j + nibble) * 256
                    uint32_t at[8];
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const uint32_t wv = w[tt][i][k];
                        at[j] = (j < 2 ? (wv << (8 - 4 * j)) : (wv >> (4 * j - 8))) & 0xF00u;
                    }
#pragma unroll
                    for (int t = 0; t < NR; ++t) {
                        if (!(i < pb[t])) continue;
                        const unsigned char *tb = lane_tables + t * kRequestBytes + tt * kLutTileBytes;
                        float s = 0.f;
#pragma unroll
                        for (int j = 0; j < 8; ++j) s += *reinterpret_cast<const float *>(tb + j * 4096 + at[j]);
                        const float alpha = uniform ? (float)alpha_u[tt][i][k]
                                                    : (float)a.scales[pb[t]][(int64_t)i * plane_scales + row_scale0[k] + g[tt]];
                        acc[k][t] = fmaf(w_ok[tt] ? alpha : 0.f, s, acc[k][t]);
                    }
                }
            }
        }
    }

#pragma unroll
    for (int k = 0; k < RPW; ++k) {
        const int64_t r = (int64_t)blockIdx.x * kRows + wave * RPW + k;
#pragma unroll
        for (int t = 0; t < NR; ++t) {
            const float v = wave_sum(acc[k][t]);
            if (lane == 0 && r <= last_row && b0 + t < a.batch) a.y[(int64_t)(b0 + t) * a.m + r] = (_Float16)v;
        }
    }
}

// rows per wave: four where that still gives the compute units two workgroups or more each, else two, else one
int lut_rows_per_wave(const GemmArgs &a) { return a.m >= 8192 ? 4 : a.m >= 2048 ? 2 : 1; }

constexpr int kLutRequests = 2;           // requests per workgroup from two requests on (64 KiB of tables: two workgroups per compute unit)

template <int PU, int RPW, int TT, int NR, bool UNI>
hipError_t lut_launch_as(const GemmArgs &a, hipStream_t stream)
{
    constexpr int lds_bytes = TT * NR * kLutTileBytes;
    auto kernel = lut_kernel<PU, RPW, TT, NR, UNI>;
    if (hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(kernel), lds_bytes)) return e;
    constexpr int rows = kLutWaves * RPW;
    dim3 grid((unsigned)((a.m + rows - 1) / rows), (unsigned)((a.batch + NR - 1) / NR));
    hipLaunchKernelGGL(kernel, grid, dim3(64 * kLutWaves), lds_bytes, stream, a);
    return hipGetLastError();
}

template <int PU, int RPW>
hipError_t lut_launch_rows(const GemmArgs &a, hipStream_t stream)
{
    // one request: two tiles per stretch (one trip to memory and one pair of barriers for 4096 columns)
    if (a.uniform_p > 0)
        return a.batch == 1 ? lut_launch_as<PU, RPW, 2, 1, true>(a, stream) : lut_launch_as<PU, RPW, 1, kLutRequests, true>(a, stream);
    return a.batch == 1 ? lut_launch_as<PU, RPW, 2, 1, false>(a, stream) : lut_launch_as<PU, RPW, 1, kLutRequests, false>(a, stream);
}

}  // namespace

bool lut_supports(const GemmArgs &a)
{
    // grid.x carries the blocks of 4, 8 or 16 rows, grid.y the pairs of requests
    // (word and scale indices inside one plane are 32-bit in the kernel)
    const int rows = kLutWaves * lut_rows_per_wave(a);
    return (a.batch + kLutRequests - 1) / kLutRequests <= 65535 && (a.m + rows - 1) / rows < (int64_t(1) << 31) &&
           a.m * (a.n / 32) < (int64_t(1) << 32);
}

hipError_t lut_launch(const GemmArgs &a, hipStream_t stream)
{
    const int rpw = lut_rows_per_wave(a);
    if (a.p_max <= 4)
        return rpw == 4 ? lut_launch_rows<4, 4>(a, stream) : rpw == 2 ? lut_launch_rows<4, 2>(a, stream) : lut_launch_rows<4, 1>(a, stream);
    return rpw == 4 ? lut_launch_rows<8, 4>(a, stream) : rpw == 2 ? lut_launch_rows<8, 2>(a, stream) : lut_launch_rows<8, 1>(a, stream);
}

}  // namespace bcq
