// Large-batch kernel: dequantise W_p = sum_i alpha_i B_i tile by tile (Fig. 1(b): p-bit inference
// reconstructs the weights from the first p planes and the scale set of precision p) and feed the
// binary16 tiles to the fp16 matrix pipe.  Once a plane word serves dozens of requests the product
// is no longer bound by HBM but by arithmetic, and one dense fp16 MFMA over dequantised weights
// costs p times fewer matrix instructions than p plane-wise products.
//
// A workgroup of four waves owns 64 weight rows and a block of 64 requests.  Per group of 128
// columns the workgroup stages the 64 x 128 activation tile in LDS; every lane fetches the 16 bytes
// of its own row's group from each plane plus the group's scales, and for each 32-column step
//   * takes ONE byte of each plane word (lane quarter kq owns columns 8kq .. 8kq+7 of the step),
//   * looks the byte up in a 256-entry LDS table of eight +-1.0 binary16 values,
//   * accumulates w_j = sum_i alpha_i * (+-1) in fp32 (one mixed-precision FMA per column and
//     plane), rounds once to binary16,
// and issues v_mfma_f32_16x16x32_f16 for the four 16-request column blocks, accumulating in fp32.
// The MFMA's M side carries requests, its N side the 16 weight rows of the wave, so a lane ends up
// with four requests of its own row.
#include <hip/hip_runtime.h>

#include "bcq_internal.hpp"

namespace bcq {
namespace {

typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kRowsPerWg = 64;              // 4 waves x 16 rows
constexpr int kReqPerWg = 64;               // 4 MFMA column blocks of 16 requests
constexpr int kMaxP = 4;
constexpr int kXRowBytes = 128 * 2 + 16;    // padded LDS row of one request's 128 activations
constexpr int kLutBytes = 256 * 16;
constexpr int kXTileBytes = kReqPerWg * kXRowBytes;

template <int P>
__global__ __launch_bounds__(256) void dequant_mfma_kernel(GemmArgs a)
{
    __shared__ __attribute__((aligned(16))) unsigned char lds[kLutBytes + 2 * kXTileBytes];
    unsigned char *lut = lds;
    unsigned char *xt0 = lds + kLutBytes;       // two activation tiles, used alternately

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int n16 = lane & 15;                // weight row inside the wave's block / request inside a column block
    const int kq = lane >> 4;                 // K quarter: columns 8kq .. 8kq+7 of each 32-column step
    const int ngroups = (int)(a.n >> 7);
    const int words = (int)(a.n >> 5);
    const int b0 = blockIdx.y * kReqPerWg;

    int64_t row = (int64_t)blockIdx.x * kRowsPerWg + wave * 16 + n16;
    const bool row_ok = row < a.m;
    if (!row_ok) row = a.m - 1;

    // table: byte -> eight binary16 values, +1.0 where the bit is set, -1.0 where it is clear
    {
        uint32_t e[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const uint32_t lo = ((tid >> (2 * c)) & 1) ? 0x3C00u : 0xBC00u;
            const uint32_t hi = ((tid >> (2 * c + 1)) & 1) ? 0x3C00u : 0xBC00u;
            e[c] = lo | (hi << 16);
        }
        *reinterpret_cast<u32x4 *>(lut + tid * 16) = u32x4{e[0], e[1], e[2], e[3]};
    }

    const _Float16 *scales = a.scales[a.uniform_p];
    v4f acc[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) acc[u] = v4f{0.f, 0.f, 0.f, 0.f};

    // staging assignment: thread t copies 16-byte units t, t+256, t+512, t+768 of the 64 x 256-byte tile
    auto stage_tile = [&](int g, unsigned char *dst) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int unit = tid + 256 * k;
            const int req = unit >> 4, part = unit & 15;            // 16 units per request row
            const int b = b0 + req;
            u32x4 v = u32x4{0, 0, 0, 0};
            if (b < a.batch) v = *reinterpret_cast<const u32x4 *>(a.x + (int64_t)b * a.n + (int64_t)g * 128 + part * 8);
            *reinterpret_cast<u32x4 *>(dst + req * kXRowBytes + part * 16) = v;
        }
    };

    stage_tile(0, xt0);
    __syncthreads();
    for (int g = 0; g < ngroups; ++g) {
        // this lane's row: one group of every plane and its scales
        u32x4 w[P];
        float alpha[P];
#pragma unroll
        for (int i = 0; i < P; ++i) {
            w[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(a.planes + ((int64_t)i * a.m + row) * words + g * 4));
            alpha[i] = (float)scales[((int64_t)i * a.m + row) * ngroups + g];
        }
        if (g + 1 < ngroups) stage_tile(g + 1, xt0 + ((g + 1) & 1) * kXTileBytes);    // next tile into the other buffer
        const unsigned char *xcur = xt0 + (g & 1) * kXTileBytes;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            float wf[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) wf[j] = 0.f;
#pragma unroll
            for (int i = 0; i < P; ++i) {
                const uint32_t byte = (w[i][t] >> (8 * kq)) & 0xffu;
                const v8h pm = *reinterpret_cast<const v8h *>(lut + byte * 16);
#pragma unroll
                for (int j = 0; j < 8; ++j) wf[j] = fmaf((float)pm[j], alpha[i], wf[j]);
            }
            v8h wb;
#pragma unroll
            for (int j = 0; j < 8; ++j) wb[j] = (_Float16)wf[j];    // the single rounding of W_p to binary16
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const v8h xa = *reinterpret_cast<const v8h *>(xcur + (16 * u + n16) * kXRowBytes + (32 * t + 8 * kq) * 2);
                acc[u] = __builtin_amdgcn_mfma_f32_16x16x32_f16(xa, wb, acc[u], 0, 0, 0);
            }
        }
        __syncthreads();                                            // next tile complete, current tile free
    }

    // lane holds requests 16u + 4kq + i (i = 0..3) of weight row `row`
    if (row_ok) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int b = b0 + 16 * u + 4 * kq + i;
                if (b < a.batch) a.y[(int64_t)b * a.m + row] = (_Float16)acc[u][i];
            }
    }
}

}  // namespace

bool dequant_mfma_supports(const GemmArgs &a)
{
    return a.uniform_p >= 1 && a.uniform_p <= kMaxP && a.group == 128 &&
           (a.batch + kReqPerWg - 1) / kReqPerWg <= 65535 && (a.m + kRowsPerWg - 1) / kRowsPerWg < (int64_t(1) << 31);
}

hipError_t dequant_mfma_launch(const GemmArgs &a, hipStream_t stream)
{
    dim3 grid((unsigned)((a.m + kRowsPerWg - 1) / kRowsPerWg), (unsigned)((a.batch + kReqPerWg - 1) / kReqPerWg));
    dim3 block(256);
    switch (a.uniform_p) {
    case 1: hipLaunchKernelGGL(dequant_mfma_kernel<1>, grid, block, 0, stream, a); break;
    case 2: hipLaunchKernelGGL(dequant_mfma_kernel<2>, grid, block, 0, stream, a); break;
    case 3: hipLaunchKernelGGL(dequant_mfma_kernel<3>, grid, block, 0, stream, a); break;
    default: hipLaunchKernelGGL(dequant_mfma_kernel<4>, grid, block, 0, stream, a); break;
    }
    return hipGetLastError();
}

}  // namespace bcq
