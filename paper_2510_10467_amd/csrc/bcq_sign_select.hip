// Generic kernel: the plane-by-plane add/subtract formulation of section 3.3
// written directly.  One wavefront owns one output row and walks the row's
// 32-column words; for each plane the word's bits choose +x or -x, the word sum
// is multiplied by the group's scale and accumulated in fp32.  It accepts every
// legal shape, group size, batch and per-request precision, and serves as the
// fallback for problems the tuned kernels do not cover.
#include <hip/hip_runtime.h>

#include "bcq_internal.hpp"

namespace bcq {
namespace {

constexpr int kWavesPerBlock = 4;
constexpr int kBatchTile = 4;

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

__global__ __launch_bounds__(64 * kWavesPerBlock) void sign_select_kernel(GemmArgs a)
{
    const int lane = threadIdx.x & 63;
    const int64_t r = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
    if (r >= a.m) return;
    const int b0 = blockIdx.y * kBatchTile;
    const int words = (int)(a.n / 32);
    const int words_per_group = a.group / 32;
    const int64_t ngroups = a.n / a.group;

    int pb[kBatchTile];
    int p_hi = 0;
#pragma unroll
    for (int t = 0; t < kBatchTile; ++t) {
        pb[t] = (b0 + t < a.batch) ? request_precision(a, b0 + t) : 0;
        p_hi = pb[t] > p_hi ? pb[t] : p_hi;
    }
    float acc[kBatchTile] = {0.f, 0.f, 0.f, 0.f};

    for (int w = lane; w < words; w += 64) {
        const int64_t g = w / words_per_group;
        uint32_t bits[BCQ_MAX_PLANES];
#pragma unroll
        for (int i = 0; i < BCQ_MAX_PLANES; ++i)
            bits[i] = (i < p_hi) ? a.planes[((int64_t)i * a.m + r) * words + w] : 0u;
#pragma unroll
        for (int t = 0; t < kBatchTile; ++t) {
            if (pb[t] == 0) continue;
            const _Float16 *xp = a.x + (int64_t)(b0 + t) * a.n + (int64_t)w * 32;
            float xv[32];
#pragma unroll
            for (int k = 0; k < 32; ++k) xv[k] = (float)xp[k];
            const _Float16 *sp = a.scales[pb[t]];
            // asymmetric scheme: the group's offset times the sum of the word's activations
            if (const _Float16 *zp = a.offsets[pb[t]]) {
                float s = 0.f;
#pragma unroll
                for (int k = 0; k < 32; ++k) s += xv[k];
                acc[t] = fmaf((float)zp[r * ngroups + g], s, acc[t]);
            }
#pragma unroll
            for (int i = 0; i < BCQ_MAX_PLANES; ++i) {
                if (i < pb[t]) {
                    float s = 0.f;
#pragma unroll
                    for (int k = 0; k < 32; ++k) s += ((bits[i] >> k) & 1u) ? xv[k] : -xv[k];
                    float alpha = (float)sp[((int64_t)i * a.m + r) * ngroups + g];
                    acc[t] = fmaf(alpha, s, acc[t]);
                }
            }
        }
    }
#pragma unroll
    for (int t = 0; t < kBatchTile; ++t) {
        float v = wave_sum(acc[t]);
        if (lane == 0 && b0 + t < a.batch) a.y[(int64_t)(b0 + t) * a.m + r] = (_Float16)v;
    }
}

}  // namespace

bool sign_select_supports(const GemmArgs &a)
{
    // grid.y carries the batch tiles
    return (a.batch + kBatchTile - 1) / kBatchTile <= 65535 && (a.m + kWavesPerBlock - 1) / kWavesPerBlock < (int64_t(1) << 31);
}

hipError_t sign_select_launch(const GemmArgs &a, hipStream_t stream)
{
    dim3 grid((unsigned)((a.m + kWavesPerBlock - 1) / kWavesPerBlock), (unsigned)((a.batch + kBatchTile - 1) / kBatchTile));
    hipLaunchKernelGGL(sign_select_kernel, grid, dim3(64 * kWavesPerBlock), 0, stream, a);
    return hipGetLastError();
}

}  // namespace bcq
