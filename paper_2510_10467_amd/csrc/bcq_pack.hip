// Bit-plane packing (section 3.3: planes are stored separately so that only the
// first p are fetched; Fig. 1 caption: a stored 0 stands for -1).
// One thread produces (or expands) one 32-column word with 16-byte accesses on
// the int8 side, so both directions are plain streaming kernels.
#include <hip/hip_runtime.h>

#include "bcq_internal.hpp"

namespace bcq {
namespace {

__global__ __launch_bounds__(256) void pack_kernel(const int8_t *__restrict__ codes, uint32_t *__restrict__ planes,
                                                   int64_t total_words)
{
    int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (w >= total_words) return;
    // codes and planes are both [plane][row][column]-ordered, so word w covers codes 32w .. 32w+31
    const uint4 *src = reinterpret_cast<const uint4 *>(codes + w * 32);
    uint32_t out = 0;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        uint4 v = src[h];
        uint32_t d[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                int8_t c = (int8_t)((d[q] >> (8 * k)) & 0xff);
                out |= (uint32_t)(c > 0) << (h * 16 + q * 4 + k);
            }
    }
    planes[w] = out;
}

__global__ __launch_bounds__(256) void unpack_kernel(const uint32_t *__restrict__ planes, int8_t *__restrict__ codes,
                                                     int64_t total_words)
{
    int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (w >= total_words) return;
    uint32_t bits = planes[w];
    uint4 *dst = reinterpret_cast<uint4 *>(codes + w * 32);
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        uint32_t d[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            uint32_t v = 0;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                uint32_t byte = ((bits >> (h * 16 + q * 4 + k)) & 1u) ? 0x01u : 0xffu;   // +1 or -1 as int8
                v |= byte << (8 * k);
            }
            d[q] = v;
        }
        dst[h] = make_uint4(d[0], d[1], d[2], d[3]);
    }
}

}  // namespace

hipError_t pack_launch(const int8_t *codes, uint32_t *planes, int n_planes, int64_t m, int64_t n, hipStream_t stream)
{
    int64_t total = (int64_t)n_planes * m * (n / 32);
    int64_t blocks = (total + 255) / 256;
    if (blocks > 0x7fffffffll) return hipErrorInvalidValue;        // beyond one grid dimension
    hipLaunchKernelGGL(pack_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, codes, planes, total);
    return hipGetLastError();
}

hipError_t unpack_launch(const uint32_t *planes, int8_t *codes, int n_planes, int64_t m, int64_t n, hipStream_t stream)
{
    int64_t total = (int64_t)n_planes * m * (n / 32);
    int64_t blocks = (total + 255) / 256;
    if (blocks > 0x7fffffffll) return hipErrorInvalidValue;        // beyond one grid dimension
    hipLaunchKernelGGL(unpack_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, planes, codes, total);
    return hipGetLastError();
}

}  // namespace bcq
