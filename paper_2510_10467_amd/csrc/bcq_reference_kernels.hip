// Reference points for the benchmark, not part of the method: what the same GPU reaches on a pure
// streaming read of as many bytes as a product call moves, and on a plain binary16 matrix-vector product
// that does not depend on a library's choice of kernel.  Both are ordinary bandwidth-bound kernels.
#include <hip/hip_runtime.h>

#include "bcq_bench.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 half8 __attribute__((ext_vector_type(8)));

constexpr int kReadUnroll = 8;                       // 16-byte loads in flight per thread

// Every thread reads kReadUnroll x 16 bytes, 4 KiB apart (a wave covers whole 1 KiB runs), and folds them
// into one word; a workgroup stores its word only if it is a value that random data never produces, so
// the loads cannot be optimised away and nothing is written.
__global__ __launch_bounds__(256) void stream_read_kernel(const u32x4 *src, uint64_t units, uint32_t *sink)
{
    const uint64_t base = (uint64_t)blockIdx.x * (256 * kReadUnroll) + threadIdx.x;
    u32x4 v[kReadUnroll];
#pragma unroll
    for (int k = 0; k < kReadUnroll; ++k) {
        const uint64_t u = base + (uint64_t)k * 256;
        v[k] = __builtin_nontemporal_load(src + (u < units ? u : units - 1));
    }
    uint32_t acc = 0;
#pragma unroll
    for (int k = 0; k < kReadUnroll; ++k) acc ^= v[k].x ^ v[k].y ^ v[k].z ^ v[k].w;
    if (acc == 0x9E3779B9u) sink[blockIdx.x & 63] = acc;
}

// y[r] = sum_j W[r][j] x[j], one wave per row, 16 bytes per lane and step, fp32 accumulation.
__global__ __launch_bounds__(256) void fp16_gemv_kernel(const _Float16 *w, const _Float16 *x, _Float16 *y, uint32_t m, uint32_t n)
{
    const uint32_t row = blockIdx.x * 4 + (threadIdx.x >> 6);
    const uint32_t lane = threadIdx.x & 63;
    if (row >= m) return;
    const half8 *wr = reinterpret_cast<const half8 *>(w + (size_t)row * n);
    const half8 *xr = reinterpret_cast<const half8 *>(x);
    float acc = 0.f;
    for (uint32_t c = lane; c < n / 8; c += 64) {
        const half8 a = __builtin_nontemporal_load(wr + c);
        const half8 b = xr[c];
#pragma unroll
        for (int e = 0; e < 8; ++e) acc = fmaf((float)a[e], (float)b[e], acc);
    }
#pragma unroll
    for (int mask = 32; mask >= 1; mask >>= 1) acc += __shfl_xor(acc, mask, 64);
    if (lane == 0) y[row] = (_Float16)acc;
}

}  // namespace

extern "C" {

int bcq_bench_stream_read(const void *src, int64_t bytes, uint32_t *sink, void *stream)
{
    if (!src || !sink) return -1;
    if (bytes < 16 || (bytes % 16) != 0 || (reinterpret_cast<uintptr_t>(src) & 15) != 0) return -3;
    const uint64_t units = (uint64_t)bytes / 16;
    const uint64_t blocks = (units + 256 * kReadUnroll - 1) / (256 * kReadUnroll);
    if (blocks > 0x7fffffffull) return -3;
    hipLaunchKernelGGL(stream_read_kernel, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                       reinterpret_cast<const u32x4 *>(src), units, sink);
    return hipGetLastError() == hipSuccess ? 0 : -5;
}

int bcq_bench_fp16_gemv(const uint16_t *w, const uint16_t *x, uint16_t *y, int64_t m, int64_t n, void *stream)
{
    if (!w || !x || !y) return -1;
    if (m < 1 || n < 8 || (n % 8) != 0 || m > (int64_t(1) << 31) || n > (int64_t(1) << 31)) return -3;
    if ((reinterpret_cast<uintptr_t>(w) & 15) != 0 || (reinterpret_cast<uintptr_t>(x) & 15) != 0) return -4;
    hipLaunchKernelGGL(fp16_gemv_kernel, dim3((unsigned)((m + 3) / 4)), dim3(256), 0, static_cast<hipStream_t>(stream),
                       reinterpret_cast<const _Float16 *>(w), reinterpret_cast<const _Float16 *>(x),
                       reinterpret_cast<_Float16 *>(y), (uint32_t)m, (uint32_t)n);
    return hipGetLastError() == hipSuccess ? 0 : -5;
}

}  // extern "C"
