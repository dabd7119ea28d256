// Reference points for the benchmark, not part of the method: what the same GPU reaches on a pure
// streaming read of as many bytes as a product call moves, and on a plain binary16 matrix-vector product
// that does not depend on a library's choice of kernel (both ordinary bandwidth-bound kernels); and what one
// SIMD issues per clock when matrix and vector instructions alternate, which is what bounds the product kernels
// once their data are there.
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

// What a SIMD can issue: `valu` independent vector FMAs behind every matrix instruction, a fixed number of times, in
// every wave of ONE workgroup (waves beyond four share SIMDs).  Lane 0 of each wave reports the shader-clock ticks and
// the 100 MHz ticks its loop took.  KIND 0: v_mfma_f32_16x16x32_f16, 1: v_mfma_f32_32x32x16_f16, 2:
// v_mfma_f32_16x16x128_f8f6f4 with an E5M2 and an FP4 operand.
typedef _Float16 half8v __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef int i32x8 __attribute__((ext_vector_type(8)));

template <int KIND, int NV>
__global__ __launch_bounds__(1024) void issue_probe_kernel(uint64_t *ticks, float *sink, int iters)
{
    half8v a, b;
    i32x8 a8, b8;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        a[j] = (_Float16)(0.001f * (float)threadIdx.x + (float)j);
        b[j] = (_Float16)(0.5f * (float)j);
        a8[j] = (int)threadIdx.x * 77 + j;
        b8[j] = 0x22222222;
    }
    f32x16 c[4];
    f32x4 d[4];
    float f[8];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
#pragma unroll
        for (int j = 0; j < 16; ++j) c[u][j] = 0.f;
        d[u] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) f[j] = (float)threadIdx.x + (float)j;
    const float k1 = 1.0001f, k2 = 0.5f;
    __syncthreads();
    const uint64_t t0 = __builtin_readcyclecounter(), r0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if constexpr (KIND == 0) d[u] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, d[u], 0, 0, 0);
            if constexpr (KIND == 1) c[u] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c[u], 0, 0, 0);
            if constexpr (KIND == 2) d[u] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a8, b8, d[u], 1, 4, 0, 0, 0, 0);
#pragma unroll
            for (int v = 0; v < NV; ++v) f[v & 7] = __builtin_fmaf(f[v & 7], k1, k2);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    const uint64_t t1 = __builtin_readcyclecounter(), r1 = wall_clock64();
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) s += f[j];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
#pragma unroll
        for (int j = 0; j < 16; ++j) s += c[u][j];
#pragma unroll
        for (int j = 0; j < 4; ++j) s += d[u][j];
    }
    sink[threadIdx.x] = s;
    if ((threadIdx.x & 63) == 0) {
        ticks[2 * (threadIdx.x >> 6)] = t1 - t0;
        ticks[2 * (threadIdx.x >> 6) + 1] = r1 - r0;
    }
}

template <int KIND>
bool launch_issue_probe(int valu, int waves, int iters, uint64_t *ticks, float *sink, hipStream_t stream)
{
    switch (valu) {
    case 0: hipLaunchKernelGGL((issue_probe_kernel<KIND, 0>), dim3(1), dim3(64 * waves), 0, stream, ticks, sink, iters); return true;
    case 4: hipLaunchKernelGGL((issue_probe_kernel<KIND, 4>), dim3(1), dim3(64 * waves), 0, stream, ticks, sink, iters); return true;
    case 8: hipLaunchKernelGGL((issue_probe_kernel<KIND, 8>), dim3(1), dim3(64 * waves), 0, stream, ticks, sink, iters); return true;
    case 16: hipLaunchKernelGGL((issue_probe_kernel<KIND, 16>), dim3(1), dim3(64 * waves), 0, stream, ticks, sink, iters); return true;
    default: return false;
    }
}

}  // namespace

extern "C" {

int bcq_bench_issue_probe(int kind, int valu, int waves, int iters, uint64_t *ticks, float *sink, void *stream)
{
    if (!ticks || !sink) return -1;
    if (waves < 1 || waves > 16 || iters < 1 || iters > (1 << 20)) return -3;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool known = kind == 0 ? launch_issue_probe<0>(valu, waves, iters, ticks, sink, st)
                     : kind == 1 ? launch_issue_probe<1>(valu, waves, iters, ticks, sink, st)
                     : kind == 2 ? launch_issue_probe<2>(valu, waves, iters, ticks, sink, st) : false;
    if (!known) return -3;
    return hipGetLastError() == hipSuccess ? 0 : -5;
}

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
