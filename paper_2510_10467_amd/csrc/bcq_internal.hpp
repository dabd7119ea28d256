// Internal launch descriptor shared by the dispatcher and the kernel files.
// Nothing here is part of the C ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "bcq.h"

namespace bcq {

// One product call, uniform or per-request precision.
struct GemmArgs {
    const uint32_t *planes;                          // [>= p_max][m][n/32]
    const _Float16 *scales[BCQ_MAX_PLANES + 1];      // [q] = scale set of precision q, or nullptr
    const _Float16 *offsets[BCQ_MAX_PLANES + 1];     // [q] = offsets [m][n/group] of precision q, or nullptr (none)
    const int32_t *p_req;                            // device int32[batch], nullptr when uniform
    int uniform_p;                                   // > 0: every request runs at this precision
    int p_max;                                       // planes stored / upper bound of any p_req
    const _Float16 *x;                               // [batch][n]
    _Float16 *y;                                     // [batch][m]
    int64_t m, n;
    int batch;
    int group;
};

// Precision of request b: the uniform one, or p_req[b] clamped to [1, p_max];
// 0 when that precision has no scale set (the request then yields zeros).
__device__ __forceinline__ int request_precision(const GemmArgs &a, int b)
{
    int p = a.uniform_p;
    if (p == 0) {
        p = a.p_req[b];
        p = p < 1 ? 1 : (p > a.p_max ? a.p_max : p);
    }
    return a.scales[p] ? p : 0;
}

// More than 64 KiB of dynamic LDS needs a per-function attribute.  It sticks to the function, so it is set once per
// kernel instance and device (and again only if a later launch asks for more); defined in bcq_api.hip.
hipError_t allow_dynamic_lds(const void *kernel, int bytes);

// Kernel families.  *_supports tells whether the family can run the problem;
// *_launch enqueues it on `stream` and returns the HIP launch status.
bool sign_select_supports(const GemmArgs &a);
hipError_t sign_select_launch(const GemmArgs &a, hipStream_t stream);

// table look-ups (section 3.3's LUT formulation): any legal shape; the fallback ahead of sign_select
bool lut_supports(const GemmArgs &a);
hipError_t lut_launch(const GemmArgs &a, hipStream_t stream);

bool plane_mfma_supports(const GemmArgs &a);
bool plane_mfma_streams(const GemmArgs &a);     // tall matrix, 2 to 8 requests: the row-streaming form takes it
hipError_t plane_mfma_launch(const GemmArgs &a, hipStream_t stream);

// `count` matrices that share n, precision, batch and activations as ONE launch
bool plane_mfma_supports_multi(const GemmArgs *mats, int count);
bool plane_mfma_streams_multi(const GemmArgs *mats, int count);   // ... and the row-streaming form takes them together
hipError_t plane_mfma_launch_multi(const GemmArgs *mats, int count, hipStream_t stream);

bool dequant_mfma_supports(const GemmArgs &a);
// benchmarks and tests: force the workgroup shape (request tiles of 64, or 0 for one tile of 16; blocks of 16 rows); (0, 0) = automatic
bool dequant_mfma_force_shape(int request_tiles, int row_blocks);
// planewise: the variant that multiplies the +-1 planes themselves and scales the group sums (groups of 128 or 256)
hipError_t dequant_mfma_launch(const GemmArgs &a, hipStream_t stream, bool planewise = false, const GemmArgs *mats = nullptr, int count = 0);
// several matrices (same n, precision, batch, activations, group size; no offsets) in one launch of the large-batch kernels
bool dequant_mfma_supports_multi(const GemmArgs *mats, int count);
hipError_t dequant_mfma_launch_multi(const GemmArgs *mats, int count, hipStream_t stream, bool planewise);

// Offline quantiser (Algorithm 1): group must be 32, 64, 128 or 256; 1 <= p_low <= p_high <= 4.
bool quantize_supports(int64_t m, int64_t n, int group);
hipError_t quantize_launch(const _Float16 *w, int p_low, int p_high, int cycles, uint32_t *planes, _Float16 *const *scales_by_p,
                           _Float16 *const *offsets_by_p, int64_t m, int64_t n, int group, bool listing_residual, hipStream_t stream);

hipError_t pack_launch(const int8_t *codes, uint32_t *planes, int n_planes, int64_t m, int64_t n, hipStream_t stream);
hipError_t unpack_launch(const uint32_t *planes, int8_t *codes, int n_planes, int64_t m, int64_t n, hipStream_t stream);

}  // namespace bcq
