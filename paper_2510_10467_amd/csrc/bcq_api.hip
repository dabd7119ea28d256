// C ABI of the library: argument checks and kernel choice.  All arithmetic
// lives in the kernel files; this file never touches tensor data.
#include <hip/hip_runtime.h>

#include <map>
#include <mutex>
#include <utility>

#include "bcq.h"
#include "bcq_bench.h"
#include "bcq_internal.hpp"

namespace {

// test and benchmark knobs (bcq_bench.h): per host thread, so that one thread's forced variant never changes
// another thread's dispatch
thread_local int g_forced = BCQ_KERNEL_AUTO;
thread_local const char *g_last = "";

bool aligned(const void *p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

int check_shape(int64_t m, int64_t n, int batch, int group)
{
    if (m < 1 || n < 1 || batch < 0 || group < 32 || (group % 32) != 0 || n < group || (n % group) != 0)
        return BCQ_ERR_BAD_SHAPE;
    // index arithmetic inside the kernels is 64-bit, but word counts per row are kept in int
    if (n > (int64_t(1) << 30) || m > (int64_t(1) << 40)) return BCQ_ERR_BAD_SHAPE;
    return BCQ_OK;
}

// pack / unpack run one thread per plane word in workgroups of 256: the word count must fit one grid dimension
bool pack_grid_fits(int n_planes, int64_t m, int64_t n)
{
    if (m > (int64_t(1) << 40) || n > (int64_t(1) << 30)) return false;
    const int64_t words_per_plane_row = n / 32;
    if (m > ((int64_t(1) << 39) - 1) / (words_per_plane_row * n_planes)) return false;      // 2^31 blocks x 256 words
    return true;
}

// The kernel family a problem runs on: the forced one, or the default choice.
int choose(const bcq::GemmArgs &a)
{
    using namespace bcq;
    int choice = g_forced;
    if (choice == BCQ_KERNEL_AUTO) {
        // Dequantising a weight tile costs the same whatever the number of requests that then use it (the time
        // of that kernel is flat up to 16 and again up to 64 requests), while the plane-wise FP4 kernel grows with
        // the batch in steps of four requests.  Measured crossovers (Llama-3-8B and 70B shapes, p = 2 and 4): on
        // matrices of at least 8192 rows 9 requests (5 for p <= 2), from 4096 rows on 9; shorter matrices
        // leave the large-batch kernels too few workgroups.
        // Up to 32 requests (one tile of 16 or 32) multiplying the +-1 planes themselves and scaling the group sums
        // beats rebuilding the weights by up to 15 %; beyond that it is the other way round.
        const bool f16_ok = a.group >= 128;                     // the fp16 plane-wise variant needs one scale per 128-column step
        // (8192 columns and more: from 5 requests at any precision, 28672 x 8192 at p = 4 and 8 requests 85 -> 70 us)
        int from = a.m >= 8192 && (a.uniform_p <= 2 || a.n >= 8192) ? 5 : 9;
        bool tiles16 = f16_ok && a.batch <= 32;                 // one tile of 16 or 32 requests
        // Per-request precision: the plane-wise fp16 variant works in tiles of 16 requests whatever mix of
        // precisions they hold (from 9 requests on); rebuilding the weights
        // takes over from 65 requests (8192 rows and more) or 97 on, as one launch of the uniform kernel's body per
        // precision (see dequant_mfma_launch), and from 28 / 40 requests where the fp16 variant cannot run (up to 64
        // requests rebuilt once per precision present).
        if (a.uniform_p == 0) {
            from = f16_ok ? 9 : (a.m >= 8192 ? 28 : 40);
            tiles16 = f16_ok && a.batch <= (a.m >= 8192 ? 64 : 96);
        }
        bool pays = a.m >= 4096 && a.batch >= from;
        // Shorter matrices give the large-batch kernel few workgroups, but the FP4 kernel's time still grows with
        // the batch: measured crossovers at 24 / 40 / 70 requests for 3072 / 2048 / 1024 rows (p = 4; a fifth later
        // for p = 2), i.e. at about 80 000 (90 000) rows x requests.  Uniform precision only.
        if (a.m < 4096 && a.m >= 1024 && a.uniform_p > 0) pays = a.batch * a.m >= (a.uniform_p >= 3 ? 80000 : 90000);
        // ... and with per-request precision the tiles of 16 from about 70 000 rows x requests on (2048 rows: 32 requests),
        // up to 256 requests
        if (a.m < 4096 && a.m >= 1024 && a.uniform_p == 0 && f16_ok) {
            pays = a.batch * a.m >= 70000;
            tiles16 = a.batch <= 256;
        }
        // Tall matrices with up to eight requests (one request: at one or two planes): the row-streaming form of the
        // FP4 kernel beats both (14336 x 4096, eight requests: 13.7 us at p = 4 and 9.0 us at p = 2 against 19.4 and 11.9 us).
        if (plane_mfma_streams(a)) choice = BCQ_KERNEL_PLANE_MFMA;
        else if (dequant_mfma_supports(a) && pays) choice = tiles16 ? BCQ_KERNEL_PLANE_F16 : BCQ_KERNEL_DEQUANT_MFMA;
        else if (plane_mfma_supports(a)) choice = BCQ_KERNEL_PLANE_MFMA;
        // shapes the plane-wise kernel does not take (groups of 64, odd widths): the generic kernel repeats all
        // of its work per request, so the dequantising one wins from the second request on
        // (the plane-wise fp16 variant up to 32 requests, as on the shapes above)
        else if (dequant_mfma_supports(a) && a.batch >= 2 && a.m >= 1024) choice = tiles16 ? BCQ_KERNEL_PLANE_F16 : BCQ_KERNEL_DEQUANT_MFMA;
        // one request on a width the plane-wise kernel does not take, not too large: the large-batch kernels, whose time is
        // flat from one request on, are ahead of the table look-ups: the plane-wise fp16 variant from 2048 rows on (14336 x
        // 4224 at p = 4: 20.8 against 26.4 us; 2048 x 4224: 7.3 against 8.5; 14336 x 640: 5.5 against 12.4) and from 1024
        // rows on narrow matrices (1024 x 640: 3.2 against 4.1), the dequantising one (groups of 64) from 4096 rows on
        // (23.1 against 26.4 us), while 1024 x 4224 (7.1 against 6.7) and 28672 x 8320 (72 against 68) stay with the look-ups
        else if (dequant_mfma_supports(a) && a.uniform_p > 0 && a.m * a.n < (int64_t)150000000 &&
                 (f16_ok ? a.m >= 2048 || (a.m >= 1024 && a.n <= 2048) : a.m >= 4096))
            choice = f16_ok ? BCQ_KERNEL_PLANE_F16 : BCQ_KERNEL_DEQUANT_MFMA;
        // everything else (groups of 32, odd widths on short or very large matrices, more than four planes): table look-ups,
        // a third of the per-bit kernel's operations
        else choice = lut_supports(a) ? BCQ_KERNEL_LUT : BCQ_KERNEL_SIGN_SELECT;
    }
    return choice;
}

int run(const bcq::GemmArgs &a, hipStream_t stream)
{
    using namespace bcq;
    hipError_t err;
    switch (choose(a)) {
    case BCQ_KERNEL_SIGN_SELECT:
        if (!sign_select_supports(a)) return BCQ_ERR_VARIANT;
        err = sign_select_launch(a, stream);
        g_last = "sign_select";
        break;
    case BCQ_KERNEL_LUT:
        if (!lut_supports(a)) return BCQ_ERR_VARIANT;
        err = lut_launch(a, stream);
        g_last = "lut";
        break;
    case BCQ_KERNEL_PLANE_MFMA:
        if (!plane_mfma_supports(a)) return BCQ_ERR_VARIANT;
        err = plane_mfma_launch(a, stream);
        g_last = plane_mfma_streams(a) ? "plane_mfma_rows" : "plane_mfma";      // (the row-streaming form of the family)
        break;
    case BCQ_KERNEL_DEQUANT_MFMA:
        if (!dequant_mfma_supports(a)) return BCQ_ERR_VARIANT;
        err = dequant_mfma_launch(a, stream);
        g_last = "dequant_mfma";
        break;
    case BCQ_KERNEL_PLANE_F16:
        // a matrix instruction sums over all 128 columns of a step: one scale per row and step, so groups of 128 or 256
        if (!dequant_mfma_supports(a) || a.group < 128) return BCQ_ERR_VARIANT;
        err = dequant_mfma_launch(a, stream, true);
        g_last = "plane_f16";
        break;
    default:
        return BCQ_ERR_VARIANT;
    }
    return err == hipSuccess ? BCQ_OK : BCQ_ERR_HIP;
}

}  // namespace

namespace bcq {

hipError_t allow_dynamic_lds(const void *kernel, int bytes)
{
    if (bytes <= 64 * 1024) return hipSuccess;
    static std::mutex lock;
    static std::map<std::pair<int, const void *>, int> granted;      // (device, kernel) -> bytes already allowed
    int dev = 0;
    if (hipError_t e = hipGetDevice(&dev)) return e;
    std::lock_guard<std::mutex> guard(lock);
    int &have = granted[{dev, kernel}];
    if (bytes <= have) return hipSuccess;
    if (hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes)) return e;
    have = bytes;
    return hipSuccess;
}

}  // namespace bcq

extern "C" {

const char *bcq_strerror(int status)
{
    switch (status) {
    case BCQ_OK: return "ok";
    case BCQ_ERR_NULL: return "a required pointer is NULL";
    case BCQ_ERR_BAD_P: return "precision or plane count out of range";
    case BCQ_ERR_BAD_SHAPE: return "shape violates m>=1, n>=group, group%32==0, n%group==0, batch>=0";
    case BCQ_ERR_ALIGN: return "pointer not aligned (planes/scales/x: 16 bytes, y: 2 bytes)";
    case BCQ_ERR_HIP: return "HIP runtime error at kernel launch";
    case BCQ_ERR_VARIANT: return "forced kernel variant unknown or unable to run this problem";
    default: return "unknown status";
    }
}

int bcq_select_kernel(int variant)
{
    if (variant < BCQ_KERNEL_AUTO || variant > BCQ_KERNEL_LUT) return BCQ_ERR_VARIANT;
    g_forced = variant;
    return BCQ_OK;
}

int bcq_selected_kernel(void) { return g_forced; }

const char *bcq_last_kernel(void) { return g_last; }

int bcq_select_dequant_shape(int request_tiles, int row_blocks)
{
    return bcq::dequant_mfma_force_shape(request_tiles, row_blocks) ? BCQ_OK : BCQ_ERR_VARIANT;
}

int bcq_pack(const int8_t *codes, uint32_t *planes, int n_planes, int64_t m, int64_t n, void *stream)
{
    if (!codes || !planes) return BCQ_ERR_NULL;
    if (n_planes < 1 || n_planes > BCQ_MAX_PLANES) return BCQ_ERR_BAD_P;
    if (m < 1 || n < 32 || (n % 32) != 0 || !pack_grid_fits(n_planes, m, n)) return BCQ_ERR_BAD_SHAPE;
    if (!aligned(codes, 16) || !aligned(planes, 4)) return BCQ_ERR_ALIGN;
    return bcq::pack_launch(codes, planes, n_planes, m, n, static_cast<hipStream_t>(stream)) == hipSuccess
               ? BCQ_OK : BCQ_ERR_HIP;
}

int bcq_unpack(const uint32_t *planes, int8_t *codes, int n_planes, int64_t m, int64_t n, void *stream)
{
    if (!codes || !planes) return BCQ_ERR_NULL;
    if (n_planes < 1 || n_planes > BCQ_MAX_PLANES) return BCQ_ERR_BAD_P;
    if (m < 1 || n < 32 || (n % 32) != 0 || !pack_grid_fits(n_planes, m, n)) return BCQ_ERR_BAD_SHAPE;
    if (!aligned(codes, 16) || !aligned(planes, 4)) return BCQ_ERR_ALIGN;
    return bcq::unpack_launch(planes, codes, n_planes, m, n, static_cast<hipStream_t>(stream)) == hipSuccess
               ? BCQ_OK : BCQ_ERR_HIP;
}

int bcq_gemv_offset(const uint32_t *planes, const bcq_half *scales_p, const bcq_half *offsets_p, int p, const bcq_half *x,
                    bcq_half *y, int64_t m, int64_t n, int batch, int group, void *stream)
{
    if (!planes || !scales_p || !x || !y) return BCQ_ERR_NULL;
    if (p < 1 || p > BCQ_MAX_PLANES) return BCQ_ERR_BAD_P;
    if (int rc = check_shape(m, n, batch, group)) return rc;
    if (!aligned(planes, 16) || !aligned(scales_p, 16) || !aligned(offsets_p, 16) || !aligned(x, 16) || !aligned(y, 2))
        return BCQ_ERR_ALIGN;
    if (batch == 0) return BCQ_OK;
    bcq::GemmArgs a{};
    a.planes = planes;
    a.scales[p] = reinterpret_cast<const _Float16 *>(scales_p);
    a.offsets[p] = reinterpret_cast<const _Float16 *>(offsets_p);
    a.p_req = nullptr;
    a.uniform_p = p;
    a.p_max = p;
    a.x = reinterpret_cast<const _Float16 *>(x);
    a.y = reinterpret_cast<_Float16 *>(y);
    a.m = m;
    a.n = n;
    a.batch = batch;
    a.group = group;
    return run(a, static_cast<hipStream_t>(stream));
}

int bcq_gemv(const uint32_t *planes, const bcq_half *scales_p, int p, const bcq_half *x, bcq_half *y,
             int64_t m, int64_t n, int batch, int group, void *stream)
{
    return bcq_gemv_offset(planes, scales_p, nullptr, p, x, y, m, n, batch, group, stream);
}

int bcq_gemm_mixed_offset(const uint32_t *planes, const bcq_half *const *scales_by_p, const bcq_half *const *offsets_by_p,
                          const int32_t *p_req, int p_max, const bcq_half *x, bcq_half *y, int64_t m, int64_t n, int batch,
                          int group, void *stream)
{
    if (!planes || !scales_by_p || !p_req || !x || !y) return BCQ_ERR_NULL;
    if (p_max < 1 || p_max > BCQ_MAX_PLANES) return BCQ_ERR_BAD_P;
    if (int rc = check_shape(m, n, batch, group)) return rc;
    if (!aligned(planes, 16) || !aligned(x, 16) || !aligned(y, 2) || !aligned(p_req, 4)) return BCQ_ERR_ALIGN;
    bcq::GemmArgs a{};
    bool any = false;
    for (int q = 1; q <= p_max; ++q) {
        if (!aligned(scales_by_p[q], 16)) return BCQ_ERR_ALIGN;
        a.scales[q] = reinterpret_cast<const _Float16 *>(scales_by_p[q]);
        any = any || scales_by_p[q] != nullptr;
        if (offsets_by_p) {
            if (!aligned(offsets_by_p[q], 16)) return BCQ_ERR_ALIGN;
            a.offsets[q] = reinterpret_cast<const _Float16 *>(offsets_by_p[q]);
        }
    }
    if (!any) return BCQ_ERR_NULL;
    if (batch == 0) return BCQ_OK;
    a.planes = planes;
    a.p_req = p_req;
    a.uniform_p = 0;
    a.p_max = p_max;
    a.x = reinterpret_cast<const _Float16 *>(x);
    a.y = reinterpret_cast<_Float16 *>(y);
    a.m = m;
    a.n = n;
    a.batch = batch;
    a.group = group;
    return run(a, static_cast<hipStream_t>(stream));
}

int bcq_gemm_mixed(const uint32_t *planes, const bcq_half *const *scales_by_p, const int32_t *p_req, int p_max,
                   const bcq_half *x, bcq_half *y, int64_t m, int64_t n, int batch, int group, void *stream)
{
    return bcq_gemm_mixed_offset(planes, scales_by_p, nullptr, p_req, p_max, x, y, m, n, batch, group, stream);
}

int bcq_gemv_multi(int count, const uint32_t *const *planes, const bcq_half *const *scales_p, const int64_t *m,
                   bcq_half *const *y, int p, const bcq_half *x, int64_t n, int batch, int group, void *stream)
{
    if (count < 1 || count > BCQ_MAX_MULTI) return BCQ_ERR_BAD_SHAPE;
    if (!planes || !scales_p || !m || !y || !x) return BCQ_ERR_NULL;
    if (p < 1 || p > BCQ_MAX_PLANES) return BCQ_ERR_BAD_P;
    bcq::GemmArgs mats[BCQ_MAX_MULTI] = {};
    for (int k = 0; k < count; ++k) {
        if (!planes[k] || !scales_p[k] || !y[k]) return BCQ_ERR_NULL;
        if (int rc = check_shape(m[k], n, batch, group)) return rc;
        if (!aligned(planes[k], 16) || !aligned(scales_p[k], 16) || !aligned(x, 16) || !aligned(y[k], 2)) return BCQ_ERR_ALIGN;
        bcq::GemmArgs &a = mats[k];
        a.planes = planes[k];
        a.scales[p] = reinterpret_cast<const _Float16 *>(scales_p[k]);
        a.uniform_p = p;
        a.p_max = p;
        a.x = reinterpret_cast<const _Float16 *>(x);
        a.y = reinterpret_cast<_Float16 *>(y[k]);
        a.m = m[k];
        a.n = n;
        a.batch = batch;
        a.group = group;
    }
    if (batch == 0) return BCQ_OK;
    // one launch when every matrix would run on the plane-wise kernel anyway
    // (or when the row-streaming form takes all their rows together: two to eight requests, or one request at one or
    // two planes, 640 row blocks in all)
    const bool forced_elsewhere = g_forced != BCQ_KERNEL_AUTO && g_forced != BCQ_KERNEL_PLANE_MFMA;
    const bool streams = count > 1 && !forced_elsewhere && bcq::plane_mfma_streams_multi(mats, count);
    bool together = count > 1 && bcq::plane_mfma_supports_multi(mats, count);
    for (int k = 0; together && !streams && k < count; ++k) together = choose(mats[k]) == BCQ_KERNEL_PLANE_MFMA;
    if (together) {
        g_last = streams ? "plane_mfma_rows" : "plane_mfma";
        return bcq::plane_mfma_launch_multi(mats, count, static_cast<hipStream_t>(stream)) == hipSuccess ? BCQ_OK : BCQ_ERR_HIP;
    }
    // larger batches: one launch of the large-batch kernels when the matrices taken together (one matrix of all their
    // rows) would run there; k and v projections of 1024 rows are too short for those kernels on their own
    if (count > 1 && bcq::dequant_mfma_supports_multi(mats, count)) {
        bcq::GemmArgs all = mats[0];
        all.m = 0;
        for (int k = 0; k < count; ++k) all.m += mats[k].m;
        const int c = choose(all);
        if ((c == BCQ_KERNEL_PLANE_F16 && group >= 128) || c == BCQ_KERNEL_DEQUANT_MFMA) {
            g_last = c == BCQ_KERNEL_PLANE_F16 ? "plane_f16" : "dequant_mfma";
            return bcq::dequant_mfma_launch_multi(mats, count, static_cast<hipStream_t>(stream), c == BCQ_KERNEL_PLANE_F16) == hipSuccess
                       ? BCQ_OK : BCQ_ERR_HIP;
        }
    }
    for (int k = 0; k < count; ++k)
        if (int rc = run(mats[k], static_cast<hipStream_t>(stream))) return rc;
    return BCQ_OK;
}

int bcq_quantize(const bcq_half *w, int p_low, int p_high, int cycles, uint32_t *planes, bcq_half *const *scales_by_p,
                 bcq_half *const *offsets_by_p, int64_t m, int64_t n, int group, void *stream)
{
    return bcq_quantize_form(w, p_low, p_high, cycles, BCQ_RESIDUAL_FROZEN_PLANES, planes, scales_by_p, offsets_by_p, m, n, group, stream);
}

int bcq_quantize_form(const bcq_half *w, int p_low, int p_high, int cycles, int residual_form, uint32_t *planes,
                      bcq_half *const *scales_by_p, bcq_half *const *offsets_by_p, int64_t m, int64_t n, int group, void *stream)
{
    if (residual_form != BCQ_RESIDUAL_FROZEN_PLANES && residual_form != BCQ_RESIDUAL_LISTING) return BCQ_ERR_VARIANT;
    if (!w || !planes || !scales_by_p) return BCQ_ERR_NULL;
    if (p_low < 1 || p_high < p_low || p_high > 4 || cycles < 0 || (cycles < 1 && p_high > p_low)) return BCQ_ERR_BAD_P;
    if (int rc = check_shape(m, n, 0, group)) return rc;
    if (!bcq::quantize_supports(m, n, group)) return BCQ_ERR_BAD_SHAPE;
    if (!aligned(w, 16) || !aligned(planes, 4)) return BCQ_ERR_ALIGN;
    for (int p = p_low; p <= p_high; ++p) {
        if (!scales_by_p[p] || (offsets_by_p && !offsets_by_p[p])) return BCQ_ERR_NULL;
        if (!aligned(scales_by_p[p], 2) || (offsets_by_p && !aligned(offsets_by_p[p], 2))) return BCQ_ERR_ALIGN;
    }
    hipError_t err = bcq::quantize_launch(reinterpret_cast<const _Float16 *>(w), p_low, p_high, cycles, planes,
                                          reinterpret_cast<_Float16 *const *>(scales_by_p),
                                          reinterpret_cast<_Float16 *const *>(offsets_by_p), m, n, group,
                                          residual_form == BCQ_RESIDUAL_LISTING, static_cast<hipStream_t>(stream));
    g_last = "quantize";
    return err == hipSuccess ? BCQ_OK : BCQ_ERR_HIP;
}

}  // extern "C"
