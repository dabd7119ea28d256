// Small-batch kernel: bit-planes go straight into the CDNA4 FP4 matrix pipe.
//
// Section 3.3 forms B_i x per plane by adding and subtracting activations and
// keeps the regime memory-bound.  On gfx950 the vector ALU cannot add/subtract
// fast enough to keep up with 8 TB/s of one-bit weights, so the sign-accumulate
// of one whole scale group (16 rows x 128 columns x 1 plane = 2048 weight bits)
// is issued as ONE v_mfma_f32_16x16x128_f8f6f4:
//
//   * weight operand (MFMA "B", 16 columns = 16 weight rows): every weight bit
//     becomes the FP4 (E2M1) code 0x2 | sign, i.e. exactly +-1: one AND-OR per
//     operand register, three of them after a shift.  Which bit lands in which
//     K slot is a fixed permutation, mirrored on the activation side.
//   * activation operand (MFMA "A", 16 rows): binary16 activations are split
//     EXACTLY, over the whole binary16 range, into four E5M2 terms (E5M2 is the
//     top byte of binary16: t_k = top byte of the running remainder, which is
//     scaled up by 4, 8, 8 between the terms so that the low bits of small
//     values stay above the 2^-16 spacing of E5M2 subnormals;
//     x = t0 + t1/4 + t2/32 + t3/256).  Row
//     4*b + k of the operand holds term k of request b, so one instruction
//     serves up to four requests.  The split is done once per workgroup and
//     parked in LDS in operand-register order.  Operand rows of absent requests
//     hold arbitrary finite or non-finite data: row m of the result depends on
//     row m of the operand only, and those result rows are never stored.
//   * result: lane (row r, request b) receives the four term sums of its own
//     row, adds them, multiplies by alpha_i[r][group] of ITS request's
//     precision, and accumulates in fp32.  Requests at different precisions
//     share the plane sweep; a lane's scales beyond p_b are zero.
//
// Asymmetric scheme (section 4.1): the offset z[r][g] of a (row, group) multiplies the plain sum of the
// group's activations, which depends on neither row nor plane; it is formed beside the operand image
// (one float per request and group, kept in the image's padding) and costs one FMA per group.
//
// Work split: a workgroup owns RB blocks of 16 rows and the whole K range;
// wave (rb, ks) handles K slice ks (1024 columns) of row block rb, issues all
// of its plane and scale loads up front (128-bit, 128 contiguous bytes per row
// and plane), and the KS partial sums are combined through LDS in a fixed
// order, so results are deterministic and no global scratch is needed.
#include <hip/hip_runtime.h>

#include <type_traits>

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

// Uniform launch parameters, computed on the host so the kernel does no address algebra of its own.
struct PlaneMfmaParams {
    const unsigned char *planes;            // plane 0
    const unsigned char *x;                 // activations of request 0 of the whole batch
    _Float16 *y;
    const unsigned char *scales[BCQ_MAX_PLANES + 1];   // scale set per precision (bytes)
    const unsigned char *offsets[BCQ_MAX_PLANES + 1];  // offsets [m][n/group] per precision, or nullptr (asymmetric scheme)
    const int32_t *p_req;                   // per-request precisions (mixed) or nullptr
    uint32_t set_mask;                      // bit k set: scales[k] is there (k = 1 .. 4)
    uint32_t offset_mask;                   // bit k set: offsets[k] is there
    uint32_t plane_stride;                  // bytes between planes:      m * n / 8
    uint32_t row_stride;                    // bytes between plane rows:  n / 8
    uint32_t scale_plane_stride;            // bytes between scale planes: m * (n/128) * 2
    uint32_t scale_row_stride;              // bytes between scale rows:   (n/128) * 2
    uint32_t x_stride;                      // bytes between requests:    n * 2
    uint32_t m;
    int batch, p_max, uniform_p;
    int KS, RB, nchunk, nslices;
    int glast;                              // 128-column groups in the last slice (8 unless n is not a multiple of 1024)
    // several matrices with the same n, p and activations in one launch (MULTI kernels): matrix k owns the
    // row blocks mat_blk0[k] .. mat_blk0[k+1]-1 of the grid; unused entries hold the total
    const unsigned char *mat_planes[BCQ_MAX_MULTI];
    const unsigned char *mat_scales[BCQ_MAX_MULTI];
    _Float16 *mat_y[BCQ_MAX_MULTI];
    uint32_t mat_m[BCQ_MAX_MULTI];
    uint32_t mat_blk0[BCQ_MAX_MULTI];
    uint32_t ntiles, nwg_rows;              // batch tiles of four requests; row-block groups (workgroups per tile)
    float inv_span;                         // 1 / (8 * ntiles)
    float inv_ks;                           // 1 / KS
};

// LDS layout for NB requests per tile, KS slices and RB row blocks per workgroup:
//   [0, image)        operand image: 16-byte rows; slice ks, group g, register half h, lane quarter qa, operand
//                     row r at ks*kSliceImage + g*kGroupBytes + h*kHalfBytes + (qa*4NB + r)*16
//   [image, red)      a tile per wave in which plane words change from row-major to operand order
//   [red, total)      one fp32 partial sum per thread for the final combine
template <int NB>
struct Lds {
    static constexpr int kRows = 4 * NB;
    static constexpr int kHalfBytes = 4 * kRows * 16 + 16;          // operand registers 0-3 (or 4-7) of all lanes, padded
    static constexpr int kGroupBytes = 2 * kHalfBytes;              // one group's image; the padding spreads LDS banks
    static constexpr int kSliceImage = kSliceGroups * kGroupBytes;   // 4 KiB * NB
    static constexpr int kTileRow = 128 + 16;                        // padded so that rows start 4 banks apart (mod 64)
    static constexpr int kWaveTile = 16 * kTileRow;                  // 16 rows x 128 bytes of one plane
    __host__ __device__ static constexpr int tile_off(int KS) { return KS * kSliceImage; }
    __host__ __device__ static constexpr int red_off(int KS, int RB) { return KS * kSliceImage + KS * RB * kWaveTile; }
    __host__ __device__ static constexpr int total(int KS, int RB) { return red_off(KS, RB) + 64 * KS * RB * 4; }
};

// 32 weight bits -> the lane's four FP4 operand registers (8 codes each).
// Register s, nibble i carries bit 4i + 3 - s in its sign position over the code of 1.0.
// `sign` and `one` hold 0x88888888 and 0x22222222 in registers so each line is one V_AND_OR_B32.
__device__ __forceinline__ v8i expand_plane_word(uint32_t w, uint32_t sign, uint32_t one)
{
    v8i r = {0, 0, 0, 0, 0, 0, 0, 0};
    r[0] = (int)((w & sign) | one);
    r[1] = (int)(((w << 1) & sign) | one);
    r[2] = (int)(((w << 2) & sign) | one);
    r[3] = (int)(((w << 3) & sign) | one);
    return r;
}

// The four E5M2 terms of an activation carry the scales 1, 4, 32 and 256 (see the conversion in `sweep`);
// their sums over a group, rows 4b .. 4b + 3 of the result, recombine to the group sum of request b.
// Every product is a power-of-two scaling, so the only roundings are those of the fp32 additions.
__device__ __forceinline__ float term_sum(v4f d)
{
    return fmaf(fmaf(d[3], 0.125f, d[2]), 0.03125f, fmaf(d[1], 0.25f, d[0]));
}

// Sum of a value over the 8 lanes l & ~7 .. l | 7 (result in all of them).
__device__ __forceinline__ float sum_over_8_lanes(float v)
{
    // quad_perm(1,0,3,2), quad_perm(2,3,0,1), row_half_mirror
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xf, 0xf, false));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xf, 0xf, false));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xf, 0xf, false));
    return v;
}

// What one wave fetches for one K slice: activations, scales, plane words.
template <int PH, int NB>
struct SliceLoads {
    u32x4 xv[NB][2];                        // 16 consecutive columns (one image unit) per request slot
    u32x4 sc[PH];                           // the 8 scales of the lane's row, per plane (groups of 64: the first 8 of 16)
    u32x4 sc2[PH];                          // groups of 64 columns only: scales 8..15 of the slice
    u32x4 zc;                               // the 8 offsets of the lane's row (asymmetric scheme only)
    u32x4 zc2;                              // groups of 64 columns only: offsets 8..15 of the slice
    u32x4 wa[PH], wb[PH];                   // plane words: rows 0-7 and rows 8-15 of the block
};

// Lane addressing of a wave, fixed for the whole kernel.
struct LaneOffsets {
    uint32_t wa, wb;                        // byte offsets into a plane of the rows of the lane's two plane loads
    uint32_t s;                             // byte offset into a scale plane: row * scale_row_stride
    uint32_t x[kMaxBatchTile];              // byte offset of each request slot's activations
    uint32_t lane;
};

// 128-bit logical shift right by 16 bits: drops the first of eight binary16 values, the last becomes 0
__device__ __forceinline__ u32x4 drop_first_half(u32x4 v)
{
    return u32x4{__builtin_amdgcn_alignbit(v.y, v.x, 16), __builtin_amdgcn_alignbit(v.z, v.y, 16),
                 __builtin_amdgcn_alignbit(v.w, v.z, 16), v.w >> 16};
}

// four binary16 values in v.x, v.y -> each of them twice: {a, a, b, b, c, c, d, d}
__device__ __forceinline__ u32x4 each_twice(u32x4 v)
{
    return u32x4{__builtin_amdgcn_perm(v.x, v.x, 0x01000100u), __builtin_amdgcn_perm(v.x, v.x, 0x03020302u),
                 __builtin_amdgcn_perm(v.y, v.y, 0x01000100u), __builtin_amdgcn_perm(v.y, v.y, 0x03020302u)};
}

// GS: scale groups of 128 columns (0: a slice has eight scales per row), of 256 (+1: four) or of 64 (-1: sixteen)
template <int PH, int NB, bool MIXED, bool OFFSET, int GS>
__device__ __forceinline__ void issue_loads(SliceLoads<PH, NB> &ld, const PlaneMfmaParams &pr, const LaneOffsets &off,
                                            const unsigned char *sbase, const unsigned char *zbase, int p_mine, int slice_c,
                                            int ngroups)
{
    // A last slice of ngroups < 8 groups: lanes whose columns or group lie past the end of the row fetch
    // the slice's first unit or group instead (valid memory, finite values; the scales of those groups
    // are zero), and the 16 bytes of scales are the LAST eight of the row, shifted into place later.
    const uint32_t x_lane = off.lane < (uint32_t)ngroups * 8 ? off.lane * 32 : 0;
    const uint32_t w_lane = (off.lane & 7) < (uint32_t)ngroups ? (off.lane & 7) * 16 : 0;
    // (scale groups of 256 columns: four scales = 8 bytes per slice, spread to eight after the loads)
    constexpr uint32_t s_bytes = GS > 0 ? kSliceGroups : GS < 0 ? kSliceGroups * 4 : kSliceGroups * 2;
    const uint32_t s_slice = ngroups < kSliceGroups ? pr.scale_row_stride - s_bytes : (uint32_t)slice_c * s_bytes;
    auto load_scales = [&](const unsigned char *p) {
        if constexpr (GS > 0) {
            const v2u t = *reinterpret_cast<const v2u *>(p);
            return u32x4{t.x, t.y, 0u, 0u};
        } else {
            return *reinterpret_cast<const u32x4 *>(p);
        }
    };
    // in the order of use: activations, scales, planes.  Every address is a wave-uniform 64-bit base plus
    // a 32-bit lane offset, which is an addressing mode of the load instruction: no 64-bit lane arithmetic.
    const unsigned char *x_base = pr.x + (uint32_t)slice_c * (kSliceCols * 2);
#pragma unroll
    for (int bb = 0; bb < NB; ++bb) {
        const uint32_t xo = off.x[bb] + x_lane;
        ld.xv[bb][0] = *reinterpret_cast<const u32x4 *>(x_base + xo);
        ld.xv[bb][1] = *reinterpret_cast<const u32x4 *>(x_base + xo + 16);
    }
#pragma unroll
    for (int i = 0; i < PH; ++i) {
        if constexpr (MIXED) {
            const int ii = min(i, max(p_mine, 1) - 1);              // stay inside the lane's own scale set
            ld.sc[i] = load_scales(sbase + (size_t)ii * pr.scale_plane_stride + off.s + s_slice);
            if constexpr (GS < 0) ld.sc2[i] = load_scales(sbase + (size_t)ii * pr.scale_plane_stride + off.s + s_slice + 16);
        } else {
            const unsigned char *s_base = sbase + (size_t)i * pr.scale_plane_stride + s_slice;
            ld.sc[i] = load_scales(s_base + off.s);
            if constexpr (GS < 0) ld.sc2[i] = load_scales(s_base + off.s + 16);
        }
    }
    if constexpr (OFFSET) {
        ld.zc = load_scales(zbase + s_slice + off.s);
        if constexpr (GS < 0) ld.zc2 = load_scales(zbase + s_slice + off.s + 16);
    }
    const uint32_t wa = off.wa + w_lane, wb = off.wb + w_lane;
#pragma unroll
    for (int i = 0; i < PH; ++i) {
        // rows 0-7, then rows 8-15 of the block: 128 contiguous bytes per row and instruction
        const unsigned char *w_base = pr.planes + (size_t)i * pr.plane_stride + (uint32_t)slice_c * (kSliceCols / 8);
        ld.wa[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(w_base + wa));
        ld.wb[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(w_base + wb));
    }
}

// Sweep of one wave over its K slices for PH planes; returns this lane's partial sum.
//   p_mine   precision of the request this lane reports on (0: none); sbase its scale set
// MIXED: lanes of different quarters may belong to requests of different precisions.
// OFFSET: asymmetric scheme; zbase is the offset set of the lane's request (any readable array of that
//         size when z_on is false: the request has none).
template <int PH, int NB, bool MIXED, bool OFFSET, int GS>
__device__ __forceinline__ float sweep(const PlaneMfmaParams &pr, unsigned char *lds, int ks, int rb, int RB, int wave, int lane,
                                       const LaneOffsets &off, int p_mine, const unsigned char *sbase,
                                       const unsigned char *zbase, bool z_on)
{
    using L = Lds<NB>;
    const int KS = pr.KS;

    float acc = 0.f;
    int chunk = 0;
    do {                                                            // nchunk >= 1
        const int slice = __builtin_amdgcn_readfirstlane(chunk * KS + ks);      // the same in all lanes of a wave
        const bool slice_ok = slice < pr.nslices;                   // the last chunk may be ragged
        const int p_eff = slice_ok ? p_mine : 0;
        const int ngroups = slice == pr.nslices - 1 ? pr.glast : kSliceGroups;   // so may the last slice

        // ---- 0. the loads go out before anything else is computed: every instruction ahead of them
        // delays the memory phase of all waves that share the SIMD.  The lane id is made opaque after
        // them so that no LDS address arithmetic is moved in front of the loop.
        SliceLoads<PH, NB> ld;
        issue_loads<PH, NB, MIXED, OFFSET, GS>(ld, pr, off, sbase, zbase, p_mine, slice_ok ? slice : 0, ngroups);
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("" : "+v"(lane));

        // constants kept in registers so that (w & sign) | one is a single three-operand instruction
        uint32_t sign = 0x88888888u, one = 0x22222222u;
        asm volatile("" : "+v"(one));
        asm volatile("" : "+s"(sign));

        const int q = lane >> 4, r16 = lane & 15;
        // operand-image address of this lane: row min(r16, 4NB-1) of quarter q, first group of the wave's slice
        const int arow = r16 < L::kRows ? r16 : L::kRows - 1;
        const unsigned char *img_lane = lds + ks * L::kSliceImage + (q * L::kRows + arow) * 16;
        // image unit `lane` of the slice = 16 consecutive columns: group lane >> 3, part u16 = lane & 7.  Column
        // 16u + low + 4i (i = 0..3) belongs to operand byte 8z + 4(u&1) + i of lane quarter 2*((u>>1)&1) + w
        // with 2w + z = 3 - low, so a unit yields one dword for each (low, term): 16 dword stores.
        const int u16 = lane & 7;
        unsigned char *img_group = lds + ks * L::kSliceImage + (lane >> 3) * L::kGroupBytes;
        unsigned char *img_unit = img_group + (u16 >> 2) * L::kHalfBytes + (2 * ((u16 >> 1) & 1) * L::kRows) * 16 + 4 * (u16 & 1);
        // asymmetric scheme: sum_j x_j of a group, one float per request slot in the padding behind the
        // first half of the group's image; this lane reads the one of its own request slot
        const unsigned char *img_xsum = lds + ks * L::kSliceImage + 4 * L::kRows * 16 + (q < NB ? q : NB - 1) * 4;
        // Plane words change hands inside the wave, row-major in, operand-major out: the wave's tile holds
        // one plane's 16 rows x 128 bytes.  Rows are 144 bytes apart, so the 64 dword reads of one group,
        // one per (row, K quarter), fall into 64 different banks.
        unsigned char *tile = lds + L::tile_off(KS) + wave * L::kWaveTile;
        unsigned char *tile_wr = tile + (lane >> 3) * L::kTileRow + (lane & 7) * 16;
        const unsigned char *tile_rd = tile + r16 * L::kTileRow + q * 4;

        // ---- 1. operand image of this slice: the RB waves that share it convert one request slot in RB each.
        // A wave reads back only what waves of its own slice wrote; with RB == 1 that is the wave itself,
        // whose LDS operations complete in order, so no barrier is needed.
#pragma unroll
        for (int bb = 0; bb < NB; ++bb) {
            const int b = rb + bb * RB;                             // request slot of the tile
            if (b >= NB) break;
            const u32x4 c0 = ld.xv[bb][0], c1 = ld.xv[bb][1];
            const uint32_t dwd[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};       // dword k = columns 2k, 2k+1
            if constexpr (OFFSET) {
                // the unit's 16 activations in fp32, then the group's 8 units (= 8 lanes)
                float xsum = 0.f;
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const h2 pair = __builtin_bit_cast(h2, dwd[k]);
                    xsum += (float)pair[0];
                    xsum += (float)pair[1];
                }
                if constexpr (GS < 0) {
                    // groups of 64 columns: the units 0-3 and 4-7 of the 128 columns are two groups; each sum goes into the
                    // padding behind its own half of the image
                    xsum += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, xsum), 0xB1, 0xf, 0xf, false));
                    xsum += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, xsum), 0x4E, 0xf, 0xf, false));
                    if ((u16 & 3) == 0) *reinterpret_cast<float *>(img_group + (u16 >> 2) * L::kHalfBytes + 4 * L::kRows * 16 + b * 4) = xsum;
                } else {
                    xsum = sum_over_8_lanes(xsum);
                    if (u16 == 0) *reinterpret_cast<float *>(img_group + 4 * L::kRows * 16 + b * 4) = xsum;
                }
            }
#pragma unroll
            for (int low = 0; low < 4; ++low) {
                const uint32_t sel = (low & 1) ? 0x07060302u : 0x05040100u;                   // upper or lower halves
                const int k0 = low >> 1;
                // packed pairs (col low, col low+4) and (col low+8, col low+12)
                h2 r01 = __builtin_bit_cast(h2, __builtin_amdgcn_perm(dwd[k0 + 2], dwd[k0], sel));
                h2 r23 = __builtin_bit_cast(h2, __builtin_amdgcn_perm(dwd[k0 + 6], dwd[k0 + 4], sel));
                const int inv = 3 - low, w = inv >> 1, z = inv & 1;
                uint32_t *d32 = reinterpret_cast<uint32_t *>(img_unit + w * (L::kRows * 16) + 8 * z + b * 64);
                // exact split into four E5M2 terms: term j is the top byte of the running binary16 remainder, and
                // the remainder is scaled by 4, 8 and 8 on the way (never past the value it came from, so nothing
                // overflows): the terms carry the scales 1, 4, 32 and 256, which term_sum() undoes.  Without the
                // scaling the terms, whose spacing ends at 2^-16, would lose the low bits of small activations.
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t t01 = __builtin_bit_cast(uint32_t, r01) & 0xFF00FF00u;
                    const uint32_t t23 = __builtin_bit_cast(uint32_t, r23) & 0xFF00FF00u;
                    if (j < 3) {
                        const _Float16 c = j == 0 ? (_Float16)4.0f : (_Float16)8.0f;
                        r01 = (r01 - __builtin_bit_cast(h2, t01)) * h2{c, c};
                        r23 = (r23 - __builtin_bit_cast(h2, t23)) * h2{c, c};
                    }
                    d32[4 * j] = __builtin_amdgcn_perm(t23, t01, 0x07050301u);              // bytes: i = 0, 1, 2, 3
                }
            }
        }
        if (RB > 1) __syncthreads();

        // scale groups of 256 columns: each of the four scales fetched serves two groups of 128
        if constexpr (GS > 0) {
#pragma unroll
            for (int i = 0; i < PH; ++i) ld.sc[i] = each_twice(ld.sc[i]);
            if constexpr (OFFSET) ld.zc = each_twice(ld.zc);
        }
        // short last slice: its scales are the last ngroups of the eight fetched; the rest become zero
        if (GS >= 0 && ngroups < kSliceGroups) {          // (groups of 64 columns come with whole slices only)
            for (int k = ngroups; k < kSliceGroups; ++k) {
#pragma unroll
                for (int i = 0; i < PH; ++i) ld.sc[i] = drop_first_half(ld.sc[i]);
                if constexpr (OFFSET) ld.zc = drop_first_half(ld.zc);
            }
        }
        if constexpr (OFFSET) {
            if (!z_on || !slice_ok) {
                ld.zc = u32x4{0, 0, 0, 0};
                if constexpr (GS < 0) ld.zc2 = u32x4{0, 0, 0, 0};
            }
        }
        // scales of planes this lane must not use (beyond its precision, or a slice past the end) become zero
        if (MIXED || !slice_ok) {
#pragma unroll
            for (int i = 0; i < PH; ++i)
                if (!(i < p_eff)) {
                    ld.sc[i] = u32x4{0, 0, 0, 0};
                    if constexpr (GS < 0) ld.sc2[i] = u32x4{0, 0, 0, 0};
                }
        }

        // ---- 2. plane words into operand order.  LDS operations of a wave complete in order: a plane
        // may overwrite the previous one as soon as its reads have been issued.
        uint32_t wt[PH][kSliceGroups];
#pragma unroll
        for (int i = 0; i < PH; ++i) {
            *reinterpret_cast<u32x4 *>(tile_wr) = ld.wa[i];
            *reinterpret_cast<u32x4 *>(tile_wr + 8 * L::kTileRow) = ld.wb[i];
#pragma unroll
            for (int g = 0; g < kSliceGroups; ++g)
                wt[i][g] = *reinterpret_cast<const uint32_t *>(tile_rd + g * 16);
        }

        // ---- 3. per group: expand plane words, one MFMA per (group, plane), scale, accumulate;
        // the operand rows of the next group are fetched while this one is in the matrix pipe
        u32x4 lo = *reinterpret_cast<const u32x4 *>(img_lane);
        u32x4 hi = *reinterpret_cast<const u32x4 *>(img_lane + L::kHalfBytes);
        float xsum = 0.f;
        if constexpr (OFFSET) xsum = *reinterpret_cast<const float *>(img_xsum);
#pragma unroll
        for (int gl = 0; gl < kSliceGroups; ++gl) {
            const v8i xa = {(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
            if constexpr (OFFSET && GS < 0) {
                // groups of 64 columns: offsets 2 gl and 2 gl + 1 of the slice times the sums of the two halves
                const uint32_t zw = gl < 4 ? ld.zc[gl & 3] : ld.zc2[gl & 3];
                const float z_lo = (float)__builtin_bit_cast(_Float16, (unsigned short)(zw & 0xffffu));
                const float z_hi = (float)__builtin_bit_cast(_Float16, (unsigned short)(zw >> 16));
                const float xsum_hi = *reinterpret_cast<const float *>(img_xsum + gl * L::kGroupBytes + L::kHalfBytes);
                acc = fmaf(z_lo, xsum, acc);
                acc = fmaf(z_hi, xsum_hi, acc);
            } else if constexpr (OFFSET) {
                // offset of the group times the sum of its activations
                const uint32_t zw = ld.zc[gl >> 1];
                const float z = (float)__builtin_bit_cast(_Float16, (unsigned short)((gl & 1) ? (zw >> 16) : (zw & 0xffffu)));
                acc = fmaf(z, xsum, acc);
            }
            if (gl + 1 < kSliceGroups) {
                lo = *reinterpret_cast<const u32x4 *>(img_lane + (gl + 1) * L::kGroupBytes);
                hi = *reinterpret_cast<const u32x4 *>(img_lane + (gl + 1) * L::kGroupBytes + L::kHalfBytes);
                if constexpr (OFFSET) xsum = *reinterpret_cast<const float *>(img_xsum + (gl + 1) * L::kGroupBytes);
            }
            if constexpr (GS < 0) {
                // Groups of 64 columns: columns 0-63 of the 128 sit in operand registers 0-3, columns 64-127 in
                // registers 4-7, so each half gets an instruction of its own with the other half zeroed.  The
                // sums of a plane are taken while the next plane is in the matrix pipe.
                const v8i xa_lo = {xa[0], xa[1], xa[2], xa[3], 0, 0, 0, 0}, xa_hi = {0, 0, 0, 0, xa[4], xa[5], xa[6], xa[7]};
                const v4f zero = {0.f, 0.f, 0.f, 0.f};
                v4f d_lo = zero, d_hi = zero;
#pragma unroll
                for (int i = 0; i <= PH; ++i) {
                    v4f n_lo = zero, n_hi = zero;
                    if (i < PH) {
                        const v8i wb = expand_plane_word(wt[i][gl], sign, one);
                        n_lo = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(xa_lo, wb, zero, 1, 4, 0, 0, 0, 0);
                        n_hi = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(xa_hi, wb, zero, 1, 4, 0, 0, 0, 0);
                    }
                    if (i > 0) {
                        // scales 2 gl and 2 gl + 1 of the slice: the two halves of dword gl of the sixteen fetched
                        const uint32_t sw = gl < 4 ? ld.sc[i - 1][gl & 3] : ld.sc2[i - 1][gl & 3];
                        const float a_lo = (float)__builtin_bit_cast(_Float16, (unsigned short)(sw & 0xffffu));
                        const float a_hi = (float)__builtin_bit_cast(_Float16, (unsigned short)(sw >> 16));
                        acc = fmaf(-a_lo, term_sum(d_lo), acc);
                        acc = fmaf(-a_hi, term_sum(d_hi), acc);
                    }
                    d_lo = n_lo;
                    d_hi = n_hi;
                }
            } else {
                v4f d[PH];
#pragma unroll
                for (int i = 0; i < PH; ++i) {
                    const v8i wb = expand_plane_word(wt[i][gl], sign, one);
                    const v4f zero = {0.f, 0.f, 0.f, 0.f};
                    // A: E5M2 activation terms (cbsz = 1), B: FP4 weight codes (blgp = 4), no block scaling
                    d[i] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(xa, wb, zero, 1, 4, 0, 0, 0, 0);
                }
#pragma unroll
                for (int i = 0; i < PH; ++i) {
                    const uint32_t sw = ld.sc[i][gl >> 1];
                    const float alpha = (float)__builtin_bit_cast(_Float16, (unsigned short)((gl & 1) ? (sw >> 16) : (sw & 0xffffu)));
                    const float sum = term_sum(d[i]);
                    // the FP4 sign bit is set for weight bit 1 (= +1), so the instruction returns -(B_i x)
                    acc = fmaf(-alpha, sum, acc);
                }
            }
            // groups stay in order: deferring the sums would keep every MFMA result register alive
            __builtin_amdgcn_sched_barrier(0);
        }
        asm volatile("" : "+v"(acc));                               // the sums are due here, not past the branch below
        if (RB > 1) __syncthreads();                                // image no longer read: the next chunk may replace it
    } while (++chunk < pr.nchunk);
    return acc;
}

// Waves per workgroup.  Four requests of mixed precision per tile need more registers than a 16-wave
// workgroup leaves a wave (128), and their operand image limits the waves per CU anyway: they stop at 8.
// So do groups of 64 columns (twice the scales and two results per plane in flight).
__host__ __device__ constexpr int max_waves(int NB, bool mixed, int gs = 0) { return (NB == 4 && mixed) || gs < 0 ? 8 : 16; }

template <int P, int NB, bool MIXED, bool OFFSET, bool MULTI = false, int GS = 0>
__global__ __launch_bounds__(64 * max_waves(NB, MIXED, GS)) void plane_mfma_kernel(PlaneMfmaParams pr_in)
{
    PlaneMfmaParams pr = pr_in;               // MULTI kernels overwrite the per-matrix fields below
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int KS = pr.KS;
    // One request per tile (NB == 1): a workgroup is one row block, wave = K slice, the grid is exact.
    // Otherwise RB row blocks share a workgroup and the batch tiles of a row-block group are spread over ids.
    int RB = 1, ks = wave, rb = 0;            // K slice of this wave inside a chunk, row block inside the workgroup
    uint32_t tile = 0, wg = blockIdx.x;
    if constexpr (NB > 1) {
        // all of this without branches, so that every kernel argument is fetched in one go
        RB = pr.RB;
        rb = (int)(((float)wave + 0.5f) * pr.inv_ks);               // wave / KS for wave < 16 (0 when RB == 1)
        ks = wave - rb * KS;
        // Workgroup id -> (row-block group, batch tile).  Ids that differ by 8 run on the same XCD (ids
        // are dealt round-robin to the 8 XCDs), so the tiles of one row-block group are placed 8 apart:
        // they start close in time on one XCD and all but the first find the planes in that XCD's L2.
        const uint32_t span_index = (uint32_t)(((float)blockIdx.x + 0.5f) * pr.inv_span);   // id / (8 * ntiles), ids < 2^21
        const uint32_t rem = blockIdx.x - span_index * 8 * pr.ntiles;
        tile = rem >> 3;
        wg = span_index * 8 + (rem & 7);                            // row-block group of this workgroup
        if (wg >= pr.nwg_rows) return;                              // padding of the last span (whole workgroup)
    }
    if constexpr (MULTI) {
        // which matrix this row block belongs to (row blocks are never shared: RB == 1), picked by comparison
        static_assert(BCQ_MAX_MULTI == 4, "the selection below is written for four matrices");
        const bool g1 = wg >= pr_in.mat_blk0[1], g2 = wg >= pr_in.mat_blk0[2], g3 = wg >= pr_in.mat_blk0[3];
        pr.planes = g3 ? pr_in.mat_planes[3] : g2 ? pr_in.mat_planes[2] : g1 ? pr_in.mat_planes[1] : pr_in.mat_planes[0];
        pr.scales[P] = g3 ? pr_in.mat_scales[3] : g2 ? pr_in.mat_scales[2] : g1 ? pr_in.mat_scales[1] : pr_in.mat_scales[0];
        pr.y = g3 ? pr_in.mat_y[3] : g2 ? pr_in.mat_y[2] : g1 ? pr_in.mat_y[1] : pr_in.mat_y[0];
        pr.m = g3 ? pr_in.mat_m[3] : g2 ? pr_in.mat_m[2] : g1 ? pr_in.mat_m[1] : pr_in.mat_m[0];
        wg -= g3 ? pr_in.mat_blk0[3] : g2 ? pr_in.mat_blk0[2] : g1 ? pr_in.mat_blk0[1] : 0u;
        pr.plane_stride = pr.m * pr.row_stride;
        pr.scale_plane_stride = pr.m * pr.scale_row_stride;
    }
    const int b0 = tile * kMaxBatchTile;
    const int nb = NB > 1 ? min(NB, pr.batch - b0) : 1;
    const uint32_t block_row0 = (wg * RB + rb) * 16;
    const uint32_t last_row = pr.m - 1;

    // rows and row strides are below 2^24 (checked on the host): full-rate 24-bit multiplies
    LaneOffsets off;
    // plane loads: lane (l >> 3, l & 7) takes group l & 7 (16 bytes) of block rows l >> 3 and 8 + (l >> 3);
    // the group part is added per slice.  Rows past the end repeat the last row.
    const uint32_t r8 = lane >> 3;
    off.wa = __umul24(min(block_row0 + r8, last_row), pr.row_stride);
    off.wb = __umul24(min(block_row0 + 8 + r8, last_row), pr.row_stride);
    off.lane = lane;
    // output side: lane (q, r16) reports row r16 of the block for request slot q
    const int q = lane >> 4;
    uint32_t row = block_row0 + (lane & 15);
    const bool row_ok = row <= last_row;
    row = min(row, last_row);
    off.s = __umul24(row, pr.scale_row_stride);
    // activations: the wave converts request slots rb, rb + RB, ... of the tile, 32 bytes per lane and
    // slot; absent slots repeat the tile's first request (their results are never stored)
#pragma unroll
    for (int bb = 0; bb < NB; ++bb) {
        const int b = rb + bb * RB;
        off.x[bb] = (uint32_t)(b0 + (b < nb ? b : 0)) * pr.x_stride;
    }

    float acc = 0.f;
    if constexpr (!MIXED) {
        acc = sweep<P, NB, false, OFFSET, GS>(pr, lds, ks, rb, RB, wave, lane, off, P, pr.scales[P], pr.offsets[P], true);
    } else {
        // precision of the request this lane reports on, and the deepest plane any request of the tile needs.
        // The four precisions of the tile are fetched together, and scale sets are picked by comparison
        // rather than by indexing memory, to keep the chain of dependent loads ahead of the sweep short.
        int p_mine = 0, p_hi = 0;
        int pq[kMaxBatchTile];
#pragma unroll
        for (int b = 0; b < kMaxBatchTile; ++b) pq[b] = pr.p_req[b0 + min(b, nb - 1)];
        const unsigned char *const set1 = pr.scales[1], *const set2 = pr.scales[2], *const set3 = pr.scales[3], *const set4 = pr.scales[4];
        const uint32_t have = pr.set_mask;     // bit k: a scale set of precision k was passed
        auto pick = [&](int k) { return k == 1 ? set1 : k == 2 ? set2 : k == 3 ? set3 : set4; };
#pragma unroll
        for (int b = 0; b < kMaxBatchTile; ++b) {
            int pb = pq[b] < 1 ? 1 : (pq[b] > pr.p_max ? pr.p_max : pq[b]);
            if (!((have >> pb) & 1) || b >= nb) pb = 0;             // no such scale set: zeros; absent slot: nothing
            p_hi = max(p_hi, pb);
            if (b == q) p_mine = pb;
        }
        const unsigned char *sbase = pick(p_mine > 0 ? p_mine : p_hi);
        // offsets of the lane's request, if its precision has any (else any readable array: the scales)
        const bool z_on = OFFSET && ((pr.offset_mask >> p_mine) & 1);
        const unsigned char *zbase = sbase;
        if constexpr (OFFSET) {
            const unsigned char *const z1 = pr.offsets[1], *const z2 = pr.offsets[2], *const z3 = pr.offsets[3], *const z4 = pr.offsets[4];
            if (z_on) zbase = p_mine == 1 ? z1 : p_mine == 2 ? z2 : p_mine == 3 ? z3 : z4;
        }
        // one straight-line sweep per possible depth: only planes 0 .. p_hi-1 are fetched
        switch (p_hi) {
        case 1: acc = sweep<1, NB, true, OFFSET, GS>(pr, lds, ks, rb, RB, wave, lane, off, p_mine, sbase, zbase, z_on); break;
        case 2: acc = sweep<2, NB, true, OFFSET, GS>(pr, lds, ks, rb, RB, wave, lane, off, p_mine, sbase, zbase, z_on); break;
        case 3: acc = sweep<3, NB, true, OFFSET, GS>(pr, lds, ks, rb, RB, wave, lane, off, p_mine, sbase, zbase, z_on); break;
        case 4: acc = sweep<4, NB, true, OFFSET, GS>(pr, lds, ks, rb, RB, wave, lane, off, p_mine, sbase, zbase, z_on); break;
        default: break;                                             // no request has a scale set: zeros
        }
    }

    // ---- combine the KS partial sums of each row block in a fixed order, store binary16 -----
    float *red = reinterpret_cast<float *>(lds + Lds<NB>::red_off(KS, RB));
    red[wave * 64 + lane] = acc;
    __syncthreads();
    if (ks == 0) {
        float v = 0.f;
        for (int k = 0; k < KS; ++k) v += red[(rb * KS + k) * 64 + lane];
        if (row_ok && q < nb) pr.y[(size_t)(b0 + q) * pr.m + row] = (_Float16)v;
    }
}

// ---------------------------------------------------------------------------------------------------------------
// Row-streaming form for tall matrices and two to eight requests (and for one request at one or two planes).  A workgroup owns four blocks of 16 rows and
// builds ONE operand image of the whole activation vectors; after that its waves run free: a wave takes a row block
// and all of its columns (KH = 1) or half of them (KH = 2, the halves meet in LDS at the end) in chunks of 1024,
// with the loads of the chunk after next already under way while it works, so that what arrives is consumed while
// the rest still streams in.  With five to eight requests a plane word is expanded once and feeds two matrix
// instructions (requests 0-3 and 4-7).  The chunks are unrolled (NS, their number per row, is a template argument):
// inside a loop the compiler waits for every outstanding load at the top of each iteration, which takes the lead away.
constexpr int kStreamWaves = 4;

// NS: scale sets a lane needs: one, or with per-request precision one per request tile (a lane reports one request of each)
template <int PH, int NSC>
struct ChunkLoads {
    u32x4 sc[NSC][PH];                      // the 8 scales of the lane's row, per plane
    u32x4 wa[PH], wb[PH];                   // plane words: rows 0-7 and rows 8-15 of the block
};

template <int PH, int NSC>
__device__ __forceinline__ void issue_chunk(ChunkLoads<PH, NSC> &ld, const PlaneMfmaParams &pr, uint32_t o_wa, uint32_t o_wb, uint32_t o_s,
                                            const unsigned char *const *sbase, const int *p_own, int slice)
{
#pragma unroll
    for (int t = 0; t < NSC; ++t)
#pragma unroll
        for (int i = 0; i < PH; ++i) {
            // (per-request precision: a lane stays inside its own request's set, which has p_own planes)
            const int ii = min(i, max(p_own[t], 1) - 1);
            ld.sc[t][i] = *reinterpret_cast<const u32x4 *>(sbase[t] + (size_t)ii * pr.scale_plane_stride + (uint32_t)slice * (kSliceGroups * 2) + o_s);
        }
#pragma unroll
    for (int i = 0; i < PH; ++i) {
        const unsigned char *w_base = pr.planes + (size_t)i * pr.plane_stride + (uint32_t)slice * (kSliceCols / 8);
        ld.wa[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(w_base + o_wa));
        ld.wb[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(w_base + o_wb));
    }
}

// The activations a wave converts into the operand image: the image is converted in NS * RG jobs (a slice of 1024
// columns x NB / RG requests), job j by wave j mod NW.  They are the first loads of a wave and depend on nothing but
// the shape, so they go out before anything else is known (with per-request precision: before the precisions are).
template <int NB, int NS, int KH>
struct StreamActivations {
    static constexpr int NW = kStreamWaves * KH;
    static constexpr int RG = NB >= KH ? KH : 1;
    static constexpr int NBC = NB / RG;
    static constexpr int XS = (NS * RG + NW - 1) / NW;               // jobs per wave
    u32x4 v[XS][NBC][2];
    __device__ __forceinline__ void load(const PlaneMfmaParams &pr)
    {
        const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
        const int nb = min(NB, pr.batch);
#pragma unroll
        for (int k = 0; k < XS; ++k) {
            const int j = wave + k * NW;
            const int slice = min(j / RG, NS - 1), b0 = (j % RG) * NBC;
            const unsigned char *x_base = pr.x + (uint32_t)slice * (kSliceCols * 2) + lane * 32;
#pragma unroll
            for (int b = 0; b < NBC; ++b) {
                const uint32_t xo = (uint32_t)(b0 + b < nb ? b0 + b : 0) * pr.x_stride;
                v[k][b][0] = *reinterpret_cast<const u32x4 *>(x_base + xo);
                v[k][b][1] = *reinterpret_cast<const u32x4 *>(x_base + xo + 16);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
};

// PH: planes fetched (the precision, or with per-request precision the deepest one present); p_own[t]: the precision of
// the request this lane reports on in tile t (PH when uniform, 0: none), sbase[t] its scale set
template <int PH, int NB, int NS, int KH, bool MIXED>
__device__ __forceinline__ void rowstream_body(const PlaneMfmaParams &pr, uint32_t wg, unsigned char *lds, const StreamActivations<NB, NS, KH> &xs,
                                               const int *p_own, const unsigned char *const *sbase)
{
    using L = Lds<NB>;
    constexpr int W = kStreamWaves;                                  // row blocks per workgroup
    constexpr int NW = W * KH;                                       // waves per workgroup: KH parts of the K range per row block
    constexpr int NC = NS / KH;                                      // chunks per wave
    static_assert(NS % KH == 0, "whole chunks per wave");
    constexpr int NT = NB > kMaxBatchTile ? 2 : 1;                   // matrix instructions per (group, plane)
    using XA = StreamActivations<NB, NS, KH>;
    constexpr int RG = XA::RG, NBC = XA::NBC, XS = XA::XS;
    constexpr int NSC = MIXED ? NT : 1;                              // scale sets per lane
    const int tid = threadIdx.x;
    int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nb = min(NB, pr.batch);
    const int rb = wave & (W - 1), kh = wave >> 2;                   // row block of the workgroup, part of the K range
    static_assert(W == 4, "wave -> (row block, K part)");
    const int c0 = kh * NC;                                          // first chunk of this wave
    const uint32_t block_row0 = (wg * (uint32_t)W + rb) * 16;        // wg: this workgroup's index inside its matrix
    const uint32_t last_row = pr.m - 1;

    // plane loads: lane (l >> 3, l & 7) takes group l & 7 (16 bytes) of block rows l >> 3 and 8 + (l >> 3); rows past
    // the end repeat the last row.  Output side: lane (q, r16) reports row r16 for request slots q and 4 + q.
    const uint32_t r8 = lane >> 3;
    const uint32_t o_wa = __umul24(min(block_row0 + r8, last_row), pr.row_stride) + (lane & 7) * 16;
    const uint32_t o_wb = __umul24(min(block_row0 + 8 + r8, last_row), pr.row_stride) + (lane & 7) * 16;
    const int q = lane >> 4, r16 = lane & 15;
    uint32_t row = block_row0 + r16;
    const bool row_ok = row <= last_row;
    row = min(row, last_row);
    const uint32_t o_s = __umul24(row, pr.scale_row_stride);

    // ---- loads in the order of use (they return in the order in which they were asked for): the activations of this
    // wave's conversion jobs are under way (xs), now its first chunk of planes and scales
    // How far the loads run ahead of the sweep: ONE chunk, asked for when the chunk before it has arrived and left
    // its registers.  With a lead of two every wave's first two chunks queue up wave after wave, and a compute unit
    // returns loads in the order asked: the last wave sees its first byte when the others are nearly done (14336 x
    // 4096, p = 4: four requests 11.7 -> 9.6 us, eight requests 14.5 -> 12.2 us; 28672 x 8192, four requests: 38.8 -> 33.0).
    constexpr int D = 1;
    ChunkLoads<PH, NSC> la, lb;
    issue_chunk<PH, NSC>(la, pr, o_wa, o_wb, o_s, sbase, p_own, c0);
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (NC > 1 && D == 2) issue_chunk<PH, NSC>(lb, pr, o_wa, o_wb, o_s, sbase, p_own, c0 + 1);
    __builtin_amdgcn_sched_barrier(0);

    // ---- operand image of the whole K range (the layout of Lds<NB>, slice after slice)
    const int u16 = lane & 7;
#pragma unroll
    for (int k = 0; k < XS; ++k) {
        const int j = wave + k * NW;
        if (j < NS * RG) {
            const int slice = j / RG, b0 = (j % RG) * NBC;
            unsigned char *img_group = lds + slice * L::kSliceImage + (lane >> 3) * L::kGroupBytes;
            unsigned char *img_unit = img_group + (u16 >> 2) * L::kHalfBytes + (2 * ((u16 >> 1) & 1) * L::kRows) * 16 + 4 * (u16 & 1);
#pragma unroll
            for (int b = 0; b < NBC; ++b) {
                const u32x4 v0 = xs.v[k][b][0], v1 = xs.v[k][b][1];
                const uint32_t dwd[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
#pragma unroll
                for (int low = 0; low < 4; ++low) {
                    const uint32_t sel = (low & 1) ? 0x07060302u : 0x05040100u;
                    const int k0 = low >> 1;
                    h2 r01 = __builtin_bit_cast(h2, __builtin_amdgcn_perm(dwd[k0 + 2], dwd[k0], sel));
                    h2 r23 = __builtin_bit_cast(h2, __builtin_amdgcn_perm(dwd[k0 + 6], dwd[k0 + 4], sel));
                    const int inv = 3 - low, w = inv >> 1, z = inv & 1;
                    uint32_t *d32 = reinterpret_cast<uint32_t *>(img_unit + w * (L::kRows * 16) + 8 * z + (b0 + b) * 64);
                    // the exact four-term split of `sweep`
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const uint32_t t01 = __builtin_bit_cast(uint32_t, r01) & 0xFF00FF00u;
                        const uint32_t t23 = __builtin_bit_cast(uint32_t, r23) & 0xFF00FF00u;
                        if (j < 3) {
                            const _Float16 c = j == 0 ? (_Float16)4.0f : (_Float16)8.0f;
                            r01 = (r01 - __builtin_bit_cast(h2, t01)) * h2{c, c};
                            r23 = (r23 - __builtin_bit_cast(h2, t23)) * h2{c, c};
                        }
                        d32[4 * j] = __builtin_amdgcn_perm(t23, t01, 0x07050301u);
                    }
                }
            }
        }
    }
    // the image is complete once every wave's LDS writes are done and the workgroup has met; the global loads under
    // way stay out of it (the barrier of __syncthreads would wait for them)
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    asm volatile("" : "+v"(lane));

    uint32_t sign = 0x88888888u, one = 0x22222222u;
    asm volatile("" : "+v"(one));
    asm volatile("" : "+s"(sign));
    constexpr int kTileRows = NT > 1 ? 16 : L::kRows;               // operand rows of one matrix instruction
    const int arow = r16 < kTileRows ? r16 : kTileRows - 1;
    const unsigned char *img_lane0 = lds + (q * L::kRows + arow) * 16;
    unsigned char *tile = lds + NS * L::kSliceImage + wave * L::kWaveTile;   // NW tiles, then the partial sums
    unsigned char *tile_wr = tile + (lane >> 3) * L::kTileRow + (lane & 7) * 16;
    const unsigned char *tile_rd = tile + r16 * L::kTileRow + q * 4;

    float acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = 0.f;
    auto process = [&](ChunkLoads<PH, NSC> &ld, auto c_tag) {
        constexpr int c = decltype(c_tag)::value;
        u32x4 sc[NSC][PH];
#pragma unroll
        for (int t = 0; t < NSC; ++t)
#pragma unroll
            for (int i = 0; i < PH; ++i) {
                sc[t][i] = ld.sc[t][i];
                // scales of planes the lane's request does not use (beyond its precision; an absent request) become zero
                if (MIXED && !(i < p_own[t])) sc[t][i] = u32x4{0, 0, 0, 0};
            }
        // plane words into operand order through the wave's tile (see `sweep`)
        uint32_t wt[PH][kSliceGroups];
#pragma unroll
        for (int i = 0; i < PH; ++i) {
            *reinterpret_cast<u32x4 *>(tile_wr) = ld.wa[i];
            *reinterpret_cast<u32x4 *>(tile_wr + 8 * L::kTileRow) = ld.wb[i];
#pragma unroll
            for (int g = 0; g < kSliceGroups; ++g)
                wt[i][g] = *reinterpret_cast<const uint32_t *>(tile_rd + g * 16);
        }
#pragma unroll
        for (int i = 0; i < PH; ++i)
#pragma unroll
            for (int g = 0; g < kSliceGroups; ++g) asm volatile("" : "+v"(wt[i][g]));
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (c + D < NC) {
            // a buffer is free (this one for a lead of two chunks, the other one for a lead of one): the next loads.
            // Their addresses depend on a value that exists only from here on, so the loads cannot be moved up.
            uint32_t l_wa = o_wa, l_wb = o_wb, l_s = o_s;
            asm volatile("" : "+v"(l_wa), "+v"(l_wb), "+v"(l_s));
            issue_chunk<PH, NSC>(D == 2 ? ld : ((c & 1) ? la : lb), pr, l_wa, l_wb, l_s, sbase, p_own, c0 + c + D);
        }
        __builtin_amdgcn_sched_barrier(0);

        const unsigned char *img_lane = img_lane0 + (c0 + c) * L::kSliceImage;
        u32x4 lo[NT], hi[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            lo[t] = *reinterpret_cast<const u32x4 *>(img_lane + t * 256);
            hi[t] = *reinterpret_cast<const u32x4 *>(img_lane + t * 256 + L::kHalfBytes);
        }
#pragma unroll
        for (int gl = 0; gl < kSliceGroups; ++gl) {
            v8i xa[NT];
#pragma unroll
            for (int t = 0; t < NT; ++t)
                xa[t] = v8i{(int)lo[t].x, (int)lo[t].y, (int)lo[t].z, (int)lo[t].w, (int)hi[t].x, (int)hi[t].y, (int)hi[t].z, (int)hi[t].w};
            if (gl + 1 < kSliceGroups) {
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    lo[t] = *reinterpret_cast<const u32x4 *>(img_lane + (gl + 1) * L::kGroupBytes + t * 256);
                    hi[t] = *reinterpret_cast<const u32x4 *>(img_lane + (gl + 1) * L::kGroupBytes + t * 256 + L::kHalfBytes);
                }
            }
            v4f d[PH][NT];
#pragma unroll
            for (int i = 0; i < PH; ++i) {
                const v8i wb = expand_plane_word(wt[i][gl], sign, one);
                const v4f zero = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int t = 0; t < NT; ++t)
                    d[i][t] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(xa[t], wb, zero, 1, 4, 0, 0, 0, 0);
            }
#pragma unroll
            for (int i = 0; i < PH; ++i)
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    const uint32_t sw = sc[MIXED ? t : 0][i][gl >> 1];
                    const float alpha = (float)__builtin_bit_cast(_Float16, (unsigned short)((gl & 1) ? (sw >> 16) : (sw & 0xffffu)));
                    acc[t] = fmaf(-alpha, term_sum(d[i][t]), acc[t]);
                }
            // the sums are due here: nothing keeps matrix results for later
#pragma unroll
            for (int t = 0; t < NT; ++t) asm volatile("" : "+v"(acc[t]));
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    auto run = [&](auto self, auto c_tag) {
        constexpr int c = decltype(c_tag)::value;
        if constexpr (c < NC) {
            process((c & 1) ? lb : la, c_tag);
            self(self, std::integral_constant<int, c + 1>{});
        }
    };
    run(run, std::integral_constant<int, 0>{});
    if constexpr (KH > 1) {
        // the parts of a row block meet in LDS, added in a fixed order
        float *red = reinterpret_cast<float *>(lds + NS * L::kSliceImage + NW * L::kWaveTile);
#pragma unroll
        for (int t = 0; t < NT; ++t) red[(wave * NT + t) * 64 + lane] = acc[t];
        __syncthreads();
        if (kh != 0) return;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            float v = 0.f;
#pragma unroll
            for (int k = 0; k < KH; ++k) v += red[((k * W + rb) * NT + t) * 64 + lane];
            acc[t] = v;
        }
    }
#pragma unroll
    for (int t = 0; t < NT; ++t)
        if (row_ok && 4 * t + q < nb) pr.y[(size_t)(4 * t + q) * pr.m + row] = (_Float16)acc[t];
}

// P: the uniform precision, or with per-request precision (MIXED) the number of planes stored
template <int P, int NB, int NS, int KH, bool MIXED = false>
__global__ __launch_bounds__(512) void plane_rowstream_kernel(PlaneMfmaParams pr_in)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    StreamActivations<NB, NS, KH> xs;
    xs.load(pr_in);
    // Several matrices with the same n, precision and activations in one launch: the grid is the concatenation of
    // their workgroups, matrix k owning the ids mat_blk0[k] .. mat_blk0[k + 1] - 1 (a single matrix: all of them); which
    // one this workgroup belongs to is picked by comparison, without a branch.
    PlaneMfmaParams pr = pr_in;
    uint32_t wg = blockIdx.x;
    if constexpr (!MIXED) {
        static_assert(BCQ_MAX_MULTI == 4, "the selection below is written for four matrices");
        const bool g1 = wg >= pr_in.mat_blk0[1], g2 = wg >= pr_in.mat_blk0[2], g3 = wg >= pr_in.mat_blk0[3];
        pr.planes = g3 ? pr_in.mat_planes[3] : g2 ? pr_in.mat_planes[2] : g1 ? pr_in.mat_planes[1] : pr_in.mat_planes[0];
        pr.scales[P] = g3 ? pr_in.mat_scales[3] : g2 ? pr_in.mat_scales[2] : g1 ? pr_in.mat_scales[1] : pr_in.mat_scales[0];
        pr.y = g3 ? pr_in.mat_y[3] : g2 ? pr_in.mat_y[2] : g1 ? pr_in.mat_y[1] : pr_in.mat_y[0];
        pr.m = g3 ? pr_in.mat_m[3] : g2 ? pr_in.mat_m[2] : g1 ? pr_in.mat_m[1] : pr_in.mat_m[0];
        wg -= g3 ? pr_in.mat_blk0[3] : g2 ? pr_in.mat_blk0[2] : g1 ? pr_in.mat_blk0[1] : 0u;
        pr.plane_stride = pr.m * pr.row_stride;
        pr.scale_plane_stride = pr.m * pr.scale_row_stride;
    }
    if constexpr (!MIXED) {
        const int p_own[1] = {P};
        const unsigned char *const sbase[1] = {pr.scales[P]};
        rowstream_body<P, NB, NS, KH, false>(pr, wg, lds, xs, p_own, sbase);
    } else {
        // Section 3.3: requests at different precisions share the plane sweep.  A lane reports one request per tile of
        // four, so it simply reads the scale set of that request's precision (zero from plane p_b on); the planes are
        // fetched to the deepest precision present, which every wave of the launch finds the same.
        constexpr int NT = NB > kMaxBatchTile ? 2 : 1;
        const int nb = min(NB, pr.batch);
        const int q = (threadIdx.x & 63) >> 4;
        const unsigned char *const set1 = pr.scales[1], *const set2 = pr.scales[2], *const set3 = pr.scales[3], *const set4 = pr.scales[4];
        auto pick = [&](int k) { return k == 1 ? set1 : k == 2 ? set2 : k == 3 ? set3 : set4; };
        int p_hi = 0, p_own[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) p_own[t] = 0;
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const int raw = pr.p_req[min(b, nb - 1)];                  // the same address in every lane: a scalar load
            int pb = raw < 1 ? 1 : (raw > pr.p_max ? pr.p_max : raw);
            if (!((pr.set_mask >> pb) & 1) || b >= nb) pb = 0;          // no such scale set: zeros; absent slot: nothing
            p_hi = max(p_hi, pb);
            if ((b & 3) == q) p_own[b >> 2] = pb;
        }
        const unsigned char *sbase[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) sbase[t] = pick(p_own[t] > 0 ? p_own[t] : p_hi);
        switch (p_hi) {           // the same in every wave of the launch
        case 1: if constexpr (P >= 1) rowstream_body<1, NB, NS, KH, true>(pr, wg, lds, xs, p_own, sbase); break;
        case 2: if constexpr (P >= 2) rowstream_body<2, NB, NS, KH, true>(pr, wg, lds, xs, p_own, sbase); break;
        case 3: if constexpr (P >= 3) rowstream_body<3, NB, NS, KH, true>(pr, wg, lds, xs, p_own, sbase); break;
        case 4: if constexpr (P >= 4) rowstream_body<4, NB, NS, KH, true>(pr, wg, lds, xs, p_own, sbase); break;
        default: {                // no request has a scale set: zeros
            const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
            const uint32_t row = (blockIdx.x * (uint32_t)kStreamWaves + (wave & 3)) * 16 + (lane & 15);
            if (wave < kStreamWaves && row < pr.m) {
#pragma unroll
                for (int t = 0; t < NT; ++t)
                    if (4 * t + q < nb) pr.y[(size_t)(4 * t + q) * pr.m + row] = (_Float16)0.f;
            }
            break;
        }
        }
    }
}

// LDS a workgroup may ask for (160 KiB on gfx950), asked of the runtime once
size_t lds_budget()
{
    static const size_t budget = [] {
        int dev = 0, bytes = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&bytes, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess || bytes <= 0)
            return (size_t)64 * 1024;
        return (size_t)bytes;
    }();
    return budget;
}

int lds_total(int NB, int KS, int RB)
{
    return NB == 1 ? Lds<1>::total(KS, RB) : NB == 2 ? Lds<2>::total(KS, RB) : Lds<4>::total(KS, RB);
}

struct Plan {
    int NB, KS, RB, nchunk;
    size_t lds_bytes;
};

Plan make_plan(const GemmArgs &a, bool share_row_blocks = true)
{
    const int nslices = (int)((a.n + kSliceCols - 1) / kSliceCols);
    Plan pl;
    pl.NB = a.batch == 1 ? 1 : a.batch == 2 ? 2 : 4;
    const int wave_cap = max_waves(pl.NB, a.uniform_p == 0, a.group == 64 ? -1 : 0);
    int ks_cap = wave_cap;
    while (ks_cap > 1 && (size_t)lds_total(pl.NB, ks_cap, 1) > lds_budget()) --ks_cap;
    int KS = 1;
    for (int d = 1; d <= ks_cap && d <= nslices; ++d)
        if (nslices % d == 0) KS = d;
    if (KS < ks_cap / 2 && nslices > ks_cap) KS = ks_cap;   // awkward factorisation: ragged last chunk instead
    pl.KS = KS;
    pl.nchunk = (nslices + KS - 1) / KS;
    // With one request a workgroup is one row block: every wave builds its own slice of the operand image and no
    // wave waits for another before the final combine.  With more, 2 or 4 row blocks share a workgroup and its
    // image (each wave converts one request slot): that halves or quarters the conversion work of a tile, at the
    // price of workgroup barriers.
    pl.RB = 1;
    const int64_t row_blocks = (a.m + 15) / 16;
    // From two requests on the conversion outweighs the barriers wherever the matrix still gives about one workgroup
    // per compute unit afterwards (14336 x 4096 at p = 2 / 4: 9.9 -> 7.9 / 12.9 -> 12.1 us with four requests); short
    // matrices with several batch tiles share down to 128 workgroups per tile.
    const int64_t min_groups = a.batch > kMaxBatchTile && row_blocks < 512 ? 128 : 224;
    if (share_row_blocks && a.batch >= 2)
        while (pl.RB * 2 <= pl.NB && pl.RB * 2 * KS <= wave_cap && row_blocks / (pl.RB * 2) >= min_groups &&
               (size_t)lds_total(pl.NB, KS, pl.RB * 2) <= lds_budget())
            pl.RB *= 2;
    pl.lds_bytes = (size_t)lds_total(pl.NB, KS, pl.RB);
    return pl;
}

template <typename K>
hipError_t launch_one(K kernel, const PlaneMfmaParams &pr, const Plan &pl, dim3 grid, dim3 block, hipStream_t stream)
{
    if (hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(kernel), (int)pl.lds_bytes)) return e;
    hipLaunchKernelGGL(kernel, grid, block, pl.lds_bytes, stream, pr);
    return hipGetLastError();
}

template <int NB, bool OFFSET, int GS>
hipError_t launch_group(const GemmArgs &a, const PlaneMfmaParams &pr, const Plan &pl, dim3 grid, dim3 block, hipStream_t stream)
{
    if (a.uniform_p == 0) return launch_one(plane_mfma_kernel<kMaxP, NB, true, OFFSET, false, GS>, pr, pl, grid, block, stream);
    switch (a.uniform_p) {
    case 1: return launch_one(plane_mfma_kernel<1, NB, false, OFFSET, false, GS>, pr, pl, grid, block, stream);
    case 2: return launch_one(plane_mfma_kernel<2, NB, false, OFFSET, false, GS>, pr, pl, grid, block, stream);
    case 3: return launch_one(plane_mfma_kernel<3, NB, false, OFFSET, false, GS>, pr, pl, grid, block, stream);
    default: return launch_one(plane_mfma_kernel<4, NB, false, OFFSET, false, GS>, pr, pl, grid, block, stream);
    }
}

template <int NB, bool OFFSET>
hipError_t launch_nb(const GemmArgs &a, const PlaneMfmaParams &pr, const Plan &pl, dim3 grid, dim3 block, hipStream_t stream)
{
    if (a.group == 64) return launch_group<NB, OFFSET, -1>(a, pr, pl, grid, block, stream);
    return a.group == 256 ? launch_group<NB, OFFSET, 1>(a, pr, pl, grid, block, stream)
                          : launch_group<NB, OFFSET, 0>(a, pr, pl, grid, block, stream);
}

template <int NB>
hipError_t launch_multi_nb(int p, const PlaneMfmaParams &pr, const Plan &pl, dim3 grid, dim3 block, hipStream_t stream)
{
    switch (p) {
    case 1: return launch_one(plane_mfma_kernel<1, NB, false, false, true>, pr, pl, grid, block, stream);
    case 2: return launch_one(plane_mfma_kernel<2, NB, false, false, true>, pr, pl, grid, block, stream);
    case 3: return launch_one(plane_mfma_kernel<3, NB, false, false, true>, pr, pl, grid, block, stream);
    default: return launch_one(plane_mfma_kernel<4, NB, false, false, true>, pr, pl, grid, block, stream);
    }
}

// Row streaming: which problems take it, and its launch.  Measured against the kernel above on 14336 x 4096,
// 17920 x 5120 and 28672 x 8192 at p = 1 .. 4 and two to eight requests: never slower, up to 45 % faster (14336 x 4096,
// p = 4: two requests 10.9 -> 9.5 us, four 12.1 -> 9.7, eight 19.4 -> 12.2; 28672 x 8192, four requests, p = 2: 33 -> 21).
// With one request it wins at one or two planes only (see make_stream_plan): one or two waves per SIMD then do all of
// a row block's arithmetic in turn, and from three planes on the waits for the next chunk outweigh the shared conversion.
struct StreamPlan {
    bool ok;
    int NB, NS, KH;
    size_t lds_bytes;
};

StreamPlan make_stream_plan(const GemmArgs &a)
{
    StreamPlan sp{};
    bool any_offsets = false;
    for (int q = 1; q <= kMaxP; ++q) any_offsets = any_offsets || a.offsets[q] != nullptr;
    const int64_t row_blocks = (a.m + 15) / 16;
    // tall enough to give most compute units a workgroup of four row blocks (measured: from 10240 rows on with up to
    // four requests, 10240 x 4096 at p = 4 13.1 -> 9.6 us, while 8192 rows lose, 8.0 -> 9.5; from 8192 rows on with
    // five to eight, 8192 x 4096 13.5 -> 11.6 us); whole chunks; 4 to 8 of them
    const bool mixed = a.uniform_p == 0;
    if ((mixed ? a.p_req == nullptr || a.p_max < 1 || a.p_max > kMaxP : a.uniform_p < 1 || a.uniform_p > kMaxP) || any_offsets ||
        a.group != 128 || a.batch < 1 || a.batch > 2 * kMaxBatchTile ||
        row_blocks < (a.batch > kMaxBatchTile ? 512 : 640) || a.n % kSliceCols != 0)
        return sp;
    // One request: only at one or two planes, where the conversion of the activations, which this form does once per
    // four row blocks, is a large part of a wave's work, and only where its one or two waves per row block spread
    // evenly over the SIMDs: from 896 row blocks on with rows of four or eight chunks (28672 x 8192: p = 1 12.0 -> 8.6 us,
    // p = 2 16.2 -> 14.9; 14336 x 4096: 4.7 -> 4.1 and 6.2 -> 6.0; gate and up projection in one launch at p = 2:
    // 9.5 -> 9.1).  Shorter matrices and other widths win or lose a few per cent at one plane and lose up to 17 % at
    // two (10240 x 8192: 8.1 -> 9.5 us), and from three planes on the kernel that asks for all of a wave's data up
    // front is ahead everywhere (28672 x 8192, p = 4: 25.6 against 27.8 us).
    if (a.batch == 1 && (mixed || a.uniform_p > 2 || row_blocks < 896 || (a.n != 4 * kSliceCols && a.n != 8 * kSliceCols))) return sp;
    sp.NS = (int)(a.n / kSliceCols);
    if (sp.NS < 4 || sp.NS > 8) return sp;
    if (mixed && sp.NS != 4) return sp;        // per-request precision (four sweep depths per kernel): instantiated for 4096 columns
    sp.NB = a.batch == 1 ? 1 : a.batch <= 2 ? 2 : a.batch <= 4 ? 4 : 8;
    sp.KH = sp.NB == 8 ? 2 : 1;                // eight requests: two waves per SIMD hide each other's matrix instructions
    // one request: two waves per row block wherever one wave per row block leaves a SIMD less than two waves
    // (rows of four chunks at either depth, rows of eight at one plane)
    if (sp.NB == 1 && (sp.NS == 4 || a.uniform_p == 1)) sp.KH = 2;
    if (sp.KH == 2 && sp.NS % 2 != 0) return sp;
    const size_t image = (size_t)sp.NS * (sp.NB == 1 ? Lds<1>::kSliceImage : sp.NB == 2 ? Lds<2>::kSliceImage
                                          : sp.NB == 4 ? Lds<4>::kSliceImage : Lds<8>::kSliceImage);
    const int waves = kStreamWaves * sp.KH;
    sp.lds_bytes = image + (size_t)waves * Lds<1>::kWaveTile + (sp.KH > 1 ? (size_t)waves * 2 * 64 * sizeof(float) : 0);
    sp.ok = sp.lds_bytes <= lds_budget() && (sp.NB < 8 || sp.NS == 4);      // (eight requests: instantiated for four chunks)
    return sp;
}

template <int P, int NB, int NS, int KH>
hipError_t launch_stream_one(const PlaneMfmaParams &pr, const StreamPlan &sp, dim3 grid, hipStream_t stream)
{
    auto kernel = plane_rowstream_kernel<P, NB, NS, KH>;
    if (hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(kernel), (int)sp.lds_bytes)) return e;
    hipLaunchKernelGGL(kernel, grid, dim3(64 * kStreamWaves * KH), sp.lds_bytes, stream, pr);
    return hipGetLastError();
}

template <int P, int NB>
hipError_t launch_stream_ns(const PlaneMfmaParams &pr, const StreamPlan &sp, dim3 grid, hipStream_t stream)
{
    switch (sp.NS) {
    case 4: return launch_stream_one<P, NB, 4, 1>(pr, sp, grid, stream);
    case 5: return launch_stream_one<P, NB, 5, 1>(pr, sp, grid, stream);
    case 6: return launch_stream_one<P, NB, 6, 1>(pr, sp, grid, stream);
    case 7: return launch_stream_one<P, NB, 7, 1>(pr, sp, grid, stream);
    default: return launch_stream_one<P, NB, 8, 1>(pr, sp, grid, stream);
    }
}

template <int P, int NB, int KH>
hipError_t launch_stream_mixed_one(const PlaneMfmaParams &pr, const StreamPlan &sp, dim3 grid, hipStream_t stream)
{
    auto kernel = plane_rowstream_kernel<P, NB, 4, KH, true>;
    if (hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(kernel), (int)sp.lds_bytes)) return e;
    hipLaunchKernelGGL(kernel, grid, dim3(64 * kStreamWaves * KH), sp.lds_bytes, stream, pr);
    return hipGetLastError();
}

template <int P>
hipError_t launch_stream_mixed(const PlaneMfmaParams &pr, const StreamPlan &sp, dim3 grid, hipStream_t stream)
{
    if (sp.NB == 2) return launch_stream_mixed_one<P, 2, 1>(pr, sp, grid, stream);
    if (sp.NB == 4) return launch_stream_mixed_one<P, 4, 1>(pr, sp, grid, stream);
    return launch_stream_mixed_one<P, 8, 2>(pr, sp, grid, stream);
}

// one request (one or two planes, rows of four or eight chunks): one or two waves per row block
template <int P>
hipError_t launch_stream_single(const PlaneMfmaParams &pr, const StreamPlan &sp, dim3 grid, hipStream_t stream)
{
    if constexpr (P <= 2) {
        if (sp.NS == 4 && sp.KH == 2) return launch_stream_one<P, 1, 4, 2>(pr, sp, grid, stream);
        if (sp.NS == 8 && sp.KH == 2) return launch_stream_one<P, 1, 8, 2>(pr, sp, grid, stream);
        if (sp.NS == 8 && sp.KH == 1) return launch_stream_one<P, 1, 8, 1>(pr, sp, grid, stream);
    }
    return hipErrorInvalidValue;                  // make_stream_plan plans nothing else
}

template <int P>
hipError_t launch_stream_p(const PlaneMfmaParams &pr, const StreamPlan &sp, dim3 grid, hipStream_t stream)
{
    if (sp.NB == 1) return launch_stream_single<P>(pr, sp, grid, stream);
    if (sp.NB == 2) return launch_stream_ns<P, 2>(pr, sp, grid, stream);
    if (sp.NB == 4) return launch_stream_ns<P, 4>(pr, sp, grid, stream);
    return launch_stream_one<P, 8, 4, 2>(pr, sp, grid, stream);
}

// `mats`: the matrices of the launch (one, or several with the same n, precision, batch and activations)
hipError_t launch_stream(const GemmArgs *mats, int count, PlaneMfmaParams pr, const StreamPlan &sp, hipStream_t stream)
{
    const GemmArgs &a = mats[0];
    uint32_t wgs = 0;
    for (int k = 0; k < BCQ_MAX_MULTI; ++k) {
        pr.mat_blk0[k] = wgs;                 // unused entries: the total, which no workgroup reaches
        if (k >= count) continue;
        pr.mat_planes[k] = reinterpret_cast<const unsigned char *>(mats[k].planes);
        pr.mat_scales[k] = reinterpret_cast<const unsigned char *>(a.uniform_p > 0 ? mats[k].scales[a.uniform_p] : nullptr);
        pr.mat_y[k] = mats[k].y;
        pr.mat_m[k] = (uint32_t)mats[k].m;
        wgs += (uint32_t)(((mats[k].m + 15) / 16 + kStreamWaves - 1) / kStreamWaves);
    }
    dim3 grid(wgs);
    if (a.uniform_p == 0) {
        switch (a.p_max) {
        case 1: return launch_stream_mixed<1>(pr, sp, grid, stream);
        case 2: return launch_stream_mixed<2>(pr, sp, grid, stream);
        case 3: return launch_stream_mixed<3>(pr, sp, grid, stream);
        default: return launch_stream_mixed<4>(pr, sp, grid, stream);
        }
    }
    switch (a.uniform_p) {
    case 1: return launch_stream_p<1>(pr, sp, grid, stream);
    case 2: return launch_stream_p<2>(pr, sp, grid, stream);
    case 3: return launch_stream_p<3>(pr, sp, grid, stream);
    default: return launch_stream_p<4>(pr, sp, grid, stream);
    }
}

}  // namespace

bool plane_mfma_streams(const GemmArgs &a) { return plane_mfma_supports(a) && make_stream_plan(a).ok; }

// Several matrices in one launch: the row-streaming form takes them when it would take one matrix of all their rows
static StreamPlan make_stream_plan_multi(const GemmArgs *mats, int count)
{
    GemmArgs all = mats[0];
    all.m = 0;
    for (int k = 0; k < count; ++k) all.m += mats[k].m;
    return make_stream_plan(all);
}

bool plane_mfma_streams_multi(const GemmArgs *mats, int count)
{
    return plane_mfma_supports_multi(mats, count) && make_stream_plan_multi(mats, count).ok;
}

bool plane_mfma_supports(const GemmArgs &a)
{
    // 32-bit byte offsets inside one plane / one scale plane / the activation matrix
    const bool small_enough = a.m * (a.n / 8) < (int64_t(1) << 31) && (int64_t)a.batch * a.n * 2 < (int64_t(1) << 31) &&
                              a.m < (int64_t(1) << 24) && a.n < (int64_t(1) << 24);
    // whole scale groups, 4-byte aligned scale rows, and at least eight groups of 128 per row (the scales of
    // a short last slice are fetched as the last ones of the row); scale groups of 128 or 256 columns
    // groups of 64 (two matrix instructions per 128 columns, one per half): whole K slices
    const bool group_ok = (a.group == 128 && (a.n % 256) == 0) || (a.group == 256 && (a.n % 512) == 0) ||
                          (a.group == 64 && (a.n % kSliceCols) == 0);
    return group_ok && a.n >= kSliceCols && a.p_max <= kMaxP && small_enough &&
           ((a.m + 15) / 16 + 8) * ((a.batch + kMaxBatchTile - 1) / kMaxBatchTile) < (int64_t(1) << 21);
}

hipError_t plane_mfma_launch(const GemmArgs &a, hipStream_t stream)
{
    const Plan pl = make_plan(a);
    PlaneMfmaParams pr{};
    pr.planes = reinterpret_cast<const unsigned char *>(a.planes);
    pr.x = reinterpret_cast<const unsigned char *>(a.x);
    pr.y = a.y;
    for (int q = 0; q <= BCQ_MAX_PLANES; ++q) pr.scales[q] = reinterpret_cast<const unsigned char *>(a.scales[q]);
    pr.p_req = a.p_req;
    for (int q = 0; q <= BCQ_MAX_PLANES; ++q) pr.offsets[q] = reinterpret_cast<const unsigned char *>(a.offsets[q]);
    for (int q = 1; q <= kMaxP; ++q) {
        if (a.scales[q]) pr.set_mask |= 1u << q;
        if (a.offsets[q] && a.scales[q]) pr.offset_mask |= 1u << q;
    }
    // the asymmetric kernels run only when an offset set will be used
    const bool with_offsets = a.uniform_p > 0 ? a.offsets[a.uniform_p] != nullptr : pr.offset_mask != 0;
    pr.plane_stride = (uint32_t)(a.m * (a.n / 8));
    pr.row_stride = (uint32_t)(a.n / 8);
    pr.scale_plane_stride = (uint32_t)(a.m * (a.n / a.group) * 2);
    pr.scale_row_stride = (uint32_t)((a.n / a.group) * 2);
    pr.x_stride = (uint32_t)(a.n * 2);
    pr.m = (uint32_t)a.m;
    pr.batch = a.batch;
    pr.p_max = a.p_max;
    pr.uniform_p = a.uniform_p;
    pr.KS = pl.KS;
    pr.RB = pl.RB;
    pr.nchunk = pl.nchunk;
    pr.nslices = (int)((a.n + kSliceCols - 1) / kSliceCols);
    pr.glast = (int)((a.n / 128 - 1) % kSliceGroups) + 1;
    const int64_t row_blocks = (a.m + 15) / 16;
    pr.ntiles = (uint32_t)((a.batch + kMaxBatchTile - 1) / kMaxBatchTile);
    pr.nwg_rows = (uint32_t)((row_blocks + pl.RB - 1) / pl.RB);
    // ids are grouped in spans of 8 row-block groups x ntiles; the last span may be partly empty
    dim3 grid(pl.NB == 1 ? pr.nwg_rows : (pr.nwg_rows + 7) / 8 * 8 * pr.ntiles);
    pr.inv_span = 1.0f / (float)(8 * pr.ntiles);
    pr.inv_ks = 1.0f / (float)pl.KS;
    dim3 block(64 * pl.KS * pl.RB);
    if (const StreamPlan sp = make_stream_plan(a); sp.ok) return launch_stream(&a, 1, pr, sp, stream);
    if (with_offsets) {
        switch (pl.NB) {
        case 1: return launch_nb<1, true>(a, pr, pl, grid, block, stream);
        case 2: return launch_nb<2, true>(a, pr, pl, grid, block, stream);
        default: return launch_nb<4, true>(a, pr, pl, grid, block, stream);
        }
    }
    switch (pl.NB) {
    case 1: return launch_nb<1, false>(a, pr, pl, grid, block, stream);
    case 2: return launch_nb<2, false>(a, pr, pl, grid, block, stream);
    default: return launch_nb<4, false>(a, pr, pl, grid, block, stream);
    }
}

// Several matrices (same n, precision, batch and activations, no offsets) as one launch: the grid is
// the concatenation of their row blocks.
bool plane_mfma_supports_multi(const GemmArgs *mats, int count)
{
    if (count < 2 || count > BCQ_MAX_MULTI) return false;
    int64_t row_blocks = 0;
    for (int k = 0; k < count; ++k) {
        const GemmArgs &a = mats[k];
        if (!plane_mfma_supports(a) || a.uniform_p < 1 || a.offsets[a.uniform_p]) return false;
        if (a.n != mats[0].n || a.uniform_p != mats[0].uniform_p || a.batch != mats[0].batch || a.x != mats[0].x ||
            a.group != 128)
            return false;
        row_blocks += (a.m + 15) / 16;
    }
    return (row_blocks + 8) * ((mats[0].batch + kMaxBatchTile - 1) / kMaxBatchTile) < (int64_t(1) << 21);
}

hipError_t plane_mfma_launch_multi(const GemmArgs *mats, int count, hipStream_t stream)
{
    const GemmArgs &a = mats[0];
    const Plan pl = make_plan(a, false);      // a row block belongs to one matrix: no sharing of workgroups
    PlaneMfmaParams pr{};
    pr.x = reinterpret_cast<const unsigned char *>(a.x);
    pr.row_stride = (uint32_t)(a.n / 8);
    pr.scale_row_stride = (uint32_t)((a.n / 128) * 2);
    pr.x_stride = (uint32_t)(a.n * 2);
    pr.batch = a.batch;
    pr.p_max = a.p_max;
    pr.uniform_p = a.uniform_p;
    if (const StreamPlan sp = make_stream_plan_multi(mats, count); sp.ok) return launch_stream(mats, count, pr, sp, stream);
    pr.KS = pl.KS;
    pr.RB = 1;
    pr.nchunk = pl.nchunk;
    pr.nslices = (int)((a.n + kSliceCols - 1) / kSliceCols);
    pr.glast = (int)((a.n / 128 - 1) % kSliceGroups) + 1;
    uint32_t blk = 0;
    for (int k = 0; k < BCQ_MAX_MULTI; ++k) {
        pr.mat_blk0[k] = blk;                 // unused entries: the total, which no row block reaches
        if (k >= count) continue;
        pr.mat_planes[k] = reinterpret_cast<const unsigned char *>(mats[k].planes);
        pr.mat_scales[k] = reinterpret_cast<const unsigned char *>(mats[k].scales[a.uniform_p]);
        pr.mat_y[k] = mats[k].y;
        pr.mat_m[k] = (uint32_t)mats[k].m;
        blk += (uint32_t)((mats[k].m + 15) / 16);
    }
    pr.ntiles = (uint32_t)((a.batch + kMaxBatchTile - 1) / kMaxBatchTile);
    pr.nwg_rows = blk;
    dim3 grid(pl.NB == 1 ? pr.nwg_rows : (pr.nwg_rows + 7) / 8 * 8 * pr.ntiles);
    pr.inv_span = 1.0f / (float)(8 * pr.ntiles);
    pr.inv_ks = 1.0f / (float)pl.KS;
    dim3 block(64 * pl.KS);
    switch (pl.NB) {
    case 1: return launch_multi_nb<1>(a.uniform_p, pr, pl, grid, block, stream);
    case 2: return launch_multi_nb<2>(a.uniform_p, pr, pl, grid, block, stream);
    default: return launch_multi_nb<4>(a.uniform_p, pr, pl, grid, block, stream);
    }
}

}  // namespace bcq
