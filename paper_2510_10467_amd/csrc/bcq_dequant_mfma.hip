// The kernels for more than a handful of requests, all built on one skeleton (activation tiles staged in LDS,
// plane words expanded to +-1.0 binary16 through a 16-entry table, fp16 matrix instructions):
//   dequant_mfma_kernel      uniform precision; rebuilds W_p in registers (below), or with PW = true multiplies the
//                            +-1 planes themselves and scales the group sums ("plane_f16", one tile of 16 requests)
//   planewise_mixed_kernel   per-request precision in tiles of 16 requests: one pass over the planes, each request's
//                            own scales applied to the group sums
//   dequant_mixed_kernel     per-request precision at 64 requests per workgroup: W_q rebuilt once per precision present
//   dequant_byclass_kernel   per-request precision beyond 64 requests: the uniform kernel's body per precision, each
//                            workgroup on the requests of its precision, picked out of the batch by rank
//
// Large-batch kernel: dequantise W_p = sum_i alpha_i B_i tile by tile (Fig. 1(b): p-bit inference
// reconstructs the weights from the first p planes and the scale set of precision p) and feed the
// binary16 tiles to the fp16 matrix pipe.  Once a plane word serves dozens of requests the product
// is no longer bound by HBM but by arithmetic, and one dense fp16 MFMA over dequantised weights
// costs p times fewer matrix instructions than p plane-wise products.
//
// A team of RW waves (RW = 4, 2 or 1) owns 16 RW weight rows (16 per wave) and TB = 16, 64, 128 or 256 requests.
// Per group of 128 columns
//   * the team stages the TB x 128 activation tile of the NEXT group in LDS with loads that write LDS
//     directly (global_load_lds_dwordx4: 64 lanes deliver 1 KiB = four requests' rows, no registers, no
//     LDS store instructions), into the tile the previous group has just left; a request's sixteen
//     16-byte parts sit XOR-permuted by the request number so that operand reads spread over all banks;
//   * lane (row, kq) of a wave holds word kq of its row's group from each plane plus the group's
//     scales (also one group ahead).  Matrix step t covers the columns 32 kq + 8 t + j of the group
//     (a permutation of K that the activation operand follows), so for each step the lane takes
//     byte t of each plane word, looks its two nibbles up in a 16-entry LDS table of four +-1.0
//     binary16 values (each entry sits in banks of its own and equal addresses are broadcast, so
//     these reads never conflict, unlike those of a 256-entry table of eight values), accumulates
//     w_j = sum_i alpha_i * (+-1) in fp32 (one mixed-precision FMA per column and plane), starting from
//     the group's offset in the asymmetric scheme (section 4.1), and rounds once to binary16: that IS
//     the B operand of v_mfma_f32_16x16x32_f16;
//   * the wave multiplies its 16 x 128 weight tile with all TB requests, reading each activation
//     operand (16 requests x 32 columns) from LDS.
// A weight is therefore dequantised once per TB requests and never leaves the registers; the
// activations are read from HBM/L2 once per workgroup.  The MFMA's M side carries requests, its N
// side the 16 weight rows of the wave, so a lane ends up with four requests of its own row per
// accumulator.  One barrier per group.
//
// A wave cannot overlap its own vector, matrix and LDS instructions, and with one wave per SIMD every
// latency is exposed.  So, LDS permitting, a workgroup has several teams (four for TB = 64, two for
// TB = 128): all work on the same rows and requests, team k on the groups k, k + TEAMS, ... with
// activation tiles and accumulators of its own; the teams meet at every barrier and add their
// accumulators through LDS at the end.  The activation tiles fill the LDS, so a CU runs one workgroup at a
// time and a short matrix needs small row blocks (RW < 4) to give every CU one; the host picks the shape
// from measured per-shape costs (cheapest_shape).  A tile of 256 requests leaves LDS for one pair of tiles:
// its second wave per SIMD comes either from eight row blocks (RW = 8) or from two teams that SHARE the
// tiles, work on every group together and split its four matrix sub-steps (SHARE).
#include <hip/hip_runtime.h>

#include <type_traits>

#include "bcq_internal.hpp"

namespace bcq {
namespace {

typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef _Float16 v4h __attribute__((ext_vector_type(4)));
typedef _Float16 h2v __attribute__((ext_vector_type(2)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kMaxP = 4;
constexpr int kClassFrom = 64;              // per-request precision: beyond this many requests the uniform kernel's body per precision
thread_local int g_forced_nt = 0, g_forced_rw = 0;       // workgroup shape forced by dequant_mfma_force_shape (0: automatic)
constexpr int kLutBytes = 256;              // 16 entries x 8 bytes, rounded up to keep what follows aligned
constexpr int kXRowBytes = 128 * 2;         // LDS row of one request's 128 activations; its sixteen parts sit XOR-permuted

// pointer into LDS from its 32-bit address
template <typename T>
__device__ __forceinline__ const T *lds_at(uint32_t addr)
{
    return (const T *)(const __attribute__((address_space(3))) T *)(uintptr_t)addr;
}

constexpr int x_tile_bytes(int nt) { return 16 * nt * kXRowBytes; }       // nt tiles of 16 requests
constexpr int lds_bytes(int nt, int teams) { return kLutBytes + teams * 2 * x_tile_bytes(nt); }

struct DequantParams {
    const unsigned char *planes;            // plane 0
    const unsigned char *scales;            // scale set of the precision
    const unsigned char *offsets;           // offsets [m][n/128] of the precision; any readable array of that size if none
    int has_offsets;
    const unsigned char *x;
    _Float16 *y;
    uint32_t plane_stride;                  // bytes between planes:        m * n / 8
    uint32_t row_stride;                    // bytes between plane rows:    n / 8
    uint32_t scale_plane_stride;            // bytes between scale planes:  m * (n/128) * 2
    uint32_t scale_row_stride;              // bytes between scale rows:    (n/128) * 2
    uint32_t x_stride;                      // bytes between requests:      n * 2
    uint32_t m;
    int batch, ngroups;                     // ngroups: steps of 128 columns
    int gshift;                             // scale groups of 64 (-1), 128 (0) or 256 (+1) columns
    // per-request precision (dequant_mixed_kernel): a scale / offset set per precision, nullptr where there is none
    const unsigned char *scale_sets[kMaxP + 1];
    const unsigned char *offset_sets[kMaxP + 1];
    const int32_t *p_req;
    int p_max;
    uint32_t class_order;                   // dequant_byclass_kernel: byte y = the precision served by the workgroups with blockIdx.y = y
    // several matrices with the same n, precision and activations in one launch (nmat > 1): matrix k owns the workgroup
    // rows mat_blk0[k] .. mat_blk0[k+1]-1 of the grid; unused entries hold the total
    int nmat;
    const unsigned char *mat_planes[BCQ_MAX_MULTI];
    const unsigned char *mat_scales[BCQ_MAX_MULTI];
    _Float16 *mat_y[BCQ_MAX_MULTI];
    uint32_t mat_m[BCQ_MAX_MULTI];
    uint32_t mat_blk0[BCQ_MAX_MULTI];
};

// What a thread fetches one group ahead into registers: the plane words of its row (its share of the next
// activation tile goes straight to LDS, the scales come in blocks of four steps).
template <int P, int XU>
struct Ahead {
    uint32_t w[P];
};

// The requests of precision q (after clamping to [1, p_max]) in the order of the batch: those of rank b0 .. b0 + TB - 1
// get their numbers written to req_of[0 .. TB - 1] by the workgroup's first wave; returns how many of these ranks
// exist (0 or less: none), the same number in every wave, each of which runs the whole ranking itself.  Sixteen
// independent loads at a time (1024 requests), so that a batch costs one memory latency, not one per 64 requests.
template <int TB>
__device__ __forceinline__ int rank_requests(const DequantParams &a, const int q, const int b0, uint32_t *req_of)
{
    const int lane = threadIdx.x & 63;
    int seen = 0;                               // requests of precision q so far
    for (int blk = 0; blk < a.batch && seen < b0 + TB; blk += 1024) {
        int pv[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int b = blk + 64 * j + lane;
            pv[j] = b < a.batch ? a.p_req[b] : 0;
        }
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int b = blk + 64 * j + lane;
            const int pc = pv[j] < 1 ? 1 : (pv[j] > a.p_max ? a.p_max : pv[j]);
            const bool is = b < a.batch && pc == q;
            const unsigned long long mask = __ballot(is);
            const int rank = seen + (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
            if (is && rank >= b0 && rank < b0 + TB && threadIdx.x < 64) req_of[rank - b0] = (uint32_t)b;
            seen += __popcll(mask);
        }
    }
    return seen - b0 > TB ? TB : seen - b0;
}

// NT: 16-request tiles per workgroup (1, 2, 4, 8 or 16); TEAMS: teams of waves (K split inside the workgroup); RW: waves per
// team = 16-row blocks per workgroup.
// PW (plane-wise): instead of rebuilding W_p, the +-1.0 values from the table are themselves the matrix operand:
//   tmp_i = B_i x over the group's 128 columns (fp16 matrix instructions, exact products, fp32 sums), then
//   acc += alpha_i * tmp_i in fp32 - y = sum_i alpha_i (B_i x) as section 3.3 writes it, group by group.
// That trades the P fused multiply-adds per weight for P times the matrix instructions, which the matrix pipe
// has room for; the offset of the asymmetric scheme multiplies the group's plain activation sum, formed by
// one more pass with an all-ones operand.
// (The small-tile shapes leave LDS for several workgroups per CU: at least four waves per SIMD keeps the compiler
// from spending the few registers that would forbid it.)
// BYCLASS (per-request precision at large batch): the workgroup serves requests whose precision is P, namely those
//   of rank b0 .. b0 + 16 NT - 1 among them, in the order of the batch; every wave ranks the batch itself (ballots
//   over p_req, no memory beyond the inputs), the first one leaves the request numbers in LDS.  A workgroup whose
//   ranks nobody holds returns at once: the grid is laid out for the case that every request has precision P.
// SHARE: the teams do not take alternate groups with tiles of their own but share one pair of tiles and split the
//   four matrix sub-steps of every group between them (team k takes sub-steps k 4/TEAMS ...): the 128- and
//   256-request tiles then fit the LDS once instead of TEAMS times, so that a CU holds eight waves on a 256-request
//   tile (two per SIMD, one computing while the other waits for its operands) instead of four.
template <int P, int NT, int TEAMS, int RW, bool PW = false, bool BYCLASS = false, bool SHARE = false>
__device__ __forceinline__ void dequant_mfma_body(const DequantParams &a, const int column, const uint32_t rowblk)
{
    constexpr int kTeamThreads = 64 * RW;
    static_assert(!(SHARE && PW), "the plane-wise variant has no shared-tile form");
    constexpr int GSTEP = SHARE ? 1 : TEAMS;  // distance between a team's groups
    constexpr int TN = SHARE ? 4 / TEAMS : 4; // matrix sub-steps of a group that a team computes
    constexpr int SW = SHARE ? RW * TEAMS : RW;       // waves that stage a tile together
    constexpr int LT = SHARE ? 1 : TEAMS;     // pairs of tiles in LDS
    constexpr int XU = 4 * NT / SW;           // 16-byte units of an activation tile per thread of those waves
    constexpr int UT = NT < 4 ? NT : 4;       // request tiles whose operands are held at a time
    static_assert(XU >= 1 && NT % UT == 0, "tile does not split over the team");
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    unsigned char *lut = lds;

    // team and wave are the same in all lanes of a wave: telling the compiler keeps group indices and
    // base addresses in scalar registers
    const int tid = threadIdx.x % kTeamThreads, team = __builtin_amdgcn_readfirstlane(threadIdx.x / kTeamThreads);
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    unsigned char *xt0 = lds + kLutBytes + (SHARE ? 0 : team) * 2 * x_tile_bytes(NT);     // the team's two activation tiles, used alternately
    const int g_first = SHARE ? 0 : team;     // the team's first group
    const int sw = SHARE ? team * RW + wave : wave;   // this wave among those that stage a tile
    const int t0 = SHARE ? team * TN : 0;     // the team's first matrix sub-step
    constexpr int kTile = x_tile_bytes(NT);
    const int n16 = lane & 15;                // weight row inside the wave's block / request inside a 16-request tile
    const int kq = lane >> 4;                 // K quarter: columns 32kq + 8t .. 32kq + 8t + 7 of the group in step t
    const uint32_t row0 = rowblk * (16 * RW) + wave * 16;
    const int b0 = column * (16 * NT);        // first request of the workgroup (BYCLASS: first rank)

    int nreq = a.batch - b0;                  // requests from b0 on (may be more than the workgroup's 16 NT)
    const uint32_t *req_of = reinterpret_cast<const uint32_t *>(lds + lds_bytes(NT, LT));
    if constexpr (BYCLASS) {
        nreq = rank_requests<16 * NT>(a, P, b0, reinterpret_cast<uint32_t *>(lds + lds_bytes(NT, LT)));
        if (nreq <= 0) return;                // (every wave of the workgroup: none has reached a barrier yet)
        __syncthreads();
    }

    // table: nibble -> four binary16 values, +1.0 where the bit is set, -1.0 where it is clear
    if (threadIdx.x < 16) {
        uint32_t e[2];
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            const uint32_t lo = ((tid >> (2 * c)) & 1) ? 0x3C00u : 0xBC00u;
            const uint32_t hi = ((tid >> (2 * c + 1)) & 1) ? 0x3C00u : 0xBC00u;
            e[c] = lo | (hi << 16);
        }
        *reinterpret_cast<u32x2 *>(lut + tid * 8) = u32x2{e[0], e[1]};
    }

    // lane offsets; rows and requests past the end repeat the last one (their results are not stored)
    // Plane words and scales are fetched with four adjacent lanes on one row (lane l: row l >> 2, word
    // l & 3), which the memory pipe combines into one request per row, and then handed to the lane
    // that uses them (row l & 15, word l >> 4) by a lane permute.
    const uint32_t frow = min(row0 + (lane >> 2), a.m - 1);
    uint32_t w_lane = frow * a.row_stride + (lane & 3) * 4;
    // Scales and offsets are fetched for FOUR of the team's steps at once: the four lanes of a row take the
    // groups of the steps 4M .. 4M + 3 (eight bytes apart, one 64-byte sector), so a load instruction asks
    // for sixteen lines once in four steps instead of every step; these requests, not the bytes, were up to a
    // sixth of the kernel's time.  With groups of 64 columns a step has two scales, fetched as one dword.
    const uint32_t s_row = frow * a.scale_row_stride;
    auto scale_col = [&](int g) { return (uint32_t)(a.gshift > 0 ? (g >> 1) * 2 : a.gshift < 0 ? g * 4 : g * 2); };
    const int pull = (4 * n16 + kq) * 4;      // byte index of the lane to take from
    const int pull_row = 4 * n16 * 4;         // first of the four lanes that hold the scales of row n16
    // groups of 64: columns 64..127 of a step use the upper scale (the plane-wise variant has no groups of 64: no shift at all)
    const uint32_t half_shift = !PW && a.gshift < 0 && kq >= 2 ? 16u : 0u;
    uint32_t sc[P], zc = 0;                   // this lane's share of the scales in flight / in use (binary16 bits)
    auto fetch_scales = [&](int block) {      // for the team's steps 4 block .. 4 block + 3
        const int gj = min(g_first + GSTEP * (4 * block + (lane & 3)), a.ngroups - 1);
        uint32_t off = s_row + scale_col(gj);
        asm volatile("" : "+v"(off));
        if (a.gshift < 0) {
#pragma unroll
            for (int i = 0; i < P; ++i) sc[i] = *reinterpret_cast<const uint32_t *>(a.scales + (size_t)i * a.scale_plane_stride + off);
            if (a.has_offsets) zc = *reinterpret_cast<const uint32_t *>(a.offsets + off);
        } else {
#pragma unroll
            for (int i = 0; i < P; ++i) sc[i] = *reinterpret_cast<const unsigned short *>(a.scales + (size_t)i * a.scale_plane_stride + off);
            if (a.has_offsets) zc = *reinterpret_cast<const unsigned short *>(a.offsets + off);
        }
    };
    // staging: unit tid + kTeamThreads * k of the tile = request (unit >> 4), 16-byte part (unit & 15) of its 256 bytes
    // Staging straight into LDS: load instruction i of a tile (i = k * RW + wave) brings the 1 KiB of requests
    // 4i .. 4i+3; lane l delivers the 16 bytes that land at chunk l of that KiB, which is part
    // (l & 15) ^ (request & 15) of request 4i + (l >> 4): rows are 256 bytes apart and the XOR spreads the
    // operand reads of sixteen requests over all banks.
    uint32_t xs_src[XU];
#pragma unroll
    for (int k = 0; k < XU; ++k) {
        const int req = 4 * (k * SW + sw) + (lane >> 4);
        const int part = (lane & 15) ^ (req & 15);
        const uint32_t source = BYCLASS ? req_of[min(req, nreq - 1)] : (uint32_t)min(b0 + req, a.batch - 1);
        xs_src[k] = source * a.x_stride + part * 16;
    }
    // A operand of request tile u, step t: request 16u + n16, part 4kq + t
    const unsigned char *xa_lane = xt0 + n16 * kXRowBytes;
    uint32_t xa_off[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) xa_off[t] = (uint32_t)(((4 * kq + ((t0 + t) & 3)) ^ n16) * 16);      // (entry t: the team's sub-step t0 + t)

    // Plane words are loaded as ordinary (cached) loads: a wave takes 16 bytes of each row per step and the
    // rest of the 128-byte line serves the other teams and the next step; marked non-temporal the line was
    // fetched from memory again and again (up to 1.4x slower).
    auto fetch_plane = [&](Ahead<P, XU> &ah, int g, int i) {
        // wave-uniform 64-bit base plus 32-bit lane offset: an addressing mode of the load instruction
        const unsigned char *w_base = a.planes + (size_t)i * a.plane_stride + (uint32_t)g * 16;
        ah.w[i] = *reinterpret_cast<const uint32_t *>(w_base + w_lane);
    };
    auto fetch_w = [&](Ahead<P, XU> &ah, int g) {
#pragma unroll
        for (int i = 0; i < P; ++i) fetch_plane(ah, g, i);
    };
    auto stage_x_unit = [&](int g, int buf, int k) {
        const unsigned char *x_base = a.x + (uint32_t)g * 256;
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(x_base + xs_src[k]),
                                         (__attribute__((address_space(3))) void *)(xt0 + buf * kTile + (k * SW + sw) * 1024), 16, 0, 0);
    };
    auto stage_x = [&](int g, int buf) {
#pragma unroll
        for (int k = 0; k < XU; ++k) stage_x_unit(g, buf, k);
    };

    // LDS address of the table as a number the compiler cannot see through (it would otherwise add a literal zero
    // to every look-up address in a separate instruction)
    uint32_t lut_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)lut;
    asm volatile("" : "+s"(lut_base));

    v4f acc[NT];
#pragma unroll
    for (int u = 0; u < NT; ++u) acc[u] = v4f{0.f, 0.f, 0.f, 0.f};

    // Group g, the team's next being g + TEAMS.  On entry `cur` holds the plane words and scales of group g
    // and the activation tile of the next group; the team's LDS tile `buf` holds the activations of group g.
    // Every wave of the workgroup passes the barrier of every step (if there is one), with or without a group of its own.
    // `mine` counts the team's steps (g = team + TEAMS * mine).
    auto step = [&](Ahead<P, XU> &cur, Ahead<P, XU> &nxt, int g, int mine, int buf) {
        if (g < a.ngroups) {
        // Everything fetched ahead is claimed here, while it is all that is outstanding: the wait is
        // then exact.  (Claimed after the next loads have been issued, it would cover those too.)
#pragma unroll
        for (int i = 0; i < P; ++i) asm volatile("" : "+v"(cur.w[i]), "+v"(sc[i]));
        asm volatile("" : "+v"(zc));
        // The lane offsets are made new values in every step: hoisted out of the loop as 64-bit numbers they
        // cost a register pair and a 64-bit add per load; widened where they are used they ride in the load's
        // own addressing mode (scalar base + 32-bit lane offset).
        asm volatile("" : "+v"(w_lane));
#pragma unroll
        for (int k = 0; k < XU; ++k) asm volatile("" : "+v"(xs_src[k]));
        const int pull_scale = pull_row + (mine & 3) * 4;       // the lane that fetched this step's scales of row n16
        uint32_t zb = (uint32_t)__builtin_amdgcn_ds_bpermute(pull_scale, (int)zc);
        if constexpr (!PW) zb >>= half_shift;
        const float z = a.has_offsets ? (float)__builtin_bit_cast(_Float16, (unsigned short)zb) : 0.f;
        uint32_t w[P];
        float alpha[P];
#pragma unroll
        for (int i = 0; i < P; ++i) {
            w[i] = (uint32_t)__builtin_amdgcn_ds_bpermute(pull, (int)cur.w[i]);
            uint32_t ab = (uint32_t)__builtin_amdgcn_ds_bpermute(pull_scale, (int)sc[i]);
            if constexpr (!PW) ab >>= half_shift;
            alpha[i] = (float)__builtin_bit_cast(_Float16, (unsigned short)ab);
        }
        // the scales of the next four steps, once the last of these four has handed its own over
        if ((mine & 3) == 3 && g + GSTEP < a.ngroups) fetch_scales((mine >> 2) + 1);
        // The loads for the team's next group are spread over the four matrix steps below: issued all at once
        // right after the barrier, by every wave of the workgroup, they queue up in the memory pipe while
        // no wave has arithmetic to do.  With three or four planes the plane words go two planes per
        // matrix step, otherwise all of them here.
        constexpr bool kSpreadPlanes = P >= 3;
        const bool more = g + GSTEP < a.ngroups;
        if (more && !kSpreadPlanes) fetch_w(nxt, g + GSTEP);
        const unsigned char *xa_cur = xa_lane + buf * kTile;
        // table offsets of all low and all high nibbles of a plane word at once: byte t of `lo8` (`hi8`) is
        // eight times the low (high) nibble of byte t
        uint32_t lo8[P], hi8[P];
#pragma unroll
        for (int i = 0; i < P; ++i) {
            lo8[i] = (w[i] << 3) & 0x78787878u;
            hi8[i] = (w[i] >> 1) & 0x78787878u;
            if constexpr (SHARE) {              // byte t below: the team's sub-step t0 + t
                lo8[i] >>= 8 * t0;
                hi8[i] >>= 8 * t0;
            }
            // kept as they are: a look-up is then one add that picks byte t (the compiler would otherwise shift
            // and mask the plane word again for every nibble)
            asm volatile("" : "+v"(lo8[i]), "+v"(hi8[i]));
        }
        if constexpr (PW) {
            constexpr int PP = NT <= 2 ? 4 : 2;              // planes per pass: PP * NT partial-sum tiles live at a time
            constexpr int NPASS = (P + PP - 1) / PP;
            constexpr int NSLOT = 4 * NPASS;                 // matrix sub-steps over which the next loads are spread
            const v4f zero4 = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int pass = 0; pass < NPASS; ++pass) {
                v4f tmp[PP][NT];
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    v8h bw[PP];
#pragma unroll
                    for (int ii = 0; ii < PP; ++ii) {
                        const int i = pass * PP + ii;
                        if (i < P) {
                            const v4h lo = *lds_at<v4h>(lut_base + ((lo8[i] >> (8 * t)) & 0xffu));
                            const v4h hi = *lds_at<v4h>(lut_base + ((hi8[i] >> (8 * t)) & 0xffu));
                            bw[ii] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                        }
                    }
                    if (more) {
                        const int slot = pass * 4 + t;
                        if (kSpreadPlanes) {
#pragma unroll
                            for (int i = 0; i < P; ++i)
                                if (i / 2 == slot) fetch_plane(nxt, g + GSTEP, i);
                        }
#pragma unroll
                        for (int k = 0; k < XU; ++k)
                            if (k * NSLOT / XU == slot) stage_x_unit(g + GSTEP, buf ^ 1, k);
                    }
#pragma unroll
                    for (int c = 0; c < NT / UT; ++c) {
                        v8h xa[UT];
#pragma unroll
                        for (int u = 0; u < UT; ++u)
                            xa[u] = *reinterpret_cast<const v8h *>(xa_cur + (UT * c + u) * (16 * kXRowBytes) + xa_off[t]);
#pragma unroll
                        for (int u = 0; u < UT; ++u)
#pragma unroll
                            for (int ii = 0; ii < PP; ++ii)
                                if (pass * PP + ii < P)
                                    tmp[ii][UT * c + u] = __builtin_amdgcn_mfma_f32_16x16x32_f16(xa[u], bw[ii], t == 0 ? zero4 : tmp[ii][UT * c + u], 0, 0, 0);
                    }
                }
#pragma unroll
                for (int ii = 0; ii < PP; ++ii)
                    if (pass * PP + ii < P) {
#pragma unroll
                        for (int u = 0; u < NT; ++u)
#pragma unroll
                            for (int k = 0; k < 4; ++k) acc[u][k] = fmaf(alpha[pass * PP + ii], tmp[ii][u][k], acc[u][k]);
                    }
            }
            if (a.has_offsets) {
                // z * (sum of the group's activations): the same product with an all-ones operand
                v8h ones;
#pragma unroll
                for (int j = 0; j < 8; ++j) ones[j] = (_Float16)1.0f;
                v4f tz[NT];
#pragma unroll
                for (int t = 0; t < 4; ++t)
#pragma unroll
                    for (int u = 0; u < NT; ++u) {
                        const v8h xo = *reinterpret_cast<const v8h *>(xa_cur + u * (16 * kXRowBytes) + xa_off[t]);
                        tz[u] = __builtin_amdgcn_mfma_f32_16x16x32_f16(xo, ones, t == 0 ? zero4 : tz[u], 0, 0, 0);
                    }
#pragma unroll
                for (int u = 0; u < NT; ++u)
#pragma unroll
                    for (int k = 0; k < 4; ++k) acc[u][k] = fmaf(z, tz[u][k], acc[u][k]);
            }
        } else {
#pragma unroll
        for (int t = 0; t < TN; ++t) {
            // every LDS read of this matrix step goes out first: the table entries, then the activation operands
            // of the first four request tiles, which arrive while the weights are being rebuilt
            v4h pl[P], ph[P];
#pragma unroll
            for (int i = 0; i < P; ++i) {
                pl[i] = *lds_at<v4h>(lut_base + ((lo8[i] >> (8 * t)) & 0xffu));
                ph[i] = *lds_at<v4h>(lut_base + ((hi8[i] >> (8 * t)) & 0xffu));
            }
            v8h xa[UT];
#pragma unroll
            for (int u = 0; u < UT; ++u) xa[u] = *reinterpret_cast<const v8h *>(xa_cur + u * (16 * kXRowBytes) + xa_off[t]);
            if (more) {
                if (kSpreadPlanes) {
#pragma unroll
                    for (int i = 0; i < P; ++i)
                        if ((i / 2 < TN ? i / 2 : TN - 1) == t) fetch_plane(nxt, g + GSTEP, i);
                }
                // tile buf ^ 1 was last read before the previous barrier
#pragma unroll
                for (int k = 0; k < XU; ++k)
                    if (k * TN / XU == t) stage_x_unit(g + GSTEP, buf ^ 1, k);
            }
            __builtin_amdgcn_sched_barrier(0);
            float wf[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) wf[j] = z;
#pragma unroll
            for (int i = 0; i < P; ++i) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    wf[j] = fmaf((float)pl[i][j], alpha[i], wf[j]);
                    wf[4 + j] = fmaf((float)ph[i][j], alpha[i], wf[4 + j]);
                }
            }
            v8h wb;
#pragma unroll
            for (int j = 0; j < 8; ++j) wb[j] = (_Float16)wf[j];    // the single rounding of W_p to binary16
#pragma unroll
            for (int c = 0; c < NT / UT; ++c) {
                // the operands of the next four tiles are fetched while these four are in the matrix pipe
                v8h xn[UT];
                if (c + 1 < NT / UT) {
#pragma unroll
                    for (int u = 0; u < UT; ++u)
                        xn[u] = *reinterpret_cast<const v8h *>(xa_cur + (UT * (c + 1) + u) * (16 * kXRowBytes) + xa_off[t]);
                }
#pragma unroll
                for (int u = 0; u < UT; ++u) acc[UT * c + u] = __builtin_amdgcn_mfma_f32_16x16x32_f16(xa[u], wb, acc[UT * c + u], 0, 0, 0);
                if (c + 1 < NT / UT) {
#pragma unroll
                    for (int u = 0; u < UT; ++u) xa[u] = xn[u];
                }
            }
        }
        }
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);     // vmcnt(0): what was staged for the next step has landed in LDS
        // tile `buf` free, the other tile complete.  A team of ONE wave stages and reads its tiles itself: no barrier,
        // and the waves of the workgroup drift apart, which lets one compute while another waits.
        if constexpr (RW > 1 || SHARE) __syncthreads();
    };

    Ahead<P, XU> ah0, ah1;
#pragma unroll
    for (int i = 0; i < P; ++i) sc[i] = 0;
    if (g_first < a.ngroups) {
        stage_x(g_first, 0);
        fetch_w(ah0, g_first);
        fetch_scales(0);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();                            // table and first tiles complete
    const int npairs = (a.ngroups + 2 * GSTEP - 1) / (2 * GSTEP);
    for (int it = 0; it < npairs; ++it) {
        const int g = 2 * it * GSTEP + g_first;
        step(ah0, ah1, g, 2 * it, 0);
        step(ah1, ah0, g + GSTEP, 2 * it + 1, 1);
    }

    if constexpr (TEAMS > 1) {
        // (teams of one wave run without step barriers: all of them must have left their tiles before these are reused)
        if constexpr (RW == 1 && !SHARE) __syncthreads();
        // the other teams hand their accumulators over through the (now free) activation tiles
        v4f *xchg = reinterpret_cast<v4f *>(lds + kLutBytes);
        if (team > 0) {
#pragma unroll
            for (int u = 0; u < NT; ++u) xchg[(((team - 1) * RW + wave) * NT + u) * 64 + lane] = acc[u];
        }
        __syncthreads();
        if (team > 0) return;
#pragma unroll
        for (int k = 1; k < TEAMS; ++k)
#pragma unroll
            for (int u = 0; u < NT; ++u) acc[u] += xchg[(((k - 1) * RW + wave) * NT + u) * 64 + lane];
    }

    // accumulator u, register i: request b0 + 16u + 4kq + i of row row0 + n16
    const uint32_t row = row0 + n16;
    if (row < a.m) {
#pragma unroll
        for (int u = 0; u < NT; ++u)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int r = 16 * u + 4 * kq + i;
                if (r < nreq) a.y[(size_t)(BYCLASS ? req_of[r] : (uint32_t)(b0 + r)) * a.m + row] = (_Float16)acc[u][i];
            }
    }
}

template <int P, int NT, int TEAMS, int RW, bool PW = false, bool SHARE = false>
__global__ __launch_bounds__(64 * RW * TEAMS) __attribute__((amdgpu_waves_per_eu(NT <= 2 ? 4 : 1))) void dequant_mfma_kernel(DequantParams a)
{
    if (a.nmat > 1) {
        // which matrix this row of workgroups belongs to, picked by comparison (no indexing of the arguments)
        static_assert(BCQ_MAX_MULTI == 4, "the selection below is written for four matrices");
        uint32_t wg = blockIdx.x;
        const bool g1 = wg >= a.mat_blk0[1], g2 = wg >= a.mat_blk0[2], g3 = wg >= a.mat_blk0[3];
        a.planes = g3 ? a.mat_planes[3] : g2 ? a.mat_planes[2] : g1 ? a.mat_planes[1] : a.mat_planes[0];
        a.scales = g3 ? a.mat_scales[3] : g2 ? a.mat_scales[2] : g1 ? a.mat_scales[1] : a.mat_scales[0];
        a.offsets = a.scales;
        a.y = g3 ? a.mat_y[3] : g2 ? a.mat_y[2] : g1 ? a.mat_y[1] : a.mat_y[0];
        a.m = g3 ? a.mat_m[3] : g2 ? a.mat_m[2] : g1 ? a.mat_m[1] : a.mat_m[0];
        wg -= g3 ? a.mat_blk0[3] : g2 ? a.mat_blk0[2] : g1 ? a.mat_blk0[1] : 0u;
        a.plane_stride = a.m * a.row_stride;
        a.scale_plane_stride = a.m * a.scale_row_stride;
        dequant_mfma_body<P, NT, TEAMS, RW, PW, false, SHARE>(a, (int)blockIdx.y, wg);
        return;
    }
    dequant_mfma_body<P, NT, TEAMS, RW, PW, false, SHARE>(a, (int)blockIdx.y, blockIdx.x);
}

// Per-request precision beyond 64 requests: byte blockIdx.y of class_order is the precision a workgroup serves, with
// the scale and offset set of that precision and the body specialised for it (the deepest precision first, those
// without a scale set, whose requests only get zeros, last); one launch covers every precision, so that the
// workgroups of all of them share the chip (on short matrices those of one precision would leave most of it idle).
// blockIdx.z is the tile of 16 NT ranks: workgroups are dispatched in the order of their ids, so the first tiles
// of every precision, which hold the work, go first, and the tiles nobody's rank reaches (each costs its
// workgroup the ranking, and a CU holds one such workgroup at a time) trail behind instead of queueing in front
// of the next precision's work.
template <int Q, int NT, int TEAMS, int RW, bool SHARE>
__device__ __forceinline__ void serve_precision(DequantParams a)
{
    if (!a.scale_sets[Q]) {
        // no scale set for this precision: its requests get zeros (the workgroup's rows of its tile of ranks)
        extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
        uint32_t *req_of = reinterpret_cast<uint32_t *>(lds + lds_bytes(NT, SHARE ? 1 : TEAMS));
        const int nreq = rank_requests<16 * NT>(a, Q, (int)blockIdx.z * (16 * NT), req_of);
        if (nreq <= 0) return;
        __syncthreads();
        const uint32_t row0 = blockIdx.x * (16 * RW);
        for (int i = threadIdx.x; i < nreq * 16 * RW; i += 64 * RW * TEAMS) {
            const uint32_t row = row0 + (uint32_t)(i % (16 * RW));
            if (row < a.m) a.y[(size_t)req_of[i / (16 * RW)] * a.m + row] = (_Float16)0.f;
        }
        return;
    }
    a.scales = a.scale_sets[Q];
    a.has_offsets = a.offset_sets[Q] != nullptr;
    a.offsets = a.has_offsets ? a.offset_sets[Q] : a.scales;
    dequant_mfma_body<Q, NT, TEAMS, RW, false, true, SHARE>(a, (int)blockIdx.z, blockIdx.x);
}

template <int NT, int TEAMS, int RW, bool SHARE = false>
__global__ __launch_bounds__(64 * RW * TEAMS) void dequant_byclass_kernel(DequantParams a)
{
    switch ((a.class_order >> (8 * blockIdx.y)) & 0xffu) {
    case 1: serve_precision<1, NT, TEAMS, RW, SHARE>(a); break;
    case 2: serve_precision<2, NT, TEAMS, RW, SHARE>(a); break;
    case 3: serve_precision<3, NT, TEAMS, RW, SHARE>(a); break;
    default: serve_precision<4, NT, TEAMS, RW, SHARE>(a); break;
    }
}

// ---- per-request precision -------------------------------------------------------------------------
// The planes are shared by all precisions and only the scale sets differ (section 3.2), so one pass over
// the planes rebuilds W_q for every precision q that occurs among the workgroup's 64 requests - the table
// look-ups are shared, the FMAs are not - and multiplies ALL 64 requests with each of them into an
// accumulator set of its own (the matrix pipe has room to spare); at the end every request keeps the
// result of its own precision.  Requests are not sorted and nothing is masked.  A precision outside
// [1, p_max] is clamped; a request whose precision has no scale set yields zeros.
struct AheadMixed {                         // the plane words fetched one group ahead
    uint32_t w[kMaxP];
};

template <int TEAMS, int RW>
__global__ __launch_bounds__(64 * RW * TEAMS) void dequant_mixed_kernel(DequantParams a)
{
    constexpr int kTeamThreads = 64 * RW;
    constexpr int XU = 16 / RW;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    unsigned char *lut = lds;
    unsigned char *preq = lds + 128;          // precision of each of the 64 requests, behind the 128-byte table

    const int tid = threadIdx.x % kTeamThreads, team = __builtin_amdgcn_readfirstlane(threadIdx.x / kTeamThreads);
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    unsigned char *xt0 = lds + kLutBytes + team * 2 * x_tile_bytes(4);
    constexpr int kTile = x_tile_bytes(4);
    const int n16 = lane & 15, kq = lane >> 4;
    const uint32_t row0 = blockIdx.x * (16 * RW) + wave * 16;
    const int b0 = blockIdx.y * 64;

    if (threadIdx.x < 16) {
        uint32_t e[2];
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            const uint32_t lo = ((tid >> (2 * c)) & 1) ? 0x3C00u : 0xBC00u;
            const uint32_t hi = ((tid >> (2 * c + 1)) & 1) ? 0x3C00u : 0xBC00u;
            e[c] = lo | (hi << 16);
        }
        *reinterpret_cast<u32x2 *>(lut + tid * 8) = u32x2{e[0], e[1]};
    }
    // which precisions occur: lane l looks at request b0 + l; every wave sees the same 64 requests
    int p_lane = 0;
    if (b0 + lane < a.batch) {
        const int pr = a.p_req[b0 + lane];
        p_lane = pr < 1 ? 1 : (pr > a.p_max ? a.p_max : pr);
        if (!a.scale_sets[p_lane]) p_lane = 0;
    }
    if (threadIdx.x < 64) preq[lane] = (unsigned char)p_lane;
    bool has[kMaxP + 1];
    int p_hi = 0;
#pragma unroll
    for (int q = 1; q <= kMaxP; ++q) {
        has[q] = __ballot(p_lane == q) != 0;
        if (has[q]) p_hi = q;
    }
    const unsigned char *const set1 = a.scale_sets[1], *const set2 = a.scale_sets[2], *const set3 = a.scale_sets[3],
                        *const set4 = a.scale_sets[4];
    const unsigned char *const off1 = a.offset_sets[1], *const off2 = a.offset_sets[2], *const off3 = a.offset_sets[3],
                        *const off4 = a.offset_sets[4];
    auto set_of = [&](int q) { return q == 1 ? set1 : q == 2 ? set2 : q == 3 ? set3 : set4; };
    auto off_of = [&](int q) { return q == 1 ? off1 : q == 2 ? off2 : q == 3 ? off3 : off4; };

    const uint32_t frow = min(row0 + (lane >> 2), a.m - 1);
    uint32_t w_lane = frow * a.row_stride + (lane & 3) * 4;
    const uint32_t s_row = frow * a.scale_row_stride;
    const uint32_t half_shift = a.gshift < 0 && kq >= 2 ? 16u : 0u;     // groups of 64: columns 64..127 of a step use the upper scale
    // scales and offsets in flight / in use (binary16 bits, two of them with groups of 64), fetched for four of the
    // team's steps at once as in dequant_mfma_kernel; set q plane i at q (q - 1) / 2 + i
    uint32_t sc[10], zc[kMaxP];
#pragma unroll
    for (int i = 0; i < 10; ++i) sc[i] = 0;
#pragma unroll
    for (int i = 0; i < kMaxP; ++i) zc[i] = 0;
    auto scale_col = [&](int g) { return (uint32_t)(a.gshift > 0 ? (g >> 1) * 2 : a.gshift < 0 ? g * 4 : g * 2); };
    const int pull = (4 * n16 + kq) * 4;
    // staging straight into LDS and the XOR placement of the parts: as in dequant_mfma_kernel
    uint32_t xs_src[XU];
#pragma unroll
    for (int k = 0; k < XU; ++k) {
        const int req = 4 * (k * RW + wave) + (lane >> 4);
        const int part = (lane & 15) ^ (req & 15);
        xs_src[k] = (uint32_t)min(b0 + req, a.batch - 1) * a.x_stride + part * 16;
    }
    const unsigned char *xa_lane = xt0 + n16 * kXRowBytes;
    uint32_t xa_off[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) xa_off[t] = (uint32_t)(((4 * kq + t) ^ n16) * 16);

    auto fetch_w = [&](AheadMixed &ah, int g) {
#pragma unroll
        for (int i = 0; i < kMaxP; ++i) {
            if (i < p_hi) {
                const unsigned char *w_base = a.planes + (size_t)i * a.plane_stride + (uint32_t)g * 16;
                ah.w[i] = *reinterpret_cast<const uint32_t *>(w_base + w_lane);     // cached, as in dequant_mfma_kernel
            }
        }
    };
    auto fetch_scales = [&](int block) {      // for the team's steps 4 block .. 4 block + 3
        const int gj = min(team + TEAMS * (4 * block + (lane & 3)), a.ngroups - 1);
        uint32_t off = s_row + scale_col(gj);
#pragma unroll
        for (int q = 1; q <= kMaxP; ++q) {
            if (has[q]) {
                asm volatile("" : "+v"(off));
                if (a.gshift < 0) {
#pragma unroll
                    for (int i = 0; i < q; ++i) sc[q * (q - 1) / 2 + i] = *reinterpret_cast<const uint32_t *>(set_of(q) + (size_t)i * a.scale_plane_stride + off);
                    if (off_of(q)) zc[q - 1] = *reinterpret_cast<const uint32_t *>(off_of(q) + off);
                } else {
#pragma unroll
                    for (int i = 0; i < q; ++i) sc[q * (q - 1) / 2 + i] = *reinterpret_cast<const unsigned short *>(set_of(q) + (size_t)i * a.scale_plane_stride + off);
                    if (off_of(q)) zc[q - 1] = *reinterpret_cast<const unsigned short *>(off_of(q) + off);
                }
            }
        }
    };
    auto stage_x_unit = [&](int g, int buf, int k) {
        const unsigned char *x_base = a.x + (uint32_t)g * 256;
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(x_base + xs_src[k]),
                                         (__attribute__((address_space(3))) void *)(xt0 + buf * kTile + (k * RW + wave) * 1024), 16, 0, 0);
    };
    auto stage_x = [&](int g, int buf) {
#pragma unroll
        for (int k = 0; k < XU; ++k) stage_x_unit(g, buf, k);
    };

    uint32_t lut_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)lut;
    asm volatile("" : "+s"(lut_base));

    v4f acc[kMaxP][4];
#pragma unroll
    for (int q = 0; q < kMaxP; ++q)
#pragma unroll
        for (int u = 0; u < 4; ++u) acc[q][u] = v4f{0.f, 0.f, 0.f, 0.f};

    auto step = [&](AheadMixed &cur, AheadMixed &nxt, int g, int mine, int buf) {
        if (g < a.ngroups) {
#pragma unroll
            for (int i = 0; i < kMaxP; ++i) asm volatile("" : "+v"(cur.w[i]));
#pragma unroll
            for (int i = 0; i < 10; ++i) asm volatile("" : "+v"(sc[i]));
#pragma unroll
            for (int i = 0; i < kMaxP; ++i) asm volatile("" : "+v"(zc[i]));
            // lane offsets made new in every step, table look-ups by byte pick: as in dequant_mfma_kernel
            asm volatile("" : "+v"(w_lane));
            const int pull_scale = 4 * n16 * 4 + (mine & 3) * 4;    // the lane that fetched this step's scales of row n16
#pragma unroll
            for (int k = 0; k < XU; ++k) asm volatile("" : "+v"(xs_src[k]));
            auto handed = [&](uint32_t v) {
                const uint32_t bits = (uint32_t)__builtin_amdgcn_ds_bpermute(pull_scale, (int)v) >> half_shift;
                return (float)__builtin_bit_cast(_Float16, (unsigned short)bits);
            };
            uint32_t w[kMaxP];
            float alpha[10], z[kMaxP];
#pragma unroll
            for (int i = 0; i < kMaxP; ++i) w[i] = i < p_hi ? (uint32_t)__builtin_amdgcn_ds_bpermute(pull, (int)cur.w[i]) : 0u;
#pragma unroll
            for (int q = 1; q <= kMaxP; ++q) {
                z[q - 1] = 0.f;
                if (has[q]) {
#pragma unroll
                    for (int i = 0; i < q; ++i) alpha[q * (q - 1) / 2 + i] = handed(sc[q * (q - 1) / 2 + i]);
                    if (off_of(q)) z[q - 1] = handed(zc[q - 1]);
                } else {
#pragma unroll
                    for (int i = 0; i < q; ++i) alpha[q * (q - 1) / 2 + i] = 0.f;
                }
            }
            const bool more = g + TEAMS < a.ngroups;
            if (more) fetch_w(nxt, g + TEAMS);
            if ((mine & 3) == 3 && more) fetch_scales((mine >> 2) + 1);
            const unsigned char *xa_cur = xa_lane + buf * kTile;
            uint32_t lo8[kMaxP], hi8[kMaxP];
#pragma unroll
            for (int i = 0; i < kMaxP; ++i) {
                lo8[i] = (w[i] << 3) & 0x78787878u;
                hi8[i] = (w[i] >> 1) & 0x78787878u;
                if (i < p_hi) asm volatile("" : "+v"(lo8[i]), "+v"(hi8[i]));
            }
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                v4h pl[kMaxP], ph[kMaxP];
#pragma unroll
                for (int i = 0; i < kMaxP; ++i) {
                    if (i < p_hi) {
                        pl[i] = *lds_at<v4h>(lut_base + ((lo8[i] >> (8 * t)) & 0xffu));
                        ph[i] = *lds_at<v4h>(lut_base + ((hi8[i] >> (8 * t)) & 0xffu));
                    } else {
                        pl[i] = ph[i] = v4h{0, 0, 0, 0};
                    }
                }
                v8h xa[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) xa[u] = *reinterpret_cast<const v8h *>(xa_cur + u * (16 * kXRowBytes) + xa_off[t]);
                if (more) {
                    // the next tile's loads spread over the matrix steps, as in dequant_mfma_kernel
#pragma unroll
                    for (int k = 0; k < XU; ++k)
                        if (k * 4 / XU == t) stage_x_unit(g + TEAMS, buf ^ 1, k);
                }
#pragma unroll
                for (int q = 1; q <= kMaxP; ++q) {
                    if (has[q]) {
                        float wf[8];
#pragma unroll
                        for (int j = 0; j < 8; ++j) wf[j] = z[q - 1];
#pragma unroll
                        for (int i = 0; i < q; ++i) {
#pragma unroll
                            for (int j = 0; j < 4; ++j) {
                                wf[j] = fmaf((float)pl[i][j], alpha[q * (q - 1) / 2 + i], wf[j]);
                                wf[4 + j] = fmaf((float)ph[i][j], alpha[q * (q - 1) / 2 + i], wf[4 + j]);
                            }
                        }
                        v8h wb;
#pragma unroll
                        for (int j = 0; j < 8; ++j) wb[j] = (_Float16)wf[j];      // the single rounding of W_q to binary16
#pragma unroll
                        for (int u = 0; u < 4; ++u) acc[q - 1][u] = __builtin_amdgcn_mfma_f32_16x16x32_f16(xa[u], wb, acc[q - 1][u], 0, 0, 0);
                    }
                }
            }
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);     // vmcnt(0): what was staged for the next step has landed in LDS
        if constexpr (RW > 1) __syncthreads();  // (a team of one wave owns its tiles: see dequant_mfma_kernel)
    };

    AheadMixed ah0{}, ah1{};
    if (team < a.ngroups) {
        stage_x(team, 0);
        fetch_w(ah0, team);
        fetch_scales(0);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
    const int npairs = (a.ngroups + 2 * TEAMS - 1) / (2 * TEAMS);
    for (int it = 0; it < npairs; ++it) {
        const int g = 2 * it * TEAMS + team;
        step(ah0, ah1, g, 2 * it, 0);
        step(ah1, ah0, g + TEAMS, 2 * it + 1, 1);
    }

    if constexpr (TEAMS > 1) {
        // (teams of one wave run without step barriers: all of them must have left their tiles before these are reused)
        if constexpr (RW == 1) __syncthreads();
        v4f *xchg = reinterpret_cast<v4f *>(lds + kLutBytes);
        if (team > 0) {
#pragma unroll
            for (int q = 0; q < kMaxP; ++q)
                if (has[q + 1]) {
#pragma unroll
                    for (int u = 0; u < 4; ++u) xchg[((((team - 1) * RW + wave) * kMaxP + q) * 4 + u) * 64 + lane] = acc[q][u];
                }
        }
        __syncthreads();
        if (team > 0) return;
#pragma unroll
        for (int k = 1; k < TEAMS; ++k)
#pragma unroll
            for (int q = 0; q < kMaxP; ++q)
                if (has[q + 1]) {
#pragma unroll
                    for (int u = 0; u < 4; ++u) acc[q][u] += xchg[((((k - 1) * RW + wave) * kMaxP + q) * 4 + u) * 64 + lane];
                }
    }

    // accumulator u, register i: request b0 + 16u + 4kq + i of row row0 + n16, at each precision; keep its own
    const uint32_t row = row0 + n16;
    if (row < a.m) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int r = 16 * u + 4 * kq + i;
                const int pb = preq[r];
                const float v = pb == 1 ? acc[0][u][i] : pb == 2 ? acc[1][u][i] : pb == 3 ? acc[2][u][i] : pb == 4 ? acc[3][u][i] : 0.f;
                if (b0 + r < a.batch) a.y[(size_t)(b0 + r) * a.m + row] = (_Float16)v;
            }
    }
}


// Per-request precision, plane-wise: the group sums B_i x of the planes are the same for every request, only the
// scale that multiplies them is the request's own (section 3.3: a request at precision q uses planes 0 .. q-1
// with the scale set of q).  One pass over the planes serves the whole tile whatever mix of precisions it
// holds; a lane picks, for each of its four requests per tile and each plane, the scale of that request's
// precision (zero from plane q on) by compare masks formed once.  NT tiles of 16 requests per workgroup.
// (At least four waves per SIMD: two of the 32-row workgroups then share a CU, which the kernel needs more than
// the dozen extra registers the compiler would otherwise take.)
template <int NT, int TEAMS, int RW>
__global__ __launch_bounds__(64 * RW * TEAMS) __attribute__((amdgpu_waves_per_eu(NT == 1 ? 4 : 2))) void planewise_mixed_kernel(DequantParams a)
{
    constexpr int kTeamThreads = 64 * RW;
    constexpr int XU = 4 * NT / RW;
    constexpr int PP = NT <= 2 ? 4 : 2;       // planes per pass
    static_assert(XU >= 1, "tile does not split over the team");
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    unsigned char *lut = lds;

    const int tid = threadIdx.x % kTeamThreads, team = __builtin_amdgcn_readfirstlane(threadIdx.x / kTeamThreads);
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    unsigned char *xt0 = lds + kLutBytes + team * 2 * x_tile_bytes(NT);
    constexpr int kTile = x_tile_bytes(NT);
    const int n16 = lane & 15, kq = lane >> 4;
    const uint32_t row0 = blockIdx.x * (16 * RW) + wave * 16;
    const int b0 = blockIdx.y * (16 * NT);

    if (threadIdx.x < 16) {
        uint32_t e[2];
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            const uint32_t lo = ((tid >> (2 * c)) & 1) ? 0x3C00u : 0xBC00u;
            const uint32_t hi = ((tid >> (2 * c + 1)) & 1) ? 0x3C00u : 0xBC00u;
            e[c] = lo | (hi << 16);
        }
        *reinterpret_cast<u32x2 *>(lut + tid * 8) = u32x2{e[0], e[1]};
    }
    const unsigned char *const set1 = a.scale_sets[1], *const set2 = a.scale_sets[2], *const set3 = a.scale_sets[3],
                        *const set4 = a.scale_sets[4];
    const unsigned char *const off1 = a.offset_sets[1], *const off2 = a.offset_sets[2], *const off3 = a.offset_sets[3],
                        *const off4 = a.offset_sets[4];
    auto set_of = [&](int q) { return q == 1 ? set1 : q == 2 ? set2 : q == 3 ? set3 : set4; };
    auto off_of = [&](int q) { return q == 1 ? off1 : q == 2 ? off2 : q == 3 ? off3 : off4; };

    const uint32_t frow = min(row0 + (lane >> 2), a.m - 1);
    uint32_t w_lane = frow * a.row_stride + (lane & 3) * 4;
    uint32_t s_lane = frow * a.scale_row_stride;
    auto scale_col = [&](int g) { return (uint32_t)(a.gshift > 0 ? (g >> 1) * 2 : g * 2); };
    const int pull = (4 * n16 + kq) * 4;
    uint32_t xs_src[XU];
#pragma unroll
    for (int k = 0; k < XU; ++k) {
        const int req = 4 * (k * RW + wave) + (lane >> 4);
        const int part = (lane & 15) ^ (req & 15);
        xs_src[k] = (uint32_t)min(b0 + req, a.batch - 1) * a.x_stride + part * 16;
    }
    const unsigned char *xa_lane = xt0 + n16 * kXRowBytes;
    uint32_t xa_off[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) xa_off[t] = (uint32_t)(((4 * kq + t) ^ n16) * 16);

    uint32_t lut_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)lut;
    asm volatile("" : "+s"(lut_base));

    v4f acc[NT];
#pragma unroll
    for (int u = 0; u < NT; ++u) acc[u] = v4f{0.f, 0.f, 0.f, 0.f};
    const v4f zero4 = v4f{0.f, 0.f, 0.f, 0.f};

    uint32_t sc[10], zc[kMaxP];               // scales and offsets in flight / in use: binary16 bits, set q plane i at q (q - 1) / 2 + i
#pragma unroll
    for (int i = 0; i < 10; ++i) sc[i] = 0;
#pragma unroll
    for (int i = 0; i < kMaxP; ++i) zc[i] = 0;

    // ---- the first loads (everything above is address arithmetic).  Which precisions occur: lane l looks at request
    // b0 + l; every wave sees the same requests.  That load goes out first, and what does not depend on its result (the
    // first activation tile, the first group's plane words to the deepest plane stored, the first block of every scale
    // set passed) is asked for before the result is looked at, so that the kernel does not begin with one memory
    // latency in which nothing else is under way (14336 x 4096, 16 requests at precisions from {2, 3, 4}: 24.4 -> 23.1 us).
    __builtin_amdgcn_sched_barrier(0);
    const bool p_known = lane < 16 * NT && b0 + lane < a.batch;
    const int p_raw = a.p_req[p_known ? b0 + lane : 0];      // (request 0 exists: batch >= 1)
    AheadMixed ah0{}, ah1{};
    if (team < a.ngroups) {
#pragma unroll
        for (int k = 0; k < XU; ++k)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(a.x + (uint32_t)team * 256 + xs_src[k]),
                                             (__attribute__((address_space(3))) void *)(xt0 + (k * RW + wave) * 1024), 16, 0, 0);
#pragma unroll
        for (int i = 0; i < kMaxP; ++i)
            if (i < a.p_max) ah0.w[i] = *reinterpret_cast<const uint32_t *>(a.planes + (size_t)i * a.plane_stride + (uint32_t)team * 16 + w_lane);
        const uint32_t off = s_lane + scale_col(min(team + TEAMS * (lane & 3), a.ngroups - 1));
#pragma unroll
        for (int q = 1; q <= kMaxP; ++q)
            if (q <= a.p_max && set_of(q)) {
#pragma unroll
                for (int i = 0; i < kMaxP; ++i)
                    if (i < q) sc[q * (q - 1) / 2 + i] = *reinterpret_cast<const unsigned short *>(set_of(q) + (size_t)i * a.scale_plane_stride + off);
                if (off_of(q)) zc[q - 1] = *reinterpret_cast<const unsigned short *>(off_of(q) + off);
            }
    }
    __builtin_amdgcn_sched_barrier(0);

    // ---- the precisions of the tile
    int p_lane = 0;
    if (p_known) {
        p_lane = p_raw < 1 ? 1 : (p_raw > a.p_max ? a.p_max : p_raw);
        if (!a.scale_sets[p_lane]) p_lane = 0;
    }
    bool has[kMaxP + 1];
    int p_hi = 0;
    bool any_offset = false;
#pragma unroll
    for (int q = 1; q <= kMaxP; ++q) {
        has[q] = __ballot(p_lane == q) != 0;
        if (has[q]) p_hi = q;
        if (has[q] && a.offset_sets[q]) any_offset = true;
    }
    // This lane's own requests: accumulator u, register k holds request 16u + 4kq + k.  The scales of a plane
    // travel as four binary16 values in two registers (sets 1 | 2 and 3 | 4); `pick` is the byte selector that
    // moves the values of TWO requests' precisions into the two halves of a register (a precision of 0 selects
    // zero bytes), from which the fused multiply-adds take them without a conversion of their own.
    uint32_t pick[NT][2];
#pragma unroll
    for (int u = 0; u < NT; ++u)
#pragma unroll
        for (int k2 = 0; k2 < 2; ++k2) {
            uint32_t sel = 0;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int pq = __shfl(p_lane, 16 * u + 4 * kq + 2 * k2 + h);
                sel |= (pq == 0 ? 0x0C0Cu : (uint32_t)((2 * pq - 1) << 8) | (uint32_t)(2 * pq - 2)) << (16 * h);
            }
            pick[u][k2] = sel;
        }

    // The sweep over the groups, with the number of planes the tile needs (its highest precision) as a
    // compile-time number: inside, a step is one straight run of instructions.
    auto sweep = [&](auto ph_tag) {
    constexpr int PH = decltype(ph_tag)::value;
    // Plane t of a group is fetched at matrix sub-step t of the step before (see dequant_mfma_kernel).  The scale sets
    // are fetched for four of the team's steps at once, as there: the four lanes of a row take the groups of the
    // steps 4 block .. 4 block + 3; sets of precisions no request of the tile has are never fetched and stay zero.
    auto fetch_part = [&](AheadMixed &ah, int g, int part) {
        if (part < PH) {
            const unsigned char *w_base = a.planes + (size_t)part * a.plane_stride + (uint32_t)g * 16;
            ah.w[part] = *reinterpret_cast<const uint32_t *>(w_base + w_lane);
        }
    };
    auto fetch_scales = [&](int block) {
        const int gj = min(team + TEAMS * (4 * block + (lane & 3)), a.ngroups - 1);
        uint32_t off = s_lane + scale_col(gj);
#pragma unroll
        for (int q = 1; q <= PH; ++q)
            if (q == PH || has[q]) {
                asm volatile("" : "+v"(off));     // (keeps the widening of the offset next to the loads, see the step)
#pragma unroll
                for (int i = 0; i < kMaxP; ++i)
                    if (i < q) sc[q * (q - 1) / 2 + i] = *reinterpret_cast<const unsigned short *>(set_of(q) + (size_t)i * a.scale_plane_stride + off);
                if (off_of(q)) zc[q - 1] = *reinterpret_cast<const unsigned short *>(off_of(q) + off);
            }
    };
    auto stage_x_unit = [&](int g, int buf, int k) {
        const unsigned char *x_base = a.x + (uint32_t)g * 256;
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(x_base + xs_src[k]),
                                         (__attribute__((address_space(3))) void *)(xt0 + buf * kTile + (k * RW + wave) * 1024), 16, 0, 0);
    };

    auto step = [&](AheadMixed &cur, AheadMixed &nxt, int g, int mine, int buf) {
        if (g < a.ngroups) {
#pragma unroll
            for (int i = 0; i < kMaxP; ++i) asm volatile("" : "+v"(cur.w[i]));
#pragma unroll
            for (int i = 0; i < 10; ++i) asm volatile("" : "+v"(sc[i]));
#pragma unroll
            for (int i = 0; i < kMaxP; ++i) asm volatile("" : "+v"(zc[i]));
            asm volatile("" : "+v"(w_lane));
            const int pull_scale = 4 * n16 * 4 + (mine & 3) * 4;    // the lane that fetched this step's scales of row n16
#pragma unroll
            for (int k = 0; k < XU; ++k) asm volatile("" : "+v"(xs_src[k]));
            // (scales of a precision no request of the tile has were never fetched: they are still zero)
            auto own_values = [](uint32_t hi, uint32_t lo, uint32_t sel) {       // of requests 2 k2 and 2 k2 + 1
                return __builtin_bit_cast(h2v, __builtin_amdgcn_perm(hi, lo, sel));
            };
            uint32_t w[kMaxP], s_lo[kMaxP], s_hi[kMaxP];
#pragma unroll
            for (int i = 0; i < kMaxP; ++i) w[i] = i < PH ? (uint32_t)__builtin_amdgcn_ds_bpermute(pull, (int)cur.w[i]) : 0u;
#pragma unroll
            for (int i = 0; i < kMaxP; ++i) {
                // plane i belongs to the sets q > i
                const uint32_t lo = (i < 1 ? sc[0] : 0u) | (i < 2 ? sc[1 + i] << 16 : 0u);
                const uint32_t hi = (i < 3 ? sc[3 + i] : 0u) | (sc[6 + i] << 16);
                s_lo[i] = i < 2 ? (uint32_t)__builtin_amdgcn_ds_bpermute(pull_scale, (int)lo) : 0u;
                s_hi[i] = (uint32_t)__builtin_amdgcn_ds_bpermute(pull_scale, (int)hi);
            }
            uint32_t z_lo = 0, z_hi = 0;
            if (any_offset) {
                z_lo = (uint32_t)__builtin_amdgcn_ds_bpermute(pull_scale, (int)(zc[0] | zc[1] << 16));
                z_hi = (uint32_t)__builtin_amdgcn_ds_bpermute(pull_scale, (int)(zc[2] | zc[3] << 16));
            }
            // the scale sets of the next four steps, once the last of these four has handed its own over
            if ((mine & 3) == 3 && g + TEAMS < a.ngroups) fetch_scales((mine >> 2) + 1);
            const bool more = g + TEAMS < a.ngroups;
            const unsigned char *xa_cur = xa_lane + buf * kTile;
            uint32_t lo8[kMaxP], hi8[kMaxP];
#pragma unroll
            for (int i = 0; i < kMaxP; ++i) {
                lo8[i] = (w[i] << 3) & 0x78787878u;
                hi8[i] = (w[i] >> 1) & 0x78787878u;
                if (i < PH) asm volatile("" : "+v"(lo8[i]), "+v"(hi8[i]));
            }
            // scale of plane i for the request in (u, k): that of the request's own precision, zero from plane p on
            auto own_scales = [&](int i, int u, int k2) { return own_values(s_hi[i], s_lo[i], pick[u][k2]); };
            constexpr int NPASS = kMaxP / PP;
#pragma unroll
            for (int pass = 0; pass < NPASS; ++pass) {
                if (pass * PP < PH) {
                    v4f tmp[PP][NT];
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        v8h bw[PP];
#pragma unroll
                        for (int ii = 0; ii < PP; ++ii) {
                            const int i = pass * PP + ii;
                            if (i < PH) {
                                const v4h lo = *lds_at<v4h>(lut_base + ((lo8[i] >> (8 * t)) & 0xffu));
                                const v4h hi = *lds_at<v4h>(lut_base + ((hi8[i] >> (8 * t)) & 0xffu));
                                bw[ii] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                            }
                        }
                        if (more && pass == 0) {
                            fetch_part(nxt, g + TEAMS, t);
#pragma unroll
                            for (int k = 0; k < XU; ++k)
                                if (k * 4 / XU == t) stage_x_unit(g + TEAMS, buf ^ 1, k);
                        }
#pragma unroll
                        for (int u = 0; u < NT; ++u) {
                            const v8h xa = *reinterpret_cast<const v8h *>(xa_cur + u * (16 * kXRowBytes) + xa_off[t]);
#pragma unroll
                            for (int ii = 0; ii < PP; ++ii)
                                if (pass * PP + ii < PH)
                                    tmp[ii][u] = __builtin_amdgcn_mfma_f32_16x16x32_f16(xa, bw[ii], t == 0 ? zero4 : tmp[ii][u], 0, 0, 0);
                        }
                    }
#pragma unroll
                    for (int ii = 0; ii < PP; ++ii)
                        if (pass * PP + ii < PH) {
#pragma unroll
                            for (int u = 0; u < NT; ++u)
#pragma unroll
                                for (int k2 = 0; k2 < 2; ++k2) {
                                    const h2v al = own_scales(pass * PP + ii, u, k2);
                                    acc[u][2 * k2] = fmaf((float)al[0], tmp[ii][u][2 * k2], acc[u][2 * k2]);
                                    acc[u][2 * k2 + 1] = fmaf((float)al[1], tmp[ii][u][2 * k2 + 1], acc[u][2 * k2 + 1]);
                                }
                        }
                }
            }
            if (any_offset) {
                v8h ones;
#pragma unroll
                for (int j = 0; j < 8; ++j) ones[j] = (_Float16)1.0f;
                v4f tz[NT];
#pragma unroll
                for (int t = 0; t < 4; ++t)
#pragma unroll
                    for (int u = 0; u < NT; ++u) {
                        const v8h xo = *reinterpret_cast<const v8h *>(xa_cur + u * (16 * kXRowBytes) + xa_off[t]);
                        tz[u] = __builtin_amdgcn_mfma_f32_16x16x32_f16(xo, ones, t == 0 ? zero4 : tz[u], 0, 0, 0);
                    }
#pragma unroll
                for (int u = 0; u < NT; ++u)
#pragma unroll
                    for (int k2 = 0; k2 < 2; ++k2) {
                        const h2v zz = own_values(z_hi, z_lo, pick[u][k2]);
                        acc[u][2 * k2] = fmaf((float)zz[0], tz[u][2 * k2], acc[u][2 * k2]);
                        acc[u][2 * k2 + 1] = fmaf((float)zz[1], tz[u][2 * k2 + 1], acc[u][2 * k2 + 1]);
                    }
            }
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);     // vmcnt(0): what was staged for the next step has landed in LDS
        if constexpr (RW > 1) __syncthreads();  // (a team of one wave owns its tiles: see dequant_mfma_kernel)
    };

    // (the first tile, plane words and scales were asked for before the precisions were known)
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
    const int npairs = (a.ngroups + 2 * TEAMS - 1) / (2 * TEAMS);
    for (int it = 0; it < npairs; ++it) {
        const int g = 2 * it * TEAMS + team;
        step(ah0, ah1, g, 2 * it, 0);
        step(ah1, ah0, g + TEAMS, 2 * it + 1, 1);
    }
    };
    switch (p_hi) {       // the same in every wave of the workgroup: all of them take the same barriers
    case 1: sweep(std::integral_constant<int, 1>{}); break;
    case 2: sweep(std::integral_constant<int, 2>{}); break;
    case 3: sweep(std::integral_constant<int, 3>{}); break;
    case 4: sweep(std::integral_constant<int, 4>{}); break;
    default: break;       // no request of the tile has a scale set: zeros
    }

    if constexpr (TEAMS > 1) {
        // (teams of one wave run without step barriers: all of them must have left their tiles before these are reused)
        if constexpr (RW == 1) __syncthreads();
        v4f *xchg = reinterpret_cast<v4f *>(lds + kLutBytes);
        if (team > 0) {
#pragma unroll
            for (int u = 0; u < NT; ++u) xchg[(((team - 1) * RW + wave) * NT + u) * 64 + lane] = acc[u];
        }
        __syncthreads();
        if (team > 0) return;
#pragma unroll
        for (int k = 1; k < TEAMS; ++k)
#pragma unroll
            for (int u = 0; u < NT; ++u) acc[u] += xchg[(((k - 1) * RW + wave) * NT + u) * 64 + lane];
    }

    const uint32_t row = row0 + n16;
    if (row < a.m) {
#pragma unroll
        for (int u = 0; u < NT; ++u)
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int b = b0 + 16 * u + 4 * kq + k;
                if (b < a.batch) a.y[(size_t)b * a.m + row] = (_Float16)acc[u][k];
            }
    }
}

template <int NT, int TEAMS, int RW>
hipError_t launch_planewise_mixed(const DequantParams &pr, const GemmArgs &a, hipStream_t stream)
{
    static_assert((TEAMS - 1) * RW * NT * 64 * 16 <= TEAMS * 2 * x_tile_bytes(NT), "accumulator exchange must fit in the tiles");
    auto kernel = planewise_mixed_kernel<NT, TEAMS, RW>;
    if (hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(kernel), lds_bytes(NT, TEAMS))) return e;
    dim3 grid((unsigned)((a.m + 16 * RW - 1) / (16 * RW)), (unsigned)((a.batch + 16 * NT - 1) / (16 * NT)));
    hipLaunchKernelGGL(kernel, grid, dim3(64 * RW * TEAMS), lds_bytes(NT, TEAMS), stream, pr);
    return hipGetLastError();
}

template <int TEAMS, int RW>
hipError_t launch_mixed(const DequantParams &pr, const GemmArgs &a, hipStream_t stream)
{
    static_assert((TEAMS - 1) * RW * kMaxP * 4 * 64 * 16 <= TEAMS * 2 * x_tile_bytes(4), "accumulator exchange must fit in the tiles");
    auto kernel = dequant_mixed_kernel<TEAMS, RW>;
    if (hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(kernel), lds_bytes(4, TEAMS))) return e;
    dim3 grid((unsigned)((a.m + 16 * RW - 1) / (16 * RW)), (unsigned)((a.batch + 63) / 64));
    hipLaunchKernelGGL(kernel, grid, dim3(64 * RW * TEAMS), lds_bytes(4, TEAMS), stream, pr);
    return hipGetLastError();
}

template <int P, int NT, int TEAMS, int RW, bool PW, bool SHARE = false>
hipError_t launch_one(const DequantParams &pr, const GemmArgs &a, hipStream_t stream)
{
    constexpr int LT = SHARE ? 1 : TEAMS;     // pairs of tiles in LDS
    static_assert((TEAMS - 1) * RW * NT * 64 * 16 <= LT * 2 * x_tile_bytes(NT), "accumulator exchange must fit in the tiles");
    auto kernel = dequant_mfma_kernel<P, NT, TEAMS, RW, PW, SHARE>;
    if (hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(kernel), lds_bytes(NT, LT))) return e;
    dim3 grid((unsigned)((a.m + 16 * RW - 1) / (16 * RW)), (unsigned)((a.batch + 16 * NT - 1) / (16 * NT)));
    if (pr.nmat > 1) {
        // several matrices: every matrix gets whole workgroups (pr.mat_m holds the row counts; the offsets are made here
        // because they depend on the rows per workgroup)
        DequantParams pm = pr;
        uint32_t blk = 0;
        for (int k = 0; k < BCQ_MAX_MULTI; ++k) {
            pm.mat_blk0[k] = blk;
            if (k < pr.nmat) blk += (pr.mat_m[k] + 16 * RW - 1) / (16 * RW);
        }
        for (int k = pr.nmat; k < BCQ_MAX_MULTI; ++k) pm.mat_blk0[k] = blk;     // never reached
        grid.x = blk;
        hipLaunchKernelGGL(kernel, grid, dim3(64 * RW * TEAMS), lds_bytes(NT, LT), stream, pm);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(kernel, grid, dim3(64 * RW * TEAMS), lds_bytes(NT, LT), stream, pr);
    return hipGetLastError();
}

template <int NT, int TEAMS, int RW, bool SHARE = false>
hipError_t launch_byclass(const DequantParams &pr, const GemmArgs &a, hipStream_t stream)
{
    constexpr int LT = SHARE ? 1 : TEAMS;
    static_assert((TEAMS - 1) * RW * NT * 64 * 16 <= LT * 2 * x_tile_bytes(NT), "accumulator exchange must fit in the tiles");
    auto kernel = dequant_byclass_kernel<NT, TEAMS, RW, SHARE>;
    constexpr int kLds = lds_bytes(NT, LT) + 16 * NT * 4;           // the workgroup's request numbers behind the tiles
    if (hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(kernel), kLds)) return e;
    dim3 grid((unsigned)((a.m + 16 * RW - 1) / (16 * RW)), (unsigned)a.p_max, (unsigned)((a.batch + 16 * NT - 1) / (16 * NT)));
    hipLaunchKernelGGL(kernel, grid, dim3(64 * RW * TEAMS), kLds, stream, pr);
    return hipGetLastError();
}

// Shape of the workgroups: NT = 1, 4, 8 or 16 tiles of 16 requests (with four, four, two and one team), RW = 4, 2
// or 1 blocks of 16 rows.  With the 64-request tiles and larger a CU holds one workgroup at a time, so the time of a
// call is about (rounds of workgroups over the 256 CUs) x (time of one workgroup per group of columns).  The
// second factor was measured for every shape on a grid that fills the chip once (microseconds per group, p = 4
// and p = 2): larger workgroups reuse dequantised weights and staged activations better, smaller ones keep CUs
// busy on short matrices; the 16-request tile saves matrix instructions and operand reads when the batch is
// that small.  The cheapest product wins; dequant_mfma_force_shape overrides the choice (benchmarks, tests).
struct WgShape {
    int nt, rw;                 // rw: row-block code (1, 2, 4: that many blocks of 16 rows; 8 and 40: see below)
    float us_p4, us_p2;         // a grid far below one workgroup per CU
    float many_p4, many_p2;     // per workgroup and 256 workgroups of the grid when that is more (0: whole rounds of the above)
};
// blocks of 16 rows per workgroup for a shape's row-block code
constexpr int row_blocks_of(int nt, int code) { return code == 40 ? 4 : code == 8 ? (nt <= 2 ? 1 : 8) : code; }
// The 16- and 32-request shapes need 32 or 64 KiB of LDS and few registers, so several of their workgroups share a
// CU and a grid beyond 256 workgroups costs less than whole rounds; they are used for a single tile only (two
// such tiles never beat one 64-request tile).
constexpr WgShape kShapes[] = {{1, 4, 0.51f, 0.32f, 0.78f, 0.39f}, {1, 2, 0.36f, 0.26f, 0.34f, 0.19f}, {1, 1, 0.31f, 0.28f, 0.175f, 0.11f},
                               {2, 4, 0.62f, 0.40f, 0.89f, 0.48f}, {2, 2, 0.41f, 0.30f, 0.44f, 0.25f}, {2, 1, 0.37f, 0.37f, 0.26f, 0.175f},
                               // row-block code 8: one row block with the K range over EIGHT teams, for matrices of few row
                               // blocks and long rows (4096x14336 at 16 requests: 30 -> 20 us)
                               {1, 8, 0.25f, 0.22f, 0.172f, 0.115f}, {2, 8, 0.30f, 0.29f, 0.30f, 0.28f},
                               {4, 4, 0.82f, 0.54f, 0.f, 0.f},     {4, 2, 0.52f, 0.36f, 0.f, 0.f},      {4, 1, 0.45f, 0.37f, 0.f, 0.f},
                               {8, 4, 1.10f, 0.80f, 0.f, 0.f},     {8, 2, 0.85f, 0.70f, 0.f, 0.f},      {16, 4, 2.10f, 1.75f, 0.f, 0.f},
                               // 256 requests with EIGHT waves on the tile instead of four (two per SIMD: one computes while the
                               // other waits for its operands).  Code 40: 64 rows, two teams that share the tiles and split the
                               // matrix sub-steps of every group (14336x4096 at 256 requests: 68 -> 57 us); code 8: 128 rows, one
                               // wave per 16 rows, for matrices that still fill the chip then (28672x8192: 254 -> 191 us).
                               {16, 40, 1.78f, 1.49f, 0.f, 0.f},   {16, 8, 2.95f, 2.42f, 0.f, 0.f},
                               // (128 requests and 128 rows the same way: 28672x8192 at 128 requests 139 -> 129 us)
                               {8, 8, 2.01f, 1.48f, 0.f, 0.f}};

// the cheapest shape for `batch` requests at precision p, among the shapes of at least min_nt tiles; `times`: that
// many such problems in one launch
void cheapest_shape(int p, int64_t m, int batch, int min_nt, int &nt, int &rw, int times = 1)
{
    nt = rw = 4;
    float best = 0.f;
    for (const WgShape &c : kShapes) {
        if (c.nt < min_nt || (c.nt <= 2 && batch > 16 * c.nt)) continue;
        const int blocks = row_blocks_of(c.nt, c.rw);
        const float wgs = (float)((m + 16 * blocks - 1) / (16 * blocks)) * (float)((batch + 16 * c.nt - 1) / (16 * c.nt)) * (float)times;
        const float one = p >= 3 ? c.us_p4 : c.us_p2, many = p >= 3 ? c.many_p4 : c.many_p2;
        float cost = one;
        if (many > 0.f) cost = wgs / 256.f * many > one ? wgs / 256.f * many : one;
        else if (wgs > 256.f) cost = __builtin_ceilf(wgs / 256.f) * one;
        if (best == 0.f || cost < best) {
            best = cost;
            nt = c.nt;
            rw = c.rw;
        }
    }
}

// A batch with per-request precision beyond 64 requests: the uniform kernel's body on the requests of each
// precision.  How many a precision has only the GPU knows; the shape is chosen for `expected` of them at the
// deepest precision and the grid for all of the batch at every precision.
hipError_t launch_classes(const DequantParams &pr, const GemmArgs &a, int expected, int nsets, int p_deepest, hipStream_t stream)
{
    int nt, rw;
    cheapest_shape(p_deepest, a.m, expected, 4, nt, rw, nsets);
    if (g_forced_nt >= 4) {
        nt = g_forced_nt;
        rw = g_forced_rw;
    }
    switch (nt * 10 + rw) {
    case 44: return launch_byclass<4, 4, 4>(pr, a, stream);
    case 42: return launch_byclass<4, 4, 2>(pr, a, stream);
    case 41: return launch_byclass<4, 4, 1>(pr, a, stream);
    case 84: return launch_byclass<8, 2, 4>(pr, a, stream);
    case 82: return launch_byclass<8, 2, 2>(pr, a, stream);
    case 164: return launch_byclass<16, 1, 4>(pr, a, stream);
    case 168: return launch_byclass<16, 1, 8>(pr, a, stream);
    case 88: return launch_byclass<8, 1, 8>(pr, a, stream);
    case 200: return launch_byclass<16, 2, 4, true>(pr, a, stream);
    default: return hipErrorInvalidValue;
    }
}

template <int P, bool PW>
hipError_t launch_p(const DequantParams &pr, const GemmArgs &a, hipStream_t stream)
{
    int nt, rw;
    cheapest_shape(P, a.m, a.batch, 1, nt, rw);
    if (g_forced_nt > 0) {
        nt = g_forced_nt;
        rw = g_forced_rw;
    }
    switch (nt * 10 + rw) {
    case 18: return launch_one<P, 1, 8, 1, PW>(pr, a, stream);      // (row-block code 8: one block, the K range over eight teams)
    case 28: return launch_one<P, 2, 8, 1, PW>(pr, a, stream);
    case 14: return launch_one<P, 1, 4, 4, PW>(pr, a, stream);
    case 12: return launch_one<P, 1, 4, 2, PW>(pr, a, stream);
    case 11: return launch_one<P, 1, 4, 1, PW>(pr, a, stream);
    case 24: return launch_one<P, 2, 4, 4, PW>(pr, a, stream);
    case 22: return launch_one<P, 2, 4, 2, PW>(pr, a, stream);
    case 21: return launch_one<P, 2, 4, 1, PW>(pr, a, stream);
    case 44: return launch_one<P, 4, 4, 4, PW>(pr, a, stream);
    case 42: return launch_one<P, 4, 4, 2, PW>(pr, a, stream);
    case 41: return launch_one<P, 4, 4, 1, PW>(pr, a, stream);
    case 84: return launch_one<P, 8, 2, 4, PW>(pr, a, stream);
    case 82: return launch_one<P, 8, 2, 2, PW>(pr, a, stream);
    case 164: return launch_one<P, 16, 1, 4, PW>(pr, a, stream);
    case 168: return launch_one<P, 16, 1, 8, PW>(pr, a, stream);
    case 88: return launch_one<P, 8, 1, 8, PW>(pr, a, stream);
    case 200:       // (16 tiles, code 40: two teams on shared tiles)
        if constexpr (!PW) return launch_one<P, 16, 2, 4, false, true>(pr, a, stream);
        else return launch_one<P, 16, 1, 4, true>(pr, a, stream);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace

// request_tiles: 1, 2 or 4 tiles of 64 requests, or 0 (with row_blocks != 0) for a single tile of 16 requests
bool dequant_mfma_force_shape(int request_tiles, int row_blocks)
{
    if (request_tiles == 0 && row_blocks == 0) {
        g_forced_nt = g_forced_rw = 0;
        return true;
    }
    const int nt = request_tiles == 0 ? 1 : request_tiles == 32 ? 2 : 4 * request_tiles;      // 32: a tile of 32 requests
    const int key = nt * 10 + row_blocks;
    const bool known = key == 14 || key == 12 || key == 11 || key == 24 || key == 22 || key == 21 || key == 44 || key == 42 || key == 41 ||
                       key == 84 || key == 82 || key == 164 || key == 18 || key == 28 || key == 168 || key == 200 || key == 88;
    if (!known || request_tiles < 0 || (row_blocks != 1 && row_blocks != 2 && row_blocks != 4 && row_blocks != 8 && row_blocks != 40)) return false;
    g_forced_nt = nt;
    g_forced_rw = row_blocks;
    return true;
}

bool dequant_mfma_supports(const GemmArgs &a)
{
    // 32-bit byte offsets inside one plane / one scale plane / the activation matrix
    const bool small_enough = a.m * (a.n / 8) < (int64_t(1) << 31) && (int64_t)a.batch * a.n * 2 < (int64_t(1) << 31);
    const bool group_ok = (a.group == 64 || a.group == 128 || a.group == 256) && (a.n % 128) == 0;
    // one precision for all requests, or one per request with planes stored to at most four
    const bool p_ok = a.uniform_p > 0 ? a.uniform_p <= kMaxP : (a.p_req != nullptr && a.p_max >= 1 && a.p_max <= kMaxP);
    return p_ok && group_ok && small_enough && (a.batch + 15) / 16 <= 65535 && (a.m + 15) / 16 < (int64_t(1) << 31);
}

// Several matrices (same n, precision, batch, activations and group size, no offsets) as one launch: the grid's rows of
// workgroups are the concatenation of theirs, the shape is chosen for the sum of their rows.
bool dequant_mfma_supports_multi(const GemmArgs *mats, int count)
{
    if (count < 2 || count > BCQ_MAX_MULTI) return false;
    int64_t rows = 0;
    for (int k = 0; k < count; ++k) {
        const GemmArgs &a = mats[k];
        if (!dequant_mfma_supports(a) || a.uniform_p < 1 || a.offsets[a.uniform_p]) return false;
        if (a.n != mats[0].n || a.uniform_p != mats[0].uniform_p || a.batch != mats[0].batch || a.x != mats[0].x || a.group != mats[0].group)
            return false;
        rows += a.m;
    }
    return (rows + 15) / 16 + count < (int64_t(1) << 31);
}

hipError_t dequant_mfma_launch_multi(const GemmArgs *mats, int count, hipStream_t stream, bool planewise)
{
    GemmArgs all = mats[0];
    all.m = 0;
    for (int k = 0; k < count; ++k) all.m += mats[k].m;
    return dequant_mfma_launch(all, stream, planewise, mats, count);
}

hipError_t dequant_mfma_launch(const GemmArgs &a, hipStream_t stream, bool planewise, const GemmArgs *mats, int count)
{
    DequantParams pr{};
    pr.planes = reinterpret_cast<const unsigned char *>(a.planes);
    pr.x = reinterpret_cast<const unsigned char *>(a.x);
    pr.y = a.y;
    pr.plane_stride = (uint32_t)(a.m * (a.n / 8));
    pr.row_stride = (uint32_t)(a.n / 8);
    pr.scale_plane_stride = (uint32_t)(a.m * (a.n / a.group) * 2);
    pr.scale_row_stride = (uint32_t)((a.n / a.group) * 2);
    pr.gshift = a.group == 256 ? 1 : a.group == 64 ? -1 : 0;
    pr.x_stride = (uint32_t)(a.n * 2);
    pr.m = (uint32_t)a.m;
    pr.batch = a.batch;
    pr.ngroups = (int)(a.n / 128);
    if (a.uniform_p == 0) {
        // per-request precision: 64 requests per workgroup, 32 or 16 rows (four accumulator sets need the registers)
        for (int q = 1; q <= kMaxP; ++q) {
            pr.scale_sets[q] = reinterpret_cast<const unsigned char *>(a.scales[q]);
            pr.offset_sets[q] = a.scales[q] ? reinterpret_cast<const unsigned char *>(a.offsets[q]) : nullptr;
        }
        pr.p_req = a.p_req;
        pr.p_max = a.p_max;
        if (planewise) {
            // tiles of 16 requests, row blocks by the cost rule of the 16-request shapes
            const float tiles16 = (float)((a.batch + 15) / 16);
            int rw16 = 4;
            float best16 = 0.f;
            for (const WgShape &c : kShapes) {
                if (c.nt != 1) continue;
                const int blocks = c.rw == 8 ? 1 : c.rw;        // (code 8: one row block, eight teams)
                const float wgs = (float)((a.m + 16 * blocks - 1) / (16 * blocks)) * tiles16;
                const float cost = wgs / 256.f * c.many_p4 > c.us_p4 ? wgs / 256.f * c.many_p4 : c.us_p4;
                if (best16 == 0.f || cost < best16) {
                    best16 = cost;
                    rw16 = c.rw;
                }
            }
            // (workgroups of 64 requests were measured too: 1.5-3x slower than four workgroups of 16)
            // beyond 16 requests tiles of 32 (16 rows per workgroup, 32 on the tallest matrices): 14336x4096 at 32 requests
            // 42 -> 33 us
            bool pairs = a.batch > 16;
            if (pairs) rw16 = a.m >= 16384 ? 2 : a.m * ((a.batch + 31) / 32) <= 4096 ? 8 : 1;     // eight teams while the grid is small
            if (g_forced_nt > 0) {
                rw16 = g_forced_rw;
                pairs = g_forced_nt == 2;
            }
            if (pairs)      // (with 64 rows per workgroup such a tile would not fit the registers of sixteen waves)
                return rw16 == 8 ? launch_planewise_mixed<2, 8, 1>(pr, a, stream)
                     : rw16 >= 2 ? launch_planewise_mixed<2, 4, 2>(pr, a, stream) : launch_planewise_mixed<2, 4, 1>(pr, a, stream);
            return rw16 == 8 ? launch_planewise_mixed<1, 8, 1>(pr, a, stream)
                 : rw16 == 4 ? launch_planewise_mixed<1, 4, 4>(pr, a, stream)
                 : rw16 == 2 ? launch_planewise_mixed<1, 4, 2>(pr, a, stream) : launch_planewise_mixed<1, 4, 1>(pr, a, stream);
        }
        if (a.batch > kClassFrom && (g_forced_nt == 0 || g_forced_nt >= 4)) {
            // Beyond 64 requests: the uniform kernel's body per precision, each on the requests of that precision
            // wherever they sit in the batch (dequant_byclass_kernel).  A weight is then rebuilt once per
            // precision and up to 256 requests, at the cost of that precision alone, instead of once per 64
            // requests at the cost of all precisions present.
            int nsets = 0, y = 0;
            pr.class_order = 0;
            for (int q = a.p_max; q >= 1; --q)
                if (a.scales[q]) {
                    ++nsets;
                    pr.class_order |= (uint32_t)q << (8 * y++);
                }
            for (int q = a.p_max; q >= 1; --q)
                if (!a.scales[q]) pr.class_order |= (uint32_t)q << (8 * y++);
            // an even split plus 1.3 standard deviations of a uniform draw: a precision that gets a few requests more
            // than its share should not need a second, nearly empty tile (which costs as much as a full one)
            const float share = nsets ? (float)a.batch / (float)nsets : (float)a.batch;
            const int expected = (int)__builtin_ceilf(share + 1.3f * __builtin_sqrtf(share * (float)(nsets > 1 ? nsets - 1 : 0) / (float)(nsets ? nsets : 1)));
            int deepest = 1;
            for (int q = 1; q <= a.p_max; ++q)
                if (a.scales[q]) deepest = q;
            return launch_classes(pr, a, expected, nsets, deepest, stream);
        }
        // 64, 32 or 16 rows per workgroup by the same two-factor cost as the uniform kernel (measured with three
        // precisions present: 1.8, 1.43 and 0.94 microseconds per workgroup and group of columns; two of the
        // 32-row workgroups fit a CU side by side, which is worth about 40 % once there are that many)
        const float tiles = (float)((a.batch + 63) / 64);
        int rw = 4;
        float best = 0.f;
        for (int r = 4; r >= 1; r >>= 1) {
            const float wgs = (float)((a.m + 16 * r - 1) / (16 * r)) * tiles;
            const float rounds = wgs <= 256.f ? 1.f : (r == 2 ? 0.6f : 1.f) * wgs / 256.f;
            const float cost = rounds * (r == 4 ? 1.8f : r == 2 ? 1.43f : 0.94f);
            if (best == 0.f || cost < best) {
                best = cost;
                rw = r;
            }
        }
        if (g_forced_nt > 0) rw = g_forced_rw;
        return rw == 4 ? launch_mixed<2, 4>(pr, a, stream) : rw == 2 ? launch_mixed<2, 2>(pr, a, stream) : launch_mixed<4, 1>(pr, a, stream);
    }
    if (mats && count > 1) {
        // (a: the matrices taken together, for the choice of the shape; each keeps its own rows, planes, scales and results)
        pr.nmat = count;
        for (int k = 0; k < count; ++k) {
            pr.mat_planes[k] = reinterpret_cast<const unsigned char *>(mats[k].planes);
            pr.mat_scales[k] = reinterpret_cast<const unsigned char *>(mats[k].scales[a.uniform_p]);
            pr.mat_y[k] = mats[k].y;
            pr.mat_m[k] = (uint32_t)mats[k].m;
        }
    }
    pr.scales = reinterpret_cast<const unsigned char *>(a.scales[a.uniform_p]);
    pr.has_offsets = a.offsets[a.uniform_p] != nullptr;
    pr.offsets = pr.has_offsets ? reinterpret_cast<const unsigned char *>(a.offsets[a.uniform_p]) : pr.scales;
    if (planewise) {
        switch (a.uniform_p) {
        case 1: return launch_p<1, true>(pr, a, stream);
        case 2: return launch_p<2, true>(pr, a, stream);
        case 3: return launch_p<3, true>(pr, a, stream);
        default: return launch_p<4, true>(pr, a, stream);
        }
    }
    switch (a.uniform_p) {
    case 1: return launch_p<1, false>(pr, a, stream);
    case 2: return launch_p<2, false>(pr, a, stream);
    case 3: return launch_p<3, false>(pr, a, stream);
    default: return launch_p<4, false>(pr, a, stream);
    }
}

}  // namespace bcq
