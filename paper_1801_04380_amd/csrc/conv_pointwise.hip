// 1x1 / stride-1 / unpadded CONV forward and backward-data on gfx950, bf16 operands
// (Sec. 3.5 of the paper: needs no workspace at all, so it serves DIRECT and STAGED alike;
// definitions in sn.h).
//
// Without taps the layer is a matrix product per image,
//     Y[n][m][px] = sum_r A[m][r] * X[n][r][px],
// forward with A = w[K][C] (m = k, r = c), backward-data with A = w transposed (m = c, r = k).
// At 50-200 FLOP per byte these layers sit under the HBM roof, and on small images they are a few
// microseconds of work: what counts is that every byte is asked for once, early, by many waves.
//
//  * NCHW has the pixels of a channel contiguous, the MFMA wants 8 reduction channels of one pixel
//    per lane.  No transposition is needed for that: a lane loads its pixel (pair) from 8 channel
//    rows with 8 loads whose addresses differ by a uniform row pitch -- a per-lane constant offset
//    plus a scalar offset -- and packs halves of the 8 registers into the operand.  With an even
//    plane size a lane takes two neighbouring pixels per load (4 bytes); the even pixels form one
//    32-column operand, the odd ones a second, and the epilogue finds both pixels of the pair in the
//    same lane again and stores them with one 4-byte store.  Odd plane sizes use 2-byte accesses.
//    The pixel index runs over the whole batch (n * HW + px), so a tile may span images and only
//    the last tile of the tensor is ragged.
//  * A is the operand all waves of a workgroup share: 64 reduction channels of it at a time are
//    staged in LDS (double buffered, one barrier per stage).  Forward reads its operands from there
//    with 16-byte reads; backward-data parks the rows of w as they are and reads them through the
//    transposing LDS read (ds_read_b64_tr_b16).
//  * X loads run three 16-channel steps ahead of the MFMAs, in registers (four rotating sets).
//  * SPLIT (few pixels, long reductions: 7x7 and 14x14 images under 1024 or 2048 channels): the four
//    waves of a workgroup share 64 pixels and each takes every fourth pair of 16-channel steps;
//    their accumulators are added through LDS in a fixed order.  Four times the waves per pixel,
//    each with a quarter of the serial chain of loads and MFMAs.
//  * Workgroups are numbered so that the output-channel tiles of one pixel tile run on the same
//    XCD one after the other: X comes from HBM once and from that XCD's L2 afterwards.
#include <algorithm>
#include "sn_internal.h"

namespace sn {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

constexpr uint32_t OUTSIDE = 0x80000000u;   // an offset past any tensor this kernel accepts: loads bring zeros, stores are dropped
constexpr int RG = 64;                      // reduction channels per LDS stage of A (SPLIT: 128, 32 per wave)

struct PwProblem {
    int M, Rd, HW;
    uint32_t npx;            // N * HW
    int mtiles, ptiles;
    int out_bf16;
    uint32_t x_bytes, a_bytes, y_bytes;
    int niter;               // main-loop trips: four 16-channel steps per wave each
    // CONV (forward of any filter, stride and padding as a matrix product over (tap, channel)): HW is the output
    // plane P * Q, Rd = R * S * C, and the input is [N][C][Hin][Win]
    int C, Hin, Win, Q, R, S, sh, sw, ph, pw;
    int spt;                 // 16-channel steps per tap: C / 16
    // backward-data of a 1x1 / stride-2 layer: pixel (p, q) of the HW = P * Q plane goes to (2p, 2q) of the
    // Hd x Wd plane of dx, and the other three pixels of its 2 x 2 cell are written as zeros
    int scat, Hd, Wd, Qd;
};

__device__ inline uint32_t pack2(float a, float b)   // two fp32 -> two bf16, round to nearest even, a in the low half
{
    f32x2 f = {a, b};
    bf16x2 h = __builtin_convertvector(f, bf16x2);
    uint32_t r;
    __builtin_memcpy(&r, &h, 4);
    return r;
}

// MS: 32-row blocks of output channels per workgroup; NW: waves per workgroup, 64 pixels each, or
// with SPLIT a share of the reduction each; AT: A[m][r] = w[r][m] (backward-data); PAIR: plane size
// even, a lane owns two neighbouring pixels.
// CONV: forward of a filter with taps, strides and padding by the same means.  The reduction runs over
// (tap, channel) with the channel innermost, A is the filter re-laid out [k][tap][c] (in the caller's
// workspace), and a lane's 8 loads of a step are the 8 channels of ITS input pixel under the step's tap:
// the per-lane offset is that of the window's first pixel plus the tap's (uniform) offset, or out of
// range where the tap falls into the padding.  No phase planes, no unfolded copy.
template <int MS, int NW, bool SPLIT, bool AT, bool PAIR, bool CONV = false>
__global__ void __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(2, 2)))
pointwise_kernel(const bf16_t *__restrict__ x, const bf16_t *__restrict__ a, void *__restrict__ y, PwProblem p)
{
    static_assert(!SPLIT || (NW == 4 && MS == 2), "the split form: four waves, 64 output channels");
    static_assert(!CONV || (!SPLIT && !AT && !PAIR), "the general forward form: single pixels, whole reduction per wave");
    constexpr int MT = 32 * MS, NT = 64 * NW;
    constexpr int RGS = SPLIT ? 2 * RG : RG;                 // reduction channels per stage
    constexpr int SPG = SPLIT ? 2 : 4;                       // 16-channel steps per wave and stage
    constexpr int GPI = 4 / SPG;                             // stages per main-loop trip
    constexpr int APITCH = AT ? 2 * MT + 64 : 2 * RGS + 16;  // bytes per LDS row (AT: a reduction channel, else an output channel)
    constexpr int AROWS = AT ? RGS : MT;
    constexpr int ABUF = AROWS * APITCH;
    constexpr int IPR = AT ? MT / 8 : RGS / 8;               // 16-byte items per row
    constexpr int AIT = AROWS * IPR / NT;                    // items per thread and stage
    constexpr int NX = PAIR ? 8 : 16;                        // registers of one X set
    static_assert(AROWS * IPR % NT == 0, "stage does not divide over the threads");
    static_assert(!SPLIT || 2 * ABUF >= 4 * 32 * 64 * 4, "the accumulators of one 32-row block of four waves fit the A buffers");
    __shared__ __attribute__((aligned(16))) char lds[2 * ABUF];

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, g = lane >> 5;

    // ---- which tile: the workgroups of an XCD (every eighth) walk the channel tiles of one pixel tile first
    const int id = blockIdx.x, xcd = id & 7, slot = id >> 3;
    const int ptile = (slot / p.mtiles) * 8 + xcd, mtile = slot % p.mtiles;
    if (ptile >= p.ptiles) return;
    const int m0 = mtile * MT;
    const uint32_t px0 = SPLIT ? (uint32_t)ptile * 64 : (uint32_t)ptile * (64 * NW) + wave * 64;

    const __amdgpu_buffer_rsrc_t xr = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(x), 0, p.x_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t ar = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(a), 0, p.a_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t yr = __builtin_amdgcn_make_buffer_rsrc(y, 0, p.y_bytes, 0x00020000);

    // ---- per-lane constants: where the lane's pixel (pair) sits in X and in Y, channel 8g / 4g of its image
    constexpr int NCOL = PAIR ? 1 : 2;
    const uint32_t esz = p.out_bf16 ? 2 : 4;
    uint32_t xlane[NCOL], ylane[NCOL];
    int ih0[NCOL], iw0[NCOL];   // CONV: the input row and column under the window's first tap
    bool okj[NCOL];
#pragma unroll
    for (int e = 0; e < NCOL; ++e) {
        const uint32_t j = PAIR ? px0 + 2 * l32 : px0 + 32 * e + l32;
        const uint32_t n = j / (uint32_t)p.HW, pp = j - n * p.HW;
        const bool ok = j < p.npx;
        okj[e] = ok;
        if (CONV) {
            const int po = (int)pp / p.Q, qo = (int)pp - po * p.Q;
            ih0[e] = po * p.sh - p.ph;
            iw0[e] = qo * p.sw - p.pw;
            // (wraps where the window starts in the padding; the taps inside the image add up to a proper offset)
            xlane[e] = (uint32_t)((((int)n * p.C + 8 * g) * p.Hin + ih0[e]) * p.Win + iw0[e]) * 2u;
        } else {
            ih0[e] = iw0[e] = 0;
            xlane[e] = ok ? ((n * p.Rd + 8 * g) * p.HW + pp) * 2 : OUTSIDE;
        }
        ylane[e] = ok ? ((n * p.M + 4 * g) * p.HW + pp) * esz : OUTSIDE;
        if (!CONV && p.scat && ok) {
            const uint32_t po = pp / (uint32_t)p.Qd, qo = pp - po * p.Qd;
            ylane[e] = (((n * p.M + 4 * g) * p.Hd + 2 * po) * p.Wd + 2 * qo) * esz;
        }
    }
    const uint32_t xrow = CONV ? (uint32_t)p.Hin * p.Win * 2 : (uint32_t)p.HW * 2;   // bytes between channels of X

    // ---- per-thread constants of the A stage
    uint32_t asrc[AIT], adst[AIT];
    int alim[AIT];   // the item is inside A while group * RG < alim
#pragma unroll
    for (int k = 0; k < AIT; ++k) {
        const int it = tid + NT * k, row = it / IPR, col = it - row * IPR;
        if (AT) {   // row = reduction channel of the group, col = 8 output channels
            const bool ok = m0 + col * 8 < p.M;
            asrc[k] = ok ? (uint32_t)(row * p.M + m0 + col * 8) * 2 : OUTSIDE;
            alim[k] = p.Rd - row;
        } else {    // row = output channel of the tile, col = 8 reduction channels
            const bool ok = m0 + row < p.M;
            asrc[k] = ok ? (uint32_t)((m0 + row) * p.Rd + col * 8) * 2 : OUTSIDE;
            alim[k] = p.Rd - col * 8;
        }
        adst[k] = row * APITCH + col * 16;
    }
    const uint32_t agroup = AT ? (uint32_t)RGS * p.M * 2 : RGS * 2;   // bytes from a stage to the next

    u32x4 areg[AIT];
    auto a_issue = [&](int grp) {
#pragma unroll
        for (int k = 0; k < AIT; ++k)
            areg[k] = __builtin_amdgcn_raw_buffer_load_b128(ar, grp * RGS < alim[k] ? asrc[k] : OUTSIDE, grp * agroup, 0);
    };
    auto a_store = [&](int buf) {
#pragma unroll
        for (int k = 0; k < AIT; ++k) *reinterpret_cast<u32x4 *>(lds + buf * ABUF + adst[k]) = areg[k];
    };

    uint32_t xraw[4][NX];
    // the q-th step of this wave is 16-channel step q, or with SPLIT step 2 * wave + q % 2 of stage q / 2
    int tap_r = 0, tap_s = 0, tap_c = 0;   // CONV: the tap and the 16-channel step within it of the next x_issue (called in step order)
    const int conv_steps = CONV ? p.R * p.S * p.spt : 0;
    auto x_issue = [&](int q, uint32_t (&dst)[NX]) {
        const int c = SPLIT ? (q >> 1) * 8 + 2 * wave + (q & 1) : q;
        const bool rows_ok = c * 16 + 8 * g < p.Rd;     // Rd is a multiple of 8: a lane's 8 rows are in or out together
        const uint32_t sb = CONV ? (uint32_t)tap_c * 16 * xrow : (uint32_t)c * 16 * xrow;
        const uint32_t tapoff = CONV ? (uint32_t)((tap_r * p.Win + tap_s) * 2) : 0u;
#pragma unroll
        for (int e = 0; e < NCOL; ++e) {
            uint32_t v;
            if (CONV) {
                const bool in = okj[e] && q < conv_steps && (unsigned)(ih0[e] + tap_r) < (unsigned)p.Hin &&
                                (unsigned)(iw0[e] + tap_s) < (unsigned)p.Win;
                v = in ? xlane[e] + tapoff : OUTSIDE;
            } else {
                v = rows_ok ? xlane[e] : OUTSIDE;
            }
#pragma unroll
            for (int jj = 0; jj < 8; ++jj) {
                if (PAIR) dst[jj] = __builtin_amdgcn_raw_buffer_load_b32(xr, v, sb + jj * xrow, 0);
                else dst[e * 8 + jj] = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(xr, v, sb + jj * xrow, 0);
            }
        }
        if (CONV && ++tap_c == p.spt) {
            tap_c = 0;
            if (++tap_s == p.S) { tap_s = 0; ++tap_r; }
        }
    };

    // ---- per-lane constants of the A operand reads (SPLIT: the wave's two steps of the stage)
    uint32_t aread;
    if (AT) {
        const int i16 = lane & 15, half = (lane >> 4) & 1;
        aread = (8 * g + (i16 >> 2)) * APITCH + (16 * half + 4 * (i16 & 3)) * 2;
        if (SPLIT) aread += wave * SPG * 16 * APITCH;
    } else {
        aread = l32 * APITCH + 8 * g * 2;
        if (SPLIT) aread += wave * SPG * 32;
    }

    f32x16 acc[MS][2];
#pragma unroll
    for (int i = 0; i < MS; ++i)
#pragma unroll
        for (int e = 0; e < 2; ++e)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][e][v] = 0.f;

    // ---- prologue: group 0 of A into LDS, three steps of X on their way
    a_issue(0);
    __builtin_amdgcn_sched_barrier(0);   // in this order: the loop's waits count on it
    x_issue(0, xraw[0]);
    __builtin_amdgcn_sched_barrier(0);
    x_issue(1, xraw[1]);
    __builtin_amdgcn_sched_barrier(0);
    x_issue(2, xraw[2]);
    __builtin_amdgcn_sched_barrier(0);
    a_store(0);
    __syncthreads();

    for (int it = 0; it < p.niter; ++it) {
#pragma unroll
        for (int h = 0; h < GPI; ++h) {
            const int grp = it * GPI + h;
            a_issue(grp + 1);   // past the last stage: zeros
            __builtin_amdgcn_sched_barrier(0);
            const char *ab = lds + (grp & 1) * ABUF;
#pragma unroll
            for (int s = 0; s < SPG; ++s) {
                const int qs = h * SPG + s;   // 0 .. 3: the register set
                x_issue(it * 4 + qs + 3, xraw[(qs + 3) & 3]);
                __builtin_amdgcn_sched_barrier(0);   // the loads go out here, three steps ahead, not where the scheduler likes them
                const uint32_t(&xs)[NX] = xraw[qs];
                bf16x8 b[2];
                {
                    u32x4 d0, d1;
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        if (PAIR) {   // low halves: the even pixel, high halves: the odd one
                            d0[t] = __builtin_amdgcn_perm(xs[2 * t + 1], xs[2 * t], 0x05040100u);
                            d1[t] = __builtin_amdgcn_perm(xs[2 * t + 1], xs[2 * t], 0x07060302u);
                        } else {
                            d0[t] = xs[2 * t] | xs[2 * t + 1] << 16;
                            d1[t] = xs[8 + 2 * t] | xs[8 + 2 * t + 1] << 16;
                        }
                    }
                    __builtin_memcpy(&b[0], &d0, 16);
                    __builtin_memcpy(&b[1], &d1, 16);
                }
                bf16x8 aop[MS];
#pragma unroll
                for (int i = 0; i < MS; ++i) {
                    if (AT) {
                        const char *q = ab + aread + s * 16 * APITCH + i * 64;
                        s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)q);
                        s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(q + 4 * APITCH));
                        u32x2 l2, h2;
                        __builtin_memcpy(&l2, &lo, 8);
                        __builtin_memcpy(&h2, &hi, 8);
                        u32x4 d = {l2[0], l2[1], h2[0], h2[1]};
                        __builtin_memcpy(&aop[i], &d, 16);
                    } else {
                        u32x4 d = *reinterpret_cast<const u32x4 *>(ab + aread + i * 32 * APITCH + s * 32);
                        __builtin_memcpy(&aop[i], &d, 16);
                    }
                }
#pragma unroll
                for (int i = 0; i < MS; ++i)
#pragma unroll
                    for (int e = 0; e < 2; ++e)
                        acc[i][e] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aop[i], b[e], acc[i][e], 0, 0, 0);
            }
            a_store((grp + 1) & 1);
            __syncthreads();
        }
    }

    // ---- epilogue: register v of a lane is output channel 8*(v/4) + 4*g + v%4 of its 32-row block
    const uint32_t yrow = (!CONV && p.scat) ? (uint32_t)p.Hd * p.Wd * esz : (uint32_t)p.HW * esz;
    // row mu + 4*g + vv of the output for the lane's pixel pair (v0: even pixel or column group 0)
    auto store_row = [&](int mu, int vv, float v0, float v1) {
        const uint32_t sb = (uint32_t)(mu + vv) * yrow;
        if (!CONV && p.scat) {   // every pixel with a zero to its right, and a row of zeros below
            const uint32_t below = (uint32_t)p.Wd * esz;
            if (PAIR) {
                if (p.out_bf16) {
                    const u32x2 d = {pack2(v0, 0.f), pack2(v1, 0.f)}, z = {0u, 0u};
                    __builtin_amdgcn_raw_buffer_store_b64(d, yr, ylane[0], sb, 0);
                    __builtin_amdgcn_raw_buffer_store_b64(z, yr, ylane[0], sb + below, 0);
                } else {
                    const u32x4 d = {__float_as_uint(v0), 0u, __float_as_uint(v1), 0u}, z = {0u, 0u, 0u, 0u};
                    __builtin_amdgcn_raw_buffer_store_b128(d, yr, ylane[0], sb, 0);
                    __builtin_amdgcn_raw_buffer_store_b128(z, yr, ylane[0], sb + below, 0);
                }
            } else {
                const float vals[2] = {v0, v1};
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    if (p.out_bf16) {
                        __builtin_amdgcn_raw_buffer_store_b32(pack2(vals[e], 0.f), yr, ylane[PAIR ? 0 : e], sb, 0);
                        __builtin_amdgcn_raw_buffer_store_b32(0u, yr, ylane[PAIR ? 0 : e], sb + below, 0);
                    } else {
                        const u32x2 d = {__float_as_uint(vals[e]), 0u}, z = {0u, 0u};
                        __builtin_amdgcn_raw_buffer_store_b64(d, yr, ylane[PAIR ? 0 : e], sb, 0);
                        __builtin_amdgcn_raw_buffer_store_b64(z, yr, ylane[PAIR ? 0 : e], sb + below, 0);
                    }
                }
            }
            return;
        }
        if (PAIR) {
            if (p.out_bf16) {
                __builtin_amdgcn_raw_buffer_store_b32(pack2(v0, v1), yr, ylane[0], sb, 0);
            } else {
                u32x2 d = {__float_as_uint(v0), __float_as_uint(v1)};
                __builtin_amdgcn_raw_buffer_store_b64(d, yr, ylane[0], sb, 0);
            }
        } else {
            const float vals[2] = {v0, v1};
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                if (p.out_bf16) __builtin_amdgcn_raw_buffer_store_b16((uint16_t)pack2(vals[e], 0.f), yr, ylane[PAIR ? 0 : e], sb, 0);
                else __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(vals[e]), yr, ylane[PAIR ? 0 : e], sb, 0);
            }
        }
    };
    if (SPLIT) {
        // the four waves hold partial sums of the same 64 x 64 block: per 32-row block, every wave parks its
        // 32 registers in LDS ([wave][e][v][lane]) and wave w then adds up and stores rows 8*w .. 8*w+7
        float *red = reinterpret_cast<float *>(lds);
#pragma unroll
        for (int i = 0; i < MS; ++i) {
            // the main loop ended with a barrier: nobody reads the A buffers any more
#pragma unroll
            for (int e = 0; e < 2; ++e)
#pragma unroll
                for (int v = 0; v < 16; ++v) red[((wave * 2 + e) * 16 + v) * 64 + lane] = acc[i][e][v];
            __syncthreads();
            const int mu = m0 + 32 * i + 8 * wave;
            if (mu < p.M) {
#pragma unroll
                for (int vv = 0; vv < 4; ++vv) {
                    float sum[2];
#pragma unroll
                    for (int e = 0; e < 2; ++e) {
                        sum[e] = red[((0 * 2 + e) * 16 + 4 * wave + vv) * 64 + lane];
#pragma unroll
                        for (int w2 = 1; w2 < 4; ++w2) sum[e] += red[((w2 * 2 + e) * 16 + 4 * wave + vv) * 64 + lane];
                    }
                    store_row(mu, vv, sum[0], sum[1]);
                }
            }
            __syncthreads();
        }
    } else {
#pragma unroll
        for (int i = 0; i < MS; ++i) {
#pragma unroll
            for (int vb = 0; vb < 4; ++vb) {
                const int mu = m0 + 32 * i + 8 * vb;   // M is a multiple of 8: the 8 rows of a block are in or out together
                if (mu < p.M) {
#pragma unroll
                    for (int vv = 0; vv < 4; ++vv) store_row(mu, vv, acc[i][0][4 * vb + vv], acc[i][1][4 * vb + vv]);
                }
            }
        }
    }
}

struct PwPlan {
    PwProblem p;
    int MS, NW;
    bool split, at, pair;
    unsigned grid;
};

bool make_plan(const ConvGeom &g, bool bwd_data, PwPlan *pl)
{
    if (!g.in_bf16 || g.R != 1 || g.S != 1 || g.ph != 0 || g.pw != 0) return false;
    // stride 1; or backward-data of stride 2 on planes of even size (whole 2 x 2 cells)
    const bool scat = bwd_data && g.sh == 2 && g.sw == 2 && g.H % 2 == 0 && g.W % 2 == 0 && g.P == g.H / 2 && g.Q == g.W / 2;
    if (!scat && (g.sh != 1 || g.sw != 1 || g.P != g.H || g.Q != g.W)) return false;
    if (g.C % 8 != 0 || g.K % 8 != 0) return false;
    const long long HW = (long long)g.P * g.Q, npx = HW * g.N;
    const long long M = bwd_data ? g.C : g.K, Rd = bwd_data ? g.K : g.C;
    const long long lim = 0x7fffffffLL - (1 << 20);
    if (npx * Rd * 2 > lim || npx * M * (g.out_bf16 ? 2 : 4) > lim || (long long)g.K * g.C * 2 > lim) return false;
    if (16 * HW * 2 * 4 > lim) return false;   // the scalar offset of a 16-channel step stays small next to the tensor
    PwProblem &p = pl->p;
    p.M = (int)M; p.Rd = (int)Rd; p.HW = (int)HW; p.npx = (uint32_t)npx;
    p.out_bf16 = g.out_bf16;
    p.x_bytes = (uint32_t)(npx * Rd * 2);
    p.y_bytes = (uint32_t)(npx * M * (g.out_bf16 ? 2 : 4));
    p.scat = scat; p.Hd = g.H; p.Wd = g.W; p.Qd = g.Q;
    if (scat) {
        const long long yb = (long long)g.N * g.C * g.H * g.W * (g.out_bf16 ? 2 : 4);
        if (yb > lim) return false;
        p.y_bytes = (uint32_t)yb;
    }
    p.a_bytes = (uint32_t)((long long)g.K * g.C * 2);
    pl->at = bwd_data;
    pl->pair = HW % 2 == 0;
    // 128 output channels x 256 pixels per workgroup where that still gives every compute unit a
    // workgroup; else smaller tiles: more workgroups, and more passes over X and A, which these
    // small problems take from L2; long reductions over few pixels are split over the waves
    auto tiles = [&](int ms, int px) { return ((M + 32 * ms - 1) / (32 * ms)) * ((npx + px - 1) / px); };
    pl->split = false;
    if (M > 64 && tiles(4, 256) >= 256) { pl->MS = 4; pl->NW = 4; }
    else if (tiles(2, 256) >= 256) { pl->MS = 2; pl->NW = 4; }
    else if (Rd >= 256 && tiles(2, 64) < 640) { pl->MS = 2; pl->NW = 4; pl->split = true; }   // measured: 7x7 and 8x8 images gain, 14x14 ones do not
    else { pl->MS = 2; pl->NW = 1; }
    const int px = pl->split ? 64 : 64 * pl->NW;
    p.mtiles = (int)((M + 32 * pl->MS - 1) / (32 * pl->MS));
    p.ptiles = (int)((npx + px - 1) / px);
    const long long per_trip = pl->split ? 4 * RG : RG;   // reduction channels a workgroup consumes per main-loop trip
    p.niter = (int)((Rd + per_trip - 1) / per_trip);
    const long long grid = 8LL * p.mtiles * ((p.ptiles + 7) / 8);
    if (grid > 0x7fffffffLL) return false;
    pl->grid = (unsigned)grid;
    return true;
}

template <int MS, int NW, bool SPLIT>
hipError_t launch_shape(const bf16_t *x, const bf16_t *a, void *y, const PwPlan &pl, hipStream_t st)
{
    const dim3 grid(pl.grid), block(64 * NW);
    if (pl.at) {
        if (pl.pair) hipLaunchKernelGGL((pointwise_kernel<MS, NW, SPLIT, true, true>), grid, block, 0, st, x, a, y, pl.p);
        else hipLaunchKernelGGL((pointwise_kernel<MS, NW, SPLIT, true, false>), grid, block, 0, st, x, a, y, pl.p);
    } else {
        if (pl.pair) hipLaunchKernelGGL((pointwise_kernel<MS, NW, SPLIT, false, true>), grid, block, 0, st, x, a, y, pl.p);
        else hipLaunchKernelGGL((pointwise_kernel<MS, NW, SPLIT, false, false>), grid, block, 0, st, x, a, y, pl.p);
    }
    return hipGetLastError();
}

// ---- forward of any filter by the CONV form of the kernel above ----------------------------------
// wp[k][tap][c] = w[k][c][tap]: the filter with the channel innermost, so that a row of A is contiguous.
__global__ void __launch_bounds__(256)
pack_tap_major_kernel(const bf16_t *__restrict__ w, bf16_t *__restrict__ wp, int C, int T, size_t total)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;   // index into wp
    if (i >= total) return;
    const size_t kt = i / C;
    const int c = (int)(i - kt * C), t = (int)(kt % T);
    const size_t k = kt / T;
    wp[i] = w[(k * C + c) * T + t];
}

bool make_conv_plan(const ConvGeom &g, PwPlan *pl)
{
    if (!g.in_bf16 || g.C % 16 != 0 || g.K % 8 != 0) return false;
    if (g.R * g.S > 121) return false;
    const long long PQ = (long long)g.P * g.Q, npx = PQ * g.N, Rd = (long long)g.C * g.R * g.S, M = g.K;
    const long long lim = 0x7fffffffLL - (1 << 20);
    const long long xb = (long long)g.N * g.C * g.H * g.W * 2;
    if (xb > lim || npx * M * (g.out_bf16 ? 2 : 4) > lim || M * Rd * 2 > lim) return false;
    if (16LL * g.H * g.W * 2 * 4 > lim) return false;
    PwProblem &p = pl->p;
    p.M = (int)M; p.Rd = (int)Rd; p.HW = (int)PQ; p.npx = (uint32_t)npx;
    p.out_bf16 = g.out_bf16;
    p.x_bytes = (uint32_t)xb;
    p.y_bytes = (uint32_t)(npx * M * (g.out_bf16 ? 2 : 4));
    p.a_bytes = (uint32_t)(M * Rd * 2);
    p.C = g.C; p.Hin = g.H; p.Win = g.W; p.Q = g.Q; p.R = g.R; p.S = g.S;
    p.sh = g.sh; p.sw = g.sw; p.ph = g.ph; p.pw = g.pw;
    p.spt = g.C / 16;
    p.scat = 0; p.Hd = p.Wd = p.Qd = 0;
    pl->at = false; pl->pair = false; pl->split = false;
    auto tiles = [&](int ms, int px) { return ((M + 32 * ms - 1) / (32 * ms)) * ((npx + px - 1) / px); };
    if (M > 64 && tiles(4, 256) >= 256) { pl->MS = 4; pl->NW = 4; }
    else if (tiles(2, 256) >= 256) { pl->MS = 2; pl->NW = 4; }
    else { pl->MS = 2; pl->NW = 1; }
    const int px = 64 * pl->NW;
    p.mtiles = (int)((M + 32 * pl->MS - 1) / (32 * pl->MS));
    p.ptiles = (int)((npx + px - 1) / px);
    p.niter = (int)((Rd + RG - 1) / RG);
    const long long grid = 8LL * p.mtiles * ((p.ptiles + 7) / 8);
    if (grid > 0x7fffffffLL) return false;
    pl->grid = (unsigned)grid;
    return true;
}

// ---- backward-filter of the same layers on small images ------------------------------------------
// dw[k][c] = sum over n and px of dy[n][k][px] * x[n][c][px]: the reduction runs along the pixels, which
// both operands have contiguous, so a lane's 8 reduction entries are one 16-byte load (at any 2-byte
// alignment) straight into the MFMA layout -- no LDS in the main loop.  A workgroup owns 64 k x 64 c; its
// four waves take a quarter of the workgroup's images each (all 64 x 64, 2 x 2 MFMA tiles) and add their
// accumulators through LDS in wave order at the end; gridDim.y slices split the batch further where
// the tiles alone do not fill the chip.  An image is ceil(HW / 16) steps; in the last one the lanes
// whose 8 pixels would pass the end of the plane read the last 8 pixels of the plane instead and
// mask the ones an earlier step already had, on both operands, so nothing outside a row is ever
// multiplied and nothing outside the tensors is read.
struct PwWgradProblem {
    int K, C, HW, N;
    int ctiles;
    int steps;     // 16-pixel steps per image
    int ipw;       // images per wave
    int atomics;
};

__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
pointwise_wgrad_kernel(const bf16_t *__restrict__ x, const bf16_t *__restrict__ dy, float *__restrict__ out, PwWgradProblem p)
{
    __shared__ __attribute__((aligned(16))) float red[4 * 32 * 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, g = lane >> 5;
    const int kt = blockIdx.x / p.ctiles, ct = blockIdx.x - kt * p.ctiles, z = blockIdx.y;
    const int k0 = kt * 64, c0 = ct * 64;

    // rows past the last channel read the last channel instead: their products land in rows / columns that are not stored
    uint32_t rowd[2], rowx[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        rowd[i] = (uint32_t)min(k0 + 32 * i + l32, p.K - 1) * p.HW * 2;
        rowx[i] = (uint32_t)min(c0 + 32 * i + l32, p.C - 1) * p.HW * 2;
    }
    const int lastcol = 16 * (p.steps - 1) + 8 * g, cnt = min(max(p.HW - lastcol, 0), 8);
    const uint32_t tailcolb = (uint32_t)(cnt < 8 ? p.HW - 8 : lastcol) * 2;
    uint32_t tailmask[4];
#pragma unroll
    for (int t = 0; t < 4; ++t)
        tailmask[t] = (2 * t >= 8 - cnt ? 0xffffu : 0u) | (2 * t + 1 >= 8 - cnt ? 0xffff0000u : 0u);

    // the wave's images: first .. first + nimg - 1
    const int first = (z * 4 + wave) * p.ipw;
    const int nimg = min(max(p.N - first, 0), p.ipw);
    const int nq = nimg * p.steps;
    const int nlast = min(first + max(nimg, 1) - 1, p.N - 1);
    const uint32_t dimg = (uint32_t)p.K * p.HW * 2, ximg = (uint32_t)p.C * p.HW * 2;   // bytes per image
    const __amdgpu_buffer_rsrc_t dr = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(dy), 0, (uint32_t)p.N * dimg, 0x00020000);
    const __amdgpu_buffer_rsrc_t xr = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(x), 0, (uint32_t)p.N * ximg, 0x00020000);

    u32x4 dreg[4][2], xreg[4][2];
    int n_iss = first, s_iss = 0;
    auto issue = [&](u32x4 (&dd)[2], u32x4 (&xd)[2]) {
        const uint32_t n = (uint32_t)min(n_iss, nlast);
        const uint32_t colb = s_iss == p.steps - 1 ? tailcolb : (uint32_t)(16 * s_iss + 8 * g) * 2;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            dd[i] = __builtin_amdgcn_raw_buffer_load_b128(dr, rowd[i] + colb, n * dimg, 0);
            xd[i] = __builtin_amdgcn_raw_buffer_load_b128(xr, rowx[i] + colb, n * ximg, 0);
        }
        if (++s_iss == p.steps) { s_iss = 0; ++n_iss; }
    };

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    issue(dreg[0], xreg[0]);
    __builtin_amdgcn_sched_barrier(0);   // in this order: the first wait of the loop is for set 0 alone
    issue(dreg[1], xreg[1]);
    __builtin_amdgcn_sched_barrier(0);
    issue(dreg[2], xreg[2]);
    __builtin_amdgcn_sched_barrier(0);
    int s_con = 0;
    for (int q0 = 0; q0 < nq; q0 += 4) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            issue(dreg[(u + 3) & 3], xreg[(u + 3) & 3]);
            __builtin_amdgcn_sched_barrier(0);
            const bool live = q0 + u < nq, last = s_con == p.steps - 1;
            if (++s_con == p.steps) s_con = 0;
            bf16x8 a[2], b[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                u32x4 dm, xm;
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const uint32_t m = live ? (last ? tailmask[t] : 0xffffffffu) : 0u;
                    dm[t] = dreg[u][i][t] & m;
                    xm[t] = xreg[u][i][t] & m;
                }
                __builtin_memcpy(&a[i], &dm, 16);
                __builtin_memcpy(&b[i], &xm, 16);
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
        }
    }

    // ---- the four waves' sums, block of 32 k at a time: [wave][j][v][lane] in LDS, wave w adds up rows 8w .. 8w+7
    float *dst = out + (p.atomics ? 0 : (size_t)z * p.K * p.C);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        __syncthreads();
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) red[((wave * 2 + j) * 16 + v) * 64 + lane] = acc[i][j][v];
        __syncthreads();
#pragma unroll
        for (int vv = 0; vv < 4; ++vv) {
            const int k = k0 + 32 * i + 8 * wave + 4 * g + vv;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                float sum = red[((0 * 2 + j) * 16 + 4 * wave + vv) * 64 + lane];
#pragma unroll
                for (int w2 = 1; w2 < 4; ++w2) sum += red[((w2 * 2 + j) * 16 + 4 * wave + vv) * 64 + lane];
                const int c = c0 + 32 * j + l32;
                if (k < p.K && c < p.C) {
                    if (p.atomics) unsafeAtomicAdd(dst + (size_t)k * p.C + c, sum);
                    else dst[(size_t)k * p.C + c] = sum;
                }
            }
        }
    }
}

struct PwWgradPlan {
    PwWgradProblem p;
    dim3 grid;
    int slices;
};

bool make_wgrad_plan(const ConvGeom &g, PwWgradPlan *pl)
{
    if (!g.in_bf16 || g.R != 1 || g.S != 1 || g.sh != 1 || g.sw != 1 || g.ph != 0 || g.pw != 0) return false;
    if (g.P != g.H || g.Q != g.W) return false;
    const long long HW = (long long)g.H * g.W;
    // the smallest planes only (7x7, 8x8): a load brings 32 bytes of each of 32 rows, which costs the memory
    // pipeline about as much as 32 separate lines; from 14x14 on the row-stationary kernel's tiles, loaded as
    // whole lines and re-laid out in LDS, are as fast (measured: 47 against 44 us on 1024 -> 256 channels)
    if (HW < 8 || HW > 64) return false;
    if ((long long)std::max(g.K, g.C) * HW * 2 * g.N > 0x7fffffffLL) return false;
    PwWgradProblem &p = pl->p;
    p.K = g.K; p.C = g.C; p.HW = (int)HW; p.N = g.N;
    p.ctiles = (g.C + 63) / 64;
    const long long tiles = (long long)((g.K + 63) / 64) * p.ctiles;
    if (tiles > 0x7fffffffLL) return false;
    p.steps = (int)((HW + 15) / 16);
    long long slices = (256 + tiles - 1) / tiles;
    slices = std::max(1LL, std::min(slices, (long long)g.N / 4));
    p.ipw = (int)((g.N + 4 * slices - 1) / (4 * slices));
    slices = (g.N + 4LL * p.ipw - 1) / (4LL * p.ipw);
    if (slices > 65535) return false;
    pl->slices = (int)slices;
    pl->grid = dim3((unsigned)tiles, (unsigned)slices);
    return true;
}

// ---- backward-filter of 1x1 layers through LDS (14x14; planes of odd sizes: 17x17, 35x35) ----------
// Same product as above, but the operands reach the MFMAs through LDS: a workgroup owns 128 k x 128 c and
// walks its images in stages of 64 pixels; the 256 rows (128 of dy, 128 of x) of a stage are fetched as
// 8-byte items, 16 consecutive lanes per row (whole 128-byte runs, which 4-pixel-aligned rows allow),
// parked [row][64 px] and read back as 16-byte operands.  Items past the end of a plane are fetched
// from an out-of-range offset and arrive as zeros, so a plane's ragged last stage needs no masks.
// Four waves, 2 x 2, 64 x 64 each; two stages ahead of the one being multiplied are under way, one in
// registers on its way from memory, one going from registers into the next of three LDS buffers (one
// barrier per stage); slices of the batch split the sum, the tiles of a slice on one XCD.
struct PwWgradLdsProblem {
    int K, C, HW, N;
    int ctiles, tiles, slices;
    int spi;       // 64-pixel stages per image
    int steps;     // 16-pixel steps per image
    int ipw;       // images per workgroup
    int atomics;
    int ragged;    // HW is not a multiple of 4
    uint32_t d_bytes, x_bytes;
};

constexpr int WL_PITCH = 144, WL_BUF = 256 * WL_PITCH, WL_NBUF = 3;

__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
pointwise_wgrad_lds_kernel(const bf16_t *__restrict__ x, const bf16_t *__restrict__ dy, float *__restrict__ out,
                           PwWgradLdsProblem p)
{
    extern __shared__ __attribute__((aligned(16))) char wl_lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, g = lane >> 5, wk = wave >> 1, wc = wave & 1;
    // workgroups go round the XCDs: all tiles of a slice (they read the same images) on one XCD
    const int xcd = blockIdx.x & 7, rest = blockIdx.x >> 3;
    const int tile = rest % p.tiles, z = (rest / p.tiles) * 8 + xcd;
    if (z >= p.slices) return;
    const int kt = tile / p.ctiles, ct = tile - kt * p.ctiles;
    const int k0 = kt * 128, c0 = ct * 128;
    const __amdgpu_buffer_rsrc_t dr = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(dy), 0, p.d_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t xr = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(x), 0, p.x_bytes, 0x00020000);

    // item j of the thread: row (tid >> 4) + 16 * j of the stage (0 .. 127 dy, 128 .. 255 x), pixels 4 * (tid & 15) .. + 3
    const int col8 = tid & 15, row0 = tid >> 4;
    uint32_t src[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) {
        const int row = row0 + 16 * (j & 7);
        const int ch = (j < 8 ? k0 : c0) + row;
        src[j] = ch < (j < 8 ? p.K : p.C) ? (uint32_t)ch * p.HW * 2 + col8 * 8 : OUTSIDE;
    }
    const uint32_t dst = row0 * WL_PITCH + col8 * 8;   // + 16 * j rows
    const uint32_t dimg = (uint32_t)p.K * p.HW * 2, ximg = (uint32_t)p.C * p.HW * 2;

    const int first = z * p.ipw, nimg = min(max(p.N - first, 0), p.ipw);
    const int nq = nimg * p.spi;

    // Planes that are no whole number of 4-pixel items: the item over a plane's end is fetched `back` pixels
    // earlier, so that it ends with the plane (nothing past a plane, or past the tensor, is read), and moved
    // down by as many pixels before it reaches LDS, which leaves zeros behind the plane's last pixel.  Only the
    // last stage of an image has such an item; stages are parked in the order they were issued.
    const int tail = p.HW - 64 * (p.spi - 1) - 4 * col8;   // pixels this thread's item has left in a last stage
    const int back = p.ragged && tail > 0 && tail < 4 ? 4 - tail : 0;
    u32x2 reg[2][16];
    int n_iss = first, js_iss = 0;
    auto issue = [&](u32x2 (&rd)[16]) {   // the stage (n_iss, js_iss); past the last stage: zeros
        const bool live = n_iss < first + nimg;
        const uint32_t off = live && 64 * js_iss + 4 * col8 < p.HW ? 0u : OUTSIDE;
        // the stage's offset within the plane, less the pixels a last item starts early by (never negative:
        // such an item is not the first of its plane)
        const uint32_t adv = js_iss * 128 - (js_iss == p.spi - 1 ? 2u * back : 0u);
        const uint32_t n = (uint32_t)min(n_iss, p.N - 1);
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const uint32_t v = (src[j] + adv) | (src[j] & OUTSIDE) | off;
            rd[j] = j < 8 ? __builtin_amdgcn_raw_buffer_load_b64(dr, v, n * dimg, 0)
                          : __builtin_amdgcn_raw_buffer_load_b64(xr, v, n * ximg, 0);
        }
        if (++js_iss == p.spi) { js_iss = 0; ++n_iss; }
    };
    int js_park = 0;
    auto park = [&](int buf, u32x2 (&rd)[16]) {
        if (p.ragged && js_park == p.spi - 1 && back) {
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const uint64_t v = (((uint64_t)rd[j].y << 32) | rd[j].x) >> (16 * back);
                rd[j].x = (uint32_t)v;
                rd[j].y = (uint32_t)(v >> 32);
            }
        }
        if (++js_park == p.spi) js_park = 0;
#pragma unroll
        for (int j = 0; j < 16; ++j) *reinterpret_cast<u32x2 *>(wl_lds + buf * WL_BUF + dst + j * 16 * WL_PITCH) = rd[j];
    };

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // stage q is multiplied out of LDS buffer q % 3 while stage q + 1 goes from registers into the next buffer
    // and stage q + 2 is on its way from memory
    issue(reg[0]);
    __builtin_amdgcn_sched_barrier(0);
    issue(reg[1]);
    __builtin_amdgcn_sched_barrier(0);
    park(0, reg[0]);
    __syncthreads();
    const uint32_t aoff = (wk * 64 + l32) * WL_PITCH + 16 * g, boff = (128 + wc * 64 + l32) * WL_PITCH + 16 * g;
    int js = 0, cur = 0;
    for (int q0 = 0; q0 < nq; q0 += 2) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            // registers h hold stage q + 2 from here on; registers 1 - h hold stage q + 1
            issue(reg[h]);
            __builtin_amdgcn_sched_barrier(0);
            const char *b = wl_lds + cur * WL_BUF;
            const int nxt = cur == 2 ? 0 : cur + 1;
            const int nst = min(4, p.steps - 4 * js);
            if (++js == p.spi) js = 0;
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                if (s < nst) {
                    bf16x8 a[2], bb[2];
#pragma unroll
                    for (int i = 0; i < 2; ++i) {
                        u32x4 da = *reinterpret_cast<const u32x4 *>(b + aoff + i * 32 * WL_PITCH + s * 32);
                        u32x4 db = *reinterpret_cast<const u32x4 *>(b + boff + i * 32 * WL_PITCH + s * 32);
                        __builtin_memcpy(&a[i], &da, 16);
                        __builtin_memcpy(&bb[i], &db, 16);
                    }
#pragma unroll
                    for (int i = 0; i < 2; ++i)
#pragma unroll
                        for (int j = 0; j < 2; ++j)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], bb[j], acc[i][j], 0, 0, 0);
                }
            }
            park(nxt, reg[1 - h]);
            __syncthreads();
            cur = nxt;
        }
    }

    float *o = out + (p.atomics ? 0 : (size_t)z * p.K * p.C);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int k = k0 + wk * 64 + 32 * i + 8 * (v >> 2) + 4 * g + (v & 3);
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int c = c0 + wc * 64 + 32 * j + l32;
                if (k < p.K && c < p.C) {
                    if (p.atomics) unsafeAtomicAdd(o + (size_t)k * p.C + c, acc[i][j][v]);
                    else o[(size_t)k * p.C + c] = acc[i][j][v];
                }
            }
        }
}

struct PwWgradLdsPlan {
    PwWgradLdsProblem p;
    dim3 grid;
    int slices;
};

bool make_wgrad_lds_plan(const ConvGeom &g, PwWgradLdsPlan *pl)
{
    if (!g.in_bf16 || g.R != 1 || g.S != 1 || g.sh != 1 || g.sw != 1 || g.ph != 0 || g.pw != 0) return false;
    if (g.P != g.H || g.Q != g.W) return false;
    const long long HW = (long long)g.H * g.W;
    // short rows (where the row-stationary kernel's 8 x 16 chunks are mostly padding) and planes of an odd size
    // (whose rows that kernel cannot fetch in aligned pieces)
    if ((HW % 4 == 0 && g.W > 16) || HW < 8) return false;
    const long long lim = 0x7fffffffLL - (1 << 20);
    if ((long long)g.K * HW * 2 * g.N > lim || (long long)g.C * HW * 2 * g.N > lim) return false;
    PwWgradLdsProblem &p = pl->p;
    p.K = g.K; p.C = g.C; p.HW = (int)HW; p.N = g.N;
    p.ragged = HW % 4 != 0;
    p.ctiles = (g.C + 127) / 128;
    const long long tiles = (long long)((g.K + 127) / 128) * p.ctiles;
    if (tiles > 0x7fffffffLL) return false;
    p.spi = (int)((HW + 63) / 64);
    p.steps = (int)((HW + 15) / 16);
    long long slices = (256 + tiles - 1) / tiles;
    slices = std::max(1LL, std::min(slices, (long long)g.N));
    p.ipw = (int)((g.N + slices - 1) / slices);
    slices = (g.N + p.ipw - 1) / p.ipw;
    if (slices > 65535) return false;
    p.d_bytes = (uint32_t)((long long)g.K * HW * 2 * g.N);
    p.x_bytes = (uint32_t)((long long)g.C * HW * 2 * g.N);
    pl->slices = (int)slices;
    p.tiles = (int)tiles;
    p.slices = (int)slices;
    const long long grid = 8 * tiles * ((slices + 7) / 8);
    if (grid > 0x7fffffffLL) return false;
    pl->grid = dim3((unsigned)grid);
    return true;
}

// ---- backward-filter of 1x1 layers with a stride or padding: the same product, x gathered ----
// dw[k][c] = sum over (n, p, q) of dy[n][k][p][q] * x[n][c][p*sh - ph][q*sw - pw].  A workgroup owns 128 k x 128 c
// and walks its images in stages of 64 output pixels: dy arrives as in the kernel above (8-byte items of the flat
// plane, the item over its end fetched early and shifted down); x is gathered element by element, a wavefront
// taking 64 consecutive output pixels of one channel per load (addresses sw elements apart within an output row;
// pixels in the padding or past the plane read as zeros from an out-of-range offset) and parking them as 2-byte
// items.  The gathers use a quarter of every cache line they touch (stride 2), and every tile of output channels
// repeats them, which bounds the kernel; a tap at a time it also ran larger filters, and lost to the fallback
// kernel on each (3x3 / stride 2: 185 - 380 against 164 - 182 us), so it is built for 1x1 filters only.
struct GwProblem {
    int K, C, N;
    int PQ, Q;          // the plane of dy
    int H, W;           // the plane of x
    int sh, sw, ph, pw;
    int d64, m64;       // 64 / Q, 64 % Q: how a stage moves a pixel's (row, column)
    int ctiles, units, slices;   // units = tiles of 128 k x 128 c
    int spi, steps, ipw, atomics, ragged;
    uint32_t d_bytes, x_bytes;
};

__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
gather_wgrad_kernel(const bf16_t *__restrict__ x, const bf16_t *__restrict__ dy, float *__restrict__ out, GwProblem p)
{
    extern __shared__ __attribute__((aligned(16))) char wl_lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, g = lane >> 5, wk = wave >> 1, wc = wave & 1;
    const int xcd = blockIdx.x & 7, rest = blockIdx.x >> 3;
    const int unit = rest % p.units, z = (rest / p.units) * 8 + xcd;
    if (z >= p.slices) return;
    const int kt = unit / p.ctiles, ct = unit - kt * p.ctiles;
    const int k0 = kt * 128, c0 = ct * 128;
    const __amdgpu_buffer_rsrc_t dr = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(dy), 0, p.d_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t xr = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(x), 0, p.x_bytes, 0x00020000);

    // dy: item j of the thread is row (tid >> 4) + 16 * j of the stage, pixels 4 * (tid & 15) .. + 3
    const int col8 = tid & 15, row0 = tid >> 4;
    uint32_t src[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int ch = k0 + row0 + 16 * j;
        src[j] = ch < p.K ? (uint32_t)ch * p.PQ * 2 + col8 * 8 : OUTSIDE;
    }
    const uint32_t dst_a = row0 * WL_PITCH + col8 * 8;   // + 16 * j rows
    // x: the thread's pixel of the stage is its lane; its wavefront takes channels c0 + wave + 4 * j
    const uint32_t xplane = (uint32_t)p.H * p.W * 2;
    const uint32_t xbase = (uint32_t)(c0 + wave) * xplane;
    const int jlim = c0 + wave < p.C ? (p.C - c0 - wave + 3) / 4 : 0;   // channels of the wavefront inside the tensor
    const uint32_t dst_b = (128 + wave) * WL_PITCH + lane * 2;           // + 4 * j rows
    const uint32_t dimg = (uint32_t)p.K * p.PQ * 2, ximg = (uint32_t)p.C * xplane;

    const int first = z * p.ipw, nimg = min(max(p.N - first, 0), p.ipw);
    const int nq = nimg * p.spi;

    const int tail = p.PQ - 64 * (p.spi - 1) - 4 * col8;   // pixels this thread's dy item has left in a last stage
    const int back = p.ragged && tail > 0 && tail < 4 ? 4 - tail : 0;
    const int pp0 = lane / p.Q, qq0 = lane - pp0 * p.Q;    // the thread's output pixel in stage 0
    u32x2 ra[2][8];
    uint32_t rb[2][32];
    int n_iss = first, js_iss = 0, pp = pp0, qq = qq0;
    auto issue = [&](u32x2 (&rd)[8], uint32_t (&rx)[32]) {   // the stage (n_iss, js_iss); past the last stage: zeros
        const bool live = n_iss < first + nimg;
        const uint32_t off = live && 64 * js_iss + 4 * col8 < p.PQ ? 0u : OUTSIDE;
        const uint32_t adv = js_iss * 128 - (js_iss == p.spi - 1 ? 2u * back : 0u);
        const uint32_t n = (uint32_t)min(n_iss, p.N - 1);
#pragma unroll
        for (int j = 0; j < 8; ++j)
            rd[j] = __builtin_amdgcn_raw_buffer_load_b64(dr, (src[j] + adv) | (src[j] & OUTSIDE) | off, n * dimg, 0);
        const int hh = pp * p.sh - p.ph, ww = qq * p.sw - p.pw;
        const bool in = live && 64 * js_iss + lane < p.PQ && (unsigned)hh < (unsigned)p.H && (unsigned)ww < (unsigned)p.W;
        const uint32_t voff = in ? xbase + (uint32_t)(hh * p.W + ww) * 2 : OUTSIDE;
#pragma unroll
        for (int j = 0; j < 32; ++j)
            rx[j] = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(xr, j < jlim ? voff : OUTSIDE, n * ximg + j * 4 * xplane, 0);
        if (++js_iss == p.spi) {
            js_iss = 0; ++n_iss; pp = pp0; qq = qq0;
        } else {
            pp += p.d64; qq += p.m64;
            if (qq >= p.Q) { qq -= p.Q; ++pp; }
        }
    };
    int js_park = 0;
    auto park = [&](int buf, u32x2 (&rd)[8], const uint32_t (&rx)[32]) {
        if (p.ragged && js_park == p.spi - 1 && back) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const uint64_t v = (((uint64_t)rd[j].y << 32) | rd[j].x) >> (16 * back);
                rd[j].x = (uint32_t)v;
                rd[j].y = (uint32_t)(v >> 32);
            }
        }
        if (++js_park == p.spi) js_park = 0;
        char *b = wl_lds + buf * WL_BUF;
#pragma unroll
        for (int j = 0; j < 8; ++j) *reinterpret_cast<u32x2 *>(b + dst_a + j * 16 * WL_PITCH) = rd[j];
#pragma unroll
        for (int j = 0; j < 32; ++j) *reinterpret_cast<uint16_t *>(b + dst_b + j * 4 * WL_PITCH) = (uint16_t)rx[j];
    };

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // as in the kernel above: stage q is multiplied out of LDS buffer q % 3 while stage q + 1 goes from registers
    // into the next buffer and stage q + 2 is on its way from memory
    issue(ra[0], rb[0]);
    __builtin_amdgcn_sched_barrier(0);
    issue(ra[1], rb[1]);
    __builtin_amdgcn_sched_barrier(0);
    park(0, ra[0], rb[0]);
    __syncthreads();
    const uint32_t aoff = (wk * 64 + l32) * WL_PITCH + 16 * g, boff = (128 + wc * 64 + l32) * WL_PITCH + 16 * g;
    int js = 0, cur = 0;
    for (int q0 = 0; q0 < nq; q0 += 2) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            issue(ra[h], rb[h]);
            __builtin_amdgcn_sched_barrier(0);
            const char *b = wl_lds + cur * WL_BUF;
            const int nxt = cur == 2 ? 0 : cur + 1;
            const int nst = min(4, p.steps - 4 * js);
            if (++js == p.spi) js = 0;
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                if (s < nst) {
                    bf16x8 a[2], bb[2];
#pragma unroll
                    for (int i = 0; i < 2; ++i) {
                        u32x4 da = *reinterpret_cast<const u32x4 *>(b + aoff + i * 32 * WL_PITCH + s * 32);
                        u32x4 db = *reinterpret_cast<const u32x4 *>(b + boff + i * 32 * WL_PITCH + s * 32);
                        __builtin_memcpy(&a[i], &da, 16);
                        __builtin_memcpy(&bb[i], &db, 16);
                    }
#pragma unroll
                    for (int i = 0; i < 2; ++i)
#pragma unroll
                        for (int j = 0; j < 2; ++j)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], bb[j], acc[i][j], 0, 0, 0);
                }
            }
            park(nxt, ra[1 - h], rb[1 - h]);
            __syncthreads();
            cur = nxt;
        }
    }

    float *o = out + (p.atomics ? 0 : (size_t)z * p.K * p.C);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int k = k0 + wk * 64 + 32 * i + 8 * (v >> 2) + 4 * g + (v & 3);
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int c = c0 + wc * 64 + 32 * j + l32;
                if (k < p.K && c < p.C) {
                    float *e = o + (size_t)k * p.C + c;
                    if (p.atomics) unsafeAtomicAdd(e, acc[i][j][v]);
                    else *e = acc[i][j][v];
                }
            }
        }
}

struct GwPlan {
    GwProblem p;
    dim3 grid;
};

bool make_gather_wgrad_plan(const ConvGeom &g, GwPlan *pl)
{
    if (!g.in_bf16 || g.R != 1 || g.S != 1) return false;
    const long long PQ = (long long)g.P * g.Q, HW = (long long)g.H * g.W;
    if (PQ < 8) return false;   // the early-fetched last item of a plane is not its first
    // every tile of output channels gathers x again: beyond eight of them the fallback kernel is faster
    // (measured on 1024 -> 2048 channels, 14x14 -> 7x7: 296 against 160 us)
    if (g.K > 1024) return false;
    const long long lim = 0x7fffffffLL - (1 << 20);
    if ((long long)g.K * PQ * 2 * g.N > lim || (long long)g.C * HW * 2 * g.N > lim) return false;
    GwProblem &p = pl->p;
    p.K = g.K; p.C = g.C; p.N = g.N;
    p.PQ = (int)PQ; p.Q = g.Q; p.H = g.H; p.W = g.W;
    p.sh = g.sh; p.sw = g.sw; p.ph = g.ph; p.pw = g.pw;
    p.d64 = 64 / g.Q; p.m64 = 64 % g.Q;
    p.ragged = PQ % 4 != 0;
    p.ctiles = (g.C + 127) / 128;
    const long long units = (long long)((g.K + 127) / 128) * p.ctiles;
    if (units > (1 << 24)) return false;
    p.units = (int)units;
    p.spi = (int)((PQ + 63) / 64);
    p.steps = (int)((PQ + 15) / 16);
    // One workgroup fits a compute unit (three stage buffers of LDS): the slices of the batch are chosen for the
    // fewest rounds of 256 workgroups times images per workgroup; among equals the fewest slices (partial sums).
    // A workgroup's epilogue (its 128 x 128 sums, and their share of the reduction that follows) is priced at 16 stages.
    long long best = 0, best_cost = -1;
    for (long long sl = 1; sl <= g.N; ++sl) {
        const long long ipw = (g.N + sl - 1) / sl;
        if ((g.N + ipw - 1) / ipw != sl) continue;   // the same images per workgroup in fewer slices
        const long long cost = ((units * sl + 255) / 256) * (ipw * p.spi + 16);
        if (best_cost < 0 || cost < best_cost) { best = sl; best_cost = cost; }
    }
    p.slices = (int)best;
    p.ipw = (int)((g.N + best - 1) / best);
    if (p.slices > 65535) return false;
    p.d_bytes = (uint32_t)((long long)g.K * PQ * 2 * g.N);
    p.x_bytes = (uint32_t)((long long)g.C * HW * 2 * g.N);
    const long long grid = 8 * units * ((best + 7) / 8);
    if (grid > 0x7fffffffLL) return false;
    pl->grid = dim3((unsigned)grid);
    return true;
}

}  // namespace

bool pointwise_supported(const ConvGeom &g, bool bwd_data)
{
    PwPlan pl;
    return make_plan(g, bwd_data, &pl);
}

hipError_t launch_pointwise(const void *in, const void *w, void *out, const ConvGeom &g, bool bwd_data, hipStream_t st)
{
    PwPlan pl;
    if (!make_plan(g, bwd_data, &pl)) return hipErrorInvalidValue;
    const bf16_t *x = static_cast<const bf16_t *>(in), *a = static_cast<const bf16_t *>(w);
    if (pl.split) return launch_shape<2, 4, true>(x, a, out, pl, st);
    if (pl.MS == 4) return launch_shape<4, 4, false>(x, a, out, pl, st);
    if (pl.NW == 4) return launch_shape<2, 4, false>(x, a, out, pl, st);
    return launch_shape<2, 1, false>(x, a, out, pl, st);
}

bool gather_conv_supported(const ConvGeom &g)
{
    PwPlan pl;
    return make_conv_plan(g, &pl);
}

size_t gather_conv_packed_bytes(const ConvGeom &g)
{
    if (g.R == 1 && g.S == 1) return 0;   // KC11 is already [k][tap][c]
    return align_up((size_t)g.K * g.C * g.R * g.S * sizeof(bf16_t), 256);
}

hipError_t launch_gather_conv_fwd(const void *x, const void *w, void *y, const ConvGeom &g, void *packed, hipStream_t st)
{
    PwPlan pl;
    // a 1x1 filter is its own tap-major form: nothing to re-lay out, no workspace
    const bool as_is = g.R == 1 && g.S == 1;
    if (!make_conv_plan(g, &pl) || (!packed && !as_is)) return hipErrorInvalidValue;
    if (!as_is) {
        const size_t total = (size_t)g.K * g.C * g.R * g.S;
        hipLaunchKernelGGL(pack_tap_major_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                           static_cast<const bf16_t *>(w), static_cast<bf16_t *>(packed), g.C, g.R * g.S, total);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    const bf16_t *xs = static_cast<const bf16_t *>(x), *a = static_cast<const bf16_t *>(as_is ? w : packed);
    const dim3 grid(pl.grid);
    if (pl.MS == 4) hipLaunchKernelGGL((pointwise_kernel<4, 4, false, false, false, true>), grid, dim3(256), 0, st, xs, a, y, pl.p);
    else if (pl.NW == 4) hipLaunchKernelGGL((pointwise_kernel<2, 4, false, false, false, true>), grid, dim3(256), 0, st, xs, a, y, pl.p);
    else hipLaunchKernelGGL((pointwise_kernel<2, 1, false, false, false, true>), grid, dim3(64), 0, st, xs, a, y, pl.p);
    return hipGetLastError();
}

bool pointwise_wgrad_supported(const ConvGeom &g)
{
    PwWgradPlan pl;
    PwWgradLdsPlan pl2;
    return make_wgrad_plan(g, &pl) || make_wgrad_lds_plan(g, &pl2);
}

int pointwise_wgrad_slices(const ConvGeom &g)
{
    PwWgradPlan pl;
    PwWgradLdsPlan pl2;
    if (make_wgrad_plan(g, &pl)) return pl.slices;
    return make_wgrad_lds_plan(g, &pl2) ? pl2.slices : 0;
}

// partial == nullptr: slices add into dw with atomics (dw is zero-filled first; one slice stores);
// otherwise slice z writes partial[z][K*C] and a reduction in slice order follows.
hipError_t launch_pointwise_wgrad(const void *x, const void *dy, float *dw, const ConvGeom &g, float *partial,
                                  hipStream_t st)
{
    PwWgradPlan pl;
    PwWgradLdsPlan pl2;
    const bool small = make_wgrad_plan(g, &pl);
    if (!small && !make_wgrad_lds_plan(g, &pl2)) return hipErrorInvalidValue;
    const int slices = small ? pl.slices : pl2.slices;
    const size_t nw = (size_t)g.K * g.C;
    const bool direct_store = slices == 1;
    const int atomics = (!partial && !direct_store) ? 1 : 0;
    if (atomics) {
        hipError_t e = launch_fill_zero(dw, nw, st);
        if (e != hipSuccess) return e;
    }
    float *out = (partial && !direct_store) ? partial : dw;
    const bf16_t *xs = static_cast<const bf16_t *>(x), *ds = static_cast<const bf16_t *>(dy);
    if (small) {
        pl.p.atomics = atomics;
        hipLaunchKernelGGL(pointwise_wgrad_kernel, pl.grid, dim3(256), 0, st, xs, ds, out, pl.p);
    } else {
        // dynamic LDS beyond 64 KB has to be enabled once per kernel
        static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(pointwise_wgrad_lds_kernel),
                                                           hipFuncAttributeMaxDynamicSharedMemorySize, WL_NBUF * WL_BUF);
        if (attr != hipSuccess) return attr;
        pl2.p.atomics = atomics;
        hipLaunchKernelGGL(pointwise_wgrad_lds_kernel, pl2.grid, dim3(256), WL_NBUF * WL_BUF, st, xs, ds, out, pl2.p);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (partial && !direct_store) return launch_reduce_partials(partial, dw, nw, slices, false, st);
    return hipSuccess;
}

bool gather_wgrad_supported(const ConvGeom &g)
{
    GwPlan pl;
    return make_gather_wgrad_plan(g, &pl);
}

int gather_wgrad_slices(const ConvGeom &g)
{
    GwPlan pl;
    return make_gather_wgrad_plan(g, &pl) ? pl.p.slices : 0;
}

// partial == nullptr: slices add into dw with atomics (dw is zero-filled first; one slice stores);
// otherwise slice z writes partial[z][K*C] and a reduction in slice order follows.
hipError_t launch_gather_wgrad(const void *x, const void *dy, float *dw, const ConvGeom &g, float *partial, hipStream_t st)
{
    GwPlan pl;
    if (!make_gather_wgrad_plan(g, &pl)) return hipErrorInvalidValue;
    const size_t nw = (size_t)g.K * g.C;
    const bool direct_store = pl.p.slices == 1;
    pl.p.atomics = (!partial && !direct_store) ? 1 : 0;
    if (pl.p.atomics) {
        hipError_t e = launch_fill_zero(dw, nw, st);
        if (e != hipSuccess) return e;
    }
    float *out = (partial && !direct_store) ? partial : dw;
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(gather_wgrad_kernel),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, WL_NBUF * WL_BUF);
    if (attr != hipSuccess) return attr;
    hipLaunchKernelGGL(gather_wgrad_kernel, pl.grid, dim3(256), WL_NBUF * WL_BUF, st, static_cast<const bf16_t *>(x),
                       static_cast<const bf16_t *>(dy), out, pl.p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (partial && !direct_store) return launch_reduce_partials(partial, dw, nw, pl.p.slices, false, st);
    return hipSuccess;
}

}  // namespace sn
