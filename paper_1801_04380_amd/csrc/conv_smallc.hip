// CONV forward and backward-filter for inputs with very few channels (C*R*S <= 32: the
// first layer of a network, 3 channels under a 3x3 filter) on gfx950, bf16 operands
// (Sec. 3.5 of the paper: the zero-workspace end of the menu; definitions in sn.h).
//
// With 27 products per output the layer is bound by memory, not by the matrix cores:
// forward writes y once, backward-filter reads dy once, and x is a few per cent of
// either.  The 16-channel chunks of the tile kernels would multiply 13 channels of
// zeros; here the whole reduction (c, r, s), padded to 32, is ONE MFMA operand.
//
//   forward          y[px][k]  += X[px][(c,r,s)] * W[(c,r,s)][k]     two 32x32x16 steps
//   backward-filter  dw[k][(c,r,s)] += DY[k][px] * X[px][(c,r,s)]    a step per 16 pixels
//
// The filter is KCRS, so W's 32 reduction entries of a channel k are contiguous; the
// X operand is gathered from a patch of x in LDS with 2-byte reads (any stride and
// padding: the gather only changes its offsets).  Every wave is a program of its own:
// it owns a private piece of LDS and walks the units u = wave, wave + nwaves, ...,
// a unit being 64 consecutive pixels of one output row for 64 output channels.  No
// barrier in the main loop; the loads of unit u+1 fly while unit u is multiplied.
//   forward: patch -> gather -> 8 MFMAs -> the 64 k x 64 px block through LDS so that a
//     lane stores 8 consecutive pixels of one channel (whole 128-byte lines); optionally
//     the per-channel statistics of the stored values for the batch normalisation that
//     follows, one (count, mean, M2) triple per wave and channel.
//   backward-filter: dy block global -> registers -> LDS [k][px] (coalesced 16-byte loads),
//     patch -> gather, 8 MFMAs into two 32x32 accumulators that live for the whole launch;
//     at the end the four waves of a workgroup add up through LDS and the workgroup either
//     writes its slice of partial sums or adds into dw with atomics.
#include "sn_internal.h"

namespace sn {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int KT = 64;           // output channels per pass (blockIdx.y)
constexpr int UPX = 64;          // pixels per unit
constexpr int RED = 32;          // the padded reduction length
constexpr int STG_PITCH = 144;   // bytes per channel row of the staged block: 64 px, and 16 so that rows spread over the banks
constexpr int STG_ROWS = 32;     // channel rows of the staged block (forward stores 32 channels at a time)
constexpr int WAVES = 4;

struct SmallProblem {
    int N, C, H, W, K, R, S, sh, sw, ph, pw, P, Q;
    int CRS, RS, CR;
    int ncb;         // 64-pixel blocks per output row
    int nunits;      // N * P * ncb
    int nslot;       // 64-lane load rounds per patch row
    int shiftc;      // columns the patch starts left of the unit's first tap (0 or 1)
    int ppitch;      // patch row pitch, elements (even)
    int patch_bytes; // per wave, multiple of 16
    int out_bf16;
    int x_bytes;     // the x tensor
    int nwaves;      // waves sharing the units of one channel pass
    int dn, dpr, dcb;   // nwaves units further on: images, rows, blocks (mixed radix)
    float *stats;    // forward: [k][nwaves][3], or null
};

struct __attribute__((packed, aligned(2))) U128u { u32x4 v; };
__device__ inline u32x4 load8_any(const void *p) { return reinterpret_cast<const U128u *>(p)->v; }
__device__ inline void store8_any(void *p, u32x4 v) { reinterpret_cast<U128u *>(p)->v = v; }

__device__ inline uint32_t pack2(float a, float b)   // two fp32 -> two bf16, round to nearest even, a in the low half
{
    f32x2 f = {a, b};
    bf16x2 h = __builtin_convertvector(f, bf16x2);
    uint32_t r;
    __builtin_memcpy(&r, &h, 4);
    return r;
}

struct Moments3 { float n, mean, m2; };
__device__ inline Moments3 join(const Moments3 &a, const Moments3 &b)   // exact pairwise combination
{
    const float nt = a.n + b.n;
    if (!(nt > 0.f)) return a;
    const float d = b.mean - a.mean, r = b.n / nt;
    Moments3 o;
    o.n = nt;
    o.mean = a.mean + d * r;
    o.m2 = a.m2 + b.m2 + d * d * a.n * r;
    return o;
}

// What is common to both kernels: the walk over the units and the patch of x.
//
// The patch of a unit holds, for every (c, r), the input row of that tap and the columns of 64
// pixels, q0*sw - pw - shiftc + 0 .. ppitch - 1, zeros outside the image; every column of it is
// rewritten for every unit, and the gathers of pixels past the end of a ragged row stay inside it.
// It travels global memory -> LDS without passing through registers: range-checked 4-byte buffer
// loads of aligned column pairs (W is even, so a pair is inside or outside the image as a whole),
// lane l of load round sl bringing pair 64 sl + l of a row to consecutive LDS addresses.  A lane
// whose pair is outside the row, or whose row is outside the image, is given an offset past the
// tensor (fewer than 2^31 bytes) and zero arrives; the row's start is a uniform offset.
struct UnitWalk {
    const SmallProblem &p;
    int lane;
    int n, pr, cb;    // the unit being staged (uniform)

    __device__ UnitWalk(const SmallProblem &pp, int lane_) : p(pp), lane(lane_) { n = pr = cb = 0; }
    __device__ void set_unit(int u)
    {
        const int per_img = p.P * p.ncb;
        n = u / per_img;
        const int rem = u - n * per_img;
        pr = rem / p.ncb;
        cb = rem - pr * p.ncb;
    }
    __device__ void advance()   // nwaves units further on
    {
        cb += p.dcb;
        pr += p.dpr;
        n += p.dn;
        if (cb >= p.ncb) { cb -= p.ncb; ++pr; }
        if (pr >= p.P) { pr -= p.P; ++n; }
    }
    __device__ void patch_fetch(const __amdgpu_buffer_rsrc_t &xr, char *__restrict__ patch) const
    {
        constexpr uint32_t OUTSIDE = 0x80000000u;
        const int h0 = pr * p.sh - p.ph, w0 = cb * UPX * p.sw - p.pw - p.shiftc;
        const uint32_t W2 = (uint32_t)p.W * 2u;
        const uint32_t cskip = (uint32_t)(p.H - p.R) * W2;   // from the last tap row of a channel to the first of the next
        const int npair = p.ppitch / 2;
        for (int sl = 0; sl < p.nslot; ++sl) {
            const int pair = sl * 64 + lane, wc = w0 + pair * 2;
            const uint32_t voff = (unsigned)wc < (unsigned)p.W ? (uint32_t)wc * 2u : OUTSIDE;
            if (pair < npair) {
                uint32_t rowb = (uint32_t)(n * p.C * p.H + h0) * W2;   // row h0 of channel 0; rows before the image are not read
                char *dst = patch + sl * 256;
                int r = 0;
                for (int i = 0; i < p.CR; ++i) {
                    const bool rowok = (unsigned)(h0 + r) < (unsigned)p.H;
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(xr, (__attribute__((address_space(3))) void *)dst, 4, rowok ? voff : OUTSIDE,
                                                             rowok ? rowb : 0u, 0, 0);
                    dst += p.ppitch * 2;
                    rowb += W2;
                    if (++r == p.R) { r = 0; rowb += cskip; }
                }
            }
        }
    }
};

__device__ inline uint32_t lds_u16(const char *p) { return *reinterpret_cast<const bf16_t *>(p); }

// ---- forward ---------------------------------------------------------------------------------
// pb0, pb1: the wave's two patch buffers (the patch of unit u + 1 lands while unit u is stored); stage: its
// staging block.  The three are distinct, which the qualifiers tell the compiler: a read of one then does
// not wait for a load into another.  Q8: the row length is a multiple of 8 pixels, so the 8-pixel pieces a
// lane stores are inside a row or outside it as a whole and the stores of a unit are always the same eight
// instructions (predicated per lane), which lets the wave leave them in flight while it goes on.
template <bool OUT_BF16, bool STATS, bool Q8>
__device__ __forceinline__ void smallc_fwd_body(const bf16_t *__restrict__ x, const bf16_t *__restrict__ w, void *__restrict__ y,
                                                const SmallProblem &p, char *__restrict__ pb0, char *__restrict__ pb1,
                                                char *__restrict__ stage, int wave)
{
    const int lane = threadIdx.x & 63;
    const int l32 = lane & 31, g = lane >> 5;
    const int k0 = blockIdx.y * KT;
    UnitWalk uw(p, lane);
    const __amdgpu_buffer_rsrc_t xr = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(x), 0, p.x_bytes, 0x00020000);

    // the filter operand: channel k0 + 32 i + l32, entries 16 b + 8 g .. + 7 (zeros past the last entry or channel)
    bf16x8 wreg[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            uint32_t d[4] = {0, 0, 0, 0};
            const int k = k0 + 32 * i + l32;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int j = 16 * b + 8 * g + e;
                const bool ok = k < p.K && j < p.CRS;
                const uint32_t v = w[ok ? (size_t)k * p.CRS + j : 0];
                d[e >> 1] |= (ok ? v : 0u) << (16 * (e & 1));
            }
            __builtin_memcpy(&wreg[i][b], d, 16);
        }
    // where the lane's pixel (l32 of the first 32; the second 32 are 32 sw columns on) finds its
    // reduction entries 16 b + 8 g + e in a patch; past the last entry any tap will do: the filter
    // operand is zero there
    int ga[2][8];
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int j = 16 * b + 8 * g + e;
            int off = 0;
            if (j < p.CRS) {
                const int c = j / p.RS, rem = j - c * p.RS, r = rem / p.S, s = rem - r * p.S;
                off = (c * p.R + r) * p.ppitch + s;
            }
            ga[b][e] = (off + p.shiftc + l32 * p.sw) * 2;
        }
    const int fstep = 32 * p.sw * 2;
    // the lane's share of the staged block on its way out: channel rows it * 8 + lane / 8, octet lane % 8
    const int oct = lane & 7, krow0 = lane >> 3;
    const uint32_t PQ2 = (uint32_t)(p.P * p.Q) * 2u;
    const uint32_t lane_y = (uint32_t)krow0 * PQ2 + (uint32_t)oct * 16u;
    const char *const sread = stage + krow0 * STG_PITCH + oct * 16;
    char *const swrite = stage + l32 * STG_PITCH + 8 * g;

    const int gw = blockIdx.x * WAVES + wave;   // this wave's number among those of the channel pass
    float cnt = 0.f, s1[2] = {0.f, 0.f}, s2[2] = {0.f, 0.f}, shift[2] = {0.f, 0.f};
    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

    auto unit = [&](const char *__restrict__ pcur, char *__restrict__ pnext, bool more) {
        const int n = uw.n, pr = uw.pr, q0 = uw.cb * UPX;
        // The loads that fill this unit's patch were sent before the last unit's stores; the compiler does not
        // count loads into LDS by itself, so wait here for everything this wave has sent.
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(0x0f70);   // vmcnt(0)
        __builtin_amdgcn_wave_barrier();
        asm volatile("" ::: "memory");
        f32x16 acc[2][2];   // [pixel group f][channel tile i]
#pragma unroll
        for (int f = 0; f < 2; ++f) {
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                uint32_t d[4];
#pragma unroll
                for (int e = 0; e < 8; e += 2)
                    d[e >> 1] = lds_u16(pcur + ga[b][e] + f * fstep) | (lds_u16(pcur + ga[b][e + 1] + f * fstep) << 16);
                bf16x8 a;
                __builtin_memcpy(&a, d, 16);
#pragma unroll
                for (int i = 0; i < 2; ++i)
                    acc[f][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, wreg[i][b], b == 0 ? zero : acc[f][i], 0, 0, 0);
            }
        }
        // the next unit's patch is on its way while this one is rounded, staged and stored
        if (more) {
            uw.advance();
            uw.patch_fetch(xr, pnext);
        }
        // acc[f][i][v]: channel k0 + 32 i + l32, pixel q0 + 32 f + 8 (v / 4) + 4 g + v % 4.  One pass over the
        // accumulators, four pixels at a time: rounded (bf16 output), into the statistics, into the staged
        // block (bf16), from where a lane stores 8 consecutive pixels of a channel, or to memory (fp32).
        const bool whole = q0 + UPX <= p.Q && k0 + KT <= p.K;   // no pixel and no channel of the block is past the end
        const bool first = cnt == 0.f;
        float add = 0.f;
        // rows of the block: 128 bytes of one channel each; a lane moves 16 of them
        char *const ub = reinterpret_cast<char *>(y) + (uint32_t)(((n * p.K + k0) * p.P + pr) * p.Q + q0) * 2u;
#pragma unroll
        for (int i = 0; i < 2; ++i) {   // 32 channels at a time through the staging block
            const int k = k0 + 32 * i + l32;
            if (STATS && first) shift[i] = OUT_BF16 ? __uint_as_float(pack2(acc[0][i][0], 0.f) << 16) : acc[0][i][0];
#pragma unroll
            for (int f = 0; f < 2; ++f)
#pragma unroll
                for (int jv = 0; jv < 4; ++jv) {
                    float v[4] = {acc[f][i][4 * jv], acc[f][i][4 * jv + 1], acc[f][i][4 * jv + 2], acc[f][i][4 * jv + 3]};
                    const int q = q0 + 32 * f + 8 * jv + 4 * g;
                    if (OUT_BF16) {
                        uint2 pk;
                        pk.x = pack2(v[0], v[1]);
                        pk.y = pack2(v[2], v[3]);
                        *reinterpret_cast<uint2 *>(swrite + (32 * f + 8 * jv) * 2) = pk;
                        if (STATS) {
                            v[0] = __uint_as_float(pk.x << 16);
                            v[1] = __uint_as_float(pk.x & 0xffff0000u);
                            v[2] = __uint_as_float(pk.y << 16);
                            v[3] = __uint_as_float(pk.y & 0xffff0000u);
                        }
                    } else {
                        float *const o32 = reinterpret_cast<float *>(y) + (uint32_t)(((n * p.K + k) * p.P + pr) * p.Q + q);
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (k < p.K && q + e < p.Q) o32[e] = v[e];
                    }
                    if (STATS) {
                        if (whole) {
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                const float d = v[e] - shift[i];
                                s1[i] += d;
                                s2[i] = __builtin_fmaf(d, d, s2[i]);
                            }
                        } else {
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                const bool ok = q + e < p.Q;
                                const float d = ok ? v[e] - shift[i] : 0.f;
                                s1[i] += d;
                                s2[i] = __builtin_fmaf(d, d, s2[i]);
                                if (i == 0) add += ok ? 1.f : 0.f;
                            }
                        }
                    }
                }
            if (OUT_BF16) {
                __builtin_amdgcn_wave_barrier();
                const int q = q0 + oct * 8;
                if (whole) {
#pragma unroll
                    for (int it = 0; it < 4; ++it) {
                        const u32x4 v = *reinterpret_cast<const u32x4 *>(sread + it * 8 * STG_PITCH);
                        store8_any(ub + (size_t)(32 * i + it * 8) * PQ2 + lane_y, v);
                    }
                } else {
#pragma unroll
                    for (int it = 0; it < 4; ++it) {
                        const u32x4 v = *reinterpret_cast<const u32x4 *>(sread + it * 8 * STG_PITCH);
                        char *const dst = ub + (size_t)(32 * i + it * 8) * PQ2 + lane_y;
                        const bool kok = k0 + 32 * i + it * 8 + krow0 < p.K;
                        if (Q8) {
                            if (kok && q < p.Q) store8_any(dst, v);
                        } else if (kok && q < p.Q) {
                            if (q + 8 <= p.Q) {
                                store8_any(dst, v);
                            } else {
                                bf16_t *const d16 = reinterpret_cast<bf16_t *>(dst);
#pragma unroll
                                for (int e = 0; e < 8; ++e)
                                    if (q + e < p.Q) d16[e] = (bf16_t)(v[e >> 1] >> (16 * (e & 1)));
                            }
                        }
                    }
                }
                __builtin_amdgcn_wave_barrier();
            }
        }
        cnt += whole ? 32.f : add;
    };

    if (gw < p.nunits) {
        uw.set_unit(gw);
        uw.patch_fetch(xr, pb0);
    }
    // two units per trip, so that which buffer is read and which is loaded is fixed in the code
    for (int u = gw; u < p.nunits; u += 2 * p.nwaves) {
        unit(pb0, pb1, u + p.nwaves < p.nunits);
        if (u + p.nwaves < p.nunits) unit(pb1, pb0, u + 2 * p.nwaves < p.nunits);
    }
    if (STATS) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            Moments3 m;
            m.n = cnt;
            m.mean = cnt > 0.f ? shift[i] + s1[i] / cnt : 0.f;
            m.m2 = cnt > 0.f ? fmaxf(s2[i] - s1[i] * s1[i] / cnt, 0.f) : 0.f;
            Moments3 o;
            o.n = __shfl_xor(m.n, 32);
            o.mean = __shfl_xor(m.mean, 32);
            o.m2 = __shfl_xor(m.m2, 32);
            const int k = k0 + 32 * i + l32;
            if (g == 0 && k < p.K) {
                m = join(m, o);
                float *e = p.stats + ((size_t)k * p.nwaves + gw) * 3;
                e[0] = m.n; e[1] = m.mean; e[2] = m.m2;
            }
        }
    }
}

template <bool OUT_BF16, bool STATS, bool Q8>
__global__ void __launch_bounds__(WAVES * 64) __attribute__((amdgpu_waves_per_eu(4, 4)))
smallc_fwd_kernel(const bf16_t *__restrict__ x, const bf16_t *__restrict__ w, void *__restrict__ y, SmallProblem p)
{
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    char *const mine = smem + wave * (2 * p.patch_bytes + STG_ROWS * STG_PITCH);
    smallc_fwd_body<OUT_BF16, STATS, Q8>(x, w, y, p, mine, mine + p.patch_bytes, mine + 2 * p.patch_bytes, wave);
}

// ---- backward-filter ----------------------------------------------------------------------------
// out: partial sums, slice blockIdx.x at out + blockIdx.x * K * CRS (use_atomics == 0), or dw itself,
// zero-filled, which every workgroup adds into (use_atomics != 0).
// The dy operand needs no staging: in NCHW a lane's 8 pixels of one channel are 16 contiguous bytes,
// loaded straight into the register the MFMA reads (a wave's load touches 32 channel planes, 32
// bytes of each; the four steps of a unit use up the 128-byte lines).  Unit u + 1 is loaded while unit
// u is multiplied.
template <bool Q8>
__device__ __forceinline__ void smallc_wgrad_body(const bf16_t *__restrict__ x, const bf16_t *__restrict__ dy,
                                                  float *__restrict__ out, int use_atomics, const SmallProblem &p,
                                                  char *__restrict__ pb0, char *__restrict__ pb1, float *__restrict__ red, int wave)
{
    const int lane = threadIdx.x & 63;
    const int l32 = lane & 31, g = lane >> 5;
    const int k0 = blockIdx.y * KT;
    UnitWalk uw(p, lane);
    const __amdgpu_buffer_rsrc_t xr = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(x), 0, p.x_bytes, 0x00020000);
    // the lane's reduction entry as an operand column: entry l32, pixels 8 g .. 8 g + 7 of a 16-pixel step
    // (entries past the last read any tap: their columns of the result are never written)
    int xa[8];
    {
        int off = 0;
        if (l32 < p.CRS) {
            const int c = l32 / p.RS, rem = l32 - c * p.RS, r = rem / p.S, s = rem - r * p.S;
            off = (c * p.R + r) * p.ppitch + s;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) xa[e] = (off + p.shiftc + (8 * g + e) * p.sw) * 2;
    }
    const int ststep = 16 * p.sw * 2;
    // dy operand of channel tile i, step st: channel k0 + 32 i + l32, pixels q0 + 16 st + 8 g .. + 7
    const uint32_t PQ2 = (uint32_t)(p.P * p.Q) * 2u;
    const uint32_t lane_y = (uint32_t)l32 * PQ2 + (uint32_t)g * 16u;
    const bool kok[2] = {k0 + l32 < p.K, k0 + 32 + l32 < p.K};
    auto dy_load = [&](u32x4 (&reg)[8]) {
        const int q0 = uw.cb * UPX;
        const char *const ub = reinterpret_cast<const char *>(dy) + (uint32_t)(((uw.n * p.K + k0) * p.P + uw.pr) * p.Q + q0) * 2u;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int st = 0; st < 4; ++st) {
                const int q = q0 + 16 * st + 8 * g;
                const char *const src = ub + (size_t)(32 * i) * PQ2 + 32 * st + lane_y;
                u32x4 v = {0, 0, 0, 0};
                if (Q8) {
                    if (kok[i] && q < p.Q) v = load8_any(src);
                } else if (kok[i] && q < p.Q) {
                    if (q + 8 <= p.Q) {
                        v = load8_any(src);
                    } else {
                        const bf16_t *const s16 = reinterpret_cast<const bf16_t *>(src);
                        uint32_t d[4] = {0, 0, 0, 0};
#pragma unroll
                        for (int e = 0; e < 8; ++e)
                            if (q + e < p.Q) d[e >> 1] |= (uint32_t)s16[e] << (16 * (e & 1));
                        v = u32x4{d[0], d[1], d[2], d[3]};
                    }
                }
                reg[i * 4 + st] = v;
            }
    };

    f32x16 acc[2];   // [channel tile i]: rows k, columns = reduction entries
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;

    const int gw = blockIdx.x * WAVES + wave;
    u32x4 yreg[2][8];
    // unit u: its patch is in pcur, its dy in ycur, both sent a unit ago
    auto unit = [&](const char *__restrict__ pcur, char *__restrict__ pnext, const u32x4 (&ycur)[8], u32x4 (&ynext)[8], bool more) {
        // Wait for them (everything this wave has in flight; the compiler does not count loads into LDS by
        // itself), then send the next unit's before the MFMAs: a wave always has a unit on its way.
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(0x0f70);   // vmcnt(0)
        __builtin_amdgcn_wave_barrier();
        asm volatile("" ::: "memory");
        if (more) {
            uw.advance();
            uw.patch_fetch(xr, pnext);
            dy_load(ynext);
        }
#pragma unroll
        for (int st = 0; st < 4; ++st) {   // 16 pixels per step
            uint32_t d[4];
#pragma unroll
            for (int e = 0; e < 8; e += 2)
                d[e >> 1] = lds_u16(pcur + xa[e] + st * ststep) | (lds_u16(pcur + xa[e + 1] + st * ststep) << 16);
            bf16x8 b;
            __builtin_memcpy(&b, d, 16);
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                bf16x8 a;
                __builtin_memcpy(&a, &ycur[i * 4 + st], 16);
                acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
            }
        }
    };
    if (gw < p.nunits) {
        uw.set_unit(gw);
        uw.patch_fetch(xr, pb0);
        dy_load(yreg[0]);
    }
    // two units per trip, so that which registers and which buffer a unit uses is fixed in the code
    for (int u = gw; u < p.nunits; u += 2 * p.nwaves) {
        unit(pb0, pb1, yreg[0], yreg[1], u + p.nwaves < p.nunits);
        if (u + p.nwaves < p.nunits) unit(pb1, pb0, yreg[1], yreg[0], u + 2 * p.nwaves < p.nunits);
    }

    // The workgroup's four waves add up through LDS (fixed order), then the slice is written.
    // acc[i][v]: column (entry) l32, row k0 + 32 i + 8 (v / 4) + 4 g + v % 4.
    __syncthreads();   // every wave is done with its patches: red takes their place
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) red[(wave * KT + 32 * i + 8 * (v / 4) + 4 * g + v % 4) * 33 + l32] = acc[i][v];
    __syncthreads();
    const size_t nw = (size_t)p.K * p.CRS;
    float *const dst = out + (use_atomics ? (size_t)0 : (size_t)blockIdx.x * nw);
    for (int e = threadIdx.x; e < KT * p.CRS; e += WAVES * 64) {
        const int kl = e / p.CRS, j = e - kl * p.CRS;
        if (k0 + kl >= p.K) continue;
        float s = red[kl * 33 + j];
#pragma unroll
        for (int wv = 1; wv < WAVES; ++wv) s += red[(wv * KT + kl) * 33 + j];
        const size_t o = (size_t)(k0 + kl) * p.CRS + j;
        if (use_atomics) unsafeAtomicAdd(dst + o, s);
        else dst[o] = s;
    }
}

template <bool Q8>
__global__ void __launch_bounds__(WAVES * 64) __attribute__((amdgpu_waves_per_eu(4, 4)))
smallc_wgrad_kernel(const bf16_t *__restrict__ x, const bf16_t *__restrict__ dy, float *__restrict__ out, int use_atomics,
                    SmallProblem p)
{
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    char *const mine = smem + wave * 2 * p.patch_bytes;
    smallc_wgrad_body<Q8>(x, dy, out, use_atomics, p, mine, mine + p.patch_bytes, reinterpret_cast<float *>(smem), wave);
}

// resident workgroups per compute unit: the kernels are built for four waves per SIMD
int workgroups_per_cu(size_t lds, bool) { return (int)std::min<size_t>(4, (160 * 1024) / lds); }

bool make_problem(const ConvGeom &g, bool wgrad, SmallProblem *p, dim3 *grid, size_t *lds)
{
    if (!g.in_bf16) return false;
    const long long crs = (long long)g.C * g.R * g.S;
    if (crs > RED) return false;
    // 32-bit byte offsets into x, dy and y (fp32 y: 4 bytes per element)
    const long long lim = 0x7fffffffLL;
    if ((long long)g.N * g.C * g.H * g.W * 2 > lim || (long long)g.N * g.K * g.P * g.Q * 4 > lim) return false;
    if (g.sh > 64 || g.sw > 64 || g.ph > 4096 || g.pw > 4096) return false;
    p->N = g.N; p->C = g.C; p->H = g.H; p->W = g.W; p->K = g.K; p->R = g.R; p->S = g.S;
    p->sh = g.sh; p->sw = g.sw; p->ph = g.ph; p->pw = g.pw; p->P = g.P; p->Q = g.Q;
    p->CRS = (int)crs; p->RS = g.R * g.S; p->CR = g.C * g.R;
    // A unit's patch always has the columns of 64 pixels, whatever the row's length, as aligned column
    // pairs (W even), starting at an even column: one left of the first tap where the padding is odd
    // (a unit starts at a multiple of 64 pixels).
    if (g.W % 2 != 0) return false;
    p->shiftc = g.pw & 1;
    const int pc = (UPX - 1) * g.sw + g.S + p->shiftc;
    p->ppitch = (pc + 1) & ~1;
    p->nslot = (p->ppitch / 2 + 63) / 64;
    if (p->nslot > 2) return false;
    p->patch_bytes = (int)align_up((size_t)p->CR * p->ppitch * 2, 16);
    p->ncb = (g.Q + UPX - 1) / UPX;
    const long long nunits = (long long)g.N * g.P * p->ncb;
    if (nunits > lim) return false;
    p->nunits = (int)nunits;
    p->out_bf16 = g.out_bf16;
    p->x_bytes = (int)((long long)g.N * g.C * g.H * g.W * 2);
    p->stats = nullptr;
    // per wave: two patch buffers, and forward's staging block; backward-filter's final sums reuse the space
    const size_t per_wave = 2 * (size_t)p->patch_bytes + (wgrad ? 0 : STG_ROWS * STG_PITCH);
    *lds = wgrad ? std::max(per_wave * WAVES, (size_t)WAVES * KT * 33 * sizeof(float)) : per_wave * WAVES;
    if (*lds > 160 * 1024) return false;
    const int ktiles = (g.K + KT - 1) / KT;
    if (ktiles > 65535) return false;
    const long long want = (nunits + WAVES - 1) / WAVES;
    const long long cap = 256LL * workgroups_per_cu(*lds, wgrad);
    const int gx = (int)std::max(1LL, std::min(want, cap));
    p->nwaves = gx * WAVES;
    const int per_img = g.P * p->ncb;
    p->dn = p->nwaves / per_img;
    p->dpr = (p->nwaves % per_img) / p->ncb;
    p->dcb = p->nwaves % p->ncb;
    *grid = dim3(gx, ktiles, 1);
    return true;
}

template <typename Kern>
hipError_t enable_lds(Kern kern)
{
    return hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
}

}  // namespace

bool smallc_supported(const ConvGeom &g)
{
    SmallProblem p;
    dim3 grid;
    size_t lds;
    return make_problem(g, false, &p, &grid, &lds) && make_problem(g, true, &p, &grid, &lds);
}

int smallc_fwd_stats_tiles(const ConvGeom &g)
{
    SmallProblem p;
    dim3 grid;
    size_t lds;
    return make_problem(g, false, &p, &grid, &lds) ? p.nwaves : 0;
}

hipError_t launch_smallc_fwd(const void *x, const void *w, void *y, const ConvGeom &g, hipStream_t st, float *stats)
{
    SmallProblem p;
    dim3 grid;
    size_t lds;
    if (!make_problem(g, false, &p, &grid, &lds)) return hipErrorInvalidValue;
    p.stats = stats;
    const bf16_t *xs = static_cast<const bf16_t *>(x), *wsrc = static_cast<const bf16_t *>(w);
    auto go = [&](auto kern) -> hipError_t {
        static const hipError_t attr = enable_lds(kern);   // one per instantiation of the lambda's call operator
        if (attr != hipSuccess) return attr;
        hipLaunchKernelGGL(kern, grid, dim3(WAVES * 64), lds, st, xs, wsrc, y, p);
        return hipGetLastError();
    };
    const bool q8 = g.Q % 8 == 0;
    if (g.out_bf16) {
        if (q8) return stats ? go(smallc_fwd_kernel<true, true, true>) : go(smallc_fwd_kernel<true, false, true>);
        return stats ? go(smallc_fwd_kernel<true, true, false>) : go(smallc_fwd_kernel<true, false, false>);
    }
    return stats ? go(smallc_fwd_kernel<false, true, false>) : go(smallc_fwd_kernel<false, false, false>);
}

int smallc_wgrad_slices(const ConvGeom &g)
{
    SmallProblem p;
    dim3 grid;
    size_t lds;
    return make_problem(g, true, &p, &grid, &lds) ? (int)grid.x : 0;
}

// partial == nullptr: the workgroups add into a zero-filled dw with atomics; otherwise workgroup z
// writes partial[z][K*C*R*S] (smallc_wgrad_slices of them) and a reduction in slice order follows.
hipError_t launch_smallc_wgrad(const void *x, const void *dy, float *dw, const ConvGeom &g, float *partial, hipStream_t st)
{
    SmallProblem p;
    dim3 grid;
    size_t lds;
    if (!make_problem(g, true, &p, &grid, &lds)) return hipErrorInvalidValue;
    const size_t nw = (size_t)g.K * p.CRS;
    const bool direct_store = !partial && grid.x == 1;
    if (!partial && !direct_store) {
        hipError_t e = launch_fill_zero(dw, nw, st);
        if (e != hipSuccess) return e;
    }
    const bf16_t *xs = static_cast<const bf16_t *>(x), *ds = static_cast<const bf16_t *>(dy);
    float *out = partial ? partial : dw;
    const int atomics = (!partial && !direct_store) ? 1 : 0;
    auto go = [&](auto kern) -> hipError_t {
        static const hipError_t attr = enable_lds(kern);
        if (attr != hipSuccess) return attr;
        hipLaunchKernelGGL(kern, grid, dim3(WAVES * 64), lds, st, xs, ds, out, atomics, p);
        return hipSuccess;
    };
    hipError_t e0 = g.Q % 8 == 0 ? go(smallc_wgrad_kernel<true>) : go(smallc_wgrad_kernel<false>);
    if (e0 != hipSuccess) return e0;
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (partial) return launch_reduce_partials(partial, dw, nw, (int)grid.x, false, st);
    return hipSuccess;
}

}  // namespace sn
