// Stride-1 bf16 backward-filter on gfx950 MFMA (Sec. 3.5 of the paper; the
// definition is in sn.h):  dw[k,c,r,s] = sum_{n,p,q} dy[n,k,p,q] * x[n,c,p+r-ph,q+s-pw].
//
// As a GEMM the reduction runs over output pixels, and in NCHW both operands are
// already contiguous along that axis (dy rows, and x rows shifted by the tap), so
// nothing has to be transposed: an MFMA lane holds 8 consecutive pixels of one
// row of dy (A operand, rows = k) or of x (B operand, columns = c).  A tap (r,s)
// is a different *shift* of the same x row, which gives one 32x32 accumulator
// tile per tap: a wave owns 32 k x 32 c x all taps of its group (9 tiles for 3x3).
//
// A 256-thread workgroup owns (2*TM*32) k x (2*TC*32) c x RG*S taps and walks a
// slice of the (n,p,q) sum in chunks of TH output rows x TWP columns of one
// image (TWP = Q rounded up to 8 for images up to 64 wide, else 32-column
// tiles).  Per chunk it stages in LDS
//   ys[k][slot]      the dy rows, slot = row*TWP + col, zero beyond the image,
//   xs[c][row][col]  the x rows with an 8-column apron on both sides, so that
//                    every 16-byte LDS access stays aligned while the tap shift
//                    s - pw of up to 3 columns is made in registers: a lane reads
//                    its aligned 8 pixels plus the neighbours it needs and builds
//                    each shifted operand with funnel shifts (v_alignbit).
// Row pitches are padded to an odd number of 16-byte units (conflict-free reads
// for 16 consecutive k or c).  Global loads are 16 bytes wide wherever the 8
// pixels lie inside the image row (whatever their alignment) and element-wise at
// the row ends.  The (n,p,q) sum is split over gridDim.z slices; a slice either
// adds its result into a zeroed dw with fp32 atomics (no workspace) or writes
// partial[slice], which is then reduced in slice order.
//
// One workgroup per CU (the 9 accumulator tiles plus the staging registers need
// more than 256 registers per lane), so the overlap is inside the workgroup: LDS
// is double buffered, the global loads of chunk i+1 fly during the MFMAs of chunk
// i and are written to the other buffer half way through them; one barrier per chunk.
#include "sn_internal.h"

namespace sn {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int PIXC_MAX = 128;   // pixel slots per chunk

struct WgradProblem {
    int N, C, H, W, K, P, Q, R, ph;
    int TH, TWP, LWX, xrows;     // chunk rows, slot columns, x row pitch, x rows = TH + RG - 1
    int apr;                     // apron columns on each side of an x row in LDS (8, or 0 when S = 1)
    int AP, CP;                  // LDS pitches (elements) of a dy row and of an x channel
    int nsteps;                  // TH*TWP/16
    int ncoltiles, rowchunks;    // per image
    int nchunks, cps;            // total chunks, chunks per slice
    int nrg;                     // tap-row groups (R / RG), folded into blockIdx.y
    int ctiles;                  // c tiles
};

struct __attribute__((packed, aligned(2))) U16x8 { unsigned short e[8]; };

__device__ inline uint4 load8_any(const bf16_t *p)
{
    U16x8 v = *reinterpret_cast<const U16x8 *>(p);
    uint4 o;
    __builtin_memcpy(&o, &v, 16);
    return o;
}

// 8 pixels starting at column v0 of a row of width W (row pointer `row`), zero outside [0,W).
__device__ inline uint4 load_row8(const bf16_t *row, int v0, int W)
{
    if (v0 >= 0 && v0 + 8 <= W) return load8_any(row + v0);
    unsigned short e[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int v = v0 + i;
        e[i] = (v >= 0 && v < W) ? row[v] : (unsigned short)0;
    }
    return make_uint4(e[0] | ((uint32_t)e[1] << 16), e[2] | ((uint32_t)e[3] << 16), e[4] | ((uint32_t)e[5] << 16),
                      e[6] | ((uint32_t)e[7] << 16));
}

// Elements d .. d+7 of a window whose dwords D[0..7] hold elements -4 .. 11.
template <int d> __device__ inline bf16x8 shifted(const uint32_t (&D)[8])
{
    constexpr int e0 = 4 + d;
    uint32_t o[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (e0 % 2 == 0) o[i] = D[e0 / 2 + i];
        else o[i] = __builtin_amdgcn_alignbit(D[(e0 + 1) / 2 + i], D[(e0 - 1) / 2 + i], 16);
    }
    bf16x8 r;
    __builtin_memcpy(&r, o, 16);
    return r;
}

template <int S, int TC, int TM, int s> struct TapLoop {
    template <typename Acc>
    __device__ static inline void run(const uint32_t (&D)[TC][8], const bf16x8 (&a)[TM], Acc &acc, int rl)
    {
        constexpr int PW = (S - 1) / 2;
#pragma unroll
        for (int tc = 0; tc < TC; ++tc) {
            const bf16x8 b = shifted<s - PW>(D[tc]);
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
                acc[tm][tc][rl * S + s] =
                    __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[tm], b, acc[tm][tc][rl * S + s], 0, 0, 0);
        }
        TapLoop<S, TC, TM, s + 1>::run(D, a, acc, rl);
    }
};
template <int S, int TC, int TM> struct TapLoop<S, TC, TM, S> {
    template <typename Acc>
    __device__ static inline void run(const uint32_t (&)[TC][8], const bf16x8 (&)[TM], Acc &, int) {}
};

template <int S, int RG, int TM, int TC>
__global__ void __launch_bounds__(256, 1)
conv_wgrad_kernel(const bf16_t *__restrict__ x, const bf16_t *__restrict__ dy, float *__restrict__ out,
                  int use_atomics, WgradProblem p)
{
    constexpr int T = RG * S, KTB = 2 * TM * 32, CTB = 2 * TC * 32;
    constexpr int YS_MAX = KTB * (PIXC_MAX + 8);
    extern __shared__ __attribute__((aligned(16))) bf16_t smem[];
    const int bufstride = YS_MAX + CTB * p.CP;   // elements per buffer: dy rows, then x channels
    __shared__ int steptab[2 * PIXC_MAX / 16];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, g = lane >> 5;
    const int wk = wave >> 1, wc = wave & 1;
    const int ctile = blockIdx.x % p.ctiles, rgi = blockIdx.x / p.ctiles;
    const int c0 = ctile * CTB, k0 = blockIdx.y * KTB, r0 = rgi * RG;
    const int OPR = p.TWP >> 3;          // octets per slot row
    const int NSG = p.nsteps * 2;        // octets (8-slot groups) per dy row
    const int NGX = p.LWX >> 3;          // octets per x row
    const int PQ = p.P * p.Q, HW = p.H * p.W;

    if (tid < NSG) {
        const int rl = tid / OPR, col = (tid - rl * OPR) * 8;
        steptab[tid] = rl * p.LWX + p.apr + col;
    }

    f32x16 acc[TM][TC][T];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TC; ++b)
#pragma unroll
            for (int t = 0; t < T; ++t)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[a][b][t][v] = 0.f;

    // staging items per thread: dy octets KTB*NSG, x octets CTB*xrows*NGX.  What depends on the
    // item only is worked out once (integer division by run-time values is slow): the LDS offset,
    // the row and column octet inside the chunk (packed), and the global offset inside the image.
    constexpr int YIT = (KTB * (PIXC_MAX / 8) + 255) / 256;
    constexpr int XIT_MAX = 10;
    uint4 yreg[YIT], xreg[XIT_MAX];
    const int ny = KTB * NSG, nx = CTB * p.xrows * NGX;
    const int xper = p.xrows * NGX;
    int ydesc[YIT], ygoff[YIT], xdesc[XIT_MAX], xgoff[XIT_MAX];   // desc = ldsoff | row << 16 | octet << 24 | zero-fill << 30; -1: no item
#pragma unroll
    for (int it = 0; it < YIT; ++it) {
        const int e = it * 256 + tid;
        ydesc[it] = -1;
        ygoff[it] = 0;
        if (e < ny) {
            const int kl = e / NSG, sg = e - kl * NSG;
            const int rl = sg / OPR, oc = sg - rl * OPR;
            if (k0 + kl < p.K) {
                ydesc[it] = (kl * p.AP + sg * 8) | (rl << 16) | (oc << 24);
                ygoff[it] = (k0 + kl) * PQ + rl * p.Q;
            } else {
                ydesc[it] = (kl * p.AP + sg * 8) | (1 << 30);   // k beyond K: zero fill
            }
        }
    }
#pragma unroll
    for (int it = 0; it < XIT_MAX; ++it) {
        const int e = it * 256 + tid;
        xdesc[it] = -1;
        xgoff[it] = 0;
        if (e < nx) {
            const int cl = e / xper, r2 = e - cl * xper;
            const int row = r2 / NGX, og = r2 - row * NGX;
            if (c0 + cl < p.C) {
                xdesc[it] = (cl * p.CP + r2 * 8) | (row << 16) | (og << 24);
                xgoff[it] = (c0 + cl) * HW + row * p.W;
            } else {
                xdesc[it] = (cl * p.CP + r2 * 8) | (1 << 30);   // c beyond C: zero fill
            }
        }
    }

    auto prefetch = [&](int chunk) {
        const int img = chunk / (p.rowchunks * p.ncoltiles);
        const int rem = chunk - img * (p.rowchunks * p.ncoltiles);
        const int rc = rem / p.ncoltiles, ct = rem - rc * p.ncoltiles;
        const int p0 = rc * p.TH, q0 = ct * p.TWP;
        const bf16_t *ybase = dy + (size_t)img * p.K * PQ + (size_t)p0 * p.Q;
        const int h0 = p0 + r0 - p.ph;
        const bf16_t *xbase = x + (size_t)img * p.C * HW + (ptrdiff_t)h0 * p.W;
#pragma unroll
        for (int it = 0; it < YIT; ++it) {
            uint4 v = make_uint4(0, 0, 0, 0);
            const int d = ydesc[it];
            if (d >= 0 && !(d >> 30)) {
                const int rl = (d >> 16) & 0xff, oc = d >> 24;
                if (p0 + rl < p.P) v = load_row8(ybase + ygoff[it], q0 + oc * 8, p.Q);
            }
            yreg[it] = v;
        }
#pragma unroll
        for (int it = 0; it < XIT_MAX; ++it) {
            if (it * 256 >= nx) break;
            uint4 v = make_uint4(0, 0, 0, 0);
            const int d = xdesc[it];
            if (d >= 0 && !(d >> 30)) {
                const int row = (d >> 16) & 0xff, og = d >> 24;
                if ((unsigned)(h0 + row) < (unsigned)p.H) v = load_row8(xbase + xgoff[it], q0 - p.apr + og * 8, p.W);
            }
            xreg[it] = v;
        }
    };

    auto stage_store = [&](int buf) {
        bf16_t *ys = smem + buf * bufstride, *xs = ys + YS_MAX;
#pragma unroll
        for (int it = 0; it < YIT; ++it)
            if (ydesc[it] >= 0) *reinterpret_cast<uint4 *>(ys + (ydesc[it] & 0xffff)) = yreg[it];
#pragma unroll
        for (int it = 0; it < XIT_MAX; ++it) {
            if (it * 256 >= nx) break;
            if (xdesc[it] >= 0) *reinterpret_cast<uint4 *>(xs + (xdesc[it] & 0xffff)) = xreg[it];
        }
    };

    auto compute = [&](int buf, int jbeg, int jend) {
        const bf16_t *ys = smem + buf * bufstride, *xs = ys + YS_MAX;
        for (int j = jbeg; j < jend; ++j) {
            const int oct = 2 * j + g;
            bf16x8 a[TM];
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
                a[tm] = *reinterpret_cast<const bf16x8 *>(ys + ((wk * TM + tm) * 32 + l32) * p.AP + oct * 8);
            const int xo = steptab[oct];
#pragma unroll
            for (int rl = 0; rl < RG; ++rl) {
                uint32_t D[TC][8];
#pragma unroll
                for (int tc = 0; tc < TC; ++tc) {
                    const bf16_t *src = xs + ((wc * TC + tc) * 32 + l32) * p.CP + xo + rl * p.LWX;
                    const uint4 m = *reinterpret_cast<const uint4 *>(src);
                    D[tc][2] = m.x; D[tc][3] = m.y; D[tc][4] = m.z; D[tc][5] = m.w;
                    if (S == 1) {
                        D[tc][0] = D[tc][1] = D[tc][6] = D[tc][7] = 0;
                    } else if (S == 3) {
                        D[tc][0] = 0;
                        D[tc][1] = (uint32_t)src[-1] << 16;
                        D[tc][6] = src[8];
                        D[tc][7] = 0;
                    } else {
                        const uint2 lo = *reinterpret_cast<const uint2 *>(src - 4);
                        const uint2 hi = *reinterpret_cast<const uint2 *>(src + 8);
                        D[tc][0] = lo.x; D[tc][1] = lo.y; D[tc][6] = hi.x; D[tc][7] = hi.y;
                    }
                }
                TapLoop<S, TC, TM, 0>::run(D, a, acc, rl);
            }
        }
    };

    const int cbeg = blockIdx.z * p.cps, cend = min(p.nchunks, cbeg + p.cps);
    if (cbeg < cend) {
        prefetch(cbeg);
        stage_store(0);
    }
    __syncthreads();
    const int half = p.nsteps >> 1;
    for (int chunk = cbeg, buf = 0; chunk < cend; ++chunk, buf ^= 1) {
        const bool more = chunk + 1 < cend;
        if (more) prefetch(chunk + 1);
        compute(buf, 0, half);
        if (more) stage_store(buf ^ 1);
        compute(buf, half, p.nsteps);
        __syncthreads();
    }

    // ---- epilogue: tile rows are k (8*(v/4) + 4*(lane/32) + v%4), columns c (lane % 32)
    const int Tall = p.R * S;
    float *dst = out + (use_atomics ? (size_t)0 : (size_t)blockIdx.z * p.K * p.C * Tall);
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int tc = 0; tc < TC; ++tc) {
            const int c = c0 + (wc * TC + tc) * 32 + l32;
            if (c >= p.C) continue;
#pragma unroll
            for (int t = 0; t < T; ++t)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int k = k0 + (wk * TM + tm) * 32 + 8 * (v >> 2) + 4 * g + (v & 3);
                    if (k >= p.K) continue;
                    const size_t off = ((size_t)k * p.C + c) * Tall + r0 * S + t;
                    if (use_atomics) unsafeAtomicAdd(dst + off, acc[tm][tc][t][v]);
                    else dst[off] = acc[tm][tc][t][v];
                }
        }
}

struct WPlan {
    WgradProblem p;
    dim3 grid;
    size_t smem;
    int S, RG, TM, TC;
};

int odd16(int elems)  // pitch in elements: a multiple of 8 whose count of 16-byte units is odd
{
    int units = (elems + 7) / 8;
    if (units % 2 == 0) ++units;
    return units * 8;
}

bool make_wplan(const ConvGeom &g, int want_slices, WPlan *pl)
{
    if (!g.in_bf16 || g.sh != 1 || g.sw != 1) return false;
    if (g.S != 1 && g.S != 3 && g.S != 5 && g.S != 7) return false;
    if (g.pw != (g.S - 1) / 2) return false;      // the column shift is built for "same" padding
    if (g.Q != g.W) return false;
    int RG, TM = 1, TC = 1;
    if (g.S == 1 && g.R == 1) { RG = 1; TM = 2; TC = 2; }
    else if (g.S == 3 && g.R == 3) RG = 3;
    else if (g.S == 1 && g.R == 7) RG = 7;
    else if ((g.S == 5 && g.R == 5) || (g.S == 7 && g.R == 1)) RG = 1;
    else return false;
    const long long lim = 0x7fffffffLL;
    if ((long long)g.N * g.C * g.H * g.W > lim || (long long)g.N * g.K * g.P * g.Q > lim) return false;
    WgradProblem p;
    p.N = g.N; p.C = g.C; p.H = g.H; p.W = g.W; p.K = g.K; p.P = g.P; p.Q = g.Q; p.R = g.R; p.ph = g.ph;
    if (g.Q <= 64) { p.TWP = (g.Q + 7) / 8 * 8; p.ncoltiles = 1; }
    else { p.TWP = 32; p.ncoltiles = (g.Q + 31) / 32; }
    int th = PIXC_MAX / p.TWP;
    if (th > g.P) th = g.P;
    while (th > 1 && (th * p.TWP) % 16 != 0) --th;
    if ((th * p.TWP) % 16 != 0) {      // a single row of 8, 24, 40 or 56 slots: pad the row pair
        th = 2;
    }
    p.TH = th;
    p.nsteps = p.TH * p.TWP / 16;
    if (p.TH * p.TWP > PIXC_MAX) return false;
    p.apr = g.S > 1 ? 8 : 0;
    p.LWX = p.TWP + 2 * p.apr;
    p.xrows = p.TH + RG - 1;
    p.AP = odd16(p.TH * p.TWP);
    p.CP = odd16(p.xrows * p.LWX);
    const int KTB = 2 * TM * 32, CTB = 2 * TC * 32;
    const long long nx = (long long)CTB * p.xrows * (p.LWX / 8);
    if (nx > 10 * 256) return false;
    p.rowchunks = (g.P + p.TH - 1) / p.TH;
    const long long nch = (long long)g.N * p.rowchunks * p.ncoltiles;
    if (nch > lim) return false;
    p.nchunks = (int)nch;
    p.nrg = g.R / RG;
    p.ctiles = (g.C + CTB - 1) / CTB;
    const int ktiles = (g.K + KTB - 1) / KTB;
    if (ktiles > 65535) return false;
    const long long tiles = (long long)p.ctiles * p.nrg * ktiles;
    long long slices = want_slices > 0 ? want_slices : (768 + tiles - 1) / tiles;
    if (slices > p.nchunks) slices = p.nchunks;
    if (slices > 65535) slices = 65535;
    if (slices < 1) slices = 1;
    p.cps = (int)((p.nchunks + slices - 1) / slices);
    slices = (p.nchunks + p.cps - 1) / p.cps;
    pl->p = p;
    pl->grid = dim3(p.ctiles * p.nrg, ktiles, (unsigned)slices);
    pl->smem = 2 * ((size_t)KTB * (PIXC_MAX + 8) + (size_t)CTB * p.CP) * sizeof(bf16_t);  // double buffered
    if (pl->smem > 156 * 1024) return false;
    pl->S = g.S; pl->RG = RG; pl->TM = TM; pl->TC = TC;
    return true;
}

template <int S, int RG, int TM, int TC>
hipError_t launch_cfg(const bf16_t *x, const bf16_t *dy, float *out, int atomics, const WPlan &pl, hipStream_t st)
{
    // dynamic LDS beyond 64 KB has to be enabled once per kernel
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(&conv_wgrad_kernel<S, RG, TM, TC>),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, 156 * 1024);
    if (attr != hipSuccess) return attr;
    hipLaunchKernelGGL((conv_wgrad_kernel<S, RG, TM, TC>), pl.grid, dim3(256), pl.smem, st, x, dy, out, atomics, pl.p);
    return hipGetLastError();
}

}  // namespace

bool tile_wgrad_supported(const ConvGeom &g)
{
    WPlan pl;
    return make_wplan(g, 0, &pl);
}

int tile_wgrad_slices(const ConvGeom &g)
{
    WPlan pl;
    return make_wplan(g, 0, &pl) ? (int)pl.grid.z : 0;
}

// partial == nullptr: slices add into dw with atomics (dw is zero-filled first);
// otherwise slice z writes partial[z][K*C*R*S] and a reduction in slice order follows.
hipError_t launch_tile_wgrad(const void *x, const void *dy, float *dw, const ConvGeom &g, float *partial,
                             hipStream_t st)
{
    WPlan pl;
    if (!make_wplan(g, 0, &pl)) return hipErrorInvalidValue;
    const size_t nw = (size_t)g.K * g.C * g.R * g.S;
    const int slices = (int)pl.grid.z;
    const bool direct_store = !partial && slices == 1;
    float *out = partial ? partial : dw;
    if (!partial && !direct_store) {
        hipError_t e = launch_fill_zero(dw, nw, st);
        if (e != hipSuccess) return e;
    }
    const int atomics = (!partial && !direct_store) ? 1 : 0;
    const bf16_t *xs = static_cast<const bf16_t *>(x), *ds = static_cast<const bf16_t *>(dy);
    hipError_t e;
    if (pl.S == 3) e = launch_cfg<3, 3, 1, 1>(xs, ds, out, atomics, pl, st);
    else if (pl.S == 1 && pl.RG == 1) e = launch_cfg<1, 1, 2, 2>(xs, ds, out, atomics, pl, st);
    else if (pl.S == 1) e = launch_cfg<1, 7, 1, 1>(xs, ds, out, atomics, pl, st);
    else if (pl.S == 5) e = launch_cfg<5, 1, 1, 1>(xs, ds, out, atomics, pl, st);
    else e = launch_cfg<7, 1, 1, 1>(xs, ds, out, atomics, pl, st);
    if (e != hipSuccess) return e;
    if (partial) return launch_reduce_partials(partial, dw, nw, slices, false, st);
    return hipSuccess;
}

}  // namespace sn
