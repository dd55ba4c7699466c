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
// for 16 consecutive k or c).  Global loads are 16 bytes wide whatever their
// alignment.  The (n,p,q) sum is split over gridDim.z slices; a slice either
// adds its result into a zeroed dw with fp32 atomics (no workspace) or writes
// partial[slice], which is then reduced in slice order.  Either way the
// accumulators go through LDS first so that global accesses are coalesced.
//
// One workgroup per CU (the 9 accumulator tiles plus the staging registers need
// more than 256 registers per lane), so the overlap is inside the workgroup: LDS
// is double buffered, the global loads of chunk i+1 fly during the MFMAs of chunk
// i and are written to the other buffer half way through them; one barrier per
// chunk.  With a single wave per SIMD every non-MFMA instruction costs issue
// time, so everything that depends only on the thread is worked out once.
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
    int ctiles;                  // c tiles
    // how the valid columns of a staged octet are found:
    //  0: a chunk spans the whole image width, the mask is fixed per thread
    //  1: column tiles and W a multiple of 8: an octet is wholly inside or outside the row
    //  2: column tiles and ragged W: recomputed per chunk
    int colmode;
};

struct __attribute__((packed, aligned(2))) U16x8 { unsigned short e[8]; };

__device__ inline uint4 load8_any(const bf16_t *p)
{
    U16x8 v = *reinterpret_cast<const U16x8 *>(p);
    uint4 o;
    __builtin_memcpy(&o, &v, 16);
    return o;
}

// Bit mask of the columns v0 .. v0+7 that lie inside a row of width W.
__device__ inline uint32_t col_mask(int v0, int W)
{
    const int lo = min(8, max(0, -v0)), hi = max(0, min(8, W - v0));
    return hi > lo ? (((1u << hi) - 1u) & ~((1u << lo) - 1u)) : 0u;
}

// Moves the elements of an octet down by sh positions (element sh becomes element 0).
__device__ inline uint4 shift_down(uint4 r, uint32_t sh)
{
    const unsigned long long lo = r.x | ((unsigned long long)r.y << 32), hi = r.z | ((unsigned long long)r.w << 32);
    const uint32_t bits = sh * 16;
    unsigned long long nlo, nhi;
    if (bits >= 64) { nlo = hi >> (bits - 64); nhi = 0; }
    else { nlo = (lo >> bits) | (bits ? hi << (64 - bits) : 0ull); nhi = hi >> bits; }
    return make_uint4((uint32_t)nlo, (uint32_t)(nlo >> 32), (uint32_t)nhi, (uint32_t)(nhi >> 32));
}

// Clears the columns of an octet that are not in vm.
__device__ inline uint4 apply_mask(uint4 r, uint32_t vm)
{
    uint32_t *d = reinterpret_cast<uint32_t *>(&r);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t b0 = (vm >> (2 * j)) & 1u, b1 = (vm >> (2 * j + 1)) & 1u;
        d[j] &= ((0u - b0) & 0xffffu) | ((0u - b1) & 0xffff0000u);
    }
    return r;
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

// desc of a staged octet: LDS element offset (bits 0-15) | chunk row (16-20) | 8-bit field (21-28)
__device__ inline int desc_lds(int d) { return d & 0xffff; }
__device__ inline int desc_row(int d) { return (d >> 16) & 31; }
__device__ inline int desc_f8(int d) { return (d >> 21) & 255; }

template <int S, int RG, int TM, int TC, int COLMODE>
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

    // ---- staging items of this thread: dy octets (KTB*NSG in all) and x octets (CTB*xrows*NGX).
    // desc: see above; its 8-bit field is the fixed column mask (colmode 0) or the octet's column
    // index (colmode 1, 2).  goff: element offset inside the chunk frame, -1 if the item's channel
    // is out of range (the item then always stores zeros).
    constexpr int YIT = (KTB * (PIXC_MAX / 8) + 255) / 256;
    constexpr int XIT_MAX = 10;
    uint4 yreg[YIT], xreg[XIT_MAX];
    uint32_t yinfo[(YIT + 1) / 2], xinfo[(XIT_MAX + 1) / 2];   // per staged octet: column mask | shift << 8
    const int ny = KTB * NSG, nx = CTB * p.xrows * NGX;
    const int xper = p.xrows * NGX;
    int ydesc[YIT], ygoff[YIT], xdesc[XIT_MAX], xgoff[XIT_MAX];
#pragma unroll
    for (int it = 0; it < YIT; ++it) {
        const int e = it * 256 + tid;
        ydesc[it] = -1;
        ygoff[it] = -1;
        if (e < ny) {
            const int kl = e / NSG, sg = e - kl * NSG;
            const int rl = sg / OPR, oc = sg - rl * OPR;
            const int f8 = COLMODE == 0 ? (int)col_mask(oc * 8, p.Q) : oc;
            ydesc[it] = (kl * p.AP + sg * 8) | (rl << 16) | (f8 << 21);
            if (k0 + kl < p.K) ygoff[it] = (k0 + kl) * PQ + rl * p.Q + oc * 8;
        }
    }
#pragma unroll
    for (int it = 0; it < XIT_MAX; ++it) {
        const int e = it * 256 + tid;
        xdesc[it] = -1;
        xgoff[it] = -1;
        if (e < nx) {
            const int cl = e / xper, r2 = e - cl * xper;
            const int row = r2 / NGX, og = r2 - row * NGX;
            const int f8 = COLMODE == 0 ? (int)col_mask(og * 8 - p.apr, p.W) : og;
            xdesc[it] = (cl * p.CP + r2 * 8) | (row << 16) | (f8 << 21);
            if (c0 + cl < p.C) xgoff[it] = (c0 + cl) * HW + row * p.W + og * 8;
        }
    }
    const unsigned ytotal = (unsigned)p.N * p.K * PQ, xtotal = (unsigned)p.N * p.C * HW;

    // chunk coordinates, advanced incrementally
    int c_img = 0, c_rc = 0, c_ct = 0;
    auto set_chunk = [&](int chunk) {
        c_img = chunk / (p.rowchunks * p.ncoltiles);
        const int rem = chunk - c_img * (p.rowchunks * p.ncoltiles);
        c_rc = rem / p.ncoltiles;
        c_ct = rem - c_rc * p.ncoltiles;
    };
    auto next_chunk = [&]() {
        if (++c_ct == p.ncoltiles) {
            c_ct = 0;
            if (++c_rc == p.rowchunks) { c_rc = 0; ++c_img; }
        }
    };

    // Issues the loads of the current chunk coordinates into yreg / xreg.  Straight-line code, so
    // that the compiler keeps all of a chunk's loads in flight: an octet that is not wanted (row
    // outside the image, columns all outside the row, channel out of range) is still loaded, from
    // element 0 of the tensor, with mask 0, and stage_store turns it into zeros.  An octet that
    // hangs over the end of its row is loaded whole and masked later; if it would run past the
    // end of the tensor itself the load starts sh elements earlier and stage_store shifts it back.
    // info keeps mask | sh << 8 per octet, two octets per register.
    auto prefetch = [&]() {
        const int p0 = c_rc * p.TH, q0 = c_ct * p.TWP;
        const int h0 = p0 + r0 - p.ph;
        const int ychunk = c_img * p.K * PQ + p0 * p.Q + q0;
        const int xchunk = c_img * p.C * HW + h0 * p.W + q0 - p.apr;
        const int yrows = p.P - p0;            // chunk rows below this are inside the image
#pragma unroll
        for (int i = 0; i < (YIT + 1) / 2; ++i) yinfo[i] = 0;
#pragma unroll
        for (int i = 0; i < (XIT_MAX + 1) / 2; ++i) xinfo[i] = 0;
#pragma unroll
        for (int it = 0; it < YIT; ++it) {
            const int d = ydesc[it];
            uint32_t vm = desc_f8(d);
            if (COLMODE == 1) vm = (q0 + (int)vm * 8 < p.Q) ? 0xffu : 0u;
            if (COLMODE == 2) vm = col_mask(q0 + (int)vm * 8, p.Q);
            if (ygoff[it] < 0 || desc_row(d) >= yrows) vm = 0;
            unsigned off = vm ? (unsigned)(ychunk + ygoff[it]) : 0u;
            uint32_t sh = 0;
            if (COLMODE != 1) {
                sh = off + 8u > ytotal ? off + 8u - ytotal : 0u;
                off -= sh;
            }
            yinfo[it >> 1] |= (vm | (sh << 8)) << (16 * (it & 1));
            yreg[it] = load8_any(dy + off);
        }
#pragma unroll
        for (int it = 0; it < XIT_MAX; ++it) {
            if (it * 256 >= nx) break;
            const int d = xdesc[it];
            uint32_t vm = desc_f8(d);
            if (COLMODE == 1) vm = ((unsigned)(q0 - p.apr + (int)vm * 8) < (unsigned)p.W) ? 0xffu : 0u;
            if (COLMODE == 2) vm = col_mask(q0 - p.apr + (int)vm * 8, p.W);
            if (xgoff[it] < 0 || (unsigned)(h0 + desc_row(d)) >= (unsigned)p.H) vm = 0;
            unsigned off = vm ? (unsigned)(xchunk + xgoff[it]) : 0u;
            uint32_t sh = 0;
            if (COLMODE != 1) {
                sh = off + 8u > xtotal ? off + 8u - xtotal : 0u;
                off -= sh;
            }
            xinfo[it >> 1] |= (vm | (sh << 8)) << (16 * (it & 1));
            xreg[it] = load8_any(x + off);
        }
    };

    // Writes the staged octets to LDS, clearing the columns that are not wanted.
    auto stage_store = [&](int buf) {
        bf16_t *ys = smem + buf * bufstride, *xs = ys + YS_MAX;
#pragma unroll
        for (int it = 0; it < YIT; ++it) {
            const int d = ydesc[it];
            if (d < 0) continue;
            const uint32_t info = (yinfo[it >> 1] >> (16 * (it & 1))) & 0xffffu, vm = info & 0xffu;
            uint4 v = yreg[it];
            if (COLMODE != 1 && (info >> 8)) v = shift_down(v, info >> 8);
            if (vm != 0xffu) v = apply_mask(v, vm);
            *reinterpret_cast<uint4 *>(ys + desc_lds(d)) = v;
        }
#pragma unroll
        for (int it = 0; it < XIT_MAX; ++it) {
            if (it * 256 >= nx) break;
            const int d = xdesc[it];
            if (d < 0) continue;
            const uint32_t info = (xinfo[it >> 1] >> (16 * (it & 1))) & 0xffffu, vm = info & 0xffu;
            uint4 v = xreg[it];
            if (COLMODE != 1 && (info >> 8)) v = shift_down(v, info >> 8);
            if (vm != 0xffu) v = apply_mask(v, vm);
            *reinterpret_cast<uint4 *>(xs + desc_lds(d)) = v;
        }
    };

    // One step = 16 pixel slots: the A operands and, per filter row, the aligned octet of x plus
    // the neighbours the column shifts need.  The LDS reads of step j+1 are issued before the
    // MFMAs of step j (two register sets, loop unrolled by two).
    struct Frag {
        bf16x8 a[TM];
        uint4 m[RG][TC];
        uint32_t lo[RG][TC][2], hi[RG][TC][2];
    };
    auto load_frag = [&](Frag &f, const bf16_t *ys, const bf16_t *xs, int j) {
        const int oct = 2 * j + g;
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
            f.a[tm] = *reinterpret_cast<const bf16x8 *>(ys + ((wk * TM + tm) * 32 + l32) * p.AP + oct * 8);
        const int xo = steptab[oct];
#pragma unroll
        for (int rl = 0; rl < RG; ++rl)
#pragma unroll
            for (int tc = 0; tc < TC; ++tc) {
                const bf16_t *src = xs + ((wc * TC + tc) * 32 + l32) * p.CP + xo + rl * p.LWX;
                f.m[rl][tc] = *reinterpret_cast<const uint4 *>(src);
                if (S == 3) {
                    f.lo[rl][tc][0] = 0;
                    f.lo[rl][tc][1] = (uint32_t)src[-1] << 16;
                    f.hi[rl][tc][0] = src[8];
                    f.hi[rl][tc][1] = 0;
                } else if (S > 3) {
                    const uint2 l2 = *reinterpret_cast<const uint2 *>(src - 4);
                    const uint2 h2 = *reinterpret_cast<const uint2 *>(src + 8);
                    f.lo[rl][tc][0] = l2.x; f.lo[rl][tc][1] = l2.y;
                    f.hi[rl][tc][0] = h2.x; f.hi[rl][tc][1] = h2.y;
                } else {
                    f.lo[rl][tc][0] = f.lo[rl][tc][1] = f.hi[rl][tc][0] = f.hi[rl][tc][1] = 0;
                }
            }
    };
    auto mma_frag = [&](const Frag &f) {
#pragma unroll
        for (int rl = 0; rl < RG; ++rl) {
            uint32_t D[TC][8];
#pragma unroll
            for (int tc = 0; tc < TC; ++tc) {
                D[tc][0] = f.lo[rl][tc][0]; D[tc][1] = f.lo[rl][tc][1];
                D[tc][2] = f.m[rl][tc].x; D[tc][3] = f.m[rl][tc].y; D[tc][4] = f.m[rl][tc].z; D[tc][5] = f.m[rl][tc].w;
                D[tc][6] = f.hi[rl][tc][0]; D[tc][7] = f.hi[rl][tc][1];
            }
            TapLoop<S, TC, TM, 0>::run(D, f.a, acc, rl);
        }
    };
    auto compute = [&](int buf) {
        const bf16_t *ys = smem + buf * bufstride, *xs = ys + YS_MAX;
        Frag f0, f1;
        load_frag(f0, ys, xs, 0);
        int j = 0;
        for (; j + 2 <= p.nsteps; j += 2) {
            load_frag(f1, ys, xs, j + 1);
            mma_frag(f0);
            if (j + 2 < p.nsteps) load_frag(f0, ys, xs, j + 2);
            mma_frag(f1);
        }
        if (j < p.nsteps) mma_frag(f0);
    };

    const int cbeg = blockIdx.z * p.cps, cend = min(p.nchunks, cbeg + p.cps);
    if (cbeg < cend) {
        set_chunk(cbeg);
        prefetch();
        stage_store(0);
    }
    __syncthreads();
    for (int chunk = cbeg, buf = 0; chunk < cend; ++chunk, buf ^= 1) {
        const bool more = chunk + 1 < cend;
        if (more) {
            next_chunk();
            prefetch();
        }
        compute(buf);
        if (more) stage_store(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue.  An accumulator tile keeps column c = lane % 32 and rows k = 8*(v/4) +
    // 4*(lane/32) + v%4 in register v.  Four passes (v/4 = 0..3) each move KTB/4 rows of the
    // workgroup's dw block through LDS as [row][c*T + t], from where consecutive lanes write
    // consecutive addresses of dw[k][c][r][s].
    constexpr int ROWS = KTB / 4, ROWLEN = CTB * T, EP = ROWLEN + 1;
    float *stage = reinterpret_cast<float *>(smem);
    const int Tall = p.R * S;
    float *dst = out + (use_atomics ? (size_t)0 : (size_t)blockIdx.z * p.K * p.C * Tall);
#pragma unroll
    for (int ps = 0; ps < 4; ++ps) {
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int tc = 0; tc < TC; ++tc)
#pragma unroll
                for (int t = 0; t < T; ++t)
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int rr = ((wk * TM + tm) * 2 + g) * 4 + i;
                        stage[rr * EP + ((wc * TC + tc) * 32 + l32) * T + t] = acc[tm][tc][t][4 * ps + i];
                    }
        __syncthreads();
        for (int e = tid; e < ROWS * ROWLEN; e += 256) {
            const int rr = e / ROWLEN, j = e - rr * ROWLEN;
            const int cl = j / T, t = j - cl * T;
            // rr = ((wk*TM + tm)*2 + g)*4 + i  ->  k = k0 + (wk*TM + tm)*32 + 8*ps + 4*g + i
            const int k = k0 + (rr >> 3) * 32 + 8 * ps + (rr & 7);
            const int c = c0 + cl;
            if (k < p.K && c < p.C && r0 * S + t < Tall) {
                const size_t off = ((size_t)k * p.C + c) * Tall + r0 * S + t;
                const float val = stage[rr * EP + j];
                if (use_atomics) unsafeAtomicAdd(dst + off, val);
                else dst[off] = val;
            }
        }
        __syncthreads();
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

bool make_wplan(const ConvGeom &g, WPlan *pl)
{
    if (!g.in_bf16 || g.sh != 1 || g.sw != 1) return false;
    if (g.S != 1 && g.S != 3 && g.S != 5 && g.S != 7) return false;
    if (g.pw != (g.S - 1) / 2) return false;      // the column shift is built for "same" padding
    if (g.Q != g.W) return false;
    int RG, TM = 1, TC = 1;
    if (g.S == 1 && g.R == 1) { RG = 1; TM = 2; TC = 2; }
    else if (g.S == 3 && g.R == 3) RG = 3;
    else if (g.S == 1 && g.R == 7) RG = 7;
    else if (g.S == 5 && g.R == 5) RG = 3;   // two groups of three filter rows; the sixth row is not written
    else if (g.S == 7 && g.R == 1) RG = 1;
    else return false;
    const long long lim = 0x7fffffffLL;
    if ((long long)g.N * g.C * g.H * g.W + 64 > lim || (long long)g.N * g.K * g.P * g.Q + 64 > lim) return false;
    if ((long long)g.N * g.C * g.H * g.W < 8 || (long long)g.N * g.K * g.P * g.Q < 8) return false;   // 16-byte loads
    WgradProblem p;
    p.N = g.N; p.C = g.C; p.H = g.H; p.W = g.W; p.K = g.K; p.P = g.P; p.Q = g.Q; p.R = g.R; p.ph = g.ph;
    if (g.Q <= 64) { p.TWP = (g.Q + 7) / 8 * 8; p.ncoltiles = 1; p.colmode = 0; }
    else { p.TWP = 32; p.ncoltiles = (g.Q + 31) / 32; p.colmode = (g.W % 8 == 0) ? 1 : 2; }
    int th = PIXC_MAX / p.TWP;
    if (th > g.P) th = g.P;
    while (th > 1 && (th * p.TWP) % 16 != 0) --th;
    if ((th * p.TWP) % 16 != 0) th = 2;      // a single row of 8, 24, 40 or 56 slots: pad to a row pair
    p.TH = th;
    p.nsteps = p.TH * p.TWP / 16;
    if (p.TH * p.TWP > PIXC_MAX || p.TH > 31) return false;
    p.apr = g.S > 1 ? 8 : 0;
    p.LWX = p.TWP + 2 * p.apr;
    p.xrows = p.TH + RG - 1;
    if (p.xrows > 31) return false;
    p.AP = odd16(p.TH * p.TWP);
    p.CP = odd16(p.xrows * p.LWX);
    const int KTB = 2 * TM * 32, CTB = 2 * TC * 32;
    const long long nx = (long long)CTB * p.xrows * (p.LWX / 8);
    if (nx > 10 * 256) return false;
    if ((long long)CTB * p.CP > 65535 || (long long)KTB * p.AP > 65535) return false;   // LDS offsets are 16 bits
    p.rowchunks = (g.P + p.TH - 1) / p.TH;
    const long long nch = (long long)g.N * p.rowchunks * p.ncoltiles;
    if (nch > lim) return false;
    p.nchunks = (int)nch;
    const int nrg = (g.R + RG - 1) / RG;
    p.ctiles = (g.C + CTB - 1) / CTB;
    const int ktiles = (g.K + KTB - 1) / KTB;
    if (ktiles > 65535) return false;
    const long long tiles = (long long)p.ctiles * nrg * ktiles;
    // slices: about two workgroups per CU in all; every slice costs a pass over dw in the epilogue
    long long slices = (512 + tiles - 1) / tiles;
    if (slices > p.nchunks) slices = p.nchunks;
    if (slices > 65535) slices = 65535;
    if (slices < 1) slices = 1;
    p.cps = (int)((p.nchunks + slices - 1) / slices);
    slices = (p.nchunks + p.cps - 1) / p.cps;
    pl->p = p;
    pl->grid = dim3(p.ctiles * nrg, ktiles, (unsigned)slices);
    const size_t stage_bytes = 2 * ((size_t)KTB * (PIXC_MAX + 8) + (size_t)CTB * p.CP) * sizeof(bf16_t);  // double buffered
    const size_t epi_bytes = (size_t)(KTB / 4) * (CTB * RG * g.S + 1) * sizeof(float);
    pl->smem = stage_bytes > epi_bytes ? stage_bytes : epi_bytes;
    if (pl->smem > 156 * 1024) return false;
    pl->S = g.S; pl->RG = RG; pl->TM = TM; pl->TC = TC;
    return true;
}

template <int S, int RG, int TM, int TC, int COLMODE>
hipError_t launch_mode(const bf16_t *x, const bf16_t *dy, float *out, int atomics, const WPlan &pl, hipStream_t st)
{
    // dynamic LDS beyond 64 KB has to be enabled once per kernel
    static const hipError_t attr =
        hipFuncSetAttribute(reinterpret_cast<const void *>(&conv_wgrad_kernel<S, RG, TM, TC, COLMODE>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, 156 * 1024);
    if (attr != hipSuccess) return attr;
    hipLaunchKernelGGL((conv_wgrad_kernel<S, RG, TM, TC, COLMODE>), pl.grid, dim3(256), pl.smem, st, x, dy, out,
                       atomics, pl.p);
    return hipGetLastError();
}

template <int S, int RG, int TM, int TC>
hipError_t launch_cfg(const bf16_t *x, const bf16_t *dy, float *out, int atomics, const WPlan &pl, hipStream_t st)
{
    if (pl.p.colmode == 0) return launch_mode<S, RG, TM, TC, 0>(x, dy, out, atomics, pl, st);
    if (pl.p.colmode == 1) return launch_mode<S, RG, TM, TC, 1>(x, dy, out, atomics, pl, st);
    return launch_mode<S, RG, TM, TC, 2>(x, dy, out, atomics, pl, st);
}

}  // namespace

bool tile_wgrad_supported(const ConvGeom &g)
{
    WPlan pl;
    return pointwise_wgrad_supported(g) || rows_wgrad_supported(g) || make_wplan(g, &pl);
}

// The kernel that takes the shape with partial sums is the row-stationary one, whose slice count can be capped.
bool tile_wgrad_cappable(const ConvGeom &g) { return !pointwise_wgrad_supported(g) && rows_wgrad_supported(g); }

int tile_wgrad_slices(const ConvGeom &g, int cap)
{
    if (pointwise_wgrad_supported(g)) return pointwise_wgrad_slices(g);
    if (rows_wgrad_supported(g)) return rows_wgrad_slices(g, cap);
    WPlan pl;
    return make_wplan(g, &pl) ? (int)pl.grid.z : 0;
}

// partial == nullptr: slices add into dw with atomics (dw is zero-filled first);
// otherwise slice z writes partial[z][K*C*R*S] and a reduction in slice order follows.
hipError_t launch_tile_wgrad(const void *x, const void *dy, float *dw, const ConvGeom &g, float *partial,
                             hipStream_t st, int cap)
{
    if (pointwise_wgrad_supported(g)) return launch_pointwise_wgrad(x, dy, dw, g, partial, st);
    WPlan pl;
    // 5x5 on the row-stationary kernel is five launches, a filter row each: with partial sums and one reduction
    // that is twice as fast as this file's kernel (measured 344 against 680 us on 96 -> 256 channels, 27x27),
    // with five rounds of atomics it is slower (758 against 700 us)
    const bool rows5 = g.R == 5 && !partial && make_wplan(g, &pl);
    if (rows_wgrad_supported(g) && !rows5) return launch_rows_wgrad(x, dy, dw, g, partial, st, partial ? cap : 0);
    if (!make_wplan(g, &pl)) return hipErrorInvalidValue;
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
    else if (pl.S == 5) e = launch_cfg<5, 3, 1, 1>(xs, ds, out, atomics, pl, st);
    else e = launch_cfg<7, 1, 1, 1>(xs, ds, out, atomics, pl, st);
    if (e != hipSuccess) return e;
    if (partial) return launch_reduce_partials(partial, dw, nw, slices, false, st);
    return hipSuccess;
}

}  // namespace sn
