// Stride-1 bf16 backward-filter for 3x3 ("same" column padding) and 1x1 filters on
// gfx950 MFMA, row-stationary form (Sec. 3.5 of the paper; the definition is in sn.h):
//   dw[k,c,r,s] = sum_{n,p,q} dy[n,k,p,q] * x[n,c,p+r-ph,q+s-pw].
//
// The reduction runs over output pixels, and in NCHW both operands are contiguous
// along an image row, so nothing is transposed: an MFMA lane holds 8 consecutive
// pixels of one row of dy (A operand, rows = k) or of x (B operand, columns = c).
// A tap (r,s) pairs dy row p with x row p+r-ph shifted by s-pw columns, one 32x32
// accumulator tile per tap.  A wave owns TM*32 k x 32 c x all taps; a 256-thread
// workgroup owns (2*TM*32) k x 64 c and walks a slice of the (n,p,q) sum in chunks
// of TH output rows x TWP columns of one image (128 pixels).  Per chunk it stages
//   ys[k][row][col]   the dy rows,
//   xs[c][row][col]   the TH+R-1 x rows, with an 8-column apron on both sides so that
//                     every 16-byte LDS access stays aligned.
// The inner loop is stationary in the x row: for one x row and 16 columns a lane
// reads its aligned 8 pixels and the two neighbours, builds the S column-shifted
// operands with funnel shifts once, and uses them for every filter row r, i.e.
// against the dy rows p = xrow - r, which sit in a rolling window of registers
// (each dy operand is read from LDS once).  That is 4 LDS reads and 8 VALU
// operations per 9*TM MFMAs for a 3x3 filter.
//
// Staging.  A thread always handles the same 8-column octet of a row, so what
// depends on the column (validity, the mask of a ragged last octet) is fixed per
// thread.  Global loads are 16 bytes wide whatever their alignment and branch free:
// an octet that is not wanted (row outside the image, channel out of range, column
// tile past the row end) is read from a page of zeros instead.  LDS is double
// buffered: the loads of chunk i+1 fly during the MFMAs of chunk i; one barrier per
// chunk.  One workgroup per CU (LDS holds two buffers of 55 KB).
//
// The (n,p,q) sum is split over gridDim.z slices; a slice either adds its result
// into a zeroed dw with fp32 atomics (no workspace) or writes partial[slice], which
// is then reduced in slice order.  Either way the accumulators go through LDS first
// so that global accesses are coalesced.
#include "sn_internal.h"

namespace sn {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Never written: the source of every load that must bring zeros.
__device__ __attribute__((aligned(16))) uint32_t zero_page[4];

constexpr int CTB = 64;   // c per workgroup

constexpr int odd16c(int elems)   // pitch in elements: a multiple of 8 whose count of 16-byte units is odd
{
    const int u = (elems + 7) / 8;
    return (u % 2 ? u : u + 1) * 8;
}

struct RowsProblem {
    int N, C, H, W, K, P, Q, R, ph;
    int rowchunks, ncoltiles;   // chunks per image
    int nchunks, cps;           // total chunks, chunks per slice
    int ctiles, ktiles;
    int xcd_slices;             // > 0: one-dimensional grid, this many slices per XCD
    int nslices;                // with xcd_slices > 0: slice z takes the chunks z, z + nslices, ...
    int Tfull, toff;            // taps of the whole filter; the first tap this launch computes (a launch may take some filter rows only)
};

struct __attribute__((packed, aligned(2))) U128u { u32x4 v; };
__device__ inline u32x4 load8_any(const bf16_t *p) { return reinterpret_cast<const U128u *>(p)->v; }

// Moves the elements of an octet down by sh (1..7) positions (element sh becomes element 0).
__device__ inline u32x4 shift_down(u32x4 r, int sh)
{
    const unsigned long long lo = r.x | ((unsigned long long)r.y << 32), hi = r.z | ((unsigned long long)r.w << 32);
    const int bits = sh * 16;
    unsigned long long nlo, nhi;
    if (bits >= 64) { nlo = hi >> (bits - 64); nhi = 0; }
    else { nlo = (lo >> bits) | (hi << (64 - bits)); nhi = hi >> bits; }
    u32x4 o = {(uint32_t)nlo, (uint32_t)(nlo >> 32), (uint32_t)nhi, (uint32_t)(nhi >> 32)};
    return o;
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

// S: filter width (1, 3, 5 or 7), RG: filter rows of this launch (R, or 1 of the 5 rows of a 5x5 filter), TM: the workgroup owns 2*TM*32 k, TH x TWP: chunk,
// WIDE: 32-column tiles of an image whose width is a multiple of 8 (otherwise the chunk spans the
// whole width, which may be ragged), TP: 2 = two sets of waves share the k x c tile and split the
// chunk's 16-column groups between them (their accumulators are added in the epilogue): a second
// wave per SIMD where K is too small for TM = 2.
template <int S, int RG, int TM, int TH, int TWP, bool WIDE, int TP>
__global__ void __launch_bounds__(TM * TP * 256) __attribute__((amdgpu_waves_per_eu(TM * TP, TM * TP)))
wgrad_rows_kernel(const bf16_t *__restrict__ x, const bf16_t *__restrict__ dy, float *__restrict__ out,
                  int use_atomics, RowsProblem p)
{
    constexpr int T = RG * S, KTB = 2 * TM * 32, NT = TM * TP * 256;   // 4*TM*TP waves: TP sets of 2*TM along k x 2 along c
    constexpr int OPR = TWP / 8, TPR = NT / OPR;      // octets per row; threads per octet column
    constexpr int XROWS = TH + RG - 1, APR = S > 1 ? 8 : 0, LWX = TWP + 2 * APR;
    constexpr int AP = odd16c(TH * TWP), CP = odd16c(XROWS * LWX);
    constexpr int YS = KTB * AP, XS = CTB * CP, BUF = YS + XS;   // elements
    constexpr int NCG = TWP / 16;
    static_assert(NCG % TP == 0, "the column groups do not split over the wave sets");
    // staging items of a thread: dy (k, row), x (c, row), apron (c, row, side)
    constexpr int YKREP = KTB >= TPR ? KTB / TPR : 1, YRPT = KTB >= TPR ? 1 : TPR / KTB;
    constexpr int YIT = KTB >= TPR ? TH * YKREP : TH / YRPT;
    constexpr int XCREP = CTB >= TPR ? CTB / TPR : 1, XRPT = CTB >= TPR ? 1 : TPR / CTB;
    constexpr int XIT = CTB >= TPR ? XROWS * XCREP : (XROWS + XRPT - 1) / XRPT;
    constexpr bool APRON = WIDE && S > 1;   // a whole-width chunk has nothing beside it
    constexpr int AIT = APRON ? (CTB * XROWS * 2 + NT - 1) / NT : 0;
    constexpr bool RAGGED = !WIDE;
    static_assert(TH % YRPT == 0, "rows do not split over the threads");
    extern __shared__ __attribute__((aligned(16))) bf16_t smem[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, g = lane >> 5;
    const int wk = (wave >> 1) % (2 * TM), wc = wave & 1, ph = wave / (4 * TM);   // ph: which set of waves
    // Which tile and slice.  With a one-dimensional grid (p.xcd_slices > 0) workgroup L runs on XCD
    // L % 8 (round-robin dispatch), and every XCD has an L2 of its own: each XCD gets a contiguous
    // range of slices, and the tiles of one slice, which read the same x and dy rows, follow each
    // other on the same XCD.
    int ctile, ktile, zslice;
    if (p.xcd_slices > 0) {
        const int tiles = p.ctiles * p.ktiles, jx = blockIdx.x >> 3, t = jx % tiles;
        zslice = (blockIdx.x & 7) * p.xcd_slices + jx / tiles;
        ctile = t % p.ctiles;
        ktile = t / p.ctiles;
    } else {
        ctile = blockIdx.x; ktile = blockIdx.y; zslice = blockIdx.z;
    }
    const int c0 = ctile * CTB, k0 = ktile * KTB;
    const int PQ = p.P * p.Q, HW = p.H * p.W;
    const int ytotal = p.N * p.K * PQ, xtotal = p.N * p.C * HW;
    const bf16_t *const zp = reinterpret_cast<const bf16_t *>(zero_page);

    // the aprons of a whole-width chunk are never written: zero for good
    if (!WIDE && S > 1) {
        for (int i = tid; i < 2 * CTB * XROWS * 2; i += NT) {
            const int buf = i / (CTB * XROWS * 2), rem = i - buf * (CTB * XROWS * 2);
            const int c = rem / (XROWS * 2), r2 = rem - c * (XROWS * 2);
            bf16_t *dst = smem + buf * BUF + YS + c * CP + (r2 >> 1) * LWX + ((r2 & 1) ? APR + TWP : 0);
            *reinterpret_cast<u32x4 *>(dst) = u32x4{0, 0, 0, 0};
        }
    }

    constexpr int WTM = 1;   // k tiles per wave
    f32x16 acc[WTM][T];
#pragma unroll
    for (int a = 0; a < WTM; ++a)
#pragma unroll
        for (int t = 0; t < T; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][t][v] = 0.f;

    // ---- per-thread constants of the staging
    const int oc = tid % OPR, tq = tid / OPR;
    auto y_row = [&](int it) { return KTB >= TPR ? it / YKREP : it * YRPT + tq / KTB; };
    auto y_k = [&](int it) { return KTB >= TPR ? (it % YKREP) * TPR + tq : tq % KTB; };
    auto x_row = [&](int it) { return CTB >= TPR ? it / XCREP : it * XRPT + tq / CTB; };
    auto x_c = [&](int it) { return CTB >= TPR ? (it % XCREP) * TPR + tq : tq % CTB; };
    const bool col_in = WIDE || oc * 8 < p.Q;   // whole-width chunk: fixed; tiles: checked per chunk
    // element offset inside the chunk frame; never wanted: -1 (the left apron can be at -8: NEVER)
    constexpr int NEVER = -(1 << 30);
    int ygoff[YIT], xgoff[XIT], agoff[APRON ? AIT : 1];
#pragma unroll
    for (int it = 0; it < YIT; ++it)
        ygoff[it] = (k0 + y_k(it) < p.K && col_in) ? (k0 + y_k(it)) * PQ + y_row(it) * p.Q + oc * 8 : -1;
#pragma unroll
    for (int it = 0; it < XIT; ++it)
        xgoff[it] = (c0 + x_c(it) < p.C && col_in && x_row(it) < XROWS) ? (c0 + x_c(it)) * HW + x_row(it) * p.W + oc * 8 : -1;
    const int aside = tid & 1, ac = (tid >> 1) & (CTB - 1);   // apron item it: side, c, row (it * NT + tid) / 128
    auto a_row = [&](int it) { return (it * NT + tid) >> 7; };
    if (APRON) {
#pragma unroll
        for (int it = 0; it < AIT; ++it)
            agoff[it] = (c0 + ac < p.C && a_row(it) < XROWS) ? (c0 + ac) * HW + a_row(it) * p.W + (aside ? TWP : -8) : NEVER;
    }
    // the valid columns of this thread's octet as dword masks (whole-width chunks only)
    u32x4 cmask = {~0u, ~0u, ~0u, ~0u};
    if (RAGGED) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int e = oc * 8 + 2 * j;
            cmask[j] = (e < p.Q ? 0xffffu : 0u) | (e + 1 < p.Q ? 0xffff0000u : 0u);
        }
    }

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

    // ---- staging, one item (a 16-byte octet) at a time.  The items of the next chunk are
    // loaded and written to the other LDS buffer in between the MFMAs of the current chunk (see
    // compute), a few at a time: a burst of all of them would wait for the L1 cache to take them
    // while the MFMA pipe runs dry.  Items 0 .. YIT-1 are dy octets, then XIT x octets, then the
    // aprons.  Nothing looks at what a load returns before it is written to LDS.  A ragged last
    // octet of the tensor is read from 8 elements before the end and moved back into place.
    constexpr int NITEMS = YIT + XIT + AIT;
    u32x4 sreg[NITEMS];
    int k_p0 = 0, k_q0 = 0, k_h0 = 0, k_ybase = 0, k_xbase = 0;   // of the chunk being staged
    bool k_colok = true;
    auto begin_chunk = [&]() {
        k_p0 = c_rc * TH;
        k_q0 = WIDE ? c_ct * TWP : 0;
        k_h0 = k_p0 - p.ph;
        k_ybase = c_img * p.K * PQ + k_p0 * p.Q + k_q0;
        k_xbase = c_img * p.C * HW + k_h0 * p.W + k_q0;
        k_colok = !WIDE || k_q0 + oc * 8 < p.Q;
    };
    auto item_load = [&](int i) {
        if (i < YIT) {
            const int it = i;
            const bool ok = ygoff[it] >= 0 && k_p0 + y_row(it) < p.P && k_colok;
            int off = k_ybase + ygoff[it];
            if (RAGGED) off = min(off, ytotal - 8);
            sreg[i] = load8_any(ok ? dy + off : zp);
        } else if (i < YIT + XIT) {
            const int it = i - YIT;
            const bool ok = xgoff[it] >= 0 && (unsigned)(k_h0 + x_row(it)) < (unsigned)p.H && k_colok;
            int off = k_xbase + xgoff[it];
            if (RAGGED) off = min(off, xtotal - 8);
            sreg[i] = load8_any(ok ? x + off : zp);
        } else {
            const int it = i - YIT - XIT;
            const bool ok = agoff[it] != NEVER && (unsigned)(k_h0 + a_row(it)) < (unsigned)p.H &&
                            (aside ? k_q0 + TWP < p.W : k_q0 > 0);
            sreg[i] = load8_any(ok ? x + (k_xbase + agoff[it]) : zp);
        }
    };
    const int ylds0 = (KTB >= TPR ? tq : tq % KTB) * AP + (KTB >= TPR ? 0 : (tq / KTB) * TWP) + oc * 8;
    const int xlds0 = (CTB >= TPR ? tq : tq % CTB) * CP + (CTB >= TPR ? 0 : (tq / CTB) * LWX) + APR + oc * 8;
    const int alds0 = ac * CP + (aside ? APR + TWP : 0);
    auto item_store = [&](int i, int buf) {
        bf16_t *ys = smem + buf * BUF, *xs = ys + YS;
        u32x4 v = sreg[i];
        if (i < YIT) {
            const int it = i;
            if (RAGGED) {
                const int over = k_ybase + ygoff[it] + 8 - ytotal;
                if (ygoff[it] >= 0 && k_p0 + y_row(it) < p.P && over > 0) v = shift_down(v, over);
                v &= cmask;
            }
            const int o = KTB >= TPR ? (it % YKREP) * TPR * AP + (it / YKREP) * TWP : it * YRPT * TWP;
            *reinterpret_cast<u32x4 *>(ys + ylds0 + o) = v;
        } else if (i < YIT + XIT) {
            const int it = i - YIT;
            if (RAGGED) {
                const int over = k_xbase + xgoff[it] + 8 - xtotal;
                if (xgoff[it] >= 0 && (unsigned)(k_h0 + x_row(it)) < (unsigned)p.H && over > 0) v = shift_down(v, over);
                v &= cmask;
            }
            const int o = CTB >= TPR ? (it % XCREP) * TPR * CP + (it / XCREP) * LWX : it * XRPT * LWX;
            if (x_row(it) < XROWS) *reinterpret_cast<u32x4 *>(xs + xlds0 + o) = v;
        } else {
            const int it = i - YIT - XIT;
            if (a_row(it) < XROWS) *reinterpret_cast<u32x4 *>(xs + alds0 + a_row(it) * LWX) = v;
        }
    };

    // ---- the MFMAs of one chunk
    const int ylane = (wk * WTM * 32 + l32) * AP + 8 * g;
    const int xlane = (wc * 32 + l32) * CP + APR + 8 * g;
    struct Raw {
        u32x4 m;
        uint32_t lo, hi, lo2, hi2;   // the elements beside the octet (S = 7: lo2 and hi2 are the outer pairs)
    };
    constexpr int NCGW = NCG / TP;       // column groups per wave
    constexpr int NSTEP = NCGW * XROWS;  // (column group, x row) steps of a chunk, per wave
    // An item is written to LDS LAG items after its load.  With one wave per SIMD nothing else
    // covers the latency of the loads: they are all issued in the first half of the chunk and
    // written after its last MFMA.
    constexpr bool LONE = TM * TP == 1;
    constexpr int LAG = LONE ? NITEMS : 4;
    auto compute = [&](int buf) {
        const bf16_t *ys = smem + buf * BUF + ylane, *xs = smem + buf * BUF + YS + xlane;
        auto load_raw = [&](Raw &r, int cg, int xr) {
            const bf16_t *src = xs + xr * LWX + cg * 16;
            r.m = *reinterpret_cast<const u32x4 *>(src);
            if (S == 3) {
                r.lo = src[-1];
                r.hi = src[8];
            } else if (S == 5) {   // two elements on either side, as dwords
                r.lo = *reinterpret_cast<const uint32_t *>(src - 2);
                r.hi = *reinterpret_cast<const uint32_t *>(src + 8);
            } else if (S == 7) {   // four on either side (three are used)
                const uint2 lo = *reinterpret_cast<const uint2 *>(src - 4), hi = *reinterpret_cast<const uint2 *>(src + 8);
                r.lo2 = lo.x; r.lo = lo.y; r.hi = hi.x; r.hi2 = hi.y;
            }
        };
        auto load_a = [&](bf16x8 (&a)[WTM], int cg, int row) {
#pragma unroll
            for (int tm = 0; tm < WTM; ++tm)
                a[tm] = *reinterpret_cast<const bf16x8 *>(ys + tm * 32 * AP + row * TWP + cg * 16);
        };
#pragma unroll
        for (int cgi = 0; cgi < NCGW; ++cgi) {
            const int cg = cgi * TP + ph;
            bf16x8 aw[RG + 1][WTM];   // dy rows in flight, by row % (RG + 1)
            Raw raw[2];
            load_raw(raw[0], cg, 0);
            load_a(aw[0], cg, 0);
#pragma unroll
            for (int xr = 0; xr < XROWS; ++xr) {
                if (xr + 1 < XROWS) load_raw(raw[(xr + 1) & 1], cg, xr + 1);
                if (xr + 1 < TH) load_a(aw[(xr + 1) % (RG + 1)], cg, xr + 1);
                __builtin_amdgcn_sched_barrier(0);   // the reads of the next row stay ahead of this row's MFMAs
                const Raw &r = raw[xr & 1];
                bf16x8 b[S];
                if (S == 3) {
                    // elements -1 .. 8 of the row: lo, the octet, hi
                    const uint32_t D[8] = {0, r.lo << 16, r.m.x, r.m.y, r.m.z, r.m.w, r.hi, 0};
                    b[0] = shifted<-1>(D);
                    b[1] = shifted<0>(D);
                    b[S - 1] = shifted<1>(D);
                } else if (S == 5) {
                    // elements -2 .. 9 of the row
                    const uint32_t D[8] = {0, r.lo, r.m.x, r.m.y, r.m.z, r.m.w, r.hi, 0};
                    b[0] = shifted<-2>(D);
                    b[1] = shifted<-1>(D);
                    b[2] = shifted<0>(D);
                    b[S > 3 ? 3 : 0] = shifted<1>(D);
                    b[S - 1] = shifted<2>(D);
                } else if (S == 7) {
                    // elements -4 .. 11 of the row
                    const uint32_t D[8] = {r.lo2, r.lo, r.m.x, r.m.y, r.m.z, r.m.w, r.hi, r.hi2};
                    b[0] = shifted<-3>(D);
                    b[S > 1 ? 1 : 0] = shifted<-2>(D);
                    b[S > 2 ? 2 : 0] = shifted<-1>(D);
                    b[S > 3 ? 3 : 0] = shifted<0>(D);
                    b[S > 4 ? 4 : 0] = shifted<1>(D);
                    b[S > 5 ? 5 : 0] = shifted<2>(D);
                    b[S - 1] = shifted<3>(D);
                } else {
                    __builtin_memcpy(&b[0], &r.m, 16);
                }
#pragma unroll
                for (int fr = 0; fr < RG; ++fr) {
                    const int pl = xr - fr;   // the dy row that meets this x row in filter row fr
                    if (pl < 0 || pl >= TH) continue;
#pragma unroll
                    for (int s = 0; s < S; ++s)
#pragma unroll
                        for (int tm = 0; tm < WTM; ++tm)
                            acc[tm][fr * S + s] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                                aw[pl % (RG + 1)][tm], b[s], acc[tm][fr * S + s], 0, 0, 0);
                }
                // this step's share of the next chunk's staging
                const int st = cgi * XROWS + xr;
                const int lo = min(NITEMS, st * NITEMS * (LONE ? 2 : 1) / NSTEP);
                const int hi = min(NITEMS, (st + 1) * NITEMS * (LONE ? 2 : 1) / NSTEP);
#pragma unroll
                for (int i = 0; i < NITEMS; ++i)
                    if (i >= lo && i < hi) item_load(i);
#pragma unroll
                for (int i = 0; i < NITEMS; ++i)
                    if (i + LAG >= lo && i + LAG < hi) item_store(i, buf ^ 1);
                // The staging instructions go between the MFMAs (a few per MFMA) rather than after them:
                // the wave has something to issue while its own MFMAs queue for the matrix pipe (measured 2-5 %).
#pragma unroll
                for (int q = 0; q < RG * S * WTM; ++q) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one MFMA
                    __builtin_amdgcn_sched_group_barrier(0x006, 4, 0);   // four vector or scalar ALU instructions
                    __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);   // one global load
                    __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);   // one LDS store
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
#pragma unroll
        for (int i = NITEMS - LAG; i < NITEMS; ++i) item_store(i, buf ^ 1);
    };

    // The chunks of a slice.  With the XCD-aware grid the slices interleave: at any time the workgroups
    // of an XCD work on neighbouring chunks -- the column tiles of the same image rows, whose 64-byte
    // row segments share cache lines and DRAM pages, and the row chunks next to them, which share halo
    // rows -- instead of 256 places far apart.  Otherwise a slice is a contiguous range.
    const int cstep = p.xcd_slices > 0 ? p.nslices : 1;
    const int cbeg = p.xcd_slices > 0 ? zslice : zslice * p.cps;
    const int cend = p.xcd_slices > 0 ? p.nchunks : min(p.nchunks, cbeg + p.cps);
    __syncthreads();   // the zero fill is complete
    if (cbeg < cend) {
        set_chunk(cbeg);
        begin_chunk();
#pragma unroll
        for (int i = 0; i < NITEMS; ++i) item_load(i);
#pragma unroll
        for (int i = 0; i < NITEMS; ++i) item_store(i, 0);
    }
    __syncthreads();
    for (int chunk = cbeg, buf = 0; chunk < cend; chunk += cstep, buf ^= 1) {
        // every round stages a chunk; past the end it is the last chunk again
        if (chunk + cstep < cend) {
            if (cstep == 1) next_chunk();
            else set_chunk(chunk + cstep);
        }
        begin_chunk();
        compute(buf);
        __syncthreads();
    }

    // ---- epilogue.  An accumulator tile keeps column c = lane % 32 and rows k = 8*(v/4) +
    // 4*(lane/32) + v%4 in register v.  Four passes (v/4 = 0..3) each move KTB/4 rows of the
    // workgroup's dw block through LDS as [row][c*T + t], from where consecutive lanes write
    // consecutive addresses of dw[k][c][r][s].
    constexpr int ROWS = KTB / 4, ROWLEN = CTB * T, EP = ROWLEN + 1;
    float *stage = reinterpret_cast<float *>(smem);
    float *dst = out + (use_atomics ? (size_t)0 : (size_t)zslice * p.K * p.C * p.Tfull);
#pragma unroll
    for (int ps = 0; ps < 4; ++ps) {
#pragma unroll
        for (int tm = 0; tm < WTM; ++tm)
#pragma unroll
            for (int t = 0; t < T; ++t)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int rr = ((wk * WTM + tm) * 2 + g) * 4 + i;
                    if (ph == 0) stage[rr * EP + (wc * 32 + l32) * T + t] = acc[tm][t][4 * ps + i];
                }
        __syncthreads();
        if (TP == 2) {   // the second set of waves adds its share
            if (ph == 1) {
#pragma unroll
                for (int tm = 0; tm < WTM; ++tm)
#pragma unroll
                    for (int t = 0; t < T; ++t)
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const int rr = ((wk * WTM + tm) * 2 + g) * 4 + i;
                            stage[rr * EP + (wc * 32 + l32) * T + t] += acc[tm][t][4 * ps + i];
                        }
            }
            __syncthreads();
        }
        if (!use_atomics && p.Tfull == T && p.C % CTB == 0 && (reinterpret_cast<uintptr_t>(dst) & 15) == 0) {
            // whole rows of 64 c x T taps are contiguous and 16-byte aligned in dw: float4 stores
            constexpr int R4 = ROWLEN / 4;
            for (int e = tid; e < ROWS * R4; e += NT) {
                const int rr = e / R4, j = (e - rr * R4) * 4;
                const int k = k0 + (rr >> 3) * 32 + 8 * ps + (rr & 7);
                if (k < p.K) {
                    const float *sp = stage + rr * EP + j;
                    const float4 v = make_float4(sp[0], sp[1], sp[2], sp[3]);
                    *reinterpret_cast<float4 *>(dst + (size_t)k * p.C * T + (size_t)c0 * T + j) = v;
                }
            }
        } else {
            for (int e = tid; e < ROWS * ROWLEN; e += NT) {
                const int rr = e / ROWLEN, j = e - rr * ROWLEN;
                // rr = ((wk*TM + tm)*2 + g)*4 + i  ->  k = k0 + (wk*TM + tm)*32 + 8*ps + 4*g + i
                const int k = k0 + (rr >> 3) * 32 + 8 * ps + (rr & 7);
                const int c = c0 + j / T;
                if (k < p.K && c < p.C) {
                    const size_t off = ((size_t)k * p.C + c) * p.Tfull + p.toff + (j - (j / T) * T);
                    const float val = stage[rr * EP + j];
                    if (use_atomics) unsafeAtomicAdd(dst + off, val);
                    else dst[off] = val;
                }
            }
        }
        __syncthreads();
    }
}

struct RPlan {
    RowsProblem p;
    dim3 grid;
    int nslices;
    int S, TM, TH, TWP, TP;
    bool wide;
};

template <int S, int RG, int TM, int TH, int TWP>
constexpr size_t rows_smem()
{
    constexpr int KTB = 2 * TM * 32, XROWS = TH + RG - 1, LWX = TWP + (S > 1 ? 16 : 0);
    constexpr size_t stage = 2 * ((size_t)KTB * odd16c(TH * TWP) + (size_t)CTB * odd16c(XROWS * LWX)) * sizeof(bf16_t);
    constexpr size_t epi = (size_t)(KTB / 4) * (CTB * RG * S + 1) * sizeof(float);
    return stage > epi ? stage : epi;
}

// cap > 0: at most that many slices (the caller's workspace holds no more partial sums)
bool make_rplan(const ConvGeom &g, RPlan *pl, int cap = 0)
{
    if (!g.in_bf16 || g.sh != 1 || g.sw != 1) return false;
    if (!((g.R == 3 && g.S == 3) || (g.R == 1 && g.S == 1) || (g.R == 5 && g.S == 5) || (g.R == 7 && g.S == 1) ||
          (g.R == 1 && g.S == 7)))
        return false;
    if (g.pw != (g.S - 1) / 2 || g.Q != g.W) return false;   // the column shift is built for "same" padding
    if (g.ph > g.R - 1 + 64) return false;
    const long long lim = 0x7fffffffLL;
    if ((long long)g.N * g.C * g.H * g.W + 64 > lim || (long long)g.N * g.K * g.P * g.Q + 64 > lim) return false;
    if ((long long)g.N * g.C * g.H * g.W < 8 || (long long)g.N * g.K * g.P * g.Q < 8) return false;   // 16-byte loads
    RowsProblem p;
    p.N = g.N; p.C = g.C; p.H = g.H; p.W = g.W; p.K = g.K; p.P = g.P; p.Q = g.Q; p.R = g.R; p.ph = g.ph;
    p.Tfull = g.R * g.S; p.toff = 0;
    bool wide;
    int TWP, TH;
    if (g.Q <= 16) { TWP = 16; TH = 8; wide = false; }
    else if (g.Q <= 32) { TWP = 32; TH = 4; wide = false; }
    else if (g.Q % 8 == 0) { TWP = 32; TH = 4; wide = true; }
    else if (g.Q <= 64 && g.R < 7) { TWP = 64; TH = 2; wide = false; }
    else return false;
    p.ncoltiles = wide ? (g.Q + TWP - 1) / TWP : 1;
    p.rowchunks = (g.P + TH - 1) / TH;
    const long long nch = (long long)g.N * p.rowchunks * p.ncoltiles;
    if (nch > lim) return false;
    p.nchunks = (int)nch;
    // 64 k per workgroup of 256 threads; 128 k per 512 threads (two waves per SIMD, half the L1
    // traffic per MFMA, but twice the bytes the slices add into dw) where there is enough work
    const int TM = (g.K >= 128 && (long long)g.N * g.P * g.Q >= 20000) ? 2 : 1, KTB = 2 * TM * 32;
    p.ctiles = (g.C + CTB - 1) / CTB;
    const int ktiles = (g.K + KTB - 1) / KTB;
    if (ktiles > 65535) return false;
    const long long tiles = (long long)p.ctiles * ktiles;
    // slices: one workgroup per CU in all; every slice costs a pass over dw in the epilogue
    long long slices = (256 + tiles - 1) / tiles;
    if (slices > p.nchunks) slices = p.nchunks;
    if (slices > 65535) slices = 65535;
    if (cap > 0 && slices > cap) slices = cap;
    if (slices < 1) slices = 1;
    p.cps = (int)((p.nchunks + slices - 1) / slices);
    slices = (p.nchunks + p.cps - 1) / p.cps;
    p.ktiles = ktiles;
    p.xcd_slices = 0;
    p.nslices = (int)slices;
    pl->nslices = (int)slices;
    pl->grid = dim3(p.ctiles, ktiles, (unsigned)slices);
    if (slices % 8 == 0 && tiles * slices <= 0x7fffffffLL) {
        p.xcd_slices = (int)(slices / 8);
        pl->grid = dim3((unsigned)(tiles * slices), 1, 1);
    }
    pl->p = p;
    pl->S = g.S; pl->TM = TM; pl->TH = TH; pl->TWP = TWP; pl->wide = wide;
    // a second set of waves on the same tile where the tile has one wave per SIMD and the chunk two column groups
    pl->TP = (TM == 1 && TWP == 32 && (long long)g.N * g.P * g.Q >= 20000) ? 2 : 1;
    return true;
}

template <int S, int RG, int TM, int TH, int TWP, bool WIDE, int TP = 1>
hipError_t launch_shape(const bf16_t *x, const bf16_t *dy, float *out, int atomics, const RPlan &pl, hipStream_t st)
{
    constexpr size_t smem = rows_smem<S, RG, TM, TH, TWP>();
    static_assert(smem <= 160 * 1024, "chunk does not fit in LDS");
    auto kern = wgrad_rows_kernel<S, RG, TM, TH, TWP, WIDE, TP>;
    // dynamic LDS beyond 64 KB has to be enabled once per kernel
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (attr != hipSuccess) return attr;
    hipLaunchKernelGGL(kern, pl.grid, dim3(TM * TP * 256), smem, st, x, dy, out, atomics, pl.p);
    return hipGetLastError();
}

template <int S, int RG, int TM>
hipError_t launch_tm(const bf16_t *x, const bf16_t *dy, float *out, int atomics, const RPlan &pl, hipStream_t st)
{
    if (pl.TWP == 16) return launch_shape<S, RG, TM, 8, 16, false>(x, dy, out, atomics, pl, st);
    if (pl.TWP == 64) {
        // seven filter rows of 64-column chunks do not fit LDS (make_rplan does not plan them)
        if constexpr (rows_smem<S, RG, TM, 2, 64>() <= 160 * 1024) return launch_shape<S, RG, TM, 2, 64, false>(x, dy, out, atomics, pl, st);
        else return hipErrorInvalidValue;
    }
    if (TM == 1 && pl.TP == 2) {
        if (pl.wide) return launch_shape<S, RG, 1, 4, 32, true, 2>(x, dy, out, atomics, pl, st);
        return launch_shape<S, RG, 1, 4, 32, false, 2>(x, dy, out, atomics, pl, st);
    }
    if (pl.wide) return launch_shape<S, RG, TM, 4, 32, true>(x, dy, out, atomics, pl, st);
    return launch_shape<S, RG, TM, 4, 32, false>(x, dy, out, atomics, pl, st);
}

}  // namespace

bool rows_wgrad_supported(const ConvGeom &g)
{
    RPlan pl;
    return make_rplan(g, &pl);
}

int rows_wgrad_slices(const ConvGeom &g, int cap)
{
    RPlan pl;
    return make_rplan(g, &pl, cap) ? pl.nslices : 0;
}

// partial == nullptr: slices add into dw with atomics (dw is zero-filled first);
// otherwise slice z writes partial[z][K*C*R*S] and a reduction in slice order follows.
hipError_t launch_rows_wgrad(const void *x, const void *dy, float *dw, const ConvGeom &g, float *partial,
                             hipStream_t st, int cap)
{
    RPlan pl;
    if (!make_rplan(g, &pl, cap)) return hipErrorInvalidValue;
    const size_t nw = (size_t)g.K * g.C * g.R * g.S;
    const int slices = pl.nslices;
    const bool direct_store = !partial && slices == 1;
    float *out = partial ? partial : dw;
    if (!partial && !direct_store) {
        hipError_t e = launch_fill_zero(dw, nw, st);
        if (e != hipSuccess) return e;
    }
    const int atomics = (!partial && !direct_store) ? 1 : 0;
    const bf16_t *xs = static_cast<const bf16_t *>(x), *ds = static_cast<const bf16_t *>(dy);
    hipError_t e;
    if (g.R == 7 && g.S == 1) {
        e = pl.TM == 2 ? launch_tm<1, 7, 2>(xs, ds, out, atomics, pl, st) : launch_tm<1, 7, 1>(xs, ds, out, atomics, pl, st);
    } else if (g.R == 1 && g.S == 7) {
        e = pl.TM == 2 ? launch_tm<7, 1, 2>(xs, ds, out, atomics, pl, st) : launch_tm<7, 1, 1>(xs, ds, out, atomics, pl, st);
    } else if (pl.S == 5) {
        // a filter row per launch (5 accumulator tiles; 25 would not fit the registers): row r0 of the filter meets
        // input row p + r0 - ph, which is the one-row problem with its padding moved by r0
        e = hipSuccess;
        for (int r0 = 0; r0 < 5 && e == hipSuccess; ++r0) {
            RPlan one = pl;
            one.p.ph = g.ph - r0;
            one.p.toff = r0 * 5;
            e = pl.TM == 2 ? launch_tm<5, 1, 2>(xs, ds, out, atomics, one, st) : launch_tm<5, 1, 1>(xs, ds, out, atomics, one, st);
        }
    } else if (pl.S == 3) e = pl.TM == 2 ? launch_tm<3, 3, 2>(xs, ds, out, atomics, pl, st) : launch_tm<3, 3, 1>(xs, ds, out, atomics, pl, st);
    else e = pl.TM == 2 ? launch_tm<1, 1, 2>(xs, ds, out, atomics, pl, st) : launch_tm<1, 1, 1>(xs, ds, out, atomics, pl, st);
    if (e != hipSuccess) return e;
    if (partial) return launch_reduce_partials(partial, dw, nw, slices, false, st);
    return hipSuccess;
}

}  // namespace sn
