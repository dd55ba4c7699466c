#pragma once
// Stride-1 implicit-GEMM convolution for bf16 on gfx950 MFMA: the fast path of
// CONV forward and CONV backward-data (Sec. 3.5 of the paper; definitions in sn.h).
//
// Backward-data of a stride-1 convolution is itself a stride-1 forward
// convolution of dy with the filter transposed in (k,c) and flipped in (r,s)
// and padding R-1-pad, so both directions run the same kernel on a "problem":
// input in[N][Cin][Hin][Win], output out[N][Kout][Pout][Qout], taps (r,s),
// padding (padh,padw), filter element A(m, red, tap) with m an output channel
// and red an input channel.
//
// Work decomposition.  A 256-thread workgroup owns KT output channels x PIXT
// output pixels (KT=128, PIXT=256 or KT=64, PIXT=512) and walks the input
// channels 16 at a time; each wave multiplies a 64-channel x 128-pixel block
// with v_mfma_f32_32x32x16_bf16 (2 x 4 tiles, 128 accumulator registers).
// Two pixel tilings:
//   WIDE    8x32 / 16x32 patches of one image; an MFMA tile is one output row,
//           and the four tiles of a wave are four consecutive rows;
//   NARROW  (images up to 64 wide) TH consecutive rows of the flattened
//           (image, output row) space times the whole width, so small images
//           fill the lanes: a tile may span several images.
// Per 16-channel chunk the workgroup keeps in LDS
//   xs: the input patch with halo, transposed to [pixel][16 channels] (32 bytes
//       per pixel, so one MFMA lane reads its 8 consecutive channels with a
//       single 16-byte load).  The transposition happens on the way in: each
//       thread gathers 8 channels of two neighbouring pixels with 4-byte loads
//       that are coalesced across lanes along the image row, and writes two
//       16-byte items.  The patch rows are padded to a multiple of 16 pixels;
//   ws: the filter slab [tap][KT][16 channels] of one stage.
// Both are XOR-swizzled on the 16-byte half index with bit 3 of the row index,
// which makes the 16-byte reads of 16 consecutive rows hit distinct banks; with
// the padded patch rows the swizzle of a pixel does not depend on the tap row.
// A tap (r,s) only shifts the pixel index by r*LWp + s, so all taps reuse one
// patch.  A chunk is worked off in stages of one filter column (all r for one
// s; all taps for 1xS filters): in the WIDE tiling the operand of output row i,
// tap row r is the operand of output row i+1, tap row r-1, so a wave reads
// 4+R-1 patch rows per stage instead of 4*R.
//
// Both LDS arrays are double buffered.  The global loads of the next stage
// (filter) and of the next chunk (patch) are issued before the MFMAs of the
// current stage and written to the other buffer after them; one barrier per
// stage.  The loads are branch free: addresses that fall outside the image or
// the tensor are clamped to a valid one, and what they return is never stored
// (the LDS buffers are zeroed once; the set of pixels outside the image is the
// same for every chunk) or belongs to output channels that are not written.
//
// The filter slab comes either from a copy pre-packed into the caller's
// workspace in exactly the LDS order, swizzle included (STAGED algorithm: a
// stage is one contiguous run of 16-byte loads), or comes straight from the KCRS
// tensor (DIRECT, no workspace).  There a thread owns one (row, 8-channel half) of
// the slab and, where the filter has at most 9 taps and the reduction channels
// come in whole chunks of 16, fetches its share of a whole chunk with 16-byte
// loads -- forward: the 8 channels x T taps of its row are one contiguous run of
// the KCRS tensor; backward-data (3x3): eight runs of T taps, one per channel,
// contiguous across the lanes -- keeps it in registers and cuts each stage's
// 16-byte LDS items out of them with byte permutes whose selectors are compile
// time constants (WM = 1 / 2).  Other shapes gather element by element (WM = 0).
#include <type_traits>
#include <utility>

#include "sn_internal.h"

namespace sn {

struct TileProblem {
    int N, Cin, Hin, Win, Kout, Pout, Qout, padh, padw;
    int out_bf16;
    int TH, TW, LW, LWp;     // tile rows, tile columns, patch width in pixels, padded patch width
    int ncoltiles;
    int tiles_per_img;       // WIDE: row tiles per image
    int Hp;                  // padded rows per image = Pout + R - 1
    int nchunks;             // ceil(Cin / 16)
    int xslots;              // pixel slots of one patch buffer in LDS
    int xt_rows, xt_cols;    // rows and columns (a multiple of 8) of the parked patch, per channel
    int ragged;              // the image width is not a multiple of 8
    // filter access: A(m, red, tap) = w[m*w_sm + red*w_sr + (tflip ? T-1-tap : tap)]
    int w_sm, w_sr, tflip;
    int Mpad;                // rows per (chunk, tap) block of the packed filter
    // conv_tile2.h only: load rounds and transposition rounds per chunk, bytes of one parked buffer
    int xg_rounds, xtr_rounds, pk_bytes;
    int xt_upc;              // units of the load size a parked channel has room for (64, 128 or 256)
    int xt_shift;            // NARROW, 16-byte loads of rows that do not start on 16-byte boundaries: 0 = off, else the
                             // number G (1 or 2) of consecutive image rows that make one parked row: G rows start on
                             // multiples of 8 bytes, and the parked row begins at the 16-byte boundary at or below it
    int xt_ncg;              // with xt_shift: 16-column groups per patch row in the transposition
    uint32_t in_bytes, w_bytes;   // sizes of the input tensor and of the packed filter
    int nptiles, nktiles, pt_per_xcd;   // pixel tiles, channel tiles, pixel tiles per XCD (the grid is 8 * pt_per_xcd * nktiles)
    // Filters too large for an XCD's L2: kmajor = min(nktiles, 8) XCDs take different channel
    // tiles (kk = nktiles / 8 of them each, at least 1) and pt_per_xcd counts the pixel tiles of
    // one of the 8 / kmajor groups of XCDs; the grid is 8 * kk * pt_per_xcd.  0: the mapping above.
    int kmajor, kk;
    // Forward only, may be null: where the tiles leave, for the BN that follows the CONV, the count,
    // mean and sum of squared deviations of their output values per channel:
    // stats[(k * nptiles + ptile) * 3 + {0, 1, 2}].
    float *stats;
};

// Which tile a workgroup computes; false if none (the grid is rounded up).  Workgroup L runs on
// XCD L % 8 (round-robin dispatch), and every XCD has an L2 of its own.  By default each XCD
// gets a contiguous range of pixel tiles, and the channel tiles of one pixel tile, which read
// the same patch, follow each other on the same XCD.  Where the filter would not stay in one L2
// (kmajor), an XCD keeps to its channel tile(s) instead, so that its share of the filter stays
// there, and walks through the pixel tiles of its group.
__device__ inline bool tile_of(const TileProblem &p, int *ktile, int *ptile)
{
    const int xcd = blockIdx.x & 7, jx = blockIdx.x >> 3;
    if (p.kmajor) {
        *ktile = xcd % p.kmajor + 8 * (jx % p.kk);
        *ptile = (xcd / p.kmajor) * p.pt_per_xcd + jx / p.kk;
        return jx / p.kk < p.pt_per_xcd && *ptile < p.nptiles;
    }
    *ktile = jx % p.nktiles;
    *ptile = xcd * p.pt_per_xcd + jx / p.nktiles;
    return *ptile < p.nptiles;
}

struct Plan {
    TileProblem p;
    int KT, NF;
    bool wide;
    int dw;                  // conv_tile2.h only: bytes per load item (16 or 4)
    int ks;                  // conv_tile2.h only: sets of waves that split a tile's chunks (1 or 2)
    size_t lds;
    dim3 grid;
};

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned short u16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int XPAIRS_MAX = 384;  // NARROW: pixel pairs gathered per chunk
constexpr int XG_MAX = 6;        // NARROW: 16-byte load rounds per chunk
constexpr int WIDE_LWP = 48;    // WIDE: padded patch row (32 + S - 1 <= 48)
constexpr int LDS_LIMIT = 160 * 1024;
constexpr int EPI_PITCH = 272;  // bytes per channel row of the output staging: 128 pixels and a pad


// f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>)
template <typename F, int... I> __device__ inline void static_for_impl(F &&f, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F> __device__ inline void static_for(F &&f)
{
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// Filter columns per stage: a 1xS filter has too little work per column.
constexpr int sg_of(int R, int S) { return (R == 1 && S > 1) ? S : 1; }

__device__ __host__ inline int swz(int row) { return (row >> 3) & 1; }

// Two consecutive bf16 as one 4-byte load, whatever the alignment.
struct __attribute__((packed, aligned(2))) U32u { uint32_t v; };
__device__ inline uint32_t load2_any(const bf16_t *p) { return reinterpret_cast<const U32u *>(p)->v; }

// Eight consecutive bf16 as one 16-byte store, whatever the alignment.
struct __attribute__((packed, aligned(2))) U128u { uint32_t v[4]; };
__device__ inline void store8_any(bf16_t *p, uint4 v)
{
    U128u u = {{v.x, v.y, v.z, v.w}};
    *reinterpret_cast<U128u *>(p) = u;
}

// Two fp32 to a pair of bf16 (round to nearest even), the first in the low half.
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
__device__ inline uint32_t pack2_bf16(float a, float b)
{
    f32x2 f = {a, b};
    bf16x2 h = __builtin_convertvector(f, bf16x2);
    uint32_t r;
    __builtin_memcpy(&r, &h, 4);
    return r;
}

// Never written: the source of every load that must bring zeros.
__device__ __attribute__((aligned(16))) uint32_t zero_page[4];

// Per-channel statistics of a tile's outputs, taken from the accumulators before they are stored
// (as the stored values: rounded to bf16 where the output is bf16), for the batch normalisation
// that follows: the count n of the tile's real output pixels, their mean, and the sum M2 of squared
// deviations from that mean.  A lane makes one pass over its registers with sums of d and d^2,
// d = value - the lane's first value (a shift next to the data keeps the variance free of
// cancellation), turns them into (n, mean, M2), and such triples combine exactly (pairwise
// formula): lane with lane + 32, then the NWP waves that hold the pixels of one channel through
// LDS, always in the same order.  acc[i][f][v]: channel kbase + 32 i + lane % 32, pixel
// (wp * NF + f) * 32 + 8 (v / 4) + 4 (lane / 32) + v % 4 of the tile; `slot` numbers the groups
// of NWP waves; red: 3 * 64 * NWP * nslots floats of LDS that nothing else uses until the function
// returns (it ends with a barrier).  Every wave of the workgroup must call it.
struct TileMoments { float n, mean, m2; };

__device__ inline TileMoments moments_join(const TileMoments &a, const TileMoments &b)
{
    const float nt = a.n + b.n;
    if (!(nt > 0.f)) return a;
    const float d = b.mean - a.mean, r = b.n / nt;
    TileMoments o;
    o.n = nt;
    o.mean = a.mean + d * r;
    o.m2 = a.m2 + b.m2 + d * d * a.n * r;
    return o;
}

template <int NF, int NWP>
__device__ inline void tile_bn_partials(const f32x16 (&acc)[2][NF], int TW, int rows_ok, int cols_ok, int wp, int slot,
                                        int l32, int g, int kbase, int Kout, bool round_bf16,
                                        float *__restrict__ stats, int nptiles, int ptile, float *red)
{
    // Which of the lane's pixels are real outputs, without the divisions of the store offsets.  A
    // tile is either 32 columns wide (32-pixel group F = wp * NF + f is row F of a column tile
    // with cols_ok real columns) or spans whole image rows, where the real pixels are the first
    // rows_ok * TW; rows_ok = min(TH, rows left).  Either way the lane's pixel v of group f,
    // 8 (v / 4) + v % 4 + 4 (lane / 32) into the group, is real iff 8 (v / 4) + v % 4 < lim[f].
    int lim[NF];
    float n = 0.f;
#pragma unroll
    for (int f = 0; f < NF; ++f) {
        const int F = wp * NF + f;
        int L = TW == 32 ? (F < rows_ok ? cols_ok - 4 * g : 0) : rows_ok * TW - F * 32 - 4 * g;
        L = min(max(L, 0), 32);
        lim[f] = L;
        n += (float)(4 * (L >> 3) + min(L & 7, 4));
    }
    // Sums of d and d^2 over the lane's real pixels, d = stored value - shift.  Four variants of
    // one loop (rounded to bf16 or not, every pixel real or not), chosen by conditions that are
    // the same for the whole wave, so that the loop itself has no selects it does not need; the
    // bf16 rounding converts two values per instruction.
    float s1[2] = {0.f, 0.f}, s2[2] = {0.f, 0.f}, shift[2];
    const bool full = __all(n == (float)(NF * 16)) != 0;   // every pixel of every lane of the wave is real
    auto sums = [&](auto rb, auto all) {
        constexpr bool RB = decltype(rb)::value, ALL = decltype(all)::value;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            shift[i] = RB ? __uint_as_float(pack2_bf16(acc[i][0][0], 0.f) << 16) : acc[i][0][0];   // any value next to the data will do
#pragma unroll
            for (int f = 0; f < NF; ++f)
#pragma unroll
                for (int v = 0; v < 16; v += 2) {
                    float x0 = acc[i][f][v], x1 = acc[i][f][v + 1];
                    if (RB) {
                        const uint32_t u = pack2_bf16(x0, x1);
                        x0 = __uint_as_float(u << 16);
                        x1 = __uint_as_float(u & 0xffff0000u);
                    }
                    float d0 = x0 - shift[i], d1 = x1 - shift[i];
                    if (!ALL) {
                        d0 = (8 * (v / 4) + v % 4 < lim[f]) ? d0 : 0.f;
                        d1 = (8 * ((v + 1) / 4) + (v + 1) % 4 < lim[f]) ? d1 : 0.f;
                    }
                    s1[i] += d0;
                    s2[i] = __builtin_fmaf(d0, d0, s2[i]);
                    s1[i] += d1;
                    s2[i] = __builtin_fmaf(d1, d1, s2[i]);
                }
        }
    };
    if (round_bf16) {
        if (full) sums(std::true_type{}, std::true_type{});
        else sums(std::true_type{}, std::false_type{});
    } else {
        if (full) sums(std::false_type{}, std::true_type{});
        else sums(std::false_type{}, std::false_type{});
    }
    __syncthreads();   // red is free
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        TileMoments m;
        m.n = n;
        m.mean = n > 0.f ? shift[i] + s1[i] / n : 0.f;
        m.m2 = n > 0.f ? fmaxf(s2[i] - s1[i] * s1[i] / n, 0.f) : 0.f;
        TileMoments o;
        o.n = __shfl_xor(m.n, 32);
        o.mean = __shfl_xor(m.mean, 32);
        o.m2 = __shfl_xor(m.m2, 32);
        if (g == 0) {
            m = moments_join(m, o);
            float *e = red + (((slot * 2 + i) * 32 + l32) * NWP + wp) * 3;
            e[0] = m.n; e[1] = m.mean; e[2] = m.m2;
        }
    }
    __syncthreads();
    if (g == 0 && wp == 0) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const float *e = red + ((slot * 2 + i) * 32 + l32) * NWP * 3;
            TileMoments m = {e[0], e[1], e[2]};
#pragma unroll
            for (int w = 1; w < NWP; ++w) {
                const TileMoments o = {e[3 * w], e[3 * w + 1], e[3 * w + 2]};
                m = moments_join(m, o);
            }
            const int k = kbase + i * 32 + l32;
            if (k < Kout) {
                float *o = stats + ((size_t)k * nptiles + ptile) * 3;
                o[0] = m.n; o[1] = m.mean; o[2] = m.m2;
            }
        }
    }
    __syncthreads();   // red may be written again
}

// Eight consecutive bf16 as one 16-byte load, whatever the alignment.
struct __attribute__((packed, aligned(2))) V128u { u32x4 v; };
__device__ inline u32x4 load8_any(const bf16_t *p) { return reinterpret_cast<const V128u *>(p)->v; }

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

__device__ inline u32x4 keep_first(u32x4 v, int n)
{
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] &= n > 2 * j + 1 ? 0xffffffffu : (n > 2 * j ? 0xffffu : 0u);
    return v;
}

// Keeps the first n (< 8) elements of an octet.
__device__ inline uint4 keep_first(uint4 v, int n)
{
    uint32_t *d = reinterpret_cast<uint32_t *>(&v);
#pragma unroll
    for (int j = 0; j < 4; ++j) d[j] &= n > 2 * j + 1 ? 0xffffffffu : (n > 2 * j ? 0xffffu : 0u);
    return v;
}

// The two 16-bit elements h0, h1 (halfword indices into wc) as one dword, h0 in the low half.
template <int N> __device__ inline uint32_t pick2(const uint32_t (&wc)[N], int h0, int h1)
{
    const uint32_t sel = (uint32_t)((h0 & 1) * 2) | (uint32_t)((h0 & 1) * 2 + 1) << 8 |
                         (uint32_t)(4 + (h1 & 1) * 2) << 16 | (uint32_t)(5 + (h1 & 1) * 2) << 24;
    return __builtin_amdgcn_perm(wc[h1 >> 1], wc[h0 >> 1], sel);
}

template <int R, int S, int KT, int NF, bool STAGED, bool WIDE, int WM = 0>
__global__ void __launch_bounds__(256, 2)
conv_tile_kernel(const bf16_t *__restrict__ in, const bf16_t *__restrict__ w, void *__restrict__ out, TileProblem p)
{
    constexpr int SG = sg_of(R, S), T = R * S, TRES = R * SG, NSUB = S / SG;
    constexpr int PIXT = (KT == 128 ? 2 : 4) * NF * 32;   // pixels per workgroup: NF tiles of 32 per wave
    constexpr int WSZ = TRES * KT * 2;                 // 16-byte items of one filter slab
    constexpr int WITEMS = (WSZ + 255) / 256;
    // gather rounds: a thread takes one pixel pair x 8 channels per round
    constexpr int XR = WIDE ? ((PIXT / 32 + R - 1) * ((32 + S) / 2) + 127) / 128 : XPAIRS_MAX / 128;
    constexpr int NB = WIDE ? NF + R - 1 : NF;
    // WIDE tiling, KT = 128, three or more stages per chunk: the patch comes in as whole 16-byte octets
    // of image rows, is parked in LDS as it is, and is transposed from there (see x_issue below).
    constexpr bool XT = WIDE && NSUB >= 3 && KT == 128;
    constexpr int XG = WIDE ? (16 * (PIXT / 32 + R - 1) * (WIDE_LWP / 8) + 255) / 256 : XG_MAX;   // load rounds
    constexpr int XTR = WIDE ? ((PIXT / 32 + R - 1) * (31 + S) + 127) / 128 : 2 * XPAIRS_MAX / 128;  // transposition rounds
    extern __shared__ __attribute__((aligned(16))) uint4 smem[];
    const int XS = p.xslots * 2;                       // 16-byte items of one patch buffer
    uint4 *const xs = smem;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, g = lane >> 5;
    const int wk = (KT == 128) ? (wave >> 1) : 0;
    const int wp = (KT == 128) ? (wave & 1) : wave;

    // ---- which tile
    int ktile, ptile;
    if (!tile_of(p, &ktile, &ptile)) return;   // uniform for the workgroup, before any barrier
    // ---- tile geometry
    const int rowtile = ptile / p.ncoltiles, coltile = ptile - rowtile * p.ncoltiles;
    const int k0 = ktile * KT;
    const int q0 = coltile * p.TW;
    const int LWp = WIDE ? WIDE_LWP : p.LWp;
    const int HWin = p.Hin * p.Win;
    int o0, NP, u0, lrows, img = 0;   // first flattened (image, row), its limit, first patch row, patch rows
    if (WIDE) {
        img = rowtile / p.tiles_per_img;
        const int pp0 = (rowtile - img * p.tiles_per_img) * p.TH;
        o0 = img * p.Pout + pp0;
        NP = (img + 1) * p.Pout;
        u0 = img * p.Hp + pp0;
        lrows = p.TH + R - 1;
    } else {
        o0 = rowtile * p.TH;
        NP = p.N * p.Pout;
        const int n0 = o0 / p.Pout;
        u0 = n0 * p.Hp + (o0 - n0 * p.Pout);
        const int olast = min(o0 + p.TH, NP) - 1, nl = olast / p.Pout;
        lrows = nl * p.Hp + (olast - nl * p.Pout) - u0 + R;
    }

    // ---- zero both patch buffers once: pixels outside the image are never written again
    for (int i = tid; i < 2 * XS; i += 256) xs[i] = make_uint4(0, 0, 0, 0);

    // ---- per-thread constants of the patch gather.  A thread takes two neighbouring
    // pixels of a patch row x 8 channels: one 4-byte load per channel (2-byte aligned)
    // brings both pixels, so that two 16-byte LDS items are built with 8 byte-permutes.
    // If only one pixel of the pair is inside the image the load is placed so that it
    // stays inside the row (rows have at least 2 pixels), and the half that holds the
    // live pixel goes to that pixel's slot.
    const int xo = tid >> 7, tp = tid & 127;
    const uint32_t xo8 = (uint32_t)xo * 8u * (uint32_t)HWin;
    uint32_t xoff[XT ? 1 : XR];       // element offset of the load for the thread's first channel of chunk 0
    int xdlo[XT ? 1 : XR], xdhi[XT ? 1 : XR];  // 16-byte LDS index for the low / high halves, -1: not stored
    const int LWh = (p.LW + 1) >> 1;
    const int xpairs = lrows * LWh;
#pragma unroll
    for (int rd = 0; rd < (XT ? 0 : XR); ++rd) {
        const int lp = rd * 128 + tp;
        int off = 0, dlo = -1, dhi = -1;
        if (lp < xpairs) {
            const int lrow = lp / LWh, lcol = (lp - lrow * LWh) * 2;
            const int u = u0 + lrow, n = WIDE ? img : u / p.Hp, h = u - n * p.Hp - p.padh;
            const int v = q0 - p.padw + lcol;
            if (n < p.N && (unsigned)h < (unsigned)p.Hin) {
                const int rowoff = (n * p.Cin * p.Hin + h) * p.Win;
                const bool va = (unsigned)v < (unsigned)p.Win;
                const bool vb = lcol + 1 < p.LW && (unsigned)(v + 1) < (unsigned)p.Win;
                const int slot = lrow * LWp + lcol;
                const int da = slot * 2 + (xo ^ swz(slot)), db = (slot + 1) * 2 + (xo ^ swz(slot + 1));
                if (va && vb) { off = rowoff + v; dlo = da; dhi = db; }
                else if (va && v >= 1) { off = rowoff + v - 1; dhi = da; }
                else if (va) { off = rowoff; dlo = da; }
                else if (vb) { off = rowoff + v + 1; dlo = db; }
            }
        }
        xoff[rd] = (uint32_t)off + xo8;
        xdlo[rd] = dlo;
        xdhi[rd] = dhi;
    }

    // ---- the same for filters with three or more stages per chunk (XT).  Loading: item e of
    // a thread's round is octet (channel e / (rows*octets), patch row, octet of the row); the
    // octets are aligned to the image columns (WIDE: from column q0 - 8), so a load never
    // leaves its row unless the width is ragged.  What is not wanted (rows outside the image,
    // the columns left of it, channels past the last) is read from a page of zeros.  The
    // octets are parked in LDS in item order, i.e. as [channel][patch row][column].
    // Transposing: a thread takes one pixel x 8 channels per round, reads its 8 elements from
    // the parked patch and writes the 16-byte item of the MFMA layout.
    constexpr int NEVER = -(1 << 30);
    const int xt_oct = p.xt_cols >> 3, xt_items = 16 * p.xt_rows * xt_oct;
    const int xtotal = p.N * p.Cin * HWin;
    const bf16_t *const zp = reinterpret_cast<const bf16_t *>(zero_page);
    int xg_off[XT ? XG : 1];   // element offset of the octet in channel chunk 0, NEVER: never wanted
    int xg_inf[XT ? XG : 1];   // channel | valid columns << 4
    uint32_t xs_sd[XT ? XTR : 1];   // parked element of the pixel's first channel | 16-byte LDS index << 16 (0xffff: no pixel)
    const int xpix = lrows * p.LW, xrounds = (xpix + 127) >> 7;
    if (XT) {
#pragma unroll
        for (int rd = 0; rd < XG; ++rd) {
            const int e = rd * 256 + tid;
            const int oct = e % xt_oct, t2 = e / xt_oct, srow = t2 % p.xt_rows, ch = t2 / p.xt_rows;
            int off = NEVER, ncols = 0;
            if (ch < 16 && srow < lrows) {
                const int u = u0 + srow, n = WIDE ? img : u / p.Hp, h = u - n * p.Hp - p.padh;
                const int col0 = (WIDE ? q0 - 8 : 0) + oct * 8;
                if (n < p.N && (unsigned)h < (unsigned)p.Hin && col0 >= 0 && col0 < p.Win) {
                    off = ((n * p.Cin + ch) * p.Hin + h) * p.Win + col0;
                    ncols = min(8, p.Win - col0);
                }
            }
            xg_off[rd] = off;
            xg_inf[rd] = (ch & 15) | (ncols << 4);
        }
#pragma unroll
        for (int rd = 0; rd < XTR; ++rd) {
            const int lp = rd * 128 + tp;
            int src = 0, dst = 0xffff;
            if (lp < xpix) {
                const int lrow = lp / p.LW, lcol = lp - lrow * p.LW;
                const int u = u0 + lrow, n = WIDE ? img : u / p.Hp, h = u - n * p.Hp - p.padh;
                const int v = q0 - p.padw + lcol;
                if (n < p.N && (unsigned)h < (unsigned)p.Hin && (unsigned)v < (unsigned)p.Win) {
                    const int slot = lrow * LWp + lcol;
                    src = (xo * 8 * p.xt_rows + lrow) * p.xt_cols + (WIDE ? v - (q0 - 8) : v);
                    dst = slot * 2 + (xo ^ swz(slot));
                }
            }
            xs_sd[rd] = (uint32_t)src | ((uint32_t)dst << 16);
        }
    }

    // ---- per-thread constants of the DIRECT filter gather: thread item = (tap, row, half)
    uint32_t wsrc[(STAGED || WM) ? 1 : WITEMS];
    int wdst[(STAGED || WM) ? 1 : WITEMS];
    if (!STAGED && !WM) {
#pragma unroll
        for (int it = 0; it < WITEMS; ++it) {
            const int e = min(it * 256 + tid, WSZ - 1);
            int tl, row, o;
            tl = e % TRES;
            const int q = e / TRES;
            if (p.tflip) { row = q % KT; o = q / KT; }   // backward-data: (m, tap) contiguous for one red
            else { o = q & 1; row = q >> 1; }            // forward: (red, tap) contiguous for one m
            const int r = tl / SG, sl = tl - r * SG, tap = r * S + sl;
            wsrc[it] = (uint32_t)(min(k0 + row, p.Kout - 1) * p.w_sm + (p.tflip ? T - 1 - tap : tap) +
                                  o * 8 * p.w_sr);
            wdst[it] = (tl * KT + row) * 2 + (o ^ swz(row));
        }
    }

    // ---- per-lane constants of the MFMA operand reads
    int pixbase[WIDE ? 1 : NF];
    if (WIDE) {
        pixbase[0] = (wp * NF) * WIDE_LWP + l32;
    } else {
#pragma unroll
        for (int f = 0; f < NF; ++f) {
            const int i = (wp * NF + f) * 32 + l32;
            const int rl = i / p.TW, cl = i - rl * p.TW;
            const int o = o0 + rl;
            int pb = 0;
            if (rl < p.TH && o < NP) {
                const int n = o / p.Pout, pp = o - n * p.Pout;
                pb = (n * p.Hp + pp - u0) * LWp + cl;
            }
            pixbase[f] = pb;
        }
    }
    const int arow = wk * 64 + l32;
    const int aidx = arow * 2 + (g ^ swz(arow));

    f32x16 acc[2][NF];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int f = 0; f < NF; ++f)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][f][v] = 0.f;

    uint32_t xraw[XT ? 1 : XR][8];
    u32x4 xg[XT ? XG : 1];
    u16x8 wreg[(STAGED || WM) ? 1 : WITEMS];

    // Global loads of the patch of one chunk; nothing here looks at what a load returns.
    auto load_x = [&](int chunk) {
        const int c0 = chunk * 16;
        if (c0 + 16 <= p.Cin) {
            const bf16_t *src = in + (size_t)c0 * HWin;
#pragma unroll
            for (int rd = 0; rd < (XT ? 0 : XR); ++rd) {
#pragma unroll
                for (int i = 0; i < 8; ++i) xraw[rd][i] = load2_any(src + (size_t)i * HWin + xoff[rd]);
            }
        } else {   // the last chunk has fewer than 16 channels: clamp, store_x clears them
#pragma unroll
            for (int rd = 0; rd < (XT ? 0 : XR); ++rd) {
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const int c = min(c0 + xo * 8 + i, p.Cin - 1);
                    xraw[rd][i] = load2_any(in + (size_t)c * HWin + (xoff[rd] - xo8));
                }
            }
        }
    };
    auto store_x = [&](int chunk, uint4 *xb) {
        const int nvalid = p.Cin - chunk * 16 - xo * 8;
#pragma unroll
        for (int rd = 0; rd < (XT ? 0 : XR); ++rd) {
            uint4 lo, hi;
            lo.x = __builtin_amdgcn_perm(xraw[rd][1], xraw[rd][0], 0x05040100u);
            lo.y = __builtin_amdgcn_perm(xraw[rd][3], xraw[rd][2], 0x05040100u);
            lo.z = __builtin_amdgcn_perm(xraw[rd][5], xraw[rd][4], 0x05040100u);
            lo.w = __builtin_amdgcn_perm(xraw[rd][7], xraw[rd][6], 0x05040100u);
            hi.x = __builtin_amdgcn_perm(xraw[rd][1], xraw[rd][0], 0x07060302u);
            hi.y = __builtin_amdgcn_perm(xraw[rd][3], xraw[rd][2], 0x07060302u);
            hi.z = __builtin_amdgcn_perm(xraw[rd][5], xraw[rd][4], 0x07060302u);
            hi.w = __builtin_amdgcn_perm(xraw[rd][7], xraw[rd][6], 0x07060302u);
            if (nvalid < 8) { lo = keep_first(lo, nvalid); hi = keep_first(hi, nvalid); }
            if (xdlo[rd] >= 0) xb[xdlo[rd]] = lo;
            if (xdhi[rd] >= 0) xb[xdhi[rd]] = hi;
        }
    };

    // XT: the loads of the patch of one chunk; nothing here looks at what a load returns.
    uint4 *const xt = smem + 2 * XS + 2 * WSZ;   // the parked patch
    auto x_issue = [&](int chunk) {
        const int c0 = chunk * 16;
#pragma unroll
        for (int rd = 0; rd < (XT ? XG : 0); ++rd) {
            const bool ok = xg_off[rd] != NEVER && c0 + (xg_inf[rd] & 15) < p.Cin;
            int off = xg_off[rd] + c0 * HWin;
            if (p.ragged) off = min(off, xtotal - 8);   // the last octet of the tensor: x_park moves it back
            xg[rd] = load8_any(ok ? in + off : zp);
        }
    };
    // XT: parks the loaded octets in LDS.
    auto x_park = [&](int chunk) {
#pragma unroll
        for (int rd = 0; rd < (XT ? XG : 0); ++rd) {
            const int e = rd * 256 + tid;
            u32x4 v = xg[rd];
            if (p.ragged) {
                const int ncols = xg_inf[rd] >> 4;
                const int over = xg_off[rd] + chunk * 16 * HWin + 8 - xtotal;
                if (xg_off[rd] != NEVER && over > 0) v = shift_down(v, over);
                if (ncols < 8) v = keep_first(v, ncols);
            }
            if (e < xt_items) reinterpret_cast<u32x4 *>(xt)[e] = v;
        }
    };
    // XT: parked patch -> MFMA layout of patch buffer xb.
    auto x_transpose = [&](uint4 *xb) {
        const bf16_t *st = reinterpret_cast<const bf16_t *>(xt);
        const int chs = p.xt_rows * p.xt_cols;
#pragma unroll
        for (int rd = 0; rd < (XT ? XTR : 0); ++rd) {
            if (!WIDE && rd >= xrounds) break;
            const int src = xs_sd[rd] & 0xffffu, dst = xs_sd[rd] >> 16;
            if (dst != 0xffff) {
                uint32_t r[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) r[i] = st[src + i * chs];
                u32x4 v = {r[0] | (r[1] << 16), r[2] | (r[3] << 16), r[4] | (r[5] << 16), r[6] | (r[7] << 16)};
                reinterpret_cast<u32x4 *>(xb)[dst] = v;
            }
        }
    };

    // Global loads of the filter slab of stage (chunk, sg).
    auto load_w = [&](int chunk, int sg) {
        if (WM) {
        } else if (STAGED) {
            const uint4 *src = reinterpret_cast<const uint4 *>(w) +
                               ((size_t)(chunk * NSUB + sg) * TRES * p.Mpad + k0) * 2;
#pragma unroll
            for (int it = 0; it < WITEMS; ++it) {
                const int e = min(it * 256 + tid, WSZ - 1);
                const int tl = e / (KT * 2), rem = e - tl * (KT * 2);
                const uint4 v = src[(size_t)tl * p.Mpad * 2 + rem];
                __builtin_memcpy(&wreg[it], &v, 16);
            }
        } else {
            const int c0 = chunk * 16;
            const int tapoff = p.tflip ? -sg * SG : sg * SG;
            if (c0 + 16 <= p.Cin) {
                const bf16_t *src = w + (ptrdiff_t)c0 * p.w_sr + tapoff;
#pragma unroll
                for (int it = 0; it < WITEMS; ++it)
#pragma unroll
                    for (int i = 0; i < 8; ++i) wreg[it][i] = src[(size_t)i * p.w_sr + wsrc[it]];
            } else {
#pragma unroll
                for (int it = 0; it < WITEMS; ++it) {
                    const int o = STAGED ? 0 : ((wdst[it] & 1) ^ swz(wdst[it] >> 1));
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        const int red = min(c0 + o * 8 + i, p.Cin - 1);
                        wreg[it][i] = w[(ptrdiff_t)red * p.w_sr + tapoff + (wsrc[it] - (uint32_t)(o * 8 * p.w_sr))];
                    }
                }
            }
        }
    };
    auto store_w = [&](uint4 *wb) {
#pragma unroll
        for (int it = 0; it < (WM ? 0 : WITEMS); ++it) {
            const int e = it * 256 + tid;
            if ((it + 1) * 256 <= WSZ || e < WSZ) {
                uint4 v;
                __builtin_memcpy(&v, &wreg[it], 16);
                wb[STAGED ? e : wdst[it]] = v;
            }
        }
    };

    // ---- DIRECT with the thread's share of a chunk's filter in registers (WM = 1 forward, 2 backward-data).
    // Thread (row, half o) of the KT x 2 items of a slab; with KT = 64 the upper two waves have none.
    constexpr int WCD = WM == 1 ? 4 * T : WM == 2 ? 40 : 1;   // dwords: 8 x T elements, or 8 runs of 10
    constexpr int NPRE = (WM && NSUB > 2) ? (NSUB - 2) * TRES : 1;
    uint32_t wc[WCD];
    u32x4 wpre[NPRE];   // the slabs of stages 2 .. NSUB-1, cut out at the end of stage 0
    const bool wc_on = KT * 2 >= 256 || tid < KT * 2;
    const int wc_row = WM == 2 ? tid % KT : tid >> 1, wc_o = WM == 2 ? (tid / KT) & 1 : tid & 1;
    const int wc_dst = wc_row * 2 + (wc_o ^ swz(wc_row));
    auto load_wc = [&](int chunk) {
        if (!WM || !wc_on) return;
        const int m = min(k0 + wc_row, p.Kout - 1);
        const bf16_t *src = w + (size_t)m * p.w_sm + (size_t)(chunk * 16 + wc_o * 8) * p.w_sr;
        if (WM == 1) {   // w_sr = T: 8 channels x T taps in one run
#pragma unroll
            for (int j = 0; j < T; ++j) {
                const u32x4 v = load8_any(src + 8 * j);
                wc[4 * j] = v.x; wc[4 * j + 1] = v.y; wc[4 * j + 2] = v.z; wc[4 * j + 3] = v.w;
            }
        } else {         // w_sm = T = 9: one run of 9 taps per channel, 8 + 1 elements
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const bf16_t *run = src + (size_t)i * p.w_sr;
                const u32x4 v = load8_any(run);
                wc[5 * i] = v.x; wc[5 * i + 1] = v.y; wc[5 * i + 2] = v.z; wc[5 * i + 3] = v.w;
                wc[5 * i + 4] = run[8];
            }
        }
    };
    // Item tl of the slab of stage sg: the thread's 8 channels at tap (tl / SG, sg * SG + tl % SG).
    auto cut_wc = [&](int sg, int tl) -> u32x4 {
        const int tap = (tl / SG) * S + sg * SG + tl % SG;
        u32x4 v;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int h0 = WM == 1 ? (2 * j) * T + tap : (2 * j) * 10 + (T - 1 - tap);
            const int h1 = WM == 1 ? (2 * j + 1) * T + tap : (2 * j + 1) * 10 + (T - 1 - tap);
            v[j] = pick2(wc, h0, h1);
        }
        return v;
    };
    auto store_wc = [&](uint4 *wb, int sg) {   // cuts the slab of stage sg and writes it
        if (!WM || !wc_on) return;
#pragma unroll
        for (int tl = 0; tl < TRES; ++tl) reinterpret_cast<u32x4 *>(wb)[tl * KT * 2 + wc_dst] = cut_wc(sg, tl);
    };

    // The MFMAs of one stage.
    auto compute = [&](const uint4 *xb, const uint4 *wb, int sg) {
#pragma unroll
        for (int sl = 0; sl < SG; ++sl) {
            const int s = sg * SG + sl;
            bf16x8 b[NB];
            if (WIDE) {
                const int slot = pixbase[0] + s;
                const uint4 *bp = xb + slot * 2 + (g ^ swz(slot));
#pragma unroll
                for (int j = 0; j < NB; ++j) b[j] = *reinterpret_cast<const bf16x8 *>(bp + j * WIDE_LWP * 2);
            }
#pragma unroll
            for (int r = 0; r < R; ++r) {
                if (!WIDE) {
#pragma unroll
                    for (int f = 0; f < NF; ++f) {
                        const int slot = pixbase[f] + s;
                        b[f] = *reinterpret_cast<const bf16x8 *>(xb + (slot + r * LWp) * 2 + (g ^ swz(slot)));
                    }
                }
                bf16x8 a[2];
#pragma unroll
                for (int i = 0; i < 2; ++i)
                    a[i] = *reinterpret_cast<const bf16x8 *>(wb + ((r * SG + sl) * KT + i * 32) * 2 + aidx);
#pragma unroll
                for (int f = 0; f < NF; ++f)
#pragma unroll
                    for (int i = 0; i < 2; ++i)
                        acc[i][f] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(WIDE ? b[f + r] : b[f], a[i], acc[i][f], 0, 0, 0);
            }
        }
    };

    if constexpr (STAGED) {
        // Packed filter: the slab of a stage is fetched two stages ahead into one of two
        // register sets (the set of a stage is its parity; two chunks are unrolled so that
        // the parity is known at compile time), and written to LDS one stage ahead.  The
        // patch of the next chunk is fetched during the first stage of a chunk and written
        // after its last.  Loads complete in order: a stage waits for the slab issued one
        // stage ago while the loads issued since stay in flight.  Every stage issues the
        // same loads, so the counts are exact; past the end they fetch the last slab / chunk
        // again, and what they bring is written to a buffer nobody reads.
        uint4 *const ws = smem + 2 * XS;
        const int nstage = p.nchunks * NSUB;
        u32x4 wr[2][WITEMS];
        auto load_ws = [&](int stage, u32x4(&dst)[WITEMS]) {
            const int st = min(stage, nstage - 1);
            const u32x4 *src = reinterpret_cast<const u32x4 *>(w) + ((size_t)st * TRES * p.Mpad + k0) * 2;
#pragma unroll
            for (int it = 0; it < WITEMS; ++it) {
                const int e = min(it * 256 + tid, WSZ - 1);
                const int tl = e / (KT * 2), rem = e - tl * (KT * 2);
                dst[it] = src[(size_t)tl * p.Mpad * 2 + rem];
            }
        };
        auto store_ws = [&](uint4 *wb, const u32x4(&srcr)[WITEMS]) {
#pragma unroll
            for (int it = 0; it < WITEMS; ++it) {
                const int e = it * 256 + tid;
                if ((it + 1) * 256 <= WSZ || e < WSZ) reinterpret_cast<u32x4 *>(wb)[e] = srcr[it];
            }
        };
        load_ws(0, wr[0]);
        load_ws(1, wr[1]);
        if (XT) {
            x_issue(0);
            x_park(0);
            __syncthreads();   // the zero fill is complete, the patch is parked
            x_transpose(xs);
        } else {
            load_x(0);
            __syncthreads();   // the zero fill is complete
            store_x(0, xs);
        }
        store_ws(ws, wr[0]);
        for (int chunk0 = 0; chunk0 < p.nchunks; chunk0 += 2) {
            static_for<2 * NSUB>([&](auto idx) {
                constexpr int c = decltype(idx)::value / NSUB, sg = decltype(idx)::value % NSUB;
                constexpr int par = decltype(idx)::value & 1;   // parity of the stage
                const int chunk = chunk0 + c;
                const int cnext = min(chunk + 1, p.nchunks - 1);
                uint4 *const xcur = xs + c * XS, *const xnext = xs + (c ^ 1) * XS;
                __syncthreads();
                if (!WIDE) {
                    // keeps the operand addresses of later stages from being worked out early
#pragma unroll
                    for (int f = 0; f < (WIDE ? 1 : NF); ++f) asm volatile("" : "+v"(pixbase[f]));
                }
                load_ws(chunk * NSUB + sg + 2, wr[par]);
                if (XT) {
                    // the next patch: loads in the first stage, parked after the second, transposed in the third
                    if (sg == 0) x_issue(cnext);
                    if (sg == 2) x_transpose(xnext);
                } else {
                    if (sg == 0) load_x(cnext);
                }
                __builtin_amdgcn_sched_barrier(0);   // the loads stay ahead of the MFMAs
                if (chunk < p.nchunks) compute(xcur, ws + par * WSZ, sg);
                __builtin_amdgcn_sched_barrier(0);
                store_ws(ws + (par ^ 1) * WSZ, wr[par ^ 1]);
                if (XT) {
                    if (sg == 1) x_park(cnext);
                } else {
                    if (sg == NSUB - 1) store_x(cnext, xnext);
                }
            });
        }
    } else if constexpr (WM != 0) {
    // Filter share of a chunk in registers.  The slab of stage 1 is cut and written at the end of
    // stage 0, those of the later stages are cut then too and wait in registers, so that the loads
    // of the next chunk's share can go out at the start of stage 1 and have until the end of the
    // chunk's last stage to arrive.  With one stage per chunk they go out at its start.
    uint4 *const ws = smem + 2 * XS;
    load_wc(0);
    if (XT) {
        x_issue(0);
        x_park(0);
        __syncthreads();   // the zero fill is complete, the patch is parked
        x_transpose(xs);
    } else {
        load_x(0);
        __syncthreads();   // the zero fill is complete
        store_x(0, xs);
    }
    store_wc(ws, 0);
    int wpar = 0;
    for (int chunk = 0; chunk < p.nchunks; ++chunk) {
        const int cnext = min(chunk + 1, p.nchunks - 1);
        uint4 *const xcur = xs + (chunk & 1) * XS, *const xnext = xs + ((chunk + 1) & 1) * XS;
        if (!WIDE) {
#pragma unroll
            for (int f = 0; f < (WIDE ? 1 : NF); ++f) asm volatile("" : "+v"(pixbase[f]));
        }
#pragma unroll
        for (int sg = 0; sg < NSUB; ++sg) {
            __syncthreads();
            if (sg == (NSUB > 1 ? 1 : 0)) load_wc(cnext);
            if (XT) {
                if (sg == 0) x_issue(cnext);
                if (sg == 2) x_transpose(xnext);
            } else {
                if (sg == 0) load_x(cnext);
            }
            __builtin_amdgcn_sched_barrier(0);   // the loads stay ahead of the MFMAs
            compute(xcur, ws + wpar * WSZ, sg);
            __builtin_amdgcn_sched_barrier(0);
            wpar ^= 1;
            if (NSUB == 1) {
                store_wc(ws + wpar * WSZ, 0);
            } else if (sg == 0) {
                store_wc(ws + wpar * WSZ, 1);
                if (wc_on) {
#pragma unroll
                    for (int s2 = 2; s2 < NSUB; ++s2)
#pragma unroll
                        for (int tl = 0; tl < TRES; ++tl) wpre[(s2 - 2) * TRES + tl] = cut_wc(s2, tl);
                }
            } else if (sg + 1 < NSUB) {
                if (wc_on) {
#pragma unroll
                    for (int tl = 0; tl < TRES; ++tl)
                        reinterpret_cast<u32x4 *>(ws + wpar * WSZ)[tl * KT * 2 + wc_dst] = wpre[(sg - 1) * TRES + tl];
                }
            } else {
                store_wc(ws + wpar * WSZ, 0);
            }
            if (XT) {
                if (sg == 1) x_park(cnext);
            } else {
                if (sg == NSUB - 1) store_x(cnext, xnext);
            }
        }
    }
    } else {
    uint4 *const ws = smem + 2 * XS;
    load_w(0, 0);
    if (XT) {
        x_issue(0);
        x_park(0);
        __syncthreads();   // the zero fill is complete, the patch is parked
        x_transpose(xs);
    } else {
        load_x(0);
        __syncthreads();   // the zero fill is complete
        store_x(0, xs);
    }
    store_w(ws);
    int wpar = 0;
    // Every stage issues the same loads and stores, so that the wait counters are exact:
    // past the end they fetch the last stage / chunk again, into a buffer nobody reads.
    for (int chunk = 0; chunk < p.nchunks; ++chunk) {
        const int cnext = min(chunk + 1, p.nchunks - 1);
        uint4 *const xcur = xs + (chunk & 1) * XS, *const xnext = xs + ((chunk + 1) & 1) * XS;
        if (!WIDE) {
            // keeps the per-tap operand addresses from being hoisted out of the loop into registers
#pragma unroll
            for (int f = 0; f < (WIDE ? 1 : NF); ++f) asm volatile("" : "+v"(pixbase[f]));
        }
#pragma unroll
        for (int sg = 0; sg < NSUB; ++sg) {
            __syncthreads();
            if (sg + 1 < NSUB) load_w(chunk, sg + 1);
            else load_w(cnext, chunk + 1 < p.nchunks ? 0 : NSUB - 1);
            if (XT) {
                if (sg == 0) x_issue(cnext);
                if (sg == 2) x_transpose(xnext);
            } else {
                if (sg == 0) load_x(cnext);
            }
            __builtin_amdgcn_sched_barrier(0);   // the loads stay ahead of the MFMAs
            compute(xcur, ws + wpar * WSZ, sg);
            __builtin_amdgcn_sched_barrier(0);
            wpar ^= 1;
            store_w(ws + wpar * WSZ);
            if (XT) {
                if (sg == 1) x_park(cnext);
            } else {
                if (sg == NSUB - 1) store_x(cnext, xnext);
            }
        }
    }
    }

    // ---- epilogue.  The MFMAs take the pixels as rows, so a lane holds, for output
    // channel lane % 32 of a tile, the pixels 8*(v/4) + 4*(lane/32) + v%4: four
    // consecutive pixels per group of four registers.
    const int PQ = p.Pout * p.Qout;
    auto pix_off = [&](int i) -> int {   // offset of pixel i of the tile in channel 0, -1: not an output
        const int rl = i / p.TW, cl = i - rl * p.TW;
        const int o = o0 + rl;
        if (!(rl < p.TH && o < NP && q0 + cl < p.Qout)) return -1;
        const int n = o / p.Pout, pp = o - n * p.Pout;
        return (n * p.Kout * p.Pout + pp) * p.Qout + q0 + cl;
    };
    if (p.stats)
        tile_bn_partials<NF, KT == 128 ? 2 : 4>(acc, p.TW, min(p.TH, NP - o0), p.Qout - q0, wp, wk, l32, g, k0 + wk * 64, p.Kout, p.out_bf16 != 0, p.stats,
                                                p.nptiles, ptile, reinterpret_cast<float *>(smem));
    if (p.out_bf16) {
        // bf16: through LDS, 32 channels x NF*32 pixels per wave and pass, so that a lane
        // writes 8 consecutive pixels of one channel with one 16-byte store
        constexpr int EP = EPI_PITCH;
        __syncthreads();   // the last stage has been read
        char *const stage = reinterpret_cast<char *>(smem) + wave * 32 * EP;
        constexpr int OCT = NF * 4, KPR = 64 / OCT;   // octets per channel row; channel rows per round
        const int oct = lane % OCT, krow = lane / OCT;
        const int i0 = wp * NF * 32 + oct * 8;
        const int off0 = pix_off(i0), off7 = pix_off(i0 + 7);
        const bool contig = off0 >= 0 && off7 == off0 + 7;
        int eoff[8];
        bool any = false;
        if (!contig) {
#pragma unroll
            for (int e = 0; e < 8; ++e) { eoff[e] = pix_off(i0 + e); any = any || eoff[e] >= 0; }
        }
        bf16_t *const o16 = reinterpret_cast<bf16_t *>(out);
#pragma unroll
        for (int i = 0; i < 2; ++i) {
#pragma unroll
            for (int f = 0; f < NF; ++f)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    uint2 v;
                    v.x = pack2_bf16(acc[i][f][4 * j], acc[i][f][4 * j + 1]);
                    v.y = pack2_bf16(acc[i][f][4 * j + 2], acc[i][f][4 * j + 3]);
                    *reinterpret_cast<uint2 *>(stage + l32 * EP + (f * 32 + 8 * j + 4 * g) * 2) = v;
                }
            __syncthreads();
#pragma unroll
            for (int rd = 0; rd < 32 / KPR; ++rd) {
                const int kl = rd * KPR + krow, k = k0 + wk * 64 + i * 32 + kl;
                const uint4 v = *reinterpret_cast<const uint4 *>(stage + kl * EP + oct * 16);
                if (k >= p.Kout) continue;
                if (contig) {
                    store8_any(o16 + (size_t)k * PQ + off0, v);
                } else if (any) {
                    const uint32_t d[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        if (eoff[e] >= 0) o16[(size_t)k * PQ + eoff[e]] = (bf16_t)(d[e >> 1] >> (16 * (e & 1)));
                }
            }
            if (i == 0) __syncthreads();
        }
    } else {
        float *const o32 = reinterpret_cast<float *>(out);
#pragma unroll
        for (int f = 0; f < NF; ++f)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int off = pix_off((wp * NF + f) * 32 + 8 * j + 4 * g + e);
                    if (off < 0) continue;
#pragma unroll
                    for (int i = 0; i < 2; ++i) {
                        const int k = k0 + wk * 64 + i * 32 + l32;
                        if (k < p.Kout) o32[(size_t)k * PQ + off] = acc[i][f][4 * j + e];
                    }
                }
    }
}



template <int R, int S, int KT, int NF, bool STAGED, bool WIDE, int WM = 0>
hipError_t launch_one(const bf16_t *in, const bf16_t *w, void *out, const Plan &pl, hipStream_t st)
{
    auto kern = conv_tile_kernel<R, S, KT, NF, STAGED, WIDE, WM>;
    // the limit of dynamic LDS is a property of the kernel, set once (thread-safe initialisation)
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, LDS_LIMIT);
    if (attr != hipSuccess) return attr;
    hipLaunchKernelGGL(kern, pl.grid, dim3(256), pl.lds, st, in, w, out, pl.p);
    return hipGetLastError();
}

// DIRECT with the filter share of a chunk in registers: 3x3 either direction, 1x1 forward; the
// reduction channels must come in whole chunks.
template <int R, int S, int NF, int WM>
hipError_t launch_wm(const bf16_t *in, const bf16_t *w, void *out, const Plan &pl, hipStream_t st)
{
    const int sel = (pl.KT == 128 ? 2 : 0) | (pl.wide ? 1 : 0);
    switch (sel) {
    case 0: return launch_one<R, S, 64, NF, false, false, WM>(in, w, out, pl, st);
    case 1: return launch_one<R, S, 64, NF, false, true, WM>(in, w, out, pl, st);
    case 2: return launch_one<R, S, 128, NF, false, false, WM>(in, w, out, pl, st);
    default: return launch_one<R, S, 128, NF, false, true, WM>(in, w, out, pl, st);
    }
}

template <int R, int S, int NF>
hipError_t launch_nf(const bf16_t *in, const bf16_t *w, void *out, const Plan &pl, bool staged, hipStream_t st)
{
    if (!staged && pl.p.Cin % 16 == 0) {
        if constexpr (R == 3 && S == 3) {
            if (pl.p.tflip) return launch_wm<R, S, NF, 2>(in, w, out, pl, st);
            return launch_wm<R, S, NF, 1>(in, w, out, pl, st);
        }
        if constexpr (R == 1 && S == 1) {
            if (!pl.p.tflip) return launch_wm<R, S, NF, 1>(in, w, out, pl, st);
        }
    }
    const int sel = (pl.KT == 128 ? 4 : 0) | (staged ? 2 : 0) | (pl.wide ? 1 : 0);
    switch (sel) {
    case 0: return launch_one<R, S, 64, NF, false, false>(in, w, out, pl, st);
    case 1: return launch_one<R, S, 64, NF, false, true>(in, w, out, pl, st);
    case 2: return launch_one<R, S, 64, NF, true, false>(in, w, out, pl, st);
    case 3: return launch_one<R, S, 64, NF, true, true>(in, w, out, pl, st);
    case 4: return launch_one<R, S, 128, NF, false, false>(in, w, out, pl, st);
    case 5: return launch_one<R, S, 128, NF, false, true>(in, w, out, pl, st);
    case 6: return launch_one<R, S, 128, NF, true, false>(in, w, out, pl, st);
    default: return launch_one<R, S, 128, NF, true, true>(in, w, out, pl, st);
    }
}

// MULTI: the filter has kernels for every tile size (NF = 4, 2, 1), else only the largest.
template <int R, int S, bool MULTI>
hipError_t launch_rs(const bf16_t *in, const bf16_t *w, void *out, const Plan &pl, bool staged, hipStream_t st)
{
    if (MULTI && pl.NF == 2) return launch_nf<R, S, MULTI ? 2 : 4>(in, w, out, pl, staged, st);
    if (MULTI && pl.NF == 1) return launch_nf<R, S, MULTI ? 1 : 4>(in, w, out, pl, staged, st);
    return launch_nf<R, S, 4>(in, w, out, pl, staged, st);
}

}  // namespace

// One translation unit per filter group, so that they compile side by side.
hipError_t launch_tile_3x3(const bf16_t *in, const bf16_t *w, void *out, const Plan &pl, bool staged, hipStream_t st);
hipError_t launch_tile_1x1(const bf16_t *in, const bf16_t *w, void *out, const Plan &pl, bool staged, hipStream_t st);
hipError_t launch_tile_other(int R, int S, const bf16_t *in, const bf16_t *w, void *out, const Plan &pl, bool staged,
                             hipStream_t st);

}  // namespace sn
