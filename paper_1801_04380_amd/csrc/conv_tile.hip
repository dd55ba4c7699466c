// Host side of the stride-1 bf16 tile convolution (the kernel is in conv_tile.h): the
// filter packing kernel, the choice of the tiling, and the entry points.
#include "conv_tile2.h"

namespace sn {
namespace {

// Packs A(m, red, tap) into [chunk = red/16][stage][tap of the stage][Mpad][16],
// zero padded, the two 8-channel halves of a row swapped where the LDS swizzle
// swaps them: a stage's slab is copied to LDS (or read by the MFMA lanes) as it is.
// One thread per 16-byte item (8 channels of one row and tap).
__global__ void __launch_bounds__(256)
pack_filter_kernel(const bf16_t *__restrict__ w, uint4 *__restrict__ wp, int M, int RED, int R, int S, int SG,
                   int w_sm, int w_sr, int tflip, int Mpad, size_t items)
{
    // Threads are numbered so that neighbours read neighbouring source elements: the tap runs
    // fastest, then (forward) the half and the row, or (backward-data) the row and the half.
    // (the filter has fewer than 2^31 elements, so there are fewer than 2^28 items: 32-bit arithmetic)
    if ((size_t)blockIdx.x * 256 + threadIdx.x >= items) return;
    uint32_t q = blockIdx.x * 256u + threadIdx.x;
    const int T = R * S, TRES = R * SG, NSUB = S / SG;
    const int tap = (int)(q % (uint32_t)T);
    q /= (uint32_t)T;
    int hs, m;
    if (tflip) { m = (int)(q % (uint32_t)Mpad); q /= (uint32_t)Mpad; hs = (int)(q & 1); q >>= 1; }
    else { hs = (int)(q & 1); q >>= 1; m = (int)(q % (uint32_t)Mpad); q /= (uint32_t)Mpad; }
    const int chunk = (int)q;
    const int r = tap / S, s = tap - r * S, sg = s / SG, tl = r * SG + (s - sg * SG);
    const size_t it = ((((size_t)chunk * NSUB + sg) * TRES + tl) * Mpad + m) * 2 + hs;
    const int red0 = chunk * 16 + (hs ^ swz(m)) * 8;
    uint32_t d[4] = {0, 0, 0, 0};
    if (m < M) {
        const bf16_t *src = w + (size_t)m * w_sm + (size_t)red0 * w_sr + (tflip ? T - 1 - tap : tap);
#pragma unroll
        for (int j = 0; j < 8; ++j)
            if (red0 + j < RED) d[j >> 1] |= (uint32_t)src[(size_t)j * w_sr] << (16 * (j & 1));
    }
    wp[it] = make_uint4(d[0], d[1], d[2], d[3]);
}

// The same packing for whole chunks of 3x3 filters with 16-byte loads: one thread per (chunk, row m,
// 8-channel half) fetches its 8 channels x 9 taps -- forward: one contiguous run of the KCRS tensor;
// backward-data: eight runs of 9 taps -- and cuts the nine 16-byte items out of registers (the
// cut the zero-workspace kernel makes per stage, see conv_tile.h).  RED must be a multiple of 16.
template <bool TFLIP>
__global__ void __launch_bounds__(256)
pack_filter9_kernel(const bf16_t *__restrict__ w, uint4 *__restrict__ wp, int M, int w_sm, int w_sr, int Mpad, uint32_t nthreads)
{
    constexpr int T = 9, S = 3, TRES = 3, NSUB = 3;
    uint32_t q = blockIdx.x * 256u + threadIdx.x;
    if (q >= nthreads) return;
    const int hs = (int)(q & 1);
    q >>= 1;
    const int m = (int)(q % (uint32_t)Mpad), chunk = (int)(q / (uint32_t)Mpad);
    const int red0 = chunk * 16 + (hs ^ swz(m)) * 8;
    constexpr int WCD = TFLIP ? 40 : 36;
    uint32_t wc[WCD];
    if (m < M) {
        const bf16_t *src = w + (size_t)m * w_sm + (size_t)red0 * w_sr;
        if (!TFLIP) {
#pragma unroll
            for (int j = 0; j < T; ++j) {
                const u32x4 v = load8_any(src + 8 * j);
                wc[4 * j] = v.x; wc[4 * j + 1] = v.y; wc[4 * j + 2] = v.z; wc[4 * j + 3] = v.w;
            }
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const bf16_t *run = src + (size_t)i * w_sr;
                const u32x4 v = load8_any(run);
                wc[5 * i] = v.x; wc[5 * i + 1] = v.y; wc[5 * i + 2] = v.z; wc[5 * i + 3] = v.w;
                wc[5 * i + 4] = run[8];
            }
        }
    } else {
#pragma unroll
        for (int i = 0; i < WCD; ++i) wc[i] = 0;
    }
#pragma unroll
    for (int tap = 0; tap < T; ++tap) {
        const int r = tap / S, s = tap - r * S;   // stage s, item r of the stage
        uint32_t d[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int h0 = TFLIP ? (2 * j) * 10 + (T - 1 - tap) : (2 * j) * T + tap;
            const int h1 = TFLIP ? (2 * j + 1) * 10 + (T - 1 - tap) : (2 * j + 1) * T + tap;
            d[j] = pick2(wc, h0, h1);
        }
        const size_t it = ((((size_t)chunk * NSUB + s) * TRES + r) * Mpad + m) * 2 + hs;
        wp[it] = make_uint4(d[0], d[1], d[2], d[3]);
    }
}

// Tiling for one problem with NF 32-pixel tiles per wave; false if the patch would not fit in LDS.
bool plan_for(const TileProblem &base, int R, int S, int NF, Plan *pl, bool prefer_narrow = false)
{
    TileProblem p = base;
    const int KT = p.Kout <= 64 ? 64 : 128;
    const int PIXT = (KT == 128 ? 2 : 4) * NF * 32;
    const long long NP = (long long)p.N * p.Pout;
    const bool xt3 = S / sg_of(R, S) >= 3;   // WIDE tiling: the patch is parked in LDS before it is transposed
    p.ragged = p.Win % 8 != 0;
    long long nrowtiles = 0;
    bool wide = p.Qout > 64;
    if (!wide) {
        // pixels of the tile that are real outputs, per tiling
        const int th = PIXT / p.Qout;
        const double eff_narrow = (double)th * p.Qout / PIXT;
        const int ct = (p.Qout + 31) / 32;
        const double eff_wide = (double)p.Qout / (ct * 32);
        wide = (prefer_narrow ? eff_wide > eff_narrow : eff_wide >= eff_narrow) && p.Pout >= PIXT / 32;
    }
    if (!wide) {
        p.TW = p.Qout;
        p.TH = PIXT / p.Qout;
        p.ncoltiles = 1;
        p.tiles_per_img = 0;
        if (p.TH > NP) p.TH = (int)NP;
        nrowtiles = (NP + p.TH - 1) / p.TH;
        p.LW = p.TW + S - 1;
        p.LWp = (p.LW + 15) / 16 * 16;
        // most patch rows a tile can need: TH rows, one halo, and one more halo per image boundary inside it
        const int crossings = p.N > 1 ? (p.TH - 1) / p.Pout + 1 : 0;
        const int lrows_max = p.TH + (crossings + 1) * (R - 1);
        if ((long long)lrows_max * ((p.LW + 1) / 2) > XPAIRS_MAX) return false;
        p.xslots = lrows_max * p.LWp;
        p.xt_rows = lrows_max;
        p.xt_cols = (p.Win + 7) / 8 * 8;
    } else {
        p.TW = 32;
        p.TH = PIXT / 32;
        p.ncoltiles = (p.Qout + 31) / 32;
        p.xslots = (p.TH + R - 1) * WIDE_LWP;
        p.xt_rows = p.TH + R - 1;
        p.xt_cols = WIDE_LWP;
        if (p.TH > p.Pout) p.TH = p.Pout;
        p.tiles_per_img = (p.Pout + p.TH - 1) / p.TH;
        nrowtiles = (long long)p.N * p.tiles_per_img;
        p.LW = p.TW + S - 1;
        p.LWp = WIDE_LWP;
        if (p.LW > WIDE_LWP) return false;
    }
    p.Hp = p.Pout + R - 1;
    p.nchunks = (p.Cin + 15) / 16;
    p.Mpad = (p.Kout + KT - 1) / KT * KT;
    size_t lds = ((size_t)2 * p.xslots * 2 + (size_t)2 * R * sg_of(R, S) * KT * 2) * 16;
    if (xt3 && wide && KT == 128) lds += (size_t)16 * p.xt_rows * p.xt_cols * sizeof(bf16_t);
    if (lds < (size_t)4 * 32 * EPI_PITCH) lds = (size_t)4 * 32 * EPI_PITCH;   // the epilogue's staging
    if (lds > (size_t)LDS_LIMIT) return false;
    if (nrowtiles * p.ncoltiles > 0x7fffffffLL) return false;
    pl->p = p;
    pl->KT = KT;
    pl->NF = NF;
    pl->wide = wide;
    pl->lds = lds;
    // one-dimensional grid, mapped to (pixel tile, channel tile) inside the kernel (see there)
    p.nptiles = (int)(nrowtiles * p.ncoltiles);
    p.nktiles = (p.Kout + KT - 1) / KT;
    p.pt_per_xcd = (p.nptiles + 7) / 8;
    long long nwg = 8LL * p.pt_per_xcd * p.nktiles;
    p.kmajor = 0;
    p.kk = 1;
    // a packed filter of more than half an XCD's L2 (4 MB), and a channel tile count that spreads evenly
    const size_t filter_bytes = (size_t)p.nchunks * R * S * p.Mpad * 16 * sizeof(bf16_t);
    if (filter_bytes > ((size_t)2 << 20) && p.nktiles >= 2 && (p.nktiles < 8 ? 8 % p.nktiles == 0 : p.nktiles % 8 == 0)) {
        p.kmajor = p.nktiles < 8 ? p.nktiles : 8;
        p.kk = p.nktiles < 8 ? 1 : p.nktiles / 8;
        const int groups = 8 / p.kmajor;
        p.pt_per_xcd = (p.nptiles + groups - 1) / groups;
        nwg = 8LL * p.kk * p.pt_per_xcd;
    }
    if (nwg > 0x7fffffffLL) return false;
    pl->p = p;
    pl->grid = dim3((unsigned)nwg, 1, 1);
    return true;
}

// The tiling for one problem: the largest tile, unless (3x3 and 1x1 filters, which have the
// kernels) that leaves compute units without work and a smaller one does not.
bool make_plan(const TileProblem &base, int R, int S, bool staged, Plan *pl, bool prefer_narrow = false)
{
    if (!plan_for(base, R, S, 4, pl, prefer_narrow)) {
        // 5x5 with at most 64 output channels: the patch of the 512-pixel tile does not fit LDS, a smaller one does
        if (!(R == 5 && S == 5)) return false;
        return plan_for(base, R, S, 2, pl, prefer_narrow) || plan_for(base, R, S, 1, pl, prefer_narrow);
    }
    const bool multi = (R == 3 && S == 3) || (R == 1 && S == 1);
    if (!multi) return true;
    // 3x3 with at most 64 output channels and the packed filter: 256-pixel tiles (twice the workgroups per
    // compute unit cover the short channel loops' start and end better; measured 216 -> 190 us on 64 x 64
    // channels at 224 x 224; with the filter gathered in the kernel the larger tile wins)
    if (staged && R == 3 && pl->KT == 64) {
        Plan alt;
        if (plan_for(base, R, S, 2, &alt, prefer_narrow)) *pl = alt;
        return true;
    }
    // fewer workgroups than compute units: halve the pixels per workgroup
    if ((long long)pl->p.nptiles * pl->p.nktiles < 256) {
        Plan alt;
        if (plan_for(base, R, S, 2, &alt, prefer_narrow)) *pl = alt;
    }
    // still under half of them (7x7 images): halve again
    if (pl->NF == 2 && (long long)pl->p.nptiles * pl->p.nktiles < 128) {
        Plan alt;
        if (plan_for(base, R, S, 1, &alt, prefer_narrow)) *pl = alt;
    }
    return true;
}

// The tiling for the second-generation kernel (conv_tile2.h), or false where it does not apply:
// 3x3 filters, an even image width (a multiple of 8 for the WIDE tiling), an input tensor of at
// most 2 GiB; with at most 64 output channels only the WIDE tiling and 96 input channels or more.
bool make_plan2(const TileProblem &base, int R, int S, Plan *pl)
{
    if (!(R == 3 && S == 3) || base.Win % 2 != 0) return false;
    if (base.Kout <= 64) {
        // one 64-channel tile: four waves along the pixels, 2 x 32 pixels each, on 8 x 32 patches.  With few
        // input channels (measured: 64) the first-generation kernel's 512-pixel tiles are faster: the loop
        // is too short to pay for this kernel's longer prologue, and the tiles are half the size.
        if (base.Win % 8 != 0 || base.Cin < 96 || !plan_for(base, R, S, 2, pl) || pl->KT != 64 || !pl->wide) return false;
    } else if (!make_plan(base, R, S, true, pl, base.Win % 8 != 0) || pl->KT != 128 || (pl->NF != 4 && pl->NF != 2)) {
        // (a width that rules out the WIDE tiling here, not a multiple of 8: whole rows where they fill the tile as well)
        return false;
    }
    TileProblem &p = pl->p;
    int dw = p.Win % 8 == 0 ? 16 : 4;
    if (pl->wide && dw != 16) return false;
    const int pixt = (pl->KT == 128 ? 2 : 4) * pl->NF * 32;
    if (pl->wide) {
        p.xt_rows = pixt / 32 + R - 1;
        p.xt_cols = WIDE_LWP;
    }
    // xt_rows = the most patch rows of a tile (set by plan_for for whole rows); a parked row holds `group` image rows
    // (0: one, on its own 16- or 4-byte boundary).  Units of d bytes per parked channel, and what follows from them:
    auto park = [&](int d, int cols, int group) {
        const int prows = group > 1 ? (p.xt_rows + group - 1) / group + 1 : p.xt_rows;
        const int units = prows * (cols * 2 / d);
        const int upc = units <= 64 ? 64 : units <= 128 ? 128 : 256;
        if (units > 256 || (d == 16 && upc != 64)) return false;
        const int ncg = group ? (p.Win + 2 + 15) / 16 : (cols + 15) / 16;
        const int xtr = (2 * p.xt_rows * ncg + 15) / 16;
        if (!pl->wide && xtr > V2_XTR_MAX_NARROW) return false;
        dw = d; p.xt_cols = cols; p.xt_shift = group; p.xt_ncg = ncg; p.xt_upc = upc;
        p.xg_rounds = 16 * upc / 256;
        p.xtr_rounds = xtr;
        return true;
    };
    // Whole rows that are not multiples of 16 bytes: 16-byte loads all the same where one row (28 columns) or two
    // consecutive rows (14 columns) are a multiple of 8 bytes and every channel starts on one: a parked row then
    // starts at the 16-byte boundary at or below its first image row.  If the longer parked rows do not fit: 4-byte loads.
    const long long HW = (long long)p.Hin * p.Win;
    const bool tight = !pl->wide && dw == 4;
    const bool shift1 = tight && p.Win % 4 == 0 && HW % 8 == 0;
    const bool shift2 = tight && !shift1 && p.Win % 2 == 0 && p.Hin % 2 == 0 && p.Hp % 2 == 0 && HW % 4 == 0 &&
                        (p.Cin * HW) % 8 == 0;
    if (!(shift1 && park(16, (p.Win + 4 + 7) / 8 * 8, 1)) && !(shift2 && park(16, (2 * p.Win + 4 + 7) / 8 * 8, 2)) &&
        !park(dw, pl->wide ? WIDE_LWP : dw == 16 ? p.Win : (p.Win + 3) / 4 * 4, 0))
        return false;
    const int chstride = p.xt_upc * dw + V2_CH_PAD;
    p.pk_bytes = (16 * chstride + V2_PK_SLACK + 15) / 16 * 16;
    if (p.pk_bytes > 0xffff) return false;   // transposition offsets are 16 bits
    if ((p.xslots * 2 + V2_TRASH) > 0xffff) return false;
    const unsigned long long in_bytes = 2ull * p.N * p.Cin * p.Hin * p.Win;
    const unsigned long long w_bytes = 32ull * p.nchunks * R * S * p.Mpad;
    if (in_bytes > 0x80000000ull || w_bytes >= 0xfffffff0ull) return false;
    p.in_bytes = (uint32_t)in_bytes;
    p.w_bytes = (uint32_t)w_bytes;
    const size_t set_bytes = (size_t)2 * (p.xslots * 2 + V2_TRASH) * 16 + (size_t)2 * p.pk_bytes;
    size_t lds = set_bytes;
    if (lds < (size_t)4 * 32 * EPI_PITCH) lds = (size_t)4 * 32 * EPI_PITCH;
    if (lds > (size_t)LDS_LIMIT) return false;
    pl->lds = lds;
    pl->dw = dw;
    pl->ks = 1;
    // Tiles that leave compute units without a workgroup (small images): two sets of waves per
    // workgroup split the tile's chunks.  LDS: both sets' buffers, the 8 waves' epilogue staging,
    // and half of a set's accumulators for the sum of the two.
    if (pl->NF == 2 && !pl->wide && p.nchunks % 2 == 0 && p.nchunks >= 4 && (long long)p.nptiles * p.nktiles <= 256) {
        size_t lds2 = 2 * set_bytes;
        if (lds2 < (size_t)8 * 32 * EPI_PITCH) lds2 = (size_t)8 * 32 * EPI_PITCH;
        if (lds2 < (size_t)4 * pl->NF * 16 * 64 * sizeof(float)) lds2 = (size_t)4 * pl->NF * 16 * 64 * sizeof(float);
        if (lds2 <= (size_t)LDS_LIMIT) {
            pl->ks = 2;
            pl->lds = lds2;
        }
    }
    return true;
}

bool problem_of(const ConvGeom &g, bool bwd_data, TileProblem *p)
{
    if (!g.in_bf16 || g.sh != 1 || g.sw != 1) return false;
    if (g.W < 2 || g.Q < 2) return false;   // the patch gather loads pixel pairs inside a row
    const long long lim = 0x7fffffffLL;
    if ((long long)g.N * g.C * g.H * g.W > lim || (long long)g.N * g.K * g.P * g.Q > lim) return false;
    if ((long long)g.K * g.C * g.R * g.S > lim) return false;
    const int T = g.R * g.S;
    if (!bwd_data) {
        p->N = g.N; p->Cin = g.C; p->Hin = g.H; p->Win = g.W;
        p->Kout = g.K; p->Pout = g.P; p->Qout = g.Q; p->padh = g.ph; p->padw = g.pw;
        p->w_sm = g.C * T; p->w_sr = T; p->tflip = 0;
    } else {
        if (g.ph > g.R - 1 || g.pw > g.S - 1) return false;
        p->N = g.N; p->Cin = g.K; p->Hin = g.P; p->Win = g.Q;
        p->Kout = g.C; p->Pout = g.H; p->Qout = g.W; p->padh = g.R - 1 - g.ph; p->padw = g.S - 1 - g.pw;
        p->w_sm = T; p->w_sr = g.C * T; p->tflip = 1;
    }
    p->out_bf16 = g.out_bf16;
    p->stats = nullptr;
    p->xt_shift = 0;
    p->xt_ncg = 0;
    return true;
}

bool filter_supported(int R, int S)
{
    return (R == 1 && S == 1) || (R == 2 && S == 2) || (R == 3 && S == 3) || (R == 5 && S == 5) || (R == 1 && S == 7) ||
           (R == 7 && S == 1);
}

}  // namespace

bool tile_conv_supported(const ConvGeom &g, bool bwd_data)
{
    TileProblem p;
    Plan pl;
    return filter_supported(g.R, g.S) && problem_of(g, bwd_data, &p) && make_plan(p, g.R, g.S, false, &pl) &&
           make_plan(p, g.R, g.S, true, &pl);
}

size_t tile_conv_packed_bytes(const ConvGeom &g, bool bwd_data)
{
    TileProblem p;
    Plan pl;
    if (!tile_conv_supported(g, bwd_data) || !problem_of(g, bwd_data, &p) || !make_plan(p, g.R, g.S, true, &pl)) return 0;
    return align_up((size_t)pl.p.nchunks * g.R * g.S * pl.p.Mpad * 16 * sizeof(bf16_t), 256);
}

// Pixel tiles of the plan launch_tile_conv would use (forward); 0 if the kernels do not apply.
int tile_conv_stats_tiles(const ConvGeom &g, bool staged, bool in_aligned16)
{
    TileProblem p;
    Plan pl, pl2;
    if (!tile_conv_supported(g, false) || !problem_of(g, false, &p) || !make_plan(p, g.R, g.S, staged, &pl)) return 0;
    if (staged && in_aligned16 && make_plan2(p, g.R, g.S, &pl2)) return pl2.p.nptiles;
    return pl.p.nptiles;
}

hipError_t launch_tile_conv(const void *in, const void *w, void *out, const ConvGeom &g, bool bwd_data,
                            void *packed, hipStream_t st, float *stats)
{
    TileProblem p;
    Plan pl;
    if (!tile_conv_supported(g, bwd_data) || !problem_of(g, bwd_data, &p) ||
        !make_plan(p, g.R, g.S, packed != nullptr, &pl))
        return hipErrorInvalidValue;
    if (stats && bwd_data) return hipErrorInvalidValue;
    if (!stats && pointwise_supported(g, bwd_data)) return launch_pointwise(in, w, out, g, bwd_data, st);
    pl.p.stats = stats;
    const bf16_t *wsrc = static_cast<const bf16_t *>(w);
    if (packed) {
        const size_t items = (size_t)pl.p.nchunks * g.R * g.S * pl.p.Mpad * 2;
        if (g.R == 3 && g.S == 3 && pl.p.Cin % 16 == 0) {
            const uint32_t nthreads = (uint32_t)(items / 9);
            const dim3 grid((nthreads + 255) / 256), block(256);
            if (pl.p.tflip)
                hipLaunchKernelGGL(pack_filter9_kernel<true>, grid, block, 0, st, wsrc, static_cast<uint4 *>(packed),
                                   pl.p.Kout, pl.p.w_sm, pl.p.w_sr, pl.p.Mpad, nthreads);
            else
                hipLaunchKernelGGL(pack_filter9_kernel<false>, grid, block, 0, st, wsrc, static_cast<uint4 *>(packed),
                                   pl.p.Kout, pl.p.w_sm, pl.p.w_sr, pl.p.Mpad, nthreads);
        } else
        hipLaunchKernelGGL(pack_filter_kernel, dim3((unsigned)((items + 255) / 256)), dim3(256), 0, st, wsrc,
                           static_cast<uint4 *>(packed), pl.p.Kout, pl.p.Cin, g.R, g.S, sg_of(g.R, g.S),
                           pl.p.w_sm, pl.p.w_sr, pl.p.tflip, pl.p.Mpad, items);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        wsrc = static_cast<const bf16_t *>(packed);
    }
    const bf16_t *src = static_cast<const bf16_t *>(in);
    const bool staged = packed != nullptr;
    Plan pl2;
    if (staged && reinterpret_cast<uintptr_t>(in) % 16 == 0 && make_plan2(p, g.R, g.S, &pl2)) {
        pl2.p.stats = stats;
        return launch_tile2_3x3(src, wsrc, out, pl2, st);
    }
    if (g.R == 1 && g.S == 1) return launch_tile_1x1(src, wsrc, out, pl, staged, st);
    if (g.R == 3 && g.S == 3) return launch_tile_3x3(src, wsrc, out, pl, staged, st);
    return launch_tile_other(g.R, g.S, src, wsrc, out, pl, staged, st);
}

}  // namespace sn
