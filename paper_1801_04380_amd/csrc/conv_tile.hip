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
// channels 16 at a time.  The pixels of a tile are TH consecutive rows of the
// flattened (image, output row) space times TW columns; TW = Qout for images up
// to 64 wide (so small images fill the lanes: a tile may span several images),
// otherwise 8x32 / 16x32 patches.  Per 16-channel chunk the workgroup keeps in
// LDS
//   xs: the input patch with halo, transposed to [pixel][16 channels] (32 bytes
//       per pixel, so one MFMA lane reads its 8 consecutive channels with a
//       single 16-byte load); the transposition happens on the way in: each lane
//       gathers 8 channels of one pixel with 2-byte loads that are coalesced
//       across lanes along the image row, and writes 16 bytes;
//   ws: the filter slab [tap][KT][16 channels].
// Both are XOR-swizzled on the 16-byte half index with bit 3 of the row index,
// which makes the 16-byte reads of 16 consecutive rows hit distinct banks.
// A tap (r,s) only shifts the pixel index by r*LW + s, so the nine taps of a 3x3
// filter reuse one patch.  Each wave multiplies a 64-channel x 128-pixel block
// with v_mfma_f32_32x32x16_bf16 (2 x 4 tiles, 128 accumulator registers).
// Global loads of the next stage are issued before the MFMAs of the current one.
//
// The filter slab comes either from a copy pre-packed into the caller's
// workspace in exactly the LDS order (STAGED algorithm: wide, contiguous loads),
// or is gathered from the KCRS tensor with 2-byte loads (DIRECT, no workspace).
#include "sn_internal.h"

namespace sn {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int XPIX_MAX = 640;  // input patch pixels held in LDS
constexpr int XROUNDS_MAX = (XPIX_MAX * 2 + 255) / 256;

struct TileProblem {
    int N, Cin, Hin, Win, Kout, Pout, Qout, padh, padw;
    int out_bf16;
    int TH, TW, LW;          // tile rows, tile columns, LDS patch width in pixels
    int ncoltiles;
    int tiles_per_img;       // > 0: row tiles never cross an image (used for wide images); 0: they may
    int Hp;                  // padded rows per image = Pout + R - 1
    int nchunks;             // ceil(Cin / 16)
    // filter access: A(m, red, tap) = w[m*w_sm + red*w_sr + (tflip ? T-1-tap : tap)]
    int w_sm, w_sr, tflip;
    int Mpad;                // rows per (chunk, tap) block of the packed filter
};

template <int R, int S, int KT> struct Cfg {
    static constexpr int T = R * S;
    // one filter row per stage: the filter slab staged through registers stays small
    // enough (S 16-byte pieces per thread at KT=128) for two workgroups per CU
    static constexpr int RG = 1;
    static constexpr int TRES = RG * S;
    static constexpr int NSUB = R / RG;  // stages per channel chunk
    static constexpr int PIXT = (KT == 128) ? 256 : 512;
    static constexpr int WITEMS = (TRES * KT * 2 + 255) / 256;
};

__device__ inline int swz(int row) { return (row >> 3) & 1; }

template <int R, int S, int KT, bool STAGED>
__global__ void __launch_bounds__(256, 2)
conv_tile_kernel(const bf16_t *__restrict__ in, const bf16_t *__restrict__ w, void *__restrict__ out, TileProblem p)
{
    typedef Cfg<R, S, KT> C;
    constexpr int T = C::T, TRES = C::TRES, NSUB = C::NSUB, WITEMS = C::WITEMS;
    __shared__ uint4 xs[XPIX_MAX * 2];
    __shared__ uint4 ws[TRES * KT * 2];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, g = lane >> 5;
    const int wk = (KT == 128) ? (wave >> 1) : 0;
    const int wp = (KT == 128) ? (wave & 1) : wave;

    // ---- tile geometry
    const int rowtile = blockIdx.x / p.ncoltiles, coltile = blockIdx.x - rowtile * p.ncoltiles;
    const int k0 = blockIdx.y * KT;
    const int q0 = coltile * p.TW;
    int o0, NP;                                  // first flattened (image, row) and the row limit
    if (p.tiles_per_img > 0) {
        const int img = rowtile / p.tiles_per_img;
        o0 = img * p.Pout + (rowtile - img * p.tiles_per_img) * p.TH;
        NP = (img + 1) * p.Pout;
    } else {
        o0 = rowtile * p.TH;
        NP = p.N * p.Pout;
    }
    const int n0 = o0 / p.Pout, u0 = n0 * p.Hp + (o0 - n0 * p.Pout);
    const int olast = min(o0 + p.TH, NP) - 1;
    const int nl = olast / p.Pout;
    const int lrows = nl * p.Hp + (olast - nl * p.Pout) - u0 + R;
    const int xpix = lrows * p.LW;
    const int HWin = p.Hin * p.Win;

    // ---- per-thread constants of the input-patch gather
    int xoff[XROUNDS_MAX];   // element offset of channel 0 of this thread's pixel, -1: zero fill
    const int xo = tid >> 7;  // which 8-channel half this thread gathers
#pragma unroll
    for (int rd = 0; rd < XROUNDS_MAX; ++rd) {
        const int lp = rd * 128 + (tid & 127);
        int off = -1;
        if (lp < xpix) {
            const int lrow = lp / p.LW, lcol = lp - lrow * p.LW;
            const int u = u0 + lrow, n = u / p.Hp, h = u - n * p.Hp - p.padh;
            const int v = q0 - p.padw + lcol;
            if (n < p.N && (unsigned)h < (unsigned)p.Hin && (unsigned)v < (unsigned)p.Win)
                off = (n * p.Cin * p.Hin + h) * p.Win + v;
        }
        xoff[rd] = off;
    }
    const int xrounds = (xpix + 127) >> 7;

    // ---- per-lane constants of the MFMA operand reads and of the output
    int pixbase[4], outoff[4];
#pragma unroll
    for (int f = 0; f < 4; ++f) {
        const int i = (wp * 4 + f) * 32 + l32;
        const int rl = i / p.TW, cl = i - rl * p.TW;
        const int o = o0 + rl;
        int pb = 0, oo = -1;
        if (rl < p.TH && o < NP && q0 + cl < p.Qout) {
            const int n = o / p.Pout, pp = o - n * p.Pout;
            pb = (n * p.Hp + pp - u0) * p.LW + cl;
            oo = (n * p.Kout * p.Pout + pp) * p.Qout + q0 + cl;
        }
        pixbase[f] = pb;
        outoff[f] = oo;
    }

    f32x16 acc[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int f = 0; f < 4; ++f)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][f][v] = 0.f;

    uint4 xreg[XROUNDS_MAX], wreg[WITEMS];

    auto prefetch = [&](int stage) {
        const int chunk = stage / NSUB, sub = stage - chunk * NSUB;
        const int c0 = chunk * 16;
        if (sub == 0) {
#pragma unroll
            for (int rd = 0; rd < XROUNDS_MAX; ++rd) {
                if (rd >= xrounds) break;
                unsigned short e[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const int c = c0 + xo * 8 + i;
                    e[i] = (xoff[rd] >= 0 && c < p.Cin) ? in[xoff[rd] + c * HWin] : (unsigned short)0;
                }
                xreg[rd] = make_uint4(e[0] | ((uint32_t)e[1] << 16), e[2] | ((uint32_t)e[3] << 16),
                                      e[4] | ((uint32_t)e[5] << 16), e[6] | ((uint32_t)e[7] << 16));
            }
        }
#pragma unroll
        for (int it = 0; it < WITEMS; ++it) {
            const int e = it * 256 + tid;
            uint4 val = make_uint4(0, 0, 0, 0);
            if (STAGED) {
                // packed filter: [chunk][tap][Mpad][16] in exactly the order of ws
                const int tl = e / (KT * 2), rem = e - tl * (KT * 2), row = rem >> 1, o = rem & 1;
                if (tl < TRES && k0 + row < p.Mpad) {
                    const size_t src = ((size_t)(chunk * T + sub * TRES + tl) * p.Mpad + k0 + row) * 2 + o;
                    val = reinterpret_cast<const uint4 *>(w)[src];
                }
            } else {
                // gather from KCRS: lanes run over taps fastest so that they follow memory
                int tl, row, o;
                if (p.tflip) {  // backward-data: (tap, m) contiguous for one red
                    tl = e % TRES; const int q = e / TRES; row = q % KT; o = q / KT;
                } else {        // forward: (red, tap) contiguous for one m
                    tl = e % TRES; const int q = e / TRES; o = q & 1; row = q >> 1;
                }
                if (e < TRES * KT * 2 && k0 + row < p.Kout) {
                    const int tap = sub * TRES + tl;
                    const int base = (k0 + row) * p.w_sm + (p.tflip ? T - 1 - tap : tap);
                    unsigned short el[8];
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        const int red = c0 + o * 8 + i;
                        el[i] = red < p.Cin ? w[base + red * p.w_sr] : (unsigned short)0;
                    }
                    val = make_uint4(el[0] | ((uint32_t)el[1] << 16), el[2] | ((uint32_t)el[3] << 16),
                                     el[4] | ((uint32_t)el[5] << 16), el[6] | ((uint32_t)el[7] << 16));
                }
            }
            wreg[it] = val;
        }
    };

    auto stage_store = [&](int stage) {
        const int sub = stage % NSUB;
        if (sub == 0) {
#pragma unroll
            for (int rd = 0; rd < XROUNDS_MAX; ++rd) {
                if (rd >= xrounds) break;
                const int lp = rd * 128 + (tid & 127);
                if (lp < xpix) xs[lp * 2 + (xo ^ swz(lp))] = xreg[rd];
            }
        }
#pragma unroll
        for (int it = 0; it < WITEMS; ++it) {
            const int e = it * 256 + tid;
            int tl, row, o;
            if (STAGED) {
                tl = e / (KT * 2); const int rem = e - tl * (KT * 2); row = rem >> 1; o = rem & 1;
            } else if (p.tflip) {
                tl = e % TRES; const int q = e / TRES; row = q % KT; o = q / KT;
            } else {
                tl = e % TRES; const int q = e / TRES; o = q & 1; row = q >> 1;
            }
            if (e < TRES * KT * 2) ws[(tl * KT + row) * 2 + (o ^ swz(row))] = wreg[it];
        }
    };

    auto compute = [&](int stage) {
        const int sub = stage % NSUB;
#pragma unroll
        for (int tl = 0; tl < TRES; ++tl) {
            const int tap = sub * TRES + tl;
            const int r = tap / S, s = tap - r * S;
            const int tapoff = r * p.LW + s;
            bf16x8 a[2], b[4];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int row = wk * 64 + i * 32 + l32;
                a[i] = *reinterpret_cast<const bf16x8 *>(&ws[(tl * KT + row) * 2 + (g ^ swz(row))]);
            }
#pragma unroll
            for (int f = 0; f < 4; ++f) {
                const int pix = pixbase[f] + tapoff;
                b[f] = *reinterpret_cast<const bf16x8 *>(&xs[pix * 2 + (g ^ swz(pix))]);
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int f = 0; f < 4; ++f)
                    acc[i][f] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[f], acc[i][f], 0, 0, 0);
        }
    };

    const int nstage = p.nchunks * NSUB;
    prefetch(0);
    for (int stage = 0; stage < nstage; ++stage) {
        __syncthreads();
        stage_store(stage);
        __syncthreads();
        if (stage + 1 < nstage) prefetch(stage + 1);
        compute(stage);
    }

    // ---- epilogue: a 32x32 tile keeps column (lane % 32), rows 8*(v/4) + 4*(lane/32) + v%4
    const int PQ = p.Pout * p.Qout;
#pragma unroll
    for (int f = 0; f < 4; ++f) {
        if (outoff[f] < 0) continue;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int k = k0 + wk * 64 + i * 32 + 8 * (v >> 2) + 4 * g + (v & 3);
                if (k >= p.Kout) continue;
                const int off = outoff[f] + k * PQ;
                if (p.out_bf16) reinterpret_cast<bf16_t *>(out)[off] = f32_to_bf16(acc[i][f][v]);
                else reinterpret_cast<float *>(out)[off] = acc[i][f][v];
            }
    }
}

// Packs A(m, red, tap) into [chunk = red/16][tap][Mpad][16], zero padded, which is
// the order the kernel's filter slab has in LDS.
__global__ void __launch_bounds__(256)
pack_filter_kernel(const bf16_t *__restrict__ w, bf16_t *__restrict__ wp, int M, int RED, int T, int w_sm,
                   int w_sr, int tflip, int Mpad, size_t total)
{
    const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= total) return;
    const int j = (int)(e & 15);
    size_t q = e >> 4;
    const int m = (int)(q % Mpad);
    q /= Mpad;
    const int tap = (int)(q % T), chunk = (int)(q / T);
    const int red = chunk * 16 + j;
    bf16_t v = 0;
    if (m < M && red < RED) v = w[(size_t)m * w_sm + (size_t)red * w_sr + (tflip ? T - 1 - tap : tap)];
    wp[e] = v;
}

struct Plan {
    TileProblem p;
    int KT;
    dim3 grid;
};

// Tiling for one problem; false if the patch would not fit the LDS budget.
bool make_plan(const TileProblem &base, int R, int S, Plan *pl)
{
    TileProblem p = base;
    const int KT = p.Kout <= 64 ? 64 : 128;
    const int PIXT = KT == 128 ? 256 : 512;
    const long long NP = (long long)p.N * p.Pout;
    long long nrowtiles;
    int lrows_max;
    if (p.Qout <= 64) {
        p.TW = p.Qout;
        p.TH = PIXT / p.Qout;
        p.ncoltiles = 1;
        p.tiles_per_img = 0;
        if (p.TH > NP) p.TH = (int)NP;
        nrowtiles = (NP + p.TH - 1) / p.TH;
        // most patch rows a tile can need: TH rows, one halo, and one more halo per image boundary inside it
        const int crossings = p.N > 1 ? (p.TH - 1) / p.Pout + 1 : 0;
        lrows_max = p.TH + (crossings + 1) * (R - 1);
    } else {
        p.TW = 32;
        p.TH = PIXT / 32;
        p.ncoltiles = (p.Qout + 31) / 32;
        if (p.TH > p.Pout) p.TH = p.Pout;
        p.tiles_per_img = (p.Pout + p.TH - 1) / p.TH;
        nrowtiles = (long long)p.N * p.tiles_per_img;
        lrows_max = p.TH + R - 1;
    }
    p.LW = p.TW + S - 1;
    p.Hp = p.Pout + R - 1;
    if ((long long)lrows_max * p.LW > XPIX_MAX) return false;
    p.nchunks = (p.Cin + 15) / 16;
    p.Mpad = (p.Kout + 63) / 64 * 64;
    if (nrowtiles * p.ncoltiles > 0x7fffffffLL) return false;
    pl->p = p;
    pl->KT = KT;
    pl->grid = dim3((unsigned)(nrowtiles * p.ncoltiles), (p.Kout + KT - 1) / KT, 1);
    return true;
}

bool problem_of(const ConvGeom &g, bool bwd_data, TileProblem *p)
{
    if (!g.in_bf16 || g.sh != 1 || g.sw != 1) return false;
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
    return true;
}

template <int R, int S>
hipError_t launch_rs(const bf16_t *in, const bf16_t *w, void *out, const Plan &pl, bool staged, hipStream_t st)
{
    dim3 block(256);
    if (pl.KT == 128) {
        if (staged) hipLaunchKernelGGL((conv_tile_kernel<R, S, 128, true>), pl.grid, block, 0, st, in, w, out, pl.p);
        else hipLaunchKernelGGL((conv_tile_kernel<R, S, 128, false>), pl.grid, block, 0, st, in, w, out, pl.p);
    } else {
        if (staged) hipLaunchKernelGGL((conv_tile_kernel<R, S, 64, true>), pl.grid, block, 0, st, in, w, out, pl.p);
        else hipLaunchKernelGGL((conv_tile_kernel<R, S, 64, false>), pl.grid, block, 0, st, in, w, out, pl.p);
    }
    return hipGetLastError();
}

bool filter_supported(int R, int S)
{
    return (R == 1 && S == 1) || (R == 3 && S == 3) || (R == 5 && S == 5) || (R == 1 && S == 7) ||
           (R == 7 && S == 1);
}

}  // namespace

bool tile_conv_supported(const ConvGeom &g, bool bwd_data)
{
    TileProblem p;
    Plan pl;
    return filter_supported(g.R, g.S) && problem_of(g, bwd_data, &p) && make_plan(p, g.R, g.S, &pl);
}

size_t tile_conv_packed_bytes(const ConvGeom &g, bool bwd_data)
{
    TileProblem p;
    Plan pl;
    if (!filter_supported(g.R, g.S) || !problem_of(g, bwd_data, &p) || !make_plan(p, g.R, g.S, &pl)) return 0;
    return align_up((size_t)pl.p.nchunks * g.R * g.S * pl.p.Mpad * 16 * sizeof(bf16_t), 256);
}

hipError_t launch_tile_conv(const void *in, const void *w, void *out, const ConvGeom &g, bool bwd_data,
                            void *packed, hipStream_t st)
{
    TileProblem p;
    Plan pl;
    if (!filter_supported(g.R, g.S) || !problem_of(g, bwd_data, &p) || !make_plan(p, g.R, g.S, &pl))
        return hipErrorInvalidValue;
    const bf16_t *wsrc = static_cast<const bf16_t *>(w);
    if (packed) {
        const int T = g.R * g.S;
        const size_t total = (size_t)pl.p.nchunks * T * pl.p.Mpad * 16;
        hipLaunchKernelGGL(pack_filter_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, wsrc,
                           static_cast<bf16_t *>(packed), pl.p.Kout, pl.p.Cin, T, pl.p.w_sm, pl.p.w_sr,
                           pl.p.tflip, pl.p.Mpad, total);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        wsrc = static_cast<const bf16_t *>(packed);
    }
    const bf16_t *src = static_cast<const bf16_t *>(in);
    const bool staged = packed != nullptr;
    if (g.R == 1 && g.S == 1) return launch_rs<1, 1>(src, wsrc, out, pl, staged, st);
    if (g.R == 3 && g.S == 3) return launch_rs<3, 3>(src, wsrc, out, pl, staged, st);
    if (g.R == 5 && g.S == 5) return launch_rs<5, 5>(src, wsrc, out, pl, staged, st);
    if (g.R == 1 && g.S == 7) return launch_rs<1, 7>(src, wsrc, out, pl, staged, st);
    return launch_rs<7, 1>(src, wsrc, out, pl, staged, st);
}

}  // namespace sn
