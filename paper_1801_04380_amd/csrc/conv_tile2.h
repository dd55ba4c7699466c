#pragma once
// Second-generation stride-1 bf16 tile convolution for the STAGED algorithm
// (packed filter in the caller's workspace): CONV forward and backward-data
// (Sec. 3.5 of the paper; definitions in sn.h).  Same problem statement, tile
// geometry, packed filter layout and epilogue as conv_tile.h; what differs is how
// the operands reach the MFMAs.
//
//  * The filter operand never touches LDS.  In the packed layout the 16 bytes a
//    lane needs for one (tap, 32 output channels) tile are one aligned item and the
//    64 items of a wave are one contiguous 1 KB run, so each wave fetches its own
//    operands from L2 straight into registers, one stage (filter column) ahead
//    into one of two register sets (five stages ahead into one of six for the
//    smaller tiles, whose stages are short).
//  * The input patch of a 16-channel chunk travels global memory -> LDS without
//    passing through registers (global_load_lds): items of DW bytes (16, or 4 when
//    the image width is not a multiple of 8) land in a "parked" buffer laid out
//    [channel][patch row][column], i.e. as the image has them.  A thread fetches the
//    same item of the patch for every channel group, so its offset into the tensor
//    is a per-thread constant plus a uniform channel offset.  The loads are
//    range-checked buffer loads: rows and columns outside the image and channels
//    past the last are given an offset past the tensor, which brings zeros.  A transposing LDS read (ds_read_b64_tr_b16: within 16 lanes, lane i
//    receives element i%4 of the 8 bytes read by lanes i/4, 4+i/4, 8+i/4, 12+i/4)
//    turns 4 channels x 16 columns into 16 pixels x 4 channels, so two reads and
//    one 16-byte write per pixel build the [pixel][16 channels] layout the MFMAs
//    read (same swizzle as conv_tile.h).
//  * Parked buffers and patch buffers are double buffered over chunks: while chunk
//    c is multiplied, chunk c+1 is transposed and chunk c+2 is in flight.  One
//    barrier per chunk.
//  * WPN = 4 (at most 64 output channels): the four waves of the workgroup all take the 64
//    channels and a quarter of the tile's pixels each (NF 32-pixel groups per wave), instead
//    of two halves of 128 channels x two halves of the pixels.
//  * KS = 2 (small images, where the tiles do not even give every compute unit a
//    workgroup): a workgroup has two sets of four waves, each with buffers of its own,
//    which run the same pipeline over the even and the odd chunks of the same tile
//    and add their accumulators through LDS before the epilogue -- twice the waves
//    per compute unit to hide latencies behind, without a second pass over memory.
#include "conv_tile.h"

namespace sn {
namespace {

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

constexpr int V2_XTR_MAX_NARROW = 4;     // transposition rounds, NARROW tiling
constexpr int V2_CH_PAD = 32;            // bytes between the channels of a parked patch: spreads them over the banks
constexpr int V2_PK_SLACK = 64;          // bytes past a parked buffer that a transposing read may touch
constexpr int V2_TRASH = 64;             // 16-byte items at the end of a patch buffer that are written and never read

__device__ inline s16x4 lds_read_tr16(const char *p)
{
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)p);
}

// The body of the kernel; the four LDS regions are distinct, which the qualifiers tell the
// compiler (loads into a parked buffer then do not hold up the reads of a patch buffer).
template <int R, int S, int NF, bool WIDE, int DW, int KS, int WPN>
__device__ __forceinline__ void conv_tile2_body(const bf16_t *__restrict__ in, const bf16_t *__restrict__ w,
                                                void *__restrict__ out, const TileProblem &p,
                                                uint4 *__restrict__ xs0, uint4 *__restrict__ xs1,
                                                char *__restrict__ pk0, char *__restrict__ pk1, uint4 *smem)
{
    constexpr int KT = WPN == 2 ? 128 : 64;
    static_assert(WPN == 2 || (WPN == 4 && KS == 1), "wave layouts");
    constexpr int SG = sg_of(R, S), TRES = R * SG, NSUB = S / SG;
    constexpr int PIXT = WPN * NF * 32;
    constexpr int NB = WIDE ? NF + R - 1 : NF;
    constexpr int WROWS = PIXT / 32 + R - 1;   // WIDE: patch rows
    constexpr int XG = DW == 16 ? 4 : 16;   // most load rounds per chunk: 16 / (channels per round)
    constexpr int XTR = WIDE ? (2 * WROWS * (WIDE_LWP / 16) + 15) / 16 : V2_XTR_MAX_NARROW;

    // tid, wave: within the set of four waves; set s of KS takes the chunks s, s + KS, ...
    const int tid = threadIdx.x & 255, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int set = KS > 1 ? __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 8) : 0;
    const int nch = p.nchunks / KS;   // chunks per set (the host gives KS > 1 only chunk counts it divides)
    const int l32 = lane & 31, g = lane >> 5;
    const int wk = WPN == 2 ? wave >> 1 : 0, wp = WPN == 2 ? wave & 1 : wave;
    const int XS = p.xslots * 2 + V2_TRASH;

    // ---- which tile
    int ktile, ptile;
    if (!tile_of(p, &ktile, &ptile)) return;   // uniform for the workgroup, before any barrier
    // ---- tile geometry (as in conv_tile.h)
    const int rowtile = ptile / p.ncoltiles, coltile = ptile - rowtile * p.ncoltiles;
    const int k0 = ktile * KT;
    const int q0 = coltile * p.TW;
    const int LWp = WIDE ? WIDE_LWP : p.LWp;
    const int HWin = p.Hin * p.Win;
    int o0, NP, u0, lrows, img = 0;
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

    // ---- both patch buffers start as zeros: the padding slots are never written
    for (int i = tid; i < XS; i += 256) {
        xs0[i] = make_uint4(0, 0, 0, 0);
        xs1[i] = make_uint4(0, 0, 0, 0);
    }

    // ---- per-thread constants of the patch loads.  A parked channel has room for upc units
    // of DW bytes (upc = 64, 128 or 256, at least rows * units per row), so one round of 256
    // loads brings 256 / upc channels: thread tid takes unit tid % upc of channel
    // rd * (256 / upc) + tid / upc.  A wave's 64 loads go to 64 * DW consecutive bytes of LDS,
    // which is what the load instruction does by itself.
    const int pitch = p.xt_cols, upr = pitch * 2 / DW;   // parked row in elements, units per row
    const int upc = p.xt_upc, gch = 256 / upc;           // units per parked channel, channels per round
    const int chstride = upc * DW + V2_CH_PAD;           // bytes from a parked channel to the next
    // An offset that is past the tensor with or without the uniform channel offset added (the
    // tensor has at most 2^31 bytes), whichever of the two the range check looks at.
    constexpr uint32_t OUTSIDE = 0x80000000u;
    const __amdgpu_buffer_rsrc_t in_rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(in), 0, p.in_bytes, 0x00020000);
    const int xg_sub = tid / upc;     // the thread's channel within a round
    // Shifted 16-byte loads (whole rows only): G image rows per parked row, groups aligned to even image rows.
    const int G = (!WIDE && DW == 16) ? p.xt_shift : 0;
    const int ubase = G > 1 ? u0 - ((u0 - p.padh) & (G - 1)) : u0;   // first patch row of the first group
    const int nprk = G > 1 ? (u0 + lrows - 1 - ubase) / G + 1 : lrows;   // parked rows of this tile
    uint32_t xg_off = OUTSIDE;        // byte offset of the thread's unit in channel xg_sub of chunk 0
    {
        const int e = tid - xg_sub * upc;
        const int unit = e % upr, srow = e / upr;
        if (srow < nprk) {
            // (G > 1: u is the first row of the group, an even image row or a padding row: n and h are then those of
            // no image row, u < 0 included, and nothing is loaded)
            const int u = G > 1 ? ubase + G * srow : u0 + srow, n = WIDE ? img : u / p.Hp, h = u - n * p.Hp - p.padh;
            const int sh = G ? (xg_sub * HWin + h * p.Win) & 7 : 0;   // the row starts sh elements into its first unit
            const int col0 = (WIDE ? q0 - 8 : -sh) + unit * (DW / 2);
            if (n < p.N && (unsigned)h < (unsigned)p.Hin && col0 > -(DW / 2) && col0 < (G > 1 ? G : 1) * p.Win)
                xg_off = (uint32_t)(((n * p.Cin + xg_sub) * p.Hin + h) * p.Win + col0) * 2u;
        }
    }
    // LDS place of the wave's 64 loads in round 0, and the step from round to round
    const int wave_dst = ((wave * 64) / upc) * chstride + ((wave * 64) % upc) * DW;
    const int round_dst = gch * chstride;
    auto dma_issue = [&](int chunk, char *__restrict__ pk) {
        const int c0 = (chunk * KS + set) * 16;
        const bool full = c0 + 16 <= p.Cin;
#pragma unroll
        for (int rd = 0; rd < XG; ++rd) {
            if (DW == 4 && rd >= p.xg_rounds) break;   // 16-byte items: always 4 rounds
            const int cr = c0 + rd * gch;   // first channel of the round
            const bool ok = xg_off != OUTSIDE && (full || cr + xg_sub < p.Cin);
            const uint32_t off = ok ? xg_off : OUTSIDE;
            const uint32_t soff = (uint32_t)cr * (uint32_t)HWin * 2u;
            char *dst = pk + wave_dst + rd * round_dst;
            if constexpr (DW == 16)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(in_rs, (__attribute__((address_space(3))) void *)dst, 16, off, soff, 0, 0);
            else
                __builtin_amdgcn_raw_ptr_buffer_load_lds(in_rs, (__attribute__((address_space(3))) void *)dst, 4, off, soff, 0, 0);
        }
    };

    // ---- per-thread constants of the transposition.  A block of 16 lanes takes one unit
    // (8-channel half, patch row, 16 columns): lane j reads the 4 columns 4*(j%4).. of
    // channels j/4 and 4+j/4 of the half, and receives the 8 channels of column j.
    uint32_t xs_sd[XTR];   // byte offset of the lane's first read | 16-byte LDS index of its pixel << 16
    {
        const int blk = tid >> 4, j = tid & 15;
        const int ncg = G ? p.xt_ncg : (pitch + 15) >> 4;
        const uint32_t trash = (uint32_t)(p.xslots * 2 + lane);   // where a lane without a pixel writes
#pragma unroll
        for (int rd = 0; rd < XTR; ++rd) {
            const int unit = rd * 16 + blk;
            const int xo = unit & 1, t2 = unit >> 1, cg = t2 % ncg, prow = t2 / ncg;
            uint32_t src = 0, dst = trash;
            if (prow < lrows) {
                // where the patch row starts in its parked row, rounded down to the 8 bytes the transposing
                // read needs; cadj: the columns that rounding puts before the row
                int grow = prow, roff = 0, cadj = 0;
                if (G) {
                    const int u = u0 + prow, n = u / p.Hp, h = u - n * p.Hp - p.padh;
                    const int jr = (u - ubase) & (G - 1);   // row within its group
                    grow = (u - ubase) / G;
                    roff = (((j >> 2) * HWin + (h - jr) * p.Win) & 7) + jr * p.Win;
                    cadj = roff & 3;
                    roff -= cadj;
                }
                src = (uint32_t)((xo * 8 + (j >> 2)) * chstride + (grow * pitch + roff + cg * 16 + (j & 3) * 4) * 2);
                const int pcol = cg * 16 + j - cadj;
                // WIDE: the parked patch starts 8 columns left of the tile, the patch buffer padw columns left of it
                const int lcol = WIDE ? pcol - 8 + p.padw : pcol + p.padw;
                const bool ok = WIDE ? (lcol >= 0 && lcol < p.LW) : (pcol >= 0 && pcol < p.Win);
                if (ok) {
                    const int slot = prow * LWp + lcol;
                    dst = (uint32_t)(slot * 2 + (xo ^ swz(slot)));
                }
            }
            xs_sd[rd] = src | (dst << 16);
        }
    }
    const int chs4 = 4 * chstride;   // bytes between channel c and c + 4 of the parked patch
    // xb0 is the start of LDS: the indices count from there for either patch buffer
    auto x_transpose = [&](const char *__restrict__ pk, uint4 *__restrict__ xb) {
        constexpr int GRP = (NF >= 4) ? XTR : 2;   // rounds whose reads are in flight together
#pragma unroll
        for (int r0 = 0; r0 < XTR; r0 += GRP) {
            if (!WIDE && r0 >= p.xtr_rounds) break;
            s16x4 lo[GRP], hi[GRP];
#pragma unroll
            for (int i = 0; i < GRP; ++i) {
                if (r0 + i >= XTR) continue;
                const uint32_t src = xs_sd[r0 + i] & 0xffffu;
                lo[i] = lds_read_tr16(pk + src);
                hi[i] = lds_read_tr16(pk + src + chs4);
            }
#pragma unroll
            for (int i = 0; i < GRP; ++i) {
                if (r0 + i >= XTR) continue;
                u32x4 v;
                __builtin_memcpy(&v, &lo[i], 8);
                __builtin_memcpy(reinterpret_cast<char *>(&v) + 8, &hi[i], 8);
                reinterpret_cast<u32x4 *>(xb)[xs_sd[r0 + i] >> 16] = v;
            }
        }
    };

    // ---- filter operands: lane (l32, g) of wave row wk takes, for tap tl and channel tile i,
    // the 16-byte item ((stage * TRES + tl) * Mpad + k0 + wk*64 + i*32 + l32) * 2 + (g ^ swz(l32)).
    const int nstage = nch * NSUB;   // stages of this set; its stage t is stage t + (t / NSUB * (KS - 1) + set) * NSUB of the tile
    const __amdgpu_buffer_rsrc_t w_rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(w), 0, p.w_bytes, 0x00020000);
    const uint32_t wlane = (uint32_t)(((k0 + wk * 64 + l32) * 2 + (g ^ swz(l32))) * 16);
    const uint32_t wtap = (uint32_t)p.Mpad * 32u;   // bytes per tap
    // Register sets of filter operands: a stage's set is loaded AD - 1 stages ahead.  (Looking five
    // stages ahead on the small tiles, whose stages are short, measured 3-8 % slower than one: the 144
    // registers of six sets cost more than the latency they cover.)
    constexpr int AD = 2;
    static_assert((2 * NSUB) % AD == 0, "a trip of the main loop must use every set equally often");
    u32x4 areg[AD][TRES * 2];
    auto load_a = [&](int stage, u32x4(&dst)[TRES * 2]) {
        const int t = min(stage, nstage - 1);
        const uint32_t sbase = (uint32_t)(KS > 1 ? t + (t / NSUB * (KS - 1) + set) * NSUB : t) * (uint32_t)TRES * wtap;
#pragma unroll
        for (int tl = 0; tl < TRES; ++tl)
#pragma unroll
            for (int i = 0; i < 2; ++i)
                dst[tl * 2 + i] = __builtin_amdgcn_raw_buffer_load_b128(w_rs, wlane + i * 1024, sbase + tl * wtap, 0);
    };

    // ---- per-lane constants of the patch reads
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

    f32x16 acc[2][NF];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int f = 0; f < NF; ++f)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][f][v] = 0.f;

    // The MFMAs of one stage.  WIDE: the operand of output row i, tap row r is the operand of
    // output row i+1, tap row r-1, so a stage reads NF+R-1 patch rows; the first R-1 of them are
    // not needed by the last tap row, during which the next stage's first R-1 rows are fetched.
    bf16x8 bw[NB];
    auto compute = [&](const uint4 *__restrict__ xb, const u32x4(&a)[TRES * 2], auto sgc) {
        constexpr int sg = decltype(sgc)::value;
        static_assert(SG == 1 || !WIDE, "the row window is written for one filter column per stage");
#pragma unroll
        for (int sl = 0; sl < SG; ++sl) {
            const int s = sg * SG + sl;
            const int wslot = pixbase[0] + s;
            const uint4 *bp = xb + wslot * 2 + (g ^ swz(wslot));        // WIDE: this stage's rows
            const uint4 *bn = xb + (wslot + 1) * 2 + (g ^ swz(wslot + 1));   // and the next stage's
            if (WIDE) {
#pragma unroll
                for (int j = (sg == 0 ? 0 : R - 1); j < NB; ++j)
                    bw[j] = *reinterpret_cast<const bf16x8 *>(bp + j * WIDE_LWP * 2);
            }
#pragma unroll
            for (int r = 0; r < R; ++r) {
                bf16x8 b[NF];
                if (!WIDE) {
#pragma unroll
                    for (int f = 0; f < NF; ++f) {
                        const int slot = pixbase[f] + s;
                        b[f] = *reinterpret_cast<const bf16x8 *>(xb + (slot + r * LWp) * 2 + (g ^ swz(slot)));
                    }
                } else {
#pragma unroll
                    for (int f = 0; f < NF; ++f) b[f] = bw[f + r];
                    if (r == R - 1 && sg + 1 < NSUB) {
#pragma unroll
                        for (int j = 0; j < R - 1; ++j)
                            bw[j] = *reinterpret_cast<const bf16x8 *>(bn + j * WIDE_LWP * 2);
                        __builtin_amdgcn_sched_barrier(0);   // issued before the last tap row's MFMAs, not after
                    }
                }
#pragma unroll
                for (int f = 0; f < NF; ++f)
#pragma unroll
                    for (int i = 0; i < 2; ++i) {
                        bf16x8 av;
                        __builtin_memcpy(&av, &a[(r * SG + sl) * 2 + i], 16);
                        acc[i][f] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[f], av, acc[i][f], 0, 0, 0);
                    }
            }
        }
    };

    // ---- prologue: chunks 0 and 1 on their way, chunk 0 transposed
#pragma unroll
    for (int i = 0; i < AD - 1; ++i) load_a(i, areg[i]);
    dma_issue(0, pk0);
    dma_issue(min(1, nch - 1), pk1);
    __syncthreads();   // zero fill done, both parked patches have landed
    x_transpose(pk0, xs0);
    __syncthreads();

    // ---- main loop, two chunks per trip so that buffers and register sets are static; a
    // last odd chunk has nothing left to fetch for the patch
    auto stage = [&](auto cc, auto sgc, auto parc, auto tailc, int chunk) {
        constexpr int c = decltype(cc)::value, sg = decltype(sgc)::value, par = decltype(parc)::value;
        constexpr bool tail = decltype(tailc)::value;
        uint4 *__restrict__ const xcur = c ? xs1 : xs0;
        uint4 *__restrict__ const xnext = c ? xs0 : xs1;
        char *__restrict__ const pcur = c ? pk1 : pk0;     // free: chunk + 2 goes here
        char *__restrict__ const pnext = c ? pk0 : pk1;    // holds chunk + 1
        if (!WIDE) {
#pragma unroll
            for (int f = 0; f < (WIDE ? 1 : NF); ++f) asm volatile("" : "+v"(pixbase[f]));
        }
        load_a(chunk * NSUB + sg + AD - 1, areg[(par + AD - 1) % AD]);   // past the end: the last stage again
        if (!tail && sg == 0) dma_issue(min(chunk + 2, nch - 1), pcur);
        __builtin_amdgcn_sched_barrier(0);   // the loads are issued a whole stage before their use
        if (!tail && sg == NSUB - 1) x_transpose(pnext, xnext);
        compute(xcur, areg[par], sgc);
        if (!tail && sg == NSUB - 1) {
            // End of a chunk: the next patch buffer has been written, and the parked patch after it
            // (chunk + 2, whose loads every wave issued in the first stage of this chunk) has to have
            // landed for every wave before the barrier, because the next chunk's last stage transposes it
            // and there is no other barrier in between.  The loads issued after it -- the filter
            // operands of this chunk's later stages, KEEP of them -- stay in flight, which a fence would
            // not allow.
            constexpr int KEEP = (NSUB - 1) * TRES * 2;
            static_assert(KEEP < 64, "the counter has 6 bits");
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_waitcnt((KEEP & 15) | ((KEEP >> 4) << 14) | (7 << 4));   // vmcnt(KEEP) lgkmcnt(0)
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
        }
    };
    int chunk0 = 0;
    for (; chunk0 + 1 < nch; chunk0 += 2) {
        static_for<2 * NSUB>([&](auto idx) {
            constexpr int c = decltype(idx)::value / NSUB, sg = decltype(idx)::value % NSUB;
            stage(std::integral_constant<int, c>{}, std::integral_constant<int, sg>{},
                  std::integral_constant<int, decltype(idx)::value % AD>{}, std::false_type{}, chunk0 + c);
        });
    }
    if (nch & 1) {
        static_for<NSUB>([&](auto idx) {
            stage(std::integral_constant<int, 0>{}, idx, std::integral_constant<int, decltype(idx)::value % AD>{},
                  std::true_type{}, chunk0);
        });
    }

    // ---- epilogue (as in conv_tile.h): a lane holds, for output channel lane % 32 of a tile,
    // the pixels 8*(v/4) + 4*(lane/32) + v%4.
    const int PQ = p.Pout * p.Qout;
    auto pix_off = [&](int i) -> int {
        const int rl = i / p.TW, cl = i - rl * p.TW;
        const int o = o0 + rl;
        if (!(rl < p.TH && o < NP && q0 + cl < p.Qout)) return -1;
        const int n = o / p.Pout, pp = o - n * p.Pout;
        return (n * p.Kout * p.Pout + pp) * p.Qout + q0 + cl;
    };
    __builtin_amdgcn_s_waitcnt(0x0f70);   // vmcnt(0): no load into LDS is still on its way
    __syncthreads();
    if constexpr (KS > 1) {
        // the second set's sums reach the first through LDS, half of the accumulators at a time
        static_assert(KS == 2, "two sets");
        float *const red = reinterpret_cast<float *>(smem) + wave * NF * 16 * 64 + lane;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            if (set == 1) {
#pragma unroll
                for (int f = 0; f < NF; ++f)
#pragma unroll
                    for (int v = 0; v < 16; ++v) red[(f * 16 + v) * 64] = acc[i][f][v];
            }
            __syncthreads();
            if (set == 0) {
#pragma unroll
                for (int f = 0; f < NF; ++f)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[i][f][v] += red[(f * 16 + v) * 64];
            }
            __syncthreads();
        }
    }
    // The second set walks through the epilogue as well (it has the same barriers to meet) but
    // owns no output channel: its channel numbers are past the last.
    const int kst = set == 0 ? k0 : (1 << 29);
    if (p.stats)
        tile_bn_partials<NF, WPN>(acc, p.TW, min(p.TH, NP - o0), p.Qout - q0, wp, wk, l32, g, kst + wk * 64, p.Kout, p.out_bf16 != 0, p.stats, p.nptiles,
                                ptile, reinterpret_cast<float *>(smem) + set * 1024);
    if (p.out_bf16) {
        constexpr int EP = EPI_PITCH;
        char *const stage = reinterpret_cast<char *>(smem) + (set * 4 + wave) * 32 * EP;
        constexpr int OCT = NF * 4, KPR = 64 / OCT;
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
                const int kl = rd * KPR + krow, k = kst + wk * 64 + i * 32 + kl;
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
                        const int k = kst + wk * 64 + i * 32 + l32;
                        if (k < p.Kout) o32[(size_t)k * PQ + off] = acc[i][f][4 * j + e];
                    }
                }
    }
}

template <int R, int S, int NF, bool WIDE, int DW, int KS, int WPN>
__global__ void __launch_bounds__(256 * KS, 2)
conv_tile2_kernel(const bf16_t *__restrict__ in, const bf16_t *__restrict__ w, void *__restrict__ out, TileProblem p)
{
    extern __shared__ __attribute__((aligned(16))) uint4 smem[];
    const int XS = p.xslots * 2 + V2_TRASH;
    // each set of waves has its two patch buffers and two parked buffers
    const int set = KS > 1 ? __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 8) : 0;
    uint4 *const xs = smem + set * (2 * XS + 2 * (p.pk_bytes / 16));
    char *const pk = reinterpret_cast<char *>(xs + 2 * XS);
    conv_tile2_body<R, S, NF, WIDE, DW, KS, WPN>(in, w, out, p, xs, xs + XS, pk, pk + p.pk_bytes, smem);
}

template <int R, int S, int NF, bool WIDE, int DW, int KS = 1, int WPN = 2>
hipError_t launch2_one(const bf16_t *in, const bf16_t *w, void *out, const Plan &pl, hipStream_t st)
{
    auto kern = conv_tile2_kernel<R, S, NF, WIDE, DW, KS, WPN>;
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, LDS_LIMIT);
    if (attr != hipSuccess) return attr;
    hipLaunchKernelGGL(kern, pl.grid, dim3(256 * KS), pl.lds, st, in, w, out, pl.p);
    return hipGetLastError();
}

}  // namespace

// 3x3 filters, 128-channel tiles; `pl` made by make_plan2.
hipError_t launch_tile2_3x3(const bf16_t *in, const bf16_t *w, void *out, const Plan &pl, hipStream_t st);

}  // namespace sn
