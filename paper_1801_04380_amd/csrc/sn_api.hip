// Host side of the C ABI: argument checks, the workspace queries, the planner of
// Sec. 3.5 (fastest algorithm whose workspace fits the budget) and the dispatch
// of each call to the HIP kernels.  No device memory is allocated here; the one
// buffer the library owns is the fixed-size `scratch` array of sn_conv2d_fwd_noalloc.
#include <algorithm>
#include <cstring>
#include <mutex>
#include <vector>

#include "sn_internal.h"

using namespace sn;

namespace {

constexpr size_t WS_ALIGN = 256;

bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

bool valid_dtype(int d) { return d == SN_F32 || d == SN_BF16; }

// Shape check shared by every CONV entry point.  On success fills g.
sn_status make_geom(const sn_conv_shape *s, ConvGeom *g)
{
    if (!s) return SN_ERR_BAD_ARG;
    if (s->N < 1 || s->C < 1 || s->H < 1 || s->W < 1 || s->K < 1 || s->R < 1 || s->S < 1) return SN_ERR_BAD_ARG;
    if (s->stride_h < 1 || s->stride_w < 1 || s->pad_h < 0 || s->pad_w < 0) return SN_ERR_BAD_ARG;
    if (!valid_dtype(s->in_dtype) || !valid_dtype(s->out_dtype)) return SN_ERR_BAD_ARG;
    if (s->in_dtype == SN_F32 && s->out_dtype != SN_F32) return SN_ERR_BAD_ARG;
    const int P = sn_out_dim(s->H, s->pad_h, s->R, s->stride_h);
    const int Q = sn_out_dim(s->W, s->pad_w, s->S, s->stride_w);
    if (P < 1 || Q < 1) return SN_ERR_BAD_ARG;
    // index ranges the kernels rely on: every GEMM dimension and every plane fits in int32
    const long long lim = 0x7fffffffLL;
    const long long CRS = (long long)s->C * s->R * s->S, KRS = (long long)s->K * s->R * s->S;
    if ((long long)s->N * P * Q > lim || (long long)s->N * s->H * s->W > lim || CRS > lim || KRS > lim)
        return SN_ERR_UNSUPPORTED;
    if ((long long)s->C * s->H * s->W > lim || (long long)s->K * P * Q > lim || (long long)s->K * CRS > lim)
        return SN_ERR_UNSUPPORTED;
    if (s->pad_h >= 32768 || s->pad_w >= 32768 || s->R >= 32768 || s->S >= 32768) return SN_ERR_UNSUPPORTED;
    g->N = s->N; g->C = s->C; g->H = s->H; g->W = s->W; g->K = s->K; g->R = s->R; g->S = s->S;
    g->sh = s->stride_h; g->sw = s->stride_w; g->ph = s->pad_h; g->pw = s->pad_w;
    g->P = P; g->Q = Q;
    g->in_bf16 = s->in_dtype == SN_BF16;
    g->out_bf16 = s->out_dtype == SN_BF16;
    return SN_OK;
}

size_t in_elem(const ConvGeom &g) { return g.in_bf16 ? 2 : 4; }

// ---- workspace layouts ------------------------------------------------------
// IM2COL_GEMM, per image of a pass:
//   forward          col                         C*R*S*P*Q * in_elem
//   backward-filter  col, plus one block of fp32 partial dw slices per call
//   backward-data    dcol (fp32)                 C*R*S*P*Q * 4
struct Im2colPlan {
    size_t per_image;  // bytes per image of a pass (256-aligned)
    size_t fixed;      // bytes needed once per call (256-aligned)
    int splits;        // backward-filter slices per pass
};

ConvGeom gemm_geom_1x1(const ConvGeom &g, int nimg);

bool im2col_supported(const ConvGeom &g)
{
    // grid.y of the unfold kernel; and the GEMM over the unfolded tensor indexes one image of it
    // (C*R*S planes of P*Q) with 32-bit integers
    return (long long)g.C * g.R * g.S <= 65535 && (long long)g.C * g.R * g.S * g.P * g.Q <= 0x7fffffffLL;
}

Im2colPlan im2col_plan(const ConvGeom &g, sn_conv_dir dir)
{
    Im2colPlan p;
    const size_t cells = (size_t)g.C * g.R * g.S * g.P * g.Q;
    p.per_image = align_up(cells * (dir == SN_CONV_BWD_DATA ? 4 : in_elem(g)), WS_ALIGN);
    p.fixed = 0;
    p.splits = 1;
    if (dir == SN_CONV_BWD_FILTER) {
        // sized for a full-batch pass, the most slices any pass can want
        p.splits = generic_bwd_filter_splits(gemm_geom_1x1(g, g.N));
        p.fixed = align_up((size_t)p.splits * g.K * g.C * g.R * g.S * sizeof(float), WS_ALIGN);
    }
    return p;
}

// The GEMM of the explicit algorithm, seen as a 1x1 stride-1 convolution over
// the unfolded tensor [nimg][C*R*S][P][Q].
ConvGeom gemm_geom_1x1(const ConvGeom &g, int nimg)
{
    ConvGeom u = g;
    u.N = nimg;
    u.C = g.C * g.R * g.S;
    u.H = g.P; u.W = g.Q;
    u.R = u.S = 1;
    u.sh = u.sw = 1;
    u.ph = u.pw = 0;
    return u;
}

// STAGED backward-filter: fp32 partial dw per slice of the (n,p,q) sum.
size_t staged_bwd_filter_bytes(const ConvGeom &g, int *splits_out)
{
    int splits = smallc_supported(g) ? smallc_wgrad_slices(g)
               : tile_wgrad_supported(g) ? tile_wgrad_slices(g)
               : gather_wgrad_supported(g) ? gather_wgrad_slices(g) : generic_bwd_filter_splits(g);
    if (splits_out) *splits_out = splits;
    return align_up((size_t)splits * g.K * g.C * g.R * g.S * sizeof(float), WS_ALIGN);
}

// The row-stationary kernel also runs with fewer slices than fill the chip (fewer, longer workgroups): a
// quarter of them is the least STAGED backward-filter takes, so its workspace is a range (Sec. 3.5: more
// workspace, more speed).  Whether the shape has that range, and its least workspace.
bool staged_bwd_filter_ranged(const ConvGeom &g)
{
    return !smallc_supported(g) && tile_wgrad_supported(g) && tile_wgrad_cappable(g);
}

size_t staged_bwd_filter_min_bytes(const ConvGeom &g)
{
    const int full = tile_wgrad_slices(g), least = tile_wgrad_slices(g, (full + 3) / 4);
    return align_up((size_t)least * g.K * g.C * g.R * g.S * sizeof(float), WS_ALIGN);
}

// Slices the row-stationary kernel may use with ws_bytes of workspace (0: all it wants).
int staged_bwd_filter_cap(const ConvGeom &g, size_t ws_bytes)
{
    if (!staged_bwd_filter_ranged(g) || ws_bytes >= staged_bwd_filter_bytes(g, nullptr)) return 0;
    const size_t per = (size_t)g.K * g.C * g.R * g.S * sizeof(float);
    return (int)std::max<size_t>(1, ws_bytes / per);
}

// ---- STAGED on strided shapes: phase decomposition (conv_phase.hip) -----------------------------
// The strided convolution becomes a stride-1 convolution over the phase planes of the input: 1x1
// filters (no padding) keep a 1x1 filter over the one phase they touch; other filters whose taps
// all have plane offsets d, e in {-1, 0, 1} become a 3x3 "same" convolution on planes of the
// output's size.  Possible where the stride-1 MFMA kernels take the inner shape.
struct PhasePlan {
    PhaseMap m;
    ConvGeom inner;
    bool plain;          // one phase and a 1x1 filter: w and dw need no transform
    bool chunkable;      // every image of x, y, dy, dx starts on a 16-byte boundary: passes over parts of the batch
    size_t wprime_bytes, dwprime_bytes;   // 256-aligned parts of the workspace (0 if plain)
};

int floor_div(int a, int b) { return (a >= 0 ? a : a - b + 1) / b; }

// The taps of one axis as plane offsets d (r - pad = d * stride + a): which residues a occur, the range
// of d, and how many plane rows beyond the output's hold input that a tap with d > 0 reads (*extra:
// convolutions without padding; the rest of such rows lies outside the image and reads as zero).
// Supported: d within -1 .. 1, or within 0 .. 2.
bool phase_axis(int R, int stride, int pad, int in, int out, int *phases, int *index, int *count, int *dmin, int *dmax,
                int *extra)
{
    if (stride > 8) return false;
    for (int a = 0; a < 8; ++a) index[a] = -1;
    *count = 0;
    *dmin = 1 << 20;
    *dmax = -(1 << 20);
    int top[8] = {0, 0, 0, 0, 0, 0, 0, 0};   // largest d of each residue
    for (int r = 0; r < R; ++r) {
        const int u = r - pad, d = floor_div(u, stride), a = u - d * stride;
        if (index[a] < 0) index[a] = 0;
        *dmin = std::min(*dmin, d);
        *dmax = std::max(*dmax, d);
        top[a] = std::max(top[a], d);
    }
    for (int a = 0; a < stride; ++a)
        if (index[a] == 0) { index[a] = *count; phases[(*count)++] = a; }
    if (*dmin < -1 || *dmax > 2 || *dmax - *dmin > 2) return false;
    *extra = 0;
    for (int a = 0; a < stride; ++a)
        for (int d = 1; d <= top[a]; ++d)
            if ((out - 1 + d) * stride + a < in) *extra = std::max(*extra, d);
    return true;
}

bool phase_plan(const ConvGeom &g, sn_conv_dir dir, PhasePlan *pp)
{
    if (!g.in_bf16 || (g.sh == 1 && g.sw == 1)) return false;
    if (g.R > 16 || g.S > 16) return false;
    // padding at least as large as the filter (the first output row or column sees padding only: every tap has
    // a negative plane offset) is not built here; such shapes run the other kernels
    if (g.ph >= g.R || g.pw >= g.S) return false;
    PhaseMap &m = pp->m;
    m.sh = g.sh; m.sw = g.sw; m.ph = g.ph; m.pw = g.pw;
    int dmin, dmax, emin, emax, xr, xc;
    if (!phase_axis(g.R, g.sh, g.ph, g.H, g.P, m.row_phase, m.row_index, &m.na, &dmin, &dmax, &xr)) return false;
    if (!phase_axis(g.S, g.sw, g.pw, g.W, g.Q, m.col_phase, m.col_index, &m.nb, &emin, &emax, &xc)) return false;
    // planes larger than the output: the inner convolution is no longer a "same" one, which the
    // backward-filter kernels are built for
    if ((xr || xc || dmax > 1 || emax > 1) && dir == SN_CONV_BWD_FILTER) return false;
    // backward-filter of larger filters on small planes: the 3x3 inner filter multiplies four times the taps, on
    // planes the row-stationary kernel fills badly; the fallback kernel is faster there (measured 3x3 / stride 2,
    // 28 -> 14: 129 against 146 us, 14 -> 7: 152 against 218 us; level at 56 -> 28)
    if (dir == SN_CONV_BWD_FILTER && g.R * g.S > 1 && g.P * g.Q <= 196) return false;
    m.nphases = m.na * m.nb;
    const bool one_tap = dmin == 0 && dmax == 0 && emin == 0 && emax == 0;
    // Offsets that span two values on either axis (3x3 / stride 2: -1 .. 0 with padding 1, 0 .. 1 without) fit a
    // 2x2 inner filter, 16 tap slots per input channel for the 9 real taps instead of 36; forward and
    // backward-data only (the backward-filter kernels are built for 3x3 "same" shapes).
    // Backward-data gains everywhere (measured 12-35 % on the ResNet- and Inception-shaped stage entries); forward
    // where the 3x3 form cannot have the packed-filter kernel anyway (planes of odd width) or has no padding
    // (measured: 384 channels 35 -> 17: 276 against 335 us; 512 channels 14 -> 7: 283 against 339 us; but
    // 256 channels 28 -> 14 with padding: 166 against 132 us, where the 3x3 form runs the faster kernel).
    const bool span2 = !one_tap && dmax - dmin <= 1 && emax - emin <= 1;
    const bool two = span2 && (dir == SN_CONV_BWD_DATA ||
                               (dir == SN_CONV_FWD && ((dmin == 0 && emin == 0) || (g.Q + xc) % 2 != 0)));
    m.Ri = m.Si = one_tap ? 1 : two ? 2 : 3;
    // offsets -1 .. 1: "same" padding; 0 .. 2: no padding (an axis with the one offset 0 goes either way);
    // two values: the first tap is the lower offset, which is -1 (a row / column of padding before the plane) or 0
    m.center_r = one_tap ? 0 : two ? -dmin : (dmax > 1 ? 0 : 1);
    m.center_c = one_tap ? 0 : two ? -emin : (emax > 1 ? 0 : 1);
    if (!two && ((dmax > 1 && dmin < 0) || (emax > 1 && emin < 0))) return false;
    m.Hs = g.P + xr;
    m.Ws = g.Q + xc;
    if ((long long)g.C * m.nphases > 0x7fffffffLL / 16) return false;
    ConvGeom &u = pp->inner;
    u = g;
    u.C = g.C * m.nphases;
    u.H = m.Hs; u.W = m.Ws;
    u.R = m.Ri; u.S = m.Si;
    u.sh = u.sw = 1;
    u.ph = m.center_r;
    u.pw = m.center_c;
    pp->plain = m.nphases == 1 && g.R == 1 && g.S == 1;
    pp->chunkable = ((long long)g.K * g.P * g.Q) % 8 == 0 && ((long long)g.C * g.H * g.W) % 8 == 0;
    if (dir == SN_CONV_BWD_FILTER ? !tile_wgrad_supported(u) : !tile_conv_supported(u, dir == SN_CONV_BWD_DATA)) return false;
    pp->wprime_bytes = pp->plain ? 0 : align_up((size_t)g.K * u.C * u.R * u.S * 2, WS_ALIGN);
    pp->dwprime_bytes = pp->plain ? 0 : align_up((size_t)g.K * u.C * u.R * u.S * 4, WS_ALIGN);
    return true;
}

// Workspace of the phase path.  Forward and backward-data: transformed filter | packed filter of the
// inner convolution | the phase planes of as many images as a pass takes (`nimg`; the passes reuse
// the same planes), so the path runs from one image's planes up.  Backward-filter: the planes of the
// whole batch | dw of the inner convolution | its partial sums.
size_t phase_fixed_bytes(const PhasePlan &pp, sn_conv_dir dir)
{
    return pp.wprime_bytes + tile_conv_packed_bytes(pp.inner, dir == SN_CONV_BWD_DATA);
}

size_t phase_plane_bytes(const PhasePlan &pp, sn_conv_dir dir, int nimg)
{
    const size_t planes = (size_t)nimg * pp.inner.C * pp.inner.H * pp.inner.W;
    return align_up(planes * (dir == SN_CONV_BWD_DATA && !pp.inner.out_bf16 ? 4 : 2), WS_ALIGN);
}

size_t phase_bytes(const PhasePlan &pp, sn_conv_dir dir, int nimg)
{
    if (dir == SN_CONV_BWD_FILTER)
        return phase_plane_bytes(pp, dir, pp.inner.N) + pp.dwprime_bytes + staged_bwd_filter_bytes(pp.inner, nullptr);
    return phase_fixed_bytes(pp, dir) + phase_plane_bytes(pp, dir, nimg);
}

// Images per pass of the phase path under this budget (forward, backward-data; at least 1: the
// caller has checked the least workspace; the whole batch where the images do not start on
// 16-byte boundaries, which the kernels' wide accesses assume of their tensors).
int phase_chunk(const PhasePlan &pp, sn_conv_dir dir, size_t ws_bytes)
{
    if (!pp.chunkable) return pp.inner.N;
    int lo = 1, hi = pp.inner.N;
    while (lo < hi) {
        const int mid = (lo + hi + 1) / 2;
        if (phase_bytes(pp, dir, mid) <= ws_bytes) lo = mid;
        else hi = mid - 1;
    }
    return lo;
}

// STAGED forward by the pixel-gathering matrix product (conv_pointwise.hip), whose only workspace is the filter
// with the channel innermost: strided shapes, and stride-1 shapes the tile kernels do not take.
bool gather_fwd(const ConvGeom &g)
{
    return gather_conv_supported(g) && (g.sh > 1 || g.sw > 1 || !tile_conv_supported(g, false));
}

// 1x1 / stride-2 backward-data on planes of even size: the 1x1 kernel writes every result with the zeros of its
// 2 x 2 cell (no workspace, under either name).
bool scatter_bwd_data(const ConvGeom &g) { return (g.sh > 1 || g.sw > 1) && pointwise_supported(g, true); }

// Where the phase planes of the whole batch fit, 1x1 strided layers with many output channels are faster
// on them (one pass to take every other pixel, then pixel pairs per load and no re-gathering per channel
// tile; measured 256 -> 512 on 56x56: 54 against 66 us, 1024 -> 2048 on 14x14: 63 against 90 us); everything
// else, and every budget below that, takes the gathering kernel.
bool phase_fwd_when_it_fits(const ConvGeom &g) { return g.R == 1 && g.S == 1 && g.K >= 512; }

sn_status query(const ConvGeom &g, sn_conv_dir dir, sn_conv_algo algo, size_t *min_b, size_t *pref_b)
{
    switch (algo) {
    case SN_ALGO_DIRECT:
        *min_b = *pref_b = 0;
        return SN_OK;
    case SN_ALGO_IM2COL_GEMM: {
        if (!im2col_supported(g)) return SN_ERR_UNSUPPORTED;
        Im2colPlan p = im2col_plan(g, dir);
        *min_b = p.fixed + p.per_image;
        *pref_b = p.fixed + p.per_image * (size_t)g.N;
        return SN_OK;
    }
    case SN_ALGO_WINOGRAD:
        if (dir == SN_CONV_BWD_FILTER || !winograd_supported(g, dir == SN_CONV_BWD_DATA)) return SN_ERR_UNSUPPORTED;
        winograd_bytes(g, dir == SN_CONV_BWD_DATA, min_b, pref_b);
        return SN_OK;
    case SN_ALGO_STAGED: {
        PhasePlan pp;
        if (dir == SN_CONV_BWD_FILTER && smallc_supported(g)) {
            *min_b = *pref_b = staged_bwd_filter_bytes(g, nullptr);
            return SN_OK;
        }
        if (dir == SN_CONV_BWD_DATA && scatter_bwd_data(g)) {
            *min_b = *pref_b = 0;
            return SN_OK;
        }
        if (dir == SN_CONV_FWD && gather_fwd(g)) {
            *min_b = *pref_b = gather_conv_packed_bytes(g);
            if (phase_fwd_when_it_fits(g) && phase_plan(g, dir, &pp)) {
                *pref_b = phase_bytes(pp, dir, g.N);
                *min_b = std::min(*min_b, pp.chunkable ? phase_bytes(pp, dir, 1) : *pref_b);
            }
            return SN_OK;
        }
        if (phase_plan(g, dir, &pp)) {
            *pref_b = phase_bytes(pp, dir, g.N);
            *min_b = pp.chunkable ? phase_bytes(pp, dir, 1) : *pref_b;
            return SN_OK;
        }
        if (dir == SN_CONV_BWD_FILTER) {
            *min_b = *pref_b = staged_bwd_filter_bytes(g, nullptr);
            if (staged_bwd_filter_ranged(g)) *min_b = staged_bwd_filter_min_bytes(g);
            return SN_OK;
        }
        if (!tile_conv_supported(g, dir == SN_CONV_BWD_DATA)) return SN_ERR_UNSUPPORTED;
        *min_b = *pref_b = tile_conv_packed_bytes(g, dir == SN_CONV_BWD_DATA);
        return SN_OK;
    }
    default:
        return SN_ERR_BAD_ARG;
    }
}

// ---- planner table ------------------------------------------------------------
struct Record {
    sn_conv_shape shape;
    int dir, algo;
    size_t ws;
    float ms;
};
std::mutex g_mu;
std::vector<Record> g_table;

bool same_shape(const sn_conv_shape &a, const sn_conv_shape &b) { return std::memcmp(&a, &b, sizeof(a)) == 0; }

// Built-in ranking used when nothing has been measured for the shape: lower is
// tried first.  The workspace-staged implicit GEMM, then the direct one; the
// explicit unfold pays a write and a read of a buffer R*S times the input, so it
// is picked on measurement only.
const sn_conv_algo kRanking[] = {SN_ALGO_WINOGRAD, SN_ALGO_STAGED, SN_ALGO_DIRECT};

sn_status plan(const sn_conv_shape *shape, const ConvGeom &g, sn_conv_dir dir, size_t budget,
               sn_conv_algo *algo, size_t *bytes, float *ms_out)
{
    // The fastest record that fits; a record with a larger workspace displaces one with a smaller
    // only if it is faster by more than the margin (measurements of a few launches differ by a few
    // per cent from run to run, and workspace is what the runtime is short of).
    constexpr float MARGIN = 0.03f;
    bool found = false;
    Record best = {};
    {
        std::lock_guard<std::mutex> lk(g_mu);
        float fastest = 0.f;
        for (const Record &r : g_table) {
            if (r.dir != (int)dir || !same_shape(r.shape, *shape) || r.ws > budget) continue;
            if (!found || r.ms < fastest) fastest = r.ms;
            found = true;
        }
        bool have = false;
        for (const Record &r : g_table) {
            if (r.dir != (int)dir || !same_shape(r.shape, *shape) || r.ws > budget) continue;
            if (r.ms > fastest * (1.f + MARGIN)) continue;
            if (!have || r.ws < best.ws || (r.ws == best.ws && r.ms < best.ms)) {
                best = r;
                have = true;
            }
        }
    }
    if (found) {
        *algo = (sn_conv_algo)best.algo;
        *bytes = best.ws;
        if (ms_out) *ms_out = best.ms;
        return SN_OK;
    }
    // Few input channels: the zero-workspace kernel is the memory-bound one (forward); backward-filter
    // runs it under either name, STAGED with a fixed summation order.
    if (dir == SN_CONV_FWD && smallc_supported(g)) {
        *algo = SN_ALGO_DIRECT;
        *bytes = 0;
        if (ms_out) *ms_out = -1.f;
        return SN_OK;
    }
    for (sn_conv_algo a : kRanking) {
        size_t mn = 0, pf = 0;
        if (query(g, dir, a, &mn, &pf) != SN_OK || mn > budget) continue;
        if (a == SN_ALGO_STAGED && pf == 0) continue;   // nothing to stage: the same kernel runs as DIRECT
        // Winograd pays four kernels per pass and streams 16 transformed values per 4 inputs: a guess in its
        // favour only where a pass has real work and the products outweigh the transforms (measured: 64 x 128
        // channels gain, 64 x 64 lose)
        if (a == SN_ALGO_WINOGRAD && ((pf > budget && winograd_pass_tiles(g, dir == SN_CONV_BWD_DATA, budget) < 2048) ||
                                      (long long)g.C * g.K < 8192)) continue;
        // The phase planes in passes: strided forward gains little over the zero-workspace kernel, so only
        // with the whole batch (below that STAGED forward is the gathering kernel, which needs the re-laid-out
        // filter alone); backward-data gains a quarter over the zero-workspace kernel, which works by residue
        // classes of the input pixels, and more than two passes' launches eat that up.
        if (a == SN_ALGO_STAGED && pf > budget && (g.sh > 1 || g.sw > 1) && dir != SN_CONV_BWD_FILTER) {
            PhasePlan pp;
            if (dir == SN_CONV_FWD) {
                if (!(gather_fwd(g) && budget >= gather_conv_packed_bytes(g))) continue;
            } else {
                if (!phase_plan(g, dir, &pp)) continue;
                const int chunk = phase_chunk(pp, dir, budget);
                if ((g.N + chunk - 1) / chunk > 2) continue;
            }
        }
        // backward-filter with fewer partial sums than it wants: a guess in its favour down to half of them
        // (below that the zero-workspace form's atomics are the better guess)
        if (a == SN_ALGO_STAGED && dir == SN_CONV_BWD_FILTER && pf > budget && budget < mn + (pf - mn) / 3) continue;
        *algo = a;
        *bytes = std::min(pf, budget);
        if (ms_out) *ms_out = -1.f;
        return SN_OK;
    }
    return SN_ERR_UNSUPPORTED;  // unreachable: DIRECT needs 0 bytes
}

sn_status check_ws(const void *ws, size_t bytes)
{
    if (bytes > 0 && !ws) return SN_ERR_BAD_ARG;
    if (ws && !aligned(ws, WS_ALIGN)) return SN_ERR_BAD_ARG;
    return SN_OK;
}

sn_status launch_status(hipError_t e) { return e == hipSuccess ? SN_OK : SN_ERR_LAUNCH; }

// Resolve AUTO and check the budget for a named algorithm.
sn_status resolve(const sn_conv_shape *shape, const ConvGeom &g, sn_conv_dir dir, sn_conv_algo *algo,
                  size_t ws_bytes)
{
    if (*algo == SN_ALGO_AUTO) {
        size_t used;
        return plan(shape, g, dir, ws_bytes, algo, &used, nullptr);
    }
    size_t mn = 0, pf = 0;
    sn_status s = query(g, dir, *algo, &mn, &pf);
    if (s != SN_OK) return s;
    if (mn > ws_bytes) return SN_ERR_WORKSPACE_TOO_SMALL;
    return SN_OK;
}

// Images per pass of the explicit algorithm under this budget.
int im2col_chunk(const ConvGeom &g, const Im2colPlan &p, size_t ws_bytes)
{
    size_t fit = (ws_bytes - p.fixed) / p.per_image;
    fit = std::min<size_t>(fit, 65535);   // grid.z of the unfold and fold kernels
    return (int)std::min<size_t>(fit, (size_t)g.N);
}

size_t out_elem(const ConvGeom &g) { return g.out_bf16 ? 2 : 4; }

// Zero-workspace implicit GEMM: the stride-1 bf16 tile kernel where it applies,
// the general kernel otherwise.
hipError_t direct_fwd(const void *x, const void *w, void *y, const ConvGeom &g, hipStream_t st)
{
    if (smallc_supported(g)) return launch_smallc_fwd(x, w, y, g, st, nullptr);
    if (tile_conv_supported(g, false)) return launch_tile_conv(x, w, y, g, false, nullptr, st);
    if (g.R == 1 && g.S == 1 && gather_fwd(g)) return launch_gather_conv_fwd(x, w, y, g, nullptr, st);
    return launch_generic_fwd(x, w, y, g, st);
}

hipError_t direct_bwd_data(const void *dy, const void *w, void *dx, const ConvGeom &g, hipStream_t st)
{
    if (scatter_bwd_data(g)) return launch_pointwise(dy, w, dx, g, true, st);
    if (tile_conv_supported(g, true)) return launch_tile_conv(dy, w, dx, g, true, nullptr, st);
    return launch_generic_bwd_data(dy, w, dx, g, st);
}

sn_status run_fwd(const void *x, const void *w, void *y, const ConvGeom &g, sn_conv_algo algo, void *ws,
                  size_t ws_bytes, hipStream_t st)
{
    if (algo == SN_ALGO_DIRECT) return launch_status(direct_fwd(x, w, y, g, st));
    if (algo == SN_ALGO_WINOGRAD) return launch_status(launch_winograd(x, w, y, g, false, ws, ws_bytes, st));
    PhasePlan pp;
    if (algo == SN_ALGO_STAGED && gather_fwd(g)) {
        const bool planes = phase_fwd_when_it_fits(g) && phase_plan(g, SN_CONV_FWD, &pp);
        const bool whole = planes && ws_bytes >= phase_bytes(pp, SN_CONV_FWD, g.N);
        if (!whole && ws_bytes >= gather_conv_packed_bytes(g)) return launch_status(launch_gather_conv_fwd(x, w, y, g, ws, st));
    }
    if (algo == SN_ALGO_STAGED && phase_plan(g, SN_CONV_FWD, &pp)) {
        char *base = static_cast<char *>(ws);
        void *wp = base, *packed = base + pp.wprime_bytes, *xs = base + phase_fixed_bytes(pp, SN_CONV_FWD);
        if (!pp.plain && launch_phase_filter(w, wp, pp.m, g, st) != hipSuccess) return SN_ERR_LAUNCH;
        const int chunk = phase_chunk(pp, SN_CONV_FWD, ws_bytes);
        for (int n0 = 0; n0 < g.N; n0 += chunk) {
            ConvGeom go = g, gi = pp.inner;
            go.N = gi.N = std::min(chunk, g.N - n0);
            const char *xo = static_cast<const char *>(x) + (size_t)n0 * g.C * g.H * g.W * in_elem(g);
            char *yo = static_cast<char *>(y) + (size_t)n0 * g.K * g.P * g.Q * out_elem(g);
            if (launch_phase_split(xo, xs, pp.m, go, st) != hipSuccess) return SN_ERR_LAUNCH;
            if (launch_tile_conv(xs, pp.plain ? w : wp, yo, gi, false, packed, st) != hipSuccess) return SN_ERR_LAUNCH;
        }
        return SN_OK;
    }
    if (algo == SN_ALGO_STAGED) return launch_status(launch_tile_conv(x, w, y, g, false, ws, st));
    if (algo == SN_ALGO_IM2COL_GEMM) {
        const Im2colPlan p = im2col_plan(g, SN_CONV_FWD);
        const int chunk = im2col_chunk(g, p, ws_bytes);
        for (int n0 = 0; n0 < g.N; n0 += chunk) {
            const int nimg = std::min(chunk, g.N - n0);
            hipError_t e = launch_im2col(x, ws, g, n0, nimg, st);
            if (e != hipSuccess) return SN_ERR_LAUNCH;
            char *yo = static_cast<char *>(y) + (size_t)n0 * g.K * g.P * g.Q * out_elem(g);
            e = direct_fwd(ws, w, yo, gemm_geom_1x1(g, nimg), st);
            if (e != hipSuccess) return SN_ERR_LAUNCH;
        }
        return SN_OK;
    }
    return SN_ERR_UNSUPPORTED;
}

sn_status run_bwd_data(const void *dy, const void *w, void *dx, const ConvGeom &g, sn_conv_algo algo, void *ws,
                       size_t ws_bytes, hipStream_t st)
{
    if (algo == SN_ALGO_DIRECT) return launch_status(direct_bwd_data(dy, w, dx, g, st));
    if (algo == SN_ALGO_WINOGRAD) return launch_status(launch_winograd(dy, w, dx, g, true, ws, ws_bytes, st));
    if (algo == SN_ALGO_STAGED && scatter_bwd_data(g)) return launch_status(launch_pointwise(dy, w, dx, g, true, st));
    PhasePlan pp;
    if (algo == SN_ALGO_STAGED && phase_plan(g, SN_CONV_BWD_DATA, &pp)) {
        char *base = static_cast<char *>(ws);
        void *wp = base, *packed = base + pp.wprime_bytes, *dxs = base + phase_fixed_bytes(pp, SN_CONV_BWD_DATA);
        if (!pp.plain && launch_phase_filter(w, wp, pp.m, g, st) != hipSuccess) return SN_ERR_LAUNCH;
        const int chunk = phase_chunk(pp, SN_CONV_BWD_DATA, ws_bytes);
        for (int n0 = 0; n0 < g.N; n0 += chunk) {
            ConvGeom go = g, gi = pp.inner;
            go.N = gi.N = std::min(chunk, g.N - n0);
            const char *dyo = static_cast<const char *>(dy) + (size_t)n0 * g.K * g.P * g.Q * in_elem(g);
            char *dxo = static_cast<char *>(dx) + (size_t)n0 * g.C * g.H * g.W * out_elem(g);
            if (launch_tile_conv(dyo, pp.plain ? w : wp, dxs, gi, true, packed, st) != hipSuccess) return SN_ERR_LAUNCH;
            if (launch_phase_merge(dxs, dxo, pp.m, go, st) != hipSuccess) return SN_ERR_LAUNCH;
        }
        return SN_OK;
    }
    if (algo == SN_ALGO_STAGED) return launch_status(launch_tile_conv(dy, w, dx, g, true, ws, st));
    if (algo == SN_ALGO_IM2COL_GEMM) {
        const Im2colPlan p = im2col_plan(g, SN_CONV_BWD_DATA);
        const int chunk = im2col_chunk(g, p, ws_bytes);
        for (int n0 = 0; n0 < g.N; n0 += chunk) {
            const int nimg = std::min(chunk, g.N - n0);
            ConvGeom u = gemm_geom_1x1(g, nimg);
            u.out_bf16 = 0;  // the column gradient stays fp32 until it is folded
            const char *dyo = static_cast<const char *>(dy) + (size_t)n0 * g.K * g.P * g.Q * in_elem(g);
            hipError_t e = direct_bwd_data(dyo, w, ws, u, st);
            if (e != hipSuccess) return SN_ERR_LAUNCH;
            e = launch_col2im(static_cast<const float *>(ws), dx, g, n0, nimg, st);
            if (e != hipSuccess) return SN_ERR_LAUNCH;
        }
        return SN_OK;
    }
    return SN_ERR_UNSUPPORTED;
}

sn_status run_bwd_filter(const void *x, const void *dy, void *dw, const ConvGeom &g, sn_conv_algo algo,
                         void *ws, size_t ws_bytes, hipStream_t st)
{
    float *dwf = static_cast<float *>(dw);
    const bool tile = tile_wgrad_supported(g);
    if (smallc_supported(g) && (algo == SN_ALGO_DIRECT || algo == SN_ALGO_STAGED))
        return launch_status(launch_smallc_wgrad(x, dy, dwf, g, algo == SN_ALGO_STAGED ? static_cast<float *>(ws) : nullptr, st));
    if (algo == SN_ALGO_DIRECT) {
        if (tile) return launch_status(launch_tile_wgrad(x, dy, dwf, g, nullptr, st));
        if (gather_wgrad_supported(g)) return launch_status(launch_gather_wgrad(x, dy, dwf, g, nullptr, st));
        return launch_status(launch_generic_bwd_filter(x, dy, dwf, g, generic_bwd_filter_splits(g), nullptr, false, st));
    }
    PhasePlan pp;
    if (algo == SN_ALGO_STAGED && phase_plan(g, SN_CONV_BWD_FILTER, &pp)) {
        // workspace: phase planes of x | dw of the inner convolution | its partial sums
        char *base = static_cast<char *>(ws);
        void *xs = base;
        char *dwp = base + align_up((size_t)pp.inner.N * pp.inner.C * pp.inner.H * pp.inner.W * 2, WS_ALIGN);
        float *partial = reinterpret_cast<float *>(dwp + pp.dwprime_bytes);
        if (launch_phase_split(x, xs, pp.m, g, st) != hipSuccess) return SN_ERR_LAUNCH;
        float *inner_dw = pp.plain ? dwf : reinterpret_cast<float *>(dwp);
        if (launch_tile_wgrad(xs, dy, inner_dw, pp.inner, partial, st) != hipSuccess) return SN_ERR_LAUNCH;
        if (pp.plain) return SN_OK;
        return launch_status(launch_phase_dw(inner_dw, dwf, pp.m, g, st));
    }
    if (algo == SN_ALGO_STAGED) {
        if (tile) return launch_status(launch_tile_wgrad(x, dy, dwf, g, static_cast<float *>(ws), st, staged_bwd_filter_cap(g, ws_bytes)));
        if (gather_wgrad_supported(g)) return launch_status(launch_gather_wgrad(x, dy, dwf, g, static_cast<float *>(ws), st));
        int splits;
        staged_bwd_filter_bytes(g, &splits);
        return launch_status(launch_generic_bwd_filter(x, dy, dwf, g, splits, static_cast<float *>(ws), false, st));
    }
    if (algo == SN_ALGO_IM2COL_GEMM) {
        const Im2colPlan p = im2col_plan(g, SN_CONV_BWD_FILTER);
        const int chunk = im2col_chunk(g, p, ws_bytes);
        float *partial = static_cast<float *>(ws);
        char *col = static_cast<char *>(ws) + p.fixed;
        // each pass reduces its slices in fixed order; passes after the first add to dw
        for (int n0 = 0, pass = 0; n0 < g.N; n0 += chunk, ++pass) {
            const int nimg = std::min(chunk, g.N - n0);
            hipError_t e = launch_im2col(x, col, g, n0, nimg, st);
            if (e != hipSuccess) return SN_ERR_LAUNCH;
            const ConvGeom u = gemm_geom_1x1(g, nimg);
            const char *dyo = static_cast<const char *>(dy) + (size_t)n0 * g.K * g.P * g.Q * in_elem(g);
            int splits = std::min(p.splits, generic_bwd_filter_splits(u));
            e = launch_generic_bwd_filter(col, dyo, dwf, u, splits, partial, pass > 0, st);
            if (e != hipSuccess) return SN_ERR_LAUNCH;
        }
        return SN_OK;
    }
    return SN_ERR_UNSUPPORTED;
}

}  // namespace

// ---- the library's own workspace, for sn_conv2d_fwd_noalloc -----------------------------------
// One array per GPU, resident from the moment the library's code is loaded on that GPU until the
// process ends.  In host code `scratch` is only a handle for hipGetSymbolAddress: the array's
// device address differs per GPU and is looked up once per device.
static __device__ __align__(256) unsigned char scratch[SN_NOALLOC_SCRATCH_BYTES];

namespace {

constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[MAX_DEVICES];   // device address of `scratch` on GPU i, nullptr until first use

sn_status scratch_of_current_device(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return SN_ERR_LAUNCH;
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return SN_ERR_LAUNCH;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return SN_OK;
}

}  // namespace

extern "C" {

int sn_version(void) { return 1; }

int sn_out_dim(int in, int pad, int window, int stride)
{
    if (in < 1 || pad < 0 || window < 1 || stride < 1) return 0;
    const long long span = (long long)in + 2LL * pad - window;
    if (span < 0) return 0;
    return (int)(span / stride) + 1;
}

sn_status sn_conv_workspace_query(const sn_conv_shape *shape, sn_conv_dir dir, sn_conv_algo algo,
                                  size_t *min_bytes, size_t *preferred_bytes)
{
    ConvGeom g;
    sn_status s = make_geom(shape, &g);
    if (s != SN_OK) return s;
    if (!min_bytes || !preferred_bytes || dir < SN_CONV_FWD || dir > SN_CONV_BWD_FILTER) return SN_ERR_BAD_ARG;
    return query(g, dir, algo, min_bytes, preferred_bytes);
}

sn_status sn_conv_plan(const sn_conv_shape *shape, sn_conv_dir dir, size_t budget_bytes, sn_conv_algo *algo,
                       size_t *bytes_used, float *predicted_ms)
{
    ConvGeom g;
    sn_status s = make_geom(shape, &g);
    if (s != SN_OK) return s;
    if (!algo || !bytes_used || dir < SN_CONV_FWD || dir > SN_CONV_BWD_FILTER) return SN_ERR_BAD_ARG;
    return plan(shape, g, dir, budget_bytes, algo, bytes_used, predicted_ms);
}

sn_status sn_planner_record(const sn_conv_shape *shape, sn_conv_dir dir, sn_conv_algo algo,
                            size_t workspace_bytes, float ms)
{
    ConvGeom g;
    sn_status s = make_geom(shape, &g);
    if (s != SN_OK) return s;
    if (dir < SN_CONV_FWD || dir > SN_CONV_BWD_FILTER || !(ms >= 0.f)) return SN_ERR_BAD_ARG;
    size_t mn = 0, pf = 0;
    s = query(g, dir, algo, &mn, &pf);
    if (s != SN_OK) return s;
    if (workspace_bytes < mn) return SN_ERR_WORKSPACE_TOO_SMALL;
    std::lock_guard<std::mutex> lk(g_mu);
    for (Record &r : g_table)
        if (r.dir == (int)dir && r.algo == (int)algo && r.ws == workspace_bytes && same_shape(r.shape, *shape)) {
            r.ms = ms;
            return SN_OK;
        }
    Record r;
    r.shape = *shape;
    r.dir = dir;
    r.algo = algo;
    r.ws = workspace_bytes;
    r.ms = ms;
    g_table.push_back(r);
    return SN_OK;
}

void sn_planner_clear(void)
{
    std::lock_guard<std::mutex> lk(g_mu);
    g_table.clear();
}

static sn_status conv_call(sn_conv_dir dir, const void *a, const void *b, void *out, const sn_conv_shape *shape,
                           sn_conv_algo algo, void *ws, size_t ws_bytes, sn_stream stream)
{
    ConvGeom g;
    sn_status s = make_geom(shape, &g);
    if (s != SN_OK) return s;
    if (!a || !b || !out || !aligned(a, 16) || !aligned(b, 16) || !aligned(out, 16)) return SN_ERR_BAD_ARG;
    if (algo < SN_ALGO_AUTO || algo >= SN_ALGO_COUNT) return SN_ERR_BAD_ARG;
    s = check_ws(ws, ws_bytes);
    if (s != SN_OK) return s;
    s = resolve(shape, g, dir, &algo, ws_bytes);
    if (s != SN_OK) return s;
    hipStream_t st = static_cast<hipStream_t>(stream);
    switch (dir) {
    case SN_CONV_FWD: return run_fwd(a, b, out, g, algo, ws, ws_bytes, st);
    case SN_CONV_BWD_DATA: return run_bwd_data(a, b, out, g, algo, ws, ws_bytes, st);
    default: return run_bwd_filter(a, b, out, g, algo, ws, ws_bytes, st);
    }
}

sn_status sn_conv2d_fwd(const void *x, const void *w, void *y, const sn_conv_shape *shape, sn_conv_algo algo,
                        void *workspace, size_t workspace_bytes, sn_stream stream)
{
    return conv_call(SN_CONV_FWD, x, w, y, shape, algo, workspace, workspace_bytes, stream);
}

sn_status sn_conv2d_fwd_noalloc(const void *x, const void *w, void *y, const sn_conv_shape *shape, sn_stream stream)
{
    ConvGeom g;
    sn_status s = make_geom(shape, &g);
    if (s != SN_OK) return s;
    if (!x || !w || !y || !aligned(x, 16) || !aligned(w, 16) || !aligned(y, 16)) return SN_ERR_BAD_ARG;
    size_t mn = 0, pf = 0;
    s = query(g, SN_CONV_FWD, SN_ALGO_STAGED, &mn, &pf);
    if (s != SN_OK) return s;
    if (mn > (size_t)SN_NOALLOC_SCRATCH_BYTES) return SN_ERR_WORKSPACE_TOO_SMALL;
    void *ws = nullptr;
    s = scratch_of_current_device(&ws);
    if (s != SN_OK) return s;
    // the packing kernel rewrites every item of the packed filter, padding included: nothing of an
    // earlier call's contents is read
    return run_fwd(x, w, y, g, SN_ALGO_STAGED, ws, SN_NOALLOC_SCRATCH_BYTES, static_cast<hipStream_t>(stream));
}

// Scratch of sn_conv2d_fwd_bn_stats: the per-tile triples of whichever tile kernel runs, or the
// partial sums of a pass over y where none does.
static size_t conv_bn_stats_need(const ConvGeom &g)
{
    size_t need = bn_stats_scratch_bytes(g.N, g.K, g.P * g.Q);
    need = std::max(need, (size_t)smallc_fwd_stats_tiles(g) * g.K * 3 * sizeof(float));
    for (int v = 0; v < 4; ++v) {
        const size_t t = (size_t)tile_conv_stats_tiles(g, (v & 1) != 0, (v & 2) != 0);
        need = std::max(need, t * g.K * 3 * sizeof(float));
    }
    return align_up(need, 256);
}

size_t sn_conv_bn_stats_scratch_bytes(const sn_conv_shape *shape)
{
    ConvGeom g;
    if (make_geom(shape, &g) != SN_OK) return 0;
    return conv_bn_stats_need(g);
}

sn_status sn_conv2d_fwd_bn_stats(const void *x, const void *w, void *y, const sn_conv_shape *shape, sn_conv_algo algo,
                                 void *workspace, size_t workspace_bytes, float *save_mean, float *save_invstd,
                                 float eps, void *scratch, size_t scratch_bytes, sn_stream stream)
{
    ConvGeom g;
    sn_status s = make_geom(shape, &g);
    if (s != SN_OK) return s;
    if (!x || !w || !y || !aligned(x, 16) || !aligned(w, 16) || !aligned(y, 16)) return SN_ERR_BAD_ARG;
    if (!save_mean || !save_invstd || !scratch || !aligned(save_mean, 4) || !aligned(save_invstd, 4) ||
        !aligned(scratch, 16) || !(eps >= 0.f))
        return SN_ERR_BAD_ARG;
    if (algo < SN_ALGO_AUTO || algo >= SN_ALGO_COUNT) return SN_ERR_BAD_ARG;
    s = check_ws(workspace, workspace_bytes);
    if (s != SN_OK) return s;
    if (scratch_bytes < conv_bn_stats_need(g)) return SN_ERR_WORKSPACE_TOO_SMALL;
    s = resolve(shape, g, SN_CONV_FWD, &algo, workspace_bytes);
    if (s != SN_OK) return s;
    hipStream_t st = static_cast<hipStream_t>(stream);
    float *part = static_cast<float *>(scratch);
    const bool staged = algo == SN_ALGO_STAGED;
    if (algo == SN_ALGO_DIRECT && smallc_supported(g)) {
        // the few-channel kernel leaves one triple per wave and channel
        if (launch_smallc_fwd(x, w, y, g, st, part) != hipSuccess) return SN_ERR_LAUNCH;
        return launch_status(launch_bn_finalize_tiles(part, g.K, smallc_fwd_stats_tiles(g), save_mean, save_invstd, eps, st));
    }
    if (tile_conv_supported(g, false) && (staged || algo == SN_ALGO_DIRECT)) {
        // the tile kernels take the statistics from their accumulators: y is not read again
        const int tiles = tile_conv_stats_tiles(g, staged, true);
        if (tiles <= 0) return SN_ERR_UNSUPPORTED;
        if (launch_tile_conv(x, w, y, g, false, staged ? workspace : nullptr, st, part) != hipSuccess) return SN_ERR_LAUNCH;
        return launch_status(launch_bn_finalize_tiles(part, g.K, tiles, save_mean, save_invstd, eps, st));
    }
    s = run_fwd(x, w, y, g, algo, workspace, workspace_bytes, st);
    if (s != SN_OK) return s;
    return launch_status(launch_bn_stats(y, part, save_mean, save_invstd, g.N, g.K, g.P * g.Q, eps, g.out_bf16, st));
}

sn_status sn_conv2d_bwd_data(const void *dy, const void *w, void *dx, const sn_conv_shape *shape,
                             sn_conv_algo algo, void *workspace, size_t workspace_bytes, sn_stream stream)
{
    return conv_call(SN_CONV_BWD_DATA, dy, w, dx, shape, algo, workspace, workspace_bytes, stream);
}

sn_status sn_conv2d_bwd_filter(const void *x, const void *dy, void *dw, const sn_conv_shape *shape,
                               sn_conv_algo algo, void *workspace, size_t workspace_bytes, sn_stream stream)
{
    return conv_call(SN_CONV_BWD_FILTER, x, dy, dw, shape, algo, workspace, workspace_bytes, stream);
}

sn_status sn_conv_autotune(sn_conv_dir dir, const void *a, const void *b, void *out, const sn_conv_shape *shape,
                           void *workspace, size_t workspace_bytes, int iters, sn_stream stream)
{
    ConvGeom g;
    sn_status s = make_geom(shape, &g);
    if (s != SN_OK) return s;
    if (dir < SN_CONV_FWD || dir > SN_CONV_BWD_FILTER || iters < 1) return SN_ERR_BAD_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return SN_ERR_LAUNCH;
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return SN_ERR_LAUNCH; }
    sn_status result = SN_OK;
    for (int algo = 0; algo < SN_ALGO_COUNT && result == SN_OK; ++algo) {
        size_t mn = 0, pf = 0;
        if (query(g, dir, (sn_conv_algo)algo, &mn, &pf) != SN_OK || mn > workspace_bytes) continue;
        const size_t used = std::min(pf, workspace_bytes);
        // one untimed run, then `iters` runs timed one by one: the median is recorded (a mean of a
        // few back-to-back launches follows whatever else disturbs one of them)
        s = conv_call(dir, a, b, out, shape, (sn_conv_algo)algo, workspace, used, stream);
        if (s != SN_OK) { result = s; break; }
        std::vector<float> times;
        for (int i = 0; i < iters; ++i) {
            float ms = 0.f;
            if (hipEventRecord(e0, st) != hipSuccess) { result = SN_ERR_LAUNCH; break; }
            s = conv_call(dir, a, b, out, shape, (sn_conv_algo)algo, workspace, used, stream);
            if (s != SN_OK) { result = s; break; }
            if (hipEventRecord(e1, st) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
                hipEventElapsedTime(&ms, e0, e1) != hipSuccess) {
                result = SN_ERR_LAUNCH;
                break;
            }
            times.push_back(ms);
        }
        if (result != SN_OK) break;
        std::sort(times.begin(), times.end());
        result = sn_planner_record(shape, dir, (sn_conv_algo)algo, used, times[times.size() / 2]);
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return result;
}

static sn_status check_cheap(int N, int C, int H, int W, int dtype)
{
    if (N < 1 || C < 1 || H < 1 || W < 1 || !valid_dtype(dtype)) return SN_ERR_BAD_ARG;
    if ((long long)H * W > 0x7fffffffLL || (long long)N * H * W > 0x7fffffffLL) return SN_ERR_UNSUPPORTED;
    if ((long long)N * C > 0x7fffffffLL) return SN_ERR_UNSUPPORTED;
    return SN_OK;
}

sn_status sn_relu_fwd(const void *x, void *y, size_t n, sn_dtype dtype, sn_stream stream)
{
    if (!valid_dtype(dtype)) return SN_ERR_BAD_ARG;
    if (n == 0) return SN_OK;
    if (!x || !y || !aligned(x, 16) || !aligned(y, 16)) return SN_ERR_BAD_ARG;
    if (n / (dtype == SN_BF16 ? 8 : 4) / 1024 > 0x7fffffffULL) return SN_ERR_UNSUPPORTED;
    return launch_status(launch_relu_fwd(x, y, n, dtype == SN_BF16, static_cast<hipStream_t>(stream)));
}

sn_status sn_relu_bwd(const void *x, const void *dy, void *dx, size_t n, sn_dtype dtype, sn_stream stream)
{
    if (!valid_dtype(dtype)) return SN_ERR_BAD_ARG;
    if (n == 0) return SN_OK;
    if (!x || !dy || !dx || !aligned(x, 16) || !aligned(dy, 16) || !aligned(dx, 16)) return SN_ERR_BAD_ARG;
    if (n / (dtype == SN_BF16 ? 8 : 4) / 1024 > 0x7fffffffULL) return SN_ERR_UNSUPPORTED;
    return launch_status(launch_relu_bwd(x, dy, dx, n, dtype == SN_BF16, static_cast<hipStream_t>(stream)));
}

static sn_status bn_fwd_common(const void *x, const float *gamma, const float *beta, void *y, float *save_mean,
                               float *save_invstd, int N, int C, int H, int W, float eps, sn_dtype dtype, int relu,
                               sn_stream stream)
{
    sn_status s = check_cheap(N, C, H, W, dtype);
    if (s != SN_OK) return s;
    if (!x || !gamma || !beta || !y || !save_mean || !save_invstd || x == y) return SN_ERR_BAD_ARG;
    if (!aligned(x, 16) || !aligned(y, 16) || !aligned(gamma, 4) || !aligned(beta, 4) || !aligned(save_mean, 4) ||
        !aligned(save_invstd, 4) || !(eps >= 0.f))
        return SN_ERR_BAD_ARG;
    if (C > 65535 * 32) return SN_ERR_UNSUPPORTED;
    return launch_status(launch_bn_fwd(x, gamma, beta, y, save_mean, save_invstd, N, C, H * W, eps,
                                       dtype == SN_BF16, relu, static_cast<hipStream_t>(stream)));
}

sn_status sn_bn_fwd(const void *x, const float *gamma, const float *beta, void *y, float *save_mean,
                    float *save_invstd, int N, int C, int H, int W, float eps, sn_dtype dtype, sn_stream stream)
{
    return bn_fwd_common(x, gamma, beta, y, save_mean, save_invstd, N, C, H, W, eps, dtype, 0, stream);
}

sn_status sn_bn_relu_fwd(const void *x, const float *gamma, const float *beta, void *y, float *save_mean,
                         float *save_invstd, int N, int C, int H, int W, float eps, sn_dtype dtype,
                         sn_stream stream)
{
    return bn_fwd_common(x, gamma, beta, y, save_mean, save_invstd, N, C, H, W, eps, dtype, 1, stream);
}

sn_status sn_bn_apply(const void *x, const float *gamma, const float *beta, const float *mean, const float *invstd,
                      void *y, int N, int C, int H, int W, int relu, sn_dtype dtype, sn_stream stream)
{
    sn_status s = check_cheap(N, C, H, W, dtype);
    if (s != SN_OK) return s;
    if (!x || !gamma || !beta || !mean || !invstd || !y || x == y) return SN_ERR_BAD_ARG;
    if (!aligned(x, 16) || !aligned(y, 16) || !aligned(gamma, 4) || !aligned(beta, 4) || !aligned(mean, 4) ||
        !aligned(invstd, 4))
        return SN_ERR_BAD_ARG;
    if (C > 65535 * 32) return SN_ERR_UNSUPPORTED;
    return launch_status(launch_bn_apply(x, gamma, beta, mean, invstd, y, N, C, H * W, dtype == SN_BF16, relu != 0,
                                         static_cast<hipStream_t>(stream)));
}

// The shapes the BN + ReLU + 2x2 pool calls take.
static sn_status check_pool2_pair(int N, int C, int H, int W, int dtype)
{
    sn_status s = check_cheap(N, C, H, W, dtype);
    if (s != SN_OK) return s;
    if ((H & 1) || (W & 1) || bn_relu_pool2_vb(W, dtype == SN_BF16) == 0) return SN_ERR_UNSUPPORTED;
    if (C > 65535 * 32) return SN_ERR_UNSUPPORTED;
    return SN_OK;
}

sn_status sn_bn_relu_pool2_fwd(const void *x, const float *gamma, const float *beta, void *pooled, int32_t *idx,
                               float *save_mean, float *save_invstd, int N, int C, int H, int W, float eps,
                               sn_dtype dtype, sn_stream stream)
{
    sn_status s = check_pool2_pair(N, C, H, W, dtype);
    if (s != SN_OK) return s;
    if (!x || !gamma || !beta || !pooled || !idx || !save_mean || !save_invstd || x == pooled ||
        x == static_cast<const void *>(idx) || pooled == static_cast<void *>(idx))
        return SN_ERR_BAD_ARG;
    if (!aligned(x, 16) || !aligned(pooled, 16) || !aligned(idx, 16) || !aligned(gamma, 4) || !aligned(beta, 4) ||
        !aligned(save_mean, 4) || !aligned(save_invstd, 4) || !(eps >= 0.f))
        return SN_ERR_BAD_ARG;
    return launch_status(launch_bn_relu_pool2_fwd(x, gamma, beta, pooled, idx, save_mean, save_invstd, N, C, H, W, eps,
                                                  dtype == SN_BF16, static_cast<hipStream_t>(stream)));
}

sn_status sn_bn_relu_pool2_apply(const void *x, const float *gamma, const float *beta, const float *mean,
                                 const float *invstd, void *pooled, int32_t *idx, int N, int C, int H, int W,
                                 sn_dtype dtype, sn_stream stream)
{
    sn_status s = check_pool2_pair(N, C, H, W, dtype);
    if (s != SN_OK) return s;
    if (!x || !gamma || !beta || !pooled || !idx || !mean || !invstd || x == pooled ||
        x == static_cast<const void *>(idx) || pooled == static_cast<void *>(idx))
        return SN_ERR_BAD_ARG;
    if (!aligned(x, 16) || !aligned(pooled, 16) || !aligned(idx, 16) || !aligned(gamma, 4) || !aligned(beta, 4) ||
        !aligned(mean, 4) || !aligned(invstd, 4))
        return SN_ERR_BAD_ARG;
    return launch_status(launch_bn_relu_pool2_apply(x, gamma, beta, mean, invstd, pooled, idx, N, C, H, W,
                                                    dtype == SN_BF16, static_cast<hipStream_t>(stream)));
}

sn_status sn_bn_relu_pool2_bwd(const void *x, const void *dpooled, const int32_t *idx, const float *gamma,
                               const float *beta, const float *save_mean, const float *save_invstd, void *dx,
                               float *dgamma, float *dbeta, int N, int C, int H, int W, sn_dtype dtype,
                               sn_stream stream)
{
    sn_status s = check_pool2_pair(N, C, H, W, dtype);
    if (s != SN_OK) return s;
    if (!x || !dpooled || !idx || !gamma || !beta || !save_mean || !save_invstd || !dx || !dgamma || !dbeta ||
        dx == x || dx == dpooled || dx == static_cast<const void *>(idx))
        return SN_ERR_BAD_ARG;
    if (!aligned(x, 16) || !aligned(dpooled, 16) || !aligned(idx, 16) || !aligned(dx, 16) || !aligned(gamma, 4) ||
        !aligned(beta, 4) || !aligned(save_mean, 4) || !aligned(save_invstd, 4) || !aligned(dgamma, 4) ||
        !aligned(dbeta, 4))
        return SN_ERR_BAD_ARG;
    return launch_status(launch_bn_bwd(x, nullptr, beta, gamma, save_mean, save_invstd, dx, dgamma, dbeta, N, C, H * W,
                                       dtype == SN_BF16, static_cast<hipStream_t>(stream), dpooled, idx, W));
}

static sn_status bn_bwd_common(const void *x, const void *dy, const float *relu_beta, const float *gamma,
                               const float *save_mean, const float *save_invstd, void *dx, float *dgamma,
                               float *dbeta, int N, int C, int H, int W, sn_dtype dtype, sn_stream stream)
{
    sn_status s = check_cheap(N, C, H, W, dtype);
    if (s != SN_OK) return s;
    if (!x || !dy || !gamma || !save_mean || !save_invstd || !dx || !dgamma || !dbeta || dx == x || dx == dy)
        return SN_ERR_BAD_ARG;
    if (!aligned(x, 16) || !aligned(dy, 16) || !aligned(dx, 16) || !aligned(gamma, 4) || !aligned(save_mean, 4) ||
        !aligned(save_invstd, 4) || !aligned(dgamma, 4) || !aligned(dbeta, 4) || (relu_beta && !aligned(relu_beta, 4)))
        return SN_ERR_BAD_ARG;
    if (C > 65535 * 32) return SN_ERR_UNSUPPORTED;
    return launch_status(launch_bn_bwd(x, dy, relu_beta, gamma, save_mean, save_invstd, dx, dgamma, dbeta, N, C, H * W,
                                       dtype == SN_BF16, static_cast<hipStream_t>(stream)));
}

sn_status sn_bn_bwd(const void *x, const void *dy, const float *gamma, const float *save_mean,
                    const float *save_invstd, void *dx, float *dgamma, float *dbeta, int N, int C, int H, int W,
                    sn_dtype dtype, sn_stream stream)
{
    return bn_bwd_common(x, dy, nullptr, gamma, save_mean, save_invstd, dx, dgamma, dbeta, N, C, H, W, dtype, stream);
}

sn_status sn_bn_relu_bwd(const void *x, const void *dy, const float *gamma, const float *beta,
                         const float *save_mean, const float *save_invstd, void *dx, float *dgamma, float *dbeta,
                         int N, int C, int H, int W, sn_dtype dtype, sn_stream stream)
{
    if (!beta) return SN_ERR_BAD_ARG;
    return bn_bwd_common(x, dy, beta, gamma, save_mean, save_invstd, dx, dgamma, dbeta, N, C, H, W, dtype, stream);
}

static sn_status lrn_common(const void *x, const void *dy, void *out, int N, int C, int H, int W, int size,
                            float alpha, float beta, float k, sn_dtype dtype, sn_stream stream, bool bwd, int relu = 0)
{
    sn_status s = check_cheap(N, C, H, W, dtype);
    if (s != SN_OK) return s;
    if (!x || !out || (bwd && !dy) || out == x || (bwd && out == dy)) return SN_ERR_BAD_ARG;
    if (!aligned(x, 16) || !aligned(out, 16) || (bwd && !aligned(dy, 16))) return SN_ERR_BAD_ARG;
    if (size < 1 || !(size & 1) || !(alpha >= 0.f) || !(k > 0.f) || !(beta == beta)) return SN_ERR_BAD_ARG;
    if (size > 9) return SN_ERR_UNSUPPORTED;
    if ((long long)N * H * W / 256 > 0x7fffffffLL) return SN_ERR_UNSUPPORTED;
    return launch_status(launch_lrn(x, bwd ? dy : nullptr, out, N, C, H * W, size, alpha, beta, k, dtype == SN_BF16,
                                    static_cast<hipStream_t>(stream), relu));
}

sn_status sn_lrn_fwd(const void *x, void *y, int N, int C, int H, int W, int size, float alpha, float beta, float k,
                     sn_dtype dtype, sn_stream stream)
{
    return lrn_common(x, nullptr, y, N, C, H, W, size, alpha, beta, k, dtype, stream, false);
}

sn_status sn_lrn_bwd(const void *x, const void *dy, void *dx, int N, int C, int H, int W, int size, float alpha,
                     float beta, float k, sn_dtype dtype, sn_stream stream)
{
    return lrn_common(x, dy, dx, N, C, H, W, size, alpha, beta, k, dtype, stream, true);
}

sn_status sn_relu_lrn_fwd(const void *x, void *y, int N, int C, int H, int W, int size, float alpha, float beta,
                          float k, sn_dtype dtype, sn_stream stream)
{
    return lrn_common(x, nullptr, y, N, C, H, W, size, alpha, beta, k, dtype, stream, false, 1);
}

sn_status sn_relu_lrn_bwd(const void *x, const void *dy, void *dx, int N, int C, int H, int W, int size, float alpha,
                          float beta, float k, sn_dtype dtype, sn_stream stream)
{
    return lrn_common(x, dy, dx, N, C, H, W, size, alpha, beta, k, dtype, stream, true, 1);
}

static sn_status check_pool(int N, int C, int H, int W, int kh, int kw, int sh, int sw, int ph, int pw, int dtype,
                            int *P, int *Q)
{
    sn_status s = check_cheap(N, C, H, W, dtype);
    if (s != SN_OK) return s;
    if (kh < 1 || kw < 1 || sh < 1 || sw < 1 || ph < 0 || pw < 0 || ph >= kh || pw >= kw) return SN_ERR_BAD_ARG;
    *P = sn_out_dim(H, ph, kh, sh);
    *Q = sn_out_dim(W, pw, kw, sw);
    if (*P < 1 || *Q < 1) return SN_ERR_BAD_ARG;
    return SN_OK;
}

sn_status sn_maxpool_fwd(const void *x, void *y, int32_t *idx, int N, int C, int H, int W, int kh, int kw, int sh,
                         int sw, int ph, int pw, sn_dtype dtype, sn_stream stream)
{
    int P, Q;
    sn_status s = check_pool(N, C, H, W, kh, kw, sh, sw, ph, pw, dtype, &P, &Q);
    if (s != SN_OK) return s;
    if (!x || !y || !idx || !aligned(x, 16) || !aligned(y, 16) || !aligned(idx, 16)) return SN_ERR_BAD_ARG;
    return launch_status(launch_maxpool_fwd(x, y, idx, N * C, H, W, P, Q, kh, kw, sh, sw, ph, pw,
                                            dtype == SN_BF16, static_cast<hipStream_t>(stream)));
}

sn_status sn_maxpool_bwd(const void *dy, const int32_t *idx, void *dx, int N, int C, int H, int W, int kh, int kw,
                         int sh, int sw, int ph, int pw, sn_dtype dtype, sn_stream stream)
{
    int P, Q;
    sn_status s = check_pool(N, C, H, W, kh, kw, sh, sw, ph, pw, dtype, &P, &Q);
    if (s != SN_OK) return s;
    if (!dy || !idx || !dx || !aligned(dy, 16) || !aligned(dx, 16) || !aligned(idx, 16)) return SN_ERR_BAD_ARG;
    return launch_status(launch_maxpool_bwd(dy, idx, dx, N * C, H, W, P, Q, kh, kw, sh, sw, ph, pw,
                                            dtype == SN_BF16, static_cast<hipStream_t>(stream)));
}

}  // extern "C"
