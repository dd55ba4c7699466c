// Layout transforms of the phase decomposition of strided convolutions (the STAGED algorithm on
// strided shapes, Sec. 3.5 of the paper: workspace bought speed).
//
// A convolution with strides (sh, sw) reads input row p*sh + r - ph for output row p and filter
// row r.  Writing r - ph = d*sh + a with 0 <= a < sh, that row is row p + d of "phase" a of the
// input, x_a[i] = x[i*sh + a] (columns likewise with e, b).  Over the phase planes as channels the
// convolution has stride 1 and a filter whose taps are the (d, e) that occur; the layers here have
// d, e in {-1, 0, 1}, i.e. a 3x3 filter with "same" padding on planes of the output's size (or 1x1
// for 1x1 filters), or in {0, 1, 2} (filters up to three strides long without padding, e.g. 11x11 /
// stride 4), a 3x3 filter without padding on planes two rows / columns larger, which the stride-1
// MFMA kernels run.  Taps that do not occur are zeros in the
// transformed filter.  This file holds the copies around that inner convolution:
//   phase_split   x  -> xs[n][phase*C + c][i][j]           (forward, backward-filter)
//   phase_filter  w  -> w'[k][phase*C + c][d+1][e+1]       (forward, backward-data)
//   phase_merge   dxs -> dx, zeros where no tap reaches    (backward-data)
//   phase_dw      dw' -> dw                                (backward-filter)
// All are HBM-bound copies; the planes are 1/(sh*sw) of the input each.
#include "sn_internal.h"

namespace sn {
namespace {

// 8 consecutive plane columns per thread, written as one 16-byte item per column phase.  With a
// column stride of 2 and rows that keep 16-byte alignment (W a multiple of 8) the thread reads the
// 16 input columns behind them with two 16-byte loads and splits them into the even and the odd
// phase; otherwise element by element.
template <bool PAIR>
__global__ void __launch_bounds__(256)
phase_split_kernel(const bf16_t *__restrict__ x, bf16_t *__restrict__ xs, PhaseMap m, int N, int C, int H, int W,
                   int Hs, int Ws, long long items)
{
    const long long it = (long long)blockIdx.x * 256 + threadIdx.x;
    if (it >= items) return;
    const int W8 = (Ws + 7) >> 3;
    const int j0 = (int)(it % W8) * 8;
    long long t = it / W8;
    const int i = (int)(t % Hs);
    t /= Hs;
    // PAIR: one thread serves every column phase of (row phase, channel); else one phase each
    const int groups = PAIR ? m.na : m.nphases;
    const int cg = (int)(t % ((long long)C * groups));
    const int n = (int)(t / ((long long)C * groups));
    const int grp = cg / C, c = cg - grp * C;
    const int ia = PAIR ? grp : grp / m.nb;
    const int a = m.row_phase[ia];
    const int h = i * m.sh + a;
    const bf16_t *src = x + (((long long)n * C + c) * H + h) * W;
    const long long plane = (long long)Hs * Ws;
    if (PAIR) {
        uint32_t in[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        if (h < H) {
            const int v0 = j0 * 2;
            if (v0 + 8 <= W) {
                const uint4 q = *reinterpret_cast<const uint4 *>(src + v0);
                in[0] = q.x; in[1] = q.y; in[2] = q.z; in[3] = q.w;
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (v0 + e < W) in[e >> 1] |= (uint32_t)src[v0 + e] << (16 * (e & 1));
            }
            if (v0 + 16 <= W) {
                const uint4 q = *reinterpret_cast<const uint4 *>(src + v0 + 8);
                in[4] = q.x; in[5] = q.y; in[6] = q.z; in[7] = q.w;
            } else {
#pragma unroll
                for (int e = 8; e < 16; ++e)
                    if (v0 + e < W) in[e >> 1] |= (uint32_t)src[v0 + e] << (16 * (e & 1));
            }
        }
#pragma unroll
        for (int ib = 0; ib < 2; ++ib) {
            if (ib >= m.nb) break;
            const int b = m.col_phase[ib];
            uint32_t d[4];
#pragma unroll
            for (int k = 0; k < 4; ++k)   // output elements 2k, 2k+1 = input dwords 2k, 2k+1, half b
                d[k] = b ? __builtin_amdgcn_perm(in[2 * k + 1], in[2 * k], 0x07060302u)
                         : __builtin_amdgcn_perm(in[2 * k + 1], in[2 * k], 0x05040100u);
            bf16_t *dst = xs + ((long long)n * C * m.nphases + (long long)(ia * m.nb + ib) * C + c) * plane + (long long)i * Ws + j0;
            if (j0 + 8 <= Ws && (reinterpret_cast<uintptr_t>(dst) & 15) == 0) {
                *reinterpret_cast<uint4 *>(dst) = make_uint4(d[0], d[1], d[2], d[3]);
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (j0 + e < Ws) dst[e] = (bf16_t)(d[e >> 1] >> (16 * (e & 1)));
            }
        }
    } else {
        const int ib = grp % m.nb, b = m.col_phase[ib];
        uint32_t d[4] = {0, 0, 0, 0};
        if (h < H) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int v = (j0 + e) * m.sw + b;
                if (j0 + e < Ws && v < W) d[e >> 1] |= (uint32_t)src[v] << (16 * (e & 1));
            }
        }
        bf16_t *dst = xs + ((long long)n * C * m.nphases + (long long)grp * C + c) * plane + (long long)i * Ws + j0;
        if (j0 + 8 <= Ws && (reinterpret_cast<uintptr_t>(dst) & 15) == 0) {
            *reinterpret_cast<uint4 *>(dst) = make_uint4(d[0], d[1], d[2], d[3]);
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (j0 + e < Ws) dst[e] = (bf16_t)(d[e >> 1] >> (16 * (e & 1)));
        }
    }
}

// One thread per element of w'.
__global__ void __launch_bounds__(256)
phase_filter_kernel(const bf16_t *__restrict__ w, bf16_t *__restrict__ wp, PhaseMap m, int K, int C, int R, int S,
                    long long total)
{
    const long long it = (long long)blockIdx.x * 256 + threadIdx.x;
    if (it >= total) return;
    const int T = m.Ri * m.Si;
    const int tap = (int)(it % T);
    long long t = it / T;
    const int cp = (int)(t % ((long long)C * m.nphases));
    const int k = (int)(t / ((long long)C * m.nphases));
    const int phase = cp / C, c = cp - phase * C;
    const int a = m.row_phase[phase / m.nb], b = m.col_phase[phase % m.nb];
    const int dd = tap / m.Si - m.center_r, ee = tap % m.Si - m.center_c;
    const int r = dd * m.sh + a + m.ph, s = ee * m.sw + b + m.pw;   // the tap with r - ph = d*sh + a
    bf16_t v = 0;
    if (r >= 0 && r < R && s >= 0 && s < S) v = w[(((long long)k * C + c) * R + r) * S + s];
    wp[it] = v;
}

// dx from the phase planes: 8 consecutive columns per thread.  PAIR (bf16, column stride 2, rows
// of dx and of the planes on 16- and 8-byte boundaries): the 8 columns are 4 of the even and 4 of
// the odd column phase, read as 8 bytes each and interleaved; otherwise element by element.
template <typename T, bool PAIR>
__global__ void __launch_bounds__(256)
phase_merge_kernel(const T *__restrict__ dxs, T *__restrict__ dx, PhaseMap m, int N, int C, int H, int W, int Hs,
                   int Ws, long long items)
{
    const long long it = (long long)blockIdx.x * 256 + threadIdx.x;
    if (it >= items) return;
    const int W8 = (W + 7) >> 3;
    const int v0 = (int)(it % W8) * 8;
    long long t = it / W8;
    const int h = (int)(t % H);
    t /= H;
    const int c = (int)(t % C), n = (int)(t / C);
    const int ia = m.row_index[h % m.sh], i = h / m.sh;
    T *dst = dx + (((long long)n * C + c) * H + h) * W + v0;
    const long long plane = (long long)Hs * Ws;
    if (PAIR) {
        uint32_t out[4] = {0, 0, 0, 0};
        if (ia >= 0 && i < Hs) {
            const int j = v0 >> 1;
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                const int ib = m.col_index[b];
                if (ib < 0) continue;
                const T *src = dxs + ((long long)n * C * m.nphases + (long long)(ia * m.nb + ib) * C + c) * plane + (long long)i * Ws + j;
                uint32_t lo = 0, hi = 0;
                if (j + 4 <= Ws) {
                    const uint2 q = *reinterpret_cast<const uint2 *>(src);
                    lo = q.x; hi = q.y;
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (j + e < Ws) (e < 2 ? lo : hi) |= (uint32_t)reinterpret_cast<const bf16_t *>(src)[e] << (16 * (e & 1));
                }
                // plane elements 0..3 go to dx columns b, 2 + b, 4 + b, 6 + b
                out[0] |= (lo & 0xffffu) << (16 * b);
                out[1] |= (lo >> 16) << (16 * b);
                out[2] |= (hi & 0xffffu) << (16 * b);
                out[3] |= (hi >> 16) << (16 * b);
            }
        }
        if (v0 + 8 <= W) {
            *reinterpret_cast<uint4 *>(dst) = make_uint4(out[0], out[1], out[2], out[3]);
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (v0 + e < W) reinterpret_cast<bf16_t *>(dst)[e] = (bf16_t)(out[e >> 1] >> (16 * (e & 1)));
        }
        return;
    }
    T vals[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int v = v0 + e;
        T val = (T)0;
        if (v < W && ia >= 0 && i < Hs) {
            const int ib = m.col_index[v % m.sw], j = v / m.sw;
            if (ib >= 0 && j < Ws)
                val = dxs[((long long)n * C * m.nphases + (long long)(ia * m.nb + ib) * C + c) * plane + (long long)i * Ws + j];
        }
        vals[e] = val;
    }
#pragma unroll
    for (int e = 0; e < 8; ++e)
        if (v0 + e < W) dst[e] = vals[e];
}

// dw[k][c][r][s] = dw'[k][phase*C + c][d + center_r][e + center_c]: one thread per element of dw.
__global__ void __launch_bounds__(256)
phase_dw_kernel(const float *__restrict__ dwp, float *__restrict__ dw, PhaseMap m, int K, int C, int R, int S,
                long long total)
{
    const long long it = (long long)blockIdx.x * 256 + threadIdx.x;
    if (it >= total) return;
    const int s = (int)(it % S);
    long long t = it / S;
    const int r = (int)(t % R);
    t /= R;
    const int c = (int)(t % C), k = (int)(t / C);
    const int u = r - m.ph, z = s - m.pw;
    // floor division and non-negative remainder
    const int d = (u >= 0 ? u : u - m.sh + 1) / m.sh, a = u - d * m.sh;
    const int e = (z >= 0 ? z : z - m.sw + 1) / m.sw, b = z - e * m.sw;
    const int phase = m.row_index[a] * m.nb + m.col_index[b];
    dw[it] = dwp[((((long long)k * m.nphases + phase) * C + c) * m.Ri + (d + m.center_r)) * m.Si + (e + m.center_c)];
}

unsigned blocks_for(long long items) { return (unsigned)((items + 255) / 256); }

}  // namespace

hipError_t launch_phase_split(const void *x, void *xs, const PhaseMap &m, const ConvGeom &g, hipStream_t st)
{
    // the paired form: column stride 2, input rows on 16-byte boundaries
    const bool pair = m.sw == 2 && g.W % 8 == 0 && reinterpret_cast<uintptr_t>(x) % 16 == 0;
    const long long items = (long long)g.N * g.C * (pair ? m.na : m.nphases) * m.Hs * ((m.Ws + 7) / 8);
    if (items > 0x7fffffffLL * 256) return hipErrorInvalidValue;
    if (pair)
        hipLaunchKernelGGL(phase_split_kernel<true>, dim3(blocks_for(items)), dim3(256), 0, st, static_cast<const bf16_t *>(x),
                           static_cast<bf16_t *>(xs), m, g.N, g.C, g.H, g.W, m.Hs, m.Ws, items);
    else
        hipLaunchKernelGGL(phase_split_kernel<false>, dim3(blocks_for(items)), dim3(256), 0, st, static_cast<const bf16_t *>(x),
                           static_cast<bf16_t *>(xs), m, g.N, g.C, g.H, g.W, m.Hs, m.Ws, items);
    return hipGetLastError();
}

hipError_t launch_phase_filter(const void *w, void *wp, const PhaseMap &m, const ConvGeom &g, hipStream_t st)
{
    const long long total = (long long)g.K * g.C * m.nphases * m.Ri * m.Si;
    hipLaunchKernelGGL(phase_filter_kernel, dim3(blocks_for(total)), dim3(256), 0, st, static_cast<const bf16_t *>(w),
                       static_cast<bf16_t *>(wp), m, g.K, g.C, g.R, g.S, total);
    return hipGetLastError();
}

hipError_t launch_phase_merge(const void *dxs, void *dx, const PhaseMap &m, const ConvGeom &g, hipStream_t st)
{
    const long long items = (long long)g.N * g.C * g.H * ((g.W + 7) / 8);
    if (items > 0x7fffffffLL * 256) return hipErrorInvalidValue;
    const dim3 grid(blocks_for(items)), block(256);
    if (g.out_bf16) {
        const bf16_t *src = static_cast<const bf16_t *>(dxs);
        bf16_t *dst = static_cast<bf16_t *>(dx);
        // rows of dx on 16-byte boundaries, rows of the planes on 8-byte boundaries
        const bool pair = m.sw == 2 && g.W % 8 == 0 && m.Ws % 4 == 0 && reinterpret_cast<uintptr_t>(dx) % 16 == 0 &&
                          reinterpret_cast<uintptr_t>(dxs) % 16 == 0;
        if (pair)
            hipLaunchKernelGGL((phase_merge_kernel<bf16_t, true>), grid, block, 0, st, src, dst, m, g.N, g.C, g.H, g.W, m.Hs, m.Ws, items);
        else
            hipLaunchKernelGGL((phase_merge_kernel<bf16_t, false>), grid, block, 0, st, src, dst, m, g.N, g.C, g.H, g.W, m.Hs, m.Ws, items);
    } else {
        hipLaunchKernelGGL((phase_merge_kernel<float, false>), grid, block, 0, st, static_cast<const float *>(dxs),
                           static_cast<float *>(dx), m, g.N, g.C, g.H, g.W, m.Hs, m.Ws, items);
    }
    return hipGetLastError();
}

hipError_t launch_phase_dw(const float *dwp, float *dw, const PhaseMap &m, const ConvGeom &g, hipStream_t st)
{
    const long long total = (long long)g.K * g.C * g.R * g.S;
    hipLaunchKernelGGL(phase_dw_kernel, dim3(blocks_for(total)), dim3(256), 0, st, dwp, dw, m, g.K, g.C, g.R, g.S, total);
    return hipGetLastError();
}

}  // namespace sn
