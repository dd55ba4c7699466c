// Winograd F(2x2, 3x3) for the fp32 path: 3x3 stride-1 CONV forward and backward-data with
// 2.25x fewer multiplications than the direct form, bought with workspace (the trade of Sec. 3.5 of
// the paper: an algorithm that needs temporary memory to deliver its speed).
//
//   Y = A^T [ (G g G^T) . (B^T d B) ] A   per 4x4 input tile d, 3x3 filter g, 2x2 output tile Y,
// summed over the input channels, with the usual matrices
//   B^T = [1 0 -1 0; 0 1 1 0; 0 -1 1 0; 0 1 0 -1],  G = [1 0 0; .5 .5 .5; .5 -.5 .5; 0 0 1],
//   A^T = [1 1 1 0; 0 1 -1 -1].
// The sum over channels is 16 independent matrix products (one per position xi of the 4x4
// transformed tile):  Mo_xi[m][t] = sum_red U_xi[red][m] * V_xi[red][t],  m = output channel,
// t = tile number, red = input channel -- plain fp32 GEMMs on v_mfma_f32_32x32x2_f32.
// Backward-data is the same computation on dy with the filter transposed in (k,c) and flipped in
// (r,s) and padding 2 - pad, as in the tile kernels.
//
// Workspace (fp32): U[16][REDp][Mp] | V[16][REDp][Tp] | Mo[16][Mp][Tp] for the images of one pass;
// REDp, Mp, Tp are RED, M, T rounded up to the GEMM's tile (16, 128, 128), the padding of U and V
// along red is zero.  Four kernels per pass: filter transform (once per call), input transform,
// GEMM, output transform; the transforms are HBM-bound.
#include <algorithm>

#include "sn_internal.h"

namespace sn {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int BM = 128, BN = 128, BK = 16;

struct WinoProblem {
    int N, RED, Hin, Win, M, Pout, Qout, padh, padw;
    int w_sm, w_sr, tflip;   // filter element A(m, red, tap) = w[m*w_sm + red*w_sr + (tflip ? 8 - tap : tap)]
    int tilesH, tilesW;
    int REDp, Mp;
};

// U[xi][red][m] = (G g G^T)[xi], zero for red >= RED or m >= M.  One thread per (red, m).
__global__ void __launch_bounds__(256)
wino_filter_kernel(const float *__restrict__ w, float *__restrict__ U, WinoProblem p)
{
    const int m = blockIdx.x * 256 + threadIdx.x, red = blockIdx.y;
    if (m >= p.Mp) return;
    float g[9];
    const bool real = m < p.M && red < p.RED;
#pragma unroll
    for (int t = 0; t < 9; ++t)
        g[t] = real ? w[(size_t)m * p.w_sm + (size_t)red * p.w_sr + (p.tflip ? 8 - t : t)] : 0.f;
    // rows of G g: t0 = g0, t1 = (g0 + g1 + g2)/2, t2 = (g0 - g1 + g2)/2, t3 = g2 (g_r = filter row r)
    float Gg[4][3];
#pragma unroll
    for (int s = 0; s < 3; ++s) {
        Gg[0][s] = g[s];
        Gg[1][s] = 0.5f * (g[s] + g[3 + s] + g[6 + s]);
        Gg[2][s] = 0.5f * (g[s] - g[3 + s] + g[6 + s]);
        Gg[3][s] = g[6 + s];
    }
    const size_t plane = (size_t)p.REDp * p.Mp;
    float *dst = U + (size_t)red * p.Mp + m;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float a = Gg[i][0], b = Gg[i][1], c = Gg[i][2];
        dst[(size_t)(i * 4 + 0) * plane] = a;
        dst[(size_t)(i * 4 + 1) * plane] = 0.5f * (a + b + c);
        dst[(size_t)(i * 4 + 2) * plane] = 0.5f * (a - b + c);
        dst[(size_t)(i * 4 + 3) * plane] = c;
    }
}

// V[xi][red][t] = (B^T d B)[xi] for the tiles of images n0 .. n0+nimg-1; zero for red >= RED and
// for t past the last tile.  One thread per (red, t); Tp = blockDim-rounded tile count.
__global__ void __launch_bounds__(256)
wino_input_kernel(const float *__restrict__ in, float *__restrict__ V, WinoProblem p, int n0, int T, int Tp)
{
    const int t = blockIdx.x * 256 + threadIdx.x, red = blockIdx.y;
    if (t >= Tp) return;
    float d[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) d[i][j] = 0.f;
    if (t < T && red < p.RED) {
        const int per = p.tilesH * p.tilesW;
        const int ni = t / per, rem = t - ni * per, th = rem / p.tilesW, tw = rem - th * p.tilesW;
        const int h0 = 2 * th - p.padh, v0 = 2 * tw - p.padw;
        const float *src = in + ((size_t)(n0 + ni) * p.RED + red) * p.Hin * p.Win;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int h = h0 + i;
            if ((unsigned)h >= (unsigned)p.Hin) continue;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int v = v0 + j;
                if ((unsigned)v < (unsigned)p.Win) d[i][j] = src[(size_t)h * p.Win + v];
            }
        }
    }
    // B^T d: rows d0 - d2, d1 + d2, d2 - d1, d1 - d3; then the same on the columns
    float Bd[4][4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        Bd[0][j] = d[0][j] - d[2][j];
        Bd[1][j] = d[1][j] + d[2][j];
        Bd[2][j] = d[2][j] - d[1][j];
        Bd[3][j] = d[1][j] - d[3][j];
    }
    const size_t plane = (size_t)p.REDp * Tp;
    float *dst = V + (size_t)red * Tp + t;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        dst[(size_t)(i * 4 + 0) * plane] = Bd[i][0] - Bd[i][2];
        dst[(size_t)(i * 4 + 1) * plane] = Bd[i][1] + Bd[i][2];
        dst[(size_t)(i * 4 + 2) * plane] = Bd[i][2] - Bd[i][1];
        dst[(size_t)(i * 4 + 3) * plane] = Bd[i][1] - Bd[i][3];
    }
}

// Mo_xi[m][t] = sum_red U_xi[red][m] * V_xi[red][t].  A 256-thread workgroup owns a 128 x 128 tile
// of one xi; a wave a 64 x 64 block (2 x 2 MFMA tiles).  Both operands are stored reduction-major, so
// a step's two LDS tiles [16][128] are plain 16-byte copies and an MFMA lane's operand is one float
// of a row of consecutive floats.  Double-buffered: the global loads of step i+1 are issued before
// the MFMAs of step i and written to the other buffer after them; one barrier per step.
__global__ void __launch_bounds__(256, 2)
wino_gemm_kernel(const float *__restrict__ U, const float *__restrict__ V, float *__restrict__ Mo, int REDp, int Mp, int Tp)
{
    __shared__ __attribute__((aligned(16))) float As[2][BK][BM];
    __shared__ __attribute__((aligned(16))) float Bs[2][BK][BN];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, g = lane >> 5;
    const int wm = wave >> 1, wn = wave & 1;
    const int t0 = blockIdx.x * BN, m0 = blockIdx.y * BM, xi = blockIdx.z;
    const float *Ux = U + (size_t)xi * REDp * Mp + m0;
    const float *Vx = V + (size_t)xi * REDp * Tp + t0;
    // a thread copies two float4 of each tile: rows tid / 32 and tid / 32 + 8, columns 4 * (tid % 32)
    const int cr = tid >> 5, cc = (tid & 31) * 4;
    float4 ra[2], rb[2];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            ra[i] = *reinterpret_cast<const float4 *>(Ux + (size_t)(k0 + cr + 8 * i) * Mp + cc);
            rb[i] = *reinterpret_cast<const float4 *>(Vx + (size_t)(k0 + cr + 8 * i) * Tp + cc);
        }
    };
    auto stash = [&](int buf) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            *reinterpret_cast<float4 *>(&As[buf][cr + 8 * i][cc]) = ra[i];
            *reinterpret_cast<float4 *>(&Bs[buf][cr + 8 * i][cc]) = rb[i];
        }
    };
    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    fetch(0);
    stash(0);
    __syncthreads();
    const int nsteps = REDp / BK;
    for (int step = 0; step < nsteps; ++step) {
        const int buf = step & 1;
        if (step + 1 < nsteps) fetch((step + 1) * BK);
#pragma unroll
        for (int s = 0; s < BK / 2; ++s) {
            float a[2], b[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                a[i] = As[buf][2 * s + g][wm * 64 + i * 32 + l32];
                b[i] = Bs[buf][2 * s + g][wn * 64 + i * 32 + l32];
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc[i][j], 0, 0, 0);
        }
        if (step + 1 < nsteps) stash(buf ^ 1);
        __syncthreads();
    }
    // acc[i][j][v]: row m = 8 (v / 4) + 4 (lane / 32) + v % 4 of tile i, column t = lane % 32 of tile j
    float *out = Mo + (size_t)xi * Mp * Tp;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + wm * 64 + i * 32 + 8 * (v / 4) + 4 * g + v % 4;
                const int t = t0 + wn * 64 + j * 32 + l32;
                out[(size_t)m * Tp + t] = acc[i][j][v];
            }
}

// y tile = A^T Mo A.  One thread per (m, t).
template <typename TOut>
__global__ void __launch_bounds__(256)
wino_output_kernel(const float *__restrict__ Mo, TOut *__restrict__ out, WinoProblem p, int n0, int T, int Tp)
{
    const int t = blockIdx.x * 256 + threadIdx.x, m = blockIdx.y;
    if (t >= T) return;
    const size_t plane = (size_t)p.Mp * Tp;
    const float *src = Mo + (size_t)m * Tp + t;
    float x[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) x[i][j] = src[(size_t)(i * 4 + j) * plane];
    float r[2][4];   // A^T x
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        r[0][j] = x[0][j] + x[1][j] + x[2][j];
        r[1][j] = x[1][j] - x[2][j] - x[3][j];
    }
    const int per = p.tilesH * p.tilesW;
    const int ni = t / per, rem = t - ni * per, th = rem / p.tilesW, tw = rem - th * p.tilesW;
    TOut *dst = out + ((size_t)(n0 + ni) * p.M + m) * p.Pout * p.Qout;
#pragma unroll
    for (int a = 0; a < 2; ++a) {
        const int pp = 2 * th + a;
        if (pp >= p.Pout) continue;
        const float y0 = r[a][0] + r[a][1] + r[a][2], y1 = r[a][1] - r[a][2] - r[a][3];
        const int q = 2 * tw;
        dst[(size_t)pp * p.Qout + q] = (TOut)y0;
        if (q + 1 < p.Qout) dst[(size_t)pp * p.Qout + q + 1] = (TOut)y1;
    }
}

bool wino_problem(const ConvGeom &g, bool bwd_data, WinoProblem *p)
{
    if (g.in_bf16 || g.out_bf16 || g.R != 3 || g.S != 3 || g.sh != 1 || g.sw != 1) return false;
    if (!bwd_data) {
        p->N = g.N; p->RED = g.C; p->Hin = g.H; p->Win = g.W; p->M = g.K; p->Pout = g.P; p->Qout = g.Q;
        p->padh = g.ph; p->padw = g.pw;
        p->w_sm = g.C * 9; p->w_sr = 9; p->tflip = 0;
    } else {
        if (g.ph > 2 || g.pw > 2) return false;
        p->N = g.N; p->RED = g.K; p->Hin = g.P; p->Win = g.Q; p->M = g.C; p->Pout = g.H; p->Qout = g.W;
        p->padh = 2 - g.ph; p->padw = 2 - g.pw;
        p->w_sm = 9; p->w_sr = g.C * 9; p->tflip = 1;
    }
    p->tilesH = (p->Pout + 1) / 2;
    p->tilesW = (p->Qout + 1) / 2;
    p->REDp = (p->RED + BK - 1) / BK * BK;
    p->Mp = (p->M + BM - 1) / BM * BM;
    if ((long long)p->tilesH * p->tilesW * p->N > 0x7fffffffLL - BN) return false;
    if (p->REDp > 65535 || p->M > 65535) return false;   // grid.y of the transforms
    return true;
}

size_t u_bytes(const WinoProblem &p) { return align_up((size_t)16 * p.REDp * p.Mp * sizeof(float), 256); }

size_t pass_bytes(const WinoProblem &p, int nimg)
{
    const size_t T = (size_t)nimg * p.tilesH * p.tilesW, Tp = (T + BN - 1) / BN * BN;
    return align_up((size_t)16 * p.REDp * Tp * sizeof(float), 256) + align_up((size_t)16 * p.Mp * Tp * sizeof(float), 256);
}

// Images per pass: the most whose V and Mo fit beside U (pass_bytes grows with the count); 0 = none.
int images_per_pass(const WinoProblem &p, size_t ws_bytes)
{
    if (ws_bytes < u_bytes(p) + pass_bytes(p, 1)) return 0;
    int lo = 1, hi = p.N;
    while (lo < hi) {
        const int mid = (lo + hi + 1) / 2;
        if (u_bytes(p) + pass_bytes(p, mid) <= ws_bytes) lo = mid;
        else hi = mid - 1;
    }
    return lo;
}

}  // namespace

long long winograd_pass_tiles(const ConvGeom &g, bool bwd_data, size_t ws_bytes)
{
    WinoProblem p;
    if (!wino_problem(g, bwd_data, &p)) return 0;
    return (long long)images_per_pass(p, ws_bytes) * p.tilesH * p.tilesW;
}

bool winograd_supported(const ConvGeom &g, bool bwd_data)
{
    WinoProblem p;
    return wino_problem(g, bwd_data, &p);
}

// Least workspace (one image per pass) and the workspace beyond which it gets no faster (one pass).
void winograd_bytes(const ConvGeom &g, bool bwd_data, size_t *min_b, size_t *pref_b)
{
    WinoProblem p;
    *min_b = *pref_b = 0;
    if (!wino_problem(g, bwd_data, &p)) return;
    *min_b = u_bytes(p) + pass_bytes(p, 1);
    *pref_b = u_bytes(p) + pass_bytes(p, p.N);
}

hipError_t launch_winograd(const void *in, const void *w, void *out, const ConvGeom &g, bool bwd_data, void *ws,
                           size_t ws_bytes, hipStream_t st)
{
    WinoProblem p;
    if (!wino_problem(g, bwd_data, &p)) return hipErrorInvalidValue;
    const int nimg = images_per_pass(p, ws_bytes);
    if (nimg < 1) return hipErrorInvalidValue;
    float *U = static_cast<float *>(ws);
    hipLaunchKernelGGL(wino_filter_kernel, dim3((p.Mp + 255) / 256, p.REDp), dim3(256), 0, st,
                       static_cast<const float *>(w), U, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int per = p.tilesH * p.tilesW;
    for (int n0 = 0; n0 < p.N; n0 += nimg) {
        const int ni = std::min(nimg, p.N - n0);
        const int T = ni * per, Tp = (T + BN - 1) / BN * BN;
        float *V = reinterpret_cast<float *>(static_cast<char *>(ws) + u_bytes(p));
        float *Mo = reinterpret_cast<float *>(reinterpret_cast<char *>(V) + align_up((size_t)16 * p.REDp * Tp * sizeof(float), 256));
        hipLaunchKernelGGL(wino_input_kernel, dim3(Tp / 256 + (Tp % 256 != 0), p.REDp), dim3(256), 0, st,
                           static_cast<const float *>(in), V, p, n0, T, Tp);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        hipLaunchKernelGGL(wino_gemm_kernel, dim3(Tp / BN, p.Mp / BM, 16), dim3(256), 0, st, U, V, Mo, p.REDp, p.Mp, Tp);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        hipLaunchKernelGGL(wino_output_kernel<float>, dim3((T + 255) / 256, p.M), dim3(256), 0, st, Mo,
                           static_cast<float *>(out), p, n0, T, Tp);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace sn
