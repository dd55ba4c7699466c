// Explicit unfolding for the IM2COL_GEMM algorithm (the workspace-hungry
// member of the algorithm menu of Sec. 3.5).  Pure copies, HBM-bound.
//
// im2col writes, for each image of the pass, the matrix col[C*R*S][P*Q]: row
// (c,r,s) holds x[n,c,p*sh+r-ph,q*sw+s-pw] for every output pixel, 0 outside
// the image.  In this layout a pass over `nimg` images is an NCHW tensor
// [nimg][C*R*S][P][Q], so the GEMM over it is a 1x1 stride-1 convolution and
// runs on the same implicit-GEMM kernels as everything else.
// col2im folds the column gradient back in gather form (each dx element adds
// the at most R*S column entries that unfolded from it): no atomics, fixed order.
#include "sn_internal.h"

namespace sn {
namespace {

template <typename T>
__global__ void __launch_bounds__(256)
im2col_kernel(const T *__restrict__ x, T *__restrict__ col, ConvGeom g, int n0)
{
    const int PQ = g.P * g.Q;
    const int pq = blockIdx.x * 256 + threadIdx.x;
    if (pq >= PQ) return;
    const int row = blockIdx.y;  // (c,r,s)
    const int i = blockIdx.z;
    const int RS = g.R * g.S;
    const int c = row / RS, rs = row - c * RS, r = rs / g.S, s = rs - r * g.S;
    const int p = pq / g.Q, q = pq - p * g.Q;
    const int h = p * g.sh + r - g.ph, v = q * g.sw + s - g.pw;
    T val = (T)0;
    if ((unsigned)h < (unsigned)g.H && (unsigned)v < (unsigned)g.W)
        val = x[(((long long)(n0 + i) * g.C + c) * g.H + h) * g.W + v];
    col[((long long)i * gridDim.y + row) * PQ + pq] = val;
}

template <typename TOut>
__global__ void __launch_bounds__(256)
col2im_kernel(const float *__restrict__ dcol, TOut *__restrict__ dx, ConvGeom g, int n0)
{
    const int HW = g.H * g.W;
    const int hw = blockIdx.x * 256 + threadIdx.x;
    if (hw >= HW) return;
    const int c = blockIdx.y, i = blockIdx.z;
    const int h = hw / g.W, v = hw - h * g.W;
    const int PQ = g.P * g.Q, RS = g.R * g.S;
    const float *base = dcol + ((long long)i * g.C * RS + (long long)c * RS) * PQ;
    float acc = 0.f;
    for (int r = 0; r < g.R; ++r) {
        const int hp = h + g.ph - r;
        if (hp < 0) break;
        const int p = hp / g.sh;
        if (p * g.sh != hp || p >= g.P) continue;
        for (int s = 0; s < g.S; ++s) {
            const int vq = v + g.pw - s;
            if (vq < 0) break;
            const int q = vq / g.sw;
            if (q * g.sw != vq || q >= g.Q) continue;
            acc += base[(long long)(r * g.S + s) * PQ + p * g.Q + q];
        }
    }
    const long long off = ((long long)(n0 + i) * g.C + c) * HW + hw;
    if (sizeof(TOut) == 2) reinterpret_cast<bf16_t *>(dx)[off] = f32_to_bf16(acc);
    else reinterpret_cast<float *>(dx)[off] = acc;
}

}  // namespace

hipError_t launch_im2col(const void *x, void *col, const ConvGeom &g, int n0, int nimg, hipStream_t st)
{
    const int PQ = g.P * g.Q;
    dim3 grid((PQ + 255) / 256, g.C * g.R * g.S, nimg), block(256);
    if (g.in_bf16)
        hipLaunchKernelGGL(im2col_kernel<bf16_t>, grid, block, 0, st, (const bf16_t *)x, (bf16_t *)col, g, n0);
    else
        hipLaunchKernelGGL(im2col_kernel<float>, grid, block, 0, st, (const float *)x, (float *)col, g, n0);
    return hipGetLastError();
}

hipError_t launch_col2im(const float *dcol, void *dx, const ConvGeom &g, int n0, int nimg, hipStream_t st)
{
    const int HW = g.H * g.W;
    dim3 grid((HW + 255) / 256, g.C, nimg), block(256);
    if (g.out_bf16)
        hipLaunchKernelGGL(col2im_kernel<bf16_t>, grid, block, 0, st, dcol, (bf16_t *)dx, g, n0);
    else
        hipLaunchKernelGGL(col2im_kernel<float>, grid, block, 0, st, dcol, (float *)dx, g, n0);
    return hipGetLastError();
}

}  // namespace sn
