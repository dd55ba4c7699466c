// Internal declarations shared by the host dispatcher and the HIP kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "sn.h"

namespace sn {

// Geometry of one CONV step, derived once on the host.
struct ConvGeom {
    int N, C, H, W, K, R, S, sh, sw, ph, pw, P, Q;
    int in_bf16;   // 1: x, w, dy are bf16; 0: fp32
    int out_bf16;  // 1: y / dx stored as bf16; 0: fp32
};

typedef unsigned short bf16_t;

__host__ __device__ inline float bf16_to_f32(bf16_t v)
{
    union { uint32_t u; float f; } c;
    c.u = (uint32_t)v << 16;
    return c.f;
}

// fp32 -> bf16, round to nearest, ties to even; NaN stays NaN.
__host__ __device__ inline bf16_t f32_to_bf16(float f)
{
    union { uint32_t u; float f; } c;
    c.f = f;
    if ((c.u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((c.u >> 16) | 0x40u);
    c.u += 0x7fffu + ((c.u >> 16) & 1u);
    return (bf16_t)(c.u >> 16);
}

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ---- launchers implemented in the .hip files (all enqueue on `st`, return hipError_t) ----

// Fallback implicit GEMM for any geometry and either dtype.  For backward-filter
// `splits` > 1 spreads the (n,p,q) sum over that many workgroup slices: with
// partial == nullptr the slices combine into dw with atomics (dw must be zeroed
// first, which the launcher does); otherwise slice z writes its own
// partial[z][K*C*R*S] and a reduction in slice order follows, which adds to the
// existing dw when `accumulate` is set.
hipError_t launch_generic_fwd(const void *x, const void *w, void *y, const ConvGeom &g, hipStream_t st);
hipError_t launch_generic_bwd_data(const void *dy, const void *w, void *dx, const ConvGeom &g, hipStream_t st);
hipError_t launch_generic_bwd_filter(const void *x, const void *dy, float *dw, const ConvGeom &g,
                                     int splits, float *partial, bool accumulate, hipStream_t st);
int generic_bwd_filter_splits(const ConvGeom &g);

// Stride-1 bf16 fast path (forward, or backward-data when bwd_data is set).
// `packed` = workspace for the re-laid-out filter (tile_conv_packed_bytes), or
// nullptr to gather the filter from the KCRS tensor inside the kernel.
bool tile_conv_supported(const ConvGeom &g, bool bwd_data);
size_t tile_conv_packed_bytes(const ConvGeom &g, bool bwd_data);
// stats (forward only, may be null): room for tile_conv_stats_tiles(...) * K * 3 floats, where every
// pixel tile leaves (count, mean, sum of squared deviations) of its outputs per channel, for
// launch_bn_finalize_tiles.
hipError_t launch_tile_conv(const void *in, const void *w, void *out, const ConvGeom &g, bool bwd_data,
                            void *packed, hipStream_t st, float *stats = nullptr);
int tile_conv_stats_tiles(const ConvGeom &g, bool staged, bool in_aligned16);

// Stride-1 bf16 backward-filter fast path.  partial == nullptr: the slices of the
// (n,p,q) sum combine with atomics into a zero-filled dw; otherwise slice z writes
// partial[z][K*C*R*S] (tile_wgrad_slices of them) and a fixed-order reduction follows.
// cap > 0 (with partial): at most that many slices, where the kernel that takes the shape can work with
// fewer (tile_wgrad_cappable: the row-stationary one) -- a workspace that holds fewer partial sums.
bool tile_wgrad_supported(const ConvGeom &g);
bool tile_wgrad_cappable(const ConvGeom &g);
int tile_wgrad_slices(const ConvGeom &g, int cap = 0);
hipError_t launch_tile_wgrad(const void *x, const void *dy, float *dw, const ConvGeom &g, float *partial,
                             hipStream_t st, int cap = 0);

// The row-stationary variant for 3x3 / 1x1 filters (same contract); launch_tile_wgrad prefers it.
bool rows_wgrad_supported(const ConvGeom &g);
int rows_wgrad_slices(const ConvGeom &g, int cap = 0);
hipError_t launch_rows_wgrad(const void *x, const void *dy, float *dw, const ConvGeom &g, float *partial,
                             hipStream_t st, int cap = 0);

// Few input channels (C*R*S <= 32, bf16 operands, any stride and padding; conv_smallc.hip): forward
// without workspace, optionally leaving smallc_fwd_stats_tiles(g) * K (count, mean, M2) triples in
// `stats` for launch_bn_finalize_tiles; backward-filter with the contract of launch_rows_wgrad
// (smallc_wgrad_slices slices).
bool smallc_supported(const ConvGeom &g);
int smallc_fwd_stats_tiles(const ConvGeom &g);
hipError_t launch_smallc_fwd(const void *x, const void *w, void *y, const ConvGeom &g, hipStream_t st, float *stats);
int smallc_wgrad_slices(const ConvGeom &g);
hipError_t launch_smallc_wgrad(const void *x, const void *dy, float *dw, const ConvGeom &g, float *partial,
                               hipStream_t st);

// 1x1 / stride-1 / unpadded layers with bf16 operands and channel counts that are multiples of 8
// (conv_pointwise.hip): forward or backward-data without workspace; launch_tile_conv prefers it
// when no statistics are asked for.
bool pointwise_supported(const ConvGeom &g, bool bwd_data);
hipError_t launch_pointwise(const void *in, const void *w, void *out, const ConvGeom &g, bool bwd_data, hipStream_t st);

// Forward of any filter, stride and padding (bf16, C a multiple of 16, K of 8) as a matrix product over
// (tap, channel) whose input operand is gathered pixel by pixel straight from x (conv_pointwise.hip);
// `packed`: gather_conv_packed_bytes for the filter re-laid out [k][tap][c], written by the call.
bool gather_conv_supported(const ConvGeom &g);
size_t gather_conv_packed_bytes(const ConvGeom &g);
hipError_t launch_gather_conv_fwd(const void *x, const void *w, void *y, const ConvGeom &g, void *packed, hipStream_t st);

// Backward-filter of the same layers on the smallest planes (8 to 64 pixels), any channel counts;
// contract of launch_rows_wgrad (pointwise_wgrad_slices slices).  launch_tile_wgrad prefers it.
bool pointwise_wgrad_supported(const ConvGeom &g);
int pointwise_wgrad_slices(const ConvGeom &g);
hipError_t launch_pointwise_wgrad(const void *x, const void *dy, float *dw, const ConvGeom &g, float *partial,
                                  hipStream_t st);
// Backward-filter of 1x1 layers with a stride or padding (up to 1024 output channels), x gathered under each
// output pixel (conv_pointwise.hip): runs where neither the stride-1 kernels nor the few-channel kernel apply.
bool gather_wgrad_supported(const ConvGeom &g);
int gather_wgrad_slices(const ConvGeom &g);
hipError_t launch_gather_wgrad(const void *x, const void *dy, float *dw, const ConvGeom &g, float *partial, hipStream_t st);

hipError_t launch_fill_zero(float *p, size_t n, hipStream_t st);
// dw[i] = (accumulate ? dw[i] : 0) + sum_z partial[z][i], z ascending.
hipError_t launch_reduce_partials(const float *partial, float *dw, size_t n, int splits, bool accumulate,
                                  hipStream_t st);

// im2col: col[i][C*R*S][P*Q] for images n0 .. n0+nimg-1 (i = n - n0), zero where
// the tap falls outside the image.  Element type as the input.
hipError_t launch_im2col(const void *x, void *col, const ConvGeom &g, int n0, int nimg, hipStream_t st);
// col2im: dx[n][c][h][v] = sum over taps of dcol[i][(c,r,s)][p][q]; dcol is fp32.
hipError_t launch_col2im(const float *dcol, void *dx, const ConvGeom &g, int n0, int nimg, hipStream_t st);

// Phase decomposition of a strided convolution (conv_phase.hip): which residues of the rows and
// columns occur as phases, and the geometry of the phase planes.  row_phase[i] = residue of the
// i-th row phase (na of them), row_index[a] = its number or -1; columns likewise (nb);
// nphases = na * nb, phase number = row number * nb + column number.  The inner filter is
// Ri x Si (1x1, or 3x3 with tap (d, e) at [d + center_r][e + center_c], the inner padding being the
// centres: 1 where the offsets are within -1 .. 1, 0 where they are 0 .. 2); planes are Hs x Ws.
struct PhaseMap {
    int sh, sw, ph, pw;
    int na, nb, nphases;
    int row_phase[8], col_phase[8], row_index[8], col_index[8];
    int Ri, Si, center_r, center_c;
    int Hs, Ws;
};
hipError_t launch_phase_split(const void *x, void *xs, const PhaseMap &m, const ConvGeom &g, hipStream_t st);
hipError_t launch_phase_filter(const void *w, void *wp, const PhaseMap &m, const ConvGeom &g, hipStream_t st);
hipError_t launch_phase_merge(const void *dxs, void *dx, const PhaseMap &m, const ConvGeom &g, hipStream_t st);
hipError_t launch_phase_dw(const float *dwp, float *dw, const PhaseMap &m, const ConvGeom &g, hipStream_t st);

// Winograd F(2x2, 3x3), fp32, 3x3 stride-1 forward / backward-data (conv_winograd.hip).
// winograd_pass_tiles: 2x2 output tiles one pass handles with ws_bytes of workspace (0: does not fit).
bool winograd_supported(const ConvGeom &g, bool bwd_data);
void winograd_bytes(const ConvGeom &g, bool bwd_data, size_t *min_b, size_t *pref_b);
long long winograd_pass_tiles(const ConvGeom &g, bool bwd_data, size_t ws_bytes);
hipError_t launch_winograd(const void *in, const void *w, void *out, const ConvGeom &g, bool bwd_data, void *ws,
                           size_t ws_bytes, hipStream_t st);

// Cheap layers.
hipError_t launch_relu_fwd(const void *x, void *y, size_t n, int bf16, hipStream_t st);
hipError_t launch_relu_bwd(const void *x, const void *dy, void *dx, size_t n, int bf16, hipStream_t st);
// relu != 0: the ReLU that follows BN is applied in the same pass (y = max(BN(x), 0)).
hipError_t launch_bn_fwd(const void *x, const float *gamma, const float *beta, void *y, float *mean,
                         float *invstd, int N, int C, int HW, float eps, int bf16, int relu, hipStream_t st);
// relu_beta != nullptr: the layer was BN + ReLU with this beta; dy is first passed through the
// ReLU backward gate, which is re-derived from x (the forward pass's own expression) and not read.
hipError_t launch_bn_bwd(const void *x, const void *dy, const float *relu_beta, const float *gamma, const float *mean,
                         const float *invstd, void *dx, float *dgamma, float *dbeta, int N, int C,
                         int HW, int bf16, hipStream_t st, const void *pool_g = nullptr,
                         const int32_t *pool_idx = nullptr, int pool_W = 0);
// BN + ReLU + 2x2 / stride-2 max-pool without padding, H and W even: the statistics of launch_bn_fwd,
// then pooled values and winner indices as launch_maxpool_fwd gives them on the BN + ReLU output,
// which is not written.  idx doubles as scratch.  bn_relu_pool2_vb: bytes per access along a row,
// 0 if W does not allow any.  Its backward is launch_bn_bwd with dy == nullptr and the pooled
// gradient, the indices and W in the pool_* arguments (relu_beta set).
int bn_relu_pool2_vb(int W, int bf16);
// The last pass of the two calls above alone, from statistics the caller has.
hipError_t launch_bn_apply(const void *x, const float *gamma, const float *beta, const float *mean,
                           const float *invstd, void *y, int N, int C, int HW, int bf16, int relu, hipStream_t st);
hipError_t launch_bn_relu_pool2_apply(const void *x, const float *gamma, const float *beta, const float *mean,
                                      const float *invstd, void *pooled, int32_t *idx, int N, int C, int H, int W,
                                      int bf16, hipStream_t st);
// Statistics alone: from the per-tile triples of launch_tile_conv (part: C * ntiles * 3 floats), or by
// a pass over x with bn_stats_scratch_bytes of scratch.
hipError_t launch_bn_finalize_tiles(const float *part, int C, int ntiles, float *mean, float *invstd, float eps,
                                    hipStream_t st);
size_t bn_stats_scratch_bytes(int N, int C, int HW);
hipError_t launch_bn_stats(const void *x, float *scratch, float *mean, float *invstd, int N, int C, int HW, float eps,
                           int bf16, hipStream_t st);
hipError_t launch_bn_relu_pool2_fwd(const void *x, const float *gamma, const float *beta, void *pooled, int32_t *idx,
                                    float *mean, float *invstd, int N, int C, int H, int W, float eps, int bf16,
                                    hipStream_t st);
// LRN across channels, size odd and at most 9; dy == nullptr: forward into out, else backward into out.
// relu != 0: the ReLU before the LRN in the same pass (forward: LRN of max(x, 0); backward: dx through both).
hipError_t launch_lrn(const void *x, const void *dy, void *out, int N, int C, int HW, int size, float alpha,
                      float beta, float k, int bf16, hipStream_t st, int relu = 0);
hipError_t launch_maxpool_fwd(const void *x, void *y, int32_t *idx, int NC, int H, int W, int P, int Q,
                              int kh, int kw, int sh, int sw, int ph, int pw, int bf16, hipStream_t st);
hipError_t launch_maxpool_bwd(const void *dy, const int32_t *idx, void *dx, int NC, int H, int W, int P,
                              int Q, int kh, int kw, int sh, int sw, int ph, int pw, int bf16,
                              hipStream_t st);

}  // namespace sn
