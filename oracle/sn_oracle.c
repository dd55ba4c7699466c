/*
 * sn_oracle.c -- TEST INFRASTRUCTURE, not part of the product.
 *
 * Plain fp64 CPU definitions of the layer math that the SuperNeurons runtime
 * (arXiv 1801.04380) delegates to its layer kernels: CONV forward / backward
 * (Sec. 3.5, Fig. 12 "f/d" steps), and the cheap-to-recompute layers ACT, BN
 * and POOL (Sec. 3.4).  The paper names these layers but does not print their
 * formulas; every function below is the standard textbook definition written
 * out with plain loops, nothing blocked, fused or reordered.
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may link
 * or call this file.  It shares no code with the HIP library.
 *
 * Layouts: x[N][C][H][W], w[K][C][R][S], y[N][K][P][Q], all row-major doubles,
 *   P = floor((H + 2*ph - R)/sh) + 1,   Q = floor((W + 2*pw - S)/sw) + 1.
 * OpenMP is used over the outermost independent loop only.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

#define IDX4(a, A, b, B, c, C, d, D) ((((size_t)(a) * (B) + (b)) * (C) + (c)) * (D) + (d))

int sn_oracle_out_dim(int in, int pad, int filt, int stride)
{
    int span = in + 2 * pad - filt;
    if (span < 0 || stride < 1) return 0;
    return span / stride + 1; /* floor: span >= 0 */
}

/* CONV forward (cross-correlation, no filter flip):
 *   y[n,k,p,q] = sum_{c,r,s} x[n,c,p*sh+r-ph,q*sw+s-pw] * w[k,c,r,s],
 * taps that fall outside the image contribute nothing. */
void sn_oracle_conv2d_fwd(const double *x, const double *w, double *y,
                          int N, int C, int H, int W, int K, int R, int S,
                          int sh, int sw, int ph, int pw)
{
    const int P = sn_oracle_out_dim(H, ph, R, sh), Q = sn_oracle_out_dim(W, pw, S, sw);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    double acc = 0.0;
                    for (int c = 0; c < C; ++c)
                        for (int r = 0; r < R; ++r)
                            for (int s = 0; s < S; ++s) {
                                int h = p * sh + r - ph, v = q * sw + s - pw;
                                if (h < 0 || h >= H || v < 0 || v >= W) continue;
                                acc += x[IDX4(n, N, c, C, h, H, v, W)] * w[IDX4(k, K, c, C, r, R, s, S)];
                            }
                    y[IDX4(n, N, k, K, p, P, q, Q)] = acc;
                }
}

/* CONV backward-data: the transpose of the forward map in x.  Written as the
 * scatter form of the same seven loops (dx[...] += dy * w), so it holds no
 * gather index algebra of its own. */
void sn_oracle_conv2d_bwd_data(const double *dy, const double *w, double *dx,
                               int N, int C, int H, int W, int K, int R, int S,
                               int sh, int sw, int ph, int pw)
{
    const int P = sn_oracle_out_dim(H, ph, R, sh), Q = sn_oracle_out_dim(W, pw, S, sw);
    memset(dx, 0, sizeof(double) * (size_t)N * C * H * W);
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    double g = dy[IDX4(n, N, k, K, p, P, q, Q)];
                    for (int c = 0; c < C; ++c)
                        for (int r = 0; r < R; ++r)
                            for (int s = 0; s < S; ++s) {
                                int h = p * sh + r - ph, v = q * sw + s - pw;
                                if (h < 0 || h >= H || v < 0 || v >= W) continue;
                                dx[IDX4(n, N, c, C, h, H, v, W)] += g * w[IDX4(k, K, c, C, r, R, s, S)];
                            }
                }
}

/* CONV backward-filter: dw[k,c,r,s] = sum_{n,p,q} dy[n,k,p,q] * x[n,c,p*sh+r-ph,q*sw+s-pw]. */
void sn_oracle_conv2d_bwd_filter(const double *x, const double *dy, double *dw,
                                 int N, int C, int H, int W, int K, int R, int S,
                                 int sh, int sw, int ph, int pw)
{
    const int P = sn_oracle_out_dim(H, ph, R, sh), Q = sn_oracle_out_dim(W, pw, S, sw);
    memset(dw, 0, sizeof(double) * (size_t)K * C * R * S);
#pragma omp parallel for schedule(static)
    for (int k = 0; k < K; ++k)
        for (int n = 0; n < N; ++n)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    double g = dy[IDX4(n, N, k, K, p, P, q, Q)];
                    for (int c = 0; c < C; ++c)
                        for (int r = 0; r < R; ++r)
                            for (int s = 0; s < S; ++s) {
                                int h = p * sh + r - ph, v = q * sw + s - pw;
                                if (h < 0 || h >= H || v < 0 || v >= W) continue;
                                dw[IDX4(k, K, c, C, r, R, s, S)] += g * x[IDX4(n, N, c, C, h, H, v, W)];
                            }
                }
}

/* Single-output versions for spot checks on tensors too large for the full
 * loops.  Each is the same definition restricted to one output element. */
double sn_oracle_conv2d_fwd_at(const double *x, const double *w,
                               int N, int C, int H, int W, int K, int R, int S,
                               int sh, int sw, int ph, int pw, int n, int k, int p, int q)
{
    double acc = 0.0;
    for (int c = 0; c < C; ++c)
        for (int r = 0; r < R; ++r)
            for (int s = 0; s < S; ++s) {
                int h = p * sh + r - ph, v = q * sw + s - pw;
                if (h < 0 || h >= H || v < 0 || v >= W) continue;
                acc += x[IDX4(n, N, c, C, h, H, v, W)] * w[IDX4(k, K, c, C, r, R, s, S)];
            }
    return acc;
}

/* dx at one (n,c,h,v): walk every forward term (k,p,q,r,s) and keep the ones
 * whose input pixel is the requested one -- the scatter form, filtered. */
double sn_oracle_conv2d_bwd_data_at(const double *dy, const double *w,
                                    int N, int C, int H, int W, int K, int R, int S,
                                    int sh, int sw, int ph, int pw, int n, int c, int h, int v)
{
    const int P = sn_oracle_out_dim(H, ph, R, sh), Q = sn_oracle_out_dim(W, pw, S, sw);
    double acc = 0.0;
    for (int k = 0; k < K; ++k)
        for (int p = 0; p < P; ++p)
            for (int q = 0; q < Q; ++q)
                for (int r = 0; r < R; ++r)
                    for (int s = 0; s < S; ++s)
                        if (p * sh + r - ph == h && q * sw + s - pw == v)
                            acc += dy[IDX4(n, N, k, K, p, P, q, Q)] * w[IDX4(k, K, c, C, r, R, s, S)];
    return acc;
}

double sn_oracle_conv2d_bwd_filter_at(const double *x, const double *dy,
                                      int N, int C, int H, int W, int K, int R, int S,
                                      int sh, int sw, int ph, int pw, int k, int c, int r, int s)
{
    const int P = sn_oracle_out_dim(H, ph, R, sh), Q = sn_oracle_out_dim(W, pw, S, sw);
    double acc = 0.0;
    for (int n = 0; n < N; ++n)
        for (int p = 0; p < P; ++p)
            for (int q = 0; q < Q; ++q) {
                int h = p * sh + r - ph, v = q * sw + s - pw;
                if (h < 0 || h >= H || v < 0 || v >= W) continue;
                acc += dy[IDX4(n, N, k, K, p, P, q, Q)] * x[IDX4(n, N, c, C, h, H, v, W)];
            }
    return acc;
}

/* Lists of output elements, for structured samples of tensors too large for the full loops:
 * out[i] = the output element at coords[4*i .. 4*i+3], in the index order of the matching _at
 * function.  Forward and backward-filter call the single-output definitions above.  For
 * backward-data the filtered walk over every (k,p,q,r,s) costs K*P*Q*R*S per element, so the
 * list version solves p*sh + r - ph = h for p (and likewise q) per tap instead of testing every
 * p; it is pinned against the scatter form on strided and padded shapes by the CPU tests. */
void sn_oracle_conv2d_fwd_points(const double *x, const double *w,
                                 int N, int C, int H, int W, int K, int R, int S,
                                 int sh, int sw, int ph, int pw,
                                 const int32_t *coords, size_t npts, double *out)
{
#pragma omp parallel for schedule(dynamic, 64)
    for (size_t i = 0; i < npts; ++i)
        out[i] = sn_oracle_conv2d_fwd_at(x, w, N, C, H, W, K, R, S, sh, sw, ph, pw,
                                         coords[4 * i], coords[4 * i + 1], coords[4 * i + 2], coords[4 * i + 3]);
}

void sn_oracle_conv2d_bwd_data_points(const double *dy, const double *w,
                                      int N, int C, int H, int W, int K, int R, int S,
                                      int sh, int sw, int ph, int pw,
                                      const int32_t *coords, size_t npts, double *out)
{
    const int P = sn_oracle_out_dim(H, ph, R, sh), Q = sn_oracle_out_dim(W, pw, S, sw);
#pragma omp parallel for schedule(dynamic, 64)
    for (size_t i = 0; i < npts; ++i) {
        const int n = coords[4 * i], c = coords[4 * i + 1], h = coords[4 * i + 2], v = coords[4 * i + 3];
        double acc = 0.0;
        for (int k = 0; k < K; ++k)
            for (int r = 0; r < R; ++r) {
                const int th = h + ph - r;           /* = p * sh for the p that reaches row h through tap row r */
                if (th < 0 || th % sh != 0 || th / sh >= P) continue;
                for (int s = 0; s < S; ++s) {
                    const int tv = v + pw - s;
                    if (tv < 0 || tv % sw != 0 || tv / sw >= Q) continue;
                    acc += dy[IDX4(n, N, k, K, th / sh, P, tv / sw, Q)] * w[IDX4(k, K, c, C, r, R, s, S)];
                }
            }
        out[i] = acc;
    }
}

void sn_oracle_conv2d_bwd_filter_points(const double *x, const double *dy,
                                        int N, int C, int H, int W, int K, int R, int S,
                                        int sh, int sw, int ph, int pw,
                                        const int32_t *coords, size_t npts, double *out)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (size_t i = 0; i < npts; ++i)
        out[i] = sn_oracle_conv2d_bwd_filter_at(x, dy, N, C, H, W, K, R, S, sh, sw, ph, pw,
                                                coords[4 * i], coords[4 * i + 1], coords[4 * i + 2], coords[4 * i + 3]);
}

/* ACT (ReLU): y = x if x > 0 else 0; the gradient passes where x > 0 (strictly). */
void sn_oracle_relu_fwd(const double *x, double *y, size_t n)
{
    for (size_t i = 0; i < n; ++i) y[i] = x[i] > 0.0 ? x[i] : 0.0;
}

void sn_oracle_relu_bwd(const double *x, const double *dy, double *dx, size_t n)
{
    for (size_t i = 0; i < n; ++i) dx[i] = x[i] > 0.0 ? dy[i] : 0.0;
}

/* BN forward, training mode, one statistic per channel over (N,H,W):
 *   mu = sum(x)/M,  var = sum((x-mu)^2)/M  (biased, two passes),
 *   invstd = 1/sqrt(var+eps),  y = gamma*(x-mu)*invstd + beta. */
void sn_oracle_bn_fwd(const double *x, const double *gamma, const double *beta, double *y,
                      double *save_mean, double *save_invstd,
                      int N, int C, int H, int W, double eps)
{
    const size_t HW = (size_t)H * W;
    const double M = (double)N * (double)HW;
#pragma omp parallel for schedule(static)
    for (int c = 0; c < C; ++c) {
        double sum = 0.0;
        for (int n = 0; n < N; ++n)
            for (size_t i = 0; i < HW; ++i) sum += x[((size_t)n * C + c) * HW + i];
        double mu = sum / M, ss = 0.0;
        for (int n = 0; n < N; ++n)
            for (size_t i = 0; i < HW; ++i) {
                double d = x[((size_t)n * C + c) * HW + i] - mu;
                ss += d * d;
            }
        double invstd = 1.0 / sqrt(ss / M + eps);
        save_mean[c] = mu;
        save_invstd[c] = invstd;
        for (int n = 0; n < N; ++n)
            for (size_t i = 0; i < HW; ++i) {
                size_t j = ((size_t)n * C + c) * HW + i;
                y[j] = gamma[c] * (x[j] - mu) * invstd + beta[c];
            }
    }
}

/* BN backward, from the saved statistics, with xhat = (x-mu)*invstd:
 *   dbeta = sum(dy), dgamma = sum(dy*xhat),
 *   dx = gamma*invstd/M * (M*dy - dbeta - xhat*dgamma). */
void sn_oracle_bn_bwd(const double *x, const double *dy, const double *gamma,
                      const double *save_mean, const double *save_invstd,
                      double *dx, double *dgamma, double *dbeta,
                      int N, int C, int H, int W)
{
    const size_t HW = (size_t)H * W;
    const double M = (double)N * (double)HW;
#pragma omp parallel for schedule(static)
    for (int c = 0; c < C; ++c) {
        double mu = save_mean[c], is = save_invstd[c], db = 0.0, dg = 0.0;
        for (int n = 0; n < N; ++n)
            for (size_t i = 0; i < HW; ++i) {
                size_t j = ((size_t)n * C + c) * HW + i;
                db += dy[j];
                dg += dy[j] * (x[j] - mu) * is;
            }
        dbeta[c] = db;
        dgamma[c] = dg;
        for (int n = 0; n < N; ++n)
            for (size_t i = 0; i < HW; ++i) {
                size_t j = ((size_t)n * C + c) * HW + i;
                double xhat = (x[j] - mu) * is;
                dx[j] = gamma[c] * is / M * (M * dy[j] - db - xhat * dg);
            }
    }
}

/* POOL (max) forward.  The window is scanned row by row, left to right, and a
 * later element replaces the running maximum only if strictly greater: of
 * several equal maxima the first in row-major order wins.  Padding positions
 * are not part of the window.  idx is the flat position h*W + v of the chosen
 * element inside its (n,c) input plane. */
void sn_oracle_maxpool_fwd(const double *x, double *y, int32_t *idx,
                           int N, int C, int H, int W,
                           int kh, int kw, int sh, int sw, int ph, int pw)
{
    const int P = sn_oracle_out_dim(H, ph, kh, sh), Q = sn_oracle_out_dim(W, pw, kw, sw);
#pragma omp parallel for schedule(static)
    for (int nc = 0; nc < N * C; ++nc) {
        const double *xp = x + (size_t)nc * H * W;
        for (int p = 0; p < P; ++p)
            for (int q = 0; q < Q; ++q) {
                int best = -1;
                double bv = 0.0;
                for (int r = 0; r < kh; ++r)
                    for (int s = 0; s < kw; ++s) {
                        int h = p * sh + r - ph, v = q * sw + s - pw;
                        if (h < 0 || h >= H || v < 0 || v >= W) continue;
                        double val = xp[(size_t)h * W + v];
                        if (best < 0 || val > bv) { best = h * W + v; bv = val; }
                    }
                y[((size_t)nc * P + p) * Q + q] = bv;
                idx[((size_t)nc * P + p) * Q + q] = best;
            }
    }
}

/* POOL backward: the transpose of the gather; overlapping windows add up. */
void sn_oracle_maxpool_bwd(const double *dy, const int32_t *idx, double *dx,
                           int N, int C, int H, int W, int P, int Q)
{
    memset(dx, 0, sizeof(double) * (size_t)N * C * H * W);
#pragma omp parallel for schedule(static)
    for (int nc = 0; nc < N * C; ++nc)
        for (int i = 0; i < P * Q; ++i)
            dx[(size_t)nc * H * W + idx[(size_t)nc * P * Q + i]] += dy[(size_t)nc * P * Q + i];
}

/* LRN across channels (the LRN1 / LRN2 layers of the paper's AlexNet example, Sec. 4; the paper
 * prints no formula, this is the normalisation of the AlexNet publication with the window's
 * alpha divided by the window size, as the cuDNN call the paper's runtime makes does):
 *   s[n,c,h,w] = k + (alpha / size) * sum_{j = c - size/2 .. c + size/2, 0 <= j < C} x[n,j,h,w]^2,
 *   y = x * s^(-beta).
 * size is odd; channels outside [0, C) contribute nothing. */
static double lrn_scale(const double *x, int C, int HW, size_t base, int c, int size, double alpha, double k)
{
    const int half = size / 2;
    double acc = 0.0;
    for (int j = c - half; j <= c + half; ++j) {
        if (j < 0 || j >= C) continue;
        const double v = x[base + (size_t)j * HW];
        acc += v * v;
    }
    return k + alpha / size * acc;
}

void sn_oracle_lrn_fwd(const double *x, double *y, int N, int C, int H, int W,
                       int size, double alpha, double beta, double k)
{
    const int HW = H * W;
    for (int n = 0; n < N; ++n)
        for (int i = 0; i < HW; ++i) {
            const size_t base = (size_t)n * C * HW + i;
            for (int c = 0; c < C; ++c)
                y[base + (size_t)c * HW] = x[base + (size_t)c * HW] * pow(lrn_scale(x, C, HW, base, c, size, alpha, k), -beta);
        }
}

/* LRN backward, the derivative of the above: y_j depends on x_c for every j whose window holds c,
 *   dx_c = dy_c * s_c^(-beta)
 *          - (2 * alpha * beta / size) * x_c * sum_{j: |j - c| <= size/2, 0 <= j < C} dy_j * x_j * s_j^(-beta-1). */
void sn_oracle_lrn_bwd(const double *x, const double *dy, double *dx, int N, int C, int H, int W,
                       int size, double alpha, double beta, double k)
{
    const int HW = H * W, half = size / 2;
    for (int n = 0; n < N; ++n)
        for (int i = 0; i < HW; ++i) {
            const size_t base = (size_t)n * C * HW + i;
            for (int c = 0; c < C; ++c) {
                const size_t e = base + (size_t)c * HW;
                double acc = 0.0;
                for (int j = c - half; j <= c + half; ++j) {
                    if (j < 0 || j >= C) continue;
                    const size_t ej = base + (size_t)j * HW;
                    acc += dy[ej] * x[ej] * pow(lrn_scale(x, C, HW, base, j, size, alpha, k), -beta - 1.0);
                }
                dx[e] = dy[e] * pow(lrn_scale(x, C, HW, base, c, size, alpha, k), -beta)
                        - 2.0 * alpha * beta / size * x[e] * acc;
            }
        }
}
