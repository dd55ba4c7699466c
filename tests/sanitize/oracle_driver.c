/* Runs every function of oracle/sn_oracle.c on small shapes, edge cases included (1x1 tensors,
 * strides larger than the filter, padding, ragged sizes), for the AddressSanitizer / UBSan build of
 * the CPU test suite.  Exit status 0 = every call returned and the sanitizers found nothing. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int sn_oracle_out_dim(int, int, int, int);
void sn_oracle_conv2d_fwd(const double *, const double *, double *, int, int, int, int, int, int, int, int, int, int, int);
void sn_oracle_conv2d_bwd_data(const double *, const double *, double *, int, int, int, int, int, int, int, int, int, int, int);
void sn_oracle_conv2d_bwd_filter(const double *, const double *, double *, int, int, int, int, int, int, int, int, int, int, int);
double sn_oracle_conv2d_fwd_at(const double *, const double *, int, int, int, int, int, int, int, int, int, int, int, int, int, int, int);
double sn_oracle_conv2d_bwd_data_at(const double *, const double *, int, int, int, int, int, int, int, int, int, int, int, int, int, int, int);
double sn_oracle_conv2d_bwd_filter_at(const double *, const double *, int, int, int, int, int, int, int, int, int, int, int, int, int, int, int);
void sn_oracle_conv2d_fwd_points(const double *, const double *, int, int, int, int, int, int, int, int, int, int, int, const int32_t *, size_t, double *);
void sn_oracle_conv2d_bwd_data_points(const double *, const double *, int, int, int, int, int, int, int, int, int, int, int, const int32_t *, size_t, double *);
void sn_oracle_conv2d_bwd_filter_points(const double *, const double *, int, int, int, int, int, int, int, int, int, int, int, const int32_t *, size_t, double *);
void sn_oracle_relu_fwd(const double *, double *, size_t);
void sn_oracle_relu_bwd(const double *, const double *, double *, size_t);
void sn_oracle_bn_fwd(const double *, const double *, const double *, double *, double *, double *, int, int, int, int, double);
void sn_oracle_bn_bwd(const double *, const double *, const double *, const double *, const double *, double *, double *, double *, int, int, int, int);
void sn_oracle_maxpool_fwd(const double *, double *, int32_t *, int, int, int, int, int, int, int, int, int, int);
void sn_oracle_maxpool_bwd(const double *, const int32_t *, double *, int, int, int, int, int, int);
void sn_oracle_lrn_fwd(const double *, double *, int, int, int, int, int, double, double, double);
void sn_oracle_lrn_bwd(const double *, const double *, double *, int, int, int, int, int, double, double, double);

static double *fill(size_t n, unsigned seed)
{
    double *p = malloc(sizeof(double) * (n ? n : 1));
    for (size_t i = 0; i < n; ++i) {
        seed = seed * 1664525u + 1013904223u;
        p[i] = (double)(int)(seed >> 20) / 2048.0 - 1.0;
    }
    return p;
}

static void conv_case(int N, int C, int H, int W, int K, int R, int S, int sh, int sw, int ph, int pw)
{
    const int P = sn_oracle_out_dim(H, ph, R, sh), Q = sn_oracle_out_dim(W, pw, S, sw);
    if (P < 1 || Q < 1) return;
    const size_t nx = (size_t)N * C * H * W, nw = (size_t)K * C * R * S, ny = (size_t)N * K * P * Q;
    double *x = fill(nx, 1), *w = fill(nw, 2), *dy = fill(ny, 3);
    double *y = malloc(sizeof(double) * ny), *dx = malloc(sizeof(double) * nx), *dw = malloc(sizeof(double) * nw);
    sn_oracle_conv2d_fwd(x, w, y, N, C, H, W, K, R, S, sh, sw, ph, pw);
    sn_oracle_conv2d_bwd_data(dy, w, dx, N, C, H, W, K, R, S, sh, sw, ph, pw);
    sn_oracle_conv2d_bwd_filter(x, dy, dw, N, C, H, W, K, R, S, sh, sw, ph, pw);
    /* the corners through the single-element and the list versions */
    int32_t cy[8] = {0, 0, 0, 0, N - 1, K - 1, P - 1, Q - 1}, cx[8] = {0, 0, 0, 0, N - 1, C - 1, H - 1, W - 1};
    int32_t cw[8] = {0, 0, 0, 0, K - 1, C - 1, R - 1, S - 1};
    double o[2];
    sn_oracle_conv2d_fwd_points(x, w, N, C, H, W, K, R, S, sh, sw, ph, pw, cy, 2, o);
    if (o[1] != sn_oracle_conv2d_fwd_at(x, w, N, C, H, W, K, R, S, sh, sw, ph, pw, N - 1, K - 1, P - 1, Q - 1)) exit(3);
    sn_oracle_conv2d_bwd_data_points(dy, w, N, C, H, W, K, R, S, sh, sw, ph, pw, cx, 2, o);
    (void)sn_oracle_conv2d_bwd_data_at(dy, w, N, C, H, W, K, R, S, sh, sw, ph, pw, N - 1, C - 1, H - 1, W - 1);
    sn_oracle_conv2d_bwd_filter_points(x, dy, N, C, H, W, K, R, S, sh, sw, ph, pw, cw, 2, o);
    if (o[1] != sn_oracle_conv2d_bwd_filter_at(x, dy, N, C, H, W, K, R, S, sh, sw, ph, pw, K - 1, C - 1, R - 1, S - 1)) exit(4);
    free(x); free(w); free(dy); free(y); free(dx); free(dw);
}

static void cheap_case(int N, int C, int H, int W, int kh, int kw, int sh, int sw, int ph, int pw, int lrn)
{
    const size_t n = (size_t)N * C * H * W;
    double *x = fill(n, 5), *g = fill(n, 6), *y = malloc(sizeof(double) * n), *dx = malloc(sizeof(double) * n);
    sn_oracle_relu_fwd(x, y, n);
    sn_oracle_relu_bwd(x, g, dx, n);
    double *gamma = fill(C, 7), *beta = fill(C, 8), *mean = malloc(sizeof(double) * C), *inv = malloc(sizeof(double) * C);
    double *dgamma = malloc(sizeof(double) * C), *dbeta = malloc(sizeof(double) * C);
    sn_oracle_bn_fwd(x, gamma, beta, y, mean, inv, N, C, H, W, 1e-5);
    sn_oracle_bn_bwd(x, g, gamma, mean, inv, dx, dgamma, dbeta, N, C, H, W);
    sn_oracle_lrn_fwd(x, y, N, C, H, W, lrn, 1e-4, 0.75, 2.0);
    sn_oracle_lrn_bwd(x, g, dx, N, C, H, W, lrn, 1e-4, 0.75, 2.0);
    const int P = sn_oracle_out_dim(H, ph, kh, sh), Q = sn_oracle_out_dim(W, pw, kw, sw);
    if (P >= 1 && Q >= 1) {
        const size_t no = (size_t)N * C * P * Q;
        double *p = malloc(sizeof(double) * no), *gp = fill(no, 9);
        int32_t *idx = malloc(sizeof(int32_t) * no);
        sn_oracle_maxpool_fwd(x, p, idx, N, C, H, W, kh, kw, sh, sw, ph, pw);
        sn_oracle_maxpool_bwd(gp, idx, dx, N, C, H, W, P, Q);
        free(p); free(gp); free(idx);
    }
    free(x); free(g); free(y); free(dx); free(gamma); free(beta); free(mean); free(inv); free(dgamma); free(dbeta);
}

int main(void)
{
    conv_case(1, 1, 1, 1, 1, 1, 1, 1, 1, 0, 0);
    conv_case(2, 3, 7, 9, 4, 3, 3, 1, 1, 1, 1);
    conv_case(1, 2, 8, 8, 3, 3, 3, 2, 2, 1, 1);
    conv_case(1, 3, 23, 19, 4, 11, 11, 4, 4, 0, 0);
    conv_case(2, 4, 9, 17, 3, 1, 7, 1, 1, 0, 3);
    conv_case(2, 2, 6, 5, 2, 2, 2, 3, 3, 0, 0);   /* stride beyond the filter: rows no window reads */
    conv_case(1, 2, 4, 4, 2, 3, 3, 1, 1, 2, 2);   /* padding as large as the filter allows */
    conv_case(1, 1, 5, 6, 1, 2, 3, 3, 2, 1, 2);
    cheap_case(1, 1, 1, 1, 1, 1, 1, 1, 0, 0, 1);
    cheap_case(2, 5, 7, 6, 3, 3, 2, 2, 0, 0, 5);
    cheap_case(3, 4, 8, 8, 2, 2, 2, 2, 0, 0, 3);
    cheap_case(2, 9, 5, 5, 3, 3, 2, 2, 1, 1, 9);
    cheap_case(1, 2, 6, 4, 3, 2, 1, 1, 1, 0, 5);
    puts("oracle driver: ok");
    return 0;
}
