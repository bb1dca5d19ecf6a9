/*
 * cgo_layers.c -- CPU oracle (test infrastructure only): the non-convolution
 * layers an AlexNet- or GoogLeNet-shaped iteration needs around its
 * convolutions (section 2.1: each iteration is a forward and a backward
 * propagation through the layers).  The paper leaves these to the stock
 * solver; each is written here from its usual definition.
 */
#include "cgo.h"
#include <math.h>
#include <stdlib.h>
#include <omp.h>

void cgo_relu_fwd(size_t n, const REAL *x, REAL *y)
{
    for (size_t i = 0; i < n; ++i) y[i] = x[i] > (REAL)0 ? x[i] : (REAL)0;
}

void cgo_relu_bwd(size_t n, const REAL *x, const REAL *dy, REAL *dx)
{
    for (size_t i = 0; i < n; ++i) dx[i] = x[i] > (REAL)0 ? dy[i] : (REAL)0;
}

int cgo_maxpool_out(int H, int k, int s, int p)
{
    int e = H + 2 * p - k;
    if (e < 0) return 0;
    int o = (e + s - 1) / s + 1;
    if ((o - 1) * s >= H + p) --o;   /* last window must start inside image+pad */
    return o;
}

void cgo_maxpool_fwd(int N, int C, int H, int W, int k, int s, int p,
                     const REAL *x, REAL *y, int32_t *argmax)
{
    const int OH = cgo_maxpool_out(H, k, s, p), OW = cgo_maxpool_out(W, k, s, p);
#pragma omp parallel for schedule(static)
    for (long nc = 0; nc < (long)N * C; ++nc) {
        const REAL *xp = x + (size_t)nc * H * W;
        for (int oh = 0; oh < OH; ++oh)
            for (int ow = 0; ow < OW; ++ow) {
                int best = -1;
                REAL bv = 0;
                for (int kh = 0; kh < k; ++kh) {
                    const int ih = oh * s - p + kh;
                    if (ih < 0 || ih >= H) continue;
                    for (int kw = 0; kw < k; ++kw) {
                        const int iw = ow * s - p + kw;
                        if (iw < 0 || iw >= W) continue;
                        const REAL val = xp[ih * W + iw];
                        if (best < 0 || val > bv) { best = ih * W + iw; bv = val; }
                    }
                }
                const size_t o = ((size_t)nc * OH + oh) * OW + ow;
                y[o] = bv;
                argmax[o] = best;
            }
    }
}

void cgo_maxpool_bwd(int N, int C, int H, int W, int k, int s, int p,
                     const REAL *dy, const int32_t *argmax, REAL *dx)
{
    const int OH = cgo_maxpool_out(H, k, s, p), OW = cgo_maxpool_out(W, k, s, p);
#pragma omp parallel for schedule(static)
    for (long nc = 0; nc < (long)N * C; ++nc) {
        double *acc = (double *)calloc((size_t)H * W, sizeof(double));
        for (int o = 0; o < OH * OW; ++o) {
            const int a = argmax[(size_t)nc * OH * OW + o];
            if (a >= 0) acc[a] += (double)dy[(size_t)nc * OH * OW + o];
        }
        for (int i = 0; i < H * W; ++i) dx[(size_t)nc * H * W + i] = (REAL)acc[i];
        free(acc);
    }
}

void cgo_lrn_fwd(int N, int C, int HW, int size, double alpha, double beta, double kappa,
                 const REAL *x, REAL *y, REAL *scale)
{
    const int half = (size - 1) / 2;
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int i = 0; i < HW; ++i) {
                double ss = 0.0;
                for (int cc = c - half; cc <= c - half + size - 1; ++cc) {
                    if (cc < 0 || cc >= C) continue;
                    const double xv = (double)x[((size_t)n * C + cc) * HW + i];
                    ss += xv * xv;
                }
                const double sc = kappa + (alpha / size) * ss;
                const size_t o = ((size_t)n * C + c) * HW + i;
                scale[o] = (REAL)sc;
                y[o] = (REAL)((double)x[o] * pow(sc, -beta));
            }
}

/* d/dx_c of sum_j dy_j x_j scale_j^-beta:
 *   dx_c = dy_c scale_c^-beta - (2 alpha beta / size) x_c sum_{j: c in window(j)} dy_j y_j / scale_j */
void cgo_lrn_bwd(int N, int C, int HW, int size, double alpha, double beta,
                 const REAL *x, const REAL *y, const REAL *scale, const REAL *dy, REAL *dx)
{
    const int half = (size - 1) / 2;
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int i = 0; i < HW; ++i) {
                const size_t o = ((size_t)n * C + c) * HW + i;
                double cross = 0.0;
                /* window(j) = [j-half, j-half+size-1] contains c  <=>  j in [c+half-size+1, c+half] */
                for (int j = c + half - size + 1; j <= c + half; ++j) {
                    if (j < 0 || j >= C) continue;
                    const size_t q = ((size_t)n * C + j) * HW + i;
                    cross += (double)dy[q] * (double)y[q] / (double)scale[q];
                }
                dx[o] = (REAL)((double)dy[o] * pow((double)scale[o], -beta) -
                               (2.0 * alpha * beta / size) * (double)x[o] * cross);
            }
}

void cgo_avgpool_fwd(int N, int C, int HW, const REAL *x, REAL *y)
{
    for (long nc = 0; nc < (long)N * C; ++nc) {
        double acc = 0.0;
        for (int i = 0; i < HW; ++i) acc += (double)x[(size_t)nc * HW + i];
        y[nc] = (REAL)(acc / HW);
    }
}

void cgo_avgpool_bwd(int N, int C, int HW, const REAL *dy, REAL *dx)
{
    for (long nc = 0; nc < (long)N * C; ++nc)
        for (int i = 0; i < HW; ++i) dx[(size_t)nc * HW + i] = (REAL)((double)dy[nc] / HW);
}

void cgo_fc_fwd(int B, int IN, int OUT, const REAL *x, const REAL *W, const REAL *bias, REAL *y)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < B; ++b)
        for (int o = 0; o < OUT; ++o) {
            double acc = bias ? (double)bias[o] : 0.0;
            for (int i = 0; i < IN; ++i) acc += (double)W[(size_t)o * IN + i] * (double)x[(size_t)b * IN + i];
            y[(size_t)b * OUT + o] = (REAL)acc;
        }
}

void cgo_fc_bwd_data(int B, int IN, int OUT, const REAL *dy, const REAL *W, REAL *dx)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < B; ++b)
        for (int i = 0; i < IN; ++i) {
            double acc = 0.0;
            for (int o = 0; o < OUT; ++o) acc += (double)dy[(size_t)b * OUT + o] * (double)W[(size_t)o * IN + i];
            dx[(size_t)b * IN + i] = (REAL)acc;
        }
}

void cgo_fc_bwd_weight(int B, int IN, int OUT, const REAL *x, const REAL *dy, REAL *dW, REAL *db)
{
#pragma omp parallel for schedule(static)
    for (int o = 0; o < OUT; ++o) {
        for (int i = 0; i < IN; ++i) {
            double acc = 0.0;
            for (int b = 0; b < B; ++b) acc += (double)dy[(size_t)b * OUT + o] * (double)x[(size_t)b * IN + i];
            dW[(size_t)o * IN + i] = (REAL)acc;
        }
        if (db) {
            double acc = 0.0;
            for (int b = 0; b < B; ++b) acc += (double)dy[(size_t)b * OUT + o];
            db[o] = (REAL)acc;
        }
    }
}

void cgo_dropout(size_t n, double p, const uint8_t *mask, const REAL *x, REAL *y)
{
    const double f = 1.0 / (1.0 - p);
    for (size_t i = 0; i < n; ++i) y[i] = mask[i] ? (REAL)((double)x[i] * f) : (REAL)0;
}

void cgo_softmax_ce(int B, int C, const REAL *z, const int32_t *labels, REAL *loss, REAL *dz)
{
    double total = 0.0;
    for (int b = 0; b < B; ++b) {
        const REAL *zb = z + (size_t)b * C;
        double mx = (double)zb[0];
        for (int c = 1; c < C; ++c) if ((double)zb[c] > mx) mx = (double)zb[c];
        double se = 0.0;
        for (int c = 0; c < C; ++c) se += exp((double)zb[c] - mx);
        const double lse = mx + log(se);
        total += lse - (double)zb[labels[b]];
        if (dz)
            for (int c = 0; c < C; ++c) {
                const double pr = exp((double)zb[c] - lse);
                dz[(size_t)b * C + c] = (REAL)((pr - (c == labels[b] ? 1.0 : 0.0)) / B);
            }
    }
    *loss = (REAL)(total / B);
}
