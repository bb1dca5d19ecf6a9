/*
 * cgo_conv.c -- CPU oracle (test infrastructure only): direct convolution and
 * its two adjoints, written as the definition.  The paper names these only as
 * the forward / backward propagation of each layer (section 2.1) and the
 * "compute local gradient" turn of Fig. 3; the formulas are the standard
 * cross-correlation of the Caffe solver it builds on.
 */
#include "cgo.h"
#include <stdlib.h>
#include <string.h>
#include <omp.h>

int cgo_num_threads(void) { return omp_get_max_threads(); }
void cgo_set_num_threads(int n) { if (n > 0) omp_set_num_threads(n); }

int cgo_conv_out_shape(const cgo_conv_desc *d, int *OH, int *OW)
{
    if (!d || d->N <= 0 || d->C <= 0 || d->H <= 0 || d->W <= 0 || d->M <= 0 ||
        d->KH <= 0 || d->KW <= 0 || d->stride_h <= 0 || d->stride_w <= 0 ||
        d->pad_h < 0 || d->pad_w < 0 || d->groups <= 0)
        return -1;
    if (d->C % d->groups || d->M % d->groups) return -1;
    int eh = d->H + 2 * d->pad_h - d->KH, ew = d->W + 2 * d->pad_w - d->KW;
    if (eh < 0 || ew < 0) return -1;
    if (OH) *OH = eh / d->stride_h + 1;
    if (OW) *OW = ew / d->stride_w + 1;
    return 0;
}

int cgo_conv_fwd(const cgo_conv_desc *d, const REAL *x, const REAL *w,
                 const REAL *bias, REAL *y)
{
    int OH, OW;
    if (cgo_conv_out_shape(d, &OH, &OW)) return -1;
    const int G = d->groups, Cg = d->C / G, Mg = d->M / G;
    const int H = d->H, W = d->W, KH = d->KH, KW = d->KW;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < d->N; ++n)
        for (int m = 0; m < d->M; ++m) {
            const int g = m / Mg;
            for (int oh = 0; oh < OH; ++oh)
                for (int ow = 0; ow < OW; ++ow) {
                    double acc = bias ? (double)bias[m] : 0.0;
                    for (int c = 0; c < Cg; ++c)
                        for (int kh = 0; kh < KH; ++kh) {
                            const int ih = oh * d->stride_h - d->pad_h + kh;
                            if (ih < 0 || ih >= H) continue;
                            for (int kw = 0; kw < KW; ++kw) {
                                const int iw = ow * d->stride_w - d->pad_w + kw;
                                if (iw < 0 || iw >= W) continue;
                                const size_t xi = (((size_t)n * d->C + g * Cg + c) * H + ih) * W + iw;
                                const size_t wi = (((size_t)m * Cg + c) * KH + kh) * KW + kw;
                                acc += (double)x[xi] * (double)w[wi];
                            }
                        }
                    y[(((size_t)n * d->M + m) * OH + oh) * OW + ow] = (REAL)acc;
                }
        }
    return 0;
}

/* Scatter form: every product dy*w of the forward sum is pushed back onto the
 * input element it was read from.  One double image per sample keeps the
 * accumulation in double; samples are independent. */
int cgo_conv_bwd_data(const cgo_conv_desc *d, const REAL *dy, const REAL *w, REAL *dx)
{
    int OH, OW;
    if (cgo_conv_out_shape(d, &OH, &OW)) return -1;
    const int G = d->groups, Cg = d->C / G, Mg = d->M / G;
    const int H = d->H, W = d->W, KH = d->KH, KW = d->KW;
    const size_t img = (size_t)d->C * H * W;
    int fail = 0;
#pragma omp parallel
    {
        double *acc = (double *)malloc(img * sizeof(double));
        if (!acc) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp barrier
        if (!fail) {
#pragma omp for schedule(static)
            for (int n = 0; n < d->N; ++n) {
                memset(acc, 0, img * sizeof(double));
                for (int m = 0; m < d->M; ++m) {
                    const int g = m / Mg;
                    for (int oh = 0; oh < OH; ++oh)
                        for (int ow = 0; ow < OW; ++ow) {
                            const double gy = (double)dy[(((size_t)n * d->M + m) * OH + oh) * OW + ow];
                            for (int c = 0; c < Cg; ++c)
                                for (int kh = 0; kh < KH; ++kh) {
                                    const int ih = oh * d->stride_h - d->pad_h + kh;
                                    if (ih < 0 || ih >= H) continue;
                                    for (int kw = 0; kw < KW; ++kw) {
                                        const int iw = ow * d->stride_w - d->pad_w + kw;
                                        if (iw < 0 || iw >= W) continue;
                                        acc[((size_t)(g * Cg + c) * H + ih) * W + iw] +=
                                            gy * (double)w[(((size_t)m * Cg + c) * KH + kh) * KW + kw];
                                    }
                                }
                        }
                }
                for (size_t i = 0; i < img; ++i) dx[(size_t)n * img + i] = (REAL)acc[i];
            }
        }
        free(acc);
    }
    return fail ? -2 : 0;
}

int cgo_conv_bwd_weight(const cgo_conv_desc *d, const REAL *x, const REAL *dy,
                        REAL *dw, REAL *db)
{
    int OH, OW;
    if (cgo_conv_out_shape(d, &OH, &OW)) return -1;
    const int G = d->groups, Cg = d->C / G, Mg = d->M / G;
    const int H = d->H, W = d->W, KH = d->KH, KW = d->KW;
#pragma omp parallel for collapse(2) schedule(static)
    for (int m = 0; m < d->M; ++m)
        for (int c = 0; c < Cg; ++c) {
            const int g = m / Mg;
            for (int kh = 0; kh < KH; ++kh)
                for (int kw = 0; kw < KW; ++kw) {
                    double acc = 0.0;
                    for (int n = 0; n < d->N; ++n)
                        for (int oh = 0; oh < OH; ++oh) {
                            const int ih = oh * d->stride_h - d->pad_h + kh;
                            if (ih < 0 || ih >= H) continue;
                            for (int ow = 0; ow < OW; ++ow) {
                                const int iw = ow * d->stride_w - d->pad_w + kw;
                                if (iw < 0 || iw >= W) continue;
                                acc += (double)dy[(((size_t)n * d->M + m) * OH + oh) * OW + ow] *
                                       (double)x[(((size_t)n * d->C + g * Cg + c) * H + ih) * W + iw];
                            }
                        }
                    dw[(((size_t)m * Cg + c) * KH + kh) * KW + kw] = (REAL)acc;
                }
        }
    if (db) {
#pragma omp parallel for schedule(static)
        for (int m = 0; m < d->M; ++m) {
            double acc = 0.0;
            for (int n = 0; n < d->N; ++n)
                for (int i = 0; i < OH * OW; ++i)
                    acc += (double)dy[((size_t)n * d->M + m) * OH * OW + i];
            db[m] = (REAL)acc;
        }
    }
    return 0;
}
