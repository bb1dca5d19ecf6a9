/*
 * cgo.h -- CPU oracle for one data-parallel worker's SGD iteration.
 *
 * TEST INFRASTRUCTURE ONLY.  This is the slow, plain reference the GPU library
 * is checked against.  It is never linked into, imported by or called from the
 * product path; it shares no source, header or table with the HIP code.
 *
 * The paper treats the layer arithmetic as the stock Caffe solver's (section
 * 2.1, "Stochastic Gradient Descend"; Fig. 1) and only fixes the data-parallel
 * update (Eq. 1) and the per-layer backward-order schedule (Fig. 3, section
 * 2.3).  Every function here writes the textbook definition of its operation
 * out as nested loops, accumulating in double and rounding once on store.
 *
 * The source is compiled twice: REAL=float (the reference the GPU is compared
 * with) and REAL=double (used for finite-difference pins of the backward
 * formulas).  All pointers are host pointers; tensors are dense NCHW / OIHW,
 * row-major.  Parallel loops run only over independent outputs, so the
 * summation order of every single output element is fixed.
 */
#ifndef CGO_H
#define CGO_H
#include <stddef.h>
#include <stdint.h>

#ifndef REAL
#define REAL float
#endif

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    int N, C, H, W;          /* input batch, channels, height, width          */
    int M, KH, KW;           /* output channels, kernel height, kernel width  */
    int stride_h, stride_w, pad_h, pad_w, groups;
} cgo_conv_desc;

/* OH = floor((H + 2*pad - KH)/stride) + 1; returns 0, or -1 if the
 * descriptor is not a valid convolution. */
int cgo_conv_out_shape(const cgo_conv_desc *d, int *OH, int *OW);

/* y[n,m,oh,ow] = b[m] + sum_{c,kh,kw} x[n, g*Cg+c, oh*s-p+kh, ow*s-p+kw] * w[m,c,kh,kw]
 * (cross-correlation, zero padding, Caffe group semantics).  bias may be NULL. */
int cgo_conv_fwd(const cgo_conv_desc *d, const REAL *x, const REAL *w,
                 const REAL *bias, REAL *y);
/* dx = adjoint of the map x -> y applied to dy (overwrites dx). */
int cgo_conv_bwd_data(const cgo_conv_desc *d, const REAL *dy, const REAL *w, REAL *dx);
/* dw = adjoint of the map w -> y applied to dy; db[m] = sum of dy over n,oh,ow
 * (overwrite; db may be NULL). */
int cgo_conv_bwd_weight(const cgo_conv_desc *d, const REAL *x, const REAL *dy,
                        REAL *dw, REAL *db);

void cgo_relu_fwd(size_t n, const REAL *x, REAL *y);
void cgo_relu_bwd(size_t n, const REAL *x, const REAL *dy, REAL *dx);

/* Max pooling, square window k, stride s, padding p.  Output size is
 * ceil((H+2p-k)/s)+1, clipped so that the last window starts inside the
 * (padded) image -- the Caffe rule.  Padded taps never win.  argmax holds
 * the flat index ih*W+iw of the first maximum in (kh,kw) row-major scan. */
int  cgo_maxpool_out(int H, int k, int s, int p);
void cgo_maxpool_fwd(int N, int C, int H, int W, int k, int s, int p,
                     const REAL *x, REAL *y, int32_t *argmax);
void cgo_maxpool_bwd(int N, int C, int H, int W, int k, int s, int p,
                     const REAL *dy, const int32_t *argmax, REAL *dx);

/* Local response normalisation across channels:
 * scale = kappa + (alpha/size) * sum_{c' in window of `size` centred on c} x^2,
 * y = x * scale^(-beta). */
void cgo_lrn_fwd(int N, int C, int HW, int size, double alpha, double beta, double kappa,
                 const REAL *x, REAL *y, REAL *scale);
void cgo_lrn_bwd(int N, int C, int HW, int size, double alpha, double beta,
                 const REAL *x, const REAL *y, const REAL *scale, const REAL *dy, REAL *dx);

/* Global average pool [N,C,H,W] -> [N,C]. */
void cgo_avgpool_fwd(int N, int C, int HW, const REAL *x, REAL *y);
void cgo_avgpool_bwd(int N, int C, int HW, const REAL *dy, REAL *dx);

/* Fully connected: y[b,o] = bias[o] + sum_i W[o,i] x[b,i]. */
void cgo_fc_fwd(int B, int IN, int OUT, const REAL *x, const REAL *W, const REAL *bias, REAL *y);
void cgo_fc_bwd_data(int B, int IN, int OUT, const REAL *dy, const REAL *W, REAL *dx);
void cgo_fc_bwd_weight(int B, int IN, int OUT, const REAL *x, const REAL *dy, REAL *dW, REAL *db);

/* Inverted dropout with a caller-supplied keep mask (1 = keep):
 * y = x * mask / (1-p); the backward pass applies the same factor. */
void cgo_dropout(size_t n, double p, const uint8_t *mask, const REAL *x, REAL *y);

/* loss = -(1/B) sum_b log softmax(z_b)[label_b]; dz = (softmax - onehot)/B. */
void cgo_softmax_ce(int B, int C, const REAL *z, const int32_t *labels, REAL *loss, REAL *dz);

/* Eq. 1 with the solver's history terms: per element, in this exact order and
 * with every operation rounded to REAL (no fused multiply-add):
 *   s = g_local; for k = 0..K-1: s = s + g_peers[k];
 *   if (grad_scale != 1) s = s * grad_scale;
 *   t = wd * w;  d = s + t;  a = mu * v;  b = lr * d;  vn = a + b;
 *   w = w - vn;  v = vn. */
void cgo_grad_reduce_sgd(REAL *w, REAL *v, const REAL *g_local,
                         const REAL *const *g_peers, int K, size_t n,
                         REAL lr, REAL mu, REAL wd, REAL grad_scale);

/* As above, with the K+1 gradients added in binomial-tree association
 * (section 3.2): rank 0 = local, rank k+1 = peer k; rank r adds the forwarded
 * sums of ranks r+1, r+2, r+4, ... (below r's lowest set bit, at most K) in
 * that order to its own gradient. */
void cgo_grad_reduce_sgd_tree(REAL *w, REAL *v, const REAL *g_local,
                              const REAL *const *g_peers, int K, size_t n,
                              REAL lr, REAL mu, REAL wd, REAL grad_scale);

int cgo_num_threads(void);
void cgo_set_num_threads(int n);

#ifdef __cplusplus
}
#endif
#endif
