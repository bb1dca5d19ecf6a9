/*
 * cgo_sgd.c -- CPU oracle (test infrastructure only): the per-layer gradient
 * aggregation and model update of the data-parallel iteration, Eq. 1:
 *     w^{l,k+1} = w^{l,k} - eps * sum_r dw_r^{l,k},
 * with the "higher order terms" the paper sets aside (solver history) written
 * in the Caffe SGD solver's form: L2 decay added to the summed gradient,
 * v <- mu*v + lr*(sum + wd*w), w <- w - v.  The s = K+1 rank gradients are
 * added left to right, the local one first (the paper adds partial gradients
 * as they arrive, section 3.2 "Reduction of the Gradient"; a fixed order is
 * chosen here so that the result has one bit pattern).
 *
 * This file must be compiled with floating-point contraction off
 * (-ffp-contract=off, SSE2 arithmetic): each operation below is individually
 * rounded to REAL.  Elements are independent, so the parallel loop does not
 * change any result.
 */
#include "cgo.h"

void cgo_grad_reduce_sgd(REAL *w, REAL *v, const REAL *g_local,
                         const REAL *const *g_peers, int K, size_t n,
                         REAL lr, REAL mu, REAL wd, REAL grad_scale)
{
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i) {
        REAL s = g_local[i];
        for (int k = 0; k < K; ++k) s = s + g_peers[k][i];
        if (grad_scale != (REAL)1) s = s * grad_scale;
        REAL t = wd * w[i];
        REAL d = s + t;
        REAL a = mu * v[i];
        REAL b = lr * d;
        REAL vn = a + b;
        w[i] = w[i] - vn;
        v[i] = vn;
    }
}
