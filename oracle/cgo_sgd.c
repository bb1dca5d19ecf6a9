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

/*
 * The same update with the K+1 rank gradients added in the association of a
 * binomial reduction tree (section 3.2: gradients travel from higher to lower
 * rank numbers and end on the master, rank 0; a rank adds what it receives to
 * its own data and forwards the result to its receiver).  Rank 0 is the local
 * worker, rank k+1 is peer k.  The receiver of rank r > 0 is r with its lowest
 * set bit cleared, so the senders of rank r are r + 1, r + 2, r + 4, ... below
 * r's own lowest set bit (any power of two for rank 0) and not above K.  The
 * paper adds senders' data as it arrives; here the senders are added in the
 * order of their distance (the smallest subtree, which is ready first, first),
 * which fixes one bit pattern.
 */
static REAL tree_sum(const REAL *g_local, const REAL *const *g_peers, int K,
                     size_t i, int r, int span)
{
    /* what rank r forwards: its own gradient plus its senders' r + d, d < span */
    REAL s = r == 0 ? g_local[i] : g_peers[r - 1][i];
    for (int d = 1; d < span && r + d <= K; d *= 2)
        s = s + tree_sum(g_local, g_peers, K, i, r + d, d);
    return s;
}

void cgo_grad_reduce_sgd_tree(REAL *w, REAL *v, const REAL *g_local,
                              const REAL *const *g_peers, int K, size_t n,
                              REAL lr, REAL mu, REAL wd, REAL grad_scale)
{
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i) {
        REAL s = tree_sum(g_local, g_peers, K, i, 0, 1 << 30);
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
