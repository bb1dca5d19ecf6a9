/*
 * cg.h -- C ABI of the MI355X (gfx950) library for one data-parallel worker's
 * share of the CaffeGPI SGD iteration.
 *
 * What the library computes.  The paper distributes Caffe's mini-batch SGD
 * (Fig. 1) over s ranks by data parallelism: every rank runs forward and
 * backward on its share of the batch, the per-layer partial gradients are
 * summed and the model of layer l is updated by
 *        w^{l,k+1} = w^{l,k} - eps * sum_{r=1..s} dw_r^{l,k}          (Eq. 1)
 * layer by layer, in inverse layer order, while the backward pass of the
 * remaining layers is still running (section 2.3, Fig. 3; the per-layer
 * update of section 3).  This library is ONE rank: the s-1 = K peer gradients
 * are buffers already resident in this GPU's memory; the inter-node transport
 * (GPI-2, section 3.1-3.2) is outside it.
 *
 * Conventions for every entry point
 *  - All tensor pointers are DEVICE pointers to dense row-major fp32 data,
 *    16-byte aligned, activations NCHW, weights [M][C/groups][KH][KW].
 *    Pointer arrays documented as HOST arrays are read during the call.
 *  - Ownership: the caller allocates and frees every device buffer, including
 *    workspaces.  The library allocates no device memory.
 *  - Asynchrony: a call validates its arguments, enqueues work on the given
 *    HIP stream (a hipStream_t passed as void*; NULL = the default stream) and
 *    returns.  Nothing synchronises.  Outputs are valid in stream order.
 *  - Errors: the return value is CG_OK (0) or a negative CG_E* code.  A call
 *    that fails validation launches nothing.  Nothing aborts or throws.
 *  - Outputs are overwritten (not accumulated into) and must not alias inputs,
 *    except where a parameter is documented as updated in place.
 *  - Every tensor must hold fewer than 2^31 bytes.
 */
#ifndef CG_H
#define CG_H
#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    CG_OK = 0,
    CG_EINVAL = -1,        /* null pointer, bad descriptor, misaligned pointer          */
    CG_ENOSPC = -2,        /* workspace smaller than cg_*_workspace_bytes() reports      */
    CG_EUNSUPPORTED = -3,  /* valid request outside what the kernels cover               */
    CG_EHIP = -4           /* a HIP runtime call failed; see cg_last_hip_error()         */
};

/* One convolution layer on a batch: input [N,C,H,W], filters [M,C/groups,KH,KW],
 * output [N,M,OH,OW] with OH = floor((H + 2*pad_h - KH)/stride_h) + 1. */
typedef struct {
    int N, C, H, W;
    int M, KH, KW;
    int stride_h, stride_w, pad_h, pad_w, groups;
} cg_conv_desc;

/* Solver constants of the update: step size eps of Eq. 1 (lr), and the
 * terms that depend on the history of the model (text after Eq. 1):
 * momentum mu and L2 weight decay wd.  grad_scale multiplies the summed
 * gradient (1 = Eq. 1 literally; 1/(K+1) gives the mean over ranks). */
typedef struct { float lr, mu, wd, grad_scale; } cg_sgd;

enum { CG_PASS_FWD = 0, CG_PASS_BWD_DATA = 1, CG_PASS_BWD_WEIGHT = 2 };

/* What the matrix instructions of a contraction multiply in.  Tensors are fp32 in
 * memory and sums are accumulated in fp32 in every mode; the mode is always the
 * caller's explicit choice, nothing selects a reduced one by itself.
 *  CG_MATH_FP32   : fp32 products (the default of every entry point without a math argument).
 *  CG_MATH_BF16   : both operands rounded to bf16 (nearest even) on their way into the
 *                   matrix cores; parity bound 2e-2 (max-abs-relative).
 *  CG_MATH_BF16X3 : every operand split into two bf16 numbers, a = ah + al, three
 *                   products al*bh + ah*bl + ah*bh; the dropped al*bl is about 2^-16
 *                   of a product, so results stay inside the fp32 parity bound. */
enum { CG_MATH_FP32 = 0, CG_MATH_BF16 = 1, CG_MATH_BF16X3 = 2 };

/* Output spatial size of a convolution.  Returns CG_EINVAL for an invalid descriptor. */
int cg_conv_out_shape(const cg_conv_desc *d, int *OH, int *OW);

/* Bytes of device workspace the given pass needs for this descriptor (0 = none). */
size_t cg_conv_workspace_bytes(const cg_conv_desc *d, int pass);

/* Forward propagation of a convolution layer (section 2.1):
 *   y[n,m,oh,ow] = bias[m] + sum_{c,kh,kw} x[n, g*C/G + c, oh*s-p+kh, ow*s-p+kw] * w[m,c,kh,kw]
 * (cross-correlation; taps outside the image read 0; output channel m belongs
 * to group g = m / (M/G)).  bias may be NULL.  ws/ws_bytes: see
 * cg_conv_workspace_bytes(d, CG_PASS_FWD). */
int cg_conv_fwd(const cg_conv_desc *d, const float *x, const float *w, const float *bias,
                float *y, void *ws, size_t ws_bytes, void *stream);

/* Backward propagation to the layer input (section 2.1): dx is the adjoint of
 * x -> y applied to dy.  dy [N,M,OH,OW], w as above, dx [N,C,H,W] overwritten. */
int cg_conv_bwd_data(const cg_conv_desc *d, const float *dy, const float *w,
                     float *dx, void *ws, size_t ws_bytes, void *stream);

/* The local gradient of a layer (Fig. 3, first step of a turn):
 *   dw[m,c,kh,kw] = sum_{n,oh,ow} dy[n,m,oh,ow] * x[n, g*C/G + c, oh*s-p+kh, ow*s-p+kw]
 *   dbias[m]      = sum_{n,oh,ow} dy[n,m,oh,ow]             (dbias may be NULL)
 * Both overwritten.  The sum over n,oh,ow is split into slices reduced in a
 * fixed order, so results are reproducible run to run. */
int cg_conv_bwd_weight(const cg_conv_desc *d, const float *x, const float *dy,
                       float *dw, float *dbias, void *ws, size_t ws_bytes, void *stream);

/* The three passes above with the arithmetic of the matrix instructions chosen by
 * the caller (math = CG_MATH_*): the optional reduced-precision path for the
 * dense linear algebra of section 2.1.  Same arguments, layouts,
 * workspaces and errors; CG_MATH_FP32 is the call without the suffix.  The bias
 * sum of backward-weight is always fp32.  CG_EUNSUPPORTED: backward-data of a
 * strided convolution with fewer than 8 (channel, stride phase) pairs per group
 * exists in fp32 only. */
int cg_conv_fwd_math(const cg_conv_desc *d, const float *x, const float *w, const float *bias,
                     float *y, void *ws, size_t ws_bytes, int math, void *stream);
int cg_conv_bwd_data_math(const cg_conv_desc *d, const float *dy, const float *w,
                          float *dx, void *ws, size_t ws_bytes, int math, void *stream);
int cg_conv_bwd_weight_math(const cg_conv_desc *d, const float *x, const float *dy,
                            float *dw, float *dbias, void *ws, size_t ws_bytes, int math, void *stream);

/* cg_conv_bwd_weight for callers that can hand over no workspace and may not
 * allocate one: code under HIP graph capture, tight serving loops, harnesses
 * that forbid allocation.  The partial sums of the pass live in a device array
 * of CG_NOALLOC_SCRATCH_BYTES that belongs to the library (one copy per GPU,
 * held from the moment the library is loaded until the process ends); the call
 * allocates and frees nothing.  Results are bit-identical to cg_conv_bwd_weight.
 * Returns CG_ENOSPC, launching nothing, if the descriptor needs more than that
 * (cg_conv_workspace_bytes(d, CG_PASS_BWD_WEIGHT) tells).  All calls on one GPU
 * share the array: calls that overlap on one GPU (two streams, two threads)
 * race and must be serialised by the caller.  The device current at the call
 * must be the one the tensors live on. */
#define CG_NOALLOC_SCRATCH_BYTES (64u << 20)
int cg_conv_bwd_weight_noalloc(const cg_conv_desc *d, const float *x, const float *dy,
                               float *dw, float *dbias, void *stream);

/* Gradient aggregation over s = K+1 ranks fused with the model update of one
 * layer (Eq. 1; gradient reduction at the receiver and update on the reduced
 * gradient, section 3.2).  Per element
 * i < n, every operation rounded to fp32 in this order, no fused multiply-add:
 *     s = g_local[i];  for k = 0..K-1:  s = s + g_peers[k][i];
 *     if (grad_scale != 1) s = s * grad_scale;
 *     d = s + wd * w[i];   vn = mu * v[i] + lr * d;   w[i] = w[i] - vn;   v[i] = vn;
 * w, v: updated in place.  g_local, g_peers[k]: read only, n floats each (the
 * gradient of a layer has the size of its model, section 3.2).
 * g_peers: HOST array of K device pointers (may be NULL when K == 0).
 * 0 <= K <= CG_MAX_PEERS.  n == 0 is a no-op. */
#define CG_MAX_PEERS 64
int cg_grad_reduce_sgd(float *w, float *v, const float *g_local,
                       const float *const *g_peers, int K, size_t n,
                       const cg_sgd *sgd, void *stream);

/* The same update for nb layer buckets in one launch per eight buckets (the
 * small layers of a net are launch-bound one by one; the layer-wise update of
 * section 3 does not care how many layers a launch carries).  w, v, g_local, n:
 * HOST arrays of nb entries (device pointers / element counts); g_peers: HOST
 * array of nb HOST arrays of K device pointers.  All buckets share K and sgd.
 * Element for element the result is that of nb calls of cg_grad_reduce_sgd.
 * Buckets must not overlap.  Entries with n[i] == 0 are skipped. */
int cg_grad_reduce_sgd_multi(int nb, float *const *w, float *const *v,
                             const float *const *g_local,
                             const float *const *const *g_peers, int K,
                             const size_t *n, const cg_sgd *sgd, void *stream);

/* cg_grad_reduce_sgd / cg_grad_reduce_sgd_multi with the K+1 gradients added in
 * the association of the binomial reduction tree of section 3.2 (gradient
 * reduction: data travels from higher to lower rank numbers and ends on the
 * master, each rank adding what it receives to its own gradient before it
 * forwards the result).  Rank 0 is the local worker, rank k+1 is g_peers[k].
 * The receiver of rank r > 0 is r with its lowest set bit cleared; rank r
 * therefore adds the forwarded sums of ranks r+1, r+2, r+4, ... (distances
 * below r's lowest set bit, ranks at most K), and does so nearest first (the
 * paper adds in order of arrival; this fixed order gives one bit pattern):
 *     K = 4:  s = ((g0 + g1) + (g2 + g3)) + g4
 * Everything after the sum, the arguments, limits and errors are those of the
 * left-to-right entry points; for K <= 2 the results are identical to theirs. */
int cg_grad_reduce_sgd_tree(float *w, float *v, const float *g_local,
                            const float *const *g_peers, int K, size_t n,
                            const cg_sgd *sgd, void *stream);
int cg_grad_reduce_sgd_tree_multi(int nb, float *const *w, float *const *v,
                                  const float *const *g_local,
                                  const float *const *const *g_peers, int K,
                                  const size_t *n, const cg_sgd *sgd, void *stream);

/* ---- whole iteration ------------------------------------------------------ */

enum {
    CG_LAYER_CONV = 0, CG_LAYER_RELU, CG_LAYER_LRN, CG_LAYER_MAXPOOL, CG_LAYER_AVGPOOL,
    CG_LAYER_FC, CG_LAYER_DROPOUT, CG_LAYER_CONCAT, CG_LAYER_SOFTMAX_CE
};

/* One layer of the net.  inputs[0..n_inputs) are producer layer indices
 * (-1 = the net input); only CONCAT takes more than one.
 *  CONV       : conv.{M,KH,KW,stride_*,pad_*,groups} (N,C,H,W are inferred)
 *  MAXPOOL    : square window k, stride, pad; output size ceil((H+2p-k)/s)+1,
 *               the last window must start inside image+pad; first maximum wins
 *  LRN        : across channels, scale = kappa + alpha/size * sum x^2, y = x*scale^-beta
 *  AVGPOOL    : global average over H x W
 *  FC         : out features; weights [out][C*H*W]
 *  DROPOUT    : y = x * mask / (1 - drop_p), keep-mask supplied per step
 *  SOFTMAX_CE : mean over the batch of -log softmax(z)[label]; must be last */
typedef struct {
    int kind;
    int n_inputs;
    int inputs[4];
    cg_conv_desc conv;
    int k, stride, pad;
    int lrn_size;
    float lrn_alpha, lrn_beta, lrn_kappa;
    int fc_out;
    float drop_p;
} cg_layer_desc;

typedef struct cg_net cg_net;

/* Records shapes and creates the per-layer HIP events; allocates no device memory.
 * B = this worker's batch, (C,H,W) = input image shape. */
int cg_net_create(const cg_layer_desc *layers, int L, int B, int C, int H, int W, cg_net **out);
int cg_net_destroy(cg_net *net);

/* Number of floats in layer's parameter bucket (weights then bias, contiguous);
 * 0 for layers without parameters, negative on error. */
long long cg_net_param_count(const cg_net *net, int layer);

/* Which tensors of a layer are not materialised (bit flags, 0 = all are;
 * negative on error):
 *  1: the layer's own output.  A convolution or fully-connected layer whose
 *     only consumer is a rectifier stores max(., 0) directly, and which = 0 of
 *     cg_net_tensor() then names the rectifier's output for both layers.
 *  2: the gradient with respect to the layer's output.  The backward of a
 *     rectifier whose only consumer is a convolution, fully-connected, LRN,
 *     max-pool or dropout layer is folded into that consumer's backward kernel,
 *     which writes the gradient of the rectifier's input directly.
 * An LRN layer whose only consumer is a max-pool runs fused with it in forward
 * and reports bit 1: its output is never written. */
int cg_net_layer_fused(const cg_net *net, int layer);

/* Attach the caller-owned buffers of a parameter layer: model w, history v,
 * this worker's gradient g_local (written by every step), and K peer gradient
 * buckets (HOST array of K device pointers, copied), each param_count floats. */
int cg_net_bind(cg_net *net, int layer, float *w, float *v, float *g_local,
                const float *const *g_peers, int K);

/* Device workspace (activations, gradients of activations, kernel scratch). */
size_t cg_net_workspace_bytes(const cg_net *net);

enum { CG_STEP_OVERLAP = 0, CG_STEP_SERIAL = 1, CG_STEP_JOIN = 2, CG_STEP_TREE_SUM = 4,
       CG_STEP_BF16 = 8, CG_STEP_BF16X3 = 16 };

/* One SGD iteration of this worker (Fig. 1 with the turn-based schedule of
 * Fig. 3): forward through layers 1..L, loss, then for l = L..1 the local
 * gradient of layer l followed, on update_stream, by its aggregation and model
 * update (cg_grad_reduce_sgd) while compute_stream continues with layer l-1.
 * Layer l's forward in the NEXT call waits only for layer l's own update
 * (the per-layer completion step of section 2.3): there is no device-wide barrier.
 *  x [B,C,H,W], labels [B] (int32, device), dropout_masks: HOST array of L
 *  device pointers (uint8 keep-masks, one per DROPOUT layer, NULL elsewhere;
 *  the array may be NULL if the net has no dropout layer), loss_dev: 1 float.
 *  flags: CG_STEP_SERIAL runs the same kernels in the same order on
 *  compute_stream alone (the separate-phases schedule the paper improves on).
 * Backward-weight passes run beside backward-data on a stream the net owns.
 * The loss and the local gradients are valid in compute_stream order, the
 * updated w and v in update_stream order.
 * The two streams must differ unless CG_STEP_SERIAL is given.
 *  CG_STEP_TREE_SUM: the K+1 gradients of every layer are added in the
 *  association of the binomial reduction tree (cg_grad_reduce_sgd_tree) instead
 *  of left to right.
 *  CG_STEP_BF16 / CG_STEP_BF16X3 (at most one of them): every convolution and
 *  fully-connected pass of the step multiplies in CG_MATH_BF16 / CG_MATH_BF16X3
 *  (see cg_conv_fwd_math); everything else, the update included, is unchanged.
 *  CG_STEP_JOIN (with the overlapped schedule): at the end of the call
 *  compute_stream also waits for the last update, so that every stream the call
 *  used has joined compute_stream and the next call depends on no event of this
 *  one.  That is the form a caller can record into a HIP graph by stream capture
 *  on compute_stream (the call allocates nothing and synchronises nothing);
 *  the call before the captured one must have been made with this flag as
 *  well, or be complete, and cg_profile_enable must be off.  The price is the
 *  overlap of the last layers' updates with the next call's forward. */
int cg_train_step(cg_net *net, const float *x, const int32_t *labels,
                  const uint8_t *const *dropout_masks, const cg_sgd *sgd,
                  void *ws, size_t ws_bytes, void *compute_stream, void *update_stream,
                  float *loss_dev, int flags);

/* Where a layer's output (which = 0), the gradient with respect to its output
 * (which = 1) or its saved forward state (which = 2: the max-pool argmax as
 * int32 flat indices ih*W+iw; empty for other layers)
 * lives inside a workspace of base address ws after a step; for inspection by
 * tests.  count receives the number of 4-byte elements. */
int cg_net_tensor(const cg_net *net, int layer, int which, void *ws, float **ptr, size_t *count);

/* Elements between consecutive images of a layer's output (which = 0 above).
 * C*H*W for a dense tensor.  A convolution whose rectifier feeds only a concat
 * layer writes straight into its channel slice of the concat's output: for it
 * and for that rectifier this is the concat's C*H*W, ptr above is the slice of
 * image 0 and count spans up to the end of the last image's slice.  (The
 * concat's backward then also applies that rectifier's gate, so the gradient
 * with respect to the rectifier's output is not materialised.) */
long long cg_net_tensor_image_stride(const cg_net *net, int layer);

const char *cg_strerror(int code);
const char *cg_version(void);
int cg_last_hip_error(void);   /* hipError_t of the most recent CG_EHIP on this thread */

#ifdef __cplusplus
}
#endif
#endif
