// The layers around the convolutions of an AlexNet- or GoogLeNet-shaped iteration (section
// 2.1: forward and backward propagation through the layers): ReLU, across-channel LRN, max and
// global-average pooling, dropout with a supplied mask, softmax cross-entropy, channel concat.
// All are streaming fp32 kernels bound by HBM bandwidth; every reduction runs in a fixed order,
// so results are reproducible run to run.
#include "cg_internal.h"

namespace cg {

namespace {

constexpr int TB = 256;

inline unsigned grid_for(size_t n, unsigned cap = 16384)
{
    size_t b = (n + TB - 1) / TB;
    if (b > cap) b = cap;
    if (b == 0) b = 1;
    return (unsigned)b;
}

__global__ __launch_bounds__(TB) void relu_fwd_kernel(const float *__restrict__ x, float *__restrict__ y, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * TB + threadIdx.x; i < n; i += (size_t)gridDim.x * TB) {
        const float a = x[i];
        y[i] = a > 0.f ? a : 0.f;
    }
}

__global__ __launch_bounds__(TB) void relu_bwd_kernel(const float *__restrict__ x, const float *__restrict__ dy,
                                                      float *__restrict__ dx, size_t n, int accumulate)
{
    for (size_t i = (size_t)blockIdx.x * TB + threadIdx.x; i < n; i += (size_t)gridDim.x * TB) {
        const float gval = x[i] > 0.f ? dy[i] : 0.f;
        dx[i] = accumulate ? dx[i] + gval : gval;
    }
}

__global__ __launch_bounds__(TB) void maxpool_fwd_kernel(const float *__restrict__ x, float *__restrict__ y,
                                                         int32_t *__restrict__ argmax, size_t total, int H, int W,
                                                         int OH, int OW, int k, int s, int p)
{
    for (size_t i = (size_t)blockIdx.x * TB + threadIdx.x; i < total; i += (size_t)gridDim.x * TB) {
        const int ow = (int)(i % OW);
        size_t r = i / OW;
        const int oh = (int)(r % OH);
        const size_t nc = r / OH;
        const float *xp = x + nc * H * W;
        int best = -1;
        float bv = 0.f;
        for (int kh = 0; kh < k; ++kh) {
            const int ih = oh * s - p + kh;
            if (ih < 0 || ih >= H) continue;
            for (int kw = 0; kw < k; ++kw) {
                const int iw = ow * s - p + kw;
                if (iw < 0 || iw >= W) continue;
                const float val = xp[ih * W + iw];
                if (best < 0 || val > bv) { best = ih * W + iw; bv = val; }
            }
        }
        y[i] = bv;
        argmax[i] = best;
    }
}

// Gather form: an input element collects dy from every window that covers it and elected it.
__global__ __launch_bounds__(TB) void maxpool_bwd_kernel(const float *__restrict__ dy,
                                                         const int32_t *__restrict__ argmax, float *__restrict__ dx,
                                                         size_t total, int H, int W, int OH, int OW, int k, int s,
                                                         int p, int accumulate)
{
    for (size_t i = (size_t)blockIdx.x * TB + threadIdx.x; i < total; i += (size_t)gridDim.x * TB) {
        const int iw = (int)(i % W);
        size_t r = i / W;
        const int ih = (int)(r % H);
        const size_t nc = r / H;
        const int me = ih * W + iw;
        // windows oh with oh*s - p <= ih <= oh*s - p + k - 1
        int oh_lo = ih + p - k + 1;
        oh_lo = oh_lo <= 0 ? 0 : (oh_lo + s - 1) / s;
        int oh_hi = (ih + p) / s;
        if (oh_hi > OH - 1) oh_hi = OH - 1;
        int ow_lo = iw + p - k + 1;
        ow_lo = ow_lo <= 0 ? 0 : (ow_lo + s - 1) / s;
        int ow_hi = (iw + p) / s;
        if (ow_hi > OW - 1) ow_hi = OW - 1;
        float acc = 0.f;
        for (int oh = oh_lo; oh <= oh_hi; ++oh)
            for (int ow = ow_lo; ow <= ow_hi; ++ow) {
                const size_t o = (nc * OH + oh) * OW + ow;
                if (argmax[o] == me) acc += dy[o];
            }
        dx[i] = accumulate ? dx[i] + acc : acc;
    }
}

__global__ __launch_bounds__(TB) void lrn_fwd_kernel(const float *__restrict__ x, float *__restrict__ y,
                                                     float *__restrict__ scale, size_t total, int C, int HW, int size,
                                                     float alpha_over_size, float beta, float kappa)
{
    const int half = (size - 1) / 2;
    for (size_t i = (size_t)blockIdx.x * TB + threadIdx.x; i < total; i += (size_t)gridDim.x * TB) {
        const int c = (int)((i / HW) % C);
        float ss = 0.f;
        for (int d = -half; d <= -half + size - 1; ++d) {
            const int cc = c + d;
            if (cc < 0 || cc >= C) continue;
            const float xv = x[(ptrdiff_t)i + (ptrdiff_t)d * HW];
            ss += xv * xv;
        }
        const float sc = kappa + alpha_over_size * ss;
        scale[i] = sc;
        y[i] = x[i] * powf(sc, -beta);
    }
}

__global__ __launch_bounds__(TB) void lrn_bwd_kernel(const float *__restrict__ x, const float *__restrict__ y,
                                                     const float *__restrict__ scale, const float *__restrict__ dy,
                                                     float *__restrict__ dx, size_t total, int C, int HW, int size,
                                                     float coef, float beta, int accumulate)
{
    const int half = (size - 1) / 2;
    for (size_t i = (size_t)blockIdx.x * TB + threadIdx.x; i < total; i += (size_t)gridDim.x * TB) {
        const int c = (int)((i / HW) % C);
        float cross = 0.f;
        // channels j whose window [j-half, j-half+size-1] contains c
        for (int d = half - size + 1; d <= half; ++d) {
            const int j = c + d;
            if (j < 0 || j >= C) continue;
            const ptrdiff_t q = (ptrdiff_t)i + (ptrdiff_t)d * HW;
            cross += dy[q] * y[q] / scale[q];
        }
        const float gval = dy[i] * powf(scale[i], -beta) - coef * x[i] * cross;
        dx[i] = accumulate ? dx[i] + gval : gval;
    }
}

// one wave per (n, c) plane; lanes stride over the plane, then a fixed-order butterfly
__global__ __launch_bounds__(64) void avgpool_fwd_kernel(const float *__restrict__ x, float *__restrict__ y, int HW)
{
    const float *xp = x + (size_t)blockIdx.x * HW;
    float s = 0.f;
    for (int i = threadIdx.x; i < HW; i += 64) s += xp[i];
    for (int o = 32; o > 0; o >>= 1) s += __shfl_down(s, o, 64);
    if (threadIdx.x == 0) y[blockIdx.x] = s / (float)HW;
}

__global__ __launch_bounds__(TB) void avgpool_bwd_kernel(const float *__restrict__ dy, float *__restrict__ dx,
                                                         size_t total, int HW, int accumulate)
{
    const float inv = 1.f / (float)HW;
    for (size_t i = (size_t)blockIdx.x * TB + threadIdx.x; i < total; i += (size_t)gridDim.x * TB) {
        const float gval = dy[i / HW] * inv;
        dx[i] = accumulate ? dx[i] + gval : gval;
    }
}

__global__ __launch_bounds__(TB) void dropout_kernel(const float *__restrict__ x, const uint8_t *__restrict__ mask,
                                                     float *__restrict__ y, size_t n, float f, int accumulate)
{
    for (size_t i = (size_t)blockIdx.x * TB + threadIdx.x; i < n; i += (size_t)gridDim.x * TB) {
        const float gval = mask[i] ? x[i] * f : 0.f;
        y[i] = accumulate ? y[i] + gval : gval;
    }
}

// one block per sample: log-sum-exp with max subtraction, per-sample loss, dz = (p - onehot)/B
__global__ __launch_bounds__(TB) void softmax_ce_kernel(const float *__restrict__ z, const int32_t *__restrict__ labels,
                                                        float *__restrict__ per_sample, float *__restrict__ dz, int B,
                                                        int C)
{
    __shared__ float red[TB];
    const int b = blockIdx.x;
    const float *zb = z + (size_t)b * C;
    float mx = -INFINITY;
    for (int c = threadIdx.x; c < C; c += TB) mx = fmaxf(mx, zb[c]);
    red[threadIdx.x] = mx;
    __syncthreads();
    for (int w = TB / 2; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) red[threadIdx.x] = fmaxf(red[threadIdx.x], red[threadIdx.x + w]);
        __syncthreads();
    }
    mx = red[0];
    __syncthreads();
    float se = 0.f;
    for (int c = threadIdx.x; c < C; c += TB) se += expf(zb[c] - mx);
    red[threadIdx.x] = se;
    __syncthreads();
    for (int w = TB / 2; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
        __syncthreads();
    }
    const float lse = mx + logf(red[0]);
    int lab = labels[b];
    lab = lab < 0 ? 0 : (lab >= C ? C - 1 : lab);   // an out-of-range label must not become a wild read
    if (threadIdx.x == 0) per_sample[b] = lse - zb[lab];
    const float invB = 1.f / (float)B;
    for (int c = threadIdx.x; c < C; c += TB) {
        const float pr = expf(zb[c] - lse);
        dz[(size_t)b * C + c] = (pr - (c == lab ? 1.f : 0.f)) * invB;
    }
}

__global__ __launch_bounds__(TB) void mean_kernel(const float *__restrict__ v, float *__restrict__ out, int n)
{
    __shared__ float red[TB];
    float s = 0.f;
    for (int i = threadIdx.x; i < n; i += TB) s += v[i];
    red[threadIdx.x] = s;
    __syncthreads();
    for (int w = TB / 2; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) *out = red[0] / (float)n;
}

__global__ __launch_bounds__(TB) void concat_copy_kernel(const float *__restrict__ src, float *__restrict__ dst,
                                                         size_t total, int Csrc, int Cdst, int c_off, int HW,
                                                         int to_concat, int accumulate)
{
    // `total` runs over the slice [N][Csrc][HW]; the concat tensor is [N][Cdst][HW]
    const size_t plane = (size_t)Csrc * HW;
    for (size_t i = (size_t)blockIdx.x * TB + threadIdx.x; i < total; i += (size_t)gridDim.x * TB) {
        const size_t n = i / plane, r = i - n * plane;
        const size_t big = (n * Cdst + c_off) * HW + r;
        if (to_concat) dst[big] = src[i];
        else dst[i] = accumulate ? dst[i] + src[big] : src[big];
    }
}

__global__ __launch_bounds__(TB) void fc_bias_grad_kernel(const float *__restrict__ dy, int B, int OUT,
                                                          float *__restrict__ db)
{
    const int o = blockIdx.x * TB + threadIdx.x;
    if (o >= OUT) return;
    float s = 0.f;
    for (int b = 0; b < B; ++b) s += dy[(size_t)b * OUT + o];
    db[o] = s;
}

}  // namespace

#define CG_LAUNCH_CHECK()                  \
    do {                                   \
        CG_HIP_TRY(hipGetLastError());     \
        return CG_OK;                      \
    } while (0)

int pool_out_size(int H, int k, int s, int p)
{
    const int e = H + 2 * p - k;
    if (e < 0) return 0;
    int o = (e + s - 1) / s + 1;
    if ((o - 1) * s >= H + p) --o;
    return o;
}

int fc_bias_grad_launch(const float *dy, int B, int OUT, float *db, hipStream_t st)
{
    hipLaunchKernelGGL(fc_bias_grad_kernel, dim3((OUT + TB - 1) / TB), dim3(TB), 0, st, dy, B, OUT, db);
    CG_LAUNCH_CHECK();
}

int relu_fwd_launch(const float *x, float *y, size_t n, hipStream_t st)
{
    if (n == 0) return CG_OK;
    hipLaunchKernelGGL(relu_fwd_kernel, dim3(grid_for(n)), dim3(TB), 0, st, x, y, n);
    CG_LAUNCH_CHECK();
}

int relu_bwd_launch(const float *x, const float *dy, float *dx, size_t n, int accumulate, hipStream_t st)
{
    if (n == 0) return CG_OK;
    hipLaunchKernelGGL(relu_bwd_kernel, dim3(grid_for(n)), dim3(TB), 0, st, x, dy, dx, n, accumulate);
    CG_LAUNCH_CHECK();
}

int maxpool_fwd_launch(const float *x, float *y, int32_t *argmax, int N, int C, int H, int W, int k, int s, int p,
                       hipStream_t st)
{
    const int OH = pool_out_size(H, k, s, p), OW = pool_out_size(W, k, s, p);
    if (OH <= 0 || OW <= 0 || p >= k) return CG_EINVAL;
    const size_t total = (size_t)N * C * OH * OW;
    hipLaunchKernelGGL(maxpool_fwd_kernel, dim3(grid_for(total)), dim3(TB), 0, st, x, y, argmax, total, H, W, OH, OW,
                       k, s, p);
    CG_LAUNCH_CHECK();
}

int maxpool_bwd_launch(const float *dy, const int32_t *argmax, float *dx, int N, int C, int H, int W, int k, int s,
                       int p, int accumulate, hipStream_t st)
{
    const int OH = pool_out_size(H, k, s, p), OW = pool_out_size(W, k, s, p);
    if (OH <= 0 || OW <= 0) return CG_EINVAL;
    const size_t total = (size_t)N * C * H * W;
    hipLaunchKernelGGL(maxpool_bwd_kernel, dim3(grid_for(total)), dim3(TB), 0, st, dy, argmax, dx, total, H, W, OH, OW,
                       k, s, p, accumulate);
    CG_LAUNCH_CHECK();
}

int lrn_fwd_launch(const float *x, float *y, float *scale, int N, int C, int HW, int size, float alpha, float beta,
                   float kappa, hipStream_t st)
{
    if (size <= 0) return CG_EINVAL;
    const size_t total = (size_t)N * C * HW;
    hipLaunchKernelGGL(lrn_fwd_kernel, dim3(grid_for(total)), dim3(TB), 0, st, x, y, scale, total, C, HW, size,
                       alpha / (float)size, beta, kappa);
    CG_LAUNCH_CHECK();
}

int lrn_bwd_launch(const float *x, const float *y, const float *scale, const float *dy, float *dx, int N, int C,
                   int HW, int size, float alpha, float beta, int accumulate, hipStream_t st)
{
    const size_t total = (size_t)N * C * HW;
    hipLaunchKernelGGL(lrn_bwd_kernel, dim3(grid_for(total)), dim3(TB), 0, st, x, y, scale, dy, dx, total, C, HW, size,
                       2.f * alpha * beta / (float)size, beta, accumulate);
    CG_LAUNCH_CHECK();
}

int avgpool_fwd_launch(const float *x, float *y, int NC, int HW, hipStream_t st)
{
    hipLaunchKernelGGL(avgpool_fwd_kernel, dim3(NC), dim3(64), 0, st, x, y, HW);
    CG_LAUNCH_CHECK();
}

int avgpool_bwd_launch(const float *dy, float *dx, int NC, int HW, int accumulate, hipStream_t st)
{
    const size_t total = (size_t)NC * HW;
    hipLaunchKernelGGL(avgpool_bwd_kernel, dim3(grid_for(total)), dim3(TB), 0, st, dy, dx, total, HW, accumulate);
    CG_LAUNCH_CHECK();
}

int dropout_launch(const float *x, const uint8_t *mask, float *y, size_t n, float p, int accumulate, hipStream_t st)
{
    if (!mask || p < 0.f || p >= 1.f) return CG_EINVAL;
    hipLaunchKernelGGL(dropout_kernel, dim3(grid_for(n)), dim3(TB), 0, st, x, mask, y, n, 1.f / (1.f - p), accumulate);
    CG_LAUNCH_CHECK();
}

int softmax_ce_launch(const float *z, const int32_t *labels, float *loss, float *dz, float *per_sample, int B, int C,
                      hipStream_t st)
{
    hipLaunchKernelGGL(softmax_ce_kernel, dim3(B), dim3(TB), 0, st, z, labels, per_sample, dz, B, C);
    CG_HIP_TRY(hipGetLastError());
    hipLaunchKernelGGL(mean_kernel, dim3(1), dim3(TB), 0, st, per_sample, loss, B);
    CG_LAUNCH_CHECK();
}

int concat_copy_launch(const float *src, float *dst, int N, int Csrc, int Cdst, int c_off, int HW, int to_concat,
                       int accumulate, hipStream_t st)
{
    const size_t total = (size_t)N * Csrc * HW;
    hipLaunchKernelGGL(concat_copy_kernel, dim3(grid_for(total)), dim3(TB), 0, st, src, dst, total, Csrc, Cdst, c_off,
                       HW, to_concat, accumulate);
    CG_LAUNCH_CHECK();
}

}  // namespace cg
