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

// Element-wise kernels move 16 bytes per lane; `n4` counts whole float4 groups, the last n % 4
// elements are handled by the first lanes of block 0.
__global__ __launch_bounds__(TB) void relu_fwd_kernel(const float *__restrict__ x, float *__restrict__ y, size_t n)
{
    const size_t n4 = n / 4;
    const float4 *x4 = reinterpret_cast<const float4 *>(x);
    float4 *y4 = reinterpret_cast<float4 *>(y);
    for (size_t i = (size_t)blockIdx.x * TB + threadIdx.x; i < n4; i += (size_t)gridDim.x * TB) {
        float4 a = x4[i];
        a.x = a.x > 0.f ? a.x : 0.f; a.y = a.y > 0.f ? a.y : 0.f;
        a.z = a.z > 0.f ? a.z : 0.f; a.w = a.w > 0.f ? a.w : 0.f;
        y4[i] = a;
    }
    if (blockIdx.x == 0 && threadIdx.x < n % 4) {
        const size_t i = n4 * 4 + threadIdx.x;
        y[i] = x[i] > 0.f ? x[i] : 0.f;
    }
}

// x may be the rectifier's input or its output: only the sign is used, and both have the same
template <int ACC>
__global__ __launch_bounds__(TB) void relu_bwd_kernel(const float *__restrict__ x, const float *__restrict__ dy,
                                                      float *__restrict__ dx, size_t n)
{
    const size_t n4 = n / 4;
    const float4 *x4 = reinterpret_cast<const float4 *>(x);
    const float4 *g4 = reinterpret_cast<const float4 *>(dy);
    float4 *d4 = reinterpret_cast<float4 *>(dx);
    for (size_t i = (size_t)blockIdx.x * TB + threadIdx.x; i < n4; i += (size_t)gridDim.x * TB) {
        const float4 a = x4[i], g = g4[i];
        float4 r;
        r.x = a.x > 0.f ? g.x : 0.f; r.y = a.y > 0.f ? g.y : 0.f;
        r.z = a.z > 0.f ? g.z : 0.f; r.w = a.w > 0.f ? g.w : 0.f;
        if (ACC) { const float4 o = d4[i]; r.x += o.x; r.y += o.y; r.z += o.z; r.w += o.w; }
        d4[i] = r;
    }
    if (blockIdx.x == 0 && threadIdx.x < n % 4) {
        const size_t i = n4 * 4 + threadIdx.x;
        const float gval = x[i] > 0.f ? dy[i] : 0.f;
        dx[i] = ACC ? dx[i] + gval : gval;
    }
}

// Pooling kernels: a block owns `ppb` consecutive (n, c) planes and first copies what it reads
// (forward: the input planes; backward: dy and the winners) into LDS, so that the window gathers,
// whose addresses depend on loaded data in backward, never go to global memory.  The copy issues
// all of a thread's loads (16 bytes each) before its first LDS write: with one load in flight
// per thread the copy would run at the latency of HBM, not at its bandwidth.  All index
// arithmetic is 32-bit and local to a plane; the divisions use multipliers computed on the host.
// KT/ST are the window and stride when known at compile time, 0 = use the run-time values.
constexpr int POOL_LDS = 8192;         // elements of LDS staging per block (floats, or float + int pairs)
constexpr int STAGE_U = 8;             // 16-byte loads a thread keeps in flight while staging

// Copies g[0..n) to s[0..n).  `s` is placed by the caller so that s and g have the same offset
// within a 16-byte group (s = base + ((address of g / 4) & 3), base 16-byte aligned): the groups
// in between are moved whole, the up to three elements before and after them one by one.
__device__ __forceinline__ void stage_to_lds(const float *__restrict__ g, float *s, uint32_t n)
{
    const uint32_t head = min(n, (4u - (uint32_t)(((uintptr_t)g >> 2) & 3u)) & 3u);
    const uint32_t n4 = (n - head) / 4, tail0 = head + n4 * 4;
    if (threadIdx.x < head) s[threadIdx.x] = g[threadIdx.x];
    if (tail0 + threadIdx.x < n) s[tail0 + threadIdx.x] = g[tail0 + threadIdx.x];
    typedef float f4 __attribute__((ext_vector_type(4)));
    const f4 *g4 = reinterpret_cast<const f4 *>(g + head);
    f4 *s4 = reinterpret_cast<f4 *>(s + head);
    for (uint32_t q0 = threadIdx.x; q0 < n4; q0 += TB * STAGE_U) {
        f4 v[STAGE_U];
#pragma unroll
        for (int u = 0; u < STAGE_U; ++u) {
            const uint32_t q = q0 + u * TB;
            if (q < n4) v[u] = __builtin_nontemporal_load(g4 + q);
        }
#pragma unroll
        for (int u = 0; u < STAGE_U; ++u) {
            const uint32_t q = q0 + u * TB;
            if (q < n4) s4[q] = v[u];
        }
    }
}

template <int KT, int ST>
__global__ __launch_bounds__(TB) void maxpool_fwd_kernel(const float *__restrict__ x, float *__restrict__ y,
                                                         int32_t *__restrict__ argmax, uint32_t planes, int ppb, int H,
                                                         int W, int OH, int OW, int k_rt, int s_rt, int p, FastDiv divP,
                                                         FastDiv divOW)
{
    extern __shared__ __align__(16) float pool_lds[];
    const int k = KT ? KT : k_rt, s = ST ? ST : s_rt;
    const uint32_t Q = (uint32_t)(H * W), P = (uint32_t)(OH * OW), plane0 = blockIdx.x * (uint32_t)ppb;
    const uint32_t np = min((uint32_t)ppb, planes - plane0);
    const float *xg = x + (size_t)plane0 * Q;
    float *xs = pool_lds + (((uintptr_t)xg >> 2) & 3u);
    stage_to_lds(xg, xs, np * Q);
    __syncthreads();
    for (uint32_t j = threadIdx.x; j < np * P; j += TB) {
        const uint32_t pl = fdiv(j, divP), o = j - pl * P;
        const int oh = (int)fdiv(o, divOW), ow = (int)(o - (uint32_t)oh * OW);
        const float *xp = xs + pl * Q;
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
        y[(size_t)plane0 * P + j] = bv;
        argmax[(size_t)plane0 * P + j] = best;
    }
}

// Gather form: an input element collects dy from every window that covers it and elected it.
// `gate`, if given, is the output of the rectifier that produced this layer's input: the result
// is then the gradient with respect to the rectifier's INPUT (zero where the gate is not positive).
// What a thread reads from global memory in the main loop (gate, dx when accumulating) is loaded
// four elements ahead of the arithmetic.
template <int KT, int ST, int ACC>
__global__ __launch_bounds__(TB) void maxpool_bwd_kernel(const float *__restrict__ dy,
                                                         const int32_t *__restrict__ argmax, float *__restrict__ dx,
                                                         const float *__restrict__ gate, uint32_t planes, int ppb,
                                                         int H, int W, int OH, int OW, int k_rt, int s_rt, int p,
                                                         FastDiv divQ, FastDiv divW, FastDiv divS)
{
    extern __shared__ __align__(16) float pool_lds[];
    const int k = KT ? KT : k_rt, s = ST ? ST : s_rt;
    const uint32_t Q = (uint32_t)(H * W), P = (uint32_t)(OH * OW), plane0 = blockIdx.x * (uint32_t)ppb;
    const uint32_t np = min((uint32_t)ppb, planes - plane0);
    const float *dyg = dy + (size_t)plane0 * P;
    const float *ag = reinterpret_cast<const float *>(argmax + (size_t)plane0 * P);      // moved as 32-bit words
    const uint32_t half = ((uint32_t)ppb * P + 4 + 3) & ~3u;
    float *gs = pool_lds + (((uintptr_t)dyg >> 2) & 3u);
    float *asf = pool_lds + half + (((uintptr_t)ag >> 2) & 3u);
    stage_to_lds(dyg, gs, np * P);
    stage_to_lds(ag, asf, np * P);
    __syncthreads();
    const int32_t *as = reinterpret_cast<const int32_t *>(asf);
    const uint32_t total = np * Q;
    const size_t g0 = (size_t)plane0 * Q;
    // (plane, row, column) of the thread's element: one division at the start, then carried along
    // as the element index advances by the block size
    const uint32_t stepW = TB % (uint32_t)W, stepH = TB / (uint32_t)W;
    uint32_t pl = fdiv(threadIdx.x, divQ);
    uint32_t ih = fdiv(threadIdx.x - pl * Q, divW), iw = threadIdx.x - pl * Q - ih * (uint32_t)W;
    constexpr int NW = KT ? (KT + ST - 1) / ST : 0;      // windows that can cover an element, per dimension
    for (uint32_t j0 = threadIdx.x; j0 < total; j0 += TB * 4) {
        float gt[4], old[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t j = j0 + u * TB;
            gt[u] = (gate && j < total) ? gate[g0 + j] : 1.f;
            old[u] = (ACC && j < total) ? dx[g0 + j] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t j = j0 + u * TB;
            if (j >= total) break;
            const int32_t me = (int32_t)(ih * (uint32_t)W + iw);
            // windows oh with oh*s - p <= ih <= oh*s - p + k - 1  (numerators below are >= 0 where divided)
            int oh_lo = (int)ih + p - k + 1;
            oh_lo = oh_lo <= 0 ? 0 : (int)(ST ? (uint32_t)(oh_lo + s - 1) / (uint32_t)(ST ? ST : 1)
                                              : fdiv((uint32_t)(oh_lo + s - 1), divS));
            int oh_hi = (int)(ST ? (ih + (uint32_t)p) / (uint32_t)(ST ? ST : 1) : fdiv(ih + (uint32_t)p, divS));
            if (oh_hi > OH - 1) oh_hi = OH - 1;
            int ow_lo = (int)iw + p - k + 1;
            ow_lo = ow_lo <= 0 ? 0 : (int)(ST ? (uint32_t)(ow_lo + s - 1) / (uint32_t)(ST ? ST : 1)
                                              : fdiv((uint32_t)(ow_lo + s - 1), divS));
            int ow_hi = (int)(ST ? (iw + (uint32_t)p) / (uint32_t)(ST ? ST : 1) : fdiv(iw + (uint32_t)p, divS));
            if (ow_hi > OW - 1) ow_hi = OW - 1;
            const int32_t *ap = as + pl * P;
            const float *gp = gs + pl * P;
            float acc = 0.f;
            if (NW) {
                // a fixed NW x NW sweep, in the same order as the loops below; windows outside
                // [lo, hi] read a clamped position and are not counted
#pragma unroll
                for (int a = NW - 1; a >= 0; --a)
#pragma unroll
                    for (int b = NW - 1; b >= 0; --b) {
                        const int oh = oh_hi - a, ow = ow_hi - b;
                        const bool in = oh >= oh_lo && ow >= ow_lo;
                        const int o = in ? oh * OW + ow : 0;
                        if (in && ap[o] == me) acc += gp[o];
                    }
            } else {
                for (int oh = oh_lo; oh <= oh_hi; ++oh)
                    for (int ow = ow_lo; ow <= ow_hi; ++ow) {
                        const int o = oh * OW + ow;
                        if (ap[o] == me) acc += gp[o];
                    }
            }
            if (!(gt[u] > 0.f)) acc = 0.f;
            dx[g0 + j] = ACC ? old[u] + acc : acc;
            iw += stepW;
            ih += stepH;
            if (iw >= (uint32_t)W) { iw -= (uint32_t)W; ++ih; }
            while (ih >= (uint32_t)H) { ih -= (uint32_t)H; ++pl; }
        }
    }
}

// Planes too large for the LDS staging (beyond POOL_LDS input elements forward, POOL_LDS / 2
// outputs backward): the same two gathers straight from global memory, one element per thread,
// `bpp` blocks per plane.  Window order and tie-break are those of the staged kernels.
__global__ __launch_bounds__(TB) void maxpool_fwd_direct_kernel(const float *__restrict__ x, float *__restrict__ y,
                                                                int32_t *__restrict__ argmax, int H, int W, int OH,
                                                                int OW, int k, int s, int p, uint32_t bpp,
                                                                FastDiv divBpp, FastDiv divOW)
{
    const uint32_t pl = fdiv(blockIdx.x, divBpp), o = (blockIdx.x - pl * bpp) * TB + threadIdx.x;
    const uint32_t P = (uint32_t)(OH * OW);
    if (o >= P) return;
    const int oh = (int)fdiv(o, divOW), ow = (int)(o - (uint32_t)oh * OW);
    const float *xp = x + (size_t)pl * (uint32_t)(H * W);
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
    y[(size_t)pl * P + o] = bv;
    argmax[(size_t)pl * P + o] = best;
}

template <int ACC>
__global__ __launch_bounds__(TB) void maxpool_bwd_direct_kernel(const float *__restrict__ dy,
                                                                const int32_t *__restrict__ argmax,
                                                                float *__restrict__ dx, const float *__restrict__ gate,
                                                                int H, int W, int OH, int OW, int k, int s, int p,
                                                                uint32_t bpp, FastDiv divBpp, FastDiv divW, FastDiv divS)
{
    const uint32_t pl = fdiv(blockIdx.x, divBpp), q = (blockIdx.x - pl * bpp) * TB + threadIdx.x;
    const uint32_t Q = (uint32_t)(H * W), P = (uint32_t)(OH * OW);
    if (q >= Q) return;
    const uint32_t ih = fdiv(q, divW), iw = q - ih * (uint32_t)W;
    // windows oh with oh*s - p <= ih <= oh*s - p + k - 1
    int oh_lo = (int)ih + p - k + 1;
    oh_lo = oh_lo <= 0 ? 0 : (int)fdiv((uint32_t)(oh_lo + s - 1), divS);
    int oh_hi = (int)fdiv(ih + (uint32_t)p, divS);
    if (oh_hi > OH - 1) oh_hi = OH - 1;
    int ow_lo = (int)iw + p - k + 1;
    ow_lo = ow_lo <= 0 ? 0 : (int)fdiv((uint32_t)(ow_lo + s - 1), divS);
    int ow_hi = (int)fdiv(iw + (uint32_t)p, divS);
    if (ow_hi > OW - 1) ow_hi = OW - 1;
    const int32_t *ap = argmax + (size_t)pl * P;
    const float *gp = dy + (size_t)pl * P;
    const size_t at = (size_t)pl * Q + q;
    const float gt = gate ? gate[at] : 1.f;
    const float old = ACC ? dx[at] : 0.f;
    float acc = 0.f;
    for (int oh = oh_lo; oh <= oh_hi; ++oh)
        for (int ow = ow_lo; ow <= ow_hi; ++ow) {
            const int o = oh * OW + ow;
            if (ap[o] == (int32_t)q) acc += gp[o];
        }
    if (!(gt > 0.f)) acc = 0.f;
    dx[at] = ACC ? old + acc : acc;
}

// Backward for a window and stride known at compile time.  A thread owns a cell of ST x ST input
// elements: the (at most NWC x NWC) windows that can cover any of them are read from LDS once,
// and every element of the cell adds the dy of the windows that elected it, in ascending window
// order (the order of the gather form above, so the sums are the same bit for bit).  The cell's
// results go to an LDS copy of the dx planes, which the block then writes out in 16-byte groups,
// applying `gate` and the accumulation there.
template <int KT, int ST, int ACC>
__global__ __launch_bounds__(TB) void maxpool_bwd_cell_kernel(const float *__restrict__ dy,
                                                              const int32_t *__restrict__ argmax,
                                                              float *__restrict__ dx, const float *__restrict__ gate,
                                                              uint32_t planes, int ppb, int H, int W, int OH, int OW,
                                                              int p, FastDiv divCells, FastDiv divCW)
{
    constexpr int NWC = (KT - 1 + ST - 1) / ST + 1;
    typedef float f4 __attribute__((ext_vector_type(4)));
    extern __shared__ __align__(16) float pool_lds[];
    const uint32_t Q = (uint32_t)(H * W), P = (uint32_t)(OH * OW), plane0 = blockIdx.x * (uint32_t)ppb;
    const uint32_t np = min((uint32_t)ppb, planes - plane0);
    const float *dyg = dy + (size_t)plane0 * P;
    const float *ag = reinterpret_cast<const float *>(argmax + (size_t)plane0 * P);      // moved as 32-bit words
    float *dxg = dx + (size_t)plane0 * Q;
    const float *gg = gate ? gate + (size_t)plane0 * Q : nullptr;
    const uint32_t half = ((uint32_t)ppb * P + 4 + 3) & ~3u;
    float *gs = pool_lds + (((uintptr_t)dyg >> 2) & 3u);
    float *asf = pool_lds + half + (((uintptr_t)ag >> 2) & 3u);
    float *os = pool_lds + 2 * half + (((uintptr_t)dxg >> 2) & 3u);
    stage_to_lds(dyg, gs, np * P);
    stage_to_lds(ag, asf, np * P);
    __syncthreads();
    const int32_t *as = reinterpret_cast<const int32_t *>(asf);
    const uint32_t CW = (uint32_t)(W + ST - 1) / ST, CH = (uint32_t)(H + ST - 1) / ST, cells = CW * CH;
    for (uint32_t j = threadIdx.x; j < np * cells; j += TB) {
        const uint32_t pl = fdiv(j, divCells), cell = j - pl * cells;
        const uint32_t ca = fdiv(cell, divCW), cb = cell - ca * CW;
        const int ih0 = (int)ca * ST, iw0 = (int)cb * ST;
        // first window that can reach the cell's first row / column (numerators >= 0 where divided)
        int oh0 = ih0 + p - KT + 1, ow0 = iw0 + p - KT + 1;
        oh0 = oh0 <= 0 ? 0 : (oh0 + ST - 1) / ST;
        ow0 = ow0 <= 0 ? 0 : (ow0 + ST - 1) / ST;
        int32_t wa[NWC][NWC];
        float wg[NWC][NWC];
#pragma unroll
        for (int a = 0; a < NWC; ++a)
#pragma unroll
            for (int b = 0; b < NWC; ++b) {
                const int oh = oh0 + a, ow = ow0 + b;
                const bool in = oh < OH && ow < OW;
                const uint32_t o = pl * P + (uint32_t)(in ? oh * OW + ow : 0);
                wa[a][b] = in ? as[o] : -1;
                wg[a][b] = gs[o];
            }
#pragma unroll
        for (int r = 0; r < ST; ++r)
#pragma unroll
            for (int c = 0; c < ST; ++c) {
                const int ih = ih0 + r, iw = iw0 + c;
                if (ih >= H || iw >= W) continue;
                const int32_t me = ih * W + iw;
                float acc = 0.f;
#pragma unroll
                for (int a = 0; a < NWC; ++a)
#pragma unroll
                    for (int b = 0; b < NWC; ++b)
                        if (wa[a][b] == me) acc += wg[a][b];
                os[pl * Q + (uint32_t)me] = acc;
            }
    }
    __syncthreads();
    // write-out: the groups of four that are aligned in global memory, then the elements around them
    const uint32_t n = np * Q;
    const uint32_t head = min(n, (4u - (uint32_t)(((uintptr_t)dxg >> 2) & 3u)) & 3u);
    const uint32_t n4 = (n - head) / 4, tail0 = head + n4 * 4;
    for (uint32_t e = threadIdx.x; e < head + (n - tail0); e += TB) {
        const uint32_t i = e < head ? e : tail0 + (e - head);
        float v = os[i];
        if (gg && !(gg[i] > 0.f)) v = 0.f;
        dxg[i] = ACC ? dxg[i] + v : v;
    }
    const f4 *s4 = reinterpret_cast<const f4 *>(os + head);
    f4 *d4 = reinterpret_cast<f4 *>(dxg + head);
    const f4 *t4 = reinterpret_cast<const f4 *>(gg ? gg + head : nullptr);
    for (uint32_t q0 = threadIdx.x; q0 < n4; q0 += TB * 4) {
        f4 gt[4], old[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t q = q0 + u * TB;
            gt[u] = (gg && q < n4) ? __builtin_nontemporal_load(t4 + q) : f4{1.f, 1.f, 1.f, 1.f};
            old[u] = (ACC && q < n4) ? d4[q] : f4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t q = q0 + u * TB;
            if (q >= n4) break;
            f4 v = s4[q];
            v.x = gt[u].x > 0.f ? v.x : 0.f;
            v.y = gt[u].y > 0.f ? v.y : 0.f;
            v.z = gt[u].z > 0.f ? v.z : 0.f;
            v.w = gt[u].w > 0.f ? v.w : 0.f;
            d4[q] = ACC ? old[u] + v : v;
        }
    }
}

// ---- local response normalisation across channels ---------------------------------------------
//   scale_c = kappa + (alpha/size) * sum_{j in win(c)} x_j^2,  y_c = x_c * scale_c^-beta,
//   win(c) = [c - half, c - half + size - 1], half = (size-1)/2.
// A thread owns four consecutive pixels and walks along the channels of a chunk with the window in registers:
// every x is read once (plus a halo of size-1 per chunk), nothing but y is written, and backward
// recomputes the scales from x instead of reading them back.

__device__ __forceinline__ float pow_neg(float sc, float beta)      // sc^-beta, sc > 0
{
    if (beta == 0.75f) { const float r = rsqrtf(sc); return r * sqrtf(r); }
    return exp2f(-beta * log2f(sc));
}

constexpr int LRN_CH = 48;        // channels per chunk
constexpr int LRN_V = 4;          // consecutive pixels per thread

// Four consecutive pixels of one channel plane move as one 16-byte access.  The planes of a tensor
// with an odd pixel count start at any multiple of 4 bytes, which these accesses allow; the last
// thread of a plane, whose group reaches beyond it, moves its `rem` < 4 pixels one by one.
typedef float f4u __attribute__((ext_vector_type(4), aligned(4)));

struct Px4 { float v[LRN_V]; };

__device__ __forceinline__ Px4 px_load(const float *__restrict__ p, int rem)
{
    Px4 r;
    if (rem >= LRN_V) {
        const f4u q = __builtin_nontemporal_load(reinterpret_cast<const f4u *>(p));
        r.v[0] = q.x; r.v[1] = q.y; r.v[2] = q.z; r.v[3] = q.w;
    } else {
#pragma unroll
        for (int e = 0; e < LRN_V; ++e) r.v[e] = e < rem ? p[e] : 0.f;
    }
    return r;
}

__device__ __forceinline__ Px4 px_zero()
{
    Px4 r;
#pragma unroll
    for (int e = 0; e < LRN_V; ++e) r.v[e] = 0.f;
    return r;
}

template <int ACC> __device__ __forceinline__ void px_store(float *__restrict__ p, int rem, const Px4 &r)
{
    if (rem >= LRN_V) {
        f4u q = {r.v[0], r.v[1], r.v[2], r.v[3]};
        if (ACC) q += *reinterpret_cast<const f4u *>(p);
        *reinterpret_cast<f4u *>(p) = q;
    } else {
#pragma unroll
        for (int e = 0; e < LRN_V; ++e)
            if (e < rem) p[e] = ACC ? p[e] + r.v[e] : r.v[e];
    }
}

template <int SIZE>
__global__ __launch_bounds__(TB) void lrn_fwd_stream_kernel(const float *__restrict__ x, float *__restrict__ y, int C,
                                                            int HW, int nchunk, float aos, float beta, float kappa)
{
    constexpr int half = (SIZE - 1) / 2;
    const int pix = (blockIdx.x * TB + threadIdx.x) * LRN_V;
    if (pix >= HW) return;
    const int rem = HW - pix;
    const int n = blockIdx.y / nchunk, c0 = (blockIdx.y % nchunk) * LRN_CH;
    const int c1 = min(C, c0 + LRN_CH);
    const float *xp = x + (size_t)n * C * HW + pix;
    float *yp = y + (size_t)n * C * HW + pix;
    Px4 win[SIZE];                 // x[c - half .. c - half + SIZE - 1] once the step's element has entered
#pragma unroll
    for (int d = 0; d < SIZE - 1; ++d) {
        const int cc = c0 - half + d;
        win[d + 1] = (cc >= 0 && cc < C) ? px_load(xp + (size_t)cc * HW, rem) : px_zero();
    }
#pragma unroll 4
    for (int c = c0; c < c1; ++c) {
        const int e = c - half + SIZE - 1;
#pragma unroll
        for (int d = 0; d < SIZE - 1; ++d) win[d] = win[d + 1];
        win[SIZE - 1] = e < C ? px_load(xp + (size_t)e * HW, rem) : px_zero();
        Px4 out;
#pragma unroll
        for (int v = 0; v < LRN_V; ++v) {
            float ss = 0.f;
#pragma unroll
            for (int d = 0; d < SIZE; ++d) ss += win[d].v[v] * win[d].v[v];
            out.v[v] = win[half].v[v] * pow_neg(kappa + aos * ss, beta);
        }
        px_store<0>(yp + (size_t)c * HW, rem, out);
    }
}

//   dx_c = dy_c * scale_c^-beta - (2 alpha beta / size) * x_c * sum_{j : c in win(j)} dy_j x_j scale_j^(-beta-1)
// Step c (from c0 - (SIZE-1), the first SIZE-1 steps only fill the rings) lets x_e enter, e = c + SIZE - 1,
// computes scale and t = dy x scale^(-beta-1) of channel j = c + half, whose window is now complete,
// and emits dx_c, whose sum over j in [c - (SIZE-1-half), c + half] is the whole t ring.
// GATE: x is the output of a rectifier and dx the gradient with respect to that rectifier's input.
template <int SIZE, int ACC, int GATE>
__global__ __launch_bounds__(TB) void lrn_bwd_stream_kernel(const float *__restrict__ x, const float *__restrict__ dy,
                                                            float *__restrict__ dx, int C, int HW, int nchunk,
                                                            float aos, float coef, float beta, float kappa)
{
    constexpr int half = (SIZE - 1) / 2;
    const int pix = (blockIdx.x * TB + threadIdx.x) * LRN_V;
    if (pix >= HW) return;
    const int rem = HW - pix;
    const int n = blockIdx.y / nchunk, c0 = (blockIdx.y % nchunk) * LRN_CH;
    const int c1 = min(C, c0 + LRN_CH);
    const size_t img = (size_t)n * C * HW + pix;
    const float *xp = x + img, *gp = dy + img;
    float *dp = dx + img;
    Px4 win[SIZE], tr[SIZE], q[half + 1];        // x window, t ring, dy*scale^-beta of the last half+1 channels
#pragma unroll
    for (int d = 0; d < SIZE; ++d) tr[d] = px_zero();
#pragma unroll
    for (int d = 0; d <= half; ++d) q[d] = px_zero();
    const int cs = c0 - (SIZE - 1);
#pragma unroll
    for (int d = 0; d < SIZE - 1; ++d) {
        const int cc = cs + d;                   // ring holds x[e-SIZE+1 .. e-1] before step cs, e = cs + SIZE - 1
        win[d + 1] = (cc >= 0 && cc < C) ? px_load(xp + (size_t)cc * HW, rem) : px_zero();
    }
#pragma unroll 2
    for (int c = cs; c < c1; ++c) {
        const int e = c + SIZE - 1, j = c + half;
#pragma unroll
        for (int d = 0; d < SIZE - 1; ++d) { win[d] = win[d + 1]; tr[d] = tr[d + 1]; }
#pragma unroll
        for (int d = 0; d < half; ++d) q[d] = q[d + 1];
        win[SIZE - 1] = (e >= 0 && e < C) ? px_load(xp + (size_t)e * HW, rem) : px_zero();
        Px4 t = px_zero(), qq = px_zero();
        if (j >= 0 && j < C) {
            const Px4 g = px_load(gp + (size_t)j * HW, rem);
#pragma unroll
            for (int v = 0; v < LRN_V; ++v) {
                float ss = 0.f;
#pragma unroll
                for (int d = 0; d < SIZE; ++d) ss += win[d].v[v] * win[d].v[v];
                const float sc = kappa + aos * ss, pw = pow_neg(sc, beta);
                qq.v[v] = g.v[v] * pw;
                t.v[v] = qq.v[v] * win[half].v[v] / sc;      // x_j sits at position half of its own window
            }
        }
        tr[SIZE - 1] = t;
        q[half] = qq;
        if (c >= c0) {
            Px4 out;
#pragma unroll
            for (int v = 0; v < LRN_V; ++v) {
                float cross = 0.f;
#pragma unroll
                for (int d = 0; d < SIZE; ++d) cross += tr[d].v[v];
                float gval = q[0].v[v] - coef * win[0].v[v] * cross;     // x_c = x_{e-SIZE+1}: the oldest ring entry
                if (GATE && !(win[0].v[v] > 0.f)) gval = 0.f;
                out.v[v] = gval;
            }
            px_store<ACC>(dp + (size_t)c * HW, rem, out);
        }
    }
}

// ---- LRN followed by max-pooling, in one pass -----------------------------------------------------
// The normalised tensor is the largest of an AlexNet-shaped net (the first layer's 96 x 55 x 55 per
// image) and exists only to be pooled: written once by the LRN, read once by the pool, and in
// backward its gradient is written by the pool and read by the LRN.  Fused, neither it nor its
// gradient touches memory.  A block owns one image, LP_CH channels (plus the window's halo) and a
// band of rows of at most 4 x 256 pixels, and walks along the channels like the stream kernels
// above, a thread holding four consecutive pixels, so that the band of the current channel is in
// the block:
//   forward:  a band is the input rows that `prb` pooled rows need (neighbouring bands share the
//             k - s rows their windows overlap in); the band of y = x * scale^-beta goes to LDS (two
//             buffers, one barrier per channel) and is pooled from there: only the pooled values
//             and the winners are written;
//   backward: a band is `hrb` input rows; the pooled rows of dy and of the winners that cover it
//             are staged in LDS, a pixel collects the dy of the windows that elected it (ascending
//             window order, as maxpool_bwd_kernel does) and feeds it to the LRN backward recurrence
//             of lrn_bwd_stream_kernel.
// The arithmetic is that of the separate kernels, operation for operation: same y, same winners.
constexpr int LP_CH = 32;
constexpr int LP_NP = 4;          // staged pooled elements per thread (at most LP_NP * TB a band)

// LDS writes of this wave have landed, then the block's barrier.  Unlike __syncthreads() this does
// not wait for the global loads in flight: the next channel's loads are issued before the barrier
// and must stay in flight across it, or every step would run at the latency of HBM.
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// KT, ST: window and stride when known at compile time (0 = run-time values); INSIDE: no window
// reaches beyond the plane (no padding, the last window ends inside), so no tap needs a range test
template <int SIZE, int KT, int ST, bool INSIDE>
__global__ __launch_bounds__(TB) void lrn_pool_fwd_kernel(const float *__restrict__ x, float *__restrict__ yp,
                                                          int32_t *__restrict__ argmax, int C, int H, int W, int OH, int OW,
                                                          int k_rt, int s_rt, int p, int nchunk, int nbands, int prb, float aos,
                                                          float beta, float kappa, FastDiv divOW)
{
    const int k = KT ? KT : k_rt, s = ST ? ST : s_rt;
    extern __shared__ __align__(16) float lp_lds[];          // [2][4 * TB]
    constexpr int half = (SIZE - 1) / 2, LB = LRN_V * TB;
    const int HW = H * W, P = OH * OW;
    int bi = blockIdx.x;
    const int band = bi % nbands; bi /= nbands;
    const int n = bi / nchunk, c0 = (bi % nchunk) * LP_CH, c1 = min(C, c0 + LP_CH);
    const int pr0 = band * prb, pr1 = min(OH, pr0 + prb);
    const int ih0 = max(0, pr0 * s - p), ih1 = min(H, (pr1 - 1) * s - p + k);
    const int base = ih0 * W, lim = ih1 * W;                 // the band's pixels in the plane
    const float *xn = x + (size_t)n * C * HW;
    const int loc = (int)threadIdx.x * LRN_V, pix = base + loc, rem = lim - pix;
    auto load_x = [&](int cc) {
        return (rem > 0 && cc >= 0 && cc < C) ? px_load(xn + (size_t)cc * HW + pix, rem) : px_zero();
    };
    Px4 win[SIZE], nxt;             // nxt: the channel that enters the window in the coming step, loaded a step ahead
#pragma unroll
    for (int d = 0; d < SIZE - 1; ++d) win[d + 1] = load_x(c0 - half + d);
    nxt = load_x(c0 - half + SIZE - 1);
    int buf = 0;
    for (int c = c0; c < c1; ++c) {
        float *ys = lp_lds + buf * LB;
        const int e = c - half + SIZE - 1;
#pragma unroll
        for (int d = 0; d < SIZE - 1; ++d) win[d] = win[d + 1];
        win[SIZE - 1] = nxt;
        nxt = c + 1 < c1 ? load_x(e + 1) : px_zero();
        if (rem > 0) {
            float out[LRN_V];
#pragma unroll
            for (int v = 0; v < LRN_V; ++v) {
                float ss = 0.f;
#pragma unroll
                for (int d = 0; d < SIZE; ++d) ss += win[d].v[v] * win[d].v[v];
                out[v] = win[half].v[v] * pow_neg(kappa + aos * ss, beta);
            }
            *reinterpret_cast<float4 *>(ys + loc) = make_float4(out[0], out[1], out[2], out[3]);   // beyond rem: never read
        }
        lds_barrier();          // the band is complete; the other buffer's readers of two channels ago are done too
        const size_t obase = ((size_t)n * C + c) * P;
        for (int o = pr0 * OW + (int)threadIdx.x; o < pr1 * OW; o += TB) {
            const int oh = (int)fdiv((uint32_t)o, divOW), ow = o - oh * OW;
            int best = -1;
            float bv = 0.f;
            if constexpr (INSIDE && KT > 0) {
                const int org = oh * s * W + ow * s;          // p = 0: the window's first element
                const float *yw = ys + org - base;
                best = org; bv = yw[0];
#pragma unroll
                for (int kh = 0; kh < KT; ++kh)
#pragma unroll
                    for (int kw = 0; kw < KT; ++kw) {
                        if (kh == 0 && kw == 0) continue;
                        const float val = yw[kh * W + kw];
                        if (val > bv) { best = org + kh * W + kw; bv = val; }
                    }
            } else {
                for (int kh = 0; kh < k; ++kh) {
                    const int ih = oh * s - p + kh;
                    if (ih < 0 || ih >= H) continue;
                    for (int kw = 0; kw < k; ++kw) {
                        const int iw = ow * s - p + kw;
                        if (iw < 0 || iw >= W) continue;
                        const float val = ys[ih * W + iw - base];
                        if (best < 0 || val > bv) { best = ih * W + iw; bv = val; }
                    }
                }
            }
            yp[obase + o] = bv;
            argmax[obase + o] = best;
        }
        buf ^= 1;
    }
}

template <int SIZE, int ACC, int GATE>
__global__ __launch_bounds__(TB) void lrn_pool_bwd_kernel(const float *__restrict__ x, const float *__restrict__ dpool,
                                                          const int32_t *__restrict__ argmax, float *__restrict__ dx, int C,
                                                          int H, int W, int OH, int OW, int k, int s, int p, int nchunk,
                                                          int nbands, int hrb, float aos, float coef, float beta,
                                                          float kappa, FastDiv divW, FastDiv divS)
{
    extern __shared__ __align__(16) float lp_lds[];          // [2][LP_NP * TB] pooled dy, then the same of winners
    constexpr int half = (SIZE - 1) / 2, LS = LP_NP * TB;
    const int HW = H * W, P = OH * OW;
    float *dps = lp_lds;
    int32_t *ams = reinterpret_cast<int32_t *>(lp_lds + 2 * LS);
    int bi = blockIdx.x;
    const int band = bi % nbands; bi /= nbands;
    const int n = bi / nchunk, c0 = (bi % nchunk) * LP_CH, c1 = min(C, c0 + LP_CH);
    const int h0 = band * hrb, h1 = min(H, h0 + hrb);
    // pooled rows with a window on the band's rows
    const int a_lo = h0 + p - k + 1;
    const int oh_lo = a_lo > 0 ? (int)fdiv((uint32_t)(a_lo + s - 1), divS) : 0;
    const int oh_hi = min(OH - 1, (int)fdiv((uint32_t)(h1 - 1 + p), divS));
    const int sbase = oh_lo * OW, scount = max(0, (oh_hi - oh_lo + 1) * OW);
    const size_t img = (size_t)n * C * HW;
    const float *xn = x + img;
    float *dn = dx + img;
    const int pix = h0 * W + (int)threadIdx.x * LRN_V, rem = h1 * W - pix;
    // the windows that cover each of the thread's pixels: first window row / column and how many
    // (at most ceil(k/s) a dimension), packed: oh0 | noh << 12 | ow0 << 16 | now << 28
    uint32_t cover[LRN_V];
#pragma unroll
    for (int v = 0; v < LRN_V; ++v) {
        const int q = min(pix + v, HW - 1);
        const int h = (int)fdiv((uint32_t)q, divW), w = q - h * W;
        const int a_h = h + p - k + 1, a_w = w + p - k + 1;
        const int oh0 = a_h > 0 ? (int)fdiv((uint32_t)(a_h + s - 1), divS) : 0, oh1 = min(OH - 1, (int)fdiv((uint32_t)(h + p), divS));
        const int ow0 = a_w > 0 ? (int)fdiv((uint32_t)(a_w + s - 1), divS) : 0, ow1 = min(OW - 1, (int)fdiv((uint32_t)(w + p), divS));
        const int noh = max(0, oh1 - oh0 + 1), now = max(0, ow1 - ow0 + 1);
        cover[v] = (uint32_t)oh0 | ((uint32_t)noh << 12) | ((uint32_t)ow0 << 16) | ((uint32_t)now << 28);
    }
    auto load_x = [&](int cc) {
        return (rem > 0 && cc >= 0 && cc < C) ? px_load(xn + (size_t)cc * HW + pix, rem) : px_zero();
    };
    // the staged part of channel jj's pooled plane (dy and winners), this thread's elements, into registers
    float pd[LP_NP];
    int32_t pa[LP_NP];
    auto load_plane = [&](int jj) {
        const size_t pb = ((size_t)n * C + jj) * P + sbase;
#pragma unroll
        for (int u = 0; u < LP_NP; ++u) {
            const int o = u * TB + (int)threadIdx.x;
            if (o < scount) { pd[u] = dpool[pb + o]; pa[u] = argmax[pb + o]; }
        }
    };
    Px4 win[SIZE], tr[SIZE], q[half + 1], nxt;
#pragma unroll
    for (int d = 0; d < SIZE; ++d) tr[d] = px_zero();
#pragma unroll
    for (int d = 0; d <= half; ++d) q[d] = px_zero();
    const int cs = c0 - (SIZE - 1);
#pragma unroll
    for (int d = 0; d < SIZE - 1; ++d) win[d + 1] = load_x(cs + d);
    nxt = load_x(cs + SIZE - 1);
    if (cs + half >= 0 && cs + half < C) load_plane(cs + half);
    int buf = 0;
    for (int c = cs; c < c1; ++c) {
        const int e = c + SIZE - 1, j = c + half;
        const bool have_j = j >= 0 && j < C;                   // uniform over the block
        if (have_j) {
            // channel j's pooled rows, loaded during the previous step, go to LDS
#pragma unroll
            for (int u = 0; u < LP_NP; ++u) {
                const int o = u * TB + (int)threadIdx.x;
                if (o < scount) { dps[buf * LS + o] = pd[u]; ams[buf * LS + o] = pa[u]; }
            }
            lds_barrier();      // staged; the other buffer's readers of the step before are done too
        }
        // what the next step needs from memory, a step ahead
        if (c + 1 < c1 && j + 1 >= 0 && j + 1 < C) load_plane(j + 1);
#pragma unroll
        for (int d = 0; d < SIZE - 1; ++d) { win[d] = win[d + 1]; tr[d] = tr[d + 1]; }
#pragma unroll
        for (int d = 0; d < half; ++d) q[d] = q[d + 1];
        win[SIZE - 1] = nxt;
        nxt = c + 1 < c1 ? load_x(e + 1) : px_zero();
        if (rem > 0) {
            Px4 t = px_zero(), qq = px_zero();
            if (have_j) {
                const float *dp = dps + buf * LS - sbase;
                const int32_t *am = ams + buf * LS - sbase;
#pragma unroll
                for (int v = 0; v < LRN_V; ++v) {
                    // the gradient of the LRN output at this pixel: dy of the windows that elected it
                    float gsum = 0.f;
                    if (v < rem) {
                        const uint32_t cv = cover[v];
                        const int oh0 = (int)(cv & 0xfffu), noh = (int)((cv >> 12) & 0xfu);
                        const int ow0 = (int)((cv >> 16) & 0xfffu), now = (int)(cv >> 28);
                        const int me = pix + v;
                        for (int a = 0; a < noh; ++a)
                            for (int b = 0; b < now; ++b) {
                                const int o = (oh0 + a) * OW + ow0 + b;
                                if (am[o] == me) gsum += dp[o];
                            }
                    }
                    float ss = 0.f;
#pragma unroll
                    for (int d = 0; d < SIZE; ++d) ss += win[d].v[v] * win[d].v[v];
                    const float sc = kappa + aos * ss, pw = pow_neg(sc, beta);
                    qq.v[v] = gsum * pw;
                    t.v[v] = qq.v[v] * win[half].v[v] / sc;
                }
            }
            tr[SIZE - 1] = t;
            q[half] = qq;
            if (c >= c0) {
                Px4 out;
#pragma unroll
                for (int v = 0; v < LRN_V; ++v) {
                    float cross = 0.f;
#pragma unroll
                    for (int d = 0; d < SIZE; ++d) cross += tr[d].v[v];
                    float gval = q[0].v[v] - coef * win[0].v[v] * cross;
                    if (GATE && !(win[0].v[v] > 0.f)) gval = 0.f;
                    out.v[v] = gval;
                }
                px_store<ACC>(dn + (size_t)c * HW + pix, rem, out);
            }
        }
        if (have_j) buf ^= 1;
    }
}

// any window size: the definition, term by term (scales recomputed per term)
__global__ __launch_bounds__(TB) void lrn_fwd_kernel(const float *__restrict__ x, float *__restrict__ y, size_t total,
                                                     int C, int HW, int size, float alpha_over_size, float beta,
                                                     float kappa)
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
        y[i] = x[i] * pow_neg(kappa + alpha_over_size * ss, beta);
    }
}

__device__ __forceinline__ float lrn_scale_at(const float *__restrict__ x, ptrdiff_t i, int c, int C, int HW, int size,
                                              float aos, float kappa)
{
    const int half = (size - 1) / 2;
    float ss = 0.f;
    for (int d = -half; d <= -half + size - 1; ++d) {
        const int cc = c + d;
        if (cc < 0 || cc >= C) continue;
        const float xv = x[i + (ptrdiff_t)d * HW];
        ss += xv * xv;
    }
    return kappa + aos * ss;
}

__global__ __launch_bounds__(TB) void lrn_bwd_kernel(const float *__restrict__ x, const float *__restrict__ dy,
                                                     float *__restrict__ dx, size_t total, int C, int HW, int size,
                                                     float aos, float coef, float beta, float kappa, int accumulate,
                                                     int gate)
{
    const int half = (size - 1) / 2;
    for (size_t i = (size_t)blockIdx.x * TB + threadIdx.x; i < total; i += (size_t)gridDim.x * TB) {
        const int c = (int)((i / HW) % C);
        float cross = 0.f;
        // channels j whose window [j-half, j-half+size-1] contains c
        for (int d = half - size + 1; d <= half; ++d) {
            const int j = c + d;
            if (j < 0 || j >= C) continue;
            const ptrdiff_t qi = (ptrdiff_t)i + (ptrdiff_t)d * HW;
            const float sc = lrn_scale_at(x, qi, j, C, HW, size, aos, kappa);
            cross += dy[qi] * x[qi] * pow_neg(sc, beta) / sc;
        }
        const float sc = lrn_scale_at(x, (ptrdiff_t)i, c, C, HW, size, aos, kappa);
        float gval = dy[i] * pow_neg(sc, beta) - coef * x[i] * cross;
        if (gate && !(x[i] > 0.f)) gval = 0.f;
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

// `gate` (backward only): output of the rectifier that produced the layer's input; see maxpool_bwd_kernel
template <int ACC>
__global__ __launch_bounds__(TB) void dropout_kernel(const float *__restrict__ x, const uint8_t *__restrict__ mask,
                                                     float *__restrict__ y, const float *__restrict__ gate, size_t n,
                                                     float f)
{
    const size_t n4 = n / 4;
    const float4 *x4 = reinterpret_cast<const float4 *>(x);
    const uchar4 *m4 = reinterpret_cast<const uchar4 *>(mask);
    float4 *y4 = reinterpret_cast<float4 *>(y);
    for (size_t i = (size_t)blockIdx.x * TB + threadIdx.x; i < n4; i += (size_t)gridDim.x * TB) {
        const float4 a = x4[i];
        const uchar4 m = m4[i];
        float4 r;
        r.x = m.x ? a.x * f : 0.f; r.y = m.y ? a.y * f : 0.f; r.z = m.z ? a.z * f : 0.f; r.w = m.w ? a.w * f : 0.f;
        if (gate) {
            const float4 g = reinterpret_cast<const float4 *>(gate)[i];
            r.x = g.x > 0.f ? r.x : 0.f; r.y = g.y > 0.f ? r.y : 0.f; r.z = g.z > 0.f ? r.z : 0.f; r.w = g.w > 0.f ? r.w : 0.f;
        }
        if (ACC) { const float4 o = y4[i]; r.x += o.x; r.y += o.y; r.z += o.z; r.w += o.w; }
        y4[i] = r;
    }
    if (blockIdx.x == 0 && threadIdx.x < n % 4) {
        const size_t i = n4 * 4 + threadIdx.x;
        float gval = mask[i] ? x[i] * f : 0.f;
        if (gate && !(gate[i] > 0.f)) gval = 0.f;
        y[i] = ACC ? y[i] + gval : gval;
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
                                                         const float *__restrict__ gate, size_t total, int Csrc,
                                                         int Cdst, int c_off, int HW, int to_concat, int accumulate)
{
    // `total` runs over the slice [N][Csrc][HW]; the concat tensor is [N][Cdst][HW].  `gate` (from the
    // concat tensor to the slice only) is a tensor of the concat's shape holding the output of the
    // rectifier that produced the slice: the result is the gradient of that rectifier's input.
    const size_t plane = (size_t)Csrc * HW;
    for (size_t i = (size_t)blockIdx.x * TB + threadIdx.x; i < total; i += (size_t)gridDim.x * TB) {
        const size_t n = i / plane, r = i - n * plane;
        const size_t big = (n * Cdst + c_off) * HW + r;
        if (to_concat) {
            dst[big] = src[i];
        } else {
            float val = src[big];
            if (gate && !(gate[big] > 0.f)) val = 0.f;
            dst[i] = accumulate ? dst[i] + val : val;
        }
    }
}

// db[o] = sum_b dy[b][o]: a block owns 32 outputs, its 8 thread rows sum interleaved samples, and
// the 8 partial sums are added in row order
__global__ __launch_bounds__(TB) void fc_bias_grad_kernel(const float *__restrict__ dy, int B, int OUT,
                                                          float *__restrict__ db)
{
    __shared__ float part[8][32];
    const int ol = threadIdx.x & 31, r = threadIdx.x >> 5, o = blockIdx.x * 32 + ol;
    float s = 0.f;
    if (o < OUT)
        for (int b = r; b < B; b += 8) s += dy[(size_t)b * OUT + o];
    part[r][ol] = s;
    __syncthreads();
    if (r == 0 && o < OUT) {
        float t = part[0][ol];
#pragma unroll
        for (int k = 1; k < 8; ++k) t += part[k][ol];
        db[o] = t;
    }
}

}  // namespace

#define CG_LAUNCH_CHECK()                  \
    do {                                   \
        CG_HIP_TRY(hipGetLastError());     \
        return CG_OK;                      \
    } while (0)

// planes per block of the pooling kernels: about four elements per thread (`work` per plane),
// and no more than fit the LDS staging (`staged` elements per plane of at most `cap`)
static int pool_planes_per_block(int work, int staged, int cap)
{
    int ppb = 1024 / (work > 0 ? work : 1);
    if (ppb < 1) ppb = 1;
    while (ppb > 1 && ppb * staged > cap) --ppb;
    return ppb;
}

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
    hipLaunchKernelGGL(fc_bias_grad_kernel, dim3((OUT + 31) / 32), dim3(TB), 0, st, dy, B, OUT, db);
    CG_LAUNCH_CHECK();
}

int relu_fwd_launch(const float *x, float *y, size_t n, hipStream_t st)
{
    if (n == 0) return CG_OK;
    if (!aligned16(x) || !aligned16(y)) return CG_EINVAL;
    hipLaunchKernelGGL(relu_fwd_kernel, dim3(grid_for(n / 4 + 1)), dim3(TB), 0, st, x, y, n);
    CG_LAUNCH_CHECK();
}

int relu_bwd_launch(const float *x, const float *dy, float *dx, size_t n, int accumulate, hipStream_t st)
{
    if (n == 0) return CG_OK;
    if (!aligned16(x) || !aligned16(dy) || !aligned16(dx)) return CG_EINVAL;
    if (accumulate) hipLaunchKernelGGL(relu_bwd_kernel<1>, dim3(grid_for(n / 4 + 1)), dim3(TB), 0, st, x, dy, dx, n);
    else hipLaunchKernelGGL(relu_bwd_kernel<0>, dim3(grid_for(n / 4 + 1)), dim3(TB), 0, st, x, dy, dx, n);
    CG_LAUNCH_CHECK();
}

int maxpool_fwd_launch(const float *x, float *y, int32_t *argmax, int N, int C, int H, int W, int k, int s, int p,
                       hipStream_t st)
{
    const int OH = pool_out_size(H, k, s, p), OW = pool_out_size(W, k, s, p);
    if (OH <= 0 || OW <= 0 || p >= k) return CG_EINVAL;
    if ((uint64_t)N * C >= (1ull << 31) || (uint64_t)H * W >= (1ull << 24)) return CG_EUNSUPPORTED;
    const uint32_t planes = (uint32_t)N * C;
    if (H * W > POOL_LDS) {        // an input plane does not fit the LDS staging
        const uint32_t bpp = ((uint32_t)(OH * OW) + TB - 1) / TB;
        if ((uint64_t)planes * bpp >= (1ull << 31)) return CG_EUNSUPPORTED;
        hipLaunchKernelGGL(maxpool_fwd_direct_kernel, dim3(planes * bpp), dim3(TB), 0, st, x, y, argmax, H, W, OH, OW, k,
                           s, p, bpp, make_fastdiv(bpp), make_fastdiv((uint32_t)OW));
        CG_LAUNCH_CHECK();
    }
    const int ppb = pool_planes_per_block(OH * OW, H * W, POOL_LDS);
    const dim3 grid((planes + ppb - 1) / ppb);
    const size_t lds = ((size_t)ppb * H * W + 4) * sizeof(float);
    const FastDiv divP = make_fastdiv((uint32_t)(OH * OW)), divOW = make_fastdiv((uint32_t)OW);
#define CG_POOL_FWD(K_, S_)                                                                                          \
    hipLaunchKernelGGL((maxpool_fwd_kernel<K_, S_>), grid, dim3(TB), lds, st, x, y, argmax, planes, ppb, H, W, OH, OW, k, \
                       s, p, divP, divOW)
    if (k == 3 && s == 2) CG_POOL_FWD(3, 2);
    else if (k == 3 && s == 1) CG_POOL_FWD(3, 1);
    else if (k == 2 && s == 2) CG_POOL_FWD(2, 2);
    else CG_POOL_FWD(0, 0);
#undef CG_POOL_FWD
    CG_LAUNCH_CHECK();
}

int maxpool_bwd_launch(const float *dy, const int32_t *argmax, float *dx, const float *gate, int N, int C, int H, int W,
                       int k, int s, int p, int accumulate, hipStream_t st)
{
    const int OH = pool_out_size(H, k, s, p), OW = pool_out_size(W, k, s, p);
    if (OH <= 0 || OW <= 0) return CG_EINVAL;
    if ((uint64_t)N * C >= (1ull << 31) || (uint64_t)H * W >= (1ull << 24)) return CG_EUNSUPPORTED;
    const uint32_t planes = (uint32_t)N * C;
    if (OH * OW > POOL_LDS / 2) {  // dy and the winners of a plane do not fit the LDS staging
        const uint32_t bpp = ((uint32_t)(H * W) + TB - 1) / TB;
        if ((uint64_t)planes * bpp >= (1ull << 31)) return CG_EUNSUPPORTED;
        const FastDiv dB = make_fastdiv(bpp), dW = make_fastdiv((uint32_t)W), dS = make_fastdiv((uint32_t)s);
        if (accumulate)
            hipLaunchKernelGGL(maxpool_bwd_direct_kernel<1>, dim3(planes * bpp), dim3(TB), 0, st, dy, argmax, dx, gate, H, W,
                               OH, OW, k, s, p, bpp, dB, dW, dS);
        else
            hipLaunchKernelGGL(maxpool_bwd_direct_kernel<0>, dim3(planes * bpp), dim3(TB), 0, st, dy, argmax, dx, gate, H, W,
                               OH, OW, k, s, p, bpp, dB, dW, dS);
        CG_LAUNCH_CHECK();
    }
    const bool cell = ((k == 3 && (s == 2 || s == 1)) || (k == 2 && s == 2)) && 2 * OH * OW + H * W + 20 <= 2 * POOL_LDS;
    if (cell) {
        // staging of dy and the winners plus an LDS copy of the dx planes
        // about 4096 elements a block, within 20 KB of LDS so that eight blocks share a compute unit
        int ppb = 4096 / (H * W);
        if (ppb < 1) ppb = 1;
        while (ppb > 1 && ppb * (2 * OH * OW + H * W) + 20 > 5120) --ppb;
        const dim3 grid((planes + ppb - 1) / ppb);
        const size_t lds = (2 * (((size_t)ppb * OH * OW + 4 + 3) & ~(size_t)3) + (size_t)ppb * H * W + 4) * sizeof(float);
        const uint32_t CW = (uint32_t)(W + s - 1) / s, CH = (uint32_t)(H + s - 1) / s;
        const FastDiv divCells = make_fastdiv(CW * CH), divCW = make_fastdiv(CW);
#define CG_POOL_CELL(K_, S_)                                                                                         \
    do {                                                                                                             \
        if (accumulate)                                                                                              \
            hipLaunchKernelGGL((maxpool_bwd_cell_kernel<K_, S_, 1>), grid, dim3(TB), lds, st, dy, argmax, dx, gate,   \
                               planes, ppb, H, W, OH, OW, p, divCells, divCW);                                       \
        else                                                                                                         \
            hipLaunchKernelGGL((maxpool_bwd_cell_kernel<K_, S_, 0>), grid, dim3(TB), lds, st, dy, argmax, dx, gate,   \
                               planes, ppb, H, W, OH, OW, p, divCells, divCW);                                       \
    } while (0)
        if (k == 3 && s == 2) CG_POOL_CELL(3, 2);
        else if (k == 3 && s == 1) CG_POOL_CELL(3, 1);
        else CG_POOL_CELL(2, 2);
#undef CG_POOL_CELL
        CG_LAUNCH_CHECK();
    }
    const int ppb = pool_planes_per_block(H * W, OH * OW, POOL_LDS / 2);
    const dim3 grid((planes + ppb - 1) / ppb);
    const size_t lds = 2 * (((size_t)ppb * OH * OW + 4 + 3) & ~(size_t)3) * sizeof(float);
    const FastDiv divQ = make_fastdiv((uint32_t)(H * W)), divW = make_fastdiv((uint32_t)W),
                  divS = make_fastdiv((uint32_t)s);
    if (accumulate)
        hipLaunchKernelGGL((maxpool_bwd_kernel<0, 0, 1>), grid, dim3(TB), lds, st, dy, argmax, dx, gate, planes, ppb, H,
                           W, OH, OW, k, s, p, divQ, divW, divS);
    else
        hipLaunchKernelGGL((maxpool_bwd_kernel<0, 0, 0>), grid, dim3(TB), lds, st, dy, argmax, dx, gate, planes, ppb, H,
                           W, OH, OW, k, s, p, divQ, divW, divS);
    CG_LAUNCH_CHECK();
}

int lrn_fwd_launch(const float *x, float *y, int N, int C, int HW, int size, float alpha, float beta, float kappa,
                   hipStream_t st)
{
    if (size <= 0 || N <= 0 || C <= 0 || HW <= 0) return CG_EINVAL;
    const float aos = alpha / (float)size;
    const int nchunk = (C + LRN_CH - 1) / LRN_CH;
    const dim3 grid(((HW + LRN_V - 1) / LRN_V + TB - 1) / TB, (unsigned)(N * nchunk));
    if (grid.y > 65535u && (size == 3 || size == 5 || size == 7)) return CG_EUNSUPPORTED;
    switch (size) {
    case 3: hipLaunchKernelGGL(lrn_fwd_stream_kernel<3>, grid, dim3(TB), 0, st, x, y, C, HW, nchunk, aos, beta, kappa); break;
    case 5: hipLaunchKernelGGL(lrn_fwd_stream_kernel<5>, grid, dim3(TB), 0, st, x, y, C, HW, nchunk, aos, beta, kappa); break;
    case 7: hipLaunchKernelGGL(lrn_fwd_stream_kernel<7>, grid, dim3(TB), 0, st, x, y, C, HW, nchunk, aos, beta, kappa); break;
    default: {
        const size_t total = (size_t)N * C * HW;
        hipLaunchKernelGGL(lrn_fwd_kernel, dim3(grid_for(total)), dim3(TB), 0, st, x, y, total, C, HW, size, aos, beta,
                           kappa);
    }
    }
    CG_LAUNCH_CHECK();
}

int lrn_bwd_launch(const float *x, const float *dy, float *dx, int N, int C, int HW, int size, float alpha, float beta,
                   float kappa, int accumulate, int gate, hipStream_t st)
{
    if (size <= 0 || N <= 0 || C <= 0 || HW <= 0) return CG_EINVAL;
    const float aos = alpha / (float)size, coef = 2.f * alpha * beta / (float)size;
    const int nchunk = (C + LRN_CH - 1) / LRN_CH;
    const dim3 grid(((HW + LRN_V - 1) / LRN_V + TB - 1) / TB, (unsigned)(N * nchunk));
    if (grid.y > 65535u && (size == 3 || size == 5 || size == 7)) return CG_EUNSUPPORTED;
#define CG_LRN_BWD(SZ)                                                                                                \
    do {                                                                                                              \
        if (accumulate && gate)                                                                                       \
            hipLaunchKernelGGL((lrn_bwd_stream_kernel<SZ, 1, 1>), grid, dim3(TB), 0, st, x, dy, dx, C, HW, nchunk,    \
                               aos, coef, beta, kappa);                                                               \
        else if (accumulate)                                                                                          \
            hipLaunchKernelGGL((lrn_bwd_stream_kernel<SZ, 1, 0>), grid, dim3(TB), 0, st, x, dy, dx, C, HW, nchunk,    \
                               aos, coef, beta, kappa);                                                               \
        else if (gate)                                                                                                \
            hipLaunchKernelGGL((lrn_bwd_stream_kernel<SZ, 0, 1>), grid, dim3(TB), 0, st, x, dy, dx, C, HW, nchunk,    \
                               aos, coef, beta, kappa);                                                               \
        else                                                                                                          \
            hipLaunchKernelGGL((lrn_bwd_stream_kernel<SZ, 0, 0>), grid, dim3(TB), 0, st, x, dy, dx, C, HW, nchunk,    \
                               aos, coef, beta, kappa);                                                               \
    } while (0)
    switch (size) {
    case 3: CG_LRN_BWD(3); break;
    case 5: CG_LRN_BWD(5); break;
    case 7: CG_LRN_BWD(7); break;
    default: {
        const size_t total = (size_t)N * C * HW;
        hipLaunchKernelGGL(lrn_bwd_kernel, dim3(grid_for(total)), dim3(TB), 0, st, x, dy, dx, total, C, HW, size, aos,
                           coef, beta, kappa, accumulate, gate);
    }
    }
#undef CG_LRN_BWD
    CG_LAUNCH_CHECK();
}

// LRN + max-pool in one pass: which layer pairs the fused kernels take (window sizes of the stream
// kernels; the rows of one pool window within a block's 1024 pixels; windows packed into 12 / 4 bits)
static int lrn_pool_fwd_rows(int W, int k, int s) { return ((LRN_V * TB) / W - k) / s + 1; }     // pooled rows per band
bool lrn_pool_fusable(int C, int H, int W, int size, int k, int s, int p)
{
    if (!(size == 3 || size == 5)) return false;
    if (H >= 4096 || W >= 4096 || k <= 0 || s <= 0 || p < 0 || p >= k || C <= 0) return false;
    if ((k + s - 1) / s > 15 || k * W > LRN_V * TB) return false;
    const int OH = pool_out_size(H, k, s, p), OW = pool_out_size(W, k, s, p);
    if (OH <= 0 || OW <= 0) return false;
    // backward: the pooled rows that cover a band of (1024 / W) input rows fit the staging
    const int hrb = (LRN_V * TB) / W < H ? (LRN_V * TB) / W : H;
    return ((hrb + k - 2) / s + 2) * OW <= LP_NP * TB;
}

int lrn_pool_fwd_launch(const float *x, float *y, int32_t *argmax, int N, int C, int H, int W, int size, float alpha,
                        float beta, float kappa, int k, int s, int p, hipStream_t st)
{
    if (!lrn_pool_fusable(C, H, W, size, k, s, p) || N <= 0) return CG_EUNSUPPORTED;
    const int OH = pool_out_size(H, k, s, p), OW = pool_out_size(W, k, s, p);
    const int nchunk = (C + LP_CH - 1) / LP_CH;
    // bands of equal height, as few as fit
    int prb = lrn_pool_fwd_rows(W, k, s);
    const int nbands = (OH + prb - 1) / prb;
    prb = (OH + nbands - 1) / nbands;
    if ((uint64_t)N * nchunk * nbands >= (1ull << 31)) return CG_EUNSUPPORTED;
    const dim3 grid((unsigned)(N * nchunk * nbands));
    const size_t lds = 2 * (size_t)LRN_V * TB * sizeof(float);
    const float aos = alpha / (float)size;
    const FastDiv divOW = make_fastdiv((uint32_t)OW);
    const bool inside = p == 0 && (OH - 1) * s + k <= H && (OW - 1) * s + k <= W;
#define CG_LP_FWD(SZ, K_, S_, IN_)                                                                                    \
    hipLaunchKernelGGL((lrn_pool_fwd_kernel<SZ, K_, S_, IN_>), grid, dim3(TB), lds, st, x, y, argmax, C, H, W, OH, OW, k, \
                       s, p, nchunk, nbands, prb, aos, beta, kappa, divOW)
    if (size == 5 && k == 3 && s == 2 && inside) CG_LP_FWD(5, 3, 2, true);
    else if (size == 5) CG_LP_FWD(5, 0, 0, false);
    else if (k == 3 && s == 2 && inside) CG_LP_FWD(3, 3, 2, true);
    else CG_LP_FWD(3, 0, 0, false);
#undef CG_LP_FWD
    CG_LAUNCH_CHECK();
}

int lrn_pool_bwd_launch(const float *x, const float *dpool, const int32_t *argmax, float *dx, int N, int C, int H, int W,
                        int size, float alpha, float beta, float kappa, int k, int s, int p, int accumulate, int gate,
                        hipStream_t st)
{
    if (!lrn_pool_fusable(C, H, W, size, k, s, p) || N <= 0) return CG_EUNSUPPORTED;
    const int OH = pool_out_size(H, k, s, p), OW = pool_out_size(W, k, s, p);
    const int nchunk = (C + LP_CH - 1) / LP_CH;
    int hrb = (LRN_V * TB) / W;
    const int nbands = (H + hrb - 1) / hrb;
    hrb = (H + nbands - 1) / nbands;
    if ((uint64_t)N * nchunk * nbands >= (1ull << 31)) return CG_EUNSUPPORTED;
    const dim3 grid((unsigned)(N * nchunk * nbands));
    const size_t lds = 4 * (size_t)LP_NP * TB * sizeof(float);
    const float aos = alpha / (float)size, coef = 2.f * alpha * beta / (float)size;
    const FastDiv divW = make_fastdiv((uint32_t)W), divS = make_fastdiv((uint32_t)s);
#define CG_LP_BWD(SZ, A_, GT_)                                                                                        \
    hipLaunchKernelGGL((lrn_pool_bwd_kernel<SZ, A_, GT_>), grid, dim3(TB), lds, st, x, dpool, argmax, dx, C, H, W, OH,  \
                       OW, k, s, p, nchunk, nbands, hrb, aos, coef, beta, kappa, divW, divS)
#define CG_LP_BWD_AG(SZ)                                                                                              \
    do {                                                                                                              \
        if (accumulate && gate) CG_LP_BWD(SZ, 1, 1);                                                                  \
        else if (accumulate) CG_LP_BWD(SZ, 1, 0);                                                                     \
        else if (gate) CG_LP_BWD(SZ, 0, 1);                                                                           \
        else CG_LP_BWD(SZ, 0, 0);                                                                                     \
    } while (0)
    if (size == 3) CG_LP_BWD_AG(3);
    else CG_LP_BWD_AG(5);
#undef CG_LP_BWD_AG
#undef CG_LP_BWD
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

int dropout_launch(const float *x, const uint8_t *mask, float *y, const float *gate, size_t n, float p, int accumulate,
                   hipStream_t st)
{
    if (!mask || p < 0.f || p >= 1.f) return CG_EINVAL;
    if (!aligned16(x) || !aligned16(y) || (reinterpret_cast<uintptr_t>(mask) & 3u)) return CG_EINVAL;
    const float f = 1.f / (1.f - p);
    if (gate && !aligned16(gate)) return CG_EINVAL;
    if (accumulate) hipLaunchKernelGGL(dropout_kernel<1>, dim3(grid_for(n / 4 + 1)), dim3(TB), 0, st, x, mask, y, gate, n, f);
    else hipLaunchKernelGGL(dropout_kernel<0>, dim3(grid_for(n / 4 + 1)), dim3(TB), 0, st, x, mask, y, gate, n, f);
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
                       int accumulate, const float *gate, hipStream_t st)
{
    const size_t total = (size_t)N * Csrc * HW;
    hipLaunchKernelGGL(concat_copy_kernel, dim3(grid_for(total)), dim3(TB), 0, st, src, dst, gate, total, Csrc, Cdst,
                       c_off, HW, to_concat, accumulate);
    CG_LAUNCH_CHECK();
}

}  // namespace cg
