// Convolution and fully-connected passes expressed as implicit-GEMM problems.
//
// Forward:          Y[m][(n,oh,ow)]   = sum_{(c,kh,kw)} W[m][(c,kh,kw)] * X(n,c,oh*s-p+kh,ow*s-p+kw)
// Backward-data:    dX[c][(n,ih,iw)]  = sum_{(m,kh,kw)} Wt[c][(m,kh,kw)] * dY(n,m,(ih+p-kh)/s,(iw+p-kw)/s)
// Backward-weight:  dW[m][(c,kh,kw)]  = sum_{(n,oh,ow)} dY[m][(n,oh,ow)] * X(n,c,oh*s-p+kh,ow*s-p+kw)
// (section 2.1: forward propagation, backward propagation, gradient on the weights; the last
// one is the first step of every turn in Fig. 3).
#include <mutex>
#include "cg_internal.h"

namespace cg {

namespace {

size_t round256(size_t v) { return (v + 255) / 256 * 256; }

// input pixel grid seen through the filter: index (n, oh, ow) -> window origin in x
IndexMap window_origin_map(const cg_conv_desc &d, int OH, int OW)
{
    IndexMap m{};
    m.count = (uint32_t)d.N * OH * OW;
    m.d1 = make_fastdiv((uint32_t)OH * OW);
    m.d2 = make_fastdiv((uint32_t)OW);
    m.s1 = d.C * d.H * d.W;
    m.s2 = d.stride_h * d.W;
    m.s3 = d.stride_w;
    m.o0 = -d.pad_h * d.W - d.pad_w;
    m.sa = d.stride_h; m.a0 = -d.pad_h;
    m.sb = d.stride_w; m.b0 = -d.pad_w;
    return m;
}

// filter tap index (c, kh, kw) -> displacement inside x
IndexMap tap_map(const cg_conv_desc &d, int Cg)
{
    IndexMap m{};
    m.count = (uint32_t)Cg * d.KH * d.KW;
    m.d1 = make_fastdiv((uint32_t)d.KH * d.KW);
    m.d2 = make_fastdiv((uint32_t)d.KW);
    m.s1 = d.H * d.W;
    m.s2 = d.W;
    m.s3 = 1;
    m.sa = 1; m.sb = 1;
    return m;
}

// wt[g][c][ml][kh][kw] = w[g*Mg + ml][c][kh][kw]: the filters as the row-major matrix that
// backward-data multiplies with (rows = input channels, reduction index = (ml, kh, kw))
__device__ __forceinline__ float transpose_filters_elem(const float *__restrict__ w, size_t i, int Mg, int Cg, int KK)
{
    const int kk = (int)(i % KK);
    size_t r = i / KK;
    const int ml = (int)(r % Mg); r /= Mg;
    const int c = (int)(r % Cg);
    const int g = (int)(r / Cg);
    return w[(((size_t)g * Mg + ml) * Cg + c) * KK + kk];
}

// Filters as the tap-major matrix the patch kernel multiplies with: dst[g][r][t][c], t = kh*KW + kw.
// Forward (bwd = 0): r = output channel, c = input channel: dst = w[g*Mg + r][c][t].
// Backward-data (bwd = 1): r = input channel, c = output channel: dst = w[g*Mg + c][r][t].
__device__ __forceinline__ float permute_filters_elem(const float *__restrict__ w, size_t i, int Mg, int Cg, int KK, int bwd)
{
    const int R = bwd ? Cg : Mg, Cr = bwd ? Mg : Cg;
    const int c = (int)(i % Cr);
    size_t q = i / Cr;
    const int t = (int)(q % KK); q /= KK;
    const int r = (int)(q % R);
    const int g = (int)(q / R);
    const int m = bwd ? c : r, ci = bwd ? r : c;
    return w[(((size_t)g * Mg + m) * Cg + ci) * KK + t];
}

// Filters as the matrix of strided backward-data (see bwd_data_strided_problem): row (c, rh, rw),
// reduction index (m, a, b) with filter tap kh = rh + sh*a, kw = rw + sw*b (zero where that tap
// does not exist).  tap_major = 1: dst[g][row][t = a*Aw + b][m] (the patch kernel's order);
// 0: dst[g][row][m][t] (the gathered kernel's).
__device__ __forceinline__ float strided_filters_elem(const float *__restrict__ w, size_t i, int Mg, int Cg, int KH, int KW,
                                                      int sh, int sw, int Ah, int Aw, int tap_major)
{
    const int R = Cg * sh * sw, T = Ah * Aw;
    int m, t;
    size_t q;
    if (tap_major) { m = (int)(i % Mg); q = i / Mg; t = (int)(q % T); q /= T; }
    else { t = (int)(i % T); q = i / T; m = (int)(q % Mg); q /= Mg; }
    const int row = (int)(q % R), g = (int)(q / R);
    const int rw = row % sw, rh = (row / sw) % sh, c = row / (sw * sh);
    const int kh = rh + sh * (t / Aw), kw = rw + sw * (t % Aw);
    return (kh < KH && kw < KW) ? w[(((size_t)g * Mg + m) * Cg + c) * KH * KW + kh * KW + kw] : 0.f;
}

__global__ __launch_bounds__(256) void transpose_filters_kernel(const float *__restrict__ w, float *__restrict__ wt,
                                                                int G, int Mg, int Cg, int KK)
{
    const size_t total = (size_t)G * Mg * Cg * KK;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256)
        wt[i] = transpose_filters_elem(w, i, Mg, Cg, KK);
}

__global__ __launch_bounds__(256) void permute_filters_kernel(const float *__restrict__ w, float *__restrict__ dst,
                                                              int G, int Mg, int Cg, int KK, int bwd)
{
    const size_t total = (size_t)G * Mg * Cg * KK;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256)
        dst[i] = permute_filters_elem(w, i, Mg, Cg, KK, bwd);
}

__global__ __launch_bounds__(256) void strided_filters_kernel(const float *__restrict__ w, float *__restrict__ dst,
                                                              int G, int Mg, int Cg, int KH, int KW, int sh, int sw,
                                                              int Ah, int Aw, int tap_major)
{
    const size_t total = (size_t)G * (Cg * sh * sw) * (Ah * Aw) * Mg;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256)
        dst[i] = strided_filters_elem(w, i, Mg, Cg, KH, KW, sh, sw, Ah, Aw, tap_major);
}

// The rearranged filters of several layers in one launch (a net prepares those of all its layers at
// the start of an iteration): block b belongs to the job whose [first_block, ...) range holds it and
// writes 1024 consecutive elements of that job's copy.
constexpr int kPrepJobs = 8;
struct PrepJob {
    const float *w;
    float *dst;
    int kind, Mg, Cg, KH, KW, sh, sw, Ah, Aw;
    unsigned first_block;
    unsigned long long total;
};
struct PrepTable {
    PrepJob j[kPrepJobs];
    int n;
};
__global__ __launch_bounds__(256) void prepare_filters_kernel(const PrepTable t)
{
    int ji = 0;
#pragma unroll
    for (int k = 1; k < kPrepJobs; ++k)
        if (k < t.n && blockIdx.x >= t.j[k].first_block) ji = k;
    const PrepJob &jb = t.j[ji];
    const size_t base = (size_t)(blockIdx.x - jb.first_block) * 1024 + threadIdx.x;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const size_t i = base + (size_t)u * 256;
        if (i >= jb.total) break;
        float v;
        if (jb.kind == CG_PREP_TRANSPOSE) v = transpose_filters_elem(jb.w, i, jb.Mg, jb.Cg, jb.KH * jb.KW);
        else if (jb.kind == CG_PREP_PERMUTE_FWD) v = permute_filters_elem(jb.w, i, jb.Mg, jb.Cg, jb.KH * jb.KW, 0);
        else if (jb.kind == CG_PREP_PERMUTE_BWD) v = permute_filters_elem(jb.w, i, jb.Mg, jb.Cg, jb.KH * jb.KW, 1);
        else v = strided_filters_elem(jb.w, i, jb.Mg, jb.Cg, jb.KH, jb.KW, jb.sh, jb.sw, jb.Ah, jb.Aw,
                                      jb.kind == CG_PREP_STRIDED_TAPS ? 1 : 0);
        jb.dst[i] = v;
    }
}

// General-stride backward-data, gather form, one thread per dx element.  Only the taps with
// (ih + p - kh) divisible by the stride contribute.
__global__ __launch_bounds__(256) void bwd_data_strided_kernel(const cg_conv_desc d, int OH, int OW,
                                                               const float *__restrict__ dy,
                                                               const float *__restrict__ w, float *__restrict__ dx,
                                                               const float *__restrict__ gate, int accumulate)
{
    const int Cg = d.C / d.groups, Mg = d.M / d.groups;
    const size_t total = (size_t)d.N * d.C * d.H * d.W;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
        const int iw = (int)(i % d.W);
        size_t r = i / d.W;
        const int ih = (int)(r % d.H); r /= d.H;
        const int c = (int)(r % d.C);
        const int n = (int)(r / d.C);
        const int g = c / Cg, cl = c - g * Cg;
        float s = 0.f;
        const int kh0 = (ih + d.pad_h) % d.stride_h, kw0 = (iw + d.pad_w) % d.stride_w;
        for (int ml = 0; ml < Mg; ++ml) {
            const int m = g * Mg + ml;
            const float *wp = w + ((size_t)m * Cg + cl) * d.KH * d.KW;
            const float *yp = dy + ((size_t)n * d.M + m) * OH * OW;
            for (int kh = kh0; kh < d.KH; kh += d.stride_h) {
                const int oh = (ih + d.pad_h - kh) / d.stride_h;
                if (ih + d.pad_h - kh < 0 || oh >= OH) continue;
                for (int kw = kw0; kw < d.KW; kw += d.stride_w) {
                    const int ow = (iw + d.pad_w - kw) / d.stride_w;
                    if (iw + d.pad_w - kw < 0 || ow >= OW) continue;
                    s += yp[oh * OW + ow] * wp[kh * d.KW + kw];
                }
            }
        }
        if (gate && !(gate[i] > 0.f)) s = 0.f;
        dx[i] = accumulate ? dx[i] + s : s;
    }
}

// Backward-data for strides > 1, by stride phase.  The input pixels with (ih mod s_h, iw mod s_w) =
// (rh, rw) all see the same filter taps, kh = kh0 + s_h*a and kw = kw0 + s_w*b, and reach dy at
// oh = ih' + qh - a, ow = iw' + qw - b for ih = s_h*ih' + rh: a stride-1 correlation of dy with the
// sub-sampled filter.  A block owns one phase, 16 x 16 of its pixels, one image and CT input
// channels of one group; it walks the group's output channels 16 at a time, with the dy window of
// the tile (zeros outside dy) and the phase's taps of the 16 filters (zeros for taps a phase does
// not have) staged in LDS, and every thread accumulates its pixel for the CT channels over a fixed
// AM x AM sweep, AM = the most taps per dimension any phase has.
// Made for few input channels per group (the first layer of a net: 3), where a matrix-core tile
// would multiply mostly padding; more channels take several blocks, each re-reading dy.  Plain
// vector arithmetic: about a third of the issued instructions are useful multiply-adds (the 11x11
// stride-4 layer at B = 256: 4.9 ms, 11 TFLOP/s; variants that shared the dy window between the
// phases of a block were slower, this kernel is bound by instruction issue, not by memory).
constexpr int PH_T = 16;          // tile edge in phase pixels
constexpr int PH_MC = 16;         // output channels per LDS stage

template <int CT, int AM>
__global__ __launch_bounds__(256) void bwd_data_phase_kernel(const cg_conv_desc d, int OH, int OW,
                                                             const float *__restrict__ dy,
                                                             const float *__restrict__ w, float *__restrict__ dx,
                                                             const float *__restrict__ gate, int accumulate, int tiles_x,
                                                             int chunks)
{
    constexpr int WT = PH_T + AM - 1, TAPS = AM * AM, TP = (TAPS + 3) / 4 * 4;
    __shared__ float dys[PH_MC * WT * WT];
    __shared__ __align__(16) float wsm[PH_MC * CT * TP];
    const int Cg = d.C / d.groups, Mg = d.M / d.groups, KK = d.KH * d.KW;
    const int tile_y = blockIdx.x / tiles_x, tile_x = blockIdx.x % tiles_x;
    const int rh = blockIdx.y / d.stride_w, rw = blockIdx.y % d.stride_w;
    int z = blockIdx.z;
    const int chunk = z % chunks; z /= chunks;
    const int g = z % d.groups, n = z / d.groups;
    const int c0 = chunk * CT;
    // taps and dy displacement of this phase
    const int kh0 = (rh + d.pad_h) % d.stride_h, kw0 = (rw + d.pad_w) % d.stride_w;
    const int qh = (rh + d.pad_h) / d.stride_h, qw = (rw + d.pad_w) / d.stride_w;
    const int ty = threadIdx.x / PH_T, tx = threadIdx.x % PH_T;
    const int oh_base = tile_y * PH_T + qh - (AM - 1), ow_base = tile_x * PH_T + qw - (AM - 1);
    float acc[CT];
#pragma unroll
    for (int c = 0; c < CT; ++c) acc[c] = 0.f;
    for (int m0 = 0; m0 < Mg; m0 += PH_MC) {
        const int mc = min(PH_MC, Mg - m0);
        __syncthreads();
        for (int i = threadIdx.x; i < PH_MC * WT * WT; i += 256) {
            const int ml = i / (WT * WT), r = i - ml * (WT * WT), wy = r / WT, wx = r - wy * WT;
            const int oh = oh_base + wy, ow = ow_base + wx;
            float v = 0.f;
            if (ml < mc && (unsigned)oh < (unsigned)OH && (unsigned)ow < (unsigned)OW)
                v = dy[(((size_t)n * d.M + g * Mg + m0 + ml) * OH + oh) * OW + ow];
            dys[i] = v;
        }
        for (int i = threadIdx.x; i < PH_MC * CT * TP; i += 256) {
            const int ml = i / (CT * TP), r = i - ml * (CT * TP), c = r / TP, t = r - c * TP;
            const int kh = kh0 + (t / AM) * d.stride_h, kw = kw0 + (t % AM) * d.stride_w;
            float v = 0.f;
            if (ml < mc && c0 + c < Cg && t < TAPS && kh < d.KH && kw < d.KW)
                v = w[((size_t)(g * Mg + m0 + ml) * Cg + c0 + c) * KK + kh * d.KW + kw];
            wsm[i] = v;
        }
        __syncthreads();
#pragma unroll 2
        for (int ml = 0; ml < PH_MC; ++ml) {          // channels beyond mc are staged as zeros
            const float *dp = dys + ml * (WT * WT) + (ty + AM - 1) * WT + (tx + AM - 1);
            float v[TP];
#pragma unroll
            for (int t = 0; t < TP; ++t)              // a tap the phase does not have reads nothing (its weight is 0)
                v[t] = (t < TAPS && kh0 + (t / AM) * d.stride_h < d.KH && kw0 + (t % AM) * d.stride_w < d.KW)
                           ? dp[-(t / AM) * WT - (t % AM)] : 0.f;
#pragma unroll
            for (int c = 0; c < CT; ++c) {
                const float4 *wq = reinterpret_cast<const float4 *>(wsm + (ml * CT + c) * TP);
#pragma unroll
                for (int t4 = 0; t4 < TP / 4; ++t4) {
                    const float4 q = wq[t4];
                    acc[c] += v[4 * t4] * q.x;
                    acc[c] += v[4 * t4 + 1] * q.y;
                    acc[c] += v[4 * t4 + 2] * q.z;
                    acc[c] += v[4 * t4 + 3] * q.w;
                }
            }
        }
    }
    const int ih = (tile_y * PH_T + ty) * d.stride_h + rh, iw = (tile_x * PH_T + tx) * d.stride_w + rw;
    if (ih < d.H && iw < d.W) {
#pragma unroll
        for (int c = 0; c < CT; ++c) {
            if (c0 + c >= Cg) continue;
            const size_t i = (((size_t)n * d.C + g * Cg + c0 + c) * d.H + ih) * d.W + iw;
            float v = acc[c];
            if (gate && !(gate[i] > 0.f)) v = 0.f;
            dx[i] = accumulate ? dx[i] + v : v;
        }
    }
}

}  // namespace

int conv_check(const cg_conv_desc *d, int *OH, int *OW)
{
    if (!d) return CG_EINVAL;
    if (d->N <= 0 || d->C <= 0 || d->H <= 0 || d->W <= 0 || d->M <= 0 || d->KH <= 0 || d->KW <= 0 ||
        d->stride_h <= 0 || d->stride_w <= 0 || d->pad_h < 0 || d->pad_w < 0 || d->groups <= 0)
        return CG_EINVAL;
    if (d->C % d->groups || d->M % d->groups) return CG_EINVAL;
    const int eh = d->H + 2 * d->pad_h - d->KH, ew = d->W + 2 * d->pad_w - d->KW;
    if (eh < 0 || ew < 0) return CG_EINVAL;
    const int oh = eh / d->stride_h + 1, ow = ew / d->stride_w + 1;
    const uint64_t lim = (1ull << 31) / 4;   // elements per tensor
    if ((uint64_t)d->N * d->C * d->H * d->W >= lim || (uint64_t)d->N * d->M * oh * ow >= lim ||
        (uint64_t)d->M * (d->C / d->groups) * d->KH * d->KW >= lim)
        return CG_EUNSUPPORTED;
    if (d->KH > 4096 || d->KW > 4096 || d->H > (1 << 20) || d->W > (1 << 20)) return CG_EUNSUPPORTED;
    if (OH) *OH = oh;
    if (OW) *OW = ow;
    return CG_OK;
}

static IgemmProblem fwd_problem(const cg_conv_desc &d, int OH, int OW, const float *x, const float *w,
                                const float *bias, float *y, int64_t y_img_stride = 0)
{
    const int G = d.groups, Cg = d.C / G, Mg = d.M / G, Kg = Cg * d.KH * d.KW, P = OH * OW;
    IgemmProblem p{};
    p.A.ptr = w;
    p.A.row = linear_map(Mg, Kg);
    p.A.k = linear_map(Kg, 1);
    p.A.limA = p.A.limB = 1;
    p.A.gstride = (int64_t)Mg * Kg;
    p.A.elems = (uint64_t)d.M * Kg;
    p.A.lanes_k = 1;
    p.B.ptr = x;
    p.B.row = window_origin_map(d, OH, OW);
    p.B.k = tap_map(d, Cg);
    p.B.limA = d.H; p.B.limB = d.W;
    p.B.gstride = (int64_t)Cg * d.H * d.W;
    p.B.elems = (uint64_t)d.N * d.C * d.H * d.W;
    p.B.lanes_k = 0;
    p.B.check = (d.pad_h || d.pad_w) ? 1 : 0;
    p.c_ptr = y;
    p.c_row_stride = P;
    p.c_col = split_map((uint32_t)d.N * P, P, y_img_stride ? (int32_t)y_img_stride : d.M * P, 1);
    p.c_gstride = (int64_t)Mg * P;
    p.bias = bias; p.bias_mode = bias ? 1 : 0; p.bias_gstride = Mg;
    p.M = Mg; p.N = (uint32_t)d.N * P; p.K = Kg;
    p.groups = G; p.splits = 1; p.k_per_split = p.K;
    return p;
}

// Describes x as the patch operand of the forward pass; true if the patch kernel can run it.
static bool fwd_patch(const cg_conv_desc &d, int OH, int OW, const float *x, IgemmProblem &p)
{
    if (d.stride_h != d.stride_w) return false;
    const int G = d.groups, Cg = d.C / G;
    PatchGeom g{};
    g.src = x; g.src_elems = (uint64_t)d.N * d.C * d.H * d.W;
    g.gstride = (int64_t)Cg * d.H * d.W;
    g.Cred = (uint32_t)Cg; g.Hs = d.H; g.Ws = d.W; g.chan_stride = d.H * d.W; g.img_stride = d.C * d.H * d.W;
    g.OHo = OH; g.OWo = OW; g.s = d.stride_h; g.oy0 = -d.pad_h; g.ox0 = -d.pad_w; g.KH = d.KH; g.KW = d.KW; g.flip = 0;
    if (!patch_plan(g, (uint32_t)(d.M / G), (uint32_t)d.N * OH * OW, (uint32_t)G)) return false;
    p.patch = g; p.use_patch = 1;
    return true;
}

// dy as the patch operand of backward-data at stride 1 (pixels = input positions, mirrored taps)
static bool bwd_data_patch(const cg_conv_desc &d, int OH, int OW, const float *dy, IgemmProblem &p)
{
    const int G = d.groups, Mg = d.M / G;
    PatchGeom g{};
    g.src = dy; g.src_elems = (uint64_t)d.N * d.M * OH * OW;
    g.gstride = (int64_t)Mg * OH * OW;
    g.Cred = (uint32_t)Mg; g.Hs = OH; g.Ws = OW; g.chan_stride = OH * OW; g.img_stride = d.M * OH * OW;
    g.OHo = d.H; g.OWo = d.W; g.s = 1; g.oy0 = d.pad_h - (d.KH - 1); g.ox0 = d.pad_w - (d.KW - 1);
    g.KH = d.KH; g.KW = d.KW; g.flip = 1;
    if (!patch_plan(g, (uint32_t)(d.C / G), (uint32_t)d.N * d.H * d.W, (uint32_t)G)) return false;
    p.patch = g; p.use_patch = 1;
    return true;
}

static int permute_filters(const float *w, float *dst, int G, int Mg, int Cg, int KK, int bwd, hipStream_t stream)
{
    const size_t total = (size_t)G * Mg * Cg * KK;
    const unsigned blocks = (unsigned)((total + 255) / 256 < 4096 ? (total + 255) / 256 : 4096);
    hipLaunchKernelGGL(permute_filters_kernel, dim3(blocks), dim3(256), 0, stream, w, dst, G, Mg, Cg, KK, bwd);
    CG_HIP_TRY(hipGetLastError());
    return CG_OK;
}

// operand A = a plain row-major [rows][K] matrix per group
static void tap_major_filters(IgemmProblem &p, const float *m, int rows, int K, uint64_t elems)
{
    p.A = Operand{};
    p.A.ptr = m;
    p.A.row = linear_map((uint32_t)rows, K);
    p.A.k = linear_map((uint32_t)K, 1);
    p.A.limA = p.A.limB = 1;
    p.A.gstride = (int64_t)rows * K;
    p.A.elems = elems;
    p.A.lanes_k = 1;
}

static bool math_ok(int math) { return math == CG_MATH_FP32 || math == CG_MATH_BF16 || math == CG_MATH_BF16X3; }

int conv_fwd_impl(const cg_conv_desc &d, const float *x, const float *w, const float *bias, float *y, void *ws,
                  size_t ws_bytes, int relu, hipStream_t stream, int64_t y_img_stride, int math, const float *prepared)
{
    if (!math_ok(math)) return CG_EINVAL;
    ProfTag tag("conv_fwd", -1);
    int OH, OW;
    const int rc = conv_check(&d, &OH, &OW);
    if (rc) return rc;
    // y_img_stride: elements between the images of y when y is a channel slice of a wider tensor
    // (0 = dense, M*OH*OW); the whole wider tensor must stay below 2^31 elements
    if (y_img_stride < 0 || (y_img_stride && (y_img_stride < (int64_t)d.M * OH * OW ||
                                              y_img_stride * (int64_t)d.N >= (1ll << 31)))) return CG_EINVAL;
    IgemmProblem p = fwd_problem(d, OH, OW, x, w, bias, y, y_img_stride);
    p.relu = relu;
    p.math = math;
    if (fwd_patch(d, OH, OW, x, p)) {
        const int G = d.groups, Cg = d.C / G, Mg = d.M / G, KK = d.KH * d.KW;
        const size_t wt_bytes = round256((size_t)d.M * Cg * KK * sizeof(float));
        if (!ws || ws_bytes < wt_bytes) return CG_ENOSPC;
        if (!aligned16(ws)) return CG_EINVAL;
        if (!prepared) {
            const int rc2 = permute_filters(w, static_cast<float *>(ws), G, Mg, Cg, KK, 0, stream);
            if (rc2) return rc2;
        }
        tap_major_filters(p, prepared ? prepared : static_cast<const float *>(ws), Mg, Cg * KK, (uint64_t)d.M * Cg * KK);
        return igemm_run(p, static_cast<char *>(ws) + wt_bytes, ws_bytes - wt_bytes, stream);
    }
    return igemm_run(p, ws, ws_bytes, stream);
}

// A 1x1 window without padding at stride 1: backward-data is the plain product of the transposed
// filter matrix with dy, and the transposed matrix can be read from w with the loader that runs the
// row index along the lanes (as the fully-connected layers do), so no transposed copy is made.
static bool bwd_data_reads_filters_in_place(const cg_conv_desc &d)
{
    return d.KH == 1 && d.KW == 1 && d.pad_h == 0 && d.pad_w == 0 && d.stride_h == 1 && d.stride_w == 1;
}

static IgemmProblem bwd_data_problem(const cg_conv_desc &d, int OH, int OW, const float *dy, const float *wt,
                                     float *dx, int accumulate)
{
    const int G = d.groups, Cg = d.C / G, Mg = d.M / G, KK = d.KH * d.KW, P = OH * OW;
    const int Kp = Mg * KK;
    IgemmProblem p{};
    p.A.ptr = wt;
    p.A.row = linear_map(Cg, Kp);
    p.A.k = linear_map(Kp, 1);
    p.A.limA = p.A.limB = 1;
    p.A.gstride = (int64_t)Cg * Kp;
    p.A.elems = (uint64_t)d.M * Cg * KK;
    p.A.lanes_k = 1;
    if (bwd_data_reads_filters_in_place(d)) {
        // one tap: A(c, m) is w[m][c] itself, rows (input channels) along the lanes -- `wt` is then w
        p.A.row = linear_map(Cg, 1);
        p.A.k = linear_map(Mg, Cg);
        p.A.lanes_k = 0;
    }
    // dy seen from an input pixel (n, ih, iw): origin (ih + p, iw + p), taps subtract (kh, kw)
    p.B.ptr = dy;
    IndexMap pix{};
    pix.count = (uint32_t)d.N * d.H * d.W;
    pix.d1 = make_fastdiv((uint32_t)d.H * d.W);
    pix.d2 = make_fastdiv((uint32_t)d.W);
    pix.s1 = d.M * P; pix.s2 = OW; pix.s3 = 1; pix.o0 = d.pad_h * OW + d.pad_w;
    pix.sa = 1; pix.a0 = d.pad_h; pix.sb = 1; pix.b0 = d.pad_w;
    IndexMap tap{};
    tap.count = (uint32_t)Kp;
    tap.d1 = make_fastdiv((uint32_t)KK);
    tap.d2 = make_fastdiv((uint32_t)d.KW);
    tap.s1 = P; tap.s2 = -OW; tap.s3 = -1;
    tap.sa = -1; tap.sb = -1;
    p.B.row = pix; p.B.k = tap;
    p.B.limA = OH; p.B.limB = OW;
    p.B.gstride = (int64_t)Mg * P;
    p.B.elems = (uint64_t)d.N * d.M * P;
    p.B.lanes_k = 0;
    p.B.check = (KK > 1 || d.pad_h || d.pad_w) ? 1 : 0;
    const int HW = d.H * d.W;
    p.c_ptr = dx;
    p.c_row_stride = HW;
    p.c_col = split_map((uint32_t)d.N * HW, HW, d.C * HW, 1);
    p.c_gstride = (int64_t)Cg * HW;
    p.M = Cg; p.N = (uint32_t)d.N * HW; p.K = Kp;
    p.groups = G; p.splits = 1; p.k_per_split = p.K;
    p.accumulate = accumulate;
    return p;
}

// Backward-data of a convolution with stride (sh, sw) > 1 as ONE stride-1 problem on the matrix
// cores.  Write an input row as ih + ph = sh*i + rh (cell i, phase rh < sh).  Only the taps
// kh = rh + sh*a reach it, from output row oh = i - a, so
//   dx[n, c, sh*i + rh - ph, sw*j + rw - pw] = sum_{m, a, b} dy[n, m, i - a, j - b] * w[m, c, rh + sh*a, rw + sw*b]:
// a correlation of dy with Ah x Aw = ceil(KH/sh) x ceil(KW/sw) taps whose "output channels" are the
// Cg * sh * sw pairs (channel, phase), the filters rearranged accordingly (zeros for taps beyond
// the window), and whose result is scattered cell by cell into dx (depth to space; phases outside
// the image are dropped).  Every dx element is the row/column pair of exactly one cell and phase,
// so dx is overwritten completely.  The first layer of the benchmark net (3 channels, 11x11,
// stride 4) becomes 48 rows x 864 reduction indices, of which 121/144 multiply a real tap.
struct StridedGeom { int sh, sw, Ah, Aw, Ch, Cw, R, Kp; uint32_t Np; };

static bool strided_geom(const cg_conv_desc &d, StridedGeom &s)
{
    s.sh = d.stride_h; s.sw = d.stride_w;
    s.Ah = (d.KH + s.sh - 1) / s.sh; s.Aw = (d.KW + s.sw - 1) / s.sw;
    s.Ch = (d.H - 1 + d.pad_h) / s.sh + 1; s.Cw = (d.W - 1 + d.pad_w) / s.sw + 1;
    const int64_t R = (int64_t)(d.C / d.groups) * s.sh * s.sw, Kp = (int64_t)(d.M / d.groups) * s.Ah * s.Aw;
    const int64_t Np = (int64_t)d.N * s.Ch * s.Cw;
    if (R < 8 || R >= (1 << 20) || Kp >= (1 << 28) || Np >= (1ll << 30) || R * Kp * d.groups >= (1ll << 29)) return false;
    s.R = (int)R; s.Kp = (int)Kp; s.Np = (uint32_t)Np;
    return true;
}

static IgemmProblem bwd_data_strided_problem(const cg_conv_desc &d, const StridedGeom &sg, int OH, int OW, const float *dy,
                                             const float *wt, float *dx, int accumulate)
{
    const int G = d.groups, Cg = d.C / G, Mg = d.M / G, P = OH * OW, T = sg.Ah * sg.Aw;
    IgemmProblem p{};
    p.A.ptr = wt;
    p.A.row = linear_map((uint32_t)sg.R, sg.Kp);
    p.A.k = linear_map((uint32_t)sg.Kp, 1);
    p.A.limA = p.A.limB = 1;
    p.A.gstride = (int64_t)sg.R * sg.Kp;
    p.A.elems = (uint64_t)G * sg.R * sg.Kp;
    p.A.lanes_k = 1;
    // dy seen from a cell (n, i, j): origin (i, j), tap (m, a, b) subtracts (a, b)
    p.B.ptr = dy;
    IndexMap cell{};
    cell.count = sg.Np;
    cell.d1 = make_fastdiv((uint32_t)sg.Ch * sg.Cw);
    cell.d2 = make_fastdiv((uint32_t)sg.Cw);
    cell.s1 = d.M * P; cell.s2 = OW; cell.s3 = 1;
    cell.sa = 1; cell.sb = 1;
    IndexMap tap{};
    tap.count = (uint32_t)sg.Kp;
    tap.d1 = make_fastdiv((uint32_t)T);
    tap.d2 = make_fastdiv((uint32_t)sg.Aw);
    tap.s1 = P; tap.s2 = -OW; tap.s3 = -1;
    tap.sa = -1; tap.sb = -1;
    p.B.row = cell; p.B.k = tap;
    p.B.limA = OH; p.B.limB = OW;
    p.B.gstride = (int64_t)Mg * P;
    p.B.elems = (uint64_t)d.N * d.M * P;
    p.B.lanes_k = 0;
    p.B.check = 1;
    // C: row (c, rh, rw) and cell (n, i, j) -> dx[n, c, sh*i + rh - ph, sw*j + rw - pw]
    const int HW = d.H * d.W;
    p.c_ptr = dx;
    p.c_scatter = 1;
    p.c_row = IndexMap{};
    p.c_row.count = (uint32_t)sg.R;
    p.c_row.d1 = make_fastdiv((uint32_t)sg.sh * sg.sw);
    p.c_row.d2 = make_fastdiv((uint32_t)sg.sw);
    p.c_row.s1 = HW; p.c_row.s2 = d.W; p.c_row.s3 = 1; p.c_row.o0 = -d.pad_h * d.W - d.pad_w;
    p.c_row.sa = 1; p.c_row.a0 = -d.pad_h; p.c_row.sb = 1; p.c_row.b0 = -d.pad_w;
    p.c_col = IndexMap{};
    p.c_col.count = sg.Np;
    p.c_col.d1 = make_fastdiv((uint32_t)sg.Ch * sg.Cw);
    p.c_col.d2 = make_fastdiv((uint32_t)sg.Cw);
    p.c_col.s1 = d.C * HW; p.c_col.s2 = sg.sh * d.W; p.c_col.s3 = sg.sw;
    p.c_col.sa = sg.sh; p.c_col.sb = sg.sw;
    p.c_limA = d.H; p.c_limB = d.W;
    p.c_gstride = (int64_t)Cg * HW;
    p.M = (uint32_t)sg.R; p.N = sg.Np; p.K = (uint32_t)sg.Kp;
    p.flops = 2.0 * Mg * Cg * d.KH * d.KW * ((double)d.N * P) * G;
    p.groups = G; p.splits = 1; p.k_per_split = p.K;
    p.accumulate = accumulate;
    return p;
}

// dy as the patch operand of that problem: cells are the pixels, the taps are mirrored
static bool bwd_data_strided_patch(const cg_conv_desc &d, const StridedGeom &sg, int OH, int OW, const float *dy,
                                   IgemmProblem &p)
{
    const int G = d.groups, Mg = d.M / G;
    PatchGeom g{};
    g.src = dy; g.src_elems = (uint64_t)d.N * d.M * OH * OW;
    g.gstride = (int64_t)Mg * OH * OW;
    g.Cred = (uint32_t)Mg; g.Hs = OH; g.Ws = OW; g.chan_stride = OH * OW; g.img_stride = d.M * OH * OW;
    g.OHo = sg.Ch; g.OWo = sg.Cw; g.s = 1; g.oy0 = -(sg.Ah - 1); g.ox0 = -(sg.Aw - 1);
    g.KH = sg.Ah; g.KW = sg.Aw; g.flip = 1;
    if (!patch_plan(g, (uint32_t)sg.R, sg.Np, (uint32_t)G)) return false;
    p.patch = g; p.use_patch = 1;
    return true;
}

static int strided_filters(const float *w, float *dst, const cg_conv_desc &d, const StridedGeom &sg, int tap_major,
                           hipStream_t stream)
{
    const int G = d.groups;
    const size_t total = (size_t)G * sg.R * sg.Kp;
    const unsigned blocks = (unsigned)((total + 255) / 256 < 4096 ? (total + 255) / 256 : 4096);
    hipLaunchKernelGGL(strided_filters_kernel, dim3(blocks), dim3(256), 0, stream, w, dst, G, d.M / G, d.C / G, d.KH, d.KW,
                       sg.sh, sg.sw, sg.Ah, sg.Aw, tap_major);
    CG_HIP_TRY(hipGetLastError());
    return CG_OK;
}

int conv_bwd_data_impl(const cg_conv_desc &d, const float *dy, const float *w, float *dx, const float *gate, void *ws,
                       size_t ws_bytes, int accumulate, hipStream_t stream, int math, const float *prepared,
                       bool beside_other_stream)
{
    if (!math_ok(math)) return CG_EINVAL;
    ProfTag tag("conv_bwd_data", -1);
    int OH, OW;
    const int rc = conv_check(&d, &OH, &OW);
    if (rc) return rc;
    StridedGeom sg;
    if ((d.stride_h != 1 || d.stride_w != 1) && strided_geom(d, sg)) {
        const size_t wt_bytes = round256((size_t)d.groups * sg.R * sg.Kp * sizeof(float));
        if (!ws || ws_bytes < wt_bytes) return CG_ENOSPC;
        if (!aligned16(ws)) return CG_EINVAL;
        float *wt = static_cast<float *>(ws);
        IgemmProblem p = bwd_data_strided_problem(d, sg, OH, OW, dy, prepared ? prepared : wt, dx, accumulate);
        p.gate = gate;
        p.math = math;
        const bool patch = bwd_data_strided_patch(d, sg, OH, OW, dy, p);
        if (!prepared) {
            const int rc2 = strided_filters(w, wt, d, sg, patch ? 1 : 0, stream);
            if (rc2) return rc2;
        }
        return igemm_run(p, static_cast<char *>(ws) + wt_bytes, ws_bytes - wt_bytes, stream);
    }
    if ((d.stride_h != 1 || d.stride_w != 1) && math != CG_MATH_FP32) return CG_EUNSUPPORTED;   // plain vector arithmetic below
    if (d.stride_h != 1 || d.stride_w != 1) {
        // few rows (channels x phases): by stride phase, for at most four taps per dimension and phase
        const int Cg = d.C / d.groups;
        const int Ahm = (d.KH + d.stride_h - 1) / d.stride_h, Awm = (d.KW + d.stride_w - 1) / d.stride_w;
        const int am = Ahm > Awm ? Ahm : Awm;
        const int th = ((d.H + d.stride_h - 1) / d.stride_h + PH_T - 1) / PH_T;
        const int tw = ((d.W + d.stride_w - 1) / d.stride_w + PH_T - 1) / PH_T;
        const int ct = Cg >= 4 ? 4 : Cg;
        const int chunks = (Cg + ct - 1) / ct;
        const uint64_t gz = (uint64_t)d.N * d.groups * chunks;
        if (am <= 4 && d.stride_h * d.stride_w <= 65535 && gz <= 65535) {
            const dim3 grid((unsigned)(th * tw), (unsigned)(d.stride_h * d.stride_w), (unsigned)gz);
#define CG_PHASE(CT_, AM_)                                                                                            \
    hipLaunchKernelGGL((bwd_data_phase_kernel<CT_, AM_>), grid, dim3(256), 0, stream, d, OH, OW, dy, w, dx, gate,      \
                       accumulate, tw, chunks)
#define CG_PHASE_AM(CT_)                                                                                              \
    do {                                                                                                              \
        if (am == 1) CG_PHASE(CT_, 1);                                                                                \
        else if (am == 2) CG_PHASE(CT_, 2);                                                                           \
        else if (am == 3) CG_PHASE(CT_, 3);                                                                           \
        else CG_PHASE(CT_, 4);                                                                                        \
    } while (0)
            if (ct == 4) CG_PHASE_AM(4);
            else if (ct == 3) CG_PHASE_AM(3);
            else if (ct == 2) CG_PHASE_AM(2);
            else CG_PHASE_AM(1);
#undef CG_PHASE_AM
#undef CG_PHASE
            CG_HIP_TRY(hipGetLastError());
            return CG_OK;
        }
        const size_t total = (size_t)d.N * d.C * d.H * d.W;
        const unsigned blocks = (unsigned)((total + 255) / 256 < 65536 ? (total + 255) / 256 : 65536);
        hipLaunchKernelGGL(bwd_data_strided_kernel, dim3(blocks), dim3(256), 0, stream, d, OH, OW, dy, w, dx, gate,
                           accumulate);
        CG_HIP_TRY(hipGetLastError());
        return CG_OK;
    }
    const int G = d.groups, Cg = d.C / G, Mg = d.M / G, KK = d.KH * d.KW;
    const size_t wt_bytes = round256((size_t)d.M * Cg * KK * sizeof(float));
    if (!ws || ws_bytes < wt_bytes) return CG_ENOSPC;
    if (!aligned16(ws)) return CG_EINVAL;
    float *wt = static_cast<float *>(ws);
    const float *wuse = prepared ? prepared : wt;
    {
        IgemmProblem pp = bwd_data_problem(d, OH, OW, dy, wuse, dx, accumulate);
        pp.gate = gate;
        pp.math = math;
        pp.beside_other_stream = beside_other_stream ? 1 : 0;
        if (bwd_data_patch(d, OH, OW, dy, pp)) {
            if (!prepared) {
                const int rc2 = permute_filters(w, wt, G, Mg, Cg, KK, 1, stream);
                if (rc2) return rc2;
            }
            tap_major_filters(pp, wuse, Cg, Mg * KK, (uint64_t)d.M * Cg * KK);
            return igemm_run(pp, static_cast<char *>(ws) + wt_bytes, ws_bytes - wt_bytes, stream);
        }
    }
    const bool in_place = bwd_data_reads_filters_in_place(d);
    if (!in_place && !prepared) {
        const size_t total = (size_t)d.M * Cg * KK;
        const unsigned blocks = (unsigned)((total + 255) / 256 < 4096 ? (total + 255) / 256 : 4096);
        hipLaunchKernelGGL(transpose_filters_kernel, dim3(blocks), dim3(256), 0, stream, w, wt, G, Mg, Cg, KK);
        CG_HIP_TRY(hipGetLastError());
    }
    IgemmProblem p = bwd_data_problem(d, OH, OW, dy, in_place ? w : wuse, dx, accumulate);
    p.gate = gate;
    p.math = math;
    return igemm_run(p, static_cast<char *>(ws) + wt_bytes, ws_bytes - wt_bytes, stream);
}

FilterPrep conv_fwd_filter_prep(const cg_conv_desc &d)
{
    FilterPrep f{};
    int OH, OW;
    if (conv_check(&d, &OH, &OW)) return f;
    IgemmProblem p = fwd_problem(d, OH, OW, nullptr, nullptr, nullptr, nullptr);
    if (!fwd_patch(d, OH, OW, nullptr, p)) return f;
    f.kind = CG_PREP_PERMUTE_FWD;
    f.Mg = d.M / d.groups; f.Cg = d.C / d.groups; f.KH = d.KH; f.KW = d.KW;
    f.floats = (size_t)d.M * f.Cg * d.KH * d.KW;
    return f;
}

FilterPrep conv_bwd_data_filter_prep(const cg_conv_desc &d)
{
    FilterPrep f{};
    int OH, OW;
    if (conv_check(&d, &OH, &OW)) return f;
    f.Mg = d.M / d.groups; f.Cg = d.C / d.groups; f.KH = d.KH; f.KW = d.KW;
    StridedGeom sg;
    if ((d.stride_h != 1 || d.stride_w != 1) && strided_geom(d, sg)) {
        IgemmProblem p = bwd_data_strided_problem(d, sg, OH, OW, nullptr, nullptr, nullptr, 0);
        f.kind = bwd_data_strided_patch(d, sg, OH, OW, nullptr, p) ? CG_PREP_STRIDED_TAPS : CG_PREP_STRIDED_ROWS;
        f.sh = sg.sh; f.sw = sg.sw; f.Ah = sg.Ah; f.Aw = sg.Aw;
        f.floats = (size_t)d.groups * sg.R * sg.Kp;
        return f;
    }
    if (d.stride_h != 1 || d.stride_w != 1) return f;            // the vector kernels read w itself
    IgemmProblem pp = bwd_data_problem(d, OH, OW, nullptr, nullptr, nullptr, 0);
    if (bwd_data_patch(d, OH, OW, nullptr, pp)) f.kind = CG_PREP_PERMUTE_BWD;
    else if (!bwd_data_reads_filters_in_place(d)) f.kind = CG_PREP_TRANSPOSE;
    else return f;
    f.floats = (size_t)d.M * f.Cg * d.KH * d.KW;
    return f;
}

size_t conv_filter_prep_max_floats(const cg_conv_desc &d)
{
    size_t m = (size_t)d.M * (d.C / d.groups) * d.KH * d.KW;
    StridedGeom sg;
    if ((d.stride_h != 1 || d.stride_w != 1) && strided_geom(d, sg)) {
        const size_t s2 = (size_t)d.groups * sg.R * sg.Kp;
        if (s2 > m) m = s2;
    }
    return m;
}

int filter_prep_launch(int n, const FilterPrep *jobs, const float *const *w, float *const *dst, hipStream_t stream)
{
    int i = 0;
    while (i < n) {
        PrepTable t{};
        unsigned long long blocks = 0;
        while (i < n && t.n < kPrepJobs) {
            const FilterPrep &f = jobs[i];
            if (f.kind == CG_PREP_NONE || f.floats == 0) { ++i; continue; }
            if (!w[i] || !dst[i] || !aligned16(dst[i])) return CG_EINVAL;
            const unsigned long long need = (f.floats + 1023) / 1024;
            if (blocks + need >= (1ull << 31)) break;
            PrepJob &j = t.j[t.n++];
            j.w = w[i]; j.dst = dst[i]; j.kind = f.kind; j.Mg = f.Mg; j.Cg = f.Cg; j.KH = f.KH; j.KW = f.KW;
            j.sh = f.sh; j.sw = f.sw; j.Ah = f.Ah; j.Aw = f.Aw;
            j.first_block = (unsigned)blocks; j.total = f.floats;
            blocks += need;
            ++i;
        }
        if (t.n == 0) {
            if (i < n) return CG_EUNSUPPORTED;
            break;
        }
        hipLaunchKernelGGL(prepare_filters_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, t);
        CG_HIP_TRY(hipGetLastError());
    }
    return CG_OK;
}

// The reduction runs over pixels (n, oh, ow).  Its index space pads every image's OH*OW pixels to
// a multiple of four (padding indices read as zero in B), so that dy, contiguous along the pixels
// of one image, can be fetched in aligned groups of four that never straddle two images.
static IgemmProblem bwd_weight_problem(const cg_conv_desc &d, int OH, int OW, const float *x, const float *dy,
                                       float *dw)
{
    const int G = d.groups, Cg = d.C / G, Mg = d.M / G, Kg = Cg * d.KH * d.KW, P = OH * OW;
    const int Pp = (P + 3) / 4 * 4;
    IgemmProblem p{};
    p.A.ptr = dy;
    p.A.row = linear_map(Mg, P);
    p.A.k = split_map((uint32_t)d.N * Pp, Pp, d.M * P, 1);
    p.A.limA = p.A.limB = 1;
    p.A.gstride = (int64_t)Mg * P;
    p.A.elems = (uint64_t)d.N * d.M * P;
    p.A.lanes_k = 1;
    p.B.ptr = x;
    p.B.row = tap_map(d, Cg);
    p.B.k = window_origin_map(d, OH, OW);
    p.B.k.count = (uint32_t)d.N * Pp;
    p.B.k.d1 = make_fastdiv((uint32_t)Pp);
    p.B.k.r1_lim = (uint32_t)P;
    p.B.limA = d.H; p.B.limB = d.W;
    p.B.gstride = (int64_t)Cg * d.H * d.W;
    p.B.elems = (uint64_t)d.N * d.C * d.H * d.W;
    p.B.lanes_k = 1;
    p.B.check = (d.pad_h || d.pad_w) ? 1 : 0;
    p.c_ptr = dw;
    p.c_row_stride = Kg;
    p.c_col = linear_map(Kg, 1);
    p.c_gstride = (int64_t)Mg * Kg;
    p.M = Mg; p.N = Kg; p.K = (uint32_t)d.N * Pp;
    p.flops = 2.0 * Mg * (double)Kg * ((double)d.N * P) * G;
    p.groups = G; p.splits = 1; p.k_per_split = p.K;
    // the band kernel, where it applies: x as padded rows in LDS, dy in tiles of 16 pixels
    if (d.stride_h == d.stride_w) {
        WgradGeom wgm{};
        wgm.x = x; wgm.x_elems = (uint64_t)d.N * d.C * d.H * d.W;
        wgm.C = d.C; wgm.Cg = Cg; wgm.H = d.H; wgm.W = d.W; wgm.OH = OH; wgm.OW = OW; wgm.s = d.stride_h;
        wgm.pad_h = d.pad_h; wgm.pad_w = d.pad_w; wgm.KH = d.KH; wgm.KW = d.KW; wgm.M = d.M;
        uint32_t splits = 1;
        if (wgrad_plan(wgm, (uint32_t)Mg, (uint32_t)Kg, (uint32_t)G, (uint32_t)d.N, &splits)) {
            p.use_wgrad = 1;
            p.wgrad = wgm;
            p.splits = splits;
        }
    }
    return p;
}

int conv_bwd_weight_impl(const cg_conv_desc &d, const float *x, const float *dy, float *dw, float *db,
                         void *ws, size_t ws_bytes, hipStream_t stream, int math, hipStream_t bias_stream,
                         void *bias_ws, size_t bias_ws_bytes)
{
    if (!math_ok(math)) return CG_EINVAL;
    ProfTag tag("conv_bwd_weight", -1);
    int OH, OW;
    const int rc = conv_check(&d, &OH, &OW);
    if (rc) return rc;
    IgemmProblem p = bwd_weight_problem(d, OH, OW, x, dy, dw);
    const size_t split_bytes = round256(igemm_ws_bytes(p));       // sized for the kernel the fp32 mode picks
    p.math = math;
    if (math != CG_MATH_FP32 && p.use_wgrad) { p.use_wgrad = 0; p.splits = 1; }    // the band kernel is fp32 only
    const size_t bias_bytes = db ? bias_grad_ws_bytes(d.N, d.M) : 0;
    if (split_bytes + bias_bytes > 0) {
        if (!ws || ws_bytes < split_bytes + bias_bytes) return CG_ENOSPC;
        if (!aligned16(ws)) return CG_EINVAL;
    }
    // The bias sums go first: they need only dy and stream through HBM while another stream's matrix
    // kernel still runs; behind the weight gradient of a net's first layer they would sit, alone on
    // the GPU, between that kernel and the update the next iteration waits for.
    // (bias_stream: a stream of the caller's that has nothing else to do meanwhile -- a net's first
    // layer has no backward-data -- so that the sums run beside the matrix kernel, not in front of it.
    // Their partial sums then live in bias_ws, scratch memory that is free in THAT stream's order: `ws`
    // is only ordered by `stream`, on which earlier launches may still be reading it.)
    // A small layer's sums (one block per channel, one launch) ride in the launch that adds the K slices.
    const bool ride = db && !bias_stream && bias_grad_single_launch(d.N, OH * OW);
    if (db && !ride) {
        int rb;
        if (bias_stream) {
            if (!bias_ws || bias_ws_bytes < bias_bytes) return CG_ENOSPC;
            rb = bias_grad_launch(dy, d.N, d.M, OH * OW, db, bias_ws, bias_bytes, bias_stream);
        } else
            rb = bias_grad_launch(dy, d.N, d.M, OH * OW, db, static_cast<char *>(ws) + split_bytes, bias_bytes, stream);
        if (rb) return rb;
    }
    const BiasRider rider{dy, d.N, d.M, OH * OW, db};
    bool taken = false;
    const int rr = igemm_run(p, ws, split_bytes, stream, ride ? &rider : nullptr, &taken);
    if (rr || !ride || taken) return rr;
    return bias_grad_launch(dy, d.N, d.M, OH * OW, db, static_cast<char *>(ws) + split_bytes, bias_bytes, stream);
}

size_t conv_ws_bytes(const cg_conv_desc &d, int pass)
{
    int OH, OW;
    if (conv_check(&d, &OH, &OW)) return 0;
    if (pass == CG_PASS_FWD) {
        IgemmProblem p = fwd_problem(d, OH, OW, nullptr, nullptr, nullptr, nullptr);
        if (fwd_patch(d, OH, OW, nullptr, p)) return round256((size_t)d.M * (d.C / d.groups) * d.KH * d.KW * sizeof(float));
        return igemm_ws_bytes(p);
    }
    if (pass == CG_PASS_BWD_DATA) {
        StridedGeom sg;
        if ((d.stride_h != 1 || d.stride_w != 1) && strided_geom(d, sg)) {
            IgemmProblem p = bwd_data_strided_problem(d, sg, OH, OW, nullptr, nullptr, nullptr, 0);
            bwd_data_strided_patch(d, sg, OH, OW, nullptr, p);
            return round256((size_t)d.groups * sg.R * sg.Kp * sizeof(float)) + igemm_ws_bytes(p);
        }
        if (d.stride_h != 1 || d.stride_w != 1) return 0;
        return round256((size_t)d.M * (d.C / d.groups) * d.KH * d.KW * sizeof(float)) +
               igemm_ws_bytes(bwd_data_problem(d, OH, OW, nullptr, nullptr, nullptr, 0));
    }
    if (pass == CG_PASS_BWD_WEIGHT)
        return round256(igemm_ws_bytes(bwd_weight_problem(d, OH, OW, nullptr, nullptr, nullptr))) +
               bias_grad_ws_bytes(d.N, d.M);
    return 0;
}

// ---- fully connected: y[b][o] = bias[o] + sum_i x[b][i] W[o][i] ------------------------------

static IgemmProblem fc_fwd_problem(int B, int IN, int OUT, const float *x, const float *W, const float *bias,
                                   float *y)
{
    IgemmProblem p{};
    p.A.ptr = x; p.A.row = linear_map(B, IN); p.A.k = linear_map(IN, 1); p.A.limA = p.A.limB = 1;
    p.A.elems = (uint64_t)B * IN; p.A.lanes_k = 1;
    p.B.ptr = W; p.B.row = linear_map(OUT, IN); p.B.k = linear_map(IN, 1); p.B.limA = p.B.limB = 1;
    p.B.elems = (uint64_t)OUT * IN; p.B.lanes_k = 1;
    p.c_ptr = y; p.c_row_stride = OUT; p.c_col = linear_map(OUT, 1);
    p.bias = bias; p.bias_mode = bias ? 2 : 0;
    p.M = B; p.N = OUT; p.K = IN;
    p.groups = 1; p.splits = 1; p.k_per_split = p.K;
    return p;
}

// dx[b][i] = sum_o dy[b][o] W[o][i]
static IgemmProblem fc_bwd_data_problem(int B, int IN, int OUT, const float *dy, const float *W, float *dx,
                                        int accumulate)
{
    IgemmProblem p{};
    p.A.ptr = dy; p.A.row = linear_map(B, OUT); p.A.k = linear_map(OUT, 1); p.A.limA = p.A.limB = 1;
    p.A.elems = (uint64_t)B * OUT; p.A.lanes_k = 1;
    p.B.ptr = W; p.B.row = linear_map(IN, 1); p.B.k = linear_map(OUT, IN); p.B.limA = p.B.limB = 1;
    p.B.elems = (uint64_t)OUT * IN; p.B.lanes_k = 0;
    p.c_ptr = dx; p.c_row_stride = IN; p.c_col = linear_map(IN, 1);
    p.M = B; p.N = IN; p.K = OUT;
    p.groups = 1; p.splits = 1; p.k_per_split = p.K;
    p.accumulate = accumulate;
    return p;
}

// dW[o][i] = sum_b dy[b][o] x[b][i];  db[o] = sum_b dy[b][o]
static IgemmProblem fc_bwd_weight_problem(int B, int IN, int OUT, const float *x, const float *dy, float *dW)
{
    IgemmProblem p{};
    p.A.ptr = dy; p.A.row = linear_map(OUT, 1); p.A.k = linear_map(B, OUT); p.A.limA = p.A.limB = 1;
    p.A.elems = (uint64_t)B * OUT; p.A.lanes_k = 0;
    p.B.ptr = x; p.B.row = linear_map(IN, 1); p.B.k = linear_map(B, IN); p.B.limA = p.B.limB = 1;
    p.B.elems = (uint64_t)B * IN; p.B.lanes_k = 0;
    p.c_ptr = dW; p.c_row_stride = IN; p.c_col = linear_map(IN, 1);
    p.M = OUT; p.N = IN; p.K = B;
    p.groups = 1; p.splits = 1; p.k_per_split = p.K;
    return p;
}

int fc_fwd_impl(int B, int IN, int OUT, const float *x, const float *W, const float *bias, float *y, void *ws,
                size_t ws_bytes, int relu, hipStream_t stream, int math)
{
    ProfTag tag("fc_fwd", -1);
    if (B <= 0 || IN <= 0 || OUT <= 0 || !math_ok(math)) return CG_EINVAL;
    IgemmProblem p = fc_fwd_problem(B, IN, OUT, x, W, bias, y);
    p.relu = relu;
    p.math = math;
    return igemm_run(p, ws, ws_bytes, stream);
}

int fc_bwd_data_impl(int B, int IN, int OUT, const float *dy, const float *W, float *dx, const float *gate,
                     int accumulate, void *ws, size_t ws_bytes, hipStream_t stream, int math)
{
    ProfTag tag("fc_bwd_data", -1);
    if (B <= 0 || IN <= 0 || OUT <= 0 || !math_ok(math)) return CG_EINVAL;
    IgemmProblem p = fc_bwd_data_problem(B, IN, OUT, dy, W, dx, accumulate);
    p.gate = gate;
    p.math = math;
    return igemm_run(p, ws, ws_bytes, stream);
}

int fc_bwd_weight_impl(int B, int IN, int OUT, const float *x, const float *dy, float *dW, float *db, void *ws,
                       size_t ws_bytes, hipStream_t stream, int math)
{
    ProfTag tag("fc_bwd_weight", -1);
    if (B <= 0 || IN <= 0 || OUT <= 0 || !math_ok(math)) return CG_EINVAL;
    IgemmProblem pw = fc_bwd_weight_problem(B, IN, OUT, x, dy, dW);
    pw.math = math;
    const int r = igemm_run(pw, ws, ws_bytes, stream);
    if (r) return r;
    if (db) return fc_bias_grad_launch(dy, B, OUT, db, stream);
    return CG_OK;
}

size_t fc_ws_bytes(int B, int IN, int OUT, int pass)
{
    if (B <= 0 || IN <= 0 || OUT <= 0) return 0;
    if (pass == CG_PASS_FWD) return igemm_ws_bytes(fc_fwd_problem(B, IN, OUT, nullptr, nullptr, nullptr, nullptr));
    if (pass == CG_PASS_BWD_DATA) return igemm_ws_bytes(fc_bwd_data_problem(B, IN, OUT, nullptr, nullptr, nullptr, 0));
    return igemm_ws_bytes(fc_bwd_weight_problem(B, IN, OUT, nullptr, nullptr, nullptr));
}

}  // namespace cg

// ---- C ABI --------------------------------------------------------------------------------

using namespace cg;

extern "C" int cg_debug_conv_operand(const cg_conv_desc *d, int pass, int operand, unsigned row, unsigned k,
                                     unsigned group, long long *elem_offset, int *valid)
{
    int OH, OW;
    const int rc = conv_check(d, &OH, &OW);
    if (rc) return rc;
    if (!elem_offset || !valid || (operand != 0 && operand != 1) || group >= (unsigned)d->groups) return CG_EINVAL;
    IgemmProblem p;
    if (pass == CG_PASS_FWD) p = fwd_problem(*d, OH, OW, nullptr, nullptr, nullptr, nullptr);
    else if (pass == CG_PASS_BWD_DATA) {
        if (d->stride_h != 1 || d->stride_w != 1) return CG_EUNSUPPORTED;
        p = bwd_data_problem(*d, OH, OW, nullptr, nullptr, nullptr, 0);
    } else if (pass == CG_PASS_BWD_WEIGHT)
        p = bwd_weight_problem(*d, OH, OW, nullptr, nullptr, nullptr);
    else return CG_EINVAL;
    const Operand &op = operand == 0 ? p.A : p.B;
    if (row >= op.row.count || k >= p.K) return CG_EINVAL;
    int64_t off;
    igemm_host_element(op, row, k, &off, valid);
    *elem_offset = off + (int64_t)group * op.gstride;
    return CG_OK;
}

extern "C" int cg_debug_band_kernel(int on)
{
    wgrad_set_enabled(on);
    return CG_OK;
}

extern "C" int cg_debug_patch_min_tiles(int tiles)
{
    if (tiles < 1) return CG_EINVAL;
    patch_set_min_tiles((uint32_t)tiles);
    return CG_OK;
}

extern "C" int cg_debug_resident_blocks(int blocks)
{
    if (blocks < 1) return CG_EINVAL;
    patch_set_resident_blocks((uint32_t)blocks);
    return CG_OK;
}

extern "C" int cg_conv_out_shape(const cg_conv_desc *d, int *OH, int *OW)
{
    return conv_check(d, OH, OW);
}

extern "C" size_t cg_conv_workspace_bytes(const cg_conv_desc *d, int pass)
{
    return d ? conv_ws_bytes(*d, pass) : 0;
}

extern "C" int cg_conv_fwd(const cg_conv_desc *d, const float *x, const float *w, const float *bias, float *y,
                           void *ws, size_t ws_bytes, void *stream)
{
    if (!d || !x || !w || !y) return CG_EINVAL;
    if (!aligned16(x) || !aligned16(w) || !aligned16(y)) return CG_EINVAL;
    return conv_fwd_impl(*d, x, w, bias, y, ws, ws_bytes, 0, static_cast<hipStream_t>(stream));
}

extern "C" int cg_conv_bwd_data(const cg_conv_desc *d, const float *dy, const float *w, float *dx, void *ws,
                                size_t ws_bytes, void *stream)
{
    if (!d || !dy || !w || !dx) return CG_EINVAL;
    if (!aligned16(dy) || !aligned16(w) || !aligned16(dx)) return CG_EINVAL;
    return conv_bwd_data_impl(*d, dy, w, dx, nullptr, ws, ws_bytes, 0, static_cast<hipStream_t>(stream));
}

extern "C" int cg_conv_bwd_weight(const cg_conv_desc *d, const float *x, const float *dy, float *dw, float *dbias,
                                  void *ws, size_t ws_bytes, void *stream)
{
    if (!d || !x || !dy || !dw) return CG_EINVAL;
    if (!aligned16(x) || !aligned16(dy) || !aligned16(dw)) return CG_EINVAL;
    return conv_bwd_weight_impl(*d, x, dy, dw, dbias, ws, ws_bytes, static_cast<hipStream_t>(stream));
}

// ---- the three passes with the arithmetic of the matrix instructions chosen by the caller -----------

extern "C" int cg_conv_fwd_math(const cg_conv_desc *d, const float *x, const float *w, const float *bias, float *y,
                                void *ws, size_t ws_bytes, int math, void *stream)
{
    if (!d || !x || !w || !y) return CG_EINVAL;
    if (!aligned16(x) || !aligned16(w) || !aligned16(y)) return CG_EINVAL;
    return conv_fwd_impl(*d, x, w, bias, y, ws, ws_bytes, 0, static_cast<hipStream_t>(stream), 0, math);
}

extern "C" int cg_conv_bwd_data_math(const cg_conv_desc *d, const float *dy, const float *w, float *dx, void *ws,
                                     size_t ws_bytes, int math, void *stream)
{
    if (!d || !dy || !w || !dx) return CG_EINVAL;
    if (!aligned16(dy) || !aligned16(w) || !aligned16(dx)) return CG_EINVAL;
    return conv_bwd_data_impl(*d, dy, w, dx, nullptr, ws, ws_bytes, 0, static_cast<hipStream_t>(stream), math);
}

extern "C" int cg_conv_bwd_weight_math(const cg_conv_desc *d, const float *x, const float *dy, float *dw, float *dbias,
                                       void *ws, size_t ws_bytes, int math, void *stream)
{
    if (!d || !x || !dy || !dw) return CG_EINVAL;
    if (!aligned16(x) || !aligned16(dy) || !aligned16(dw)) return CG_EINVAL;
    return conv_bwd_weight_impl(*d, x, dy, dw, dbias, ws, ws_bytes, static_cast<hipStream_t>(stream), math);
}

// ---- backward-weight without a caller's workspace ------------------------------------------------
//
// The partial sums of the K slices and of the bias gradient live in a device array that is part of
// the library's code object: every GPU the library runs on holds its own copy, at its own address,
// from the moment the module is loaded until the process ends.  In host code the array's name is
// only a handle for hipGetSymbolAddress; the address that call returns for the current device is
// what the kernels are given.  Nothing has to start at zero: the matrix kernel writes every partial
// sum the finishing kernels read.  All calls on one GPU share the array, so two calls that overlap
// on that GPU (different streams, or threads) race.
static __device__ __align__(256) unsigned char scratch[CG_NOALLOC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[kMaxDevices];       // per device, filled on the first call with that device current

int scratch_for_current_device(void **out)
{
    int dev = -1;
    CG_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return CG_EUNSUPPORTED;
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        CG_HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr || !aligned16(ptr)) return CG_EHIP;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return CG_OK;
}
}  // namespace

extern "C" int cg_conv_bwd_weight_noalloc(const cg_conv_desc *d, const float *x, const float *dy, float *dw,
                                          float *dbias, void *stream)
{
    if (!d || !x || !dy || !dw) return CG_EINVAL;
    if (!aligned16(x) || !aligned16(dy) || !aligned16(dw)) return CG_EINVAL;
    int OH, OW;
    const int rc = conv_check(d, &OH, &OW);
    if (rc) return rc;
    if (conv_ws_bytes(*d, CG_PASS_BWD_WEIGHT) > (size_t)CG_NOALLOC_SCRATCH_BYTES) return CG_ENOSPC;
    void *ptr = nullptr;
    const int rs = scratch_for_current_device(&ptr);
    if (rs) return rs;
    return conv_bwd_weight_impl(*d, x, dy, dw, dbias, ptr, (size_t)CG_NOALLOC_SCRATCH_BYTES,
                                static_cast<hipStream_t>(stream));
}
