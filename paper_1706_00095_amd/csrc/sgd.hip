// Gradient aggregation over K+1 ranks fused with the layer's model update (Eq. 1 plus the
// solver's history terms).  Pure streaming: every element is read once from each of the K+1
// gradient buffers and from w and v, and w and v are written once -- 4K+20 bytes per
// parameter, so the kernel is bound by HBM bandwidth and nothing else.
//
// This translation unit is compiled with -ffp-contract=off: the operation order documented in
// cg.h is also the rounding order, which makes the result bit-reproducible.
#include <cstdio>
#include "cg_internal.h"

namespace cg {

typedef float f4 __attribute__((ext_vector_type(4)));

struct PeerTable { const float *p[CG_MAX_PEERS]; };

__device__ __forceinline__ float upd(float w, float v, float s, const cg_sgd c, float &vn_out)
{
    if (c.grad_scale != 1.0f) s = s * c.grad_scale;
    const float t = c.wd * w;
    const float d = s + t;
    const float a = c.mu * v;
    const float b = c.lr * d;
    const float vn = a + b;
    vn_out = vn;
    return w - vn;
}

// K known at compile time: the K+1 gradient loads of a f4 group are issued back to back.
// KRT > 0 means "K is a run-time value" (K > 16).
template <int KC>
__global__ __launch_bounds__(256) void reduce_sgd_kernel(float *__restrict__ w, float *__restrict__ v,
                                                         const float *__restrict__ g, const PeerTable peers,
                                                         int K_rt, size_t n4, size_t n, const cg_sgd c)
{
    const int K = KC >= 0 ? KC : K_rt;
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += stride) {
        f4 s = __builtin_nontemporal_load(reinterpret_cast<const f4 *>(g) + i);
        if constexpr (KC >= 0) {
            f4 q[KC > 0 ? KC : 1];
#pragma unroll
            for (int k = 0; k < KC; ++k)
                q[k] = __builtin_nontemporal_load(reinterpret_cast<const f4 *>(peers.p[k]) + i);
#pragma unroll
            for (int k = 0; k < KC; ++k) { s.x = s.x + q[k].x; s.y = s.y + q[k].y; s.z = s.z + q[k].z; s.w = s.w + q[k].w; }
        } else {
            for (int k = 0; k < K; ++k) {
                const f4 q = __builtin_nontemporal_load(reinterpret_cast<const f4 *>(peers.p[k]) + i);
                s.x = s.x + q.x; s.y = s.y + q.y; s.z = s.z + q.z; s.w = s.w + q.w;
            }
        }
        const f4 wi = reinterpret_cast<const f4 *>(w)[i];
        const f4 vi = reinterpret_cast<const f4 *>(v)[i];
        f4 wo, vo;
        float v0, v1, v2, v3;
        wo.x = upd(wi.x, vi.x, s.x, c, v0);
        wo.y = upd(wi.y, vi.y, s.y, c, v1);
        wo.z = upd(wi.z, vi.z, s.z, c, v2);
        wo.w = upd(wi.w, vi.w, s.w, c, v3);
        vo.x = v0; vo.y = v1; vo.z = v2; vo.w = v3;
        reinterpret_cast<f4 *>(w)[i] = wo;
        reinterpret_cast<f4 *>(v)[i] = vo;
    }
    // ragged tail (n % 4 elements), handled by the first threads of block 0
    const size_t tail = n4 * 4 + (size_t)blockIdx.x * 256 + threadIdx.x;
    if (blockIdx.x == 0 && tail < n) {
        float s = g[tail];
        for (int k = 0; k < K; ++k) s = s + peers.p[k][tail];
        float vn;
        const float wn = upd(w[tail], v[tail], s, c, vn);
        w[tail] = wn;
        v[tail] = vn;
    }
}

namespace {

template <int KC>
void launch(float *w, float *v, const float *g, const PeerTable &pt, int K, size_t n, const cg_sgd &c,
            unsigned blocks, hipStream_t stream)
{
    hipLaunchKernelGGL((reduce_sgd_kernel<KC>), dim3(blocks), dim3(256), 0, stream, w, v, g, pt, K, n / 4, n, c);
}

}  // namespace

int grad_reduce_sgd_impl(float *w, float *v, const float *g_local, const float *const *g_peers, int K, size_t n,
                         const cg_sgd &sgd, hipStream_t stream)
{
    if (K < 0 || K > CG_MAX_PEERS) return CG_EINVAL;
    if (n == 0) return CG_OK;
    if (!w || !v || !g_local || (K > 0 && !g_peers)) return CG_EINVAL;
    if (!aligned16(w) || !aligned16(v) || !aligned16(g_local)) return CG_EINVAL;
    if (w == v) return CG_EINVAL;
    PeerTable pt{};
    for (int k = 0; k < K; ++k) {
        if (!g_peers[k] || !aligned16(g_peers[k])) return CG_EINVAL;
        pt.p[k] = g_peers[k];
    }
    // 256 compute units x 8 resident blocks saturate HBM; small buckets get one f4 per thread
    const size_t n4 = n / 4;
    size_t blocks = (n4 + 255) / 256;
    if (blocks > 2048) blocks = 2048;
    if (blocks == 0) blocks = 1;
    const unsigned b = (unsigned)blocks;
    int rec = -1;
    if (prof_on()) {
        ProfTag tag("reduce_sgd", -1);
        char name[64];
        snprintf(name, sizeof name, "reduce_sgd_kernel<%d>", K <= 16 ? K : -1);
        rec = prof_begin(name, 0.0, (4.0 * K + 20.0) * (double)n, stream);
    }
    switch (K) {
#define CG_CASE(k) case k: launch<k>(w, v, g_local, pt, K, n, sgd, b, stream); break;
        CG_CASE(0) CG_CASE(1) CG_CASE(2) CG_CASE(3) CG_CASE(4) CG_CASE(5) CG_CASE(6) CG_CASE(7) CG_CASE(8)
        CG_CASE(9) CG_CASE(10) CG_CASE(11) CG_CASE(12) CG_CASE(13) CG_CASE(14) CG_CASE(15) CG_CASE(16)
#undef CG_CASE
    default: launch<-1>(w, v, g_local, pt, K, n, sgd, b, stream); break;
    }
    prof_end(rec, stream);
    CG_HIP_TRY(hipGetLastError());
    return CG_OK;
}

}  // namespace cg

extern "C" int cg_grad_reduce_sgd(float *w, float *v, const float *g_local, const float *const *g_peers, int K,
                                  size_t n, const cg_sgd *sgd, void *stream)
{
    if (!sgd) return CG_EINVAL;
    return cg::grad_reduce_sgd_impl(w, v, g_local, g_peers, K, n, *sgd, static_cast<hipStream_t>(stream));
}
