// Gradient aggregation over K+1 ranks fused with the layer's model update (Eq. 1 plus the
// solver's history terms).  Pure streaming: every element is read once from each of the K+1
// gradient buffers and from w and v, and w and v are written once -- 4K+20 bytes per
// parameter, so the kernel is bound by HBM bandwidth and nothing else.
//
// Two associations of the sum exist: left to right (local first, then peers 0..K-1), and that of
// the binomial reduction tree of section 3.2 (rank 0 = local, rank k+1 = peer k; rank r adds the
// sums forwarded by ranks r+1, r+2, r+4, ... below its own lowest set bit, nearest first).
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

__device__ __forceinline__ void add4(f4 &a, const f4 b)
{
    a.x = a.x + b.x; a.y = a.y + b.y; a.z = a.z + b.z; a.w = a.w + b.w;
}
__device__ __forceinline__ void add4(float &a, const float b) { a = a + b; }

// Sum of rank 0 (s) and ranks 1..KC (q[0..KC-1]).  TREE: the message rounds of the binomial tree,
// distance 1, 2, 4, ...: in the round of distance d rank r (a multiple of 2d) adds what rank r + d
// holds.  KC is a compile-time constant, so the array lives in registers.
template <int KC, bool TREE, typename T>
__device__ __forceinline__ T rank_sum(const T s, const T *q)
{
    if constexpr (!TREE || KC < 3) {
        T t = s;
#pragma unroll
        for (int k = 0; k < KC; ++k) add4(t, q[k]);
        return t;
    } else {
        T a[KC + 1];
        a[0] = s;
#pragma unroll
        for (int k = 0; k < KC; ++k) a[k + 1] = q[k];
#pragma unroll
        for (int d = 1; d <= KC; d *= 2) {
#pragma unroll
            for (int r = 0; r + d <= KC; r += 2 * d) add4(a[r], a[r + d]);
        }
        return a[0];
    }
}

// One launch serves up to MAXB buckets: block b belongs to the bucket whose [first, first + blocks)
// range contains it and updates UNR x TB consecutive float4 groups there, every load of a group
// issued before the first use.  No loop: one short-lived block per few KB of each stream keeps far
// more loads in flight than a persistent grid does, which is what the memory system rewards here.
// Every access is non-temporal, the reads of w and v and the two stores included: each byte is
// touched once per launch, and with the model and its history read through the caches and written
// back through them the same kernel ran 5 % slower (K = 4: 72 -> 76 % of 8 TB/s on one array of
// the eight buckets' size; either hint alone gained nothing or lost).
constexpr int MAXB = 8;          // buckets per launch
constexpr int KMAX_TAB = 16;     // peers per bucket in the table (more: the run-time-K kernel)
// Launch shape: blocks of ONE wave, one float4 group per thread -- 1 KB of every stream per block --
// for every K.  Measured on the eight buckets in one launch, same box, percent of 8 TB/s
// (groups per thread x threads per block): K = 4: 1x64 76.2, 1x128 72.5, 1x256 72.6, 2x64 71.1,
// 2x128 72.7, 2x256 72.6, 4x64 72.2, 4x128 72.5; K = 8: 1x64 74.2, 1x128 69.9, 1x256 71.1, 2x64 69.7,
// 4x64 70.5, 4x128 71.5, 4x256 72.3; K = 16: 1x64 73.5, 1x128 72.0, 1x192 68.7, 1x256 67.5, 1x512 69.3.
// A wave that is its own block leaves as soon as its own loads have come back and been stored;
// nothing in the kernel needs a second wave.
constexpr int unr_for(int) { return 1; }
constexpr int tb_for(int) { return 64; }

struct Bucket {
    float *w, *v;
    const float *g;
    const float *peer[KMAX_TAB];
    unsigned long long n;        // elements
    unsigned first_block;        // of this bucket in the launch
};
struct BucketTable {
    int nb;
    Bucket b[MAXB];
};

template <int KC, bool TREE>
__global__ __launch_bounds__(tb_for(KC)) void reduce_sgd_kernel(const BucketTable tab, const cg_sgd c)
{
    constexpr int UNR = unr_for(KC), TB = tb_for(KC);
    int bi = 0;
#pragma unroll
    for (int j = 1; j < MAXB; ++j)
        if (j < tab.nb && blockIdx.x >= tab.b[j].first_block) bi = j;
    const Bucket &bk = tab.b[bi];
    const size_t n = bk.n, n4 = n / 4;
    const size_t i0 = (size_t)(blockIdx.x - bk.first_block) * (TB * UNR) + threadIdx.x;
    const f4 *g4 = reinterpret_cast<const f4 *>(bk.g);
    f4 *w4 = reinterpret_cast<f4 *>(bk.w), *v4 = reinterpret_cast<f4 *>(bk.v);
    f4 s[UNR], q[UNR][KC > 0 ? KC : 1], wi[UNR], vi[UNR];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
        const size_t i = i0 + (size_t)u * TB;
        if (i < n4) {
            s[u] = __builtin_nontemporal_load(g4 + i);
#pragma unroll
            for (int k = 0; k < KC; ++k) q[u][k] = __builtin_nontemporal_load(reinterpret_cast<const f4 *>(bk.peer[k]) + i);
            wi[u] = __builtin_nontemporal_load(w4 + i);
            vi[u] = __builtin_nontemporal_load(v4 + i);
        }
    }
    // every load above is issued before the first addition below: left to itself the instruction
    // scheduler saves registers by adding each peer's values as they arrive, which halves the loads a
    // thread has in flight (K = 16, one group per thread: 1.71 ms instead of 0.89 for the eight buckets)
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
        const size_t i = i0 + (size_t)u * TB;
        if (i < n4) {
            const f4 t = rank_sum<KC, TREE, f4>(s[u], q[u]);
            f4 wo, vo;
            float v0, v1, v2, v3;
            wo.x = upd(wi[u].x, vi[u].x, t.x, c, v0);
            wo.y = upd(wi[u].y, vi[u].y, t.y, c, v1);
            wo.z = upd(wi[u].z, vi[u].z, t.z, c, v2);
            wo.w = upd(wi[u].w, vi[u].w, t.w, c, v3);
            vo.x = v0; vo.y = v1; vo.z = v2; vo.w = v3;
            __builtin_nontemporal_store(wo, w4 + i);
            __builtin_nontemporal_store(vo, v4 + i);
        }
    }
    // ragged tail (n % 4 elements), handled by the first threads of the bucket's first block
    const size_t tail = n4 * 4 + threadIdx.x;
    if (blockIdx.x == bk.first_block && tail < n) {
        float qt[KC > 0 ? KC : 1];
#pragma unroll
        for (int k = 0; k < KC; ++k) qt[k] = bk.peer[k][tail];
        const float t = rank_sum<KC, TREE, float>(bk.g[tail], qt);
        float vn;
        const float wn = upd(bk.w[tail], bk.v[tail], t, c, vn);
        bk.w[tail] = wn;
        bk.v[tail] = vn;
    }
}

// Run-time K, tree association: ranks are visited from K down to 0.  When rank r is reached the
// sums of its senders r + 2^j (2^j below r's lowest set bit) are complete, and each is the latest
// sum filed under its own lowest set bit 2^j; r adds them nearest first and files its own sum
// under its lowest set bit.  Seven slots cover ranks up to 64.
template <typename T, typename LOAD>
__device__ __forceinline__ T tree_sum_anyk(int K, LOAD load)
{
    T slot[7];
    T s = T();
    for (int r = K; r >= 0; --r) {
        s = load(r);
        const int b = r ? __builtin_ctz((unsigned)r) : 7;
#pragma unroll
        for (int j = 0; j < 7; ++j)
            if (j < b && r + (1 << j) <= K) add4(s, slot[j]);
#pragma unroll
        for (int j = 0; j < 7; ++j)
            if (j == b) slot[j] = s;
    }
    return s;
}

// any K up to CG_MAX_PEERS: one bucket, grid-stride
template <bool TREE>
__global__ __launch_bounds__(256) void reduce_sgd_anyk_kernel(float *__restrict__ w, float *__restrict__ v,
                                                              const float *__restrict__ g, const PeerTable peers,
                                                              int K, size_t n4, size_t n, const cg_sgd c)
{
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += stride) {
        f4 s;
        if constexpr (TREE) {
            s = tree_sum_anyk<f4>(K, [&](int r) {
                return __builtin_nontemporal_load(reinterpret_cast<const f4 *>(r ? peers.p[r - 1] : g) + i);
            });
        } else {
            s = __builtin_nontemporal_load(reinterpret_cast<const f4 *>(g) + i);
            for (int k = 0; k < K; ++k)
                add4(s, __builtin_nontemporal_load(reinterpret_cast<const f4 *>(peers.p[k]) + i));
        }
        const f4 wi = __builtin_nontemporal_load(reinterpret_cast<const f4 *>(w) + i);
        const f4 vi = __builtin_nontemporal_load(reinterpret_cast<const f4 *>(v) + i);
        f4 wo, vo;
        float v0, v1, v2, v3;
        wo.x = upd(wi.x, vi.x, s.x, c, v0);
        wo.y = upd(wi.y, vi.y, s.y, c, v1);
        wo.z = upd(wi.z, vi.z, s.z, c, v2);
        wo.w = upd(wi.w, vi.w, s.w, c, v3);
        vo.x = v0; vo.y = v1; vo.z = v2; vo.w = v3;
        __builtin_nontemporal_store(wo, reinterpret_cast<f4 *>(w) + i);
        __builtin_nontemporal_store(vo, reinterpret_cast<f4 *>(v) + i);
    }
    const size_t tail = n4 * 4 + (size_t)blockIdx.x * 256 + threadIdx.x;
    if (blockIdx.x == 0 && tail < n) {
        float s;
        if constexpr (TREE) {
            s = tree_sum_anyk<float>(K, [&](int r) { return r ? peers.p[r - 1][tail] : g[tail]; });
        } else {
            s = g[tail];
            for (int k = 0; k < K; ++k) s = s + peers.p[k][tail];
        }
        float vn;
        const float wn = upd(w[tail], v[tail], s, c, vn);
        w[tail] = wn;
        v[tail] = vn;
    }
}

namespace {

// [a, a+n) and [b, b+n) share an element
bool overlap(const float *a, const float *b, size_t n)
{
    const uintptr_t x = reinterpret_cast<uintptr_t>(a), y = reinterpret_cast<uintptr_t>(b), len = n * sizeof(float);
    return x < y + len && y < x + len;
}

// w and v are written while every gradient buffer is still being read by other blocks: none of the
// gradients may share memory with w or v, nor w with v (gradient buffers may alias each other)
int check_bucket(const float *w, const float *v, const float *g, const float *const *peers, int K, size_t n)
{
    if (!w || !v || !g || (K > 0 && !peers)) return CG_EINVAL;
    if (!aligned16(w) || !aligned16(v) || !aligned16(g)) return CG_EINVAL;
    if (overlap(w, v, n) || overlap(g, w, n) || overlap(g, v, n)) return CG_EINVAL;
    for (int k = 0; k < K; ++k)
        if (!peers[k] || !aligned16(peers[k]) || overlap(peers[k], w, n) || overlap(peers[k], v, n)) return CG_EINVAL;
    return CG_OK;
}

void launch_table(const BucketTable &tab, unsigned blocks, int K, bool tree, const cg_sgd &c, hipStream_t stream)
{
    // up to three ranks the two associations are the same sum
    switch (tree && K >= 3 ? 100 + K : K) {
#define CG_CASE(k)                                                                                         \
    case k: hipLaunchKernelGGL((reduce_sgd_kernel<k, false>), dim3(blocks), dim3(tb_for(k)), 0, stream, tab, c); break; \
    case 100 + k: hipLaunchKernelGGL((reduce_sgd_kernel<k, true>), dim3(blocks), dim3(tb_for(k)), 0, stream, tab, c); break;
        CG_CASE(0) CG_CASE(1) CG_CASE(2) CG_CASE(3) CG_CASE(4) CG_CASE(5) CG_CASE(6) CG_CASE(7) CG_CASE(8)
        CG_CASE(9) CG_CASE(10) CG_CASE(11) CG_CASE(12) CG_CASE(13) CG_CASE(14) CG_CASE(15) CG_CASE(16)
#undef CG_CASE
    default: break;
    }
}

}  // namespace

// nb buckets with the same K and constants; launches ceil(nb / MAXB) kernels
int grad_reduce_sgd_multi_impl(int nb, float *const *w, float *const *v, const float *const *g_local,
                               const float *const *const *g_peers, int K, const size_t *n, const cg_sgd &sgd,
                               hipStream_t stream, bool tree)
{
    if (K < 0 || K > CG_MAX_PEERS || nb < 0) return CG_EINVAL;
    if (nb == 0) return CG_OK;
    if (!w || !v || !g_local || !n || (K > 0 && !g_peers)) return CG_EINVAL;
    for (int i = 0; i < nb; ++i) {
        if (n[i] == 0) continue;
        const int rc = check_bucket(w[i], v[i], g_local[i], K > 0 ? g_peers[i] : nullptr, K, n[i]);
        if (rc) return rc;
        if (n[i] >= (1ull << 40)) return CG_EUNSUPPORTED;
    }
    ProfTag tag("reduce_sgd", -1);
    if (K > KMAX_TAB) {
        for (int i = 0; i < nb; ++i) {
            if (n[i] == 0) continue;
            PeerTable pt{};
            for (int k = 0; k < K; ++k) pt.p[k] = g_peers[i][k];
            size_t blocks = (n[i] / 4 + 255) / 256;
            if (blocks > 4096) blocks = 4096;
            if (blocks == 0) blocks = 1;
            const int rec = prof_on() ? prof_begin("reduce_sgd_kernel<any>", 0.0, (4.0 * K + 20.0) * (double)n[i], stream) : -1;
            if (tree)
                hipLaunchKernelGGL(reduce_sgd_anyk_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, stream, w[i], v[i],
                                   g_local[i], pt, K, n[i] / 4, n[i], sgd);
            else
                hipLaunchKernelGGL(reduce_sgd_anyk_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, stream, w[i], v[i],
                                   g_local[i], pt, K, n[i] / 4, n[i], sgd);
            prof_end(rec, stream);
        }
        CG_HIP_TRY(hipGetLastError());
        return CG_OK;
    }
    int i = 0;
    while (i < nb) {
        BucketTable tab{};
        unsigned long long blocks = 0;
        double bytes = 0.0;
        while (i < nb && tab.nb < MAXB) {
            if (n[i] == 0) { ++i; continue; }
            const unsigned long long per_block = (unsigned long long)tb_for(K) * unr_for(K);
            const unsigned long long bb = (n[i] / 4 + per_block - 1) / per_block;
            const unsigned long long need = bb ? bb : 1;           // a bucket of 1..3 elements still needs its tail block
            if (blocks + need >= (1ull << 31)) break;
            Bucket &bk = tab.b[tab.nb++];
            bk.w = w[i]; bk.v = v[i]; bk.g = g_local[i];
            for (int k = 0; k < K; ++k) bk.peer[k] = g_peers[i][k];
            bk.n = n[i];
            bk.first_block = (unsigned)blocks;
            blocks += need;
            bytes += (4.0 * K + 20.0) * (double)n[i];
            ++i;
        }
        if (tab.nb == 0) {
            if (i < nb) return CG_EUNSUPPORTED;     // a single bucket too large for one grid
            break;
        }
        int rec = -1;
        if (prof_on()) {
            char name[64];
            snprintf(name, sizeof name, tree ? "reduce_sgd_kernel<%d,tree>" : "reduce_sgd_kernel<%d>", K);
            rec = prof_begin(name, 0.0, bytes, stream);
        }
        launch_table(tab, (unsigned)blocks, K, tree, sgd, stream);
        prof_end(rec, stream);
        CG_HIP_TRY(hipGetLastError());
    }
    return CG_OK;
}

int grad_reduce_sgd_impl(float *w, float *v, const float *g_local, const float *const *g_peers, int K, size_t n,
                         const cg_sgd &sgd, hipStream_t stream, bool tree)
{
    if (n == 0) return (K < 0 || K > CG_MAX_PEERS) ? CG_EINVAL : CG_OK;
    return grad_reduce_sgd_multi_impl(1, &w, &v, &g_local, &g_peers, K, &n, sgd, stream, tree);
}

}  // namespace cg

extern "C" int cg_grad_reduce_sgd(float *w, float *v, const float *g_local, const float *const *g_peers, int K,
                                  size_t n, const cg_sgd *sgd, void *stream)
{
    if (!sgd) return CG_EINVAL;
    return cg::grad_reduce_sgd_impl(w, v, g_local, g_peers, K, n, *sgd, static_cast<hipStream_t>(stream), false);
}

extern "C" int cg_grad_reduce_sgd_tree(float *w, float *v, const float *g_local, const float *const *g_peers, int K,
                                       size_t n, const cg_sgd *sgd, void *stream)
{
    if (!sgd) return CG_EINVAL;
    return cg::grad_reduce_sgd_impl(w, v, g_local, g_peers, K, n, *sgd, static_cast<hipStream_t>(stream), true);
}

extern "C" int cg_grad_reduce_sgd_multi(int nb, float *const *w, float *const *v, const float *const *g_local,
                                        const float *const *const *g_peers, int K, const size_t *n, const cg_sgd *sgd,
                                        void *stream)
{
    if (!sgd) return CG_EINVAL;
    return cg::grad_reduce_sgd_multi_impl(nb, w, v, g_local, g_peers, K, n, *sgd, static_cast<hipStream_t>(stream), false);
}

extern "C" int cg_grad_reduce_sgd_tree_multi(int nb, float *const *w, float *const *v, const float *const *g_local,
                                             const float *const *const *g_peers, int K, const size_t *n,
                                             const cg_sgd *sgd, void *stream)
{
    if (!sgd) return CG_EINVAL;
    return cg::grad_reduce_sgd_multi_impl(nb, w, v, g_local, g_peers, K, n, *sgd, static_cast<hipStream_t>(stream), true);
}
