// Implicit-GEMM kernel on the fp32 matrix cores of gfx950.
//
// One kernel template computes C[m][n] = sum_k A(m,k) * B(n,k) for every dense contraction of
// the iteration: convolution forward, backward-data and backward-weight, and the three
// fully-connected passes.  Operand elements are addressed through index maps (cg_internal.h),
// so the im2col matrix is never materialised: a tile of it is gathered straight from the NCHW
// tensor into LDS, with zero padding folded into the validity test.
//
// Work decomposition: a block of 4 waves owns an MT x 128 tile of C; each wave owns TM x TN
// sub-tiles of 32x32, accumulated by v_mfma_f32_32x32x2_f32.  The K loop advances KT = 16 at a
// time; the global loads of tile i+1 are issued into registers before the MFMAs of tile i and
// written to the other LDS buffer afterwards, so one barrier per K-tile suffices.
#include <cstdio>
#include "cg_internal.h"

namespace cg {

typedef float v16f __attribute__((ext_vector_type(16)));

namespace {

constexpr int KT = 16;

// ---- tile loaders -----------------------------------------------------------------------
// A loader moves one R x KT operand tile global -> registers (gload) -> LDS (sstore) and says
// where the MFMA fragment of a lane lives in LDS (frag).  Two LDS layouts:
//   k-major  [row][k], row stride KT+4: for operands that are contiguous along k in memory;
//   row-major [k][row], row stride R+8: for operands that are contiguous along the row index.
// In both, lane (i = lane&31, h = lane>>5) of a wave fetches for one 8-wide k step the four
// values k = kb + 4h + t, t = 0..3 of row i; MFMA number t of the step consumes value t.  Which
// k a lane half holds is immaterial as long as A and B agree.

template <int MODE, int R, int NTHR> struct Loader;

template <int R, int NTHR> struct Loader<LD_RMAJ_S, R, NTHR> {
    static_assert(NTHR % R == 0, "row-major loader: threads must be a multiple of tile rows");
    static constexpr int NP = NTHR / R;
    static_assert(KT % NP == 0, "row-major loader: KT must be a multiple of the k phases");
    static constexpr int CNT = KT / NP;
    static constexpr int RS = R + 8;
    static constexpr int SZ = KT * RS;
    static constexpr int RTAB = 1;
    float v[CNT];
    Info ri;
    int r, kp;

    __device__ void init(const Operand &op, uint32_t row0, uint32_t row_limit, int t, int4 *)
    {
        r = t % R;
        kp = t / R;
        ri = map_info(op.row, row0 + r, row_limit);
    }
    __device__ void gload(const float *base, uint32_t limA, uint32_t limB, const int4 *ktab, const int4 *)
    {
#pragma unroll
        for (int i = 0; i < CNT; ++i) {
            const int4 ki = ktab[kp + i * NP];
            const bool ok = (uint32_t)(ri.a + ki.y) < limA && (uint32_t)(ri.b + ki.z) < limB;
            const uint32_t off = ok ? (uint32_t)(ri.off + ki.x) : 0u;
            const float x = base[off];
            v[i] = ok ? x : 0.f;
        }
    }
    __device__ void sstore(float *s) const
    {
#pragma unroll
        for (int i = 0; i < CNT; ++i) s[(kp + i * NP) * RS + r] = v[i];
    }
    // fragment: 4 scalars
    __device__ static void frag(const float *s, int row, int kb, int h, float out[4])
    {
#pragma unroll
        for (int t = 0; t < 4; ++t) out[t] = s[(kb + 4 * h + t) * RS + row];
    }
};

template <int R, int NTHR> struct Loader<LD_KMAJ_S, R, NTHR> {
    static_assert(NTHR % KT == 0, "");
    static constexpr int RP = NTHR / KT;
    static constexpr int CNT = (R + RP - 1) / RP;
    static constexpr int RS = KT + 4;
    static constexpr int SZ = R * RS;
    static constexpr int RTAB = R;
    float v[CNT];
    int kl, r0;

    __device__ void init(const Operand &op, uint32_t row0, uint32_t row_limit, int t, int4 *rtab)
    {
        kl = t % KT;
        r0 = t / KT;
        for (int r = t; r < R; r += NTHR) {
            const Info ri = map_info(op.row, row0 + r, row_limit);
            rtab[r] = make_int4(ri.off, ri.a, ri.b, 0);
        }
    }
    __device__ void gload(const float *base, uint32_t limA, uint32_t limB, const int4 *ktab, const int4 *rtab)
    {
        const int4 ki = ktab[kl];
#pragma unroll
        for (int i = 0; i < CNT; ++i) {
            const int r = r0 + i * RP;
            if (R % RP == 0 || r < R) {
                const int4 ri = rtab[r];
                const bool ok = (uint32_t)(ri.y + ki.y) < limA && (uint32_t)(ri.z + ki.z) < limB;
                const uint32_t off = ok ? (uint32_t)(ri.x + ki.x) : 0u;
                const float x = base[off];
                v[i] = ok ? x : 0.f;
            }
        }
    }
    __device__ void sstore(float *s) const
    {
#pragma unroll
        for (int i = 0; i < CNT; ++i) {
            const int r = r0 + i * RP;
            if (R % RP == 0 || r < R) s[r * RS + kl] = v[i];
        }
    }
    __device__ static void frag(const float *s, int row, int kb, int h, float out[4])
    {
        const float4 q = *reinterpret_cast<const float4 *>(s + row * RS + kb + 4 * h);
        out[0] = q.x; out[1] = q.y; out[2] = q.z; out[3] = q.w;
    }
};

template <int R, int NTHR> struct Loader<LD_KMAJ_V4, R, NTHR> {
    static constexpr int KQ = KT / 4;
    static constexpr int RP = NTHR / KQ;
    static constexpr int CNT = (R + RP - 1) / RP;
    static constexpr int RS = KT + 4;
    static constexpr int SZ = R * RS;
    static constexpr int RTAB = R;
    float4 v[CNT];
    int k4, r0;

    __device__ void init(const Operand &op, uint32_t row0, uint32_t row_limit, int t, int4 *rtab)
    {
        k4 = t % KQ;
        r0 = t / KQ;
        for (int r = t; r < R; r += NTHR) {
            const Info ri = map_info(op.row, row0 + r, row_limit);
            rtab[r] = make_int4(ri.off, ri.a, ri.b, 0);
        }
    }
    __device__ void gload(const float *base, uint32_t limA, uint32_t limB, const int4 *ktab, const int4 *rtab)
    {
        const int4 ki = ktab[4 * k4];
#pragma unroll
        for (int i = 0; i < CNT; ++i) {
            const int r = r0 + i * RP;
            if (R % RP == 0 || r < R) {
                const int4 ri = rtab[r];
                const bool ok = (uint32_t)(ri.y + ki.y) < limA && (uint32_t)(ri.z + ki.z) < limB;
                const uint32_t off = ok ? (uint32_t)(ri.x + ki.x) : 0u;
                const float4 x = *reinterpret_cast<const float4 *>(base + off);
                v[i] = ok ? x : make_float4(0.f, 0.f, 0.f, 0.f);
            }
        }
    }
    __device__ void sstore(float *s) const
    {
#pragma unroll
        for (int i = 0; i < CNT; ++i) {
            const int r = r0 + i * RP;
            if (R % RP == 0 || r < R) *reinterpret_cast<float4 *>(s + r * RS + 4 * k4) = v[i];
        }
    }
    __device__ static void frag(const float *s, int row, int kb, int h, float out[4])
    {
        const float4 q = *reinterpret_cast<const float4 *>(s + row * RS + kb + 4 * h);
        out[0] = q.x; out[1] = q.y; out[2] = q.z; out[3] = q.w;
    }
};

}  // namespace

template <int WM, int WN, int TM, int TN, int AMODE, int BMODE>
__global__ __launch_bounds__(WM *WN * 64) void igemm_kernel(const IgemmProblem p)
{
    constexpr int NTHR = WM * WN * 64;
    constexpr int MT = WM * TM * 32, NT = WN * TN * 32;
    using LA = Loader<AMODE, MT, NTHR>;
    using LB = Loader<BMODE, NT, NTHR>;

    __shared__ __attribute__((aligned(16))) float sA[2][LA::SZ];
    __shared__ __attribute__((aligned(16))) float sB[2][LB::SZ];
    __shared__ int4 kA[2][KT];
    __shared__ int4 kB[2][KT];
    __shared__ int4 rA[LA::RTAB];
    __shared__ int4 rB[LB::RTAB];

    const int t = threadIdx.x;
    const int lane = t & 63, wave = t >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int h = lane >> 5, li = lane & 31;

    const uint32_t m0 = blockIdx.y * MT, n0 = blockIdx.x * NT;
    const uint32_t g = blockIdx.z / p.splits, sp = blockIdx.z % p.splits;
    const uint32_t kbeg = sp * p.k_per_split;
    const uint32_t kend = min(p.K, kbeg + p.k_per_split);
    const int n_iter = (int)((kend - kbeg + KT - 1) / KT);

    const float *a_base = p.A.ptr + (int64_t)g * p.A.gstride;
    const float *b_base = p.B.ptr + (int64_t)g * p.B.gstride;

    LA la;
    LB lb;
    la.init(p.A, m0, p.M, t, rA);
    lb.init(p.B, n0, p.N, t, rB);

    // k-info of K-tile `it` is produced by the first 2*KT threads into table (it & 1)
    auto put_kinfo = [&](int it) {
        if (t < 2 * KT) {
            const uint32_t k = kbeg + (uint32_t)it * KT + (uint32_t)(t & (KT - 1));
            const Info ki = map_info(t < KT ? p.A.k : p.B.k, k, kend);
            (t < KT ? kA : kB)[it & 1][t & (KT - 1)] = make_int4(ki.off, ki.a, ki.b, 0);
        }
    };

    v16f acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    put_kinfo(0);
    __syncthreads();
    la.gload(a_base, p.A.limA, p.A.limB, kA[0], rA);
    lb.gload(b_base, p.B.limA, p.B.limB, kB[0], rB);
    if (n_iter > 1) put_kinfo(1);
    la.sstore(sA[0]);
    lb.sstore(sB[0]);
    __syncthreads();

    for (int it = 0; it < n_iter; ++it) {
        const int cur = it & 1;
        if (it + 1 < n_iter) {
            la.gload(a_base, p.A.limA, p.A.limB, kA[cur ^ 1], rA);
            lb.gload(b_base, p.B.limA, p.B.limB, kB[cur ^ 1], rB);
        }
        if (it + 2 < n_iter) put_kinfo(it + 2);

        const float *a_s = sA[cur];
        const float *b_s = sB[cur];
#pragma unroll
        for (int kb = 0; kb < KT; kb += 8) {
            float af[TM][4], bf[TN][4];
#pragma unroll
            for (int i = 0; i < TM; ++i) LA::frag(a_s, (wm * TM + i) * 32 + li, kb, h, af[i]);
#pragma unroll
            for (int j = 0; j < TN; ++j) LB::frag(b_s, (wn * TN + j) * 32 + li, kb, h, bf[j]);
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[i][s], bf[j][s], acc[i][j], 0, 0, 0);
        }

        if (it + 1 < n_iter) {
            la.sstore(sA[cur ^ 1]);
            lb.sstore(sB[cur ^ 1]);
        }
        __syncthreads();
    }

    // Epilogue.  Accumulator register r of lane (h, li) holds C row 8*(r/4) + 4*h + r%4,
    // column li of its 32x32 sub-tile.
    float *c_base = p.c_ptr + (int64_t)g * p.c_gstride + (int64_t)sp * p.c_split_stride;
    const float *bias = p.bias_mode ? p.bias + (int64_t)g * p.bias_gstride : nullptr;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const uint32_t n = n0 + (uint32_t)((wn * TN + j) * 32 + li);
        if (n >= p.N) continue;
        const Info ci = map_info(p.c_col, n, p.N);
        const float bcol = p.bias_mode == 2 ? bias[n] : 0.f;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const uint32_t m = m0 + (uint32_t)((wm * TM + i) * 32 + (r >> 2) * 8 + h * 4 + (r & 3));
                if (m < p.M) {
                    float val = acc[i][j][r] + bcol;
                    if (p.bias_mode == 1) val += bias[m];
                    float *dst = c_base + ((int32_t)m * p.c_row_stride + ci.off);
                    if (p.accumulate) val += *dst;
                    *dst = val;
                }
            }
        }
    }
}

namespace {

template <int WM, int WN, int TM, int TN, int AMODE, int BMODE>
int launch_cfg(const IgemmProblem &p, hipStream_t stream)
{
    constexpr int MT = WM * TM * 32, NT = WN * TN * 32;
    dim3 grid((p.N + NT - 1) / NT, (p.M + MT - 1) / MT, p.groups * p.splits);
    if (grid.y > 65535u || grid.z > 65535u) return CG_EUNSUPPORTED;
    int rec = -1;
    if (prof_on()) {
        char name[64];
        snprintf(name, sizeof name, "igemm_kernel<%d,%d,%d,%d,%d,%d>", WM, WN, TM, TN, AMODE, BMODE);
        rec = prof_begin(name, 2.0 * p.M * (double)p.N * p.K * p.groups, 0.0, stream);
    }
    hipLaunchKernelGGL((igemm_kernel<WM, WN, TM, TN, AMODE, BMODE>), grid, dim3(WM * WN * 64), 0, stream, p);
    prof_end(rec, stream);
    CG_HIP_TRY(hipGetLastError());
    return CG_OK;
}

template <int AMODE, int BMODE>
int launch_modes(const IgemmProblem &p, int mt, hipStream_t stream)
{
    switch (mt) {
    case 128: return launch_cfg<2, 2, 2, 2, AMODE, BMODE>(p, stream);
    case 96:
        if constexpr (AMODE != LD_RMAJ_S) return launch_cfg<1, 4, 3, 1, AMODE, BMODE>(p, stream);
        else return CG_EUNSUPPORTED;
    case 64: return launch_cfg<1, 4, 2, 1, AMODE, BMODE>(p, stream);
    default: return launch_cfg<1, 4, 1, 1, AMODE, BMODE>(p, stream);
    }
}

int pick_mt(uint32_t M, bool allow96)
{
    const int cand[4] = {128, 96, 64, 32};
    int best = 0;
    uint64_t best_cost = ~0ull;
    for (int c : cand) {
        if (c == 96 && !allow96) continue;
        const uint64_t cost = (uint64_t)((M + c - 1) / c) * c;
        if (cost < best_cost) { best_cost = cost; best = c; }   // ties keep the larger tile
    }
    return best;
}

bool operand_ok(const Operand &o)
{
    return o.ptr && aligned16(o.ptr) && o.row.count > 0 && o.k.count > 0;
}

}  // namespace

FastDiv make_fastdiv(uint32_t d)
{
    // mul = ceil(2^(31+L) / d) with L = ceil(log2 d): exact quotients for all n < 2^31.
    FastDiv f;
    f.d = d ? d : 1;
    uint32_t L = 0;
    while ((1ull << L) < f.d) ++L;
    f.sh = 31 + L;
    f.mul = (uint32_t)(((1ull << f.sh) + f.d - 1) / f.d);
    return f;
}

IndexMap linear_map(uint32_t count, int32_t stride)
{
    IndexMap m{};
    m.count = count;
    m.d1 = make_fastdiv(1);
    m.d2 = make_fastdiv(1);
    m.s1 = stride;
    return m;
}

IndexMap split_map(uint32_t count, uint32_t d, int32_t sq, int32_t sr)
{
    IndexMap m{};
    m.count = count;
    m.d1 = make_fastdiv(d);
    m.d2 = make_fastdiv(1);
    m.s1 = sq;
    m.s2 = sr;
    return m;
}

void igemm_host_element(const Operand &op, uint32_t row, uint32_t k, uint32_t K, int64_t *off, int *valid)
{
    const Info r = map_info(op.row, row, op.row.count), q = map_info(op.k, k, K);
    *valid = (uint32_t)(r.a + q.a) < op.limA && (uint32_t)(r.b + q.b) < op.limB;
    *off = (int64_t)r.off + q.off;
}

int igemm_launch(const IgemmProblem &p, hipStream_t stream)
{
    if (!operand_ok(p.A) || !operand_ok(p.B) || !p.c_ptr || !aligned16(p.c_ptr)) return CG_EINVAL;
    if (p.M == 0 || p.N == 0 || p.K == 0 || p.groups == 0 || p.splits == 0) return CG_EINVAL;
    if (p.M >= (1u << 31) || p.N >= (1u << 31) || p.K >= (1u << 31)) return CG_EUNSUPPORTED;
    if (p.A.row.count != p.M || p.B.row.count != p.N || p.A.k.count != p.K || p.B.k.count != p.K) return CG_EINVAL;
    if (p.splits > 1 && (p.k_per_split % KT != 0)) return CG_EINVAL;
    if ((uint64_t)p.k_per_split * p.splits < p.K || (uint64_t)p.k_per_split * (p.splits - 1) >= p.K) return CG_EINVAL;
    if (p.bias_mode && !p.bias) return CG_EINVAL;
    if (p.a_mode == LD_KMAJ_V4 && (!p.A.vec4_ok || p.K % 4)) return CG_EINVAL;
    if (p.b_mode == LD_KMAJ_V4 && (!p.B.vec4_ok || p.K % 4)) return CG_EINVAL;

    const int mt = pick_mt(p.M, p.a_mode != LD_RMAJ_S);
    const int am = p.a_mode, bm = p.b_mode;
    if (am == LD_KMAJ_V4 && bm == LD_RMAJ_S) return launch_modes<LD_KMAJ_V4, LD_RMAJ_S>(p, mt, stream);
    if (am == LD_KMAJ_S && bm == LD_RMAJ_S) return launch_modes<LD_KMAJ_S, LD_RMAJ_S>(p, mt, stream);
    if (am == LD_KMAJ_S && bm == LD_KMAJ_S) return launch_modes<LD_KMAJ_S, LD_KMAJ_S>(p, mt, stream);
    if (am == LD_KMAJ_V4 && bm == LD_KMAJ_V4) return launch_modes<LD_KMAJ_V4, LD_KMAJ_V4>(p, mt, stream);
    if (am == LD_RMAJ_S && bm == LD_RMAJ_S) return launch_modes<LD_RMAJ_S, LD_RMAJ_S>(p, mt, stream);
    return CG_EUNSUPPORTED;
}

// ---- split-K: more blocks for problems whose C has few tiles ---------------------------------

namespace {

struct FinishArgs {
    const float *part;
    int64_t plane;            // floats between consecutive K slices: groups * M * N
    int splits;
    float *c_ptr;
    int32_t c_row_stride;
    IndexMap c_col;
    int64_t c_gstride;
    const float *bias;
    int bias_mode;
    int32_t bias_gstride;
    uint32_t M, N;
    FastDiv divN, divMN;
    int accumulate;
    uint32_t total;           // groups * M * N
};

// C = (sum over K slices, in slice order) + bias, written through the problem's output map.
__global__ __launch_bounds__(256) void splitk_finish_kernel(const FinishArgs a)
{
    for (uint32_t i = blockIdx.x * 256 + threadIdx.x; i < a.total; i += gridDim.x * 256) {
        float s = a.part[i];
        for (int k = 1; k < a.splits; ++k) s += a.part[(int64_t)k * a.plane + i];
        const uint32_t g = fdiv(i, a.divMN), r = i - g * a.divMN.d;
        const uint32_t m = fdiv(r, a.divN), n = r - m * a.divN.d;
        if (a.bias_mode == 1) s += a.bias[(int64_t)g * a.bias_gstride + m];
        else if (a.bias_mode == 2) s += a.bias[(int64_t)g * a.bias_gstride + n];
        const Info ci = map_info(a.c_col, n, a.N);
        float *dst = a.c_ptr + (int64_t)g * a.c_gstride + ((int32_t)m * a.c_row_stride + ci.off);
        if (a.accumulate) s += *dst;
        *dst = s;
    }
}

}  // namespace

SplitPlan plan_split(uint32_t M, uint32_t N, uint32_t K, uint32_t groups, int a_mode)
{
    SplitPlan pl{1, K, 0};
    const uint32_t mt = (uint32_t)pick_mt(M, a_mode != LD_RMAJ_S);
    const uint64_t tiles = (uint64_t)((M + mt - 1) / mt) * ((N + 127) / 128) * groups;
    if (tiles >= 512) return pl;
    uint64_t want = (1024 + tiles - 1) / tiles;      // aim at ~4 resident blocks per compute unit
    const uint64_t max_by_k = K / 128;               // keep at least 8 K-tiles per slice
    if (want > max_by_k) want = max_by_k;
    if (want > 512) want = 512;
    if (want < 2) return pl;
    if ((uint64_t)groups * M * N >= (1ull << 31)) return pl;
    uint64_t per = (K + want - 1) / want;
    per = (per + KT - 1) / KT * KT;
    pl.k_per_split = (uint32_t)per;
    pl.splits = (uint32_t)((K + per - 1) / per);
    if (pl.splits < 2) return SplitPlan{1, K, 0};
    pl.ws_bytes = (size_t)pl.splits * groups * M * N * sizeof(float);
    return pl;
}

size_t igemm_ws_bytes(const IgemmProblem &p)
{
    return plan_split(p.M, p.N, p.K, p.groups, p.a_mode).ws_bytes;
}

int igemm_run(const IgemmProblem &p0, void *ws, size_t ws_bytes, hipStream_t stream)
{
    const SplitPlan pl = plan_split(p0.M, p0.N, p0.K, p0.groups, p0.a_mode);
    if (pl.splits <= 1) {
        IgemmProblem p = p0;
        p.splits = 1; p.k_per_split = p.K;
        return igemm_launch(p, stream);
    }
    if (!ws || ws_bytes < pl.ws_bytes) return CG_ENOSPC;
    if (!aligned16(ws) || !p0.c_ptr) return CG_EINVAL;
    if (p0.bias_mode && !p0.bias) return CG_EINVAL;
    IgemmProblem p = p0;
    p.c_ptr = static_cast<float *>(ws);
    p.c_row_stride = (int32_t)p0.N;
    p.c_col = linear_map(p0.N, 1);
    p.c_gstride = (int64_t)p0.M * p0.N;
    p.c_split_stride = (int64_t)p0.groups * p0.M * p0.N;
    p.bias = nullptr; p.bias_mode = 0; p.accumulate = 0;
    p.splits = pl.splits; p.k_per_split = pl.k_per_split;
    const int rc = igemm_launch(p, stream);
    if (rc) return rc;
    FinishArgs a{};
    a.part = static_cast<const float *>(ws);
    a.plane = p.c_split_stride;
    a.splits = (int)pl.splits;
    a.c_ptr = p0.c_ptr; a.c_row_stride = p0.c_row_stride; a.c_col = p0.c_col; a.c_gstride = p0.c_gstride;
    a.bias = p0.bias; a.bias_mode = p0.bias_mode; a.bias_gstride = p0.bias_gstride;
    a.M = p0.M; a.N = p0.N;
    a.divN = make_fastdiv(p0.N);
    a.divMN = make_fastdiv(p0.M * p0.N);
    a.accumulate = p0.accumulate;
    a.total = p0.groups * p0.M * p0.N;
    const unsigned blocks = (a.total + 255) / 256 < 8192 ? (a.total + 255) / 256 : 8192;
    hipLaunchKernelGGL(splitk_finish_kernel, dim3(blocks), dim3(256), 0, stream, a);
    CG_HIP_TRY(hipGetLastError());
    return CG_OK;
}

// ---- bias gradient of a convolution: db[m] = sum over n and pixels of dy[n][m][pix] ------------

namespace {

// block (m, s) sums the samples of slice s; the slices are added afterwards in slice order
__global__ __launch_bounds__(256) void bias_grad_partial_kernel(const float *__restrict__ dy, int N, int M, int P,
                                                                int n_per, float *__restrict__ part)
{
    const int m = blockIdx.x, sl = blockIdx.y;
    const int n_beg = sl * n_per, n_end = min(N, n_beg + n_per);
    float s = 0.f;
    for (int n = n_beg; n < n_end; ++n) {
        const float *src = dy + ((size_t)n * M + m) * P;
        for (int q = threadIdx.x; q < P; q += 256) s += src[q];
    }
    __shared__ float red[256];
    red[threadIdx.x] = s;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) part[(size_t)sl * M + m] = red[0];
}

__global__ __launch_bounds__(256) void bias_grad_finish_kernel(const float *__restrict__ part, int M, int S,
                                                               float *__restrict__ db)
{
    const int m = blockIdx.x * 256 + threadIdx.x;
    if (m >= M) return;
    float s = 0.f;
    for (int k = 0; k < S; ++k) s += part[(size_t)k * M + m];
    db[m] = s;
}

int bias_slices(int N, int M)
{
    int S = (2048 + M - 1) / M;
    if (S > N) S = N;
    return S < 1 ? 1 : S;
}

}  // namespace

size_t bias_grad_ws_bytes(int N, int M)
{
    return (size_t)bias_slices(N, M) * M * sizeof(float);
}

int bias_grad_launch(const float *dy, int N, int M, int P, float *db, void *ws, size_t ws_bytes,
                     hipStream_t stream)
{
    if (!dy || !db || N <= 0 || M <= 0 || P <= 0) return CG_EINVAL;
    if (!ws || ws_bytes < bias_grad_ws_bytes(N, M)) return CG_ENOSPC;
    const int S = bias_slices(N, M);
    const int n_per = (N + S - 1) / S;
    const int S2 = (N + n_per - 1) / n_per;
    float *part = static_cast<float *>(ws);
    hipLaunchKernelGGL(bias_grad_partial_kernel, dim3(M, S2), dim3(256), 0, stream, dy, N, M, P, n_per, part);
    CG_HIP_TRY(hipGetLastError());
    hipLaunchKernelGGL(bias_grad_finish_kernel, dim3((M + 255) / 256), dim3(256), 0, stream, part, M, S2, db);
    CG_HIP_TRY(hipGetLastError());
    return CG_OK;
}

}  // namespace cg
