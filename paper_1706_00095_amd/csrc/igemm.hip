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
#include <cstdlib>
#include <type_traits>
#include <utility>
#include "cg_internal.h"

namespace cg {

typedef float v16f __attribute__((ext_vector_type(16)));

namespace {

#ifndef CG_KT
#define CG_KT 16
#endif
constexpr int KT = CG_KT;
#ifndef CG_SIDE
#define CG_SIDE 15   // timing experiments only: which loader step kinds run in the K loop
#endif
#ifndef CG_EXP
#define CG_EXP 0   // timing experiments only: 1 = no loader steps in the K loop
#endif

// ---- tile loaders -----------------------------------------------------------------------
// A loader moves one R x KT operand tile global -> registers -> LDS and says where the MFMA
// fragment of a lane lives in LDS (frag).  Two LDS layouts:
//   k-major  [row][k], row stride KT+4: for operands that are contiguous along k in memory;
//   row-major [k][row], row stride R+8: for operands that are contiguous along the row index.
// In both, lane (i = lane&31, h = lane>>5) of a wave fetches for one 8-wide k step the four
// values k = kb + 4h + t, t = 0..3 of row i; MFMA number t of the step consumes value t.  Which
// k a lane half holds is immaterial as long as A and B agree.
//
// The work of a loader is cut into single-element steps so that the K loop can place one step
// behind each MFMA: tables() reads the index tables of a tile into registers, issue<I, SET>()
// starts global load I into register set SET, store<I, SET>() writes it to LDS.  Whether an
// element is a real one or zero padding is kept as a bit and applied at store time, so no
// instruction between issue and store depends on the loaded value.

template <int B, class F, int... Is>
__device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, Is...>)
{
    (f(std::integral_constant<int, B + Is>{}), ...);
}
template <int B, int E, class F> __device__ __forceinline__ void static_for(F &&f)
{
    static_for_impl<B>(f, std::make_integer_sequence<int, (E > B ? E - B : 0)>{});
}

#define CG_SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)

// Validity of an element as a sign mask, in vector arithmetic only (a compare that goes through
// scalar registers costs the in-order wave more latency than the MFMA shadow hides):
// all-ones if a or b lies outside [0, limA) x [0, limB), zero otherwise.  Coordinates and limits
// are far below 2^30, so the sign bit of each term is exact.
__device__ __forceinline__ int32_t invalid_mask(int32_t a, int32_t b, int32_t limA1, int32_t limB1)
{
    return ((limA1 - a) | (limB1 - b) | a | b) >> 31;
}

template <int MODE, int R, int NTHR> struct Loader;

template <int R, int NTHR> struct Loader<LD_RMAJ_S, R, NTHR> {
    static_assert(NTHR % R == 0, "row-major loader: threads must be a multiple of tile rows");
    static constexpr int NP = NTHR / R;
    static_assert(KT % NP == 0, "row-major loader: KT must be a multiple of the k phases");
    static constexpr int CNT = KT / NP;
    static constexpr int RS = R + 8;
    static constexpr int SZ = KT * RS;
    static constexpr int RTAB = 1;
    float v[2][CNT];
    uint32_t badm[2];
    int4 ke[2];          // ring of k-table entries: step I uses ke[I & 1] and fetches the next one
    Info ri;
    int r, kp;

    __device__ __forceinline__ void init(const Operand &op, uint32_t row0, uint32_t row_limit, int t, int4 *)
    {
        r = t % R;
        kp = t / R;
        ri = map_info(op.row, row0 + r, row_limit);
    }
    __device__ __forceinline__ void tables(const int4 *ktab, const int4 *) { ke[0] = ktab[kp]; }
    template <int I, int SET>
    __device__ __forceinline__ void issue(const float *base, uint32_t limA, uint32_t limB, const int4 *ktab,
                                          const int4 *)
    {
        if constexpr (I + 1 < CNT) ke[(I + 1) & 1] = ktab[kp + (I + 1) * NP];
        const int4 e = ke[I & 1];
        const int32_t m = invalid_mask(ri.a + e.y, ri.b + e.z, (int32_t)limA - 1, (int32_t)limB - 1);
        badm[SET] = (I == 0 ? 0u : badm[SET]) | ((uint32_t)m & (1u << I));
        v[SET][I] = base[(uint32_t)((ri.off + e.x) & ~m)];
    }
    template <int I, int SET> __device__ __forceinline__ void store(float *s) const
    {
#if CG_SIDE & 16
        asm volatile("" ::"v"(v[SET][I]));            // timing experiment: wait for the load, no LDS store
#elif CG_SIDE & 32
        s[(kp + I * NP) * RS + r] = (float)I;          // timing experiment: LDS store without the load
#else
        s[(kp + I * NP) * RS + r] = (badm[SET] >> I) & 1u ? 0.f : v[SET][I];
#endif
    }
    __device__ __forceinline__ static void frag(const float *s, int row, int kb, int h, float out[4])
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
    float v[2][CNT];
    uint32_t badm[2];
    int4 ki;
    int4 re[2];          // ring of row-table entries
    int kl, r0;

    __device__ __forceinline__ void init(const Operand &op, uint32_t row0, uint32_t row_limit, int t, int4 *rtab)
    {
        kl = t % KT;
        r0 = t / KT;
        for (int rr = t; rr < R; rr += NTHR) {
            const Info q = map_info(op.row, row0 + rr, row_limit);
            rtab[rr] = make_int4(q.off, q.a, q.b, 0);
        }
    }
    __device__ __forceinline__ int row_of(int i) const { return (R % RP == 0 || r0 + i * RP < R) ? r0 + i * RP : 0; }
    __device__ __forceinline__ void tables(const int4 *ktab, const int4 *rtab)
    {
        ki = ktab[kl];
        re[0] = rtab[row_of(0)];
    }
    template <int I, int SET>
    __device__ __forceinline__ void issue(const float *base, uint32_t limA, uint32_t limB, const int4 *,
                                          const int4 *rtab)
    {
        if constexpr (I + 1 < CNT) re[(I + 1) & 1] = rtab[row_of(I + 1)];
        const int4 e = re[I & 1];
        const int32_t m = invalid_mask(e.y + ki.y, e.z + ki.z, (int32_t)limA - 1, (int32_t)limB - 1);
        badm[SET] = (I == 0 ? 0u : badm[SET]) | ((uint32_t)m & (1u << I));
        v[SET][I] = base[(uint32_t)((e.x + ki.x) & ~m)];
    }
    template <int I, int SET> __device__ __forceinline__ void store(float *s) const
    {
        const int rr = r0 + I * RP;
        if (R % RP == 0 || rr < R) s[rr * RS + kl] = (badm[SET] >> I) & 1u ? 0.f : v[SET][I];
    }
    __device__ __forceinline__ static void frag(const float *s, int row, int kb, int h, float out[4])
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
    float4 v[2][CNT];
    uint32_t badm[2];
    int4 ki;
    int4 re[2];          // ring of row-table entries
    int k4, r0;

    __device__ __forceinline__ void init(const Operand &op, uint32_t row0, uint32_t row_limit, int t, int4 *rtab)
    {
        k4 = t % KQ;
        r0 = t / KQ;
        for (int rr = t; rr < R; rr += NTHR) {
            const Info q = map_info(op.row, row0 + rr, row_limit);
            rtab[rr] = make_int4(q.off, q.a, q.b, 0);
        }
    }
    __device__ __forceinline__ int row_of(int i) const { return (R % RP == 0 || r0 + i * RP < R) ? r0 + i * RP : 0; }
    __device__ __forceinline__ void tables(const int4 *ktab, const int4 *rtab)
    {
        ki = ktab[4 * k4];
        re[0] = rtab[row_of(0)];
    }
    template <int I, int SET>
    __device__ __forceinline__ void issue(const float *base, uint32_t limA, uint32_t limB, const int4 *,
                                          const int4 *rtab)
    {
        if constexpr (I + 1 < CNT) re[(I + 1) & 1] = rtab[row_of(I + 1)];
        const int4 e = re[I & 1];
        const int32_t m = invalid_mask(e.y + ki.y, e.z + ki.z, (int32_t)limA - 1, (int32_t)limB - 1);
        badm[SET] = (I == 0 ? 0u : badm[SET]) | ((uint32_t)m & (1u << I));
        v[SET][I] = *reinterpret_cast<const float4 *>(base + (uint32_t)((e.x + ki.x) & ~m));
    }
    template <int I, int SET> __device__ __forceinline__ void store(float *s) const
    {
        const int rr = r0 + I * RP;
        if (R % RP == 0 || rr < R) {
            const int32_t keep = (badm[SET] >> I) & 1u ? 0 : -1;
            float4 q = v[SET][I];
            q.x = __int_as_float(__float_as_int(q.x) & keep); q.y = __int_as_float(__float_as_int(q.y) & keep);
            q.z = __int_as_float(__float_as_int(q.z) & keep); q.w = __int_as_float(__float_as_int(q.w) & keep);
#if CG_SIDE & 16
            asm volatile("" ::"v"(q.x), "v"(q.y), "v"(q.z), "v"(q.w));
#elif CG_SIDE & 32
            *reinterpret_cast<float4 *>(s + rr * RS + 4 * k4) = make_float4(1.f, 2.f, 3.f, 4.f);
#else
            *reinterpret_cast<float4 *>(s + rr * RS + 4 * k4) = q;
#endif
        }
    }
    __device__ __forceinline__ static void frag(const float *s, int row, int kb, int h, float out[4])
    {
        const float4 q = *reinterpret_cast<const float4 *>(s + row * RS + kb + 4 * h);
        out[0] = q.x; out[1] = q.y; out[2] = q.z; out[3] = q.w;
    }
};

}  // namespace

#if CG_EXP == 3
__device__ long long g_trace[8][8];
#define CG_T() __builtin_readcyclecounter()
#endif

// Wave-specialised K loop.  On gfx950 vector-ALU instructions of a wave do not overlap with an
// MFMA of the SAME wave (measured: MFMA + N v_add costs 64 + 12 + 4N cycles), but an MFMA-only
// wave runs at the full 64 cycles per v_mfma_f32_32x32x2_f32 while ANOTHER wave on its SIMD issues
// vector-ALU, LDS and memory instructions.  So a block is 8 waves, two per SIMD:
//   waves 0-3, consumers: LDS fragment reads and MFMAs only, each owns TM x TN 32x32 tiles;
//   waves 4-7, producers: all address arithmetic, global loads and LDS stores of the block's
//                         A and B tiles (the loaders above run on these 256 threads).
// LDS holds a ring of three K-tiles.  In iteration `it` the consumers multiply tile it (and
// prefetch the first fragments of tile it+1, complete since the previous barrier) while the
// producers store tile it+2, loaded one iteration earlier into the other register set, and issue
// the global loads of tile it+3.  One s_barrier per iteration; nobody waits for memory unless a
// load takes longer than a whole iteration.  Tiles past the end of the K range are produced as
// all padding (offset 0, stored as zeros) and never multiplied, so the loops carry no conditions.
template <int WM, int WN, int TM, int TN, int AMODE, int BMODE>
__global__ __launch_bounds__(512) void igemm_kernel(const IgemmProblem p)
{
    static_assert(WM * WN == 4, "four consumer waves");
    constexpr int NPROD = 256;
    constexpr int MT = WM * TM * 32, NT = WN * TN * 32;
    constexpr int NKS = KT / 8;                       // 8-wide k-steps per K-tile
    constexpr int NST = 3;                            // LDS ring depth
    using LA = Loader<AMODE, MT, NPROD>;
    using LB = Loader<BMODE, NT, NPROD>;
    constexpr int CA = LA::CNT, CB = LB::CNT;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    float *sA = reinterpret_cast<float *>(smem);                 // [NST][LA::SZ]
    float *sB = sA + NST * LA::SZ;                               // [NST][LB::SZ]
    int4 *kA = reinterpret_cast<int4 *>(sB + NST * LB::SZ);      // [4][KT]  k-info ring of operand A
    int4 *kB = kA + 4 * KT;                                      // [4][KT]
    int4 *rA = kB + 4 * KT;                                      // [LA::RTAB]
    int4 *rB = rA + LA::RTAB;                                    // [LB::RTAB]

    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);     // wave-uniform: lives in a scalar register

    const uint32_t m0 = blockIdx.y * MT, n0 = blockIdx.x * NT;
    const uint32_t g = blockIdx.z / p.splits, sp = blockIdx.z % p.splits;
    const uint32_t kbeg = sp * p.k_per_split;
    const uint32_t kend = min(p.K, kbeg + p.k_per_split);
    const int n_iter = (int)((kend - kbeg + KT - 1) / KT);

    if (wave >= 4) {
        // ------------------------------- producers -------------------------------------------
        const int tp = t - NPROD;
        const int pw = wave - 4;
        const float *a_base = p.A.ptr + (int64_t)g * p.A.gstride;
        const float *b_base = p.B.ptr + (int64_t)g * p.B.gstride;
        const uint32_t a_limA = p.A.limA, a_limB = p.A.limB, b_limA = p.B.limA, b_limB = p.B.limB;
        LA la;
        LB lb;
        la.init(p.A, m0, p.M, tp, rA);
        lb.init(p.B, n0, p.N, tp, rB);

        // k-info of K-tile `tile` goes to ring slot tile & 3.  Producer wave 0 makes operand A's
        // entries, producer wave 1 operand B's; the choice is wave-uniform, so the selected map
        // constants are scalar values (never a pointer into the argument block, which would put
        // a memory wait into the loop).
        const bool kw0 = pw == 0;
#define CG_KSEL(f) (kw0 ? p.A.k.f : p.B.k.f)
        const FastDiv kd1{CG_KSEL(d1.d), CG_KSEL(d1.mul), CG_KSEL(d1.sh)}, kd2{CG_KSEL(d2.d), CG_KSEL(d2.mul), CG_KSEL(d2.sh)};
        const int32_t ks1 = CG_KSEL(s1), ks2 = CG_KSEL(s2), ks3 = CG_KSEL(s3), ko0 = CG_KSEL(o0);
        const int32_t ksa = CG_KSEL(sa), ka0 = CG_KSEL(a0), ksb = CG_KSEL(sb), kb0 = CG_KSEL(b0);
#undef CG_KSEL
        int4 *const ktab_mine = kw0 ? kA : kB;
        auto put_kinfo = [&](int tile) {
            if (pw < 2 && lane < KT) {
                const uint32_t k = kbeg + (uint32_t)tile * KT + (uint32_t)lane;
                const uint32_t q1 = fdiv(k, kd1), r1 = k - q1 * kd1.d;
                const uint32_t q2 = fdiv(r1, kd2), r2 = r1 - q2 * kd2.d;
                const bool ok = k < kend;
                const int32_t off = (int32_t)q1 * ks1 + (int32_t)q2 * ks2 + (int32_t)r2 * ks3 + ko0;
                const int32_t a = (int32_t)q2 * ksa + ka0, b = (int32_t)r2 * ksb + kb0;
                ktab_mine[(tile & 3) * KT + lane] = make_int4(ok ? off : 0, ok ? a : kInvalidA, ok ? b : 0, 0);
            }
        };
        auto issue_tile = [&](auto SETC, int tile) {
            constexpr int SET = decltype(SETC)::value;
            const int4 *ka = kA + (tile & 3) * KT, *kb = kB + (tile & 3) * KT;
            la.tables(ka, rA);
            lb.tables(kb, rB);
            static_for<0, CB>([&](auto I) { lb.template issue<decltype(I)::value, SET>(b_base, b_limA, b_limB, kb, rB); });
            static_for<0, CA>([&](auto I) { la.template issue<decltype(I)::value, SET>(a_base, a_limA, a_limB, ka, rA); });
        };
        auto store_tile = [&](auto SETC, int tile) {
            constexpr int SET = decltype(SETC)::value;
            float *a_d = sA + (tile % NST) * LA::SZ, *b_d = sB + (tile % NST) * LB::SZ;
            static_for<0, CA>([&](auto I) { la.template store<decltype(I)::value, SET>(a_d); });
            static_for<0, CB>([&](auto I) { lb.template store<decltype(I)::value, SET>(b_d); });
        };
        const std::integral_constant<int, 0> S0{};
        const std::integral_constant<int, 1> S1{};

        // prologue: tiles 0 and 1 in LDS, tile 2 in flight in register set 0, k-info up to tile 3
        put_kinfo(0); put_kinfo(1); put_kinfo(2); put_kinfo(3);
        __syncthreads();
        issue_tile(S0, 0);
        issue_tile(S1, 1);
        store_tile(S0, 0);
        store_tile(S1, 1);
        issue_tile(S0, 2);
        __syncthreads();
        // iteration it: issue tile it+3 into set (it+1)&1, store tile it+2 from set it&1
#if CG_EXP == 3
        long long tw = 0, tb = 0, ti = 0;
        const long long tbeg = CG_T();
#define CG_TR_A() const long long q0 = CG_T();
#define CG_TR_I() const long long qi = CG_T();
#define CG_TR_B() const long long q1 = CG_T();
#define CG_TR_C() { const long long q2 = CG_T(); ti += qi - q0; tw += q1 - qi; tb += q2 - q1; }
#else
#define CG_TR_A()
#define CG_TR_I()
#define CG_TR_B()
#define CG_TR_C()
#endif
        for (int it = 0; it < n_iter; it += 2) {
            {
                CG_TR_A()
                issue_tile(S1, it + 3);
                put_kinfo(it + 4);
                CG_TR_I()
                store_tile(S0, it + 2);
                CG_TR_B()
                __syncthreads();
                CG_TR_C()
            }
            if (it + 1 < n_iter) {
                CG_TR_A()
                issue_tile(S0, it + 4);
                put_kinfo(it + 5);
                CG_TR_I()
                store_tile(S1, it + 3);
                CG_TR_B()
                __syncthreads();
                CG_TR_C()
            }
        }
#if CG_EXP == 3
        if (blockIdx.x == 7 && blockIdx.y == 0 && blockIdx.z == 0 && lane == 0) {
            g_trace[wave][0] = ti; g_trace[wave][1] = tw; g_trace[wave][2] = tb; g_trace[wave][3] = CG_T() - tbeg;
            g_trace[wave][4] = n_iter;
        }
#endif
        return;
    }

    // ----------------------------------- consumers -----------------------------------------------
    const int wm = wave / WN, wn = wave % WN;
    const int h = lane >> 5, li = lane & 31;
    v16f acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    float af[2][TM][4], bf[2][TN][4];      // fragments of k-step ks live in ring slot ks & 1
    auto fetch = [&](auto SLOTC, int tile, int ks) {
        constexpr int SL = decltype(SLOTC)::value;
        const float *a_s = sA + (tile % NST) * LA::SZ, *b_s = sB + (tile % NST) * LB::SZ;
#pragma unroll
        for (int i = 0; i < TM; ++i) LA::frag(a_s, (wm * TM + i) * 32 + li, ks * 8, h, af[SL][i]);
#pragma unroll
        for (int j = 0; j < TN; ++j) LB::frag(b_s, (wn * TN + j) * 32 + li, ks * 8, h, bf[SL][j]);
    };
    __syncthreads();     // producers: k-info ready
    __syncthreads();     // producers: tiles 0 and 1 stored
    fetch(std::integral_constant<int, 0>{}, 0, 0);
#if CG_EXP == 3
    long long tw = 0, tb = 0;
    const long long tbeg = CG_T();
#endif
    for (int it = 0; it < n_iter; ++it) {
#if CG_EXP == 3
        const long long q0 = CG_T();
#endif
        static_for<0, NKS>([&](auto KS) {
            constexpr int ks = decltype(KS)::value;
            // next fragments first: the LDS reads run under this k-step's MFMAs.  The last k-step
            // fetches from tile it+1, which has been complete since the previous barrier.
            if constexpr (ks + 1 < NKS) fetch(std::integral_constant<int, (ks + 1) & 1>{}, it, ks + 1);
            else fetch(std::integral_constant<int, 0>{}, it + 1, 0);
            CG_SCHED_FENCE();
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[ks & 1][i][s], bf[ks & 1][j][s], acc[i][j], 0, 0, 0);
            CG_SCHED_FENCE();
        });
#if CG_EXP == 3
        const long long q1 = CG_T();
        __syncthreads();
        const long long q2 = CG_T();
        tw += q1 - q0; tb += q2 - q1;
#else
        __syncthreads();
#endif
    }
#if CG_EXP == 3
    if (blockIdx.x == 7 && blockIdx.y == 0 && blockIdx.z == 0 && lane == 0) {
        g_trace[wave][0] = 0; g_trace[wave][1] = tw; g_trace[wave][2] = tb; g_trace[wave][3] = CG_T() - tbeg;
        g_trace[wave][4] = n_iter;
    }
#endif

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

// LDS bytes of one block of the kernel instance (ring of three K-tiles + index tables)
template <int WM, int WN, int TM, int TN, int AMODE, int BMODE> constexpr size_t igemm_lds_bytes()
{
    using LA = Loader<AMODE, WM * TM * 32, 256>;
    using LB = Loader<BMODE, WN * TN * 32, 256>;
    return 3 * (LA::SZ + LB::SZ) * sizeof(float) + (8 * KT + LA::RTAB + LB::RTAB) * sizeof(int4);
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
    constexpr size_t lds = igemm_lds_bytes<WM, WN, TM, TN, AMODE, BMODE>();
    static_assert(lds <= 160 * 1024, "tile does not fit the LDS of a compute unit");
    static bool attr_set = false;      // raising the dynamic-LDS limit is a per-kernel, one-time host call
    if (!attr_set) {
        CG_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(&igemm_kernel<WM, WN, TM, TN, AMODE, BMODE>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        attr_set = true;
    }
    hipLaunchKernelGGL((igemm_kernel<WM, WN, TM, TN, AMODE, BMODE>), grid, dim3(512), lds, stream, p);
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


#if CG_EXP == 3
extern "C" int cg_debug_read_trace(long long *host)
{
    return hipMemcpyFromSymbol(host, HIP_SYMBOL(g_trace), sizeof(long long) * 64) == hipSuccess ? 0 : -4;
}
#endif

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
#if CG_EXP
    if (getenv("CG_NO_SPLIT")) return pl;
#endif
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
