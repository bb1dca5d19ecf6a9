// Implicit-GEMM kernel on the fp32 matrix cores of gfx950.
//
// One kernel template computes C[m][n] = sum_k A(m,k) * B(n,k) for every dense contraction of
// the iteration: convolution forward, backward-data and backward-weight, and the three
// fully-connected passes.  Operand elements are addressed through index maps (cg_internal.h),
// so the im2col matrix is never materialised: a tile of it is gathered straight from the NCHW
// tensor into LDS, with zero padding folded into the load address.
//
// Work decomposition: a block of 4 waves owns an MT x 128 tile of C; each wave owns TM x TN
// sub-tiles of 32x32, accumulated by v_mfma_f32_32x32x2_f32.  The K loop advances KT = 16 at a
// time through a ring of NST LDS stages.  Operand tiles travel global memory -> LDS directly
// (buffer loads with the LDS modifier: no register round trip, no LDS store instructions), and an
// element that is zero padding, lies beyond the tile's rows or beyond K gets an offset outside the
// buffer descriptor's range, for which the hardware writes 0.  The loads of tile it+NST-1 are
// issued while tile it is multiplied; one s_barrier per K-tile.
#include <atomic>
#include <cstdio>
#include <cstdlib>
#include <type_traits>
#include <utility>
#include "cg_internal.h"

// This file is compiled three times.  CG_MATH = 0 (the default) multiplies in fp32 and holds
// everything: kernels, planning, K slices, bias gradient.  CG_MATH = 1 and 2 build only the two
// main kernels and their launchers once more, for the bf16 matrix instructions: the tiles travel
// and lie in LDS as fp32 exactly as before, a lane rounds its fragments to bf16 (nearest even)
// and one v_mfma_f32_32x32x16_bf16 per accumulator multiplies a whole K-tile of 16.
//   1 (CG_MATH_BF16):   a*b with a, b rounded to bf16, accumulated in fp32.
//   2 (CG_MATH_BF16X3): a = ah + al, b = bh + bl (ah = bf16(a), al = bf16(a - ah)), three products
//                       al*bh + ah*bl + ah*bh: what is dropped is al*bl, about 2^-16 of a product.
#ifndef CG_MATH
#define CG_MATH 0
#endif
#if CG_MATH == 0
#define CG_IGEMM_LAUNCH igemm_launch
#elif CG_MATH == 1
#define CG_IGEMM_LAUNCH igemm_launch_bf16
#else
#define CG_IGEMM_LAUNCH igemm_launch_bf16x3
#endif

namespace cg {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) float lds_float;
typedef uint32_t BufferRsrc __attribute__((ext_vector_type(4)));   // the four descriptor words of a raw buffer

namespace {

// Blocks a split-K launch aims at, from below: two blocks are resident per compute unit, so up to
// 512 blocks start together and finish together.  A few blocks more than a whole number of such
// rounds run an extra round on a nearly empty GPU (1040 blocks took 19 % longer than 1000 on the
// backward-weight shapes of the benchmark), and one round measured faster than two or three.
#ifndef CG_SPLIT_BLOCKS
#define CG_SPLIT_BLOCKS 512
#endif
constexpr uint64_t kSplitBlocks = CG_SPLIT_BLOCKS;
// Blocks of the matrix kernels the GPU keeps resident at once: two per compute unit of the current
// device (512 on the 256 units of an MI355X), unless a test has set a lower count.
static std::atomic<uint32_t> g_resident_override{0};
uint32_t resident_blocks()
{
    const uint32_t o = g_resident_override.load(std::memory_order_relaxed);
    if (o) return o;
    static std::atomic<uint32_t> cached{0};
    uint32_t c = cached.load(std::memory_order_relaxed);
    if (!c) {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0)
            c = 2u * (uint32_t)cus;
        else
            c = 512;
        cached.store(c, std::memory_order_relaxed);
    }
    return c;
}

constexpr int KT = 16;                       // reduction indices per LDS stage (a ring of NST stages)
constexpr int NPART = KT / 2;                // MFMA steps per tile = parts the loads of a tile are issued in
// Offsets that no buffer descriptor of this library covers (descriptors span < 0x7fffff00 bytes).
// Their sum does not wrap, and either one added to a valid offset (< 2^31) stays out of range.
constexpr uint32_t OOB_ROW = 0x80000000u, OOB_K = 0x7fffff00u;
constexpr uint64_t kMaxBufferBytes = 0x7fffff00ull;

template <int B, class F, int... Is>
__device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, Is...>)
{
    (f(std::integral_constant<int, B + Is>{}), ...);
}
template <int B, int E, class F> __device__ __forceinline__ void static_for(F &&f)
{
    static_for_impl<B>(f, std::make_integer_sequence<int, (E > B ? E - B : 0)>{});
}

// The eight fp32 fragment values a lane holds of a K-tile (k = 8*ks + 4*h + t, ks = 0..1, t = 0..3)
// as the bf16 operand vector of v_mfma_f32_32x32x16_bf16, whose lane half h supplies k slots
// 8h..8h+7: slot 4*ks + t.  Which k sits in which slot is immaterial as long as A and B agree.
template <bool SPLIT>
__device__ __forceinline__ void to_bf16(const float (&f)[KT / 8][4], bf16x8 &hi, bf16x8 &lo)
{
#pragma unroll
    for (int ks = 0; ks < KT / 8; ++ks)
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const float x = f[ks][t];
            const __bf16 xh = (__bf16)x;
            hi[4 * ks + t] = xh;
            if (SPLIT) lo[4 * ks + t] = (__bf16)(x - (float)xh);
        }
}

// 64 lanes x 4 bytes, global memory -> LDS: lane l's element lands at lds + 4*l.  `lds` and `soff`
// are wave-uniform.  Written as assembly so that the waits stay under this file's control: the
// kernel below waits for exactly the tile it is about to read (s_waitcnt vmcnt(n)), whereas the
// compiler, told that a load writes LDS, drains every load in flight before each LDS read.
// The hazard recognizer does not look inside assembly: a scalar register written by a preceding
// vector instruction (a readfirstlane, or a v_readlane that restores a spilled register, the buffer
// descriptor included) may not be read by a vector-memory instruction for five wait states (one for
// M0), so the s_mov and the s_nop 3 of this form supply them.  The short forms below (s_nop 0) are
// for kernels that spill no scalar register, which the build checks (build.py).
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void load_to_lds(BufferRsrc rsrc, const float *lds, uint32_t voff, uint32_t soff)
{
    const uint32_t lds_addr = (uint32_t)(size_t)(const lds_float *)lds;
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 3\n\tbuffer_load_dword %1, %2, %3 offen lds"
                 ::"s"(lds_addr), "v"(voff), "s"(rsrc), "s"(__builtin_amdgcn_readfirstlane(soff))
                 : "memory", "m0");
}
// The same without a scalar offset: no scalar register a vector instruction may just have written is
// read, and the one wait state M0 needs is enough.  A load with its set-up costs the matrix pipeline
// about 6 % of a four-MFMA step with four wait states and 4 % with one (measured on a loop of MFMAs).
__device__ __forceinline__ void load_to_lds(BufferRsrc rsrc, const float *lds, uint32_t voff)
{
    const uint32_t lds_addr = (uint32_t)(size_t)(const lds_float *)lds;
#if CG_MATH == 0
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, 0 offen lds"
                 ::"s"(lds_addr), "v"(voff), "s"(rsrc) : "memory", "m0");
#else   // the bf16 instances of the gathered kernel spill scalar registers: the long form throughout
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 3\n\tbuffer_load_dword %1, %2, 0 offen lds"
                 ::"s"(lds_addr), "v"(voff), "s"(rsrc) : "memory", "m0");
#endif
}
// 64 lanes x 16 bytes: lane l's four elements land at lds + 16*l.
constexpr int kShortWS = CG_MATH == 0 ? 1 : 4;
template <int WS = kShortWS>
__device__ __forceinline__ void load4_to_lds(BufferRsrc rsrc, const float *lds, uint32_t voff)
{
    const uint32_t lds_addr = (uint32_t)(size_t)(const lds_float *)lds;
    if constexpr (WS == 1)
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                     ::"s"(lds_addr), "v"(voff), "s"(rsrc) : "memory", "m0");
    else
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 3\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                     ::"s"(lds_addr), "v"(voff), "s"(rsrc) : "memory", "m0");
}
#pragma clang diagnostic pop

// ---- tile loaders -------------------------------------------------------------------------------
// A loader brings one R x KT operand tile into an LDS stage and says where the MFMA fragment of a
// lane lives there.  One load instruction moves 64 elements that land contiguously in LDS, so the
// lanes run along whichever index is contiguous in memory:
//   RowsLoader: lanes = 64 consecutive rows at one k.  Stage layout [k][RS], RS = 64*chunks + 8.
//               Row offsets (and window origins) live in registers for the whole K loop; the k part
//               is wave-uniform and travels in the scalar offset of the load.
//   KLoader:    lanes = 4 rows x 16 consecutive k.  Stage layout [row/4][68] with row%4 and k inside
//               the 64-float group.  The k part is computed per lane once per tile.
// In both, lane (i = lane&31, h = lane>>5) of a wave fetches for one 8-wide k step the four values
// k = 8*ks + 4h + t, t = 0..3 of row i; MFMA number t of the step consumes value t.  Which k a
// lane half holds is immaterial as long as A and B agree.  The paddings (8, 4) put the two lane
// halves, and neighbouring row groups, on different LDS banks.
// Wave w of the block issues the loads of k = 4w..4w+3 (RowsLoader) or of rows R/4*w.. (KLoader).

template <int R, bool CHECK> struct RowsLoader {
    static constexpr int NCH = (R + 63) / 64;
    static constexpr int RS = NCH * 64 + 8;
    static constexpr int SZ = KT * RS;
    static constexpr int LPT = 4 * NCH;          // load instructions per tile and wave
    uint32_t roff[NCH];
    int32_t ra[NCH], rb[NCH];

    __device__ __forceinline__ void init(const Operand &op, uint32_t row0, uint32_t nrows, int, int lane)
    {
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const uint32_t rl = (uint32_t)(c * 64 + lane), row = row0 + rl;
            const Info q = map_info(op.row, row);
            roff[c] = (rl < (uint32_t)R && row < nrows) ? (uint32_t)q.off * 4u : OOB_ROW;
            ra[c] = q.a; rb[c] = q.b;
        }
    }
    // scalar info of the k this wave is loading (set by the part that issues chunk 0 of that k)
    Info kq;
    uint32_t ksoff;

    // The loads of one tile are cut into NPART parts so that the K loop can place one part behind
    // each MFMA step: part P issues loads [P*LPT/NPART, (P+1)*LPT/NPART), load i = (t, chunk).
    template <int P>
    __device__ __forceinline__ void issue_part(BufferRsrc rsrc, float *stage, const Operand &op, uint32_t k0,
                                               uint32_t kend, int wave, int)
    {
#pragma unroll
        for (int i = P * LPT / NPART; i < (P + 1) * LPT / NPART; ++i) {
            const int t = i / NCH, c = i % NCH;
            const uint32_t kl = (uint32_t)(4 * wave + t), k = k0 + kl;       // wave-uniform
            if (c == 0) {
                kq = map_info(op.k, k);
                ksoff = (k < kend && (op.k.r1_lim == 0 || kq.r1 < op.k.r1_lim)) ? (uint32_t)kq.off * 4u : OOB_K;
            }
            uint32_t voff = roff[c];
            if (CHECK) {
                const bool ok = (uint32_t)(ra[c] + kq.a) < op.limA && (uint32_t)(rb[c] + kq.b) < op.limB;
                voff = ok ? voff : OOB_ROW;
            }
            load_to_lds(rsrc, stage + kl * RS + c * 64, voff, ksoff);
        }
    }
    __device__ __forceinline__ static void frag(const float *stage, int row, int ks, int h, float out[4])
    {
#pragma unroll
        for (int t = 0; t < 4; ++t) out[t] = stage[(8 * ks + 4 * h + t) * RS + row];
    }
};

template <int R, bool CHECK> struct KLoader {
    static_assert(R % 16 == 0, "four waves, four rows per load");
    static constexpr int NI = R / 4;             // load instructions per tile
    static constexpr int NJ = NI / 4;            // ... and wave
    static constexpr int GS = 68;
    static constexpr int SZ = NI * GS;
    static constexpr int LPT = NJ;
    uint32_t roff[NJ];
    int32_t ra[NJ], rb[NJ];

    __device__ __forceinline__ void init(const Operand &op, uint32_t row0, uint32_t nrows, int wave, int lane)
    {
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            const uint32_t row = row0 + (uint32_t)(4 * (wave * NJ + j) + (lane >> 4));
            const Info q = map_info(op.row, row);
            roff[j] = row < nrows ? (uint32_t)q.off * 4u : OOB_ROW;
            ra[j] = q.a; rb[j] = q.b;
        }
    }
    Info kq;              // this lane's k of the tile being loaded (set by part 0)
    uint32_t koff;

    template <int P>
    __device__ __forceinline__ void issue_part(BufferRsrc rsrc, float *stage, const Operand &op, uint32_t k0,
                                               uint32_t kend, int wave, int lane)
    {
        if (P == 0) {
            const uint32_t k = k0 + (uint32_t)(lane & 15);
            kq = map_info(op.k, k);
            koff = (k < kend && (op.k.r1_lim == 0 || kq.r1 < op.k.r1_lim)) ? (uint32_t)kq.off * 4u : OOB_K;
        }
#pragma unroll
        for (int j = P * LPT / NPART; j < (P + 1) * LPT / NPART; ++j) {
            uint32_t voff = roff[j] + koff;
            if (CHECK) {
                const bool ok = (uint32_t)(ra[j] + kq.a) < op.limA && (uint32_t)(rb[j] + kq.b) < op.limB;
                voff = ok ? voff : OOB_ROW;
            }
            load_to_lds(rsrc, stage + (wave * NJ + j) * GS, voff);
        }
    }
    __device__ __forceinline__ static void frag(const float *stage, int row, int ks, int h, float out[4])
    {
        const float4 q = *reinterpret_cast<const float4 *>(stage + (row >> 2) * GS + (row & 3) * 16 + 8 * ks + 4 * h);
        out[0] = q.x; out[1] = q.y; out[2] = q.z; out[3] = q.w;
    }
};

// KLoader4: for an operand in which every aligned group of four reduction indices is four
// consecutive floats in memory (a row-major matrix; or runs of pixels, one run per image, the run
// length padded to a multiple of four in the index space).  One load moves 16 rows x 16 k: lane l
// fetches quad (l&3) ^ ((row>>2)&3) of row l>>2, so that the four quads of a row sit in its 64-byte
// LDS line in an order that spreads a fragment read of 16 rows over all banks.  Addresses need
// only 4-byte alignment, and the range check is per float: a quad that reaches beyond K, a run or
// the tensor delivers the floats that exist and zeros (or the neighbouring row's values) for the
// rest, which meet zeros of operand B.
template <int R, int WS = kShortWS> struct KLoader4 {       // WS: wait states behind the M0 set-up of a load (1 or 4)
    static constexpr int NJ = (R + 63) / 64;     // load instructions per tile and wave
    static constexpr int SZ = 4 * NJ * 256;      // rows beyond R are loaded as zeros
    static constexpr int LPT = NJ;
    uint32_t roff[NJ];
    uint32_t kq4;                                // first k of this lane's quad inside the tile
    uint32_t koff;                               // byte offset of that quad (set by part 0 of a tile)

    __device__ __forceinline__ void init(const Operand &op, uint32_t row0, uint32_t nrows, int wave, int lane)
    {
        const uint32_t r = (uint32_t)lane >> 2;
        kq4 = 4u * (((uint32_t)lane & 3u) ^ ((r >> 2) & 3u));
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            const uint32_t rl = (uint32_t)(16 * (wave * NJ + j)) + r, row = row0 + rl;
            const Info q = map_info(op.row, row);
            roff[j] = (rl < (uint32_t)R && row < nrows) ? (uint32_t)q.off * 4u : OOB_ROW;
        }
    }
    template <int P>
    __device__ __forceinline__ void issue_part(BufferRsrc rsrc, float *stage, const Operand &op, uint32_t k0,
                                               uint32_t kend, int wave, int)
    {
        if (P == 0) {
            const uint32_t k = k0 + kq4;
            // a plain matrix (wave-uniform test) needs no index arithmetic: its k is its offset
            const uint32_t off = op.k.d1.d == 1 ? k + (uint32_t)op.k.o0 : (uint32_t)map_info(op.k, k).off;
            koff = k < kend ? off * 4u : OOB_K;
        }
#pragma unroll
        for (int j = P * LPT / NPART; j < (P + 1) * LPT / NPART; ++j)
            load4_to_lds<WS>(rsrc, stage + (wave * NJ + j) * 256, roff[j] + koff);
    }
    __device__ __forceinline__ static void frag(const float *stage, int row, int ks, int h, float out[4])
    {
        const int unit = row * 4 + ((2 * ks + h) ^ ((row >> 2) & 3));
        const float4 q = *reinterpret_cast<const float4 *>(stage + unit * 4);
        out[0] = q.x; out[1] = q.y; out[2] = q.z; out[3] = q.w;
    }
};

// Buffer descriptor over the part of an operand's tensor that starts at group g (+ the shift that
// keeps per-index offsets non-negative).  igemm_launch has checked that the span fits the format.
// Words: base address (48 bits, stride 0), number of bytes, format word of a raw dword buffer.
__device__ __forceinline__ BufferRsrc operand_rsrc(const Operand &op, uint32_t g)
{
    const int64_t first = (int64_t)g * op.gstride + op.shift;
    const uint64_t base = (uint64_t)reinterpret_cast<uintptr_t>(op.ptr) + (uint64_t)(first * 4);
    const uint32_t bytes = (uint32_t)(((int64_t)op.elems - first) * 4);
    BufferRsrc r;       // wave-uniform by construction; readfirstlane pins the words to scalar registers
    r.x = __builtin_amdgcn_readfirstlane((uint32_t)base);
    r.y = __builtin_amdgcn_readfirstlane((uint32_t)(base >> 32) & 0xffffu);
    r.z = __builtin_amdgcn_readfirstlane(bytes);
    r.w = 0x00020000u;
    return r;
}

// Epilogue of the matrix kernels: a wave's TM x TN accumulator tiles, whose first row / column
// are (mw, nw), go to C (columns below n_end) with bias, rectifier, gate and accumulation applied.
// Accumulator register r of lane (h, li) holds C row 8*(r/4) + 4*h + r%4, column li of its 32x32
// sub-tile: stored from there, every store instruction would write 4 bytes per lane in runs of
// 128 bytes.  Instead each 32-row slab of the wave's tile is turned around in LDS (`wlds`, private
// to the wave, EpiLds<TN>::FLOATS floats, free once the block has left the K loop) so that a lane
// owns four consecutive columns of a row and a store instruction writes whole runs of 32*TN
// columns, 16 bytes per lane (4-byte aligned).  Columns whose C offsets are not consecutive
// (a pixel tile that crosses into the next image) or that reach beyond n_end go one by one.
typedef float f4u __attribute__((ext_vector_type(4), aligned(4)));

template <int TN> struct EpiLds {
    static constexpr int W = TN * 32, LS = W + 8, FLOATS = 32 * LS;
};

// PLAIN: no gate, no accumulation, no scattered rows (forward, ungated backward-data, K-slice partial
// planes): that instance has a third of the other's instructions, and a block's epilogue is time in
// which its waves issue no matrix instruction.
template <int TM, int TN, bool PLAIN>
__device__ __forceinline__ void store_tile_impl(const IgemmProblem &p, const v16f (&acc)[TM][TN], uint32_t g, uint32_t sp,
                                                uint32_t mw, uint32_t nw, uint32_t n_end, int lane, float *wlds)
{
    constexpr int LS = EpiLds<TN>::LS, QR = TN * 8, RPI = 64 / QR;      // quads per row, rows per instruction
    constexpr int NRG = 32 / RPI;                   // row groups (one store instruction each) of a 32-row slab
    constexpr int PB = TM >= 4 ? 2 : NRG < 4 ? NRG : 4;      // row groups per batch (fewer beside 128 accumulator registers)
    constexpr int NBS = NRG / PB, NBT = TM * NBS;   // batches per slab and of the whole tile
    const int h = lane >> 5, li = lane & 31, qd = lane % QR, rr = lane / QR;
    float *c_base = p.c_ptr + (int64_t)g * p.c_gstride + (int64_t)sp * p.c_split_stride;
    const float *bias = p.bias_mode ? p.bias + (int64_t)g * p.bias_gstride : nullptr;
    const float *gate = (!PLAIN && p.gate) ? p.gate + (int64_t)g * p.c_gstride : nullptr;
    const bool accumulate = !PLAIN && p.accumulate, scatter = !PLAIN && p.c_scatter;
    const uint32_t n = nw + 4u * (uint32_t)qd;
    int32_t off[4], ca[4], cb[4];
    float bcol[4];
    uint32_t okbits = 0u;       // bit e: column n + e exists (kept in a vector register: lane masks are scalar-register pairs)
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const bool ok = n + (uint32_t)e < n_end;
        const Info ci = map_info(p.c_col, ok ? n + (uint32_t)e : 0u);
        off[e] = ok ? ci.off : 0;
        ca[e] = ci.a; cb[e] = ci.b;
        bcol[e] = (p.bias_mode == 2 && ok) ? bias[n + (uint32_t)e] : 0.f;
        okbits |= ok ? 1u << e : 0u;
    }
    const bool quad = !scatter && (okbits & 8u) && off[1] == off[0] + 1 && off[2] == off[0] + 2 && off[3] == off[0] + 3;
    // Loads and stores leave the vector-memory counter in the order they were issued, so a load
    // issued behind stores is waited for together with them, a whole write latency.  Hence what a
    // batch of row groups reads from global memory (per-row bias, gate, C when accumulating) is
    // requested one batch ahead, before the stores of the batch in front of it: the wait for it
    // then leaves those stores outstanding.
    struct Batch {
        f4u gt[PB], old[PB];
        float brow[PB];
        int32_t roff[PB];
        uint32_t okm;           // bit 4u+e: element e of row group u is inside C (a vector register, not 16 lane masks)
    };
    Batch bt[2];
    auto prepare = [&](auto BC, Batch &t) {
        constexpr int b = decltype(BC)::value, i = b / NBS, p0 = (b % NBS) * PB;
#pragma unroll
        for (int u = 0; u < PB; ++u) {
            const int row = (p0 + u) * RPI + rr;
            const uint32_t m = mw + (uint32_t)(i * 32 + row);
            t.gt[u] = f4u{1.f, 1.f, 1.f, 1.f};
            t.old[u] = f4u{0.f, 0.f, 0.f, 0.f};
            t.roff[u] = (int32_t)m * p.c_row_stride;
            t.brow[u] = (p.bias_mode == 1 && m < p.M) ? bias[m] : 0.f;
            uint32_t bits = m < p.M ? okbits : 0u;
            if (scatter && m < p.M) {
                const Info ri = map_info(p.c_row, m);
                t.roff[u] = ri.off;
                bits = 0u;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    bits |= ((okbits >> e & 1u) && (uint32_t)(ri.a + ca[e]) < p.c_limA && (uint32_t)(ri.b + cb[e]) < p.c_limB) ? 1u << e : 0u;
            }
            if (u == 0) t.okm = 0u;
            t.okm |= bits << (4 * u);
            if (m < p.M && (gate || accumulate)) {
                const int32_t row_off = t.roff[u];
                if (quad) {
                    if (gate) t.gt[u] = *reinterpret_cast<const f4u *>(gate + row_off + off[0]);
                    if (accumulate) t.old[u] = *reinterpret_cast<const f4u *>(c_base + row_off + off[0]);
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        if (gate && (bits >> e & 1u)) t.gt[u][e] = gate[row_off + off[e]];
                        if (accumulate && (bits >> e & 1u)) t.old[u][e] = c_base[row_off + off[e]];
                    }
                }
            }
        }
    };
    prepare(std::integral_constant<int, 0>{}, bt[0]);
    static_for<0, NBT>([&](auto BC) {
        constexpr int b = decltype(BC)::value, i = b / NBS, p0 = (b % NBS) * PB;
        if constexpr (b % NBS == 0) {
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) wlds[((r >> 2) * 8 + h * 4 + (r & 3)) * LS + j * 32 + li] = acc[i][j][r];
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");       // the slab is in LDS (one wave: no barrier)
        }
        float4 q[PB];
#pragma unroll
        for (int u = 0; u < PB; ++u) q[u] = *reinterpret_cast<const float4 *>(wlds + ((p0 + u) * RPI + rr) * LS + 4 * qd);
        if constexpr (b + 1 < NBT) prepare(std::integral_constant<int, b + 1>{}, bt[(b + 1) & 1]);
        const Batch &t = bt[b & 1];
#pragma unroll
        for (int u = 0; u < PB; ++u) {
            const int row = (p0 + u) * RPI + rr;
            const uint32_t m = mw + (uint32_t)(i * 32 + row);
            if (m >= p.M || !(okbits & 1u)) continue;
            float val[4] = {q[u].x + bcol[0], q[u].y + bcol[1], q[u].z + bcol[2], q[u].w + bcol[3]};
            const float br = t.brow[u];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                val[e] += br;
                if (p.relu) val[e] = fmaxf(val[e], 0.f);
            }
            const int32_t row_off = t.roff[u];
            if constexpr (!PLAIN) {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (!(t.gt[u][e] > 0.f)) val[e] = 0.f;
            }
            f4u out = {val[0], val[1], val[2], val[3]};
            if (accumulate) out += t.old[u];
            if (quad) {
                *reinterpret_cast<f4u *>(c_base + row_off + off[0]) = out;
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (t.okm >> (4 * u + e) & 1u) c_base[row_off + off[e]] = out[e];
            }
        }
        if constexpr (b % NBS == NBS - 1)
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");       // slab read before the next one overwrites it
    });
}

template <int TM, int TN>
__device__ __forceinline__ void store_tile(const IgemmProblem &p, const v16f (&acc)[TM][TN], uint32_t g, uint32_t sp,
                                           uint32_t mw, uint32_t nw, uint32_t n_end, int lane, float *wlds)
{
    if (!p.gate && !p.accumulate && !p.c_scatter) store_tile_impl<TM, TN, true>(p, acc, g, sp, mw, nw, n_end, lane, wlds);
    else store_tile_impl<TM, TN, false>(p, acc, g, sp, mw, nw, n_end, lane, wlds);
}

}  // namespace

template <int WM, int WN, int TM, int TN, int NST, class LA, class LB, int MATH>
__global__ __launch_bounds__(256, 2) void igemm_kernel(const IgemmProblem p)
{
    static_assert(WM * WN == 4, "four waves");
    constexpr int MT = WM * TM * 32, NT = WN * TN * 32;
    constexpr int STAGE = LA::SZ + LB::SZ;
    constexpr int LPT = LA::LPT + LB::LPT;
    static_assert((NST - 1) * LPT <= 63, "the vector-memory counter holds 63 loads");

    extern __shared__ __attribute__((aligned(16))) float smem[];     // [NST][LA::SZ + LB::SZ]

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    const uint32_t m0 = blockIdx.y * MT, n0 = blockIdx.x * NT;
    const uint32_t g = blockIdx.z / p.splits, sp = blockIdx.z % p.splits;
    const uint32_t kbeg = sp * p.k_per_split;
    const uint32_t kend = min(p.K, kbeg + p.k_per_split);
    const int n_iter = (int)((kend - kbeg + KT - 1) / KT);

    const BufferRsrc rsrcA = operand_rsrc(p.A, g), rsrcB = operand_rsrc(p.B, g);
    LA la;
    LB lb;
    la.init(p.A, m0, p.M, wave, lane);
    lb.init(p.B, n0, p.N, wave, lane);

    // Tiles past the end of the K range are all padding: they cost no memory traffic and keep the
    // count of outstanding loads the same in every iteration.
    auto issue_part = [&](auto PC, int tile) {
        constexpr int P = decltype(PC)::value;
        float *st = smem + (tile % NST) * STAGE;
        const uint32_t k0 = kbeg + (uint32_t)tile * KT;
        la.template issue_part<P>(rsrcA, st, p.A, k0, kend, wave, lane);
        lb.template issue_part<P>(rsrcB, st + LA::SZ, p.B, k0, kend, wave, lane);
    };

    const int wm = wave / WN, wn = wave % WN;
    const int h = lane >> 5, li = lane & 31;
    v16f acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

#pragma unroll
    for (int d = 0; d < NST - 1; ++d) static_for<0, NPART>([&](auto PC) { issue_part(PC, d); });

    for (int it = 0; it < n_iter; ++it) {
        // This wave's loads of tile `it` have landed (all but the NST-2 newer tiles are complete);
        // behind the barrier that holds for every wave, and everyone is done reading tile it-1,
        // whose stage the loads issued below overwrite.
        asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"((NST - 2) * LPT) : "memory");
        const float *a_s = smem + (it % NST) * STAGE, *b_s = a_s + LA::SZ;
        if constexpr (MATH != 0) {
            // bf16 matrix instructions: all fragments of the tile, rounded (and split), one MFMA per
            // accumulator and product, then the next tile's loads
            float af[TM][KT / 8][4], bf[TN][KT / 8][4];
#pragma unroll
            for (int ks = 0; ks < KT / 8; ++ks) {
#pragma unroll
                for (int i = 0; i < TM; ++i) LA::frag(a_s, (wm * TM + i) * 32 + li, ks, h, af[i][ks]);
#pragma unroll
                for (int j = 0; j < TN; ++j) LB::frag(b_s, (wn * TN + j) * 32 + li, ks, h, bf[j][ks]);
            }
            bf16x8 ah[TM], al[TM], bh[TN], bl[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) to_bf16<MATH == 2>(af[i], ah[i], al[i]);
#pragma unroll
            for (int j = 0; j < TN; ++j) to_bf16<MATH == 2>(bf[j], bh[j], bl[j]);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    if constexpr (MATH == 2) {
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al[i], bh[j], acc[i][j], 0, 0, 0);
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[i], bl[j], acc[i][j], 0, 0, 0);
                    }
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[i], bh[j], acc[i][j], 0, 0, 0);
                }
            static_for<0, NPART>([&](auto PC) { issue_part(PC, it + NST - 1); });
            continue;
        }
        float af[KT / 8][TM][4], bf[KT / 8][TN][4];
        // the fragments of the tile's first eight k now, those of the second eight behind the first
        // MFMA step: half the reads are waited for at the start of a tile
#pragma unroll
        for (int i = 0; i < TM; ++i) LA::frag(a_s, (wm * TM + i) * 32 + li, 0, h, af[0][i]);
#pragma unroll
        for (int j = 0; j < TN; ++j) LB::frag(b_s, (wn * TN + j) * 32 + li, 0, h, bf[0][j]);
        __builtin_amdgcn_sched_barrier(0);
        // One part of the next tile's loads behind each MFMA step: the address pipeline and the
        // matrix pipeline both stay fed, instead of taking turns.
        static_for<0, NPART>([&](auto PC) {
            constexpr int P = decltype(PC)::value, ks = P / 4, s4 = P % 4;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[ks][i][s4], bf[ks][j][s4], acc[i][j], 0, 0, 0);
            if constexpr (P == 0) {
#pragma unroll
                for (int ks2 = 1; ks2 < KT / 8; ++ks2) {
#pragma unroll
                    for (int i = 0; i < TM; ++i) LA::frag(a_s, (wm * TM + i) * 32 + li, ks2, h, af[ks2][i]);
#pragma unroll
                    for (int j = 0; j < TN; ++j) LB::frag(b_s, (wn * TN + j) * 32 + li, ks2, h, bf[ks2][j]);
                }
            }
            issue_part(PC, it + NST - 1);
            __builtin_amdgcn_sched_barrier(0);
        });
    }
    // the padding tiles still in flight write into this block's LDS: let them finish before it is released
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();            // every wave has read its last fragments: the stages are free for the epilogue
    store_tile<TM, TN>(p, acc, g, sp, m0 + (uint32_t)(wm * TM * 32), n0 + (uint32_t)(wn * TN * 32), p.N, lane,
                       smem + wave * EpiLds<TN>::FLOATS);
}

// ---- patch kernel: convolutions whose B operand is staged as raw padded image rows ---------------
//
// The gathered im2col tile of the kernel above re-reads every input element once per filter tap
// (9 or 25 times), and the address pipeline, one load instruction per 64 elements, is what limits
// it.  Here a block keeps, for its 128 output pixels and 16 reduction channels at a time, the
// zero-padded source rows those pixels' windows touch ("patch", PatchGeom in cg_internal.h) in
// LDS, loaded once per channel block, and multiplies tap after tap from it: the B fragment of
// pixel p, tap t, channel c is  patch[c][sigma(p) + tapoff(t)],  sigma fixed per lane for the
// whole kernel and tapoff uniform per tap.  The reduction runs tap-major inside a channel block:
// K-tile number cb*KK + t holds tap t of channels 16cb..16cb+15, and operand A is the filter
// matrix permuted to [row][tap][channel], whose tiles the aligned-quad loader fetches.
//
// Pipeline: A tiles in a ring of NSTA stages as above.  The patch is double buffered; the loads
// of channel block cb+1 are issued during the first K-tile (t = 0) of channel block cb, part by
// part behind the MFMA steps and so interleaved with the loads of A tile t + NSTA-1.  The count a
// wave may leave outstanding at a tile's barrier is (NSTA-2) A tiles, plus the patch loads while
// the awaited A tile is older than all of them, t = 1..NSTA-2; from t = NSTA-1 on the wait covers
// the patch too, long before the next channel block starts (KK >= 5 > NSTA-1).

template <int NSL, int PAD = 8> struct PatchB {
    static constexpr int CS = NSL * 64 + PAD;        // LDS floats between channels (+8: lane halves on different banks)
    static constexpr int BUF = 16 * CS;              // one buffer: 16 channels
    static constexpr int NB = 4 * NSL;               // load instructions per wave and channel block
};

template <int WM, int WN, int TM, int TN, int NSTA, int NSL, int MATH>
__global__ __launch_bounds__(256, 2) void igemm_patch_kernel(const IgemmProblem p)
{
    static_assert(WM * WN == 4 && WN * TN == 4, "four waves, 128 pixels per block");
    constexpr int MT = WM * TM * 32, NT = 128;
    using LA = KLoader4<MT, 4>;
    using PB = PatchB<NSL>;
    constexpr int LAW = LA::LPT, NB = PB::NB;
    static_assert((NSTA - 1) * LAW + NB <= 63, "the vector-memory counter holds 63 loads");

    extern __shared__ __attribute__((aligned(16))) float smem[];     // [NSTA][LA::SZ] then [2][PB::BUF]
    float *const sB = smem + NSTA * LA::SZ;

    const PatchGeom &pg = p.patch;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t m0 = blockIdx.y * MT, g = blockIdx.z;
    const int KK = pg.KH * pg.KW, ncb = (int)(pg.Cred / 16), n_iter = ncb * KK;
    // this block's pixels n0..n1
    const uint32_t P = pg.divP.d;
    uint32_t n0, n1;
    const uint32_t tile = blockIdx.x + pg.tile0;
    if (pg.tiles_per_img) {
        const uint32_t b = fdiv(tile, pg.divTpi), ti = tile - b * pg.divTpi.d;
        n0 = b * P + ti * NT;
        n1 = min(n0 + NT - 1, (b + 1) * P - 1);
    } else {
        n0 = tile * NT;
        n1 = min(n0 + NT - 1, p.N - 1);
    }

    const BufferRsrc rsrcA = operand_rsrc(p.A, g);
    BufferRsrc rsrcB;
    {
        const uint64_t base = (uint64_t)reinterpret_cast<uintptr_t>(pg.src) + (uint64_t)((int64_t)g * pg.gstride * 4);
        rsrcB.x = __builtin_amdgcn_readfirstlane((uint32_t)base);
        rsrcB.y = __builtin_amdgcn_readfirstlane((uint32_t)(base >> 32) & 0xffffu);
        rsrcB.z = __builtin_amdgcn_readfirstlane((uint32_t)(((int64_t)pg.src_elems - (int64_t)g * pg.gstride) * 4));
        rsrcB.w = 0x00020000u;
    }
    LA la;
    la.init(p.A, m0, p.M, wave, lane);

    // ---- where this block's pixels sit: images bA..bB, pixel rows oyA (in bA) .. oyB (in bB) -------
    const uint32_t bA = fdiv(n0, pg.divP), oyA = fdiv(n0 - bA * P, pg.divOW);
    const uint32_t bB = fdiv(n1, pg.divP), oyB = fdiv(n1 - bB * P, pg.divOW);
    // slots of the first image's segment; later images start at R0 + (d-1)*Rfull
    const int32_t R0 = (int32_t)((((bA == bB) ? oyB : (uint32_t)pg.OHo - 1) - oyA) * pg.s + pg.KH) * pg.Wp;

    // global byte offset of every patch slot this lane loads (or out of range: padding, unused slots)
    uint32_t voff[NSL];
#pragma unroll
    for (int e = 0; e < NSL; ++e) {
        const int32_t j = e * 64 + lane;
        const uint32_t d = j < R0 ? 0u : 1u + fdiv((uint32_t)(j - R0), pg.divRfull);
        const int32_t local = j - (d == 0 ? 0 : R0 + (int32_t)(d - 1) * pg.Rfull);
        const uint32_t r = fdiv((uint32_t)local, pg.divWp), c = (uint32_t)local - r * (uint32_t)pg.Wp;
        const uint32_t b = bA + d, oylo = d == 0 ? oyA : 0u;
        const uint32_t oyhi = b == bB ? oyB : (uint32_t)pg.OHo - 1;
        const int32_t sy = (int32_t)(oylo * pg.s) + pg.oy0 + (int32_t)r, sx = pg.ox0 + (int32_t)c;
        const bool ok = b <= bB && r < (oyhi - oylo) * pg.s + pg.KH && (uint32_t)sy < (uint32_t)pg.Hs &&
                        (uint32_t)sx < (uint32_t)pg.Ws;
        voff[e] = ok ? (uint32_t)((int32_t)b * pg.img_stride + sy * pg.Ws + sx) * 4u : OOB_ROW;
    }

    const int wm = wave / WN, wn = wave % WN;
    const int h = lane >> 5, li = lane & 31;
    // sigma of this lane's pixels (floats into a patch buffer), with the lane half's channel offset folded in
    int32_t sig[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const uint32_t n = n0 + (uint32_t)((wn * TN + j) * 32 + li);
        int32_t sg = 0;
        if (n <= n1) {
            const uint32_t b = fdiv(n, pg.divP), rem = n - b * P, oy = fdiv(rem, pg.divOW), ox = rem - oy * pg.divOW.d;
            const uint32_t d = b - bA, oylo = d == 0 ? oyA : 0u;
            sg = (d == 0 ? 0 : R0 + (int32_t)(d - 1) * pg.Rfull) + (int32_t)((oy - oylo) * pg.s) * pg.Wp + (int32_t)(ox * pg.s);
        }
        sig[j] = sg + 4 * h * PB::CS;
    }

    v16f acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // part P of the patch loads of channel block cb: load q = (channel wave + 4*(q/NSL), chunk q%NSL)
    auto issue_patch_part = [&](auto PC, int cb) {
        constexpr int Pn = decltype(PC)::value;
        float *buf = sB + (cb & 1) * PB::BUF;
#pragma unroll
        for (int q = Pn * NB / NPART; q < (Pn + 1) * NB / NPART; ++q) {
            const int cl = wave + 4 * (q / NSL), e = q % NSL;
            load_to_lds(rsrcB, buf + cl * PB::CS + e * 64, voff[e], (uint32_t)((cb * 16 + cl) * pg.chan_stride) * 4u);
        }
    };
    // part P of the A loads of K-tile `tile` = (cb, t); tiles past the end are all padding
    auto issue_a_part = [&](auto PC, int tile, int cb, int t) {
        constexpr int Pn = decltype(PC)::value;
        const uint32_t k0 = (uint32_t)t * pg.Cred + (uint32_t)cb * 16u;
        la.template issue_part<Pn>(rsrcA, smem + (tile % NSTA) * LA::SZ, p.A, k0, tile < n_iter ? p.K : 0u, wave, lane);
    };

    // prologue: the first patch, then A tiles 0..NSTA-2
    static_for<0, NPART>([&](auto PC) { issue_patch_part(PC, 0); });
    int icb = 0, it_ = 0;                       // (cb, t) of the next A tile to issue
    auto advance_issue = [&]() { if (++it_ == KK) { it_ = 0; ++icb; } };
#pragma unroll
    for (int d = 0; d < NSTA - 1; ++d) {
        static_for<0, NPART>([&](auto PC) { issue_a_part(PC, d, icb, it_); });
        advance_issue();
    }

    int ccb = 0, ct = 0, cky = 0, ckx = 0;      // (cb, t = cky*KW + ckx) of the tile being multiplied
    for (int it = 0; it < n_iter; ++it) {
        const bool burst = ccb + 1 < ncb;       // this channel block issues the next one's patch in its tile 0
        if (burst && ct >= 1 && ct <= NSTA - 2)
            asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"((NSTA - 2) * LAW + NB) : "memory");
        else
            asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"((NSTA - 2) * LAW) : "memory");
        const float *a_s = smem + (it % NSTA) * LA::SZ;
        const int py = pg.flip ? pg.KH - 1 - cky : cky, px = pg.flip ? pg.KW - 1 - ckx : ckx;
        const float *b_s = sB + (ccb & 1) * PB::BUF + (py * pg.Wp + px);
        if constexpr (MATH != 0) {
            float af[TM][KT / 8][4], bf[TN][KT / 8][4];
#pragma unroll
            for (int ks = 0; ks < KT / 8; ++ks) {
#pragma unroll
                for (int i = 0; i < TM; ++i) LA::frag(a_s, (wm * TM + i) * 32 + li, ks, h, af[i][ks]);
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int t = 0; t < 4; ++t) bf[j][ks][t] = b_s[sig[j] + (8 * ks + t) * PB::CS];
            }
            bf16x8 ah[TM], al[TM], bh[TN], bl[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) to_bf16<MATH == 2>(af[i], ah[i], al[i]);
#pragma unroll
            for (int j = 0; j < TN; ++j) to_bf16<MATH == 2>(bf[j], bh[j], bl[j]);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    if constexpr (MATH == 2) {
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al[i], bh[j], acc[i][j], 0, 0, 0);
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[i], bl[j], acc[i][j], 0, 0, 0);
                    }
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[i], bh[j], acc[i][j], 0, 0, 0);
                }
            const bool do_patch_b = burst && ct == 0;
            static_for<0, NPART>([&](auto PC) {
                issue_a_part(PC, it + NSTA - 1, icb, it_);
                if (do_patch_b) issue_patch_part(PC, ccb + 1);
            });
            advance_issue();
            if (++ckx == pg.KW) { ckx = 0; ++cky; }
            if (++ct == KK) { ct = 0; cky = 0; ++ccb; }
            continue;
        }
        float af[KT / 8][TM][4], bf[KT / 8][TN][4];
        // Fragments are read one MFMA step ahead (A once per eight k, B per step): only the first step's
        // reads are waited for at the start of a tile, the others arrive while the matrix pipeline works.
#pragma unroll
        for (int i = 0; i < TM; ++i) LA::frag(a_s, (wm * TM + i) * 32 + li, 0, h, af[0][i]);
#pragma unroll
        for (int j = 0; j < TN; ++j) bf[0][j][0] = b_s[sig[j]];
        __builtin_amdgcn_sched_barrier(0);
        const bool do_patch = burst && ct == 0;
        static_for<0, NPART>([&](auto PC) {
            constexpr int Pn = decltype(PC)::value, ks = Pn / 4, s4 = Pn % 4;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[ks][i][s4], bf[ks][j][s4], acc[i][j], 0, 0, 0);
            if constexpr (Pn + 1 < NPART) {
                constexpr int nks = (Pn + 1) / 4, nt = (Pn + 1) % 4;
                if constexpr (nt == 0) {
#pragma unroll
                    for (int i = 0; i < TM; ++i) LA::frag(a_s, (wm * TM + i) * 32 + li, nks, h, af[nks][i]);
                }
#pragma unroll
                for (int j = 0; j < TN; ++j) bf[nks][j][nt] = b_s[sig[j] + (8 * nks + nt) * PB::CS];
            }
            issue_a_part(PC, it + NSTA - 1, icb, it_);
            if (do_patch) issue_patch_part(PC, ccb + 1);
            __builtin_amdgcn_sched_barrier(0);
        });
        advance_issue();
        if (++ckx == pg.KW) { ckx = 0; ++cky; }
        if (++ct == KK) { ct = 0; cky = 0; ++ccb; }
    }
    // the padding tiles still in flight write into this block's LDS: let them finish before it is released
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();            // every wave has read its last fragments: the stages are free for the epilogue
    store_tile<TM, TN>(p, acc, g, 0u, m0 + (uint32_t)(wm * TM * 32), n0 + (uint32_t)(wn * TN * 32), n1 + 1, lane,
                       smem + wave * EpiLds<TN>::FLOATS);
}

#if CG_MATH == 0
// ---- patch kernel for at most 48 rows ------------------------------------------------------------
//
// The same data movement as igemm_patch_kernel, multiplied with v_mfma_f32_16x16x4_f32: a block
// owns 16*TM rows (TM <= 3) x 128 pixels, each of its four waves all the rows and 32 pixels.  A
// group of 48 channels (backward-data of a 5x5 layer whose groups have 48 input channels) then
// fills its tile, where the 32x32 tiles above would multiply 64 rows for 48.
// Lane (q = lane / 16, l = lane % 16) supplies A[row l][k = 4q + t] and B[k = 4q + t][pixel l] in
// step t = 0..3 of a K-tile and holds C[row 4q + r][pixel l], r = 0..3, of each 16x16 sub-tile.
// The patch buffers put channels NSL*64 + 4 floats apart, so that the four k of a step fall on
// different quarters of the banks.
typedef float v4f __attribute__((ext_vector_type(4)));

template <int TM, int NSTA, int NSL>
__global__ __launch_bounds__(256, 3) void igemm_patch16_kernel(const IgemmProblem p)
{
    constexpr int MT = TM * 16, NT = 128, TN = 2;
    using LA = KLoader4<MT, 4>;
    using PB = PatchB<NSL, 4>;
    constexpr int LAW = LA::LPT, NB = PB::NB;
    static_assert(TM >= 1 && TM <= 3 && LA::NJ == 1, "at most 48 rows: one A load per wave and K-tile");
    static_assert((NSTA - 1) * LAW + NB <= 63, "the vector-memory counter holds 63 loads");

    extern __shared__ __attribute__((aligned(16))) float smem[];     // [NSTA][LA::SZ] then [2][PB::BUF]
    float *const sB = smem + NSTA * LA::SZ;

    const PatchGeom &pg = p.patch;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t m0 = blockIdx.y * MT, g = blockIdx.z;
    const int KK = pg.KH * pg.KW, ncb = (int)(pg.Cred / 16), n_iter = ncb * KK;
    const uint32_t P = pg.divP.d;
    uint32_t n0, n1;
    const uint32_t tile = blockIdx.x + pg.tile0;
    if (pg.tiles_per_img) {
        const uint32_t b = fdiv(tile, pg.divTpi), ti = tile - b * pg.divTpi.d;
        n0 = b * P + ti * NT;
        n1 = min(n0 + NT - 1, (b + 1) * P - 1);
    } else {
        n0 = tile * NT;
        n1 = min(n0 + NT - 1, p.N - 1);
    }

    const BufferRsrc rsrcA = operand_rsrc(p.A, g);
    BufferRsrc rsrcB;
    {
        const uint64_t base = (uint64_t)reinterpret_cast<uintptr_t>(pg.src) + (uint64_t)((int64_t)g * pg.gstride * 4);
        rsrcB.x = __builtin_amdgcn_readfirstlane((uint32_t)base);
        rsrcB.y = __builtin_amdgcn_readfirstlane((uint32_t)(base >> 32) & 0xffffu);
        rsrcB.z = __builtin_amdgcn_readfirstlane((uint32_t)(((int64_t)pg.src_elems - (int64_t)g * pg.gstride) * 4));
        rsrcB.w = 0x00020000u;
    }
    LA la;
    la.init(p.A, m0, p.M, wave, lane);

    // where this block's pixels sit (as in igemm_patch_kernel)
    const uint32_t bA = fdiv(n0, pg.divP), oyA = fdiv(n0 - bA * P, pg.divOW);
    const uint32_t bB = fdiv(n1, pg.divP), oyB = fdiv(n1 - bB * P, pg.divOW);
    const int32_t R0 = (int32_t)((((bA == bB) ? oyB : (uint32_t)pg.OHo - 1) - oyA) * pg.s + pg.KH) * pg.Wp;
    uint32_t voff[NSL];
#pragma unroll
    for (int e = 0; e < NSL; ++e) {
        const int32_t j = e * 64 + lane;
        const uint32_t d = j < R0 ? 0u : 1u + fdiv((uint32_t)(j - R0), pg.divRfull);
        const int32_t local = j - (d == 0 ? 0 : R0 + (int32_t)(d - 1) * pg.Rfull);
        const uint32_t r = fdiv((uint32_t)local, pg.divWp), c = (uint32_t)local - r * (uint32_t)pg.Wp;
        const uint32_t b = bA + d, oylo = d == 0 ? oyA : 0u;
        const uint32_t oyhi = b == bB ? oyB : (uint32_t)pg.OHo - 1;
        const int32_t sy = (int32_t)(oylo * pg.s) + pg.oy0 + (int32_t)r, sx = pg.ox0 + (int32_t)c;
        const bool ok = b <= bB && r < (oyhi - oylo) * pg.s + pg.KH && (uint32_t)sy < (uint32_t)pg.Hs &&
                        (uint32_t)sx < (uint32_t)pg.Ws;
        voff[e] = ok ? (uint32_t)((int32_t)b * pg.img_stride + sy * pg.Ws + sx) * 4u : OOB_ROW;
    }

    const int q = lane >> 4, l16 = lane & 15;
    int32_t sig[TN];                 // this lane's pixels in a patch buffer, with its k group's channel offset folded in
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const uint32_t n = n0 + (uint32_t)((wave * TN + j) * 16 + l16);
        int32_t sg = 0;
        if (n <= n1) {
            const uint32_t b = fdiv(n, pg.divP), rem = n - b * P, oy = fdiv(rem, pg.divOW), ox = rem - oy * pg.divOW.d;
            const uint32_t d = b - bA, oylo = d == 0 ? oyA : 0u;
            sg = (d == 0 ? 0 : R0 + (int32_t)(d - 1) * pg.Rfull) + (int32_t)((oy - oylo) * pg.s) * pg.Wp + (int32_t)(ox * pg.s);
        }
        sig[j] = sg + 4 * q * PB::CS;
    }

    v4f acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.f;

    auto issue_patch_part = [&](auto PC, int cb) {
        constexpr int Pn = decltype(PC)::value;
        float *buf = sB + (cb & 1) * PB::BUF;
#pragma unroll
        for (int qq = Pn * NB / NPART; qq < (Pn + 1) * NB / NPART; ++qq) {
            const int cl = wave + 4 * (qq / NSL), e = qq % NSL;
            load_to_lds(rsrcB, buf + cl * PB::CS + e * 64, voff[e], (uint32_t)((cb * 16 + cl) * pg.chan_stride) * 4u);
        }
    };
    auto issue_a_part = [&](auto PC, int tile, int cb, int t) {
        constexpr int Pn = decltype(PC)::value;
        const uint32_t k0 = (uint32_t)t * pg.Cred + (uint32_t)cb * 16u;
        la.template issue_part<Pn>(rsrcA, smem + (tile % NSTA) * LA::SZ, p.A, k0, tile < n_iter ? p.K : 0u, wave, lane);
    };

    static_for<0, NPART>([&](auto PC) { issue_patch_part(PC, 0); });
    int icb = 0, it_ = 0;
    auto advance_issue = [&]() { if (++it_ == KK) { it_ = 0; ++icb; } };
#pragma unroll
    for (int d = 0; d < NSTA - 1; ++d) {
        static_for<0, NPART>([&](auto PC) { issue_a_part(PC, d, icb, it_); });
        advance_issue();
    }

    int ccb = 0, ct = 0, cky = 0, ckx = 0;
    for (int it = 0; it < n_iter; ++it) {
        const bool burst = ccb + 1 < ncb;
        if (burst && ct >= 1 && ct <= NSTA - 2)
            asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"((NSTA - 2) * LAW + NB) : "memory");
        else
            asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"((NSTA - 2) * LAW) : "memory");
        const float *a_s = smem + (it % NSTA) * LA::SZ;
        const int py = pg.flip ? pg.KH - 1 - cky : cky, px = pg.flip ? pg.KW - 1 - ckx : ckx;
        const float *b_s = sB + (ccb & 1) * PB::BUF + (py * pg.Wp + px);
        float af[TM][4], bf[TN][4];
#pragma unroll
        for (int i = 0; i < TM; ++i) LA::frag(a_s, i * 16 + l16, q >> 1, q & 1, af[i]);      // the quad k = 4q .. 4q+3
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int t = 0; t < 4; ++t) bf[j][t] = b_s[sig[j] + t * PB::CS];
        const bool do_patch = burst && ct == 0;
        static_for<0, NPART>([&](auto PC) {
            constexpr int Pn = decltype(PC)::value, t = Pn / 2, j = Pn % 2;
#pragma unroll
            for (int i = 0; i < TM; ++i)
                acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(af[i][t], bf[j][t], acc[i][j], 0, 0, 0);
            issue_a_part(PC, it + NSTA - 1, icb, it_);
            if (do_patch) issue_patch_part(PC, ccb + 1);
            __builtin_amdgcn_sched_barrier(0);
        });
        advance_issue();
        if (++ckx == pg.KW) { ckx = 0; ++cky; }
        if (++ct == KK) { ct = 0; cky = 0; ++ccb; }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

    // epilogue: rectifier, gate and accumulation as in store_tile (this kernel is launched without
    // split-K; bias modes as there)
    float *c_base = p.c_ptr + (int64_t)g * p.c_gstride;
    const float *bias = p.bias_mode ? p.bias + (int64_t)g * p.bias_gstride : nullptr;
    const float *gate = p.gate ? p.gate + (int64_t)g * p.c_gstride : nullptr;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const uint32_t n = n0 + (uint32_t)((wave * TN + j) * 16 + l16);
        if (n > n1) continue;
        const Info ci = map_info(p.c_col, n);
        const int32_t coff = ci.off;
        const float bcol = p.bias_mode == 2 ? bias[n] : 0.f;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const uint32_t m = m0 + (uint32_t)(i * 16 + q * 4 + r);
                if (m < p.M) {
                    int32_t idx = (int32_t)m * p.c_row_stride + coff;
                    if (p.c_scatter) {
                        const Info ri = map_info(p.c_row, m);
                        if (!((uint32_t)(ri.a + ci.a) < p.c_limA && (uint32_t)(ri.b + ci.b) < p.c_limB)) continue;
                        idx = ri.off + coff;
                    }
                    float val = acc[i][j][r] + bcol;
                    if (p.bias_mode == 1) val += bias[m];
                    if (p.relu) val = fmaxf(val, 0.f);
                    if (gate && !(gate[idx] > 0.f)) val = 0.f;
                    float *dst = c_base + idx;
                    if (p.accumulate) val += *dst;
                    *dst = val;
                }
            }
        }
    }
}

// ---- band kernel: backward-weight with the input staged as raw padded rows ------------------------
//
//   dw[m][(c,kh,kw)] = sum over pixels (n,oh,ow) of dy[n][m][oh][ow] * x[n][c][oh*s-p+kh][ow*s-p+kw]
//
// The gathered kernel fetches x once per filter tap and column tile.  Here the reduction walks
// "units" = (image, band of output rows); for a unit a block keeps the zero-padded source rows of
// the CPB input channels its 128 columns (c,kh,kw) belong to in LDS (loaded once per unit), and
// the B fragment of column (c,kh,kw) at pixel (r,ow) of the band is
//   patch[c - c0][ (r*s + kh)*Wp + ow*s + kw ] = patch[colbase(lane) + sigma(pixel)],
// colbase fixed per lane for the whole kernel, sigma computed per K-tile for the eight pixels a
// lane half multiplies.  dy arrives in K-tiles of 16 consecutive pixels of the band (aligned quads;
// what a quad reads beyond the band's last pixel meets B values forced to zero).  Pipeline and
// waits as in the patch kernel above: A ring of NSTA stages, the patch double buffered, the next
// unit's patch loads issued during the current unit's first K-tile (a unit has >= 5 K-tiles).

template <int WM, int WN, int TM, int TN, int NSTA, int CPB, int NSL>
__global__ __launch_bounds__(256, 2) void igemm_wgrad_kernel(const IgemmProblem p)
{
    static_assert(WM * WN == 4 && WN * TN == 4, "four waves, 128 columns per block");
    static_assert(CPB % 4 == 0, "whole channels per wave");
    constexpr int MT = WM * TM * 32, NT = 128;
    using LA = KLoader4<MT, 4>;
    constexpr int LAW = LA::LPT;
    constexpr int CS = NSL * 64 + 1;            // odd: the channels of one tap fall on different banks
    constexpr int BUF = CPB * CS;
    constexpr int NB = CPB / 4 * NSL;           // patch load instructions per wave and unit
    static_assert((NSTA - 1) * LAW + NB <= 63, "the vector-memory counter holds 63 loads");

    extern __shared__ __attribute__((aligned(16))) float smem[];     // [NSTA][LA::SZ] then [2][BUF]
    float *const sB = smem + NSTA * LA::SZ;

    const WgradGeom &wg = p.wgrad;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t m0 = blockIdx.y * MT, n0 = blockIdx.x * NT;
    const uint32_t g = blockIdx.z / p.splits, sp = blockIdx.z % p.splits;
    const int KK = wg.KH * wg.KW, P = wg.OH * wg.OW, HW = wg.H * wg.W;
    const int u0 = (int)sp * wg.units_per_split, u1 = min(wg.units, u0 + wg.units_per_split);

    const BufferRsrc rsrcA = operand_rsrc(p.A, g);
    BufferRsrc rsrcX;
    {
        const int64_t first = (int64_t)g * wg.Cg * HW;
        const uint64_t base = (uint64_t)reinterpret_cast<uintptr_t>(wg.x) + (uint64_t)(first * 4);
        rsrcX.x = __builtin_amdgcn_readfirstlane((uint32_t)base);
        rsrcX.y = __builtin_amdgcn_readfirstlane((uint32_t)(base >> 32) & 0xffffu);
        rsrcX.z = __builtin_amdgcn_readfirstlane((uint32_t)(((int64_t)wg.x_elems - first) * 4));
        rsrcX.w = 0x00020000u;
    }
    LA la;
    la.init(p.A, m0, p.M, wave, lane);

    const int wm = wave / WN, wn = wave % WN;
    const int h = lane >> 5, li = lane & 31;
    const uint32_t c0 = fdiv(n0, wg.divKK);                  // first input channel of this block's columns
    int32_t colbase[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const uint32_t n = n0 + (uint32_t)((wn * TN + j) * 32 + li);
        int32_t cb = 0;
        if (n < p.N) {
            const uint32_t c = fdiv(n, wg.divKK), tap = n - c * (uint32_t)KK;
            const uint32_t kh = fdiv(tap, wg.divKW), kw = tap - kh * (uint32_t)wg.KW;
            cb = (int32_t)(c - c0) * CS + (int32_t)kh * wg.Wp + (int32_t)kw;
        }
        colbase[j] = cb;
    }

    // a unit's band: first output row, number of output rows, pixels, K-tiles
    auto band_of = [&](int u, int &img, int &oy0, int &rows) {
        img = u / wg.nb;
        const int jb = u - img * wg.nb;
        oy0 = jb * wg.Rb;
        rows = min(wg.Rb, wg.OH - oy0);
    };
    int n_iter = 0;
    for (int u = u0; u < u1; ++u) {
        int img, oy0, rows;
        band_of(u, img, oy0, rows);
        n_iter += (rows * wg.OW + KT - 1) / KT;
    }

    v16f acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // ---- patch loads of unit u (a burst, issued in NPART parts) -----------------------------------
    uint32_t pvoff[NSL];
    auto patch_offsets = [&](int u) {          // global byte offset of every slot this lane loads, or out of range
        int img, oy0, rows;
        band_of(u, img, oy0, rows);
        const int prow = (rows - 1) * wg.s + wg.KH, sy0 = oy0 * wg.s - wg.pad_h;
#pragma unroll
        for (int e = 0; e < NSL; ++e) {
            const uint32_t jslot = (uint32_t)(e * 64 + lane);
            const uint32_t r = fdiv(jslot, wg.divWp), cc = jslot - r * (uint32_t)wg.Wp;
            const int sy = sy0 + (int)r, sx = (int)cc - wg.pad_w;
            const bool ok = (int)r < prow && (uint32_t)sy < (uint32_t)wg.H && (uint32_t)sx < (uint32_t)wg.W;
            pvoff[e] = ok ? (uint32_t)(sy * wg.W + sx) * 4u : OOB_ROW;
        }
    };
    auto issue_patch_part = [&](auto PC, int u) {
        constexpr int Pn = decltype(PC)::value;
        if (Pn == 0) patch_offsets(u);
        const int img = u / wg.nb;
        float *buf = sB + (u & 1) * BUF;
#pragma unroll
        for (int q = Pn * NB / NPART; q < (Pn + 1) * NB / NPART; ++q) {
            const int cl = wave + 4 * (q / NSL), e = q % NSL;
            const uint32_t c = c0 + (uint32_t)cl;
            const uint32_t soff = c < (uint32_t)wg.Cg ? (uint32_t)((img * wg.C + (int)c) * HW) * 4u : OOB_K;
            load_to_lds(rsrcX, buf + cl * CS + e * 64, pvoff[e], soff);
        }
    };
    // ---- A loads of the K-tile t of unit u: 16 consecutive pixels of dy ---------------------------
    auto issue_a_part = [&](auto PC, int tile, int u, int t) {
        constexpr int Pn = decltype(PC)::value;
        if (Pn == 0) {
            int img, oy0, rows;
            band_of(u, img, oy0, rows);
            const uint32_t k = (uint32_t)(oy0 * wg.OW + t * KT) + la.kq4;            // pixel of this lane's quad in its image
            la.koff = tile < n_iter ? ((uint32_t)(img * wg.M) * (uint32_t)P + k) * 4u : OOB_K;
        }
#pragma unroll
        for (int j = Pn * LAW / NPART; j < (Pn + 1) * LAW / NPART; ++j)
            load4_to_lds<4>(rsrcA, smem + (tile % NSTA) * LA::SZ + (wave * LA::NJ + j) * 256, la.roff[j] + la.koff);
    };
    auto tiles_of = [&](int u) {
        int img, oy0, rows;
        band_of(u, img, oy0, rows);
        return (rows * wg.OW + KT - 1) / KT;
    };

    // prologue: the first unit's patch, then A tiles 0..NSTA-2
    static_for<0, NPART>([&](auto PC) { issue_patch_part(PC, u0); });
    int iu = u0, it_ = 0, itiles = tiles_of(u0);        // (unit, tile) of the next A tile to issue
    auto advance_issue = [&]() {
        if (++it_ == itiles) { it_ = 0; ++iu; itiles = iu < u1 ? tiles_of(iu) : 1 << 30; }
    };
#pragma unroll
    for (int d = 0; d < NSTA - 1; ++d) {
        static_for<0, NPART>([&](auto PC) { issue_a_part(PC, d, iu, it_); });
        advance_issue();
    }

    int cu = u0, ct = 0, ctiles = tiles_of(u0);         // (unit, tile) being multiplied
    for (int it = 0; it < n_iter; ++it) {
        const bool burst = cu + 1 < u1;                 // this unit issues the next one's patch in its tile 0
        if (burst && ct >= 1 && ct <= NSTA - 2)
            asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"((NSTA - 2) * LAW + NB) : "memory");
        else
            asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"((NSTA - 2) * LAW) : "memory");
        const float *a_s = smem + (it % NSTA) * LA::SZ;
        const float *b_s = sB + (cu & 1) * BUF;
        int img, oy0, rows;
        band_of(cu, img, oy0, rows);
        const int npix = rows * wg.OW;
        float af[KT / 8][TM][4], bf[KT / 8][TN][4];
#pragma unroll
        for (int ks = 0; ks < KT / 8; ++ks) {
#pragma unroll
            for (int i = 0; i < TM; ++i) LA::frag(a_s, (wm * TM + i) * 32 + li, ks, h, af[ks][i]);
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int pix = ct * KT + 8 * ks + 4 * h + t;
                const uint32_t r = fdiv((uint32_t)pix, wg.divOW), ox = (uint32_t)pix - r * (uint32_t)wg.OW;
                const int sg = (int)(r * (uint32_t)wg.s) * wg.Wp + (int)(ox * (uint32_t)wg.s);
                const bool live = pix < npix;
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const float vv = b_s[live ? colbase[j] + sg : 0];
                    bf[ks][j][t] = live ? vv : 0.f;
                }
            }
        }
        const bool do_patch = burst && ct == 0;
        static_for<0, NPART>([&](auto PC) {
            constexpr int Pn = decltype(PC)::value, ks = Pn / 4, s4 = Pn % 4;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[ks][i][s4], bf[ks][j][s4], acc[i][j], 0, 0, 0);
            issue_a_part(PC, it + NSTA - 1, iu, it_);
            if (do_patch) issue_patch_part(PC, cu + 1);
            __builtin_amdgcn_sched_barrier(0);
        });
        advance_issue();
        if (++ct == ctiles) { ct = 0; ++cu; ctiles = cu < u1 ? tiles_of(cu) : 1 << 30; }
    }
    // the padding tiles still in flight write into this block's LDS: let them finish before it is released
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();            // every wave has read its last fragments: the stages are free for the epilogue
    store_tile<TM, TN>(p, acc, g, sp, m0 + (uint32_t)(wm * TM * 32), n0 + (uint32_t)(wn * TN * 32), p.N, lane,
                       smem + wave * EpiLds<TN>::FLOATS);
}

#endif  // CG_MATH == 0

namespace {

template <int WM, int WN, int TM, int TN, int NST, class LA, class LB>
int launch_cfg(const IgemmProblem &p, const char *modes, hipStream_t stream)
{
    constexpr int MT = WM * TM * 32, NT = WN * TN * 32;
    dim3 grid((p.N + NT - 1) / NT, (p.M + MT - 1) / MT, p.groups * p.splits);
    if (grid.y > 65535u || grid.z > 65535u) return CG_EUNSUPPORTED;
    int rec = -1;
    if (prof_on()) {
        char name[64];
        snprintf(name, sizeof name, CG_MATH == 0 ? "igemm_kernel<%dx%d,%s>" : CG_MATH == 1 ? "igemm_kernel<%dx%d,%s,bf16>" : "igemm_kernel<%dx%d,%s,bf16x3>", MT, NT, modes);
        rec = prof_begin(name, p.flops > 0 ? p.flops : 2.0 * p.M * (double)p.N * p.K * p.groups, 0.0, stream);
    }
    constexpr size_t lds = (size_t)NST * (LA::SZ + LB::SZ) * sizeof(float);
    static_assert(lds >= 4 * EpiLds<TN>::FLOATS * sizeof(float), "the epilogue turns the tile around in the stages' LDS");
    static_assert(2 * lds <= 160 * 1024, "two blocks of this tile do not fit the LDS of a compute unit");
    static std::atomic<bool> attr_set{false};      // raising the dynamic-LDS limit: once per kernel (repeating it is harmless)
    if (!attr_set.load(std::memory_order_acquire)) {
        CG_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(&igemm_kernel<WM, WN, TM, TN, NST, LA, LB, CG_MATH>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        attr_set.store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL((igemm_kernel<WM, WN, TM, TN, NST, LA, LB, CG_MATH>), grid, dim3(256), lds, stream, p);
    prof_end(rec, stream);
    CG_HIP_TRY(hipGetLastError());
    return CG_OK;
}

// How an operand's tile is fetched: rows along the lanes, k along the lanes, or aligned quads of k.
enum { LD_ROWS = 0, LD_K = 1, LD_K4 = 2 };
template <int MODE, int R, bool CHECK>
using LoaderOf = std::conditional_t<MODE == LD_K4, KLoader4<R>,
                                    std::conditional_t<MODE == LD_K, KLoader<R, CHECK>, RowsLoader<R, CHECK>>>;

template <int AM, int BM, bool BC>
int launch_modes(const IgemmProblem &p, int mt, hipStream_t stream)
{
    static const char modes[4] = {"rk4"[AM], "rk4"[BM], BC ? 'c' : '-', 0};
    switch (mt) {
    case 256: return launch_cfg<2, 2, 4, 2, 3, LoaderOf<AM, 256, false>, LoaderOf<BM, 128, BC>>(p, modes, stream);
    case 192: return launch_cfg<2, 2, 3, 2, 3, LoaderOf<AM, 192, false>, LoaderOf<BM, 128, BC>>(p, modes, stream);
    case 128: return launch_cfg<2, 2, 2, 2, 4, LoaderOf<AM, 128, false>, LoaderOf<BM, 128, BC>>(p, modes, stream);
    case 96: return launch_cfg<1, 4, 3, 1, 4, LoaderOf<AM, 96, false>, LoaderOf<BM, 128, BC>>(p, modes, stream);
    case 64: return launch_cfg<1, 4, 2, 1, 4, LoaderOf<AM, 64, false>, LoaderOf<BM, 128, BC>>(p, modes, stream);
    default: return launch_cfg<1, 4, 1, 1, 4, LoaderOf<AM, 32, false>, LoaderOf<BM, 128, BC>>(p, modes, stream);
    }
}

// every aligned group of four reduction indices is four consecutive floats: k is unit-stride, either
// throughout or inside runs whose padded length is a multiple of four
bool quad_ok(const Operand &o, uint32_t)
{
    if (!o.lanes_k || o.check) return false;
    const bool linear = o.k.d1.d == 1 && o.k.d2.d == 1 && o.k.s1 == 1;
    const bool runs = o.k.d1.d % 4 == 0 && o.k.d2.d == 1 && o.k.s2 == 1;
    return linear || runs;
}

// Row-tile height for a problem.  A taller tile gathers the B operand (the costly one: one load
// instruction per 64 elements) fewer times, but leaves fewer blocks to spread over the 256 compute
// units, two resident per unit.  The cost model is the number of blocks the busiest unit runs (an
// odd one out runs alone and a little slower than a pair) times a block's duration, rows + a fixed
// per-block part; problems with few tiles are cut along K afterwards, which fills the chip for any
// tile height, so there only the per-block efficiency counts.
int pick_mt(uint32_t M, uint32_t N, uint32_t groups, uint32_t K = 0)
{
    const int cand[6] = {256, 192, 128, 96, 64, 32};
    int best = 32;
    double best_cost = 1e300;
    for (int c : cand) {
        const uint64_t tiles = (uint64_t)((M + c - 1) / c) * ((N + 127) / 128) * groups;
        double cost;
        if (tiles < 512 && K && K / 128 < kSplitBlocks / tiles) {
            // a short reduction cannot be cut into enough slices to fill the chip: the blocks all run
            // at once (or two to a unit), and what counts is how long one of them takes, in the same
            // unit as below (block duration per K-tile of the whole reduction, blocks per unit)
            const uint64_t splits = K / 128 >= 2 ? K / 128 : 1;
            const uint64_t kt = (K + KT - 1) / KT, kt_per = (kt + splits - 1) / splits;
            cost = (double)((tiles * splits + 255) / 256) * (c + 50) * (double)kt_per / (double)kt;
        } else if (tiles < 512) {
            cost = (double)tiles * (c + 50) / 256.0;                  // cut along K afterwards into one round of resident blocks
        } else {
            const uint64_t n = (tiles + 255) / 256;
            cost = ((n & 1) ? (double)(n - 1) + 1.2 : (double)n) * (c + 50);
        }
        if (cost < best_cost * 0.999) { best_cost = cost; best = c; }   // ties keep the larger tile
    }
    return best;
}

// lower bound of a map's offsets over its index range
int64_t map_min_off(const IndexMap &m)
{
    if (m.count == 0) return m.o0;
    const int64_t q1max = (m.count - 1) / m.d1.d;
    const int64_t q2max = (int64_t)((m.count - 1 < m.d1.d - 1 ? m.count - 1 : m.d1.d - 1)) / m.d2.d;
    const int64_t r2max = (int64_t)m.d2.d - 1;
    int64_t lo = m.o0;
    if (m.s1 < 0) lo += q1max * m.s1;
    if (m.s2 < 0) lo += q2max * m.s2;
    if (m.s3 < 0) lo += r2max * m.s3;
    return lo;
}
int64_t map_max_off(const IndexMap &m)
{
    if (m.count == 0) return m.o0;
    const int64_t q1max = (m.count - 1) / m.d1.d;
    const int64_t q2max = (int64_t)((m.count - 1 < m.d1.d - 1 ? m.count - 1 : m.d1.d - 1)) / m.d2.d;
    const int64_t r2max = (int64_t)m.d2.d - 1;
    int64_t hi = m.o0;
    if (m.s1 > 0) hi += q1max * m.s1;
    if (m.s2 > 0) hi += q2max * m.s2;
    if (m.s3 > 0) hi += r2max * m.s3;
    return hi;
}

// Moves the most negative part of both maps' offsets into the base pointer and checks that the
// buffer descriptor of every group, and every offset the kernel can form, fit 31 bits of bytes.
int normalise_operand(Operand &o, uint32_t groups)
{
    if (!o.ptr || !aligned16(o.ptr) || o.row.count == 0 || o.k.count == 0 || o.elems == 0) return CG_EINVAL;
    const int64_t lo_r = map_min_off(o.row), lo_k = map_min_off(o.k);
    o.row.o0 -= (int32_t)lo_r;
    o.k.o0 -= (int32_t)lo_k;
    o.shift = lo_r + lo_k;
    const int64_t span = (int64_t)o.elems - o.shift;          // floats behind the shifted base of group 0
    if (span <= 0 || (uint64_t)span * 4 > kMaxBufferBytes) return CG_EUNSUPPORTED;
    if ((uint64_t)(map_max_off(o.row) + 1) * 4 > kMaxBufferBytes || (uint64_t)(map_max_off(o.k) + 1) * 4 > kMaxBufferBytes)
        return CG_EUNSUPPORTED;
    if ((int64_t)(groups - 1) * o.gstride + o.shift >= (int64_t)o.elems) return CG_EINVAL;
    return CG_OK;
}

}  // namespace

namespace {

// pixel tiles (blocks along x) of a patch-kernel problem
uint32_t patch_pixel_tiles(const IgemmProblem &p)
{
    return p.patch.tiles_per_img ? (p.N / p.patch.divP.d) * (uint32_t)p.patch.tiles_per_img : (p.N + 127) / 128;
}

template <int TM, int NSTA, int NSL>
int launch_patch_cfg(const IgemmProblem &p, hipStream_t stream)
{
    constexpr int MT = 2 * TM * 32;
    using LA = KLoader4<MT, 4>;
    dim3 grid(p.patch.tile_count ? p.patch.tile_count : patch_pixel_tiles(p), (p.M + MT - 1) / MT, p.groups);
    if (grid.y > 65535u || grid.z > 65535u) return CG_EUNSUPPORTED;
    int rec = -1;
    if (prof_on()) {
        char name[64];
        snprintf(name, sizeof name, CG_MATH == 0 ? "igemm_patch_kernel<%dx128,%d>" : CG_MATH == 1 ? "igemm_patch_kernel<%dx128,%d,bf16>" : "igemm_patch_kernel<%dx128,%d,bf16x3>", MT, NSL);
        rec = prof_begin(name, p.flops > 0 ? p.flops : 2.0 * p.M * (double)p.N * p.K * p.groups, 0.0, stream);
    }
    constexpr size_t lds = ((size_t)NSTA * LA::SZ + 2 * PatchB<NSL>::BUF) * sizeof(float);
    static_assert(lds >= 4 * EpiLds<2>::FLOATS * sizeof(float), "the epilogue turns the tile around in the stages' LDS");
    static_assert(2 * lds <= 160 * 1024, "two blocks of this tile do not fit the LDS of a compute unit");
    static std::atomic<bool> attr_set{false};
    if (!attr_set.load(std::memory_order_acquire)) {
        CG_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(&igemm_patch_kernel<2, 2, TM, 2, NSTA, NSL, CG_MATH>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        attr_set.store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL((igemm_patch_kernel<2, 2, TM, 2, NSTA, NSL, CG_MATH>), grid, dim3(256), lds, stream, p);
    prof_end(rec, stream);
    CG_HIP_TRY(hipGetLastError());
    return CG_OK;
}

#if CG_MATH == 0
template <int TM, int NSTA, int NSL>
int launch_patch16_cfg(const IgemmProblem &p, hipStream_t stream)
{
    constexpr int MT = TM * 16;
    using LA = KLoader4<MT, 4>;
    dim3 grid(p.patch.tile_count ? p.patch.tile_count : patch_pixel_tiles(p), (p.M + MT - 1) / MT, p.groups);
    if (grid.y > 65535u || grid.z > 65535u) return CG_EUNSUPPORTED;
    int rec = -1;
    if (prof_on()) {
        char name[64];
        snprintf(name, sizeof name, "igemm_patch16_kernel<%dx128,%d>", MT, NSL);
        rec = prof_begin(name, p.flops > 0 ? p.flops : 2.0 * p.M * (double)p.N * p.K * p.groups, 0.0, stream);
    }
    constexpr size_t lds = ((size_t)NSTA * LA::SZ + 2 * PatchB<NSL, 4>::BUF) * sizeof(float);
    static_assert(2 * lds <= 160 * 1024, "two blocks of this tile do not fit the LDS of a compute unit");
    static std::atomic<bool> attr_set{false};
    if (!attr_set.load(std::memory_order_acquire)) {
        CG_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(&igemm_patch16_kernel<TM, NSTA, NSL>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        attr_set.store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL((igemm_patch16_kernel<TM, NSTA, NSL>), grid, dim3(256), lds, stream, p);
    prof_end(rec, stream);
    CG_HIP_TRY(hipGetLastError());
    return CG_OK;
}

#endif

// row-tile height of the patch kernel: 64, 128 or 192 rows
int patch_mt(uint32_t M, uint32_t N, uint32_t groups)
{
    const int mt = pick_mt(M, N, groups);
    return mt >= 192 && mt != 256 ? 192 : mt >= 96 ? 128 : 64;
}

int patch_launch_tiles(const IgemmProblem &p, int mt, hipStream_t stream)
{
    if (p.patch.nsl == 4) {
        if (mt == 192) return launch_patch_cfg<3, 3, 4>(p, stream);
        if (mt == 128) return launch_patch_cfg<2, 4, 4>(p, stream);
        return launch_patch_cfg<1, 4, 4>(p, stream);
    }
    if (p.patch.nsl == 6) {      // 2 x 50 KB of patch buffers: no 192-row tile beside them
        if (mt >= 128) return launch_patch_cfg<2, 3, 6>(p, stream);
        return launch_patch_cfg<1, 4, 6>(p, stream);
    }
    if (mt == 192) return launch_patch_cfg<3, 3, 5>(p, stream);
    if (mt == 128) return launch_patch_cfg<2, 4, 5>(p, stream);
    return launch_patch_cfg<1, 4, 5>(p, stream);
}

int patch_launch(const IgemmProblem &p, hipStream_t stream)
{
#if CG_MATH == 0
    // (three filter stages, not four, for the four- and five-chunk instances: 50.5 KB of LDS a block instead
    // of 53.7, so that three blocks fit a compute unit.  Alone on the GPU the kernel runs as before; beside
    // the weight-gradient kernel of the same layer on another stream the whole AlexNet-shaped step went
    // from 10.77 to 10.44 ms.)
    if (p.M <= 48) {             // the 16-row tiles waste less of a small row count than a 64-row tile
        const int tm = (int)(p.M + 15) / 16;
        if (p.patch.nsl == 4)
            return tm == 3 ? launch_patch16_cfg<3, 3, 4>(p, stream) : tm == 2 ? launch_patch16_cfg<2, 3, 4>(p, stream)
                                                                              : launch_patch16_cfg<1, 3, 4>(p, stream);
        if (p.patch.nsl == 6)
            return tm == 3 ? launch_patch16_cfg<3, 4, 6>(p, stream) : tm == 2 ? launch_patch16_cfg<2, 4, 6>(p, stream)
                                                                              : launch_patch16_cfg<1, 4, 6>(p, stream);
        return tm == 3 ? launch_patch16_cfg<3, 3, 5>(p, stream) : tm == 2 ? launch_patch16_cfg<2, 3, 5>(p, stream)
                                                                          : launch_patch16_cfg<1, 3, 5>(p, stream);
    }
#endif
    int mt = patch_mt(p.M, p.N, p.groups);
    // six chunks: no 192-row instance; 128-row tiles unless they would pad the rows by half a tile or more
    if (p.patch.nsl == 6 && mt > 64) mt = (p.M + 127) / 128 * 128 - p.M >= 64 ? 64 : 128;
    // Two blocks are resident per compute unit, so blocks run in rounds of g_resident_blocks that
    // start and end together.  When the last round would be less than three quarters full, the
    // pixel tiles of the whole rounds go out as one launch and the rest as a second launch of
    // 64-row tiles: three or two small blocks in place of a large one fill the compute units that
    // the short round would leave idle (676 blocks of 192 rows: 512 + 492 of 64 rows).  Forward only:
    // backward-data shares the GPU with backward-weight on another stream, whose blocks already
    // fill those compute units, and a second dependent launch then only delays it (measured).
    // Backward-data (mirrored taps) in the same situation takes 64-row tiles for the whole launch: three
    // of those blocks fit a compute unit, and twice or three times as many, shorter blocks quantise
    // better (676 blocks of 192 rows = 1.32 rounds of 512; 2028 of 64 rows = 2.64 rounds of 768).
    // Alone on the GPU: conv4-shaped 0.516 -> 0.461 ms, conv5-shaped 0.352 -> 0.315 ms at B = 256 (a
    // one-stream step 11.17 -> 10.82 ms); beside backward-weight on another stream, whose blocks fill the
    // short round anyway, the step was 0.07 ms slower with it, so a caller that runs such a stream says
    // so (beside_other_stream) and keeps the large tiles.
    if (mt > 64 && p.patch.tile_count == 0 && p.patch.flip && p.patch.nsl == 4 && !p.beside_other_stream) {
        const uint32_t rb = resident_blocks();
        const uint64_t blocks = (uint64_t)patch_pixel_tiles(p) * ((p.M + mt - 1) / mt) * p.groups;
        const uint32_t rest = (uint32_t)(blocks % rb);
        if (blocks / rb >= 1 && rest > 0 && rest < rb * 3 / 4) mt = 64;
    }
    if (mt > 64 && p.patch.tile_count == 0 && !p.patch.flip) {
        const uint32_t g_resident_blocks = resident_blocks();
        const uint32_t px = patch_pixel_tiles(p), per_px = ((p.M + mt - 1) / mt) * p.groups;
        const uint64_t blocks = (uint64_t)px * per_px;
        const uint32_t rounds = (uint32_t)(blocks / g_resident_blocks);
        const uint32_t rest = (uint32_t)(blocks - (uint64_t)rounds * g_resident_blocks);
        const uint32_t px_main = rounds * g_resident_blocks / per_px;
        const uint32_t tail_blocks = (px - px_main) * ((p.M + 63) / 64) * p.groups;
        if (rounds >= 1 && rest > 0 && rest < g_resident_blocks * 3 / 4 && px_main > 0 && px_main < px &&
            tail_blocks <= g_resident_blocks) {
            IgemmProblem a = p, b = p;
            a.patch.tile0 = 0;
            a.patch.tile_count = px_main;
            b.patch.tile0 = px_main;
            b.patch.tile_count = px - px_main;
            const double fl = p.flops > 0 ? p.flops : 2.0 * p.M * (double)p.N * p.K * p.groups;
            a.flops = fl * px_main / px;
            b.flops = fl - a.flops;
            const int rc = patch_launch_tiles(a, mt, stream);
            return rc != CG_OK ? rc : patch_launch_tiles(b, 64, stream);
        }
    }
    return patch_launch_tiles(p, mt, stream);
}

}  // namespace

#if CG_MATH == 0
namespace {

template <int TM, int NSTA, int CPB, int NSL>
int launch_wgrad_cfg(const IgemmProblem &p, hipStream_t stream)
{
    constexpr int MT = 2 * TM * 32;
    using LA = KLoader4<MT, 4>;
    dim3 grid((p.N + 127) / 128, (p.M + MT - 1) / MT, p.groups * p.splits);
    if (grid.y > 65535u || grid.z > 65535u) return CG_EUNSUPPORTED;
    int rec = -1;
    if (prof_on()) {
        char name[64];
        snprintf(name, sizeof name, "igemm_wgrad_kernel<%dx128,%d,%d>", MT, CPB, NSL);
        rec = prof_begin(name, p.flops > 0 ? p.flops : 2.0 * p.M * (double)p.N * p.K * p.groups, 0.0, stream);
    }
    constexpr size_t lds = ((size_t)NSTA * LA::SZ + 2 * CPB * (NSL * 64 + 1)) * sizeof(float);
    static_assert(lds >= 4 * EpiLds<2>::FLOATS * sizeof(float), "the epilogue turns the tile around in the stages' LDS");
    static_assert(2 * lds <= 160 * 1024, "two blocks of this tile do not fit the LDS of a compute unit");
    static std::atomic<bool> attr_set{false};
    if (!attr_set.load(std::memory_order_acquire)) {
        CG_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(&igemm_wgrad_kernel<2, 2, TM, 2, NSTA, CPB, NSL>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        attr_set.store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL((igemm_wgrad_kernel<2, 2, TM, 2, NSTA, CPB, NSL>), grid, dim3(256), lds, stream, p);
    prof_end(rec, stream);
    CG_HIP_TRY(hipGetLastError());
    return CG_OK;
}

int wgrad_mt(uint32_t M) { return M > 128 && (M + 191) / 192 * 192 <= (M + 127) / 128 * 128 ? 192 : M > 64 ? 128 : 64; }

int wgrad_launch(const IgemmProblem &p, hipStream_t stream)
{
    const int mt = wgrad_mt(p.M);
    if (p.wgrad.cpb == 16) {
        if (mt == 192) return launch_wgrad_cfg<3, 3, 16, 4>(p, stream);
        if (mt == 128) return launch_wgrad_cfg<2, 4, 16, 4>(p, stream);
        return launch_wgrad_cfg<1, 4, 16, 4>(p, stream);
    }
    if (mt == 192) return launch_wgrad_cfg<3, 3, 8, 8>(p, stream);
    if (mt == 128) return launch_wgrad_cfg<2, 4, 8, 8>(p, stream);
    return launch_wgrad_cfg<1, 4, 8, 8>(p, stream);
}

}  // namespace

static std::atomic<uint32_t> g_wgrad_enabled{0};
void wgrad_set_enabled(int on) { g_wgrad_enabled.store(on ? 1 : 0, std::memory_order_relaxed); }

bool wgrad_plan(WgradGeom &g, uint32_t M, uint32_t N, uint32_t groups, uint32_t images, uint32_t *splits)
{
    g.cpb = g.nsl = 0;
    const int KK = g.KH * g.KW;
    if (!g_wgrad_enabled.load(std::memory_order_relaxed) || KK < 9 || g.s <= 0 || g.Cg <= 0 || images == 0) return false;
    if (g.x_elems * 4 > kMaxBufferBytes || (uint64_t)images * g.M * g.OH * g.OW * 4 > kMaxBufferBytes) return false;
    g.Wp = (g.OW - 1) * g.s + g.KW;
    // channels a block of 128 columns can touch: at most 127/KK + 2
    const int chans = 127 / KK + 2;
    const int cpb = chans > 8 ? 16 : 8, nsl = cpb == 16 ? 4 : 8;
    if (chans > 16) return false;
    const int max_prow = nsl * 64 / g.Wp;                   // padded source rows that fit the staging
    const int max_rows = (max_prow - g.KH) / g.s + 1;       // output rows per band
    if (max_prow < g.KH || max_rows < 1) return false;
    g.nb = (g.OH + max_rows - 1) / max_rows;
    g.Rb = (g.OH + g.nb - 1) / g.nb;
    // every unit needs at least five K-tiles of 16 pixels (the patch of the next unit lands during four)
    const int last_rows = g.OH - (g.nb - 1) * g.Rb;
    if (last_rows < 1 || last_rows * g.OW < 5 * KT) return false;
    if ((uint64_t)images * g.nb >= (1u << 30)) return false;
    g.units = (int32_t)(images * (uint32_t)g.nb);
    g.divOW = make_fastdiv((uint32_t)g.OW);
    g.divWp = make_fastdiv((uint32_t)g.Wp);
    g.divKK = make_fastdiv((uint32_t)KK);
    g.divKW = make_fastdiv((uint32_t)g.KW);
    // K slices: at most kSplitBlocks blocks, whole units per slice
    const int mt = wgrad_mt(M);
    const uint64_t tiles = (uint64_t)((M + mt - 1) / mt) * ((N + 127) / 128) * groups;
    uint64_t want = kSplitBlocks / tiles;
    if (want > (uint64_t)g.units) want = (uint64_t)g.units;
    if (want < 1) want = 1;
    if (want > 4096) want = 4096;
    g.units_per_split = (int32_t)(((uint64_t)g.units + want - 1) / want);
    *splits = (uint32_t)(((uint64_t)g.units + g.units_per_split - 1) / g.units_per_split);
    if ((uint64_t)*splits * groups * M * N >= (1ull << 31)) return false;
    g.cpb = cpb; g.nsl = nsl;
    return true;
}

static std::atomic<uint32_t> g_patch_min_tiles{512};
void patch_set_min_tiles(uint32_t t) { g_patch_min_tiles.store(t, std::memory_order_relaxed); }
void patch_set_resident_blocks(uint32_t b) { g_resident_override.store(b, std::memory_order_relaxed); }

bool patch_plan(PatchGeom &g, uint32_t M, uint32_t N, uint32_t groups)
{
    g.nsl = 0;
    const int KK = g.KH * g.KW;
    if (g.Cred == 0 || g.Cred % 16 || KK < 5 || g.s <= 0 || g.OHo <= 0 || g.OWo <= 0) return false;
    if (g.src_elems * 4 > kMaxBufferBytes || N >= (1u << 30)) return false;
    g.Wp = (g.OWo - 1) * g.s + g.KW;
    const int64_t rfull = (int64_t)((g.OHo - 1) * g.s + g.KH) * g.Wp;
    if (rfull >= (1 << 24)) return false;
    g.Rfull = (int32_t)rfull;
    const uint32_t P = (uint32_t)g.OHo * (uint32_t)g.OWo;
    g.divP = make_fastdiv(P);
    g.divOW = make_fastdiv((uint32_t)g.OWo);
    g.divWp = make_fastdiv((uint32_t)g.Wp);
    g.divRfull = make_fastdiv((uint32_t)g.Rfull);
    // enough tiles to fill the chip without cutting K (the patch kernel has no K slices)
    const int mt = patch_mt(M, N, groups);
    if ((uint64_t)((M + mt - 1) / mt) * ((N + 127) / 128) * groups < g_patch_min_tiles.load(std::memory_order_relaxed)) return false;
    // The largest patch any block needs: a fragment read reaches (KH-1)*Wp + KW-1 beyond sigma, and
    // sigma + that stays below the slot count of the block's segments, which is what is counted.
    auto slots = [&](uint32_t n0, uint32_t n1) {
        const uint32_t bA = n0 / P, oyA = (n0 % P) / (uint32_t)g.OWo, bB = n1 / P, oyB = (n1 % P) / (uint32_t)g.OWo;
        if (bA == bB) return (int64_t)((oyB - oyA) * g.s + g.KH) * g.Wp;
        return (int64_t)(((uint32_t)g.OHo - 1 - oyA) * g.s + g.KH) * g.Wp + (int64_t)(bB - bA - 1) * g.Rfull +
               (int64_t)(oyB * g.s + g.KH) * g.Wp;
    };
    int64_t smax = 0;
    for (uint32_t n0 = 0; n0 < N; n0 += 128) {
        const int64_t sl = slots(n0, (n0 + 127 < N - 1) ? n0 + 127 : N - 1);
        if (sl > smax) smax = sl;
    }
    g.tiles_per_img = 0;
    g.divTpi = make_fastdiv(1);
    if (smax <= 4 * 64) { g.nsl = 4; return true; }
    // large images: blocks that stay inside one image need smaller patches (every image is the same)
    if (N % P) return false;
    int64_t amax = 0;
    for (uint32_t n0 = 0; n0 < P; n0 += 128) {
        const int64_t sl = slots(n0, (n0 + 127 < P - 1) ? n0 + 127 : P - 1);
        if (sl > amax) amax = sl;
    }
    // six chunks (planes 56 wide with a 3x3 window: four pixel rows, 348 slots) leave room for 128-row
    // tiles with a three-stage filter ring
    if (amax > 6 * 64) return false;
    g.nsl = amax > 5 * 64 ? 6 : 5;
    g.tiles_per_img = (int32_t)((P + 127) / 128);
    g.divTpi = make_fastdiv((uint32_t)g.tiles_per_img);
    return true;
}

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

void igemm_host_element(const Operand &op, uint32_t row, uint32_t k, int64_t *off, int *valid)
{
    const Info r = map_info(op.row, row), q = map_info(op.k, k);
    *valid = (uint32_t)(r.a + q.a) < op.limA && (uint32_t)(r.b + q.b) < op.limB &&
             (op.k.r1_lim == 0 || q.r1 < op.k.r1_lim);
    *off = (int64_t)r.off + q.off + op.shift;
}

#endif  // CG_MATH == 0

int CG_IGEMM_LAUNCH(const IgemmProblem &p0, hipStream_t stream)
{
#if CG_MATH == 0
    if (p0.math == CG_MATH_BF16) return igemm_launch_bf16(p0, stream);
    if (p0.math == CG_MATH_BF16X3) return igemm_launch_bf16x3(p0, stream);
    if (p0.math != CG_MATH_FP32) return CG_EINVAL;
#endif
    IgemmProblem p = p0;
    if (!p.c_ptr || !aligned16(p.c_ptr)) return CG_EINVAL;
    if (p.M == 0 || p.N == 0 || p.K == 0 || p.groups == 0 || p.splits == 0) return CG_EINVAL;
    if (p.M >= (1u << 30) || p.N >= (1u << 30) || p.K >= (1u << 30)) return CG_EUNSUPPORTED;
    if (p.bias_mode && !p.bias) return CG_EINVAL;
#if CG_MATH != 0
    if (p.use_wgrad) return CG_EUNSUPPORTED;      // the band kernel multiplies in fp32 only
#else
    if (p.use_wgrad) {         // K slices are whole units here, not k ranges
        if (!p.wgrad.x || !aligned16(p.wgrad.x) || p.wgrad.cpb == 0 || p.A.check) return CG_EINVAL;
        p.A.shift = 0;
        const int rcw = normalise_operand(p.A, p.groups);
        if (rcw) return rcw;
        return wgrad_launch(p, stream);
    }
#endif
    if (p.splits > 1 && (p.k_per_split % KT != 0)) return CG_EINVAL;
    if ((uint64_t)p.k_per_split * p.splits < p.K || (uint64_t)p.k_per_split * (p.splits - 1) >= p.K) return CG_EINVAL;
    if (p.bias_mode && !p.bias) return CG_EINVAL;
    if (p.A.check) return CG_EUNSUPPORTED;
    p.A.shift = p.B.shift = 0;
    int rc = normalise_operand(p.A, p.groups);
    if (rc) return rc;
    if (p.use_patch) {
        if (!p.patch.src || !aligned16(p.patch.src) || p.patch.nsl == 0 || p.splits != 1 || !quad_ok(p.A, p.K) ||
            p.K != p.patch.Cred * (uint32_t)(p.patch.KH * p.patch.KW))
            return CG_EINVAL;
        return patch_launch(p, stream);
    }
    if (p.A.row.count != p.M || p.B.row.count != p.N || p.A.k.count != p.K || p.B.k.count != p.K) return CG_EINVAL;
    rc = normalise_operand(p.B, p.groups);
    if (rc) return rc;
    if (!p.A.check) { p.A.limA = p.A.limB = 1; }
    if (!p.B.check) { p.B.limA = p.B.limB = 1; }

    const int mt = pick_mt(p.M, p.N, p.groups, p.K);
    const bool bc = p.B.check != 0;
    const int am = quad_ok(p.A, p.K) ? LD_K4 : p.A.lanes_k ? LD_K : LD_ROWS;
    int bm = quad_ok(p.B, p.K) ? LD_K4 : p.B.lanes_k ? LD_K : LD_ROWS;
    // A quad that reaches beyond K, or into the padding of a run of reduction indices, delivers the
    // floats that follow in memory (the next row's first elements): harmless only if the other
    // operand delivers exact zeros there, which the loaders that check every element do and the quad
    // loader does not.  Quads on both sides need a reduction range without any such position.
    if (am == LD_K4 && bm == LD_K4 && (p.K % 4 != 0 || p.A.k.r1_lim != 0 || p.B.k.r1_lim != 0)) bm = LD_K;
    if (am == LD_K4 && bm == LD_ROWS) return bc ? launch_modes<LD_K4, LD_ROWS, true>(p, mt, stream) : launch_modes<LD_K4, LD_ROWS, false>(p, mt, stream);
    if (am == LD_K4 && bm == LD_K4) return launch_modes<LD_K4, LD_K4, false>(p, mt, stream);
    if (am == LD_K4 && bm == LD_K) return bc ? launch_modes<LD_K4, LD_K, true>(p, mt, stream) : launch_modes<LD_K4, LD_K, false>(p, mt, stream);
    if (am == LD_K && bm == LD_ROWS) return bc ? launch_modes<LD_K, LD_ROWS, true>(p, mt, stream) : launch_modes<LD_K, LD_ROWS, false>(p, mt, stream);
    if (am == LD_K && (bm == LD_K || bm == LD_K4)) return bc ? launch_modes<LD_K, LD_K, true>(p, mt, stream) : launch_modes<LD_K, LD_K, false>(p, mt, stream);
    if (am == LD_ROWS && bm == LD_ROWS && !bc) return launch_modes<LD_ROWS, LD_ROWS, false>(p, mt, stream);
    return CG_EUNSUPPORTED;
}

#if CG_MATH == 0
// ---- split-K: more blocks for problems whose C has few tiles ---------------------------------

namespace {

struct FinishArgs {
    const float *part;
    int64_t plane;            // floats between consecutive K slices: groups * M * N
    int splits;
    float *c_ptr;
    int32_t c_row_stride;
    IndexMap c_col;
    int c_scatter;
    IndexMap c_row;
    uint32_t c_limA, c_limB;
    int64_t c_gstride;
    const float *bias;
    int bias_mode;
    int32_t bias_gstride;
    uint32_t M, N;
    FastDiv divN, divMN;
    int accumulate, relu;
    const float *gate;
    uint32_t total;           // groups * M * N
    // a convolution's bias gradient riding in the same launch: blocks finish_blocks.. sum one channel each
    const float *r_dy;
    int rN, rM, rP;
    FastDiv r_divQP;
    float *r_db;
    uint32_t finish_blocks;
};

typedef float f4u_b __attribute__((ext_vector_type(4), aligned(4)));

// Sum of dy[n][m][0..P) over the images n_beg..n_end-1, by one block; thread 0 returns it.
// The (image, group of four pixels) pairs are spread over the threads, each moving 16 bytes
// (4-byte aligned: planes of an odd pixel count start anywhere) with four loads in flight.
__device__ __forceinline__ float bias_channel_sum(const float *__restrict__ dy, int M, int P, int m, int n_beg, int n_end,
                                                  FastDiv divQP)
{
    const uint32_t QP = divQP.d, total = (uint32_t)(n_end - n_beg) * QP;
    float s = 0.f;
    for (uint32_t i0 = threadIdx.x; i0 < total; i0 += 256 * 4) {
        f4u_b v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t i = i0 + u * 256;
            v[u] = f4u_b{0.f, 0.f, 0.f, 0.f};
            if (i < total) {
                const uint32_t n = fdiv(i, divQP), qd = i - n * QP;
                const float *src = dy + ((size_t)(n_beg + (int)n) * M + m) * P + 4 * qd;
                const int rem = P - 4 * (int)qd;
                if (rem >= 4) v[u] = __builtin_nontemporal_load(reinterpret_cast<const f4u_b *>(src));
                else {
                    v[u].x = src[0];
                    if (rem > 1) v[u].y = src[1];
                    if (rem > 2) v[u].z = src[2];
                }
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) s += (v[u].x + v[u].y) + (v[u].z + v[u].w);
    }
    __shared__ float red[256];
    red[threadIdx.x] = s;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
        __syncthreads();
    }
    return red[0];
}

// C = (sum over the K slices) + bias, written through the problem's output map.  With few slices a
// thread adds them in slice order.  With many (ROWS = 8) a block owns 32 consecutive elements, its
// 8 thread rows add interleaved slices (row r: slices r, r+8, ...), and the 8 row sums are added
// in row order.  Either way the association is fixed by the number of slices alone, so the result
// does not depend on scheduling.
__device__ __forceinline__ void finish_store(const FinishArgs &a, uint32_t i, float s)
{
    const uint32_t g = fdiv(i, a.divMN), rem = i - g * a.divMN.d;
    const uint32_t m = fdiv(rem, a.divN), n = rem - m * a.divN.d;
    if (a.bias_mode == 1) s += a.bias[(int64_t)g * a.bias_gstride + m];
    else if (a.bias_mode == 2) s += a.bias[(int64_t)g * a.bias_gstride + n];
    if (a.relu) s = fmaxf(s, 0.f);
    const Info ci = map_info(a.c_col, n);
    int32_t in_group = (int32_t)m * a.c_row_stride + ci.off;
    if (a.c_scatter) {
        const Info ri = map_info(a.c_row, m);
        if (!((uint32_t)(ri.a + ci.a) < a.c_limA && (uint32_t)(ri.b + ci.b) < a.c_limB)) return;
        in_group = ri.off + ci.off;
    }
    const int64_t idx = (int64_t)g * a.c_gstride + in_group;
    if (a.gate && !(a.gate[idx] > 0.f)) s = 0.f;
    float *dst = a.c_ptr + idx;
    if (a.accumulate) s += *dst;
    *dst = s;
}

template <int ROWS> __global__ __launch_bounds__(256) void splitk_finish_kernel(const FinishArgs a)
{
    if (a.r_dy && blockIdx.x >= a.finish_blocks) {       // a rider block: one channel of the bias gradient
        const int m = (int)(blockIdx.x - a.finish_blocks);
        const float s = bias_channel_sum(a.r_dy, a.rM, a.rP, m, 0, a.rN, a.r_divQP);
        if (threadIdx.x == 0) a.r_db[m] = s;
        return;
    }
    const uint32_t nblk = a.r_dy ? a.finish_blocks : gridDim.x;
    if (ROWS == 1) {
        for (uint32_t i = blockIdx.x * 256 + threadIdx.x; i < a.total; i += nblk * 256) {
            float s = a.part[i];
            for (int k = 1; k < a.splits; ++k) s += a.part[(int64_t)k * a.plane + i];
            finish_store(a, i, s);
        }
        return;
    }
    __shared__ float part[8][33];
    const int el = threadIdx.x & 31, r = threadIdx.x >> 5;
    for (uint32_t i0 = blockIdx.x * 32; i0 < a.total; i0 += nblk * 32) {
        const uint32_t i = i0 + el;
        float s = 0.f;
        if (i < a.total)
            for (int k = r; k < a.splits; k += 8) s += a.part[(int64_t)k * a.plane + i];
        part[r][el] = s;
        __syncthreads();
        if (r == 0 && i < a.total) {
            s = part[0][el];
#pragma unroll
            for (int k = 1; k < 8; ++k) s += part[k][el];
            finish_store(a, i, s);
        }
        __syncthreads();
    }
}

}  // namespace

SplitPlan plan_split(uint32_t M, uint32_t N, uint32_t K, uint32_t groups)
{
    SplitPlan pl{1, K, 0};
    const uint32_t mt = (uint32_t)pick_mt(M, N, groups, K);
    const uint64_t tiles = (uint64_t)((M + mt - 1) / mt) * ((N + 127) / 128) * groups;
    if (tiles >= 512) return pl;
    uint64_t want = kSplitBlocks / tiles;
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
    if (p.use_patch) return 0;
    if (p.use_wgrad) return p.splits > 1 ? (size_t)p.splits * p.groups * p.M * p.N * sizeof(float) : 0;
    return plan_split(p.M, p.N, p.K, p.groups).ws_bytes;
}

int igemm_run(const IgemmProblem &p0, void *ws, size_t ws_bytes, hipStream_t stream, const BiasRider *rider, bool *rider_taken)
{
    if (rider_taken) *rider_taken = false;
    const SplitPlan pl = p0.use_patch   ? SplitPlan{1, p0.K, 0}
                         : p0.use_wgrad ? SplitPlan{p0.splits, p0.K, igemm_ws_bytes(p0)}
                                        : plan_split(p0.M, p0.N, p0.K, p0.groups);
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
    p.c_scatter = 0;
    p.bias = nullptr; p.bias_mode = 0; p.accumulate = 0; p.relu = 0; p.gate = nullptr;
    p.splits = pl.splits; p.k_per_split = pl.k_per_split;
    const int rc = igemm_launch(p, stream);
    if (rc) return rc;
    FinishArgs a{};
    a.part = static_cast<const float *>(ws);
    a.plane = p.c_split_stride;
    a.splits = (int)pl.splits;
    a.c_ptr = p0.c_ptr; a.c_row_stride = p0.c_row_stride; a.c_col = p0.c_col; a.c_gstride = p0.c_gstride;
    a.c_scatter = p0.c_scatter; a.c_row = p0.c_row; a.c_limA = p0.c_limA; a.c_limB = p0.c_limB;
    a.bias = p0.bias; a.bias_mode = p0.bias_mode; a.bias_gstride = p0.bias_gstride;
    a.M = p0.M; a.N = p0.N;
    a.divN = make_fastdiv(p0.N);
    a.divMN = make_fastdiv(p0.M * p0.N);
    a.accumulate = p0.accumulate; a.relu = p0.relu; a.gate = p0.gate;
    a.total = p0.groups * p0.M * p0.N;
    unsigned riders = 0;
    if (rider && rider->dy && rider->db && rider->M > 0 && rider->M <= 65536 &&
        (uint64_t)rider->N * (uint64_t)((rider->P + 3) / 4) < (1ull << 31)) {
        a.r_dy = rider->dy; a.rN = rider->N; a.rM = rider->M; a.rP = rider->P; a.r_db = rider->db;
        a.r_divQP = make_fastdiv((uint32_t)(rider->P + 3) / 4);
        riders = (unsigned)rider->M;
        if (rider_taken) *rider_taken = true;
    }
    if (pl.splits >= 16) {
        const unsigned blocks = (a.total + 31) / 32 < 65536 ? (a.total + 31) / 32 : 65536;
        a.finish_blocks = blocks;
        hipLaunchKernelGGL(splitk_finish_kernel<8>, dim3(blocks + riders), dim3(256), 0, stream, a);
    } else {
        const unsigned blocks = (a.total + 255) / 256 < 16384 ? (a.total + 255) / 256 : 16384;
        a.finish_blocks = blocks;
        hipLaunchKernelGGL(splitk_finish_kernel<1>, dim3(blocks + riders), dim3(256), 0, stream, a);
    }
    CG_HIP_TRY(hipGetLastError());
    return CG_OK;
}

// ---- bias gradient of a convolution: db[m] = sum over n and pixels of dy[n][m][pix] ------------

namespace {

// block (m, s) sums the samples of slice s; the slices are added afterwards in slice order.
// The (image, group of four pixels) pairs of the slice are spread over the threads, each moving
// 16 bytes (4-byte aligned: planes of an odd pixel count start anywhere) with four loads in flight.
typedef float f4u __attribute__((ext_vector_type(4), aligned(4)));

__global__ __launch_bounds__(256) void bias_grad_partial_kernel(const float *__restrict__ dy, int N, int M, int P,
                                                                int n_per, FastDiv divQP, float *__restrict__ part)
{
    const int m = blockIdx.x, sl = blockIdx.y;
    const int n_beg = sl * n_per, n_end = min(N, n_beg + n_per);
    const float s = bias_channel_sum(dy, M, P, m, n_beg, n_end, divQP);
    if (threadIdx.x == 0) part[(size_t)sl * M + m] = s;
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

bool bias_grad_single_launch(int N, int P) { return (uint64_t)N * (uint64_t)P <= 32768; }

int bias_grad_launch(const float *dy, int N, int M, int P, float *db, void *ws, size_t ws_bytes,
                     hipStream_t stream)
{
    if (!dy || !db || N <= 0 || M <= 0 || P <= 0) return CG_EINVAL;
    if (!ws || ws_bytes < bias_grad_ws_bytes(N, M)) return CG_ENOSPC;
    // a small layer: one block per channel sums all images and writes db itself (one launch)
    const int S = bias_grad_single_launch(N, P) ? 1 : bias_slices(N, M);
    const int n_per = (N + S - 1) / S;
    const int S2 = (N + n_per - 1) / n_per;
    float *part = static_cast<float *>(ws);
    if ((uint64_t)n_per * (uint64_t)((P + 3) / 4) >= (1ull << 31)) return CG_EUNSUPPORTED;     // 32-bit pair index
    hipLaunchKernelGGL(bias_grad_partial_kernel, dim3(M, S2), dim3(256), 0, stream, dy, N, M, P, n_per,
                       make_fastdiv((uint32_t)(P + 3) / 4), S2 == 1 ? db : part);
    CG_HIP_TRY(hipGetLastError());
    if (S2 == 1) return CG_OK;
    hipLaunchKernelGGL(bias_grad_finish_kernel, dim3((M + 255) / 256), dim3(256), 0, stream, part, M, S2, db);
    CG_HIP_TRY(hipGetLastError());
    return CG_OK;
}

#endif  // CG_MATH == 0

}  // namespace cg
