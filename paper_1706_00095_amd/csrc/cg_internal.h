// Internal declarations shared by the translation units of libcg (never installed).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "cg.h"
#include "cg_debug.h"

namespace cg {

// Every kernel launch of the library is counted (cg_debug_launch_count): nets of many small layers
// are bound by the number of launches, and benchmarks report it.
void note_launch();
}  // namespace cg
#undef hipLaunchKernelGGL
#define hipLaunchKernelGGL(kernelName, ...)                          \
    do {                                                             \
        ::cg::note_launch();                                         \
        hipLaunchKernelGGLInternal((kernelName), __VA_ARGS__);       \
    } while (0)

namespace cg {

// Records the failing hipError_t for cg_last_hip_error() and maps it to CG_EHIP.
int hip_fail(hipError_t e);

#define CG_HIP_TRY(expr)                                   \
    do {                                                   \
        hipError_t e__ = (expr);                           \
        if (e__ != hipSuccess) return ::cg::hip_fail(e__); \
    } while (0)

// ---- per-launch timing (api.hip) ---------------------------------------------------------------
// When enabled through cg_profile_enable(), every implicit-GEMM and reduce+update launch is
// bracketed by two HIP events on the stream it is launched on and logged with its
// algorithmic work.  ProfTag names the pass (and layer) that issues the launches in its scope.
struct ProfTag {
    ProfTag(const char *pass, int layer);
    ~ProfTag();
    const char *prev_pass;
    int prev_layer;
};
bool prof_on();
// returns a record index (or -1) after recording the start event
int prof_begin(const char *kernel, double flops, double bytes, hipStream_t s);
void prof_end(int rec, hipStream_t s);

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// ---- index maps: how a GEMM coordinate becomes a tensor element ---------------------------
//
// Every operand of every pass (forward, backward-data, backward-weight, fully connected) is
// addressed as  element(row, k) = ptr[ R.off + K.off ],  valid iff
//   (unsigned)(R.a + K.a) < limA  &&  (unsigned)(R.b + K.b) < limB,
// where R = info(row index) and K = info(reduction index).  An index is split twice,
// idx = q1*d1 + r1, r1 = q2*d2 + r2, and
//   off = q1*s1 + q2*s2 + r2*s3 + o0,   a = q2*sa + a0,   b = r2*sb + b0.
// A pixel index (n,oh,ow) of a convolution input uses d1 = OH*OW, d2 = OW, a = oh*s - p,
// b = ow*s - p; a filter-tap index (c,kh,kw) uses d1 = KH*KW, d2 = KW, a = kh, b = kw; a plain
// matrix dimension uses d1 = d2 = 1.  The sum a_row + a_k is then the input row ih, and the
// unsigned compare against H implements zero padding.

struct FastDiv {       // exact n / d for n < 2^31:  q = (uint64(n) * mul) >> sh
    uint32_t d, mul, sh;
};

struct IndexMap {
    uint32_t count;    // indices >= count are out of range (read as 0 / not stored)
    FastDiv d1, d2;
    int32_t s1, s2, s3, o0;
    int32_t sa, a0, sb, b0;
    uint32_t r1_lim;   // if non-zero: indices with r1 >= r1_lim are padding (read as 0): runs of r1_lim real
                       // indices, each padded to d1 (a reduction over images whose pixel count is rounded
                       // up to a multiple of 4 so that aligned groups of four never straddle two images)
};

struct Info { int32_t off, a, b; uint32_t r1; };

FastDiv make_fastdiv(uint32_t d);
IndexMap linear_map(uint32_t count, int32_t stride);
// idx = q*d + r  ->  off = q*sq + r*sr
IndexMap split_map(uint32_t count, uint32_t d, int32_t sq, int32_t sr);

__host__ __device__ inline uint32_t fdiv(uint32_t n, const FastDiv &f)
{
    return (uint32_t)(((uint64_t)n * f.mul) >> f.sh);
}

// offset and window coordinates of index idx (any idx < 2^31; the caller checks the range)
__host__ __device__ inline Info map_info(const IndexMap &m, uint32_t idx)
{
    Info r;
    const uint32_t q1 = fdiv(idx, m.d1), r1 = idx - q1 * m.d1.d;
    const uint32_t q2 = fdiv(r1, m.d2), r2 = r1 - q2 * m.d2.d;
    r.off = (int32_t)q1 * m.s1 + (int32_t)q2 * m.s2 + (int32_t)r2 * m.s3 + m.o0;
    r.a = (int32_t)q2 * m.sa + m.a0;
    r.b = (int32_t)r2 * m.sb + m.b0;
    r.r1 = r1;
    return r;
}

struct Operand {
    const float *ptr;
    IndexMap row, k;
    uint32_t limA, limB;
    int64_t gstride;      // elements between groups
    uint64_t elems;       // floats behind ptr (all groups): the bound of the kernel's buffer descriptor
    int lanes_k;          // which index runs along the 64 lanes of one load, i.e. the direction that is
                          // (nearly) contiguous in memory: 1 = the reduction index, 0 = the row index
    int check;            // 1 = the (a, b) window test is needed (zero padding); 0 = always valid
    int64_t shift;        // set by igemm_launch: elements moved from the maps' offsets into the base
                          // pointer so that both per-index offsets are non-negative
};

// Operand B of a convolution seen as raw image patches instead of gathered im2col rows.  The N
// rows of B are output pixels (img, oy, ox) of a grid OHo x OWo; the reduction index is
// (tap t = ky*KW + kx, channel c), tap-major, with Cred % 16 == 0 channels per group; element
// (pixel, t, c) is src[img][group*Cred + c][oy*s + oy0 + py(t)][ox*s + ox0 + px(t)] or zero outside
// the Hs x Ws plane, where (py, px) = (ky, kx) in forward and (KH-1-ky, KW-1-kx) in backward-data.
// The kernel keeps, per block of 128 pixels and 16 channels, the padded source rows those pixels'
// windows touch in LDS and reads each tap's operand fragment from there at a per-tap offset.
struct PatchGeom {
    const float *src;
    uint64_t src_elems;       // floats behind src
    int64_t gstride;          // elements between groups: Cred * Hs * Ws
    uint32_t Cred;
    int32_t Hs, Ws, chan_stride;
    int32_t img_stride;       // Ctot * Hs * Ws (elements)
    int32_t OHo, OWo, s, oy0, ox0, KH, KW;
    int32_t Wp;               // padded patch width: (OWo-1)*s + KW
    int32_t Rfull;            // slots of a whole image: ((OHo-1)*s + KH) * Wp
    int32_t flip;             // 0: (py, px) = (ky, kx); 1: mirrored taps
    FastDiv divP, divOW, divWp, divRfull;
    int32_t nsl;              // 64-slot chunks per channel the kernel instance stages (4 or 5); 0 = not usable
    int32_t tiles_per_img;    // 0: blocks own 128 consecutive pixels across image boundaries; > 0: every image is
                              // cut into this many blocks of its own (smaller patches for large images)
    FastDiv divTpi;
    uint32_t tile0;           // first pixel tile of this launch (blockIdx.x counts from it)
    uint32_t tile_count;      // pixel tiles of this launch; 0 = all
};

// Backward-weight seen as  dw[m][(c,kh,kw)] = sum over pixels of dy[m][pix] * x[c][window of pix at (kh,kw)]
// with the input staged as raw padded rows: the reduction walks "units" = (image, band of Rb output
// rows), whose padded source rows (((rows-1)*s + KH) x Wp slots per channel) a block keeps in LDS for
// the channels its 128 columns (c,kh,kw) belong to, while dy arrives in K-tiles of 16 pixels.
struct WgradGeom {
    const float *x;
    uint64_t x_elems;
    int32_t C, Cg, H, W, OH, OW, s, pad_h, pad_w, KH, KW;
    int32_t M;                // all output channels (dy's channel count)
    int32_t Wp;               // padded patch width (OW-1)*s + KW
    int32_t nb, Rb;           // bands per image, output rows per band (the last band of an image takes the rest)
    int32_t units;            // images * nb
    int32_t units_per_split;
    int32_t cpb, nsl;         // channels and 64-slot chunks per channel a block stages: (16, 4) or (8, 8); 0 = unusable
    FastDiv divOW, divWp, divKK, divKW;
};

// C[m][n] = sum_k A(m,k) * B(n,k)   (+ bias), for `groups` independent problems, the K range
// optionally cut into `splits` slices whose partial results go to consecutive output planes.
struct IgemmProblem {
    Operand A, B;
    float *c_ptr;
    int32_t c_row_stride;     // C row m lives at m * c_row_stride (+ column offset)
    IndexMap c_col;           // column n -> offset
    // Scattered output (c_scatter != 0): row m lives at map_info(c_row, m).off instead, and element
    // (m, n) exists only if (unsigned)(row.a + col.a) < c_limA && (unsigned)(row.b + col.b) < c_limB
    // (backward-data of a strided convolution: rows are (channel, stride phase), columns are cells of
    // stride x stride input pixels, and phases that fall outside the image are not stored).
    int c_scatter;
    IndexMap c_row;
    uint32_t c_limA, c_limB;
    int64_t c_gstride, c_split_stride;
    const float *bias;        // per row (bias_mode 1) or per column (2); NULL / 0 = none
    int bias_mode;
    int32_t bias_gstride;
    uint32_t M, N, K;
    uint32_t groups, splits, k_per_split;
    double flops;             // algorithmic work to report (0: 2*M*N*K*groups; set when K counts padding)
    int accumulate;           // C += result instead of C = result
    int relu;                 // C = max(result, 0) after bias (forward passes followed by a rectifier)
    const float *gate;        // same layout as C, or NULL: result = 0 where gate <= 0 (backward-data into a
                              // rectifier: the gradient with respect to the rectifier's input), before accumulate
    int math;                 // CG_MATH_FP32, CG_MATH_BF16 or CG_MATH_BF16X3: what the matrix instructions multiply in
    int beside_other_stream;  // the caller runs matrix kernels on another stream meanwhile (tile choice of the patch kernel)
    int use_patch;            // B is described by `patch` (and A is the matching tap-major matrix); B unused
    PatchGeom patch;
    int use_wgrad;            // backward-weight from image bands (`wgrad`): A = dy rows, B unused, K counted in pixels
    WgradGeom wgrad;
};

// Fills the derived fields of a patch description (Wp, Rfull, dividers) and decides whether the
// patch kernel can run it for N output pixels and M rows: sets g.nsl, returns true if usable.
bool patch_plan(PatchGeom &g, uint32_t M, uint32_t N, uint32_t groups);
// The same for backward-weight: fills Wp, bands, dividers, chooses the staging and the number of K
// slices (p.splits, units_per_split); returns true if the band kernel can run the problem.
bool wgrad_plan(WgradGeom &g, uint32_t M, uint32_t N, uint32_t groups, uint32_t images, uint32_t *splits);
void wgrad_set_enabled(int on);     // tests compare the band kernel with the gathered one
// smallest number of C tiles for which the patch kernel is chosen (512; tests lower it)
void patch_set_resident_blocks(uint32_t blocks);
void patch_set_min_tiles(uint32_t t);

// Validates the problem against what the kernels assume and launches it.
int igemm_launch(const IgemmProblem &p, hipStream_t stream);
// The same for the bf16 matrix instructions (igemm_launch dispatches on p.math)
int igemm_launch_bf16(const IgemmProblem &p, hipStream_t stream);
int igemm_launch_bf16x3(const IgemmProblem &p, hipStream_t stream);
// Host-side evaluation of one operand element: offset and validity (for tests of the maps).
void igemm_host_element(const Operand &op, uint32_t row, uint32_t k, int64_t *off, int *valid);

// Split-K front end: when C has too few tiles to fill the chip, the K range is cut into slices
// whose partial results go to `ws` and are then added in slice order (so results do not depend
// on scheduling).  igemm_ws_bytes() says how much workspace igemm_run() needs for a problem.
struct SplitPlan { uint32_t splits, k_per_split; size_t ws_bytes; };
SplitPlan plan_split(uint32_t M, uint32_t N, uint32_t K, uint32_t groups);
size_t igemm_ws_bytes(const IgemmProblem &p);
// rider: a small convolution's bias gradient (db[m] = sum of dy over images and pixels), summed by
// extra blocks of the K-slice finishing launch, one block per channel, instead of a launch of its
// own; *rider_taken says whether that happened (it does not when the problem runs without K slices).
struct BiasRider { const float *dy; int N, M, P; float *db; };
int igemm_run(const IgemmProblem &p, void *ws, size_t ws_bytes, hipStream_t stream, const BiasRider *rider = nullptr,
              bool *rider_taken = nullptr);
// db[m] = sum over n and pixels of dy[n][m][pix]; two passes over `ws`, fixed order
size_t bias_grad_ws_bytes(int N, int M);
bool bias_grad_single_launch(int N, int P);       // small enough for one block per channel, no partial sums
int bias_grad_launch(const float *dy, int N, int M, int P, float *db, void *ws, size_t ws_bytes,
                     hipStream_t stream);


// ---- convolution / fully-connected passes (conv.hip) ----------------------------------------
int conv_check(const cg_conv_desc *d, int *OH, int *OW);
size_t conv_ws_bytes(const cg_conv_desc &d, int pass);
size_t fc_ws_bytes(int B, int IN, int OUT, int pass);
// relu != 0: y = max(conv + bias, 0), the rectifier that follows folded into the store
// math: CG_MATH_* (what the matrix instructions multiply in; workspace sizes do not depend on it)
// prepared: if not null, the rearranged copy of the filters this pass multiplies with (what
// conv_fwd_filter_prep / conv_bwd_data_filter_prep describe for this descriptor), made beforehand by
// filter_prep_launch from the same w; the pass then launches no rearrangement of its own
int conv_fwd_impl(const cg_conv_desc &d, const float *x, const float *w, const float *bias, float *y, void *ws,
                  size_t ws_bytes, int relu, hipStream_t stream, int64_t y_img_stride = 0, int math = 0,
                  const float *prepared = nullptr);
int conv_bwd_data_impl(const cg_conv_desc &d, const float *dy, const float *w, float *dx, const float *gate, void *ws,
                       size_t ws_bytes, int accumulate, hipStream_t stream, int math = 0, const float *prepared = nullptr,
                       bool beside_other_stream = false);
// Which rearranged copy of its filters a pass needs (kind CG_PREP_NONE: it reads w itself), and how
// many floats the copy has.  The answer follows the same kernel choice the pass itself makes.
enum { CG_PREP_NONE = 0, CG_PREP_TRANSPOSE, CG_PREP_PERMUTE_FWD, CG_PREP_PERMUTE_BWD, CG_PREP_STRIDED_TAPS, CG_PREP_STRIDED_ROWS };
struct FilterPrep {
    int kind;
    size_t floats;
    int Mg, Cg, KH, KW, sh, sw, Ah, Aw;
};
FilterPrep conv_fwd_filter_prep(const cg_conv_desc &d);
FilterPrep conv_bwd_data_filter_prep(const cg_conv_desc &d);
size_t conv_filter_prep_max_floats(const cg_conv_desc &d);      // upper bound of either copy, for sizing
// n copies, eight per launch: job i reads w[i] and writes dst[i] (16-byte aligned, jobs[i].floats floats)
int filter_prep_launch(int n, const FilterPrep *jobs, const float *const *w, float *const *dst, hipStream_t stream);
// bias_stream: if not null, the bias sums are enqueued there instead of on `stream` (dy must be complete
// in that stream's order as well, and the caller joins both streams before db is used)
int conv_bwd_weight_impl(const cg_conv_desc &d, const float *x, const float *dy, float *dw, float *db,
                         void *ws, size_t ws_bytes, hipStream_t stream, int math = 0, hipStream_t bias_stream = nullptr,
                         void *bias_ws = nullptr, size_t bias_ws_bytes = 0);
int fc_fwd_impl(int B, int IN, int OUT, const float *x, const float *W, const float *bias, float *y, void *ws,
                size_t ws_bytes, int relu, hipStream_t stream, int math = 0);
int fc_bwd_data_impl(int B, int IN, int OUT, const float *dy, const float *W, float *dx, const float *gate,
                     int accumulate, void *ws, size_t ws_bytes, hipStream_t stream, int math = 0);
int fc_bwd_weight_impl(int B, int IN, int OUT, const float *x, const float *dy, float *dW, float *db, void *ws,
                       size_t ws_bytes, hipStream_t stream, int math = 0);

// ---- gradient aggregation + update (sgd.hip) --------------------------------------------------
int grad_reduce_sgd_impl(float *w, float *v, const float *g_local, const float *const *g_peers, int K,
                         size_t n, const cg_sgd &sgd, hipStream_t stream, bool tree = false);
int grad_reduce_sgd_multi_impl(int nb, float *const *w, float *const *v, const float *const *g_local,
                               const float *const *const *g_peers, int K, const size_t *n, const cg_sgd &sgd,
                               hipStream_t stream, bool tree = false);

// ---- the other layers (layers.hip) -------------------------------------------------------------
int fc_bias_grad_launch(const float *dy, int B, int OUT, float *db, hipStream_t stream);
int relu_fwd_launch(const float *x, float *y, size_t n, hipStream_t s);
int relu_bwd_launch(const float *x, const float *dy, float *dx, size_t n, int accumulate, hipStream_t s);
int pool_out_size(int H, int k, int s, int p);
int maxpool_fwd_launch(const float *x, float *y, int32_t *argmax, int N, int C, int H, int W, int k, int s, int p,
                       hipStream_t st);
// `gate` (maxpool, dropout: a pointer or NULL; LRN: a flag, the gate being its own input x): the
// layer's input is the output of a rectifier, and dx is the gradient with respect to that
// rectifier's input, i.e. zero wherever the gate is not positive.
int maxpool_bwd_launch(const float *dy, const int32_t *argmax, float *dx, const float *gate, int N, int C, int H, int W,
                       int k, int s, int p, int accumulate, hipStream_t st);
int lrn_fwd_launch(const float *x, float *y, int N, int C, int HW, int size, float alpha, float beta, float kappa,
                   hipStream_t st);
// recomputes the scales from x; nothing saved by forward is read
int lrn_bwd_launch(const float *x, const float *dy, float *dx, int N, int C, int HW, int size, float alpha, float beta,
                   float kappa, int accumulate, int gate, hipStream_t st);
// LRN followed by max-pooling in one pass (neither the normalised tensor nor its gradient is
// materialised); lrn_pool_fusable says whether the fused kernels take a layer pair
bool lrn_pool_fusable(int C, int H, int W, int size, int k, int s, int p);
int lrn_pool_fwd_launch(const float *x, float *y, int32_t *argmax, int N, int C, int H, int W, int size, float alpha,
                        float beta, float kappa, int k, int s, int p, hipStream_t st);
int lrn_pool_bwd_launch(const float *x, const float *dpool, const int32_t *argmax, float *dx, int N, int C, int H, int W,
                        int size, float alpha, float beta, float kappa, int k, int s, int p, int accumulate, int gate,
                        hipStream_t st);
int avgpool_fwd_launch(const float *x, float *y, int NC, int HW, hipStream_t st);
int avgpool_bwd_launch(const float *dy, float *dx, int NC, int HW, int accumulate, hipStream_t st);
int dropout_launch(const float *x, const uint8_t *mask, float *y, const float *gate, size_t n, float p, int accumulate,
                   hipStream_t st);
// per_sample: B floats of scratch
int softmax_ce_launch(const float *z, const int32_t *labels, float *loss, float *dz, float *per_sample, int B, int C,
                      hipStream_t st);
// dst[n][c_off + c][hw] = src[n][c][hw]  (forward of a channel concat) or the reverse slice copy
int concat_copy_launch(const float *src, float *dst, int N, int Csrc, int Cdst, int c_off, int HW, int to_concat,
                       int accumulate, const float *gate, hipStream_t st);

}  // namespace cg
