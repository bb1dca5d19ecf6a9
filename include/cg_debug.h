/*
 * cg_debug.h -- test hooks and measurement aids of libcg.  Not part of the
 * product boundary (cg.h): nothing here is needed to run the iteration.  The
 * hooks that change which kernel a call selects are process-wide switches
 * (stored atomically); a test that flips one must not run beside other users
 * of the library.
 */
#ifndef CG_DEBUG_H
#define CG_DEBUG_H
#include "cg.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Test hook: forward and stride-1 backward-data convolutions with enough
 * output tiles to fill the chip without cutting the reduction (512 by default)
 * run a kernel that stages raw image rows instead of gathered im2col tiles;
 * tests lower the threshold so that small shapes the oracle can check element
 * by element take that path too.  Process-wide. */
int cg_debug_patch_min_tiles(int tiles);

/* Test hook: the number of blocks the GPU keeps resident at once (512 = 256
 * compute units x 2), which decides where a patch-kernel launch is cut into a
 * launch of whole rounds and a launch of smaller tiles for the rest.  Tests
 * lower it so that small shapes take the two-launch path.  Process-wide. */
int cg_debug_resident_blocks(int blocks);

/* Switch for an alternative backward-weight kernel that stages bands of raw
 * image rows in LDS (convolutions with at least nine taps).  Off by default:
 * alone on the GPU it is a few percent faster than the gathered kernel at the
 * 3x3 AlexNet shapes, but beside the backward-data kernels of the three-stream
 * schedule the whole iteration is slower with it.  on = 1 selects it where it
 * applies, so that tests can compare the two.  Process-wide. */
int cg_debug_band_kernel(int on);

/* Measurement aid: dst[0..bytes) = src[0..bytes) by a plain kernel (16-byte
 * aligned device pointers, bytes % 16 == 0): a dispatch of known HBM traffic to
 * scale hardware-counter readings of the other kernels by. */
int cg_debug_copy(void *dst, const void *src, size_t bytes, void *stream);

/* Test hook (host only, launches nothing): which element of which tensor the
 * implicit-GEMM view of a convolution pass reads for operand A (0) or B (1) at
 * (row, k) of the given group.  elem_offset is in floats from the tensor's base
 * (forward: A = w, B = x; backward-data, stride 1 only: A = the group-wise
 * transposed filter copy [g][c][m][kh][kw], or w itself for a 1x1 window
 * without padding, B = dy; backward-weight: A = dy, B = x); valid = 0 means the
 * element is a zero-padding tap. */
int cg_debug_conv_operand(const cg_conv_desc *d, int pass, int operand, unsigned row, unsigned k,
                          unsigned group, long long *elem_offset, int *valid);

/* Per-launch timing for benchmarks: while enabled, every matrix-core (implicit
 * GEMM) launch and every gradient-aggregation launch is bracketed by two HIP
 * events on its own stream and logged with its algorithmic work (flops =
 * 2*M*N*K*groups for a contraction; bytes = (4K+20)*n for the update).
 * cg_profile_enable(1) starts a fresh log, cg_profile_enable(0) stops logging;
 * cg_profile_get waits for record i to finish and returns its duration. */
typedef struct {
    char kernel[64];   /* kernel template instance, as a profiler prints it (abridged) */
    char pass[32];     /* conv_fwd, conv_bwd_data, conv_bwd_weight, fc_fwd, ..., reduce_sgd */
    int layer;         /* layer index inside cg_train_step, -1 for stand-alone calls */
    float ms;
    double flops, bytes;
} cg_profile_record;
int cg_profile_enable(int on);
int cg_profile_count(void);
int cg_profile_get(int i, cg_profile_record *out);

/* How nets created from now on run an LRN layer whose only consumer is a
 * max-pool.  mode 0: two kernels per direction.  mode 1 (the default): forward
 * as one kernel, the LRN's output is not materialised (cg_net_layer_fused
 * reports 1 for that LRN layer).  mode 3: backward as one kernel as well,
 * neither the LRN's output nor the gradient with respect to it exists
 * (reports 3); built and tested, slower than the two kernels it replaces.
 * Process-wide. */
int cg_debug_fuse_lrn_pool(int mode);

/* Measurement aid: kernels launched by the library in this process so far
 * (every entry point, every stream). */
unsigned long long cg_debug_launch_count(void);

/* Measurement aid: the streaming rates the memory system reaches with the
 * simplest possible kernels, to quote beside the published peak.  mode 0:
 * dst[i] = src[i]; mode 1: read src only (dst receives one float4 if the sum
 * happens to hit a sentinel, i.e. practically never); mode 2: fill dst;
 * mode 3: dst[i] = src[i] + 3 * src2[i].  16-byte aligned device pointers,
 * bytes % 16 == 0; src2 is needed for mode 3 only.  All accesses non-temporal. */
int cg_debug_stream(void *dst, const void *src, const void *src2, size_t bytes, int mode, void *stream);

/* Measurement aid: the rate the fp32 matrix pipeline reaches with nothing else
 * to do.  `blocks` blocks of four waves; every wave issues `iters` times four
 * independent v_mfma_f32_32x32x2_f32 (no loads, no LDS), i.e. 2*32*32*2 *
 * 16 * iters * blocks floating-point operations in all, and then stores its
 * accumulators' sum: `out` receives 256 * blocks floats (16-byte aligned
 * device pointer; the values mean nothing).  blocks in 1..65536, iters >= 1. */
int cg_debug_mfma_loop(float *out, int blocks, int iters, void *stream);

#ifdef __cplusplus
}
#endif
#endif
