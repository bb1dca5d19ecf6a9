// Error strings, version and the per-thread record of the last HIP failure.
#include <atomic>
#include <cstdio>
#include <mutex>
#include <vector>
#include "cg_internal.h"

namespace cg {

static thread_local int g_last_hip_error = 0;

static std::atomic<unsigned long long> g_launches{0};
void note_launch() { g_launches.fetch_add(1, std::memory_order_relaxed); }

int hip_fail(hipError_t e)
{
    g_last_hip_error = (int)e;
    return CG_EHIP;
}

// ---- per-launch timing ---------------------------------------------------------------------------
namespace {
struct ProfRec {
    hipEvent_t e0 = nullptr, e1 = nullptr;
    char kernel[64];
    char pass[32];
    int layer;
    double flops, bytes;
    bool open;
};
std::mutex g_prof_mu;
std::vector<ProfRec> g_prof;      // records of the current session (events are reused across sessions)
size_t g_prof_used = 0;
std::atomic<bool> g_prof_enabled{false};
thread_local const char *g_pass = "";
thread_local int g_layer = -1;
}  // namespace

ProfTag::ProfTag(const char *pass, int layer) : prev_pass(g_pass), prev_layer(g_layer)
{
    g_pass = pass;
    if (layer >= 0 || g_layer < 0) g_layer = layer;
}
ProfTag::~ProfTag() { g_pass = prev_pass; g_layer = prev_layer; }

bool prof_on() { return g_prof_enabled; }

int prof_begin(const char *kernel, double flops, double bytes, hipStream_t s)
{
    if (!g_prof_enabled) return -1;
    std::lock_guard<std::mutex> lk(g_prof_mu);
    if (g_prof_used == g_prof.size()) {
        ProfRec r;
        if (hipEventCreate(&r.e0) != hipSuccess || hipEventCreate(&r.e1) != hipSuccess) return -1;
        g_prof.push_back(r);
    }
    ProfRec &r = g_prof[g_prof_used];
    snprintf(r.kernel, sizeof r.kernel, "%s", kernel);
    snprintf(r.pass, sizeof r.pass, "%s", g_pass);
    r.layer = g_layer; r.flops = flops; r.bytes = bytes; r.open = true;
    if (hipEventRecord(r.e0, s) != hipSuccess) return -1;
    return (int)g_prof_used++;
}

void prof_end(int rec, hipStream_t s)
{
    if (rec < 0) return;
    std::lock_guard<std::mutex> lk(g_prof_mu);
    if ((size_t)rec < g_prof_used && hipEventRecord(g_prof[rec].e1, s) == hipSuccess) g_prof[rec].open = false;
}

}  // namespace cg

extern "C" int cg_profile_enable(int on)
{
    std::lock_guard<std::mutex> lk(cg::g_prof_mu);
    cg::g_prof_enabled = on != 0;
    if (on) cg::g_prof_used = 0;
    return CG_OK;
}

extern "C" int cg_profile_count(void)
{
    std::lock_guard<std::mutex> lk(cg::g_prof_mu);
    return (int)cg::g_prof_used;
}

extern "C" int cg_profile_get(int i, cg_profile_record *out)
{
    if (!out) return CG_EINVAL;
    std::lock_guard<std::mutex> lk(cg::g_prof_mu);
    if (i < 0 || (size_t)i >= cg::g_prof_used || cg::g_prof[i].open) return CG_EINVAL;
    const cg::ProfRec &r = cg::g_prof[i];
    CG_HIP_TRY(hipEventSynchronize(r.e1));
    float ms = 0.f;
    CG_HIP_TRY(hipEventElapsedTime(&ms, r.e0, r.e1));
    snprintf(out->kernel, sizeof out->kernel, "%s", r.kernel);
    snprintf(out->pass, sizeof out->pass, "%s", r.pass);
    out->layer = r.layer; out->ms = ms; out->flops = r.flops; out->bytes = r.bytes;
    return CG_OK;
}

// A plain copy of known size: the yardstick that hardware-counter readings (bytes fetched from and
// written to HBM per dispatch) of the other kernels are scaled by.
namespace cg {
__global__ __launch_bounds__(256) void debug_copy_kernel(float4 *__restrict__ dst, const float4 *__restrict__ src, size_t n4)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n4) dst[i] = src[i];
}
}  // namespace cg

extern "C" int cg_debug_copy(void *dst, const void *src, size_t bytes, void *stream)
{
    if (!dst || !src || !cg::aligned16(dst) || !cg::aligned16(src) || bytes % 16) return CG_EINVAL;
    if (bytes == 0) return CG_OK;
    const size_t n4 = bytes / 16;
    if ((n4 + 255) / 256 >= (1ull << 31)) return CG_EUNSUPPORTED;
    hipLaunchKernelGGL(cg::debug_copy_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), static_cast<float4 *>(dst), static_cast<const float4 *>(src), n4);
    CG_HIP_TRY(hipGetLastError());
    return CG_OK;
}

// The simplest streaming kernels, for the rates the memory system reaches (quoted beside the
// published peak): one float4 per thread, non-temporal, one short-lived block per 4 KB.
namespace cg {
typedef float f4nt __attribute__((ext_vector_type(4)));
template <int MODE>
__global__ __launch_bounds__(256) void debug_stream_kernel(f4nt *__restrict__ dst, const f4nt *__restrict__ src,
                                                           const f4nt *__restrict__ src2, size_t n4)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n4) return;
    if (MODE == 0) {
        __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
    } else if (MODE == 1) {
        const f4nt a = __builtin_nontemporal_load(src + i);
        if (a.x + a.y + a.z + a.w == 123.456f) dst[0] = a;
    } else if (MODE == 2) {
        __builtin_nontemporal_store(f4nt{1.f, 2.f, 3.f, 4.f}, dst + i);
    } else {
        __builtin_nontemporal_store(__builtin_nontemporal_load(src + i) + 3.f * __builtin_nontemporal_load(src2 + i), dst + i);
    }
}
}  // namespace cg

extern "C" int cg_debug_stream(void *dst, const void *src, const void *src2, size_t bytes, int mode, void *stream)
{
    if (mode < 0 || mode > 3 || !dst || !cg::aligned16(dst) || bytes % 16) return CG_EINVAL;
    if (mode != 2 && (!src || !cg::aligned16(src))) return CG_EINVAL;
    if (mode == 3 && (!src2 || !cg::aligned16(src2))) return CG_EINVAL;
    if (bytes == 0) return CG_OK;
    const size_t n4 = bytes / 16;
    if ((n4 + 255) / 256 >= (1ull << 31)) return CG_EUNSUPPORTED;
    const dim3 grid((unsigned)((n4 + 255) / 256));
    hipStream_t s = static_cast<hipStream_t>(stream);
    cg::f4nt *d = static_cast<cg::f4nt *>(dst);
    const cg::f4nt *a = static_cast<const cg::f4nt *>(src), *b = static_cast<const cg::f4nt *>(src2);
    if (mode == 0) hipLaunchKernelGGL(cg::debug_stream_kernel<0>, grid, dim3(256), 0, s, d, a, b, n4);
    else if (mode == 1) hipLaunchKernelGGL(cg::debug_stream_kernel<1>, grid, dim3(256), 0, s, d, a, b, n4);
    else if (mode == 2) hipLaunchKernelGGL(cg::debug_stream_kernel<2>, grid, dim3(256), 0, s, d, a, b, n4);
    else hipLaunchKernelGGL(cg::debug_stream_kernel<3>, grid, dim3(256), 0, s, d, a, b, n4);
    CG_HIP_TRY(hipGetLastError());
    return CG_OK;
}

// The fp32 matrix pipeline alone: four independent accumulators a wave, so that an instruction
// never waits for the one before it; operands are lane-dependent numbers the compiler cannot fold.
namespace cg {
typedef float v16f_dbg __attribute__((ext_vector_type(16)));
__global__ __launch_bounds__(256) void debug_mfma_kernel(float *__restrict__ out, int iters)
{
    v16f_dbg a0 = {}, a1 = {}, a2 = {}, a3 = {};
    const float x = 1.f + (float)threadIdx.x * 0x1p-10f, y = 1.f - (float)(threadIdx.x & 31) * 0x1p-12f;
    for (int i = 0; i < iters; ++i) {
        a0 = __builtin_amdgcn_mfma_f32_32x32x2f32(x, y, a0, 0, 0, 0);
        a1 = __builtin_amdgcn_mfma_f32_32x32x2f32(y, x, a1, 0, 0, 0);
        a2 = __builtin_amdgcn_mfma_f32_32x32x2f32(x, x, a2, 0, 0, 0);
        a3 = __builtin_amdgcn_mfma_f32_32x32x2f32(y, y, a3, 0, 0, 0);
    }
    float sum = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) sum += a0[r] + a1[r] + a2[r] + a3[r];
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = sum;
}
}  // namespace cg

extern "C" int cg_debug_mfma_loop(float *out, int blocks, int iters, void *stream)
{
    if (!out || !cg::aligned16(out) || blocks < 1 || blocks > 65536 || iters < 1) return CG_EINVAL;
    hipLaunchKernelGGL(cg::debug_mfma_kernel, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(stream), out, iters);
    CG_HIP_TRY(hipGetLastError());
    return CG_OK;
}

extern "C" unsigned long long cg_debug_launch_count(void)
{
    return cg::g_launches.load(std::memory_order_relaxed);
}

extern "C" const char *cg_strerror(int code)
{
    switch (code) {
    case CG_OK: return "ok";
    case CG_EINVAL: return "invalid argument (null or misaligned pointer, bad descriptor)";
    case CG_ENOSPC: return "workspace too small";
    case CG_EUNSUPPORTED: return "valid request outside what the kernels cover";
    case CG_EHIP: return "HIP runtime error";
    default: return "unknown error code";
    }
}

extern "C" const char *cg_version(void) { return "cg 0.1 (gfx950)"; }

extern "C" int cg_last_hip_error(void) { return cg::g_last_hip_error; }
