// Error strings, version and the per-thread record of the last HIP failure.
#include "cg_internal.h"

namespace cg {

static thread_local int g_last_hip_error = 0;

int hip_fail(hipError_t e)
{
    g_last_hip_error = (int)e;
    return CG_EHIP;
}

}  // namespace cg

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
