// Error reporting and version entry points of libmoegps.
#include "common.h"

namespace moegps {
static thread_local int g_last_hip_error = 0;
void set_last_hip_error(hipError_t e) { g_last_hip_error = (int)e; }
}  // namespace moegps

extern "C" const char* moe_strerror(int code) {
    switch (code) {
        case MOE_OK: return "ok";
        case MOE_ERR_INVALID_ARG: return "invalid argument";
        case MOE_ERR_UNSUPPORTED: return "shape or dtype not supported by this library";
        case MOE_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
        case MOE_ERR_HIP: return "HIP runtime error (see moe_last_hip_error)";
        default: return "unknown error code";
    }
}

extern "C" int moe_last_hip_error(void) { return moegps::g_last_hip_error; }

extern "C" int moe_abi_version(void) { return 1; }
