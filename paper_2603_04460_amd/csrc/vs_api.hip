// Error reporting and version string of libvsprefill.
#include "vs_common.h"

namespace {
thread_local int g_last_hip_error = 0;
}

namespace vs {
void set_hip_error(hipError_t e) { g_last_hip_error = static_cast<int>(e); }
}  // namespace vs

extern "C" {

const char* vs_strerror(int status) {
    switch (status) {
        case VS_OK: return "ok";
        case VS_ERR_INVALID_ARG: return "invalid argument";
        case VS_ERR_UNSUPPORTED: return "unsupported shape or mode";
        case VS_ERR_WORKSPACE: return "workspace missing or too small";
        case VS_ERR_CAPACITY: return "index list capacity too small for the forced entries";
        case VS_ERR_HIP: return "HIP runtime error (see vs_last_hip_error)";
        case VS_ERR_STATIC_LIMIT: return "sizes exceed the library's fixed scratch array (use the workspace entry point)";
        default: return "unknown status";
    }
}

int vs_last_hip_error(void) { return g_last_hip_error; }

const char* vs_version(void) { return "vsprefill-gfx950 0.1"; }

}  // extern "C"
