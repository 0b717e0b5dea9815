// Error reporting and version string of libvsprefill.
#include "vs_common.h"

namespace {
thread_local int g_last_hip_error = 0;
}

namespace vs {
void set_hip_error(hipError_t e) { g_last_hip_error = static_cast<int>(e); }
}  // namespace vs

namespace {

// report[h]: 0 when head h's list is usable as it is; else a bit-or of VS_LIST_* flags
__global__ void validate_lists_kernel(const int32_t* idx, const int32_t* cnt, int cap, int n, int32_t* report) {
    const int h = blockIdx.x;
    const int c = cnt[h];
    int bad = 0;
    if (c < 0 || c > cap) bad |= VS_LIST_BAD_COUNT;
    const int m = c < 0 ? 0 : (c > cap ? cap : c);
    const int32_t* list = idx + static_cast<size_t>(h) * cap;
    for (int t = threadIdx.x; t < m; t += blockDim.x) {
        const int e = list[t];
        if (e < 0 || e >= n) bad |= VS_LIST_OUT_OF_RANGE;
        if (t > 0 && list[t - 1] >= e) bad |= VS_LIST_NOT_ASCENDING;
    }
    __shared__ int any;
    if (threadIdx.x == 0) any = 0;
    __syncthreads();
    if (bad) atomicOr(&any, bad);
    __syncthreads();
    if (threadIdx.x == 0) report[h] = any;
}

}  // namespace

extern "C" {

int vs_validate_lists(const int32_t* idx, const int32_t* cnt, int cap, int heads, int64_t n, int32_t* report, void* stream) {
    if (!idx || !cnt || !report || cap <= 0 || heads <= 0 || n <= 0) return VS_ERR_INVALID_ARG;
    if (n > VS_MAX_SEQ) return VS_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(validate_lists_kernel, dim3(heads), dim3(256), 0, static_cast<hipStream_t>(stream), idx, cnt, cap,
                       static_cast<int>(n), report);
    VS_LAUNCH_CHECK();
    return VS_OK;
}

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
