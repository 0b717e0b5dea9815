// Rotary embedding on [heads, n, 128] bf16, in place (Appendix, "RoPE Matrix Representation").
//
// One thread owns one (position, plane): the angle position * base^(-2p/128) and its sine / cosine
// are evaluated once in fp64 (positions reach 2^20, far beyond what fp32 angles resolve) and reused
// for every head.  The rotated pair is rounded once from fp64 to bf16, nearest even.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "vs_common.h"

namespace {

__device__ __forceinline__ double bf16_to_f64(uint16_t b) { return static_cast<double>(__uint_as_float(static_cast<uint32_t>(b) << 16)); }

// fp64 -> bf16 with a single rounding: truncate to fp32, fold the lost bits into a sticky bit
// (round to odd), then round the fp32 to nearest-even bf16.
__device__ __forceinline__ uint16_t f64_to_bf16(double x) {
    float f = __double2float_rz(x);
    uint32_t u = __float_as_uint(f);
    if (static_cast<double>(f) != x) u |= 1u;
    u += 0x7fffu + ((u >> 16) & 1u);
    return static_cast<uint16_t>(u >> 16);
}

__global__ __launch_bounds__(256) void rope_kernel(uint16_t* x, int heads, long long n, long long pos0, double theta_base,
                                                   int pairing) {
    const long long gid = static_cast<long long>(blockIdx.x) * blockDim.x + threadIdx.x;
    const long long t = gid >> 6;
    const int p = static_cast<int>(gid & 63);
    if (t >= n) return;
    const double theta = pow(theta_base, -2.0 * p / 128.0);
    const double phi = static_cast<double>(pos0 + t) * theta;
    double s, c;
    sincos(phi, &s, &c);
    const int ia = pairing == 0 ? 2 * p : p;
    const int ib = pairing == 0 ? 2 * p + 1 : p + 64;
    for (int h = 0; h < heads; ++h) {
        uint16_t* row = x + (static_cast<long long>(h) * n + t) * 128;
        const double xa = bf16_to_f64(row[ia]), xb = bf16_to_f64(row[ib]);
        row[ia] = f64_to_bf16(xa * c - xb * s);
        row[ib] = f64_to_bf16(xa * s + xb * c);
    }
}

}  // namespace

extern "C" int vs_rope_apply(void* x_bf16, int heads, int64_t n, int64_t pos0, double theta_base, int pairing,
                             void* stream) {
    if (!x_bf16 || !vs::aligned16(x_bf16) || heads <= 0 || n <= 0 || pos0 < 0) return VS_ERR_INVALID_ARG;
    if (!(theta_base > 1.0) || !isfinite(theta_base)) return VS_ERR_INVALID_ARG;
    if (pairing != 0 && pairing != 1) return VS_ERR_INVALID_ARG;
    if (n > VS_MAX_SEQ) return VS_ERR_UNSUPPORTED;
    const long long threads = static_cast<long long>(n) * 64;
    hipLaunchKernelGGL(rope_kernel, dim3(static_cast<unsigned>((threads + 255) / 256)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), static_cast<uint16_t*>(x_bf16), heads, static_cast<long long>(n),
                       static_cast<long long>(pos0), theta_base, pairing);
    VS_LAUNCH_CHECK();
    return VS_OK;
}
