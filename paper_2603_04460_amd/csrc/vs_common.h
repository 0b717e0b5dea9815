// Internal helpers shared by the translation units of libvsprefill (host side only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "vsprefill.h"

namespace vs {

void set_hip_error(hipError_t e);

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

}  // namespace vs

#define VS_HIP(call)                       \
    do {                                   \
        hipError_t e_ = (call);            \
        if (e_ != hipSuccess) {            \
            vs::set_hip_error(e_);         \
            return VS_ERR_HIP;             \
        }                                  \
    } while (0)

#define VS_LAUNCH_CHECK() VS_HIP(hipGetLastError())
