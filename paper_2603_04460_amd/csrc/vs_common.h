// Internal helpers shared by the translation units of libvsprefill (host side only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <mutex>
#include "vsprefill.h"

namespace vs {

void set_hip_error(hipError_t e);

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }


// Per-device one-time set-up (kernel attributes, device facts) for entry points that may be called from several
// threads and on several devices: `setup(dev)` runs once per device under a lock; its failure is reported and retried
// by the next call.
constexpr int kMaxDevices = 64;
struct PerDeviceOnce {
    std::mutex mu;
    bool done[kMaxDevices] = {};
    template <class F>
    int run(int* dev_out, F setup) {
        int dev = 0;
        const hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) {
            set_hip_error(e);
            return VS_ERR_HIP;
        }
        if (dev < 0 || dev >= kMaxDevices) return VS_ERR_UNSUPPORTED;
        if (dev_out) *dev_out = dev;
        std::lock_guard<std::mutex> lock(mu);
        if (done[dev]) return VS_OK;
        const int rc = setup(dev);
        if (rc == VS_OK) done[dev] = true;
        return rc;
    }
};

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
