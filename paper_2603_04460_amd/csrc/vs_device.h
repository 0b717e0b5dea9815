// Device-side helpers shared by the attention and aggregation kernels: bitmaps built from index lists.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

// 64 bits of a bitmap starting at bit `bitpos` (the bitmap must have two readable words after the first one touched)
__device__ __forceinline__ uint64_t window64(const uint32_t* __restrict__ bm, int bitpos) {
    const int w = bitpos >> 5, sh = bitpos & 31;
    const uint32_t a = bm[w], b = bm[w + 1], c = bm[w + 2];
    uint64_t r = ((static_cast<uint64_t>(b) << 32) | a) >> sh;
    if (sh) r |= static_cast<uint64_t>(c) << (64 - sh);
    return r;
}

// ---- index lists -> bitmaps ----
__global__ void fill_zero_kernel(uint32_t* p, size_t words) {
    const size_t i = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < words) p[i] = 0u;
}

// bit (e + bit_shift) of head ih's bitmap is set for every valid list entry e in [0, n)
__global__ void set_bits_kernel(const int32_t* idx, const int32_t* cnt, int cap, int n, uint32_t* bits, int words_per_head,
                                int bit_shift) {
    const int ih = blockIdx.y;
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= min(cnt[ih], cap)) return;
    const int e = idx[static_cast<size_t>(ih) * cap + t];
    if (e < 0 || e >= n) return;
    const int bit = e + bit_shift;
    atomicOr(bits + static_cast<size_t>(ih) * words_per_head + (bit >> 5), 1u << (bit & 31));
}

}  // namespace
