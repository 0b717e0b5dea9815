// Reductions over the 64 lanes of a wavefront on the vector ALU (data-parallel-primitive operand modifiers inside a row of
// 16 lanes, then the gfx950 row and half swaps): every lane ends with the result.  The shuffle intrinsics go through the
// LDS crossbar instead, a round trip of its own per step.
#pragma once
#include <hip/hip_runtime.h>

namespace {

template <typename F>
__device__ __forceinline__ float wave_reduce(float x, F op) {
    auto dpp = [](float v, auto ctrl) __attribute__((always_inline)) {
        return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), decltype(ctrl)::value, 0xf, 0xf, true));
    };
    x = op(x, dpp(x, std::integral_constant<int, 0xB1>{}));    // lane ^ 1 (quad_perm 1,0,3,2)
    x = op(x, dpp(x, std::integral_constant<int, 0x4E>{}));    // lane ^ 2 (quad_perm 2,3,0,1): the quad's result in its four lanes
    x = op(x, dpp(x, std::integral_constant<int, 0x141>{}));   // mirror inside 8 lanes: the other quad
    x = op(x, dpp(x, std::integral_constant<int, 0x140>{}));   // mirror inside the row of 16: the other half row
    // (the swaps exchange rows between their two operands and return both.  Their elements are copied to scalars before the
    // bit cast: applied to an element of the returned vector the cast reads element 0 with this compiler.)
    auto r = __builtin_amdgcn_permlane16_swap(__builtin_bit_cast(unsigned, x), __builtin_bit_cast(unsigned, x), false, false);
    const unsigned r0 = r[0], r1 = r[1];
    x = op(__builtin_bit_cast(float, r0), __builtin_bit_cast(float, r1));        // the neighbouring row
    auto q = __builtin_amdgcn_permlane32_swap(__builtin_bit_cast(unsigned, x), __builtin_bit_cast(unsigned, x), false, false);
    const unsigned q0 = q[0], q1 = q[1];
    return op(__builtin_bit_cast(float, q0), __builtin_bit_cast(float, q1));     // the other half of the wavefront
}

__device__ __forceinline__ float wave_sum(float x) {
    return wave_reduce(x, [](float a, float b) { return a + b; });
}

__device__ __forceinline__ float wave_max(float x) {
    return wave_reduce(x, [](float a, float b) { return fmaxf(a, b); });
}

}  // namespace
