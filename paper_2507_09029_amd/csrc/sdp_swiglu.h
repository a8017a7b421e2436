// SwiGLU elementwise step and its backward, and bf16 <-> fp32 conversion (device code).
//
//   act = silu(g) * u,  silu(z) = z * s(z),  s(z) = 1 / (1 + exp(-z))
//   d act / d u = silu(g)              d act / d g = u * silu'(g),  silu'(z) = s(z) (1 + z (1 - s(z)))
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sdp {

__device__ inline float bf16_to_f32(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

// round to nearest, ties to even; NaN stays NaN (quiet)
__device__ inline uint16_t f32_to_bf16(float f) {
    uint32_t x = __float_as_uint(f);
    if ((x & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((x >> 16) | 0x0040u);
    x += 0x7FFFu + ((x >> 16) & 1u);
    return (uint16_t)(x >> 16);
}

// PRECISE selects libm-grade expf and an IEEE division (fp32 path); otherwise the hardware
// exponential and reciprocal (bf16 path, where the result is rounded to 8 bits of mantissa anyway).
template <bool PRECISE>
__device__ inline float sigmoidf(float z) {
    if (PRECISE) return 1.0f / (1.0f + expf(-z));
    return __builtin_amdgcn_rcpf(1.0f + __expf(-z));
}

template <bool PRECISE>
__device__ inline float swiglu_fwd(float g, float u) {
    return g * sigmoidf<PRECISE>(g) * u;
}

template <bool PRECISE>
__device__ inline void swiglu_bwd(float da, float g, float u, float& dg, float& du, float& act) {
    const float s = sigmoidf<PRECISE>(g);
    const float silu = g * s;
    du = da * silu;
    dg = da * u * (s * (1.0f + g * (1.0f - s)));
    act = silu * u;
}

} // namespace sdp
