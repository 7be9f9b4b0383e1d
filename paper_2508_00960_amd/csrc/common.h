// Scalar helpers shared by the kernels: storage types, activations.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace phantom {

typedef __bf16 bf16_t;

enum { ACT_IDENTITY = 0, ACT_RELU = 1, ACT_GELU = 2 };

template <typename T> __device__ __forceinline__ float to_f32(T v) { return (float)v; }
template <typename T> __device__ __forceinline__ T from_f32(float v) { return (T)v; }

// sigma(a): identity, ReLU, or GELU = a * Phi(a) in its erf form (no tanh approximation)
__device__ __forceinline__ float act_apply(int act, float a)
{
    if (act == ACT_RELU) return a > 0.f ? a : 0.f;
    if (act == ACT_GELU) return 0.5f * a * (1.f + erff(a * 0.70710678118654752f));
    return a;
}

// sigma'(a).  ReLU'(0) = 0.  GELU' = Phi(a) + a * phi(a).
__device__ __forceinline__ float act_deriv(int act, float a)
{
    if (act == ACT_RELU) return a > 0.f ? 1.f : 0.f;
    if (act == ACT_GELU) {
        float Phi = 0.5f * (1.f + erff(a * 0.70710678118654752f));
        float phi = 0.39894228040143268f * __expf(-0.5f * a * a);
        return Phi + a * phi;
    }
    return 1.f;
}

}  // namespace phantom
