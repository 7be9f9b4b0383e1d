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

// GELU and its derivative together, for bf16 outputs: erf by the five-term rational formula of Abramowitz &
// Stegun 7.1.26 (absolute error of erf below 1.5e-7, far under a bf16 rounding step), whose exp(-z^2) with
// z = a / sqrt(2) is the same exponential that phi(a) needs.  One v_exp, one v_rcp and a dozen FMAs instead of
// two library calls per element: the epilogues that evaluate it run on every element of a layer's output
// with nothing left to overlap them with.
__device__ __forceinline__ void gelu_both(float a, float &y, float &d)
{
    const float z = fabsf(a) * 0.70710678118654752f;
    const float t = __frcp_rn(1.f + 0.3275911f * z);
    const float e = __expf(-0.5f * a * a);
    const float poly = t * (0.254829592f + t * (-0.284496736f + t * (1.421413741f + t * (-1.453152027f + t * 1.061405429f))));
    const float h = 0.5f * poly * e;                   // = (1 - erf(z)) / 2 = Phi(-|a|)
    const float Phi = a < 0.f ? h : 1.f - h;
    y = a * Phi;
    d = Phi + a * (0.39894228040143268f * e);
}

}  // namespace phantom
