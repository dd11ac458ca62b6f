// GELU and its derivative in fp32 (section 3, nonlinear activations), shared by the elementwise
// kernels and by the product kernels' result paths that apply them.
#pragma once
#include <hip/hip_runtime.h>

#include "nntile_mi.h"

namespace nnt {

// tanh form through the logistic function: 0.5 (1 + tanh u) = 1 / (1 + e^(-2u)), so
//   gelu(x) = x r,   r = 1 / (1 + e),   e = 2^(-2 u log2(e)),   u = sqrt(2/pi) (x + 0.044715 x^3),
// with the hardware's 2^x and reciprocal (about 1 ulp each; the library tanh costs some thirty
// instructions).  The exponent is clamped so that e stays finite for very negative x (r ~ 1e-24 there).
__device__ __forceinline__ float gelu_tanh_e(float x) {
    constexpr float k = 2.302208198144325f;             // 2 sqrt(2/pi) log2(e)
    const float z = -x * fmaf(0.044715f * k, x * x, k);
    return __builtin_amdgcn_exp2f(fminf(z, 80.f));
}

__device__ __forceinline__ float gelu_f(float x, int variant) {
    if (variant == NNT_GELU_TANH) return x * __builtin_amdgcn_rcpf(1.f + gelu_tanh_e(x));
    return 0.5f * x * (1.f + erff(x * 0.7071067811865476f));
}
__device__ __forceinline__ float gelu_grad_f(float x, int variant) {
    if (variant == NNT_GELU_TANH) {
        // d/dx (x r) = r + x r (1 - r) 2 u',  1 - r = e r,  u' = sqrt(2/pi) (1 + 3 * 0.044715 x^2)
        const float e = gelu_tanh_e(x);
        const float r = __builtin_amdgcn_rcpf(1.f + e);
        const float du2 = fmaf(2.f * 0.7978845608028654f * 3.f * 0.044715f, x * x, 2.f * 0.7978845608028654f);
        return fmaf(x * (e * r * r), du2, r);
    }
    return 0.5f * (1.f + erff(x * 0.7071067811865476f)) + x * 0.3989422804014327f * expf(-0.5f * x * x);
}

}  // namespace nnt
