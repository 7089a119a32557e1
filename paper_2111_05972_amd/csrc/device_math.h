// Scalar device helpers shared by the HIP kernels: storage conversion and the exact GeLU.
#pragma once
#include <hip/hip_runtime.h>

namespace tpl {

typedef __bf16 bf16_t;

template <typename T> __device__ __forceinline__ float to_f32(T v) { return (float)v; }
template <typename T> __device__ __forceinline__ T from_f32(float v) { return (T)v; }

// gelu(u) = u * Phi(u) with the erf form of the normal CDF.
__device__ __forceinline__ float gelu_f(float u) {
    return 0.5f * u * (1.0f + erff(u * 0.70710678118654752440f));
}
// d/du gelu(u) = Phi(u) + u * phi(u)
__device__ __forceinline__ float gelu_grad_f(float u) {
    float Phi = 0.5f * (1.0f + erff(u * 0.70710678118654752440f));
    float phi = 0.39894228040143267794f * __expf(-0.5f * u * u);
    return Phi + u * phi;
}

}  // namespace tpl
