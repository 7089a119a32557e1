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

// Eight consecutive elements <-> eight floats with 16-byte accesses (pointer 16-byte aligned).
__device__ __forceinline__ void load8(const float* p, float (&v)[8]) {
    float4 a = reinterpret_cast<const float4*>(p)[0], b = reinterpret_cast<const float4*>(p)[1];
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
__device__ __forceinline__ void load8(const bf16_t* p, float (&v)[8]) {
    uint4 u = *reinterpret_cast<const uint4*>(p);
    const unsigned w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        v[2 * i] = __uint_as_float(w[i] << 16);
        v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
}
__device__ __forceinline__ void store8(float* p, const float (&v)[8]) {
    reinterpret_cast<float4*>(p)[0] = make_float4(v[0], v[1], v[2], v[3]);
    reinterpret_cast<float4*>(p)[1] = make_float4(v[4], v[5], v[6], v[7]);
}
__device__ __forceinline__ void store8(bf16_t* p, const float (&v)[8]) {
    unsigned u[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        bf16_t lo = (bf16_t)v[2 * i], hi = (bf16_t)v[2 * i + 1];
        u[i] = (unsigned)__builtin_bit_cast(unsigned short, lo) |
               ((unsigned)__builtin_bit_cast(unsigned short, hi) << 16);
    }
    *reinterpret_cast<uint4*>(p) = make_uint4(u[0], u[1], u[2], u[3]);
}

}  // namespace tpl
