// Scalar device helpers shared by the HIP kernels: storage conversion and the exact GeLU.
#pragma once
#include <hip/hip_runtime.h>

namespace tpl {

typedef __bf16 bf16_t;

template <typename T> __device__ __forceinline__ float to_f32(T v) { return (float)v; }
template <typename T> __device__ __forceinline__ T from_f32(float v) { return (T)v; }

// The exact (erf) GeLU: gelu(u) = u * Phi(u), Phi the normal CDF, Phi(u) = 0.5 * (1 + erf(u / sqrt 2)).
// Phi is evaluated through the lower tail, Phi(-|u|) = 0.5 * erfc(|u| / sqrt 2), with the rational
// approximation erfc(x) = t (a1 + t (a2 + t (a3 + t (a4 + t a5)))) exp(-x^2), t = 1 / (1 + p x)
// (Abramowitz & Stegun 7.1.26, absolute error below 1.5e-7, i.e. float rounding level for values in [0, 1]);
// no cancellation for negative u, one exp and one reciprocal per element, and the same exp(-u^2 / 2)
// serves the density in the derivative.  About a third of the instructions of the library erff.
struct PhiParts { float Phi, e; };   // Phi(u) and exp(-u^2 / 2)
__device__ __forceinline__ PhiParts normal_cdf(float u) {
    const float x = fabsf(u) * 0.70710678118654752440f;
    const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, x, 1.0f));
    const float e = __expf(-x * x);
    float q = fmaf(1.061405429f, t, -1.453152027f);
    q = fmaf(q, t, 1.421413741f);
    q = fmaf(q, t, -0.284496736f);
    q = fmaf(q, t, 0.254829592f);
    q = 0.5f * q * t * e;
    return PhiParts{u < 0.0f ? q : 1.0f - q, e};
}
__device__ __forceinline__ float gelu_f(float u) { return u * normal_cdf(u).Phi; }
// d/du gelu(u) = Phi(u) + u * phi(u), phi the normal density
__device__ __forceinline__ float gelu_grad_f(float u) {
    const PhiParts c = normal_cdf(u);
    return fmaf(u * 0.39894228040143267794f, c.e, c.Phi);
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
