// LayerNorm over the hidden dimension, forward and backward, float or bfloat16 storage with float
// arithmetic.  In the speed-optimised distribution layer normalisation is not distributed (Sec. I.1
// of the paper): every tensor-parallel rank normalises the full replicated [M, H] activation, so this
// is a plain HBM-bound row kernel.  One 256-thread workgroup holds a whole row in registers (16-byte
// accesses, up to 8 chunks of 8 elements per thread: H <= 16384), so every tensor is read or written
// exactly once:
//   forward : reads a (and b), writes z = a + b (optional) and y          -> up to 4 M H elements
//   backward: reads dy and z, writes dz; per-workgroup column partials of dgamma, dbeta are then
//             summed in workgroup order by a second small kernel (fixed order: deterministic).
#include <hip/hip_runtime.h>

#include "device_math.h"
#include "kernels.h"

namespace tpl {

constexpr int LN_THREADS = 256;
constexpr int LN_MAX_BLOCKS = 256;     // backward: rows are strided over this many workgroups

// Sum over the workgroup, same value returned to every thread; fixed combination order.
__device__ __forceinline__ float block_sum(float v, float* red) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    const int w = threadIdx.x >> 6;
    __syncthreads();                   // red may still be read from the previous reduction
    if ((threadIdx.x & 63) == 0) red[w] = v;
    __syncthreads();
    return ((red[0] + red[1]) + red[2]) + red[3];
}

template <typename T, int MAXC>
__global__ __launch_bounds__(LN_THREADS) void ln_fwd_kernel(int64_t M, int64_t H, const T* __restrict__ a,
                                                            const T* __restrict__ b,
                                                            const T* __restrict__ gamma,
                                                            const T* __restrict__ beta, float eps,
                                                            T* __restrict__ z, T* __restrict__ y,
                                                            float* __restrict__ mean,
                                                            float* __restrict__ rstd) {
    __shared__ float red[4];
    const int t = threadIdx.x;
    const float inv_h = 1.0f / (float)H;
    for (int64_t row = blockIdx.x; row < M; row += gridDim.x) {
        float v[MAXC][8];
        float s = 0.0f;
#pragma unroll
        for (int i = 0; i < MAXC; ++i) {
            const int64_t col = ((int64_t)t + LN_THREADS * i) * 8;
            if (col < H) {
                load8(a + row * H + col, v[i]);
                if (b) {
                    float w[8];
                    load8(b + row * H + col, w);
#pragma unroll
                    for (int e = 0; e < 8; ++e) v[i][e] += w[e];
                }
                if (z) store8(z + row * H + col, v[i]);
#pragma unroll
                for (int e = 0; e < 8; ++e) s += v[i][e];
            }
        }
        const float mu = block_sum(s, red) * inv_h;
        float q = 0.0f;
#pragma unroll
        for (int i = 0; i < MAXC; ++i) {
            const int64_t col = ((int64_t)t + LN_THREADS * i) * 8;
            if (col < H) {
#pragma unroll
                for (int e = 0; e < 8; ++e) { v[i][e] -= mu; q = fmaf(v[i][e], v[i][e], q); }
            }
        }
        const float rs = 1.0f / sqrtf(block_sum(q, red) * inv_h + eps);
#pragma unroll
        for (int i = 0; i < MAXC; ++i) {
            const int64_t col = ((int64_t)t + LN_THREADS * i) * 8;
            if (col < H) {
                float g[8], bt[8];
                load8(gamma + col, g);
                load8(beta + col, bt);
#pragma unroll
                for (int e = 0; e < 8; ++e) v[i][e] = fmaf(v[i][e] * rs, g[e], bt[e]);
                store8(y + row * H + col, v[i]);
            }
        }
        if (t == 0) { mean[row] = mu; rstd[row] = rs; }
    }
}

template <typename T, int MAXC>
__global__ __launch_bounds__(LN_THREADS) void ln_bwd_kernel(int64_t M, int64_t H, const T* __restrict__ dy,
                                                            const T* __restrict__ z,
                                                            const float* __restrict__ mean,
                                                            const float* __restrict__ rstd,
                                                            const T* __restrict__ gamma,
                                                            T* __restrict__ dz,
                                                            float* __restrict__ partials) {
    __shared__ float red[4];
    const int t = threadIdx.x;
    const float inv_h = 1.0f / (float)H;
    float gam[MAXC][8], dgam[MAXC][8], dbet[MAXC][8];
#pragma unroll
    for (int i = 0; i < MAXC; ++i) {
        const int64_t col = ((int64_t)t + LN_THREADS * i) * 8;
#pragma unroll
        for (int e = 0; e < 8; ++e) { gam[i][e] = 0.0f; dgam[i][e] = 0.0f; dbet[i][e] = 0.0f; }
        if (col < H) load8(gamma + col, gam[i]);
    }
    for (int64_t row = blockIdx.x; row < M; row += gridDim.x) {
        const float mu = mean[row], rs = rstd[row];
        float g[MAXC][8], zh[MAXC][8];
        float s1 = 0.0f, s2 = 0.0f;
#pragma unroll
        for (int i = 0; i < MAXC; ++i) {
            const int64_t col = ((int64_t)t + LN_THREADS * i) * 8;
            if (col < H) {
                load8(dy + row * H + col, g[i]);
                load8(z + row * H + col, zh[i]);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    zh[i][e] = (zh[i][e] - mu) * rs;
                    dbet[i][e] += g[i][e];
                    dgam[i][e] = fmaf(g[i][e], zh[i][e], dgam[i][e]);
                    g[i][e] *= gam[i][e];
                    s1 += g[i][e];
                    s2 = fmaf(g[i][e], zh[i][e], s2);
                }
            }
        }
        const float c1 = block_sum(s1, red) * inv_h;
        const float c2 = block_sum(s2, red) * inv_h;
#pragma unroll
        for (int i = 0; i < MAXC; ++i) {
            const int64_t col = ((int64_t)t + LN_THREADS * i) * 8;
            if (col < H) {
#pragma unroll
                for (int e = 0; e < 8; ++e) g[i][e] = (g[i][e] - c1 - zh[i][e] * c2) * rs;
                store8(dz + row * H + col, g[i]);
            }
        }
    }
    // this workgroup's share of the column sums: partials[block][0][:] = dgamma, [block][1][:] = dbeta
    float* pg = partials + (int64_t)blockIdx.x * 2 * H;
#pragma unroll
    for (int i = 0; i < MAXC; ++i) {
        const int64_t col = ((int64_t)t + LN_THREADS * i) * 8;
        if (col < H) { store8(pg + col, dgam[i]); store8(pg + H + col, dbet[i]); }
    }
}

bool ln_supported(int64_t H) { return H > 0 && H % 8 == 0 && H <= 8 * 8 * LN_THREADS; }
int64_t ln_partial_rows(int64_t M) { return M < LN_MAX_BLOCKS ? M : LN_MAX_BLOCKS; }

template <typename T, int MAXC>
static hipError_t fwd_t(const LnArgs& a) {
    const unsigned grid = (unsigned)(a.M < 65535 * 16 ? a.M : 65535 * 16);
    hipLaunchKernelGGL((ln_fwd_kernel<T, MAXC>), dim3(grid), dim3(LN_THREADS), 0, a.stream, a.M, a.H,
                       (const T*)a.a, (const T*)a.b, (const T*)a.gamma, (const T*)a.beta, a.eps, (T*)a.z,
                       (T*)a.y, a.mean, a.rstd);
    return hipGetLastError();
}
template <typename T, int MAXC>
static hipError_t bwd_t(const LnArgs& a) {
    const int64_t blocks = ln_partial_rows(a.M);
    hipLaunchKernelGGL((ln_bwd_kernel<T, MAXC>), dim3((unsigned)blocks), dim3(LN_THREADS), 0, a.stream, a.M,
                       a.H, (const T*)a.dy, (const T*)a.z, a.mean, a.rstd, (const T*)a.gamma, (T*)a.dz,
                       a.partials);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    // partial rows are [block][2][H]: summing over blocks with row length 2H yields dgamma | dbeta
    // into a [2H] vector; gamma and beta gradients are separate buffers, so two calls with stride 2H.
    e = sum_partials_strided(a.dtype, blocks, a.H, a.partials, 2 * a.H, a.dgamma, a.stream);
    if (e != hipSuccess) return e;
    return sum_partials_strided(a.dtype, blocks, a.H, a.partials + a.H, 2 * a.H, a.dbeta, a.stream);
}

template <typename T>
static hipError_t dispatch(const LnArgs& a, bool bwd) {
    const int64_t chunks = (a.H / 8 + LN_THREADS - 1) / LN_THREADS;
    if (chunks <= 2) return bwd ? bwd_t<T, 2>(a) : fwd_t<T, 2>(a);
    if (chunks <= 4) return bwd ? bwd_t<T, 4>(a) : fwd_t<T, 4>(a);
    return bwd ? bwd_t<T, 8>(a) : fwd_t<T, 8>(a);
}

hipError_t ln_fwd(const LnArgs& a) { return a.dtype == F32 ? dispatch<float>(a, false) : dispatch<bf16_t>(a, false); }
hipError_t ln_bwd(const LnArgs& a) { return a.dtype == F32 ? dispatch<float>(a, true) : dispatch<bf16_t>(a, true); }

}  // namespace tpl
