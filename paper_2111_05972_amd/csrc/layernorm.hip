// LayerNorm over the hidden dimension, forward and backward, float or bfloat16 storage with float
// arithmetic.  In the speed-optimised distribution layer normalisation is not distributed (Sec. I.1
// of the paper): every tensor-parallel rank normalises the full replicated [M, H] activation, so this
// is a plain HBM-bound row kernel.  One 256-thread workgroup holds a whole row in registers (16-byte
// accesses, up to 8 chunks of 8 elements per thread: H <= 16384), so every tensor is read or written
// exactly once:
//   forward : reads a (and b), writes z = a + b (optional) and y          -> up to 4 M H elements
//   backward: a row pass reads dy, z for the two per-row means; a tile pass (32 rows x 512 columns per
//             workgroup) reads dy, z again (served by the infinity cache), writes dz and per-slab column
//             partials of dgamma, dbeta, which a small kernel sums in slab order (deterministic).
#include <hip/hip_runtime.h>

#include "device_math.h"
#include "kernels.h"

namespace tpl {

constexpr int LN_THREADS = 256;

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

// Backward, pass 1: per-row means c1 = mean_H(dy*gamma), c2 = mean_H(dy*gamma*zh) (one workgroup per row).
template <typename T, int MAXC>
__global__ __launch_bounds__(LN_THREADS) void ln_bwd_rowstat_kernel(int64_t M, int64_t H,
                                                                    const T* __restrict__ dy,
                                                                    const T* __restrict__ z,
                                                                    const float* __restrict__ mean,
                                                                    const float* __restrict__ rstd,
                                                                    const T* __restrict__ gamma,
                                                                    float* __restrict__ c12) {
    __shared__ float red[4];
    const int t = threadIdx.x;
    const float inv_h = 1.0f / (float)H;
    for (int64_t row = blockIdx.x; row < M; row += gridDim.x) {
        const float mu = mean[row], rs = rstd[row];
        float s1 = 0.0f, s2 = 0.0f;
#pragma unroll
        for (int i = 0; i < MAXC; ++i) {
            const int64_t col = ((int64_t)t + LN_THREADS * i) * 8;
            if (col < H) {
                float g[8], zz[8], gm[8];
                load8(dy + row * H + col, g);
                load8(z + row * H + col, zz);
                load8(gamma + col, gm);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    float gg = g[e] * gm[e];
                    s1 += gg;
                    s2 = fmaf(gg, (zz[e] - mu) * rs, s2);
                }
            }
        }
        const float c1 = block_sum(s1, red) * inv_h;
        const float c2 = block_sum(s2, red) * inv_h;
        if (t == 0) { c12[2 * row] = c1; c12[2 * row + 1] = c2; }
    }
}

// Backward, pass 2: a workgroup owns LN_SLAB rows x 512 columns (64 column groups of 8 x 4 row lanes):
// writes dz for its tile and its column partial sums of dgamma, dbeta (row lanes combined through LDS
// in lane order).  partials[slab][0][:] = dgamma, partials[slab][1][:] = dbeta.
constexpr int LN_SLAB = 32;
template <typename T>
__global__ __launch_bounds__(LN_THREADS) void ln_bwd_tile_kernel(int64_t M, int64_t H, const T* __restrict__ dy,
                                                                 const T* __restrict__ z,
                                                                 const float* __restrict__ mean,
                                                                 const float* __restrict__ rstd,
                                                                 const T* __restrict__ gamma,
                                                                 const float* __restrict__ c12,
                                                                 T* __restrict__ dz,
                                                                 float* __restrict__ partials) {
    __shared__ float red[2][4][64][8];
    const int cg = threadIdx.x & 63, rl = threadIdx.x >> 6;
    const int64_t col = ((int64_t)blockIdx.x * 64 + cg) * 8;
    const int64_t m0 = (int64_t)blockIdx.y * LN_SLAB, m1 = m0 + LN_SLAB < M ? m0 + LN_SLAB : M;
    float dgam[8] = {0, 0, 0, 0, 0, 0, 0, 0}, dbet[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (col < H) {
        float gm[8];
        load8(gamma + col, gm);
        for (int64_t row = m0 + rl; row < m1; row += 4) {
            const float mu = mean[row], rs = rstd[row], c1 = c12[2 * row], c2 = c12[2 * row + 1];
            float g[8], zz[8];
            load8(dy + row * H + col, g);
            load8(z + row * H + col, zz);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float zh = (zz[e] - mu) * rs;
                dbet[e] += g[e];
                dgam[e] = fmaf(g[e], zh, dgam[e]);
                g[e] = (g[e] * gm[e] - c1 - zh * c2) * rs;
            }
            store8(dz + row * H + col, g);
        }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) { red[0][rl][cg][e] = dgam[e]; red[1][rl][cg][e] = dbet[e]; }
    __syncthreads();
    if (rl == 0 && col < H) {
        float* pg = partials + (int64_t)blockIdx.y * 2 * H + col;
        float a[8], b[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            a[e] = ((red[0][0][cg][e] + red[0][1][cg][e]) + red[0][2][cg][e]) + red[0][3][cg][e];
            b[e] = ((red[1][0][cg][e] + red[1][1][cg][e]) + red[1][2][cg][e]) + red[1][3][cg][e];
        }
        store8(pg, a);
        store8(pg + H, b);
    }
}

bool ln_supported(int64_t H) { return H > 0 && H % 8 == 0 && H <= 8 * 8 * LN_THREADS; }
int64_t ln_partial_rows(int64_t M) { return (M + LN_SLAB - 1) / LN_SLAB; }
size_t ln_scratch_bytes(int64_t M, int64_t H) {
    return ((size_t)2 * M + (size_t)ln_partial_rows(M) * 2 * H) * sizeof(float);
}

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
    float* c12 = a.partials;                       // [M][2], then the column partials
    float* part = a.partials + 2 * a.M;
    const unsigned grid = (unsigned)(a.M < 65535 * 16 ? a.M : 65535 * 16);
    hipLaunchKernelGGL((ln_bwd_rowstat_kernel<T, MAXC>), dim3(grid), dim3(LN_THREADS), 0, a.stream, a.M, a.H,
                       (const T*)a.dy, (const T*)a.z, a.mean, a.rstd, (const T*)a.gamma, c12);
    const int64_t slabs = ln_partial_rows(a.M);
    hipLaunchKernelGGL((ln_bwd_tile_kernel<T>), dim3((unsigned)((a.H + 511) / 512), (unsigned)slabs),
                       dim3(LN_THREADS), 0, a.stream, a.M, a.H, (const T*)a.dy, (const T*)a.z, a.mean, a.rstd,
                       (const T*)a.gamma, c12, (T*)a.dz, part);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    // partial rows are [slab][2][H]: gamma and beta gradients are separate buffers, so two strided sums
    e = sum_partials_strided(a.dtype, slabs, a.H, part, 2 * a.H, a.dgamma, a.stream);
    if (e != hipSuccess) return e;
    return sum_partials_strided(a.dtype, slabs, a.H, part + a.H, 2 * a.H, a.dbeta, a.stream);
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
