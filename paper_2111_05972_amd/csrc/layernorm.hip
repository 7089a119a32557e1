// LayerNorm over the hidden dimension, forward and backward, float or bfloat16 storage with float
// arithmetic.  In the speed-optimised distribution layer normalisation is not distributed (Sec. I.1
// of the paper): every tensor-parallel rank normalises the full replicated [M, H] activation, so this
// is a plain HBM-bound row kernel.  One 256-thread workgroup holds a whole row in registers (16-byte
// accesses, up to 8 chunks of 8 elements per thread: H <= 16384), so every tensor is read or written
// exactly once:
//   forward : reads a (and b), writes z = a + b (optional) and y          -> up to 4 M H elements
//   backward: one kernel; a workgroup walks its rows (row, row + G, ...) holding dy and z of a row in registers
//             (next row prefetched), reduces the two per-row means, writes dz, and accumulates its column
//             sums of dgamma, dbeta in registers; the G per-workgroup partials are then summed in workgroup
//             order by a small kernel (deterministic)                         -> 3 M H elements + 4 G H floats
//   (the distributed variant below keeps the older two-pass form: row sums first, because there the
//   caller all-reduces them between the passes)
#include <hip/hip_runtime.h>

#include "device_math.h"
#include "kernels.h"

namespace tpl {

constexpr int LN_THREADS = 256;

// Sum over the workgroup, same value returned to every thread; fixed combination order.
template <int NW = 4>
__device__ __forceinline__ float block_sum(float v, float* red) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    const int w = threadIdx.x >> 6;
    __syncthreads();                   // red may still be read from the previous reduction
    if ((threadIdx.x & 63) == 0) red[w] = v;
    __syncthreads();
    float s = red[0];
#pragma unroll
    for (int i = 1; i < NW; ++i) s += red[i];
    return s;
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
                                                                    float out_scale,
                                                                    float* __restrict__ c12) {
    __shared__ float red[4];
    const int t = threadIdx.x;
    const float inv_h = out_scale;   // 1/H: row means (replicated); 1: plain sums (distributed, summed over ranks later)
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
                                                                 float c_scale,
                                                                 const T* __restrict__ add,
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
            const float mu = mean[row], rs = rstd[row], c1 = c12[2 * row] * c_scale, c2 = c12[2 * row + 1] * c_scale;
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
            if (add) {                               // gradient arriving over the residual branch
                float r[8];
                load8(add + row * H + col, r);
#pragma unroll
                for (int e = 0; e < 8; ++e) g[e] += r[e];
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

// Eight consecutive elements as they sit in memory (16 or 32 bytes), converted only when used: rows that are
// still in flight cost half the registers in bfloat16.
template <typename T> struct Raw8;
template <> struct Raw8<float> {
    float4 a, b;
    __device__ __forceinline__ void load(const float* p) { a = reinterpret_cast<const float4*>(p)[0]; b = reinterpret_cast<const float4*>(p)[1]; }
    __device__ __forceinline__ void get(float (&v)[8]) const {
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    }
};
template <> struct Raw8<bf16_t> {
    uint4 u;
    __device__ __forceinline__ void load(const bf16_t* p) { u = *reinterpret_cast<const uint4*>(p); }
    __device__ __forceinline__ void get(float (&v)[8]) const {
        const unsigned w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = __uint_as_float(w[i] << 16);
            v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
};

// Two sums over the workgroup at once (same values returned to every thread; fixed combination order).
template <int NW>
__device__ __forceinline__ void block_sum2(float& a, float& b, float (*red)[NW]) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) { a += __shfl_xor(a, o, 64); b += __shfl_xor(b, o, 64); }
    const int w = threadIdx.x >> 6;
    __syncthreads();                   // red may still be read from the previous row
    if ((threadIdx.x & 63) == 0) { red[0][w] = a; red[1][w] = b; }
    __syncthreads();
    a = red[0][0];
    b = red[1][0];
#pragma unroll
    for (int i = 1; i < NW; ++i) { a += red[0][i]; b += red[1][i]; }
}

// Backward in one pass (replicated LayerNorm).  Workgroup g of G walks rows g, g + G, ...; the next DEPTH rows of
// dy and z are always in flight (unconverted, in a ring of registers: the kernel is bound by how many bytes a CU
// keeps outstanding, not by arithmetic).  partials[g][0][:] = dgamma, partials[g][1][:] = dbeta of its rows.
constexpr int LN_BWD_GROUPS = 256;     // most workgroups of the backward kernel = rows of its partial sums
template <typename T, int MAXC, int THREADS, int DEPTH>
__global__ __launch_bounds__(THREADS) void ln_bwd_fused_kernel(int64_t M, int64_t H, const T* __restrict__ dy,
                                                                  const T* __restrict__ z,
                                                                  const float* __restrict__ mean,
                                                                  const float* __restrict__ rstd,
                                                                  const T* __restrict__ gamma,
                                                                  T* __restrict__ dz,
                                                                  float* __restrict__ partials) {
    constexpr int NW = THREADS / 64;
    __shared__ float red[2][NW];
    const int t = threadIdx.x;
    const int64_t G = gridDim.x;
    const float inv_h = 1.0f / (float)H;
    float gm[MAXC][8], dgam[MAXC][8], dbet[MAXC][8];
#pragma unroll
    for (int i = 0; i < MAXC; ++i) {
        const int64_t col = ((int64_t)t + THREADS * i) * 8;
#pragma unroll
        for (int e = 0; e < 8; ++e) { gm[i][e] = 0.0f; dgam[i][e] = 0.0f; dbet[i][e] = 0.0f; }
        if (col < H) load8(gamma + col, gm[i]);
    }
    Raw8<T> rg[DEPTH][MAXC], rz[DEPTH][MAXC];
    auto fetch = [&](int64_t row, Raw8<T> (&a)[MAXC], Raw8<T> (&b)[MAXC]) {
#pragma unroll
        for (int i = 0; i < MAXC; ++i) {
            const int64_t col = ((int64_t)t + THREADS * i) * 8;
            if (col < H && row < M) { a[i].load(dy + row * H + col); b[i].load(z + row * H + col); }
        }
    };
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) fetch(blockIdx.x + d * G, rg[d], rz[d]);
    for (int64_t row0 = blockIdx.x; row0 < M; row0 += DEPTH * G) {
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            const int64_t row = row0 + d * G;
            if (row < M) {                                     // uniform over the workgroup
                float g[MAXC][8], zz[MAXC][8];
#pragma unroll
                for (int i = 0; i < MAXC; ++i) { rg[d][i].get(g[i]); rz[d][i].get(zz[i]); }
                fetch(row + DEPTH * G, rg[d], rz[d]);          // the ring slot is free again
                const float mu = mean[row], rs = rstd[row];
                float c1 = 0.0f, c2 = 0.0f;
#pragma unroll
                for (int i = 0; i < MAXC; ++i) {
                    const int64_t col = ((int64_t)t + THREADS * i) * 8;
                    if (col < H) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            zz[i][e] = (zz[i][e] - mu) * rs;   // zh
                            const float gg = g[i][e] * gm[i][e];
                            c1 += gg;
                            c2 = fmaf(gg, zz[i][e], c2);
                        }
                    }
                }
                block_sum2<NW>(c1, c2, red);
                c1 *= inv_h;
                c2 *= inv_h;
#pragma unroll
                for (int i = 0; i < MAXC; ++i) {
                    const int64_t col = ((int64_t)t + THREADS * i) * 8;
                    if (col < H) {
                        float o[8];
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            dbet[i][e] += g[i][e];
                            dgam[i][e] = fmaf(g[i][e], zz[i][e], dgam[i][e]);
                            o[e] = (g[i][e] * gm[i][e] - c1 - zz[i][e] * c2) * rs;
                        }
                        store8(dz + row * H + col, o);
                    }
                }
            }
        }
    }
    float* pg = partials + (int64_t)blockIdx.x * 2 * H;
#pragma unroll
    for (int i = 0; i < MAXC; ++i) {
        const int64_t col = ((int64_t)t + THREADS * i) * 8;
        if (col < H) { store8(pg + col, dgam[i]); store8(pg + H + col, dbet[i]); }
    }
}

// dgamma, dbeta = sums of the per-workgroup partials [groups][2][H]: group lane g of 16 adds groups g, g + 16, ... in
// order, then the 16 lanes are combined in lane order (fixed order).  A thread owns four adjacent columns (16-byte
// loads); 16 such threads x 16 group lanes per workgroup, so that [256][2][12288] is spread over 384 workgroups;
// blockIdx.y picks gamma or beta.
constexpr int LN_SUM_LANES = 16, LN_SUM_COLS = 256 / LN_SUM_LANES * 4;     // columns per workgroup
template <typename T>
__global__ __launch_bounds__(256) void ln_sum_partials_kernel(int64_t groups, int64_t H, const float* __restrict__ part,
                                                             T* __restrict__ dgamma, T* __restrict__ dbeta) {
    constexpr int CT = 256 / LN_SUM_LANES;                            // column threads
    __shared__ float4 red[LN_SUM_LANES][CT];
    const int cl = threadIdx.x % CT, gl = threadIdx.x / CT;
    const int64_t col = ((int64_t)blockIdx.x * CT + cl) * 4;          // H is a multiple of 8
    const float* src = part + (int64_t)blockIdx.y * H + col;
    float4 s = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    auto add = [&](const float4& v) { s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w; };
    if (col < H) {
        int64_t g = gl;
        for (; g + 3 * LN_SUM_LANES < groups; g += 4 * LN_SUM_LANES) {   // four independent loads in flight per thread
            const float4 a = *reinterpret_cast<const float4*>(src + g * 2 * H);
            const float4 b = *reinterpret_cast<const float4*>(src + (g + LN_SUM_LANES) * 2 * H);
            const float4 c = *reinterpret_cast<const float4*>(src + (g + 2 * LN_SUM_LANES) * 2 * H);
            const float4 d = *reinterpret_cast<const float4*>(src + (g + 3 * LN_SUM_LANES) * 2 * H);
            add(a); add(b); add(c); add(d);
        }
        for (; g < groups; g += LN_SUM_LANES) add(*reinterpret_cast<const float4*>(src + g * 2 * H));
    }
    red[gl][cl] = s;
    __syncthreads();
    if (gl == 0 && col < H) {
        float4 r = red[0][cl];
#pragma unroll
        for (int i = 1; i < LN_SUM_LANES; ++i) { const float4 v = red[i][cl]; r.x += v.x; r.y += v.y; r.z += v.z; r.w += v.w; }
        T* out = (blockIdx.y == 0 ? dgamma : dbeta) + col;
        out[0] = from_f32<T>(r.x); out[1] = from_f32<T>(r.y); out[2] = from_f32<T>(r.z); out[3] = from_f32<T>(r.w);
    }
}

bool ln_supported(int64_t H) { return H > 0 && H % 8 == 0 && H <= 8 * 8 * LN_THREADS; }
int64_t ln_partial_rows(int64_t M) { return (M + LN_SLAB - 1) / LN_SLAB; }
static int64_t ln_bwd_groups(int64_t M) { return M < LN_BWD_GROUPS ? M : LN_BWD_GROUPS; }
size_t ln_scratch_bytes(int64_t M, int64_t H) { return (size_t)ln_bwd_groups(M) * 2 * H * sizeof(float); }

template <typename T, int MAXC>
static hipError_t fwd_t(const LnArgs& a) {
    const unsigned grid = (unsigned)(a.M < 65535 * 16 ? a.M : 65535 * 16);
    hipLaunchKernelGGL((ln_fwd_kernel<T, MAXC>), dim3(grid), dim3(LN_THREADS), 0, a.stream, a.M, a.H,
                       (const T*)a.a, (const T*)a.b, (const T*)a.gamma, (const T*)a.beta, a.eps, (T*)a.z,
                       (T*)a.y, a.mean, a.rstd);
    return hipGetLastError();
}
// MAXC counts the 8-element chunks per thread of a 256-thread workgroup; rows of more than two such chunks go to
// 512-thread workgroups with half the chunks, so that two wavefronts share each SIMD.
template <typename T, int MAXC>
static hipError_t bwd_t(const LnArgs& a) {
    float* part = a.partials;                      // [groups][2][H]
    const int64_t groups = ln_bwd_groups(a.M);
    // Rows in flight per workgroup beyond the one being worked on.  Measured at [2048, 12288] bfloat16: 1 -> 47 us,
    // 2 -> 41 us, 3 and 4 -> 42 us for both kernels together (the compiler drains the whole ring once per DEPTH rows).
    constexpr int DEPTH = (sizeof(T) == 2 && MAXC <= 6) ? 2 : 1;   // the widest rows have no registers left for two
    if constexpr (MAXC > 2)
        hipLaunchKernelGGL((ln_bwd_fused_kernel<T, MAXC / 2, 512, DEPTH>), dim3((unsigned)groups), dim3(512), 0, a.stream,
                           a.M, a.H, (const T*)a.dy, (const T*)a.z, a.mean, a.rstd, (const T*)a.gamma, (T*)a.dz, part);
    else
        hipLaunchKernelGGL((ln_bwd_fused_kernel<T, MAXC, LN_THREADS, DEPTH>), dim3((unsigned)groups), dim3(LN_THREADS), 0,
                           a.stream, a.M, a.H, (const T*)a.dy, (const T*)a.z, a.mean, a.rstd, (const T*)a.gamma,
                           (T*)a.dz, part);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((ln_sum_partials_kernel<T>), dim3((unsigned)((a.H + LN_SUM_COLS - 1) / LN_SUM_COLS), 2), dim3(256), 0, a.stream,
                       groups, a.H, part, (T*)a.dgamma, (T*)a.dbeta);
    return hipGetLastError();
}

template <typename T>
static hipError_t dispatch(const LnArgs& a, bool bwd) {
    const int64_t chunks = (a.H / 8 + LN_THREADS - 1) / LN_THREADS;
    if (chunks <= 2) return bwd ? bwd_t<T, 2>(a) : fwd_t<T, 2>(a);
    if (chunks <= 4) return bwd ? bwd_t<T, 4>(a) : fwd_t<T, 4>(a);
    if (chunks <= 6) return bwd ? bwd_t<T, 6>(a) : fwd_t<T, 6>(a);
    return bwd ? bwd_t<T, 8>(a) : fwd_t<T, 8>(a);
}

// ------------------------------------------------------------------------------------------------
// Distributed layer normalisation (memory-optimised distribution, App. F.2 of the paper): a rank holds
// the channel slice [M, Hs] of the activation.  Forward: per-token moments (sum x, sum x^2) of the
// slice; after the caller's all-reduce over ranks, `ln_dist_stats` turns the totals into mean and
// 1/sqrt(var + eps), and `ln_dist_apply` normalises the slice element-wise with them.  Backward: the
// per-token sums (sum dy*gamma, sum dy*gamma*xhat) of the slice, all-reduced by the caller, then dx,
// dgamma, dbeta of the slice.  The backward runs the two kernels above with x in place of the saved
// z, plain sums out of the row pass and the totals scaled by 1/H going into the tile pass.
// ------------------------------------------------------------------------------------------------
template <typename T, int MAXC>
__global__ __launch_bounds__(LN_THREADS) void ln_moments_kernel(int64_t M, int64_t Hs, const T* __restrict__ x,
                                                                float* __restrict__ sums) {
    __shared__ float red[4];
    const int t = threadIdx.x;
    for (int64_t row = blockIdx.x; row < M; row += gridDim.x) {
        float s1 = 0.0f, s2 = 0.0f;
#pragma unroll
        for (int i = 0; i < MAXC; ++i) {
            const int64_t col = ((int64_t)t + LN_THREADS * i) * 8;
            if (col < Hs) {
                float v[8];
                load8(x + row * Hs + col, v);
#pragma unroll
                for (int e = 0; e < 8; ++e) { s1 += v[e]; s2 = fmaf(v[e], v[e], s2); }
            }
        }
        const float a = block_sum(s1, red), b = block_sum(s2, red);
        if (t == 0) { sums[2 * row] = a; sums[2 * row + 1] = b; }
    }
}

__global__ void ln_stats_kernel(int64_t M, float inv_h, float eps, const float* __restrict__ totals,
                                float* __restrict__ mean, float* __restrict__ rstd) {
    const int64_t row = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (row < M) {
        const float mu = totals[2 * row] * inv_h;
        const float var = fmaf(-mu, mu, totals[2 * row + 1] * inv_h);
        mean[row] = mu;
        rstd[row] = 1.0f / sqrtf(fmaxf(var, 0.0f) + eps);
    }
}

// LN_SLAB rows x 512 columns per workgroup, as the backward tile pass.
template <typename T>
__global__ __launch_bounds__(LN_THREADS) void ln_apply_kernel(int64_t M, int64_t Hs, const T* __restrict__ x,
                                                              const float* __restrict__ mean,
                                                              const float* __restrict__ rstd,
                                                              const T* __restrict__ gamma,
                                                              const T* __restrict__ beta, T* __restrict__ y) {
    const int cg = threadIdx.x & 63, rl = threadIdx.x >> 6;
    const int64_t col = ((int64_t)blockIdx.x * 64 + cg) * 8;
    const int64_t m0 = (int64_t)blockIdx.y * LN_SLAB, m1 = m0 + LN_SLAB < M ? m0 + LN_SLAB : M;
    if (col >= Hs) return;
    float gm[8], bt[8];
    load8(gamma + col, gm);
    load8(beta + col, bt);
    for (int64_t row = m0 + rl; row < m1; row += 4) {
        const float mu = mean[row], rs = rstd[row];
        float v[8];
        load8(x + row * Hs + col, v);
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = fmaf((v[e] - mu) * rs, gm[e], bt[e]);
        store8(y + row * Hs + col, v);
    }
}

template <typename T, int MAXC>
static hipError_t moments_t(int64_t M, int64_t Hs, const void* x, float* sums, hipStream_t s) {
    const unsigned grid = (unsigned)(M < 65535 * 16 ? M : 65535 * 16);
    hipLaunchKernelGGL((ln_moments_kernel<T, MAXC>), dim3(grid), dim3(LN_THREADS), 0, s, M, Hs, (const T*)x, sums);
    return hipGetLastError();
}
template <typename T, int MAXC>
static hipError_t bwd_sums_t(int64_t M, int64_t Hs, const void* dy, const void* x, const float* mean,
                             const float* rstd, const void* gamma, float* sums, hipStream_t s) {
    const unsigned grid = (unsigned)(M < 65535 * 16 ? M : 65535 * 16);
    hipLaunchKernelGGL((ln_bwd_rowstat_kernel<T, MAXC>), dim3(grid), dim3(LN_THREADS), 0, s, M, Hs, (const T*)dy,
                       (const T*)x, mean, rstd, (const T*)gamma, 1.0f, sums);
    return hipGetLastError();
}
#define TPL_LN_CHUNKS(Hs, CALL2, CALL4, CALL8)                                   \
    do {                                                                         \
        const int64_t chunks_ = ((Hs) / 8 + LN_THREADS - 1) / LN_THREADS;        \
        if (chunks_ <= 2) return CALL2;                                          \
        if (chunks_ <= 4) return CALL4;                                          \
        return CALL8;                                                            \
    } while (0)

hipError_t ln_dist_moments(int dtype, int64_t M, int64_t Hs, const void* x, float* sums, hipStream_t s) {
    if (dtype == F32) TPL_LN_CHUNKS(Hs, (moments_t<float, 2>(M, Hs, x, sums, s)), (moments_t<float, 4>(M, Hs, x, sums, s)),
                                    (moments_t<float, 8>(M, Hs, x, sums, s)));
    TPL_LN_CHUNKS(Hs, (moments_t<bf16_t, 2>(M, Hs, x, sums, s)), (moments_t<bf16_t, 4>(M, Hs, x, sums, s)),
                  (moments_t<bf16_t, 8>(M, Hs, x, sums, s)));
}

hipError_t ln_dist_stats(int64_t M, int64_t H, float eps, const float* totals, float* mean, float* rstd,
                         hipStream_t s) {
    hipLaunchKernelGGL(ln_stats_kernel, dim3((unsigned)((M + 255) / 256)), dim3(256), 0, s, M, 1.0f / (float)H, eps,
                       totals, mean, rstd);
    return hipGetLastError();
}

hipError_t ln_dist_apply(int dtype, int64_t M, int64_t Hs, const void* x, const float* mean, const float* rstd,
                         const void* gamma, const void* beta, void* y, hipStream_t s) {
    const dim3 grid((unsigned)((Hs + 511) / 512), (unsigned)ln_partial_rows(M));
    if (dtype == F32)
        hipLaunchKernelGGL((ln_apply_kernel<float>), grid, dim3(LN_THREADS), 0, s, M, Hs, (const float*)x, mean, rstd,
                           (const float*)gamma, (const float*)beta, (float*)y);
    else
        hipLaunchKernelGGL((ln_apply_kernel<bf16_t>), grid, dim3(LN_THREADS), 0, s, M, Hs, (const bf16_t*)x, mean,
                           rstd, (const bf16_t*)gamma, (const bf16_t*)beta, (bf16_t*)y);
    return hipGetLastError();
}

hipError_t ln_dist_bwd_sums(int dtype, int64_t M, int64_t Hs, const void* dy, const void* x, const float* mean,
                            const float* rstd, const void* gamma, float* sums, hipStream_t s) {
    if (dtype == F32)
        TPL_LN_CHUNKS(Hs, (bwd_sums_t<float, 2>(M, Hs, dy, x, mean, rstd, gamma, sums, s)),
                      (bwd_sums_t<float, 4>(M, Hs, dy, x, mean, rstd, gamma, sums, s)),
                      (bwd_sums_t<float, 8>(M, Hs, dy, x, mean, rstd, gamma, sums, s)));
    TPL_LN_CHUNKS(Hs, (bwd_sums_t<bf16_t, 2>(M, Hs, dy, x, mean, rstd, gamma, sums, s)),
                  (bwd_sums_t<bf16_t, 4>(M, Hs, dy, x, mean, rstd, gamma, sums, s)),
                  (bwd_sums_t<bf16_t, 8>(M, Hs, dy, x, mean, rstd, gamma, sums, s)));
}

// partials: ln_partial_rows(M) * 2 * Hs floats.
hipError_t ln_dist_bwd_apply(int dtype, int64_t M, int64_t Hs, int64_t H, const void* dy, const void* x,
                             const float* mean, const float* rstd, const void* gamma, const float* totals,
                             const void* dx_add, void* dx, void* dgamma, void* dbeta, float* partials,
                             hipStream_t s) {
    const int64_t slabs = ln_partial_rows(M);
    const dim3 grid((unsigned)((Hs + 511) / 512), (unsigned)slabs);
    const float c_scale = 1.0f / (float)H;
    if (dtype == F32)
        hipLaunchKernelGGL((ln_bwd_tile_kernel<float>), grid, dim3(LN_THREADS), 0, s, M, Hs, (const float*)dy,
                           (const float*)x, mean, rstd, (const float*)gamma, totals, c_scale, (const float*)dx_add,
                           (float*)dx, partials);
    else
        hipLaunchKernelGGL((ln_bwd_tile_kernel<bf16_t>), grid, dim3(LN_THREADS), 0, s, M, Hs, (const bf16_t*)dy,
                           (const bf16_t*)x, mean, rstd, (const bf16_t*)gamma, totals, c_scale, (const bf16_t*)dx_add,
                           (bf16_t*)dx, partials);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    e = sum_partials_strided(dtype, slabs, Hs, partials, 2 * Hs, dgamma, s);
    if (e != hipSuccess) return e;
    return sum_partials_strided(dtype, slabs, Hs, partials + Hs, 2 * Hs, dbeta, s);
}
size_t ln_dist_scratch_bytes(int64_t M, int64_t Hs) { return (size_t)ln_partial_rows(M) * 2 * Hs * sizeof(float); }

// ------------------------------------------------------------------------------------------------
// What a rank does to the slice [M, N] it keeps after a reduce-scatter (the product of an input-split
// linear is a partial sum, so bias, residual and activation cannot ride in the GEMM epilogue):
// v = in + bias (+ resid); with GeLU u = v is kept and out = gelu(v), otherwise out = v.
// Backward with GeLU: din = dout * gelu'(u).
// ------------------------------------------------------------------------------------------------
template <typename T, bool GELU>
__global__ __launch_bounds__(256) void slice_epilogue_fwd_kernel(int64_t M, int64_t N, const T* __restrict__ in,
                                                                 const T* __restrict__ bias,
                                                                 const T* __restrict__ resid, T* __restrict__ u,
                                                                 T* __restrict__ out) {
    const int64_t chunks = N / 8, total = M * chunks;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        const int64_t col = (i % chunks) * 8, off = (i / chunks) * N + col;
        float v[8], b[8];
        load8(in + off, v);
        load8(bias + col, b);
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] += b[e];
        if (resid) {
            load8(resid + off, b);
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] += b[e];
        }
        if (GELU) {
            store8(u + off, v);
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = gelu_f(v[e]);
        }
        store8(out + off, v);
    }
}
template <typename T>
__global__ __launch_bounds__(256) void gelu_bwd_kernel(int64_t total8, const T* __restrict__ dg,
                                                       const T* __restrict__ u, T* __restrict__ du) {
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total8; i += (int64_t)gridDim.x * 256) {
        float v[8], w[8];
        load8(dg + i * 8, v);
        load8(u + i * 8, w);
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] *= gelu_grad_f(w[e]);
        store8(du + i * 8, v);
    }
}
static unsigned ew_grid(int64_t items) {
    int64_t b = (items + 255) / 256;
    return (unsigned)(b < 1 ? 1 : (b > 256 * 32 ? 256 * 32 : b));
}
template <typename T>
static hipError_t slice_fwd_t(bool gelu, int64_t M, int64_t N, const void* in, const void* bias, const void* resid,
                              void* u, void* out, hipStream_t s) {
    const unsigned grid = ew_grid(M * (N / 8));
    if (gelu)
        hipLaunchKernelGGL((slice_epilogue_fwd_kernel<T, true>), dim3(grid), dim3(256), 0, s, M, N, (const T*)in,
                           (const T*)bias, (const T*)resid, (T*)u, (T*)out);
    else
        hipLaunchKernelGGL((slice_epilogue_fwd_kernel<T, false>), dim3(grid), dim3(256), 0, s, M, N, (const T*)in,
                           (const T*)bias, (const T*)resid, (T*)u, (T*)out);
    return hipGetLastError();
}
hipError_t slice_epilogue_fwd(int dtype, bool gelu, int64_t M, int64_t N, const void* in, const void* bias,
                              const void* resid, void* u, void* out, hipStream_t s) {
    return dtype == F32 ? slice_fwd_t<float>(gelu, M, N, in, bias, resid, u, out, s)
                        : slice_fwd_t<bf16_t>(gelu, M, N, in, bias, resid, u, out, s);
}
hipError_t gelu_bwd(int dtype, int64_t M, int64_t N, const void* dg, const void* u, void* du, hipStream_t s) {
    const int64_t total8 = M * N / 8;
    const unsigned grid = ew_grid(total8);
    if (dtype == F32)
        hipLaunchKernelGGL((gelu_bwd_kernel<float>), dim3(grid), dim3(256), 0, s, total8, (const float*)dg,
                           (const float*)u, (float*)du);
    else
        hipLaunchKernelGGL((gelu_bwd_kernel<bf16_t>), dim3(grid), dim3(256), 0, s, total8, (const bf16_t*)dg,
                           (const bf16_t*)u, (bf16_t*)du);
    return hipGetLastError();
}

hipError_t ln_fwd(const LnArgs& a) { return a.dtype == F32 ? dispatch<float>(a, false) : dispatch<bf16_t>(a, false); }
hipError_t ln_bwd(const LnArgs& a) { return a.dtype == F32 ? dispatch<float>(a, true) : dispatch<bf16_t>(a, true); }

}  // namespace tpl
