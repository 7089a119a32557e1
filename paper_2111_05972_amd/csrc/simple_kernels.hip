// Generic kernels: any shape, float or bfloat16 storage, float accumulation.
// They are the only path for float tensors and cover bfloat16 shapes the MFMA kernels do not take.
#include <hip/hip_runtime.h>

#include <mutex>

#include "device_math.h"
#include "kernels.h"

namespace tpl {

// ------------------------------------------------------------------------------------------------
// GEMM: 64x64 output tile per 256-thread block, 4x4 outputs per thread, operands addressed through
// (row, column) strides so all four transpose combinations share one kernel.
// ------------------------------------------------------------------------------------------------
constexpr int SG_BM = 64, SG_BN = 64, SG_BK = 16;

template <typename T>
__global__ __launch_bounds__(256) void gemm_simple_kernel(
    int64_t M, int64_t N, int64_t K, const T* __restrict__ A, int64_t a_rs, int64_t a_cs,
    const T* __restrict__ B, int64_t b_rs, int64_t b_cs, T* __restrict__ C,
    const T* __restrict__ bias, const T* __restrict__ resid, T* __restrict__ aux, int epi) {
    __shared__ float As[SG_BK][SG_BM + 1];
    __shared__ float Bs[SG_BK][SG_BN + 1];
    const int t = threadIdx.x;
    const int64_t m0 = (int64_t)blockIdx.y * SG_BM, n0 = (int64_t)blockIdx.x * SG_BN;
    const int tm = (t / 16) * 4, tn = (t % 16) * 4;
    float acc[4][4] = {};
    for (int64_t k0 = 0; k0 < K; k0 += SG_BK) {
        for (int i = 0; i < 4; ++i) {
            int mm, kk;
            if (a_cs == 1) { kk = t % SG_BK; mm = t / SG_BK + 16 * i; }
            else           { mm = t % SG_BM; kk = t / SG_BM + 4 * i; }
            int64_t gm = m0 + mm, gk = k0 + kk;
            As[kk][mm] = (gm < M && gk < K) ? to_f32(A[gm * a_rs + gk * a_cs]) : 0.0f;
            int nn, kb;
            if (b_rs == 1) { kb = t % SG_BK; nn = t / SG_BK + 16 * i; }
            else           { nn = t % SG_BN; kb = t / SG_BN + 4 * i; }
            int64_t gn = n0 + nn, gkb = k0 + kb;
            Bs[kb][nn] = (gn < N && gkb < K) ? to_f32(B[gkb * b_rs + gn * b_cs]) : 0.0f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < SG_BK; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { a[i] = As[kk][tm + i]; b[i] = Bs[kk][tn + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
    for (int i = 0; i < 4; ++i) {
        int64_t gm = m0 + tm + i;
        if (gm >= M) continue;
        for (int j = 0; j < 4; ++j) {
            int64_t gn = n0 + tn + j;
            if (gn >= N) continue;
            float v = acc[i][j];
            if (bias) v += to_f32(bias[gn]);
            if (resid) v += to_f32(resid[gm * N + gn]);
            if (epi == EPI_GELU) {
                aux[gm * N + gn] = from_f32<T>(v);
                v = gelu_f(v);
            } else if (epi == EPI_DGELU) {
                v *= gelu_grad_f(to_f32(aux[gm * N + gn]));
            }
            C[gm * N + gn] = from_f32<T>(v);
        }
    }
}

template <typename T>
static hipError_t gemm_simple_t(const GemmArgs& a) {
    dim3 grid((unsigned)((a.N + SG_BN - 1) / SG_BN), (unsigned)((a.M + SG_BM - 1) / SG_BM));
    int64_t a_rs = a.trans_a ? 1 : a.K, a_cs = a.trans_a ? a.M : 1;   // A(m,k)
    int64_t b_rs = a.trans_b ? 1 : a.N, b_cs = a.trans_b ? a.K : 1;   // B(k,n)
    hipLaunchKernelGGL(gemm_simple_kernel<T>, grid, dim3(256), 0, a.stream, a.M, a.N, a.K,
                       (const T*)a.A, a_rs, a_cs, (const T*)a.B, b_rs, b_cs, (T*)a.C,
                       (const T*)a.bias, (const T*)a.resid, (T*)a.aux, a.epi);
    return hipGetLastError();
}

hipError_t gemm_simple(const GemmArgs& a) {
    return a.dtype == F32 ? gemm_simple_t<float>(a) : gemm_simple_t<bf16_t>(a);
}

// ------------------------------------------------------------------------------------------------
// Attention, one wavefront per query row (forward, dQ) or per key row (dK, dV).
// qkv is [B*S, 3*nl*dh] with columns (q|k|v, head, dh).  Keys are visited 64 at a time: lane j of
// the wavefront owns key j0+j for the logits, then lane d owns output column d for the
// value-weighted sums, with the weights passed across lanes by shuffles.
// ------------------------------------------------------------------------------------------------
constexpr int AT_WAVES = 4;
constexpr int AT_MAXDH = 256;

__device__ __forceinline__ float wave_max(float v) {
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

template <typename T>
__global__ __launch_bounds__(64 * AT_WAVES) void attn_simple_fwd_kernel(
    int B, int S, int nl, int dh, int causal, const T* __restrict__ qkv, T* __restrict__ o,
    float* __restrict__ lse) {
    __shared__ float q_s[AT_WAVES][AT_MAXDH];
    const int w = threadIdx.x / 64, lane = threadIdx.x % 64;
    const int i_raw = blockIdx.x * AT_WAVES + w;
    const bool valid = i_raw < S;          // a tail wavefront recomputes the last row and stores nothing
    const int i = valid ? i_raw : S - 1;
    const int b = blockIdx.y / nl, h = blockIdx.y % nl;
    const int64_t ld = 3LL * nl * dh;
    const T* qp = qkv + ((int64_t)b * S + i) * ld + (int64_t)h * dh;
    const T* kbase = qkv + (int64_t)b * S * ld + (int64_t)nl * dh + (int64_t)h * dh;
    const T* vbase = kbase + (int64_t)nl * dh;
    for (int d = lane; d < dh; d += 64) q_s[w][d] = to_f32(qp[d]);
    __syncthreads();
    const float scale = 1.0f / sqrtf((float)dh);
    const int jend = causal ? i + 1 : S;
    // pass 1: row maximum and sum of exponentials
    float mx = -INFINITY, sum = 0.0f;
    for (int j0 = 0; j0 < jend; j0 += 64) {
        int j = j0 + lane;
        if (j < jend) {
            const T* kp = kbase + (int64_t)j * ld;
            float s = 0.0f;
            for (int d = 0; d < dh; ++d) s = fmaf(q_s[w][d], to_f32(kp[d]), s);
            s *= scale;
            float nm = fmaxf(mx, s);
            sum = sum * expf(mx - nm) + expf(s - nm);
            mx = nm;
        }
    }
    float gmx = wave_max(mx);
    sum = wave_sum(mx == -INFINITY ? 0.0f : sum * expf(mx - gmx));
    const float inv = 1.0f / sum;
    // pass 2: O = sum_j p_j V_j
    float acc[AT_MAXDH / 64] = {};
    for (int j0 = 0; j0 < jend; j0 += 64) {
        int j = j0 + lane;
        float p = 0.0f;
        if (j < jend) {
            const T* kp = kbase + (int64_t)j * ld;
            float s = 0.0f;
            for (int d = 0; d < dh; ++d) s = fmaf(q_s[w][d], to_f32(kp[d]), s);
            p = expf(s * scale - gmx) * inv;
        }
        int cnt = min(64, jend - j0);
        for (int jj = 0; jj < cnt; ++jj) {
            float pj = __shfl(p, jj, 64);
            const T* vp = vbase + (int64_t)(j0 + jj) * ld;
#pragma unroll
            for (int t = 0; t < AT_MAXDH / 64; ++t) {
                int d = lane + 64 * t;
                if (d < dh) acc[t] = fmaf(pj, to_f32(vp[d]), acc[t]);
            }
        }
    }
    T* op = o + ((int64_t)b * S + i) * ((int64_t)nl * dh) + (int64_t)h * dh;
#pragma unroll
    for (int t = 0; t < AT_MAXDH / 64; ++t) {
        int d = lane + 64 * t;
        if (valid && d < dh) op[d] = from_f32<T>(acc[t]);
    }
    if (valid && lane == 0) lse[((int64_t)b * nl + h) * S + i] = gmx + logf(sum);
}

// dQ_i = sum_j dS_ij K_j / sqrt(dh), dS_ij = P_ij (dO_i.V_j - D_i), D_i = dO_i.O_i; also stores D.
template <typename T>
__global__ __launch_bounds__(64 * AT_WAVES) void attn_simple_dq_kernel(
    int B, int S, int nl, int dh, int causal, const T* __restrict__ qkv, const T* __restrict__ o,
    const float* __restrict__ lse, const T* __restrict__ d_o, T* __restrict__ dqkv,
    float* __restrict__ dsum) {
    __shared__ float q_s[AT_WAVES][AT_MAXDH];
    __shared__ float do_s[AT_WAVES][AT_MAXDH];
    const int w = threadIdx.x / 64, lane = threadIdx.x % 64;
    const int i_raw = blockIdx.x * AT_WAVES + w;
    const bool valid = i_raw < S;
    const int i = valid ? i_raw : S - 1;
    const int b = blockIdx.y / nl, h = blockIdx.y % nl;
    const int64_t ld = 3LL * nl * dh, ldo = (int64_t)nl * dh;
    const T* qp = qkv + ((int64_t)b * S + i) * ld + (int64_t)h * dh;
    const T* kbase = qkv + (int64_t)b * S * ld + (int64_t)nl * dh + (int64_t)h * dh;
    const T* vbase = kbase + (int64_t)nl * dh;
    const T* dop = d_o + ((int64_t)b * S + i) * ldo + (int64_t)h * dh;
    const T* op = o + ((int64_t)b * S + i) * ldo + (int64_t)h * dh;
    float dpart = 0.0f;
    for (int d = lane; d < dh; d += 64) {
        float g = to_f32(dop[d]);
        q_s[w][d] = to_f32(qp[d]);
        do_s[w][d] = g;
        dpart = fmaf(g, to_f32(op[d]), dpart);
    }
    const float Di = wave_sum(dpart);
    __syncthreads();
    const float scale = 1.0f / sqrtf((float)dh);
    const float L = lse[((int64_t)b * nl + h) * S + i];
    const int jend = causal ? i + 1 : S;
    float acc[AT_MAXDH / 64] = {};
    for (int j0 = 0; j0 < jend; j0 += 64) {
        int j = j0 + lane;
        float ds = 0.0f;
        if (j < jend) {
            const T* kp = kbase + (int64_t)j * ld;
            const T* vp = vbase + (int64_t)j * ld;
            float s = 0.0f, dp = 0.0f;
            for (int d = 0; d < dh; ++d) {
                s = fmaf(q_s[w][d], to_f32(kp[d]), s);
                dp = fmaf(do_s[w][d], to_f32(vp[d]), dp);
            }
            ds = expf(s * scale - L) * (dp - Di);
        }
        int cnt = min(64, jend - j0);
        for (int jj = 0; jj < cnt; ++jj) {
            float dsj = __shfl(ds, jj, 64);
            const T* kp = kbase + (int64_t)(j0 + jj) * ld;
#pragma unroll
            for (int t = 0; t < AT_MAXDH / 64; ++t) {
                int d = lane + 64 * t;
                if (d < dh) acc[t] = fmaf(dsj, to_f32(kp[d]), acc[t]);
            }
        }
    }
    T* dqp = dqkv + ((int64_t)b * S + i) * ld + (int64_t)h * dh;
#pragma unroll
    for (int t = 0; t < AT_MAXDH / 64; ++t) {
        int d = lane + 64 * t;
        if (valid && d < dh) dqp[d] = from_f32<T>(acc[t] * scale);
    }
    if (valid && lane == 0) dsum[((int64_t)b * nl + h) * S + i] = Di;
}

// dK_j = sum_i dS_ij Q_i / sqrt(dh), dV_j = sum_i P_ij dO_i.
template <typename T>
__global__ __launch_bounds__(64 * AT_WAVES) void attn_simple_dkv_kernel(
    int B, int S, int nl, int dh, int causal, const T* __restrict__ qkv,
    const float* __restrict__ lse, const T* __restrict__ d_o, T* __restrict__ dqkv,
    const float* __restrict__ dsum) {
    __shared__ float k_s[AT_WAVES][AT_MAXDH];
    __shared__ float v_s[AT_WAVES][AT_MAXDH];
    const int w = threadIdx.x / 64, lane = threadIdx.x % 64;
    const int j_raw = blockIdx.x * AT_WAVES + w;
    const bool valid = j_raw < S;
    const int j = valid ? j_raw : S - 1;
    const int b = blockIdx.y / nl, h = blockIdx.y % nl;
    const int64_t ld = 3LL * nl * dh, ldo = (int64_t)nl * dh;
    const T* qbase = qkv + (int64_t)b * S * ld + (int64_t)h * dh;
    const T* kp = qbase + (int64_t)j * ld + (int64_t)nl * dh;
    const T* vp = kp + (int64_t)nl * dh;
    const T* dobase = d_o + (int64_t)b * S * ldo + (int64_t)h * dh;
    for (int d = lane; d < dh; d += 64) { k_s[w][d] = to_f32(kp[d]); v_s[w][d] = to_f32(vp[d]); }
    __syncthreads();
    const float scale = 1.0f / sqrtf((float)dh);
    const float* lrow = lse + ((int64_t)b * nl + h) * S;
    const float* drow = dsum + ((int64_t)b * nl + h) * S;
    const int ibeg = causal ? j : 0;
    float dk[AT_MAXDH / 64] = {}, dv[AT_MAXDH / 64] = {};
    for (int i0 = ibeg; i0 < S; i0 += 64) {
        int i = i0 + lane;
        float p = 0.0f, ds = 0.0f;
        if (i < S) {
            const T* qp = qbase + (int64_t)i * ld;
            const T* dop = dobase + (int64_t)i * ldo;
            float s = 0.0f, dp = 0.0f;
            for (int d = 0; d < dh; ++d) {
                s = fmaf(to_f32(qp[d]), k_s[w][d], s);
                dp = fmaf(to_f32(dop[d]), v_s[w][d], dp);
            }
            p = expf(s * scale - lrow[i]);
            ds = p * (dp - drow[i]);
        }
        int cnt = min(64, S - i0);
        for (int ii = 0; ii < cnt; ++ii) {
            float pi = __shfl(p, ii, 64), dsi = __shfl(ds, ii, 64);
            const T* qp = qbase + (int64_t)(i0 + ii) * ld;
            const T* dop = dobase + (int64_t)(i0 + ii) * ldo;
#pragma unroll
            for (int t = 0; t < AT_MAXDH / 64; ++t) {
                int d = lane + 64 * t;
                if (d < dh) {
                    dk[t] = fmaf(dsi, to_f32(qp[d]), dk[t]);
                    dv[t] = fmaf(pi, to_f32(dop[d]), dv[t]);
                }
            }
        }
    }
    T* dkp = dqkv + ((int64_t)b * S + j) * ld + (int64_t)nl * dh + (int64_t)h * dh;
    T* dvp = dkp + (int64_t)nl * dh;
#pragma unroll
    for (int t = 0; t < AT_MAXDH / 64; ++t) {
        int d = lane + 64 * t;
        if (valid && d < dh) { dkp[d] = from_f32<T>(dk[t] * scale); dvp[d] = from_f32<T>(dv[t]); }
    }
}

template <typename T>
static hipError_t attn_fwd_t(const AttnArgs& a) {
    dim3 grid((a.S + AT_WAVES - 1) / AT_WAVES, a.B * a.nl);
    hipLaunchKernelGGL(attn_simple_fwd_kernel<T>, grid, dim3(64 * AT_WAVES), 0, a.stream, a.B, a.S,
                       a.nl, a.dh, a.causal, (const T*)a.qkv, (T*)a.o, a.lse);
    return hipGetLastError();
}
template <typename T>
static hipError_t attn_bwd_t(const AttnArgs& a) {
    dim3 grid((a.S + AT_WAVES - 1) / AT_WAVES, a.B * a.nl);
    hipLaunchKernelGGL(attn_simple_dq_kernel<T>, grid, dim3(64 * AT_WAVES), 0, a.stream, a.B, a.S,
                       a.nl, a.dh, a.causal, (const T*)a.qkv, (const T*)a.o, a.lse,
                       (const T*)a.d_o, (T*)a.dqkv, a.dsum);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(attn_simple_dkv_kernel<T>, grid, dim3(64 * AT_WAVES), 0, a.stream, a.B, a.S,
                       a.nl, a.dh, a.causal, (const T*)a.qkv, a.lse, (const T*)a.d_o, (T*)a.dqkv,
                       a.dsum);
    return hipGetLastError();
}

hipError_t attn_simple_fwd(const AttnArgs& a) {
    return a.dtype == F32 ? attn_fwd_t<float>(a) : attn_fwd_t<bf16_t>(a);
}
hipError_t attn_simple_bwd(const AttnArgs& a) {
    return a.dtype == F32 ? attn_bwd_t<float>(a) : attn_bwd_t<bf16_t>(a);
}

// ------------------------------------------------------------------------------------------------
// Column sums (bias gradients): out[n] = sum_m X[m,n].  HBM-bound: X is read once with 16-byte loads.
// Two fixed-order stages so results do not depend on scheduling: a block sums a slab of CS_ROWS rows
// for 512 columns (64 column groups of 8 x 4 row lanes, combined through LDS in lane order) into
// scratch[slab][n]; then the slabs of a column are added in a fixed order (four interleaved lanes).
// ------------------------------------------------------------------------------------------------
constexpr int CS_ROWS = 64;

template <typename T>
__global__ __launch_bounds__(256) void colsum_stage1(int64_t M, int64_t N, const T* __restrict__ X,
                                                     float* __restrict__ part) {
    __shared__ float red[4][64][8];
    const int cg = threadIdx.x & 63, rl = threadIdx.x >> 6;
    const int64_t n = ((int64_t)blockIdx.x * 64 + cg) * 8;
    const int64_t m0 = (int64_t)blockIdx.y * CS_ROWS, m1 = m0 + CS_ROWS < M ? m0 + CS_ROWS : M;
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    const int cnt = n + 8 <= N ? 8 : (n < N ? (int)(N - n) : 0);     // columns this thread owns
    if (cnt == 8) {
        int64_t m = m0 + rl;
        for (; m + 12 < m1; m += 16) {                               // four rows in flight, added in row order
            float v[4][8];
#pragma unroll
            for (int r = 0; r < 4; ++r) load8(X + (m + 4 * r) * N + n, v[r]);
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[e] += v[r][e];
        }
        for (; m < m1; m += 4) {
            float v[8];
            load8(X + m * N + n, v);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] += v[e];
        }
    } else if (cnt > 0) {                                            // ragged tail of a float matrix
        for (int64_t m = m0 + rl; m < m1; m += 4)
            for (int e = 0; e < cnt; ++e) acc[e] += to_f32(X[m * N + n + e]);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) red[rl][cg][e] = acc[e];
    __syncthreads();
    if (rl == 0) {
        float* dst = part + (int64_t)blockIdx.y * N + n;
        for (int e = 0; e < cnt; ++e) dst[e] = ((red[0][cg][e] + red[1][cg][e]) + red[2][cg][e]) + red[3][cg][e];
    }
}
// 64 columns x 4 slab lanes per workgroup: lane g adds slabs g, g+4, ... in order (four loads in flight), the four
// lanes are combined through LDS in lane order.
template <typename T>
__global__ __launch_bounds__(256) void colsum_stage2(int64_t slabs, int64_t N, int64_t stride,
                                                     const float* __restrict__ part,
                                                     T* __restrict__ out) {
    __shared__ float red[4][64];
    const int cl = threadIdx.x & 63, gl = threadIdx.x >> 6;
    const int64_t n = (int64_t)blockIdx.x * 64 + cl;
    float s = 0.0f;
    if (n < N) {
        const float* src = part + n;
        int64_t i = gl;
        for (; i + 12 < slabs; i += 16) {
            const float a = src[i * stride], b = src[(i + 4) * stride], c = src[(i + 8) * stride],
                        d = src[(i + 12) * stride];
            s += a; s += b; s += c; s += d;
        }
        for (; i < slabs; i += 4) s += src[i * stride];
    }
    red[gl][cl] = s;
    __syncthreads();
    if (gl == 0 && n < N) out[n] = from_f32<T>(((red[0][cl] + red[1][cl]) + red[2][cl]) + red[3][cl]);
}

size_t colsum_scratch_bytes(int64_t M, int64_t N) {
    return (size_t)((M + CS_ROWS - 1) / CS_ROWS) * (size_t)N * sizeof(float);
}

hipError_t sum_partials_strided(int dtype, int64_t slabs, int64_t N, const float* part, int64_t stride,
                                void* out, hipStream_t s) {
    dim3 g2((unsigned)((N + 63) / 64));
    if (dtype == F32) hipLaunchKernelGGL(colsum_stage2<float>, g2, dim3(256), 0, s, slabs, N, stride, part, (float*)out);
    else hipLaunchKernelGGL(colsum_stage2<bf16_t>, g2, dim3(256), 0, s, slabs, N, stride, part, (bf16_t*)out);
    return hipGetLastError();
}

// Scratch for the entry points that may not allocate: one array per GPU, held until the process ends.  In host
// code the array's name is only a handle; its device address is looked up once per device (with that device
// current) and that pointer is what every launch and copy uses.
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

hipError_t static_scratch(void** ptr) {
    constexpr int MAX_DEV = 64;
    static void* per_device[MAX_DEV] = {};
    static std::mutex mu;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= MAX_DEV) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (!per_device[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        per_device[dev] = p;
    }
    *ptr = per_device[dev];
    return hipSuccess;
}

hipError_t colsum(int dtype, int64_t M, int64_t N, const void* X, void* out, float* scratch,
                  hipStream_t s) {
    int64_t slabs = (M + CS_ROWS - 1) / CS_ROWS;
    dim3 g1((unsigned)((N + 511) / 512), (unsigned)slabs), g2((unsigned)((N + 63) / 64));
    if (dtype == F32) {
        hipLaunchKernelGGL(colsum_stage1<float>, g1, dim3(256), 0, s, M, N, (const float*)X, scratch);
        hipLaunchKernelGGL(colsum_stage2<float>, g2, dim3(256), 0, s, slabs, N, N, scratch, (float*)out);
    } else {
        hipLaunchKernelGGL(colsum_stage1<bf16_t>, g1, dim3(256), 0, s, M, N, (const bf16_t*)X, scratch);
        hipLaunchKernelGGL(colsum_stage2<bf16_t>, g2, dim3(256), 0, s, slabs, N, N, scratch, (bf16_t*)out);
    }
    return hipGetLastError();
}

}  // namespace tpl
