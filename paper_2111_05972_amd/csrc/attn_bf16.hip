// bf16 flash-style softmax attention for gfx950 (head size 64 or 128), forward and backward.
//
// qkv is [B*S, 3*nl*dh] with columns (q | k | v, local head, dh); o is [B*S, nl*dh].  The S x S
// score matrix is never stored: scores are recomputed tile by tile on the matrix cores (MFMA
// 32x32x16 bf16, float accumulation), softmax statistics stay in registers, and only
// LSE = max + log(sum) per row is kept for the backward pass.
//
// Register layouts.  An MFMA 32x32 accumulator gives lane l column (l % 32) and rows
// 8*i + 4*(l/32) + j (register 4*i + j).  The forward and the dQ kernel compute the TRANSPOSED score
// tile (rows = keys, columns = queries), so one lane owns one query: row max / row sum are in-lane
// reductions plus one exchange with lane l^32, and the probabilities are already laid out as the
// K-operand of the next MFMA (P never passes through LDS).  The dK/dV kernel computes the
// untransposed tile (lane = key) for the same reason.  Operands that are needed with the other
// dimension contiguous (V in forward, Q and dO in dK/dV, K in dQ) are read from LDS with the
// transposing ds_read_b64_tr_b16.
//
// Backward is two kernels (dK/dV per key block, dQ per query block), each accumulating in registers
// in a fixed order: no atomics, results are run-to-run identical.
#include <hip/hip_runtime.h>

#include "device_math.h"
#include "kernels.h"

namespace tpl {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((address_space(3))) s16x4* lds_s16x4_ptr;

constexpr int AW = 4;              // wavefronts per workgroup
constexpr int ATHREADS = 64 * AW;
constexpr int BLK = 32 * AW;       // rows (queries or keys) owned by a workgroup
constexpr int TILE = 64;           // rows of the streamed operand staged in LDS per step
constexpr float LOG2E = 1.44269504088896340736f;
constexpr float LN2 = 0.69314718055994530942f;

// ---- LDS tile of TILE rows x DH bf16, 16-byte chunks XOR-swizzled by row -------------------------
// Two kinds of read hit these tiles: 16-byte reads of 16 consecutive rows at one chunk (operand with
// the head dimension as K), and transposing 8-byte reads of 4 consecutive rows at two neighbouring
// 32-byte column groups.  The XOR below makes both conflict-free over the 64 banks (256 bytes): the
// bits that separate the 4 rows of a transposing read move the 64-byte column group, the remaining
// row bits move the chunk inside it.
template <int DH> __device__ __forceinline__ int swz(int row) {
    return DH == 64 ? ((((row >> 1) & 1) << 2) | ((row >> 2) & 3))     // 128-byte rows, 8 chunks
                    : (((row & 3) << 2) | ((row >> 2) & 3));           // 256-byte rows, 16 chunks
}
template <int DH> constexpr int tile_bytes() { return TILE * DH * 2; }
template <int DH, int NT> constexpr int NCHUNKS = TILE * DH / 8 / NT;     // 16-byte chunks per thread and tile
template <int DH> constexpr int chunks_per_thread() { return NCHUNKS<DH, ATHREADS>; }

// global -> registers; rows >= nrows read as zero.  base points at row 0, column 0 of the head.
template <int DH, int NT = ATHREADS>
__device__ __forceinline__ void tile_g2r(uint4 (&r)[(NCHUNKS<DH, NT>)], const bf16_t* base,
                                         int64_t ld, int row0, int nrows, int t) {
    constexpr int NC = DH / 8;
#pragma unroll
    for (int i = 0; i < NCHUNKS<DH, NT>; ++i) {
        int q = t + NT * i;
        int row = q / NC, c = q % NC;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (row0 + row < nrows) v = *reinterpret_cast<const uint4*>(base + (int64_t)(row0 + row) * ld + c * 8);
        r[i] = v;
    }
}
template <int DH, int NT = ATHREADS>
__device__ __forceinline__ void tile_r2s(char* tile, const uint4 (&r)[(NCHUNKS<DH, NT>)], int t) {
    constexpr int NC = DH / 8;
#pragma unroll
    for (int i = 0; i < NCHUNKS<DH, NT>; ++i) {
        int q = t + NT * i;
        int row = q / NC, c = q % NC;
        *reinterpret_cast<uint4*>(tile + row * (DH * 2) + ((c ^ swz<DH>(row)) << 4)) = r[i];
    }
}
// MFMA operand with the head dimension as K: row (row_base + lane%32), dh = 16*ks + 8*(lane/32) + 0..7
template <int DH>
__device__ __forceinline__ bf16x8 frag_k(const char* tile, int row_base, int ks, int lane) {
    int row = row_base + (lane & 31);
    int c = 2 * ks + (lane >> 5);
    return *reinterpret_cast<const bf16x8*>(tile + row * (DH * 2) + ((c ^ swz<DH>(row)) << 4));
}
// MFMA operand with the tile's ROW index as K: column (d_base + lane%32); element e = 4h + j holds
// row r_base + 8h + 4*(lane/32) + j, which is the order accumulator registers 0..7 hold their rows.
template <int DH>
__device__ __forceinline__ bf16x8 frag_t(const char* tile, int d_base, int r_base, int lane) {
    int l16 = lane & 15;
    int d = d_base + (lane & 16) + 4 * (l16 & 3);
    bf16x8 out;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        int row = r_base + 8 * h + 4 * (lane >> 5) + (l16 >> 2);
        int off = row * (DH * 2) + ((((d >> 3) ^ swz<DH>(row))) << 4) + (d & 7) * 2;
        s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(tile + off));
        bf16x4 b = __builtin_bit_cast(bf16x4, v);
        out[4 * h + 0] = b[0]; out[4 * h + 1] = b[1]; out[4 * h + 2] = b[2]; out[4 * h + 3] = b[3];
    }
    return out;
}
// The same operand straight from global memory (loop-invariant fragments kept in registers).
template <int DH>
__device__ __forceinline__ bf16x8 frag_k_global(const bf16_t* base, int64_t ld, int row, int nrows,
                                                int ks, int lane) {
    bf16x8 z;
#pragma unroll
    for (int e = 0; e < 8; ++e) z[e] = (bf16_t)0.0f;
    if (row >= nrows) return z;
    return *reinterpret_cast<const bf16x8*>(base + (int64_t)row * ld + 16 * ks + 8 * (lane >> 5));
}
__device__ __forceinline__ bf16x8 pack_regs(const f32x16& a, int first) {
    bf16x8 o;
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = (bf16_t)a[first + e];
    return o;
}
__device__ __forceinline__ f32x16 zero16() {
    f32x16 z;
#pragma unroll
    for (int v = 0; v < 16; ++v) z[v] = 0.0f;
    return z;
}
__device__ __forceinline__ void store4(bf16_t* p, float a, float b, float c, float d) {
    bf16x4 o;
    o[0] = (bf16_t)a; o[1] = (bf16_t)b; o[2] = (bf16_t)c; o[3] = (bf16_t)d;
    *reinterpret_cast<bf16x4*>(p) = o;
}
// 2^x on the hardware transcendental unit (arguments here are <= ~0; results below 2^-126 flush to 0).
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
#define MFMA(a, b, c) __builtin_amdgcn_mfma_f32_32x32x16_bf16((a), (b), (c), 0, 0, 0)

// =================================================================================================
// Forward.  Workgroup = (query block of 128, batch*head), 8 wavefronts: wavefront w owns the 32
// queries of sub-block w % 4 and, of every 64-key tile streamed through double-buffered LDS, the key
// half w / 4.  The two wavefronts of a query sub-block therefore walk half the keys each (half the
// dependent chain, two wavefronts per SIMD to overlap softmax arithmetic with matrix-core work) and
// their (max, sum, O) partials are merged through LDS at the end, always in the same order.
// =================================================================================================
constexpr int FTHREADS = 512;

template <int DH> constexpr int fwd_lds_bytes() {
    constexpr int ring = 4 * tile_bytes<DH>();
    constexpr int merge = 4 * 64 * (2 + DH / 2) * 4;      // per query sub-block and lane: m, l, O[DH/2]
    return ring > merge ? ring : merge;
}

template <int DH, bool CAUSAL>
__global__ __launch_bounds__(FTHREADS) void attn_fwd_kernel(const bf16_t* __restrict__ qkv,
                                                            bf16_t* __restrict__ o,
                                                            float* __restrict__ lse, int S, int nl) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    constexpr int TB = tile_bytes<DH>();
    constexpr int NCH = NCHUNKS<DH, FTHREADS>;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6, half = lane >> 5;
    const int qs = wave & 3, kvh = wave >> 2;
    const int nqb = (S + BLK - 1) / BLK;
    const int qb = nqb - 1 - (int)blockIdx.x;            // longest (last) causal blocks first
    const int b = blockIdx.y / nl, h = blockIdx.y % nl;
    const int64_t ld = 3LL * nl * DH;
    const bf16_t* qbase = qkv + (int64_t)b * S * ld + (int64_t)h * DH;
    const bf16_t* kbase = qbase + (int64_t)nl * DH;
    const bf16_t* vbase = kbase + (int64_t)nl * DH;
    const int q0 = qb * BLK + qs * 32;                    // first query of this wavefront
    const int q = q0 + (lane & 31);                       // this lane's query
    const float c2 = LOG2E / sqrtf((float)DH);

    bf16x8 qf[DH / 16];
#pragma unroll
    for (int ks = 0; ks < DH / 16; ++ks) qf[ks] = frag_k_global<DH>(qbase, ld, q, S, ks, lane);

    f32x16 oacc[DH / 32];
#pragma unroll
    for (int dt = 0; dt < DH / 32; ++dt) oacc[dt] = zero16();
    float m = -INFINITY, lsum = 0.0f;

    const int kv_end = CAUSAL ? min(S, (qb + 1) * BLK) : S;
    const int ntiles = (kv_end + TILE - 1) / TILE;
    uint4 rk[NCH], rv[NCH];
    tile_g2r<DH, FTHREADS>(rk, kbase, ld, 0, S, t);
    tile_g2r<DH, FTHREADS>(rv, vbase, ld, 0, S, t);
    tile_r2s<DH, FTHREADS>(smem, rk, t);
    tile_r2s<DH, FTHREADS>(smem + TB, rv, t);
    __syncthreads();
    for (int kt = 0; kt < ntiles; ++kt) {
        const char* ks_ = smem + (kt & 1) * 2 * TB;
        const char* vs_ = ks_ + TB;
        char* nxt = smem + ((kt + 1) & 1) * 2 * TB;
        const bool more = kt + 1 < ntiles;
        if (more) {
            tile_g2r<DH, FTHREADS>(rk, kbase, ld, (kt + 1) * TILE, S, t);
            tile_g2r<DH, FTHREADS>(rv, vbase, ld, (kt + 1) * TILE, S, t);
        }
        const int kv0 = kt * TILE + kvh * 32;
        if (kv0 < kv_end && !(CAUSAL && kv0 > q0 + 31)) {                 // wavefront-uniform
            f32x16 s = zero16();
#pragma unroll
            for (int ks = 0; ks < DH / 16; ++ks) s = MFMA(frag_k<DH>(ks_, kvh * 32, ks, lane), qf[ks], s);
            // masking is needed only in tiles that straddle the diagonal or the end of the sequence
            if (kv0 + 31 >= S || (CAUSAL && kv0 + 31 > q0)) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    int kv = kv0 + (v >> 2) * 8 + half * 4 + (v & 3);
                    bool ok = kv < S && (!CAUSAL || kv <= q);
                    s[v] = ok ? s[v] : -INFINITY;
                }
            }
            float mb = s[0];
#pragma unroll
            for (int v = 1; v < 16; ++v) mb = fmaxf(mb, s[v]);
            mb = fmaxf(mb, __shfl_xor(mb, 32, 64)) * c2;      // c2 > 0: scaling commutes with max
            float mn = fmaxf(m, mb);
            float mu = mn == -INFINITY ? 0.0f : mn;
            float alpha = fast_exp2(m - mu);
            m = mn;
            float ps = 0.0f;
#pragma unroll
            for (int v = 0; v < 16; ++v) { s[v] = fast_exp2(fmaf(s[v], c2, -mu)); ps += s[v]; }
            lsum = lsum * alpha + ps;
            if (__any(alpha != 1.0f)) {                       // the running maximum rarely moves
#pragma unroll
                for (int dt = 0; dt < DH / 32; ++dt)
#pragma unroll
                    for (int v = 0; v < 16; ++v) oacc[dt][v] *= alpha;
            }
            bf16x8 pb0 = pack_regs(s, 0), pb1 = pack_regs(s, 8);
#pragma unroll
            for (int dt = 0; dt < DH / 32; ++dt) {
                oacc[dt] = MFMA(frag_t<DH>(vs_, dt * 32, kvh * 32, lane), pb0, oacc[dt]);
                oacc[dt] = MFMA(frag_t<DH>(vs_, dt * 32, kvh * 32 + 16, lane), pb1, oacc[dt]);
            }
        }
        if (more) {
            tile_r2s<DH, FTHREADS>(nxt, rk, t);
            tile_r2s<DH, FTHREADS>(nxt + TB, rv, t);
        }
        __syncthreads();
    }
    lsum += __shfl_xor(lsum, 32, 64);
    // merge the two key halves: wavefronts 4..7 hand (m, l, O) to wavefronts 0..3 through LDS
    constexpr int NV = 2 + DH / 2;
    float* mg = reinterpret_cast<float*>(smem) + (qs * NV) * 64 + lane;   // element i at mg[i * 64]
    if (kvh == 1) {
        mg[0] = m; mg[64] = lsum;
#pragma unroll
        for (int dt = 0; dt < DH / 32; ++dt)
#pragma unroll
            for (int v = 0; v < 16; ++v) mg[(2 + dt * 16 + v) * 64] = oacc[dt][v];
    }
    __syncthreads();
    if (kvh == 0) {
        const float m1 = mg[0], l1 = mg[64];
        const float mn = fmaxf(m, m1);
        const float mu = mn == -INFINITY ? 0.0f : mn;
        const float f0 = fast_exp2(m - mu), f1 = fast_exp2(m1 - mu);
        const float ltot = lsum * f0 + l1 * f1;
        const float inv = ltot > 0.0f ? 1.0f / ltot : 0.0f;
        if (q < S) {
            bf16_t* op = o + ((int64_t)b * S + q) * ((int64_t)nl * DH) + (int64_t)h * DH;
#pragma unroll
            for (int dt = 0; dt < DH / 32; ++dt)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    float r[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        r[j] = (oacc[dt][4 * i + j] * f0 + mg[(2 + dt * 16 + 4 * i + j) * 64] * f1) * inv;
                    store4(op + dt * 32 + 8 * i + 4 * half, r[0], r[1], r[2], r[3]);
                }
            if (half == 0) lse[((int64_t)b * nl + h) * S + q] = (mn + log2f(ltot)) * LN2;
        }
    }
}

// =================================================================================================
// D[b,h,s] = sum_d dO[s,d] * O[s,d]   (one wavefront per token row, 8 elements per lane per pass)
// =================================================================================================
template <int DH>
__global__ __launch_bounds__(256) void attn_dsum_kernel(const bf16_t* __restrict__ o,
                                                        const bf16_t* __restrict__ d_o,
                                                        float* __restrict__ dsum, int B, int S, int nl) {
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= (int64_t)B * S) return;
    const int b = (int)(row / S), s = (int)(row % S);
    const int Hl = nl * DH;
    constexpr int LPH = DH / 8;     // lanes per head
    for (int c0 = 0; c0 < Hl; c0 += 512) {
        int c = c0 + lane * 8;
        float acc = 0.0f;
        if (c < Hl) {
            bf16x8 a = *reinterpret_cast<const bf16x8*>(o + row * Hl + c);
            bf16x8 g = *reinterpret_cast<const bf16x8*>(d_o + row * Hl + c);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc = fmaf((float)a[e], (float)g[e], acc);
        }
#pragma unroll
        for (int off = LPH / 2; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
        if (c < Hl && (lane % LPH) == 0) dsum[((int64_t)b * nl + c / DH) * S + s] = acc;
    }
}

// =================================================================================================
// dK, dV.  Workgroup = (key block of 128, batch*head), 8 wavefronts: wavefront w owns the 32 keys of
// sub-block w % 4; wavefronts 0..3 accumulate dV = P^T dO (they need the scores only), wavefronts 4..7
// accumulate dK = dS^T Q (scores and dP).  The scores are computed by both, which costs a quarter more
// matrix-core work but halves the accumulators and fragments a wavefront holds (two wavefronts per
// SIMD) and shortens its dependent chain per tile.  Q, dO (and LSE, D) are streamed in tiles of 64
// queries.  Score tile is untransposed: lane = key (l%32), registers = queries 8i + 4*(l/32) + j.
// =================================================================================================
template <int DH, bool CAUSAL, bool DK_ROLE>
__device__ __forceinline__ void attn_dkv_body(char* smem, const bf16_t* __restrict__ qkv,
                                              const bf16_t* __restrict__ d_o, const float* __restrict__ lse,
                                              const float* __restrict__ dsum, bf16_t* __restrict__ dqkv,
                                              int S, int nl) {
    constexpr int TB = tile_bytes<DH>();
    constexpr int NCH = NCHUNKS<DH, FTHREADS>;
    constexpr int STAGE = 2 * TB + 2 * TILE * 4;          // Q tile, dO tile, LSE*log2e, D
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6, half = lane >> 5;
    const int kb = blockIdx.x;
    const int b = blockIdx.y / nl, h = blockIdx.y % nl;
    const int64_t ld = 3LL * nl * DH, ldo = (int64_t)nl * DH;
    const bf16_t* qbase = qkv + (int64_t)b * S * ld + (int64_t)h * DH;
    const bf16_t* kbase = qbase + (int64_t)nl * DH;
    const bf16_t* vbase = kbase + (int64_t)nl * DH;
    const bf16_t* dobase = d_o + (int64_t)b * S * ldo + (int64_t)h * DH;
    const float* lrow = lse + ((int64_t)b * nl + h) * S;
    const float* drow = dsum + ((int64_t)b * nl + h) * S;
    const int k0 = kb * BLK + (wave & 3) * 32;
    const int kv = k0 + (lane & 31);
    const float scale = 1.0f / sqrtf((float)DH);
    const float c2 = LOG2E * scale;

    bf16x8 kf[DH / 16], vf[DK_ROLE ? DH / 16 : 1];
#pragma unroll
    for (int ks = 0; ks < DH / 16; ++ks) {
        kf[ks] = frag_k_global<DH>(kbase, ld, kv, S, ks, lane);
        if (DK_ROLE) vf[ks] = frag_k_global<DH>(vbase, ld, kv, S, ks, lane);
    }
    f32x16 acc[DH / 32];                                   // dK (DK_ROLE) or dV
#pragma unroll
    for (int dt = 0; dt < DH / 32; ++dt) acc[dt] = zero16();

    const int qt0 = CAUSAL ? (kb * BLK) / TILE : 0;       // first query tile that can see this key block
    const int ntiles = (S + TILE - 1) / TILE;
    uint4 rq[NCH], rdo[NCH];
    float rl = 0.0f, rd = 0.0f;
    auto g2r = [&](int qt) {
        tile_g2r<DH, FTHREADS>(rq, qbase, ld, qt * TILE, S, t);
        tile_g2r<DH, FTHREADS>(rdo, dobase, ldo, qt * TILE, S, t);
        if (t < TILE) {
            int qi = qt * TILE + t;
            rl = qi < S ? lrow[qi] * LOG2E : 0.0f;
            rd = qi < S ? drow[qi] : 0.0f;
        }
    };
    auto r2s = [&](char* st) {
        tile_r2s<DH, FTHREADS>(st, rq, t);
        tile_r2s<DH, FTHREADS>(st + TB, rdo, t);
        if (t < TILE) {
            reinterpret_cast<float*>(st + 2 * TB)[t] = rl;
            reinterpret_cast<float*>(st + 2 * TB)[TILE + t] = rd;
        }
    };
    if (qt0 < ntiles) { g2r(qt0); r2s(smem); }
    __syncthreads();
    for (int qt = qt0; qt < ntiles; ++qt) {
        const char* st = smem + ((qt - qt0) & 1) * STAGE;
        char* nxt = smem + ((qt - qt0 + 1) & 1) * STAGE;
        const char* qs = st;
        const char* dos = st + TB;
        const float* ls = reinterpret_cast<const float*>(st + 2 * TB);
        const float* ds_ = ls + TILE;
        const bool more = qt + 1 < ntiles;
        if (more) g2r(qt + 1);
#pragma unroll
        for (int sb = 0; sb < 2; ++sb) {
            const int qs0 = qt * TILE + sb * 32;
            if (qs0 >= S || (CAUSAL && qs0 + 31 < k0)) continue;          // wavefront-uniform
            f32x16 s = zero16(), dp = zero16();
#pragma unroll
            for (int ks = 0; ks < DH / 16; ++ks) {
                s = MFMA(frag_k<DH>(qs, sb * 32, ks, lane), kf[ks], s);
                if (DK_ROLE) dp = MFMA(frag_k<DH>(dos, sb * 32, ks, lane), vf[ks], dp);
            }
            const bool need_mask = qs0 + 31 >= S || k0 + 31 >= S || (CAUSAL && k0 + 31 > qs0);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float4 l4 = *reinterpret_cast<const float4*>(ls + sb * 32 + 8 * i + 4 * half);
                float4 d4 = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
                if (DK_ROLE) d4 = *reinterpret_cast<const float4*>(ds_ + sb * 32 + 8 * i + 4 * half);
                const float lv[4] = {l4.x, l4.y, l4.z, l4.w}, dvv[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    int v = 4 * i + j;
                    float p = fast_exp2(fmaf(s[v], c2, -lv[j]));
                    if (need_mask) {
                        int qi = qs0 + 8 * i + 4 * half + j;
                        bool ok = qi < S && kv < S && (!CAUSAL || kv <= qi);
                        p = ok ? p : 0.0f;
                    }
                    s[v] = DK_ROLE ? p * (dp[v] - dvv[j]) : p;             // dS, or P
                }
            }
            bf16x8 g0 = pack_regs(s, 0), g1 = pack_regs(s, 8);
            const char* src = DK_ROLE ? qs : dos;                          // dK += dS^T Q ; dV += P^T dO
#pragma unroll
            for (int dt = 0; dt < DH / 32; ++dt) {
                acc[dt] = MFMA(frag_t<DH>(src, dt * 32, sb * 32, lane), g0, acc[dt]);
                acc[dt] = MFMA(frag_t<DH>(src, dt * 32, sb * 32 + 16, lane), g1, acc[dt]);
            }
        }
        if (more) r2s(nxt);
        __syncthreads();
    }
    if (kv < S) {
        bf16_t* outp = dqkv + ((int64_t)b * S + kv) * ld + (int64_t)(DK_ROLE ? 1 : 2) * nl * DH + (int64_t)h * DH;
        const float f = DK_ROLE ? scale : 1.0f;
#pragma unroll
        for (int dt = 0; dt < DH / 32; ++dt)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                store4(outp + dt * 32 + 8 * i + 4 * half, acc[dt][4 * i] * f, acc[dt][4 * i + 1] * f,
                       acc[dt][4 * i + 2] * f, acc[dt][4 * i + 3] * f);
    }
}

template <int DH, bool CAUSAL>
__global__ __launch_bounds__(FTHREADS) void attn_dkv_kernel(const bf16_t* __restrict__ qkv,
                                                            const bf16_t* __restrict__ d_o,
                                                            const float* __restrict__ lse,
                                                            const float* __restrict__ dsum,
                                                            bf16_t* __restrict__ dqkv, int S, int nl) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    // the role is uniform per wavefront; both bodies run the same loop and the same barriers
    if ((threadIdx.x >> 6) < 4) attn_dkv_body<DH, CAUSAL, false>(smem, qkv, d_o, lse, dsum, dqkv, S, nl);
    else attn_dkv_body<DH, CAUSAL, true>(smem, qkv, d_o, lse, dsum, dqkv, S, nl);
}

// =================================================================================================
// dQ.  Same decomposition as the forward: 8 wavefronts, wavefront w owns query sub-block w % 4 (its Q
// and dO fragments stay in registers) and key half w / 4 of every streamed 64-key tile; the two dQ
// partials of a sub-block are added through LDS in a fixed order.  Transposed score tile: lane = query.
// =================================================================================================
template <int DH> constexpr int dq_lds_bytes() {
    constexpr int ring = 4 * tile_bytes<DH>();
    constexpr int merge = 4 * 64 * (DH / 2) * 4;
    return ring > merge ? ring : merge;
}

template <int DH, bool CAUSAL>
__global__ __launch_bounds__(FTHREADS) void attn_dq_kernel(const bf16_t* __restrict__ qkv,
                                                           const bf16_t* __restrict__ d_o,
                                                           const float* __restrict__ lse,
                                                           const float* __restrict__ dsum,
                                                           bf16_t* __restrict__ dqkv, int S, int nl) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    constexpr int TB = tile_bytes<DH>();
    constexpr int NCH = NCHUNKS<DH, FTHREADS>;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6, half = lane >> 5;
    const int qs = wave & 3, kvh = wave >> 2;
    const int nqb = (S + BLK - 1) / BLK;
    const int qb = nqb - 1 - (int)blockIdx.x;
    const int b = blockIdx.y / nl, h = blockIdx.y % nl;
    const int64_t ld = 3LL * nl * DH, ldo = (int64_t)nl * DH;
    const bf16_t* qbase = qkv + (int64_t)b * S * ld + (int64_t)h * DH;
    const bf16_t* kbase = qbase + (int64_t)nl * DH;
    const bf16_t* vbase = kbase + (int64_t)nl * DH;
    const bf16_t* dobase = d_o + (int64_t)b * S * ldo + (int64_t)h * DH;
    const int q0 = qb * BLK + qs * 32;
    const int q = q0 + (lane & 31);
    const float scale = 1.0f / sqrtf((float)DH);
    const float c2 = LOG2E * scale;
    const float l2 = q < S ? lse[((int64_t)b * nl + h) * S + q] * LOG2E : 0.0f;
    const float dq_d = q < S ? dsum[((int64_t)b * nl + h) * S + q] : 0.0f;

    bf16x8 qf[DH / 16], dof[DH / 16];
#pragma unroll
    for (int ks = 0; ks < DH / 16; ++ks) {
        qf[ks] = frag_k_global<DH>(qbase, ld, q, S, ks, lane);
        dof[ks] = frag_k_global<DH>(dobase, ldo, q, S, ks, lane);
    }
    f32x16 dq[DH / 32];
#pragma unroll
    for (int dt = 0; dt < DH / 32; ++dt) dq[dt] = zero16();

    const int kv_end = CAUSAL ? min(S, (qb + 1) * BLK) : S;
    const int ntiles = (kv_end + TILE - 1) / TILE;
    uint4 rk[NCH], rv[NCH];
    tile_g2r<DH, FTHREADS>(rk, kbase, ld, 0, S, t);
    tile_g2r<DH, FTHREADS>(rv, vbase, ld, 0, S, t);
    tile_r2s<DH, FTHREADS>(smem, rk, t);
    tile_r2s<DH, FTHREADS>(smem + TB, rv, t);
    __syncthreads();
    for (int kt = 0; kt < ntiles; ++kt) {
        const char* ks_ = smem + (kt & 1) * 2 * TB;
        const char* vs_ = ks_ + TB;
        char* nxt = smem + ((kt + 1) & 1) * 2 * TB;
        const bool more = kt + 1 < ntiles;
        if (more) {
            tile_g2r<DH, FTHREADS>(rk, kbase, ld, (kt + 1) * TILE, S, t);
            tile_g2r<DH, FTHREADS>(rv, vbase, ld, (kt + 1) * TILE, S, t);
        }
        const int kv0 = kt * TILE + kvh * 32;
        if (kv0 < kv_end && !(CAUSAL && kv0 > q0 + 31)) {                 // wavefront-uniform
            f32x16 s = zero16(), dp = zero16();
#pragma unroll
            for (int ks = 0; ks < DH / 16; ++ks) {
                s = MFMA(frag_k<DH>(ks_, kvh * 32, ks, lane), qf[ks], s);
                dp = MFMA(frag_k<DH>(vs_, kvh * 32, ks, lane), dof[ks], dp);
            }
            const bool need_mask = q0 + 31 >= S || kv0 + 31 >= S || (CAUSAL && kv0 + 31 > q0);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                float p = fast_exp2(fmaf(s[v], c2, -l2));
                if (need_mask) {
                    int kv = kv0 + (v >> 2) * 8 + half * 4 + (v & 3);
                    bool ok = q < S && kv < S && (!CAUSAL || kv <= q);
                    p = ok ? p : 0.0f;
                }
                dp[v] = p * (dp[v] - dq_d);
            }
            bf16x8 g0 = pack_regs(dp, 0), g1 = pack_regs(dp, 8);
#pragma unroll
            for (int dt = 0; dt < DH / 32; ++dt) {
                dq[dt] = MFMA(frag_t<DH>(ks_, dt * 32, kvh * 32, lane), g0, dq[dt]);
                dq[dt] = MFMA(frag_t<DH>(ks_, dt * 32, kvh * 32 + 16, lane), g1, dq[dt]);
            }
        }
        if (more) {
            tile_r2s<DH, FTHREADS>(nxt, rk, t);
            tile_r2s<DH, FTHREADS>(nxt + TB, rv, t);
        }
        __syncthreads();
    }
    float* mg = reinterpret_cast<float*>(smem) + (qs * (DH / 2)) * 64 + lane;   // element i at mg[i * 64]
    if (kvh == 1) {
#pragma unroll
        for (int dt = 0; dt < DH / 32; ++dt)
#pragma unroll
            for (int v = 0; v < 16; ++v) mg[(dt * 16 + v) * 64] = dq[dt][v];
    }
    __syncthreads();
    if (kvh == 0 && q < S) {
        bf16_t* dqp = dqkv + ((int64_t)b * S + q) * ld + (int64_t)h * DH;
#pragma unroll
        for (int dt = 0; dt < DH / 32; ++dt)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float r[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) r[j] = (dq[dt][4 * i + j] + mg[(dt * 16 + 4 * i + j) * 64]) * scale;
                store4(dqp + dt * 32 + 8 * i + 4 * half, r[0], r[1], r[2], r[3]);
            }
    }
}

// ---- host side ----------------------------------------------------------------------------------
bool attn_bf16_supported(const AttnArgs& a) {
    return a.dtype == BF16 && (a.dh == 64 || a.dh == 128) && a.S >= 1 && (int64_t)a.B * a.nl <= 65535;
}

template <typename K>
static hipError_t set_lds(K kernel, int bytes) {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
}

template <int DH, bool CAUSAL>
static hipError_t fwd_t(const AttnArgs& a) {
    constexpr int LDS = fwd_lds_bytes<DH>();
    static bool once = false;
    if (!once) {
        hipError_t e = set_lds(&attn_fwd_kernel<DH, CAUSAL>, LDS);
        if (e != hipSuccess) return e;
        once = true;
    }
    dim3 grid((a.S + BLK - 1) / BLK, a.B * a.nl);
    hipLaunchKernelGGL((attn_fwd_kernel<DH, CAUSAL>), grid, dim3(FTHREADS), LDS, a.stream,
                       (const bf16_t*)a.qkv, (bf16_t*)a.o, a.lse, a.S, a.nl);
    return hipGetLastError();
}

template <int DH, bool CAUSAL>
static hipError_t bwd_t(const AttnArgs& a) {
    constexpr int LDS_KV = 2 * (2 * tile_bytes<DH>() + 2 * TILE * 4);
    constexpr int LDS_Q = dq_lds_bytes<DH>();
    static bool once = false;
    if (!once) {
        hipError_t e = set_lds(&attn_dkv_kernel<DH, CAUSAL>, LDS_KV);
        if (e != hipSuccess) return e;
        e = set_lds(&attn_dq_kernel<DH, CAUSAL>, LDS_Q);
        if (e != hipSuccess) return e;
        once = true;
    }
    const int64_t rows = (int64_t)a.B * a.S;
    hipLaunchKernelGGL((attn_dsum_kernel<DH>), dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, a.stream,
                       (const bf16_t*)a.o, (const bf16_t*)a.d_o, a.dsum, a.B, a.S, a.nl);
    dim3 grid((a.S + BLK - 1) / BLK, a.B * a.nl);
    hipLaunchKernelGGL((attn_dkv_kernel<DH, CAUSAL>), grid, dim3(FTHREADS), LDS_KV, a.stream,
                       (const bf16_t*)a.qkv, (const bf16_t*)a.d_o, a.lse, a.dsum, (bf16_t*)a.dqkv, a.S, a.nl);
    hipLaunchKernelGGL((attn_dq_kernel<DH, CAUSAL>), grid, dim3(FTHREADS), LDS_Q, a.stream,
                       (const bf16_t*)a.qkv, (const bf16_t*)a.d_o, a.lse, a.dsum, (bf16_t*)a.dqkv, a.S, a.nl);
    return hipGetLastError();
}

hipError_t attn_bf16_fwd(const AttnArgs& a) {
    if (a.dh == 64) return a.causal ? fwd_t<64, true>(a) : fwd_t<64, false>(a);
    return a.causal ? fwd_t<128, true>(a) : fwd_t<128, false>(a);
}
hipError_t attn_bf16_bwd(const AttnArgs& a) {
    if (a.dh == 64) return a.causal ? bwd_t<64, true>(a) : bwd_t<64, false>(a);
    return a.causal ? bwd_t<128, true>(a) : bwd_t<128, false>(a);
}

}  // namespace tpl
