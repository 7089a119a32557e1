// bf16 GEMM for gfx950: C[M,N] = epi(opA(A) opB(B)), float accumulation on the matrix cores.
//
// One 512-thread workgroup (8 wavefronts, 2 x 4) owns a 256 x 256 output tile and walks K in steps
// of 64.  Operand tiles are staged global -> registers -> LDS, double buffered, one barrier per
// step.  Each wavefront accumulates a 128 x 64 sub-tile as 4 x 2 MFMA 32x32x16 blocks (128
// accumulator registers per lane).
//
// Either operand may be stored with K contiguous ("K-major": A as [M,K], B as [N,K]) or with its
// M/N dimension contiguous ("MN-major": A as [K,M], B as [K,N]).  K-major tiles are read from LDS
// with 16-byte reads; MN-major tiles with the transposing ds_read_b64_tr_b16, which hands each lane
// four K-consecutive values of one column, so no operand is ever transposed in HBM or registers.
//
// The epilogue goes through LDS (per-wavefront regions, no workgroup barrier) so that every global
// access of the epilogue is a 16-byte access and eight lanes cover 128 contiguous bytes of a row.
#include <hip/hip_runtime.h>

#include "device_math.h"
#include "kernels.h"

namespace tpl {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((address_space(3))) s16x4* lds_s16x4_ptr;

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int NTHREADS = 512;
constexpr int STAGE_BYTES = (BM + BN) * BK * 2;          // 64 KiB: A tile then B tile
constexpr int EPI_ROW_BYTES = 64 * 4 + 16;               // one 64-float row of a wavefront's staging area
constexpr int EPI_WAVE_BYTES = 32 * EPI_ROW_BYTES;       // 32 rows per round
constexpr int LDS_BYTES = 2 * STAGE_BYTES;               // 128 KiB (epilogue staging reuses it)
static_assert(8 * EPI_WAVE_BYTES <= LDS_BYTES, "epilogue staging must fit in the operand buffers");

struct GemmParams {
    const bf16_t* A; const bf16_t* B; bf16_t* C;
    const bf16_t* bias; const bf16_t* resid; bf16_t* aux;
    int M, N, K;
    int lda, ldb;          // row strides (elements) of A and B as stored
    int epi;
    int tiles_m, tiles_n;
};

// ---- LDS layouts -------------------------------------------------------------------------------
// K-major tile: 128-byte rows (64 k), eight 16-byte chunks per row, chunk index XOR-swizzled by row.
__device__ __forceinline__ int swz_k(int row) { return (row >> 1) & 7; }
// MN-major tile: 512-byte rows (256 m or n) per k, thirty-two 16-byte chunks, swizzled by k.
__device__ __forceinline__ int swz_mn(int k) { return (k & 3) << 2; }

// ---- global -> registers (4 x 16 bytes per thread and operand), zero filled outside the matrix ---
template <bool KMAJ>
__device__ __forceinline__ void load_global(uint4 (&r)[4], const bf16_t* __restrict__ base, int ld,
                                            int mn0, int k0, int MN, int K, int t) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int row, col;   // row of the stored matrix, first element column of the chunk
        bool ok;
        if (KMAJ) {
            row = mn0 + (t >> 3) + 64 * i; col = k0 + (t & 7) * 8;
            ok = row < MN && col < K;
        } else {
            row = k0 + (t >> 5) + 16 * i; col = mn0 + (t & 31) * 8;
            ok = row < K && col < MN;
        }
        uint4 v = make_uint4(0, 0, 0, 0);
        if (ok) v = *reinterpret_cast<const uint4*>(base + (int64_t)row * ld + col);
        r[i] = v;
    }
}

template <bool KMAJ>
__device__ __forceinline__ void store_lds(char* tile, const uint4 (&r)[4], int t) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int off;
        if (KMAJ) {
            int row = (t >> 3) + 64 * i, c = t & 7;
            off = row * 128 + ((c ^ swz_k(row)) << 4);
        } else {
            int k = (t >> 5) + 16 * i, c = t & 31;
            off = k * 512 + ((c ^ swz_mn(k)) << 4);
        }
        *reinterpret_cast<uint4*>(tile + off) = r[i];
    }
}

// ---- LDS -> MFMA fragment: rows mn_base + (lane % 32), k = ks*16 + 8*(lane/32) + 0..7 -----------
template <bool KMAJ>
__device__ __forceinline__ bf16x8 load_frag(const char* tile, int mn_base, int ks, int lane) {
    if (KMAJ) {
        int row = mn_base + (lane & 31);
        int c = 2 * ks + (lane >> 5);
        return *reinterpret_cast<const bf16x8*>(tile + row * 128 + ((c ^ swz_k(row)) << 4));
    } else {
        // Two transposing reads; in each 16-lane group lane l points at (k = kb + l/4, 4 columns at
        // 4*(l%4)) and receives k = kb..kb+3 of column l.
        int l16 = lane & 15;
        int mn = mn_base + (lane & 16) + 4 * (l16 & 3);
        int kq = l16 >> 2;
        int kb = ks * 16 + 8 * (lane >> 5);
        bf16x8 out;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            int k = kb + 4 * h + kq;
            int off = k * 512 + ((((mn >> 3) ^ swz_mn(k))) << 4) + (mn & 7) * 2;
            s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(tile + off));
            bf16x4 b = __builtin_bit_cast(bf16x4, v);
            out[4 * h + 0] = b[0]; out[4 * h + 1] = b[1]; out[4 * h + 2] = b[2]; out[4 * h + 3] = b[3];
        }
        return out;
    }
}

__device__ __forceinline__ void unpack8(const uint4& v, float (&f)[8]) {
    const unsigned u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        f[2 * i] = __uint_as_float(u[i] << 16);
        f[2 * i + 1] = __uint_as_float(u[i] & 0xffff0000u);
    }
}
__device__ __forceinline__ uint4 pack8(const float (&f)[8]) {
    unsigned u[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        bf16_t lo = (bf16_t)f[2 * i], hi = (bf16_t)f[2 * i + 1];
        u[i] = (unsigned)__builtin_bit_cast(unsigned short, lo) |
               ((unsigned)__builtin_bit_cast(unsigned short, hi) << 16);
    }
    return make_uint4(u[0], u[1], u[2], u[3]);
}

// XCD-aware tile order: consecutive workgroup ids go to different XCDs (each with its own L2), so
// ids are first regrouped so that one XCD works on a contiguous run of tiles, and runs are laid out
// column-major in bands of 8 tile rows so that the tiles in flight on an XCD share A and B panels.
__device__ __forceinline__ void tile_of_block(int bid, int nblocks, int tiles_m, int tiles_n,
                                              int& tm, int& tn) {
    constexpr int NXCD = 8, BAND = 8;
    int per = nblocks / NXCD, rem = nblocks % NXCD;
    int xcd = bid % NXCD, idx = bid / NXCD;
    int logical = xcd * per + (xcd < rem ? xcd : rem) + idx;
    int band_tiles = BAND * tiles_n;
    int band = logical / band_tiles, within = logical % band_tiles;
    int rows = tiles_m - band * BAND;
    rows = rows < BAND ? rows : BAND;
    tm = band * BAND + within % rows;
    tn = within / rows;
}

template <bool A_KMAJ, bool B_KMAJ>
__global__ __launch_bounds__(NTHREADS) void gemm_bf16_kernel(GemmParams p) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave >> 2, wn = wave & 3;      // 2 x 4 wavefronts, each 128 x 64
    int tm, tn;
    tile_of_block(blockIdx.x, gridDim.x, p.tiles_m, p.tiles_n, tm, tn);
    const int m0 = tm * BM, n0 = tn * BN;

    f32x16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    const int nk = (p.K + BK - 1) / BK;
    uint4 ra[4], rb[4];
    load_global<A_KMAJ>(ra, p.A, p.lda, m0, 0, p.M, p.K, t);
    load_global<B_KMAJ>(rb, p.B, p.ldb, n0, 0, p.N, p.K, t);
    store_lds<A_KMAJ>(smem, ra, t);
    store_lds<B_KMAJ>(smem + BM * BK * 2, rb, t);
    __syncthreads();

    for (int kt = 0; kt < nk; ++kt) {
        char* cur = smem + (kt & 1) * STAGE_BYTES;
        char* nxt = smem + ((kt + 1) & 1) * STAGE_BYTES;
        const bool more = kt + 1 < nk;
        if (more) {
            load_global<A_KMAJ>(ra, p.A, p.lda, m0, (kt + 1) * BK, p.M, p.K, t);
            load_global<B_KMAJ>(rb, p.B, p.ldb, n0, (kt + 1) * BK, p.N, p.K, t);
        }
        const char* sa = cur;
        const char* sb = cur + BM * BK * 2;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            bf16x8 fa[4], fb[2];
#pragma unroll
            for (int i = 0; i < 4; ++i) fa[i] = load_frag<A_KMAJ>(sa, wm * 128 + i * 32, ks, lane);
#pragma unroll
            for (int j = 0; j < 2; ++j) fb[j] = load_frag<B_KMAJ>(sb, wn * 64 + j * 32, ks, lane);
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
        if (more) {
            store_lds<A_KMAJ>(nxt, ra, t);
            store_lds<B_KMAJ>(nxt + BM * BK * 2, rb, t);
        }
        __syncthreads();
    }

    // ---- epilogue: accumulators -> per-wavefront LDS staging -> 16-byte row accesses ------------
    char* stage = smem + wave * EPI_WAVE_BYTES;
    const int er = lane >> 3, ec = (lane & 7) * 8;     // this lane's row (of 8) and first column
    const int gn = n0 + wn * 64 + ec;
    float bias8[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (p.bias && gn < p.N) unpack8(*reinterpret_cast<const uint4*>(p.bias + gn), bias8);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        // accumulator register v of block (i,j): row (v/4)*8 + (lane/32)*4 + v%4, column j*32 + lane%32
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                int row = (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
                *reinterpret_cast<float*>(stage + row * EPI_ROW_BYTES + (j * 32 + (lane & 31)) * 4) = acc[i][j][v];
            }
#pragma unroll
        for (int pass = 0; pass < 4; ++pass) {
            int row = pass * 8 + er;
            int gm = m0 + wm * 128 + i * 32 + row;
            const float4* src = reinterpret_cast<const float4*>(stage + row * EPI_ROW_BYTES + ec * 4);
            float4 x0 = src[0], x1 = src[1];
            if (gm < p.M && gn < p.N) {
                float v8[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
                const int64_t idx = (int64_t)gm * p.N + gn;
#pragma unroll
                for (int e = 0; e < 8; ++e) v8[e] += bias8[e];
                if (p.resid) {
                    float r8[8];
                    unpack8(*reinterpret_cast<const uint4*>(p.resid + idx), r8);
#pragma unroll
                    for (int e = 0; e < 8; ++e) v8[e] += r8[e];
                }
                if (p.epi == EPI_GELU) {
                    *reinterpret_cast<uint4*>(p.aux + idx) = pack8(v8);
#pragma unroll
                    for (int e = 0; e < 8; ++e) v8[e] = gelu_f(v8[e]);
                } else if (p.epi == EPI_DGELU) {
                    float u8[8];
                    unpack8(*reinterpret_cast<const uint4*>(p.aux + idx), u8);
#pragma unroll
                    for (int e = 0; e < 8; ++e) v8[e] *= gelu_grad_f(u8[e]);
                }
                *reinterpret_cast<uint4*>(p.C + idx) = pack8(v8);
            }
        }
    }
}

bool gemm_bf16_supported(const GemmArgs& a) {
    if (a.dtype != BF16) return false;
    if (a.M % 8 || a.N % 8 || a.K % 8) return false;
    if (a.M > (1 << 30) || a.N > (1 << 30) || a.K > (1 << 30)) return false;
    int64_t tiles = ((a.M + BM - 1) / BM) * ((a.N + BN - 1) / BN);
    return tiles < (1 << 30);
}

size_t gemm_bf16_workspace_bytes(int64_t, int64_t, int64_t) { return 0; }

template <bool AK, bool BK_>
static hipError_t launch(const GemmParams& p, hipStream_t s) {
    static bool attr_set = false;   // raising the dynamic LDS limit is a per-function, one-off call
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_bf16_kernel<AK, BK_>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL((gemm_bf16_kernel<AK, BK_>), dim3(p.tiles_m * p.tiles_n), dim3(NTHREADS),
                       LDS_BYTES, s, p);
    return hipGetLastError();
}

hipError_t gemm_bf16(const GemmArgs& a) {
    GemmParams p;
    p.A = (const bf16_t*)a.A; p.B = (const bf16_t*)a.B; p.C = (bf16_t*)a.C;
    p.bias = (const bf16_t*)a.bias; p.resid = (const bf16_t*)a.resid; p.aux = (bf16_t*)a.aux;
    p.M = (int)a.M; p.N = (int)a.N; p.K = (int)a.K;
    p.lda = a.trans_a ? (int)a.M : (int)a.K;
    p.ldb = a.trans_b ? (int)a.K : (int)a.N;
    p.epi = a.epi;
    p.tiles_m = (int)((a.M + BM - 1) / BM);
    p.tiles_n = (int)((a.N + BN - 1) / BN);
    const bool a_kmaj = !a.trans_a, b_kmaj = a.trans_b;
    if (a_kmaj && b_kmaj) return launch<true, true>(p, a.stream);
    if (a_kmaj && !b_kmaj) return launch<true, false>(p, a.stream);
    if (!a_kmaj && b_kmaj) return launch<false, true>(p, a.stream);
    return launch<false, false>(p, a.stream);
}

}  // namespace tpl
