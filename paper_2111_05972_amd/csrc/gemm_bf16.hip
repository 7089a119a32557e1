// bf16 GEMM for gfx950: C[M,N] = epi(opA(A) opB(B)), float accumulation on the matrix cores.
//
// Tile and pipeline.  A 256-thread workgroup (4 wavefronts, 2 x 2) owns a 256 x 256 output tile;
// each wavefront accumulates 128 x 128 as 4 x 4 MFMA 32x32x16 blocks (256 accumulator registers).
// K is walked in stages of 32 through a 4-deep LDS ring (4 x 32 KiB) that is filled by
// buffer_load ... lds: global memory goes straight into LDS, no staging registers, and anything
// outside the matrix is zero filled by the buffer bounds check.  Loads run about 3.5 stages ahead of
// the math.  There is one barrier per stage, placed between the two 16-MFMA halves of the stage so
// that its wait and the LDS reads that follow it overlap with matrix-core work already queued.
//
// Operand layouts.  Either operand may be stored with K contiguous ("K-major": A as [M,K], B as
// [N,K]) or with its M/N dimension contiguous ("MN-major": A as [K,M], B as [K,N]).  K-major tiles
// are read from LDS with 16-byte reads; MN-major tiles with the transposing ds_read_b64_tr_b16,
// which hands each lane four K-consecutive values of one column, so no operand is ever transposed
// in HBM or in registers.  LDS chunk positions are XOR-swizzled (applied on the global-address side
// of the direct loads) so that both kinds of read are bank-conflict free.
//
// Scheduling over the chip.  One workgroup per output tile.  Workgroup ids are dealt round-robin to
// the 8 XCDs (each with its own L2), so ids are regrouped to give every XCD a contiguous run of
// tiles, and tiles are ordered column-major inside bands of 8 tile rows: the 32 tiles in flight on
// an XCD form an 8 x 4 block that shares 12 operand panels in that XCD's L2.
//
// Epilogue.  Accumulators go through per-wavefront LDS staging so that every global access of the
// epilogue (bias, residual, GeLU input, output) is a 16-byte access and 16 lanes cover 256
// contiguous bytes of a row.
#include <hip/hip_runtime.h>

#include "device_math.h"
#include "kernels.h"

namespace tpl {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((address_space(3))) s16x4* lds_s16x4_ptr;
typedef __attribute__((address_space(3))) void* lds_void_ptr;

constexpr int DK = 32;                      // k per stage
constexpr int DSTAGES = 4;
constexpr int DT = 256;                     // tile edge
constexpr int D_OP_BYTES = DT * DK * 2;     // one operand tile of one stage: 16 KiB
constexpr int D_STAGE_BYTES = 2 * D_OP_BYTES;
constexpr int D_LDS_BYTES = DSTAGES * D_STAGE_BYTES;
constexpr unsigned OOB_OFFSET = 0xFFFFFFF0u;   // beyond any buffer this kernel accepts
constexpr int EROW = 4 * 32 * 4 + 16;          // one 128-float row of a wavefront's epilogue staging
constexpr int EWAVE = 32 * EROW;
static_assert(4 * EWAVE <= D_LDS_BYTES, "epilogue staging must fit in the ring");

struct GemmParams {
    const bf16_t* A; const bf16_t* B; bf16_t* C;
    const bf16_t* bias; const bf16_t* resid; bf16_t* aux;
    int M, N, K;
    int lda, ldb;          // row strides (elements) of A and B as stored
    int epi;
    int tiles_m, tiles_n, nk;
};

// ---- LDS layouts -------------------------------------------------------------------------------
// K-major stage tile: 64-byte rows (32 k), four 16-byte chunks, swizzled by row.
__device__ __forceinline__ int swz_k32(int row) { return (row >> 2) & 3; }
// MN-major stage tile: 512-byte rows (256 m or n) per k, thirty-two 16-byte chunks, swizzled by k.
__device__ __forceinline__ int swz_mn(int k) { return (k & 3) << 2; }

// Raw buffer descriptor over `bytes` bytes at p (stride 0): loads at offsets >= bytes return zero
// instead of touching memory.
__device__ __forceinline__ i32x4 make_rsrc(const void* p, unsigned bytes) {
    const uint64_t a = (uint64_t)(uintptr_t)p;
    i32x4 r;
    r[0] = __builtin_amdgcn_readfirstlane((int)(unsigned)a);
    r[1] = __builtin_amdgcn_readfirstlane((int)(unsigned)(a >> 32) & 0xffff);
    r[2] = __builtin_amdgcn_readfirstlane((int)bytes);
    r[3] = 0x00020000;
    return r;
}

// One 16-byte-per-lane buffer load straight into LDS (lane l lands at lds_addr + 16*l).  Issued as
// inline assembly on purpose: the compiler then keeps no record of an LDS write in flight, so it does
// not drain the whole prefetch ring (vmcnt(0)) in front of later LDS reads; the kernel waits on
// vmcnt itself, with the exact number of loads allowed to remain in flight.
__device__ __forceinline__ void buffer_load_lds_b128(i32x4 rsrc, unsigned lds_addr, unsigned voffset) {
    asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :: "s"(lds_addr), "v"(voffset), "s"(rsrc) : "memory", "m0");
}

// Byte offsets (relative to the operand base, for tile origin mn0 and k = 0) of the four 16-byte
// chunks this lane fetches per stage; chunk j of wavefront w lands in LDS block w*4 + j at 16*lane.
template <bool KMAJ>
__device__ __forceinline__ void dma_offsets(unsigned (&off)[4], bool (&mn_ok)[4], int& kcol, int ld,
                                            int mn0, int MN, int wave, int lane) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        int block = wave * 4 + j;
        if (KMAJ) {
            int row = block * 16 + (lane >> 2);
            int c = (lane & 3) ^ swz_k32(row);
            kcol = c * 8;                                   // same for every j
            mn_ok[j] = true;                                // rows beyond MN fall outside the buffer
            off[j] = (unsigned)(((int64_t)(mn0 + row) * ld + c * 8) * 2);
        } else {
            int k = block * 2 + (lane >> 5);
            int c = (lane & 31) ^ swz_mn(k);
            kcol = 0;
            mn_ok[j] = mn0 + c * 8 < MN;
            off[j] = (unsigned)(((int64_t)k * ld + mn0 + c * 8) * 2);
        }
    }
}

// Stage starting at k0; k >= kend is zero filled (the end of K, or the end of this workgroup's share).
template <bool KMAJ>
__device__ __forceinline__ void dma_issue(i32x4 rsrc, unsigned tile_lds, const unsigned (&off)[4],
                                          const bool (&mn_ok)[4], int kcol, int ld, int k0, int kend, int wave) {
    const unsigned step = KMAJ ? (unsigned)k0 * 2u : (unsigned)((int64_t)k0 * ld * 2);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        bool ok = KMAJ ? (k0 + kcol < kend) : (mn_ok[j] && k0 < kend);
        unsigned o = ok ? off[j] + step : OOB_OFFSET;
        buffer_load_lds_b128(rsrc, tile_lds + (wave * 4 + j) * 1024, o);
    }
}

// LDS -> MFMA fragment: rows mn_base + (lane % 32), k = ks*16 + 8*(lane/32) + 0..7.
template <bool KMAJ>
__device__ __forceinline__ bf16x8 dma_frag(const char* tile, int mn_base, int ks, int lane) {
    if (KMAJ) {
        int row = mn_base + (lane & 31);
        int c = 2 * ks + (lane >> 5);
        return *reinterpret_cast<const bf16x8*>(tile + row * 64 + ((c ^ swz_k32(row)) << 4));
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
            int off = k * (DT * 2) + ((((mn >> 3) ^ swz_mn(k))) << 4) + (mn & 7) * 2;
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

// Workgroup id -> position in the tile list.  Consecutive ids go to different XCDs (each with its
// own L2), so ids are regrouped to give every XCD one contiguous run of the list.
__device__ __forceinline__ int share_of_block(int bid, int nblocks) {
    constexpr int NXCD = 8;
    int per = nblocks / NXCD, rem = nblocks % NXCD;
    int xcd = bid % NXCD, idx = bid / NXCD;
    return xcd * per + (xcd < rem ? xcd : rem) + idx;
}
// Tile order: column-major inside bands of 8 tile rows, so tiles adjacent in the list (in flight
// together on one XCD) share A and B panels in that XCD's L2.
__device__ __forceinline__ void tile_coords(int tile, int tiles_m, int tiles_n, int& tm, int& tn) {
    constexpr int BAND = 8;
    int band_tiles = BAND * tiles_n;
    int band = tile / band_tiles, within = tile % band_tiles;
    int rows = tiles_m - band * BAND;
    rows = rows < BAND ? rows : BAND;
    tm = band * BAND + within % rows;
    tn = within / rows;
}

template <bool A_KMAJ, bool B_KMAJ>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(GemmParams p) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const int tile = share_of_block(blockIdx.x, gridDim.x);
    const int ks0 = 0, ks1 = p.nk;

    const i32x4 ra = make_rsrc(p.A, (unsigned)((int64_t)(A_KMAJ ? p.M : p.K) * p.lda * 2));
    const i32x4 rb = make_rsrc(p.B, (unsigned)((int64_t)(B_KMAJ ? p.N : p.K) * p.ldb * 2));
    const unsigned lds0 = (unsigned)(uintptr_t)(lds_void_ptr)smem;
    constexpr int READS = (A_KMAJ ? 4 : 8) + (B_KMAJ ? 4 : 8);   // LDS reads per fragment set
    {
        int tm, tn;
        tile_coords(tile, p.tiles_m, p.tiles_n, tm, tn);
        const int m0 = tm * DT, n0 = tn * DT;
        const int kend = ks1 * DK < p.K ? ks1 * DK : p.K;

        f32x16 acc[4][4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

        unsigned offa[4], offb[4];
        bool oka[4], okb[4];
        int kca, kcb;
        dma_offsets<A_KMAJ>(offa, oka, kca, p.lda, m0, p.M, wave, lane);
        dma_offsets<B_KMAJ>(offb, okb, kcb, p.ldb, n0, p.N, wave, lane);

        // ring slot of stage s is (s - ks0) % 4; stages >= ks1 are issued too (zero fill, no memory
        // traffic) so that the number of loads in flight is the same in every iteration.
        auto issue = [&](int s) {
            const unsigned buf = lds0 + ((s - ks0) % DSTAGES) * D_STAGE_BYTES;
            dma_issue<A_KMAJ>(ra, buf, offa, oka, kca, p.lda, s * DK, kend, wave_u);
            dma_issue<B_KMAJ>(rb, buf + D_OP_BYTES, offb, okb, kcb, p.ldb, s * DK, kend, wave_u);
        };
        auto read_frags = [&](bf16x8 (&fa)[4], bf16x8 (&fb)[4], int s, int ks) {
            const char* buf = smem + ((s - ks0) % DSTAGES) * D_STAGE_BYTES;
#pragma unroll
            for (int i = 0; i < 4; ++i) fa[i] = dma_frag<A_KMAJ>(buf, (wm * 4 + i) * 32, ks, lane);
#pragma unroll
            for (int j = 0; j < 4; ++j) fb[j] = dma_frag<B_KMAJ>(buf + D_OP_BYTES, (wn * 4 + j) * 32, ks, lane);
        };
        auto mma = [&](const bf16x8 (&fa)[4], const bf16x8 (&fb)[4]) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        };

        issue(ks0); issue(ks0 + 1); issue(ks0 + 2); issue(ks0 + 3);
        asm volatile("s_waitcnt vmcnt(24)" ::: "memory");        // first stage has landed (8 loads per stage)
        __builtin_amdgcn_s_barrier();
        bf16x8 fa0[4], fb0[4], fa1[4], fb1[4];
        read_frags(fa0, fb0, ks0, 0);

        for (int kt = ks0; kt < ks1; ++kt) {
            // first half: math on k-substep 0 while the fragments of substep 1 are read
            read_frags(fa1, fb1, kt, 1);
            mma(fa0, fb0);
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // math first: no LDS wait at the loop top
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x100, READS / 8, 0);
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            }
            __builtin_amdgcn_sched_group_barrier(0x008, 7, 0);
            // stage kt+1 has landed for this wavefront once at most two newer stages are in flight;
            // after the barrier it has landed for all, and nobody reads stage kt's slot any more.
            asm volatile("s_waitcnt vmcnt(16) lgkmcnt(0)" ::: "memory");
            __builtin_amdgcn_s_barrier();
            issue(kt + 4);
            read_frags(fa0, fb0, kt + 1, 0);
            mma(fa1, fb1);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, READS / 8, 0);
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            }
            __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
        }
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");   // drain the ring before LDS is reused
        __builtin_amdgcn_s_barrier();

        // ---- epilogue: accumulators -> per-wavefront LDS staging -> 16-byte row accesses ----------
        char* stage = smem + wave * EWAVE;
        const int er = lane >> 4, ec = (lane & 15) * 8;
        const int ln = wn * 128 + ec;             // column inside the tile
        const int gn = n0 + ln;
        float bias8[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        if (p.bias && gn < p.N) unpack8(*reinterpret_cast<const uint4*>(p.bias + gn), bias8);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            // accumulator register v of block (i,j): row (v/4)*8 + (lane/32)*4 + v%4, column j*32 + lane%32
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    int row = (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
                    *reinterpret_cast<float*>(stage + row * EROW + (j * 32 + (lane & 31)) * 4) = acc[i][j][v];
                }
#pragma unroll
            for (int pass = 0; pass < 8; ++pass) {
                const int row = pass * 4 + er;
                const int lm = (wm * 4 + i) * 32 + row;      // row inside the tile
                const int gm = m0 + lm;
                const float4* src = reinterpret_cast<const float4*>(stage + row * EROW + ec * 4);
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
}

bool gemm_bf16_supported(const GemmArgs& a) {
    if (a.dtype != BF16) return false;
    if (a.M % 8 || a.N % 8 || a.K % 8) return false;
    // 32-bit buffer offsets: operands below 2 GiB
    if (a.M * a.K * 2 >= 0x7FFFFFFFll || a.N * a.K * 2 >= 0x7FFFFFFFll) return false;
    int64_t tiles = ((a.M + DT - 1) / DT) * ((a.N + DT - 1) / DT);
    return tiles < (1 << 24) && a.K < (1 << 24);
}

size_t gemm_bf16_workspace_bytes(int64_t, int64_t, int64_t) { return 0; }

template <bool AK, bool BK_>
static hipError_t launch(const GemmParams& p, int grid, hipStream_t s) {
    static bool attr_set = false;   // raising the dynamic LDS limit is a per-function, one-off call
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_bf16_kernel<AK, BK_>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, D_LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL((gemm_bf16_kernel<AK, BK_>), dim3(grid), dim3(256), D_LDS_BYTES, s, p);
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
    p.tiles_m = (int)((a.M + DT - 1) / DT);
    p.tiles_n = (int)((a.N + DT - 1) / DT);
    p.nk = (int)((a.K + DK - 1) / DK);
    const int grid = p.tiles_m * p.tiles_n;
    const bool a_kmaj = !a.trans_a, b_kmaj = a.trans_b;
    if (a_kmaj && b_kmaj) return launch<true, true>(p, grid, a.stream);
    if (a_kmaj && !b_kmaj) return launch<true, false>(p, grid, a.stream);
    if (!a_kmaj && b_kmaj) return launch<false, true>(p, grid, a.stream);
    return launch<false, false>(p, grid, a.stream);
}

}  // namespace tpl
