// bf16 GEMM for gfx950: C[M,N] = epi(opA(A) opB(B)), float accumulation on the matrix cores.
//
// Kernels (the host picks one per GEMM by an estimate of its time, see make_plan):
//   gemm_bf16_kernel          4 wavefronts that fetch and compute, MFMA 32x32x16; tiles 256x256, 256x192, and
//                             192x192 / 128x128 with two workgroups per compute unit
//   gemm_bf16_spec_kernel     256x192, 4 math + 4 fetch wavefronts, MFMA 32x32x16      (forward GEMMs: NN)
//   gemm_bf16_spec16_kernel   the same roles on MFMA 16x16x32, K-major A               (data gradients: NT)
//   gemm_bf16_x16s_kernel     192x192, two workgroups per compute unit, MFMA 16x16x32  (weight gradients: TN; short-K
//                             forward GEMMs such as the out-projection)
//   gemm_bf16_x16w8_kernel    256x192, 8 wavefronts that fetch and compute, 16x16x32   (short K, one GEMM at a time)
//   gemm_sum_shares_kernel    adds the partial sums of a GEMM whose K was cut into shares, applies the epilogue
//
// Pipeline.  K is walked in stages of 32 through LDS rings filled by buffer_load ... lds: global memory goes
// straight into LDS, no staging registers, and anything outside the matrix is zero filled by the buffer bounds
// check.  Loads run 2 to 4 stages ahead of the math; there is one workgroup barrier per stage.  The loop bodies
// are written as single pieces (one matrix instruction, one fragment read, one direct load) separated by
// scheduling fences, so the instruction order is the one written.
//
// What decides the design (measured on the device):
//  * With random operands these GEMMs run at the board's power limit with the clock pulled down; throughput then
//    follows energy per flop.  MFMA 16x16x32 needs less than 32x32x16 (each instruction carries 32 k, so the float
//    accumulators are read and written half as often per flop): a pure matrix-instruction loop on random data
//    sustains 15 % more with it.
//  * Issuing a 1 KiB memory instruction (fragment read or direct load) holds a wavefront for about 35 cycles.  Under
//    a 32-cycle 32x32x16 instruction that is almost hidden, under a 16-cycle 16x16x32 it is not.  Hence fetch-only
//    wavefronts beside the math wavefronts, or two wavefronts per SIMD.
//  * Two wavefronts per SIMD leave 256 registers each, 144 to 192 of them accumulators: the 16x16x32 kernels
//    single-buffer their fragments and refill each register as soon as its last use of the k-step is issued.
//
// Operand layouts.  Either operand may be stored with K contiguous ("K-major": A as [M,K], B as [N,K]) or with
// its M/N dimension contiguous ("MN-major": A as [K,M], B as [K,N]).  K-major tiles are read from LDS with
// 16-byte reads; MN-major tiles with the transposing ds_read_b64_tr_b16, which hands each lane four
// K-consecutive values of one column, so no operand is ever transposed in HBM or in registers.  LDS chunk
// positions are XOR-swizzled (applied on the global-address side of the direct loads) so that the reads are
// free of bank conflicts; the XOR depends on the fragment shape that reads the tile.
//
// Scheduling over the chip.  One workgroup per (output tile, K share).  Workgroup ids are dealt round-robin to
// the 8 XCDs (each with its own L2), so ids are regrouped to give every XCD a contiguous run of tiles, and tiles
// are ordered column-major inside bands of a few tile rows (the height that minimises what the tiles in flight on
// an XCD fetch together, see choose_band): the tiles in flight on an XCD share operand panels in that XCD's L2.
//
// Epilogue.  Accumulators go through per-wavefront LDS staging so that every global access of the epilogue
// (bias, residual, GeLU input, output) is a 16-byte access and a staged row is contiguous.
#include <hip/hip_runtime.h>
#include <type_traits>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <mutex>

#include "device_math.h"
#include "kernels.h"
#include "lds_dma.h"

namespace tpl {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((address_space(3))) s16x4* lds_s16x4_ptr;

constexpr int DK = 32;                      // k per stage
constexpr unsigned OOB_OFFSET = 0xFFFFFFF0u;   // beyond any buffer this kernel accepts

// Tile variant: 2 x 2 wavefronts, each owning TM x TN MFMA 32x32 blocks -> a (64 TM) x (64 TN) tile.
template <int TM_, int TN_, int STAGES_>
struct Tile {
    static constexpr int TM = TM_, TN = TN_, STAGES = STAGES_;
    static constexpr int BM = 64 * TM, BN = 64 * TN;
    static constexpr int A_BYTES = BM * DK * 2, B_BYTES = BN * DK * 2;   // one stage of each operand
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr int LOADS = TM + TN;                                // direct loads per lane and stage
    static constexpr int EROW = TN * 32 * 4 + 16;                        // staged epilogue row of a wavefront
    static constexpr int EWAVE = 32 * EROW;
    static constexpr int LDS_BYTES = STAGES * STAGE_BYTES > 4 * EWAVE ? STAGES * STAGE_BYTES : 4 * EWAVE;
    static_assert((STAGES - 1) * LOADS <= 63, "vmcnt is a 6-bit counter");
};

struct GemmParams {
    const bf16_t* A; const bf16_t* B; bf16_t* C;
    const bf16_t* bias; const bf16_t* resid; bf16_t* aux;
    int M, N, K;
    int lda, ldb;          // row strides (elements) of A and B as stored
    int epi;
    int tiles_m, tiles_n;
    int band;              // tile rows per band of the tile order (see tile_coords)
    int nt_store;          // C stored with the non-temporal hint
    int nk;                // k-steps of one workgroup (one K share when K is split)
    int nk_total;          // k-steps of the whole K
    float* partial;        // K split over several workgroups: float partial sums [share][M][N], else null
    bf16_t* colsum;        // [N]: sum over k of B[k][n], written by the kernels that can (see gemm_bf16), else null
};

// Which K share a workgroup computes.  The workgroup list is share-major (all tiles of share 0, then all
// tiles of share 1, ...), so the tiles in flight together on an XCD walk the same k range and share panels.
struct KShare { int tile, kt0, nk, kend; float* partial; };
__device__ __forceinline__ KShare k_share(const GemmParams& p, int list_pos) {
    KShare s;
    const int ntiles = p.tiles_m * p.tiles_n;
    const int share = list_pos / ntiles;
    s.tile = list_pos - share * ntiles;
    s.kt0 = share * p.nk;
    s.nk = p.nk_total - s.kt0 < p.nk ? p.nk_total - s.kt0 : p.nk;
    s.kend = (s.kt0 + s.nk) * DK < p.K ? (s.kt0 + s.nk) * DK : p.K;
    s.partial = p.partial ? p.partial + (int64_t)share * p.M * p.N : nullptr;
    return s;
}

// ---- LDS layouts -------------------------------------------------------------------------------
// K-major stage tile: 64-byte rows (32 k), four 16-byte chunks, swizzled by row.
__device__ __forceinline__ int swz_k32(int row) { return (row >> 2) & 3; }
// MN-major stage tile: one row of R (m or n) bf16 per k = R/8 16-byte chunks, R*2 bytes per k.
// A transposing read touches four consecutive k at the same 64 bytes of columns (two 16-lane groups,
// 32 bytes each); the four k must land in four different 64-byte quarters of the 256-byte bank line.
//  * R*2 a multiple of 256 (R = 128, 256): every k starts at the same bank offset, so the 64-byte
//    column group is XORed with k & 3.
//  * R = 192 (384-byte rows): k and k+1 already differ by 128 bytes, so k+2, k+3 are moved one
//    64-byte group further (cyclically over the row's 6 groups; 6 = 2 mod 4 keeps the four distinct).
template <int R> __device__ __forceinline__ int mn_swz(int c, int k) {
    constexpr int CPR = R / 8;
    const int half = ((k >> 3) & 1) << 1;       // k and k + 8 (16x16x32 fragments read both at once): other 32 bytes
    if ((CPR & (CPR - 1)) == 0) return c ^ ((k & 3) << 2) ^ half;
    int g = (c >> 2) + ((k >> 1) & 1);
    g = g >= CPR / 4 ? g - CPR / 4 : g;
    return (g << 2) | ((c & 3) ^ half);
}
template <int R> __device__ __forceinline__ int mn_unswz(int c, int k) {
    constexpr int CPR = R / 8;
    const int half = ((k >> 3) & 1) << 1;
    if ((CPR & (CPR - 1)) == 0) return c ^ ((k & 3) << 2) ^ half;
    int g = (c >> 2) - ((k >> 1) & 1);
    g = g < 0 ? g + CPR / 4 : g;
    return (g << 2) | ((c & 3) ^ half);
}

constexpr unsigned OOB_HALF = 0x80000000u;     // out of bounds for operands below 2 GiB, and no wrap when a
                                               // scalar offset below 2 GiB is added

// Byte offsets (relative to the operand base, for tile origin mn0 and k = 0) of the T 16-byte chunks
// this lane fetches per stage (operand tile of R = 64 T rows); chunk j of wavefront w lands in LDS
// block w*T + j (1 KiB blocks) at 16*lane.
// XOR16: MN-major chunk positions for the kernel that reads 16x16x32 fragments with per-lane base registers
// (chunk c of row k at position c ^ xor16(k)); otherwise mn_swz.
__device__ __forceinline__ int xor16(int k) { return (((k >> 1) & 1) << 1) | (((k >> 3) & 1) << 2); }
// K16: K-major chunk positions for tiles read as 16-row fragments (swz_k32_16 below).
__device__ __forceinline__ int swz_k32_16(int row) { return (row >> 1) & 3; }
// k row (0..31) of the MN-major stage tile of R = 64 T columns that load j of wavefront `wave` fetches for this lane.
template <int T> __device__ __forceinline__ int mn_krow(int wave, int j, int lane) {
    return ((wave * T + j) * 64 + lane) / (64 * T / 8);
}
template <bool KMAJ, int T, bool XOR16 = false, bool K16 = false>
__device__ __forceinline__ void dma_offsets(unsigned (&off)[T], bool (&mn_ok)[T], int& kcol, int ld,
                                            int mn0, int MN, int wave, int lane) {
    constexpr int R = 64 * T;
#pragma unroll
    for (int j = 0; j < T; ++j) {
        int block = wave * T + j;
        if (KMAJ) {
            int row = block * 16 + (lane >> 2);
            int c = (lane & 3) ^ (K16 ? swz_k32_16(row) : swz_k32(row));
            kcol = c * 8;                                   // same for every j
            mn_ok[j] = true;                                // rows beyond MN point past the buffer
            off[j] = mn0 + row < MN ? (unsigned)(((int64_t)(mn0 + row) * ld + c * 8) * 2) : OOB_HALF;
        } else {
            int idx = block * 64 + lane;                    // physical chunk index inside the stage tile
            int k = idx / (R / 8);
            int c = XOR16 ? (idx % (R / 8)) ^ xor16(k) : mn_unswz<R>(idx % (R / 8), k);   // logical chunk stored there
            kcol = 0;
            mn_ok[j] = mn0 + c * 8 < MN;
            off[j] = (unsigned)(((int64_t)k * ld + mn0 + c * 8) * 2);
        }
    }
}

// LDS -> MFMA fragment: rows mn_base + (lane % 32), k = ks*16 + 8*(lane/32) + 0..7.
template <bool KMAJ, int R>
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
            int off = k * (R * 2) + (mn_swz<R>(mn >> 3, k) << 4) + (mn & 7) * 2;
            s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(tile + off));
            bf16x4 b = __builtin_bit_cast(bf16x4, v);
            out[4 * h + 0] = b[0]; out[4 * h + 1] = b[1]; out[4 * h + 2] = b[2]; out[4 * h + 3] = b[3];
        }
        return out;
    }
}

// LDS -> fragment of the 16x16x32 matrix instruction: rows mn_base + (lane % 16), k = 8*(lane/16) + 0..7 of
// the 32-k stage.  For this lane pattern a K-major tile of 64-byte rows is free of bank conflicts with the chunk
// XOR (row >> 1) & 3 (measured: 223 B/clk/CU, against 125 with the (row >> 2) & 3 of the 32-row fragments).
template <bool KMAJ, int R>
__device__ __forceinline__ bf16x8 dma_frag16(const char* tile, int mn_base, int lane) {
    if (KMAJ) {
        int row = mn_base + (lane & 15);
        int c = lane >> 4;
        return *reinterpret_cast<const bf16x8*>(tile + row * 64 + ((c ^ swz_k32_16(row)) << 4));
    } else {
        int l16 = lane & 15;
        int mn = mn_base + 4 * (l16 & 3);
        int kq = l16 >> 2;
        int kb = 8 * (lane >> 4);
        bf16x8 out;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            int k = kb + 4 * h + kq;
            int off = k * (R * 2) + (mn_swz<R>(mn >> 3, k) << 4) + (mn & 7) * 2;
            s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(tile + off));
            bf16x4 b = __builtin_bit_cast(bf16x4, v);
            out[4 * h + 0] = b[0]; out[4 * h + 1] = b[1]; out[4 * h + 2] = b[2]; out[4 * h + 3] = b[3];
        }
        return out;
    }
}

template <int N> __device__ __forceinline__ void wait_vmcnt() {
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
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
// Tile order: column-major inside bands of `band` tile rows.  Every XCD (own L2) works through one contiguous run
// of this list (share_of_block), i.e. a block of band rows x some columns of the tile grid: it fetches the A panels
// of its band and the B panels of its columns once.  The host picks the band height that minimises the sum over
// XCDs of those fetches (choose_band).
__device__ __forceinline__ void tile_coords(int tile, int tiles_m, int tiles_n, int band_rows, int& tm, int& tn) {
    int band_tiles = band_rows * tiles_n;
    int band = tile / band_tiles, within = tile % band_tiles;
    int rows = tiles_m - band * band_rows;
    rows = rows < band_rows ? rows : band_rows;
    tm = band * band_rows + within % rows;
    tn = within / rows;
}

// Epilogue of one wavefront: accumulators -> its LDS staging area -> 16-byte row accesses.  The wavefront's
// part of the tile goes through the staging area in slabs of 32 rows; store_slab(i, stage) writes slab i
// (row r, column c of the wavefront's part at stage + r * EROW + 4 c).
// One pass over a staged slab: 64 / LPR rows, 8 columns per lane (bias, residual, GeLU or its derivative, or the raw
// float sums of one K share).
template <typename TL>
__device__ __forceinline__ void epilogue_pass(const GemmParams& p, const char* stage, int pass, int i, int wm, int lane,
                                              int m0, int gn, const float (&bias8)[8], float* partial) {
    constexpr int TM = TL::TM, TN = TL::TN;
    constexpr int LPR = TN * 4;               // lanes per staged row (8 columns each)
    constexpr int RPP = 64 / LPR;             // rows per pass (lanes beyond RPP*LPR idle when TN = 3)
    const int er = lane / LPR, ec = (lane % LPR) * 8;
    const int row = pass * RPP + er;
    const int gm = m0 + (wm * TM + i) * 32 + row;
    if (er < RPP && row < 32 && gm < p.M && gn < p.N) {
        const float4* src = reinterpret_cast<const float4*>(stage + row * TL::EROW + ec * 4);
        float4 x0 = src[0], x1 = src[1];
        float v8[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
        const int64_t idx = (int64_t)gm * p.N + gn;
        if (partial) {                     // one K share: the raw float sums; the epilogue is applied
            float4* dst = reinterpret_cast<float4*>(partial + idx);   // when the shares are summed
            dst[0] = x0; dst[1] = x1;
            return;
        }
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
        const uint4 out = pack8(v8);
        if (p.nt_store) {
            typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
            u32x4 o4 = {out.x, out.y, out.z, out.w};
            __builtin_nontemporal_store(o4, reinterpret_cast<u32x4*>(p.C + idx));
        } else {
            *reinterpret_cast<uint4*>(p.C + idx) = out;
        }
    }
}
template <typename TL, typename StoreSlab>
__device__ __forceinline__ void epilogue_rows(const GemmParams& p, char* smem, int wave, int lane, int m0, int n0,
                                              float* partial, StoreSlab store_slab) {
    constexpr int TM = TL::TM, TN = TL::TN;
    const int wm = wave >> 1, wn = wave & 1;
    constexpr int LPR = TN * 4, RPP = 64 / LPR, PASSES = (32 + RPP - 1) / RPP;
    char* stage = smem + wave * TL::EWAVE;
    const int gn = n0 + wn * TN * 32 + (lane % LPR) * 8;
    float bias8[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (p.bias && !partial && gn < p.N) unpack8(*reinterpret_cast<const uint4*>(p.bias + gn), bias8);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        store_slab(i, stage);
#pragma unroll
        for (int pass = 0; pass < PASSES; ++pass) epilogue_pass<TL>(p, stage, pass, i, wm, lane, m0, gn, bias8, partial);
    }
}
// The same for kernels whose fetching wavefronts 4..7 have nothing left to do: math wavefront w stages slab i into
// one of two buffers, and after a workgroup barrier it and wavefront w + 4 (helper) take alternate passes over it.
// Two buffers: the math wavefront stages slab i + 1 while its helper may still read slab i; buffer (i & 1) is
// written again only after the barrier of slab i + 1, which the helper reaches after it has finished slab i.
// Every wavefront of the workgroup executes exactly TM barriers here.
template <typename TL, typename StoreSlab>
__device__ __forceinline__ void epilogue_rows_shared(const GemmParams& p, char* smem, int wave, int lane, int m0, int n0,
                                                     float* partial, bool helper, StoreSlab store_slab) {
    constexpr int TM = TL::TM, TN = TL::TN;
    const int w4 = wave & 3, wm = w4 >> 1, wn = w4 & 1;
    constexpr int LPR = TN * 4, RPP = 64 / LPR, PASSES = (32 + RPP - 1) / RPP;
    const int gn = n0 + wn * TN * 32 + (lane % LPR) * 8;
    float bias8[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (p.bias && !partial && gn < p.N) unpack8(*reinterpret_cast<const uint4*>(p.bias + gn), bias8);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        char* stage = smem + (w4 * 2 + (i & 1)) * TL::EWAVE;
        if (!helper) store_slab(i, stage);
        __syncthreads();
        // the helper takes the even passes (one more when their number is odd): the math wavefront also stages
#pragma unroll
        for (int pass = 0; pass < PASSES; ++pass)
            if (((pass & 1) == 0) == helper) epilogue_pass<TL>(p, stage, pass, i, wm, lane, m0, gn, bias8, partial);
    }
}

// 32x32x16 accumulators: register v of block (i,j) is row (v/4)*8 + (lane/32)*4 + v%4, column j*32 + lane%32.
template <typename TL>
__device__ __forceinline__ void epilogue(const GemmParams& p, const f32x16 (&acc)[TL::TM][TL::TN], char* smem,
                                         int wave, int lane, int m0, int n0, float* partial) {
    epilogue_rows<TL>(p, smem, wave, lane, m0, n0, partial, [&](int i, char* stage) {
#pragma unroll
        for (int j = 0; j < TL::TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                int row = (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
                *reinterpret_cast<float*>(stage + row * TL::EROW + (j * 32 + (lane & 31)) * 4) = acc[i][j][v];
            }
    });
}
// 16x16x32 accumulators: register v of block (i,j) is row i*16 + (lane/16)*4 + v, column j*16 + lane%16.
template <typename TL>
__device__ __forceinline__ void epilogue16(const GemmParams& p, const f32x4 (&acc)[2 * TL::TM][2 * TL::TN], char* smem,
                                           int wave, int lane, int m0, int n0, float* partial) {
    epilogue_rows<TL>(p, smem, wave, lane, m0, n0, partial, [&](int i, char* stage) {
#pragma unroll
        for (int ii = 0; ii < 2; ++ii)
#pragma unroll
            for (int j = 0; j < 2 * TL::TN; ++j)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    int row = ii * 16 + (lane >> 4) * 4 + v;
                    *reinterpret_cast<float*>(stage + row * TL::EROW + (j * 16 + (lane & 15)) * 4) = acc[2 * i + ii][j][v];
                }
    });
}
// Shared forms (see epilogue_rows_shared): the math wavefronts pass their accumulators, the helpers nothing.
template <typename TL>
__device__ __forceinline__ void epilogue_shared(const GemmParams& p, const f32x16 (&acc)[TL::TM][TL::TN], char* smem,
                                                int wave, int lane, int m0, int n0, float* partial) {
    epilogue_rows_shared<TL>(p, smem, wave, lane, m0, n0, partial, false, [&](int i, char* stage) {
#pragma unroll
        for (int j = 0; j < TL::TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                int row = (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
                *reinterpret_cast<float*>(stage + row * TL::EROW + (j * 32 + (lane & 31)) * 4) = acc[i][j][v];
            }
    });
}
template <typename TL>
__device__ __forceinline__ void epilogue16_shared(const GemmParams& p, const f32x4 (&acc)[2 * TL::TM][2 * TL::TN],
                                                  char* smem, int wave, int lane, int m0, int n0, float* partial) {
    epilogue_rows_shared<TL>(p, smem, wave, lane, m0, n0, partial, false, [&](int i, char* stage) {
#pragma unroll
        for (int ii = 0; ii < 2; ++ii)
#pragma unroll
            for (int j = 0; j < 2 * TL::TN; ++j)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    int row = ii * 16 + (lane >> 4) * 4 + v;
                    *reinterpret_cast<float*>(stage + row * TL::EROW + (j * 16 + (lane & 15)) * 4) = acc[2 * i + ii][j][v];
                }
    });
}
template <typename TL>
__device__ __forceinline__ void epilogue_helper(const GemmParams& p, char* smem, int wave, int lane, int m0, int n0,
                                                float* partial) {
    epilogue_rows_shared<TL>(p, smem, wave, lane, m0, n0, partial, true, [](int, char*) {});
}

template <typename TL, bool A_KMAJ, bool B_KMAJ>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(GemmParams p) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    constexpr int TM = TL::TM, TN = TL::TN, BM = TL::BM, BN = TL::BN, DSTAGES = TL::STAGES;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const KShare sh = k_share(p, share_of_block(blockIdx.x, gridDim.x));

    const i32x4 ra = make_rsrc(p.A, (unsigned)((int64_t)(A_KMAJ ? p.M : p.K) * p.lda * 2));
    const i32x4 rb = make_rsrc(p.B, (unsigned)((int64_t)(B_KMAJ ? p.N : p.K) * p.ldb * 2));
    const unsigned lds0 = (unsigned)(uintptr_t)(lds_void_ptr)smem;
    constexpr int NM = TM * TN;                                   // matrix instructions per half stage

    int tm, tn;
    tile_coords(sh.tile, p.tiles_m, p.tiles_n, p.band, tm, tn);
    const int m0 = tm * BM, n0 = tn * BN;

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    unsigned offa[TM], offb[TN];
    bool oka[TM], okb[TN];
    int kca, kcb;
    dma_offsets<A_KMAJ, TM>(offa, oka, kca, p.lda, m0, p.M, wave, lane);
    dma_offsets<B_KMAJ, TN>(offb, okb, kcb, p.ldb, n0, p.N, wave, lane);

    // Ring slot of stage s (counted from the start of this workgroup's K share) is s % STAGES.  Stages past
    // the end of the share are issued too (all chunks out of
    // bounds: zero fill, no memory traffic) so the number of loads in flight never changes.  The loads
    // of a stage are numbered 0..LOADS-1 (A chunks, then B chunks); every piece of the loop body below
    // is fenced so that the instruction order is the one written: one fragment read or one direct
    // load between matrix instructions, never a burst that fills the memory queue and holds up the
    // wavefront's next matrix instruction.
    constexpr int L = TL::LOADS, L1 = L / 2;                     // part 1: loads [0,L1), part 2: [L1,L)
    auto dma_one = [&](int s, int d) {
        const unsigned buf = lds0 + (s % DSTAGES) * TL::STAGE_BYTES;
        const int k0 = (sh.kt0 + s) * DK;
        if (d < TM) {
            bool ok = A_KMAJ ? (k0 + kca < sh.kend) : (oka[d] && k0 < sh.kend);
            unsigned step = A_KMAJ ? (unsigned)k0 * 2u : (unsigned)((int64_t)k0 * p.lda * 2);
            buffer_load_lds_b128(ra, buf + (wave_u * TM + d) * 1024, ok ? offa[d] + step : OOB_OFFSET);
        } else {
            const int e = d - TM;
            bool ok = B_KMAJ ? (k0 + kcb < sh.kend) : (okb[e] && k0 < sh.kend);
            unsigned step = B_KMAJ ? (unsigned)k0 * 2u : (unsigned)((int64_t)k0 * p.ldb * 2);
            buffer_load_lds_b128(rb, buf + TL::A_BYTES + (wave_u * TN + e) * 1024, ok ? offb[e] + step : OOB_OFFSET);
        }
    };
    auto read_one = [&](bf16x8 (&fa)[TM], bf16x8 (&fb)[TN], int s, int ks, int r) {
        const char* buf = smem + (s % DSTAGES) * TL::STAGE_BYTES;
        if (r < TM) fa[r] = dma_frag<A_KMAJ, BM>(buf, (wm * TM + r) * 32, ks, lane);
        else fb[r - TM] = dma_frag<B_KMAJ, BN>(buf + TL::A_BYTES, (wn * TN + r - TM) * 32, ks, lane);
    };
    // one half stage: NM matrix instructions on (fa, fb); after instruction m, fragment m of the
    // next set is read, and the direct loads d0..d1-1 of stage ds are spread evenly over the half
    auto half = [&](const bf16x8 (&fa)[TM], const bf16x8 (&fb)[TN], bf16x8 (&na)[TM], bf16x8 (&nb)[TN],
                    int rs, int rks, int ds, auto d0c, auto d1c) {
        constexpr int D0 = decltype(d0c)::value, D1 = decltype(d1c)::value, NL = D1 - D0;
#pragma unroll
        for (int m = 0; m < NM; ++m) {
            acc[m / TN][m % TN] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[m / TN], fb[m % TN], acc[m / TN][m % TN], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            if (m < TM + TN) {
                read_one(na, nb, rs, rks, m);
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int d = 0; d < NL; ++d)
                if (m == ((2 * d + 1) * NM) / (2 * NL)) {
                    dma_one(ds, D0 + d);
                    __builtin_amdgcn_sched_barrier(0);
                }
        }
    };
    using IC0 = std::integral_constant<int, 0>;
    using ICL1 = std::integral_constant<int, L1>;
    using ICL = std::integral_constant<int, L>;

#pragma unroll
    for (int s0 = 0; s0 < DSTAGES - 1; ++s0)
#pragma unroll
        for (int d = 0; d < L; ++d) dma_one(s0, d);
#pragma unroll
    for (int d = 0; d < L1; ++d) dma_one(DSTAGES - 1, d);
    wait_vmcnt<(DSTAGES - 2) * L + L1>();                        // first stage has landed
    __builtin_amdgcn_s_barrier();
    bf16x8 fa0[TM], fb0[TN], fa1[TM], fb1[TN];
#pragma unroll
    for (int r = 0; r < TM + TN; ++r) read_one(fa0, fb0, 0, 0, r);
    __builtin_amdgcn_sched_barrier(0);

    for (int kt = 0; kt < sh.nk; ++kt) {
        // first half: math on k-substep 0, fragments of substep 1 are read, rest of stage kt+STAGES-1 is fetched
        half(fa0, fb0, fa1, fb1, kt, 1, kt + DSTAGES - 1, ICL1{}, ICL{});
        // stage kt+1 has landed for this wavefront once only the newer stages are in flight; after the
        // barrier it has landed for all, and nobody reads stage kt's slot any more.
        wait_vmcnt<(DSTAGES - 2) * L>();
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        half(fa1, fb1, fa0, fb0, kt + 1, 0, kt + DSTAGES, IC0{}, ICL1{});
    }
    wait_vmcnt<0>();                                             // drain the ring before LDS is reused
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    epilogue<TL>(p, acc, smem, wave, lane, m0, n0, sh.partial);
}

// =================================================================================================
// Eight wavefronts on the 16x16x32 matrix instruction: 4 x 2 wavefronts, two per SIMD, each owning
// (2 TM) x (2 TN) blocks of 16 x 16 (64 x 96 of a 256 x 192 tile).
// Why this instruction.  For random operands the chip runs these GEMMs at its power limit, and the 16x16x32
// form needs less energy per flop than 32x32x16 (a pure matrix-instruction loop on random data sustains about
// 15 % more with it: each instruction carries 32 k, so the float accumulators are read and written half as
// often per flop).  What it costs is twice the fragment registers per k and matrix instructions of only 16
// cycles: issuing a 1 KiB memory instruction (fragment read or direct load) holds a wavefront for about 34
// cycles (measured), so a single wavefront per SIMD that also feeds itself leaves the matrix pipe idle; with
// two per SIMD one issues matrix instructions while the other is held.
// Pipeline.  A stage of 32 k is one k-substep; one barrier per stage at its start makes stage kt+1 visible
// (its fragments are read during the matrix instructions of stage kt) and frees the slot of stage kt (read
// during stage kt-1) for stage kt+STAGES.  Wavefronts 0..3 fetch the A stage (2 TM blocks of 1 KiB each),
// wavefronts 4..7 the B stage (TN blocks each); the lane's offset is loop invariant and the k position is
// the scalar offset of the load, checked against the end of the K share only in the last few stages.
// Where it is used.  Its fixed cost per tile is lower than that of the kernel with fetch-only wavefronts
// and its time per k-step higher (K-major operands arrive as half cache lines in 32-k stages), so the host
// picks it for short K.
// =================================================================================================
// acc += a b, the accumulator tied to one AGPR quad.  Written as assembly because the compiler otherwise
// moves the four-register accumulators between registers around every matrix instruction.  No other
// matrix or vector instruction touches an accumulator within a stage, so no wait states are needed between
// these; the reader after the loop inserts them itself (mfma16_drain).
__device__ __forceinline__ void mfma16_inplace(f32x4& acc, const bf16x8& a, const bf16x8& b) {
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}
__device__ __forceinline__ void mfma16_drain() { asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7" ::: "memory"); }

template <int TM_, int TN_, int STAGES_>
struct Tile8 {
    static constexpr int TM = TM_, TN = TN_, STAGES = STAGES_;          // 32-row / 32-column units per wavefront
    static constexpr int BM = 4 * 32 * TM, BN = 2 * 32 * TN;
    static constexpr int A_BYTES = BM * DK * 2, B_BYTES = BN * DK * 2;
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr int LA = 2 * TM, LB = TN;                          // direct loads per stage of an A / B fetcher
    static constexpr int LMAX = LA > LB ? LA : LB;
    static constexpr int EROW = TN * 32 * 4 + 16, EWAVE = 32 * EROW;
    static constexpr int LDS_BYTES = STAGES * STAGE_BYTES > 8 * EWAVE ? STAGES * STAGE_BYTES : 8 * EWAVE;
    static_assert(STAGES * LMAX <= 63, "vmcnt is a 6-bit counter");
};

template <typename TL, bool A_KMAJ, bool B_KMAJ>
__global__ __launch_bounds__(512) void gemm_bf16_x16w8_kernel(GemmParams p) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    constexpr int TM = TL::TM, TN = TL::TN, BM = TL::BM, BN = TL::BN, DSTAGES = TL::STAGES;
    constexpr int FM = 2 * TM, FN = 2 * TN, NM = FM * FN;
    constexpr int LA = TL::LA, LB = TL::LB, LMAX = TL::LMAX;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const bool is_a = wave_u < 4;                                 // which operand this wavefront fetches
    const int wq = wave_u & 3;
    const KShare sh = k_share(p, share_of_block(blockIdx.x, gridDim.x));
    int tm, tn;
    tile_coords(sh.tile, p.tiles_m, p.tiles_n, p.band, tm, tn);
    const int m0 = tm * BM, n0 = tn * BN;

    // fetch state of this wavefront: descriptor, LDS position of its first block inside a stage, bytes per k,
    // per-lane offsets (rows / columns outside the matrix folded in) and the lane's k column (K-major only)
    const i32x4 ra = make_rsrc(p.A, (unsigned)((int64_t)(A_KMAJ ? p.M : p.K) * p.lda * 2));
    const i32x4 rb = make_rsrc(p.B, (unsigned)((int64_t)(B_KMAJ ? p.N : p.K) * p.ldb * 2));
    i32x4 rs;
#pragma unroll
    for (int q = 0; q < 4; ++q) rs[q] = is_a ? ra[q] : rb[q];
    const unsigned lds0 = (unsigned)(uintptr_t)(lds_void_ptr)smem;
    const unsigned lds_first = lds0 + (is_a ? wq * LA * 1024 : TL::A_BYTES + wq * LB * 1024);
    const unsigned kbytes = is_a ? (A_KMAJ ? 2u : (unsigned)p.lda * 2u) : (B_KMAJ ? 2u : (unsigned)p.ldb * 2u);
    const int nload = is_a ? LA : LB;
    unsigned vo[LMAX];
    int kc = 0;
    if (is_a) {
        unsigned off[LA]; bool ok[LA];
        dma_offsets<A_KMAJ, LA, false, true>(off, ok, kc, p.lda, m0, p.M, wq, lane);
#pragma unroll
        for (int d = 0; d < LMAX; ++d) vo[d] = d < LA ? ((A_KMAJ || ok[d < LA ? d : 0]) ? off[d < LA ? d : 0] : OOB_HALF) : OOB_HALF;
        if (!A_KMAJ) kc = 0;
    } else {
        unsigned off[LB]; bool ok[LB];
        dma_offsets<B_KMAJ, LB, false, true>(off, ok, kc, p.ldb, n0, p.N, wq, lane);
#pragma unroll
        for (int d = 0; d < LMAX; ++d) vo[d] = d < LB ? ((B_KMAJ || ok[d < LB ? d : 0]) ? off[d < LB ? d : 0] : OOB_HALF) : OOB_HALF;
        if (!B_KMAJ) kc = 0;
    }
    // load d of stage s (of this K share); CHECKED: the stage may reach past the end of the share
    auto dma_one = [&](int s, int d, auto checkedc) {
        if (d >= LA && is_a) return;
        if (d >= LB && !is_a) return;
        const unsigned k0 = (unsigned)(sh.kt0 + s) * DK;
        unsigned v = vo[d];
        if (decltype(checkedc)::value) v = (int)k0 + kc < sh.kend ? v : OOB_HALF;
        buffer_load_lds_b128_s(rs, lds_first + (s % DSTAGES) * TL::STAGE_BYTES + d * 1024, v, k0 * kbytes);
    };
    auto read_one = [&](bf16x8 (&fa)[FM], bf16x8 (&fb)[FN], int s, int r) {
        const char* buf = smem + (s % DSTAGES) * TL::STAGE_BYTES;
        if (r < FM) fa[r] = dma_frag16<A_KMAJ, BM>(buf, (wm * FM + r) * 16, lane);
        else fb[r - FM] = dma_frag16<B_KMAJ, BN>(buf + TL::A_BYTES, (wn * FN + r - FM) * 16, lane);
    };

    f32x4 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[i][j][v] = 0.0f;

    auto stage = [&](const bf16x8 (&fa)[FM], const bf16x8 (&fb)[FN], bf16x8 (&na)[FM], bf16x8 (&nb)[FN], int kt, auto checkedc) {
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j) {
                const int m = i * FN + j;
                mfma16_inplace(acc[i][j], fa[i], fb[j]);
                __builtin_amdgcn_sched_barrier(0);
                if (m < FM + FN) {
                    read_one(na, nb, kt + 1, m);
                    __builtin_amdgcn_sched_barrier(0);
                }
#pragma unroll
                for (int d = 0; d < LMAX; ++d)
                    if (m == ((2 * d + 1) * NM) / (2 * LMAX)) {
                        dma_one(kt + DSTAGES, d, checkedc);
                        __builtin_amdgcn_sched_barrier(0);
                    }
            }
    };
    using Fast = std::integral_constant<bool, false>;
    using Checked = std::integral_constant<bool, true>;
    // loads this wavefront may leave in flight with stage s+1 landed: those of the D-2 newer stages
    auto wait_stage = [&]() {
        if (LA == LB) wait_vmcnt<(DSTAGES - 2) * LA>();
        else if (is_a) wait_vmcnt<(DSTAGES - 2) * LA>();
        else wait_vmcnt<(DSTAGES - 2) * LB>();
    };

#pragma unroll
    for (int s0 = 0; s0 < DSTAGES; ++s0)
#pragma unroll
        for (int d = 0; d < LMAX; ++d) dma_one(s0, d, Checked{});
    if (LA == LB) wait_vmcnt<(DSTAGES - 1) * LA>();              // stage 0 has landed
    else if (is_a) wait_vmcnt<(DSTAGES - 1) * LA>();
    else wait_vmcnt<(DSTAGES - 1) * LB>();
    __builtin_amdgcn_s_barrier();
    bf16x8 fa0[FM], fb0[FN], fa1[FM], fb1[FN];
#pragma unroll
    for (int r = 0; r < FM + FN; ++r) read_one(fa0, fb0, 0, r);
    __builtin_amdgcn_sched_barrier(0);

    auto sync = [&]() {
        wait_stage();
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
    };
    const int nfast = (sh.kend - sh.kt0 * DK) / DK - DSTAGES;
    int kt = 0;
    for (; kt + 1 < nfast; kt += 2) {
        sync();
        stage(fa0, fb0, fa1, fb1, kt, Fast{});
        sync();
        stage(fa1, fb1, fa0, fb0, kt + 1, Fast{});
    }
    for (; kt + 1 < sh.nk; kt += 2) {
        sync();
        stage(fa0, fb0, fa1, fb1, kt, Checked{});
        sync();
        stage(fa1, fb1, fa0, fb0, kt + 1, Checked{});
    }
    if (kt < sh.nk) {
        sync();
        stage(fa0, fb0, fa1, fb1, kt, Checked{});
    }
    mfma16_drain();
    wait_vmcnt<0>();
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    epilogue16<TL>(p, acc, smem, wave, lane, m0, n0, sh.partial);
}

// =================================================================================================
// Variant with specialised wavefronts: 512 threads, wavefronts 0..3 only compute (2 x 2, each
// TM x TN blocks), wavefronts 4..7 only fetch.  Both roles meet at the same barriers: one before the
// loop, one per k-step of 32, one after.
//
// LDS rings.  B lives in a ring of NB slots of 32 k.  A K-major A lives in a ring of 3 slots of 64 k
// (rows of 128 bytes): a direct load then covers 8 whole 128-byte lines instead of 16 half lines,
// which the vector memory path serves about 1.4 times faster (measured), and global->LDS
// throughput is what bounds this kernel once the loads no longer hold up matrix instructions.
// (B stays at 32 k: three 64-k slots of both operands do not fit in 160 KiB.)  An MN-major A uses
// a ring of NB slots of 32 k like B.  Slot of k-step kt: B kt % NB; wide A (kt / 2) % 3.
//
// Fetch order.  After the barrier of k-step kt the B slot of kt is free and is refilled with k-step
// kt + NB.  A wide A slot (unit u = k-steps 2u, 2u+1) is free after the barrier of k-step 2u+1; unit
// u+3 is fetched in two halves, after that barrier and after the next one, so every k-step issues
// TM + TN loads per fetching wavefront.
// =================================================================================================
template <int TM_, int TN_>
struct SpecTile {
    static constexpr int TM = TM_, TN = TN_, BM = 64 * TM, BN = 64 * TN;
    static constexpr int NB = 5, NA_WIDE = 3;
    static constexpr int B_SLOT = BN * DK * 2;                           // 32 k of B
    static constexpr int A_SLOT32 = BM * DK * 2, A_SLOT64 = BM * 64 * 2;
    static constexpr int EROW = TN * 32 * 4 + 16, EWAVE = 32 * EROW;     // epilogue staging, as in Tile
    template <bool A_KMAJ> static constexpr int a_bytes() { return A_KMAJ ? NA_WIDE * A_SLOT64 : NB * A_SLOT32; }
    template <bool A_KMAJ> static constexpr int lds_bytes() {
        return a_bytes<A_KMAJ>() + NB * B_SLOT > 8 * EWAVE ? a_bytes<A_KMAJ>() + NB * B_SLOT : 8 * EWAVE;   // 8: two staging buffers per math wavefront
    }
};

// One operand's loads of one k range [k0, k0 + KSPAN) by a fetching wavefront: NL loads, load i to LDS block
// lds_first + 1024 i.  off[i] is the lane's loop-invariant byte offset (k = 0; rows or columns outside the matrix
// already point past the buffer), kin[i] the lane's k position inside the range (K-major: its chunk's first k;
// MN-major: its row), kstep_bytes the bytes per unit of k (2 for K-major, 2 ld for MN-major).
//  * range inside the K share: the k position is the load's SCALAR offset, the lane offset is used as it is;
//  * range past the end of the share: a descriptor of zero records (nothing is read, zeros land in LDS);
//  * range that straddles the end (K not a multiple of the range): per-lane check, the only case with vector
//    instructions.  A vector instruction issued by a fetching wavefront takes an issue slot from the matrix
//    instructions of the math wavefront on the same SIMD (measured: about 2 cycles of matrix-pipe time each), which
//    is why the steady state has none.
template <int NL, int KSPAN>
__device__ __forceinline__ void fetch_range(const i32x4& rsrc, unsigned lds_first, const unsigned (&off)[NL],
                                            const int (&kin)[NL], int k0, int kend, unsigned kstep_bytes) {
    if (k0 >= kend) {
        i32x4 r = rsrc;
        r[2] = 0;
#pragma unroll
        for (int i = 0; i < NL; ++i) buffer_load_lds_b128_s(r, lds_first + i * 1024, off[i], 0u);
    } else if (k0 + KSPAN <= kend) {
        // (the compiler does not always see that the product is wave-uniform)
        const unsigned so = (unsigned)__builtin_amdgcn_readfirstlane((int)((unsigned)k0 * kstep_bytes));
#pragma unroll
        for (int i = 0; i < NL; ++i) buffer_load_lds_b128_s(rsrc, lds_first + i * 1024, off[i], so);
    } else {
#pragma unroll
        for (int i = 0; i < NL; ++i)
            buffer_load_lds_b128(rsrc, lds_first + i * 1024,
                                 k0 + kin[i] < kend ? off[i] + (unsigned)k0 * kstep_bytes : OOB_OFFSET);
    }
}

// K-major tile with rows of 128 bytes (64 k): 16-byte chunk c of row r sits at position c ^ ((r >> 1) & 7),
// so the 16 rows a quarter-wavefront reads at one k are spread over all banks.
__device__ __forceinline__ int swz_k64(int row) { return (row >> 1) & 7; }
__device__ __forceinline__ bf16x8 wide_frag(const char* tile, int mn_base, int k16, int lane) {
    int row = mn_base + (lane & 31);
    int c = 2 * k16 + (lane >> 5);
    return *reinterpret_cast<const bf16x8*>(tile + row * 128 + ((c ^ swz_k64(row)) << 4));
}

template <typename ST, bool A_KMAJ, bool B_KMAJ>
__global__ __launch_bounds__(512) void gemm_bf16_spec_kernel(GemmParams p) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    constexpr int TM = ST::TM, TN = ST::TN, BM = ST::BM, BN = ST::BN, NB = ST::NB, NAW = ST::NA_WIDE;
    constexpr bool WIDE = A_KMAJ;
    constexpr int A_BYTES = ST::template a_bytes<A_KMAJ>();
    constexpr int LPS = TM + TN;                                  // loads per k-step and fetching wavefront
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const KShare sh = k_share(p, share_of_block(blockIdx.x, gridDim.x));   // sh.kt0 is even (host)
    int tm, tn;
    tile_coords(sh.tile, p.tiles_m, p.tiles_n, p.band, tm, tn);
    const int m0 = tm * BM, n0 = tn * BN;

    if (wave >= 4) {
        // ---------------- fetching wavefronts ----------------
        const int w = __builtin_amdgcn_readfirstlane(wave) & 3;
        const i32x4 ra = make_rsrc(p.A, (unsigned)((int64_t)(A_KMAJ ? p.M : p.K) * p.lda * 2));
        const i32x4 rb = make_rsrc(p.B, (unsigned)((int64_t)(B_KMAJ ? p.N : p.K) * p.ldb * 2));
        const unsigned lds_a = (unsigned)(uintptr_t)(lds_void_ptr)smem, lds_b = lds_a + A_BYTES;
        // Lane offsets of this wavefront's loads (see fetch_range): B and a narrow A as in the kernel above; a wide A
        // unit is 2 TM loads, load q covering rows 8 (2 TM w + q) .. + 7, lane l the chunk at LDS position l % 8 of
        // row l / 8.
        unsigned offb[TN], offa[TM], offw0[TM], offw1[TM];
        int kinb[TN], kina[TM], kinw0[TM], kinw1[TM];
        {
            bool okb[TN];
            int kc;
            dma_offsets<B_KMAJ, TN>(offb, okb, kc, p.ldb, n0, p.N, w, lane);
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                if (!B_KMAJ) offb[j] = okb[j] ? offb[j] : OOB_HALF;
                kinb[j] = B_KMAJ ? kc : mn_krow<TN>(w, j, lane);
            }
        }
        if (WIDE) {
#pragma unroll
            for (int q = 0; q < 2 * TM; ++q) {
                const int row = (w * 2 * TM + q) * 8 + (lane >> 3);
                const int c = (lane & 7) ^ swz_k64(row);
                const unsigned o = m0 + row < p.M ? (unsigned)(((int64_t)(m0 + row) * p.lda + c * 8) * 2) : OOB_HALF;
                if (q < TM) { offw0[q] = o; kinw0[q] = c * 8; }
                else { offw1[q - TM] = o; kinw1[q - TM] = c * 8; }
            }
        } else {
            bool oka[TM];
            int kc;
            dma_offsets<A_KMAJ, TM>(offa, oka, kc, p.lda, m0, p.M, w, lane);
#pragma unroll
            for (int j = 0; j < TM; ++j) {
                if (!A_KMAJ) offa[j] = oka[j] ? offa[j] : OOB_HALF;
                kina[j] = A_KMAJ ? kc : mn_krow<TM>(w, j, lane);
            }
        }
        const unsigned kb_bytes = B_KMAJ ? 2u : (unsigned)p.ldb * 2u, ka_bytes = A_KMAJ ? 2u : (unsigned)p.lda * 2u;
        // k-steps kt and wide units u below count from the start of this workgroup's K share
        auto load_b = [&](int kt) {                               // k-step kt of B into its slot
            fetch_range<TN, DK>(rb, lds_b + (kt % NB) * ST::B_SLOT + w * TN * 1024, offb, kinb, (sh.kt0 + kt) * DK, sh.kend,
                                kb_bytes);
        };
        auto load_a32 = [&](int kt) {
            fetch_range<TM, DK>(ra, lds_a + (kt % NB) * ST::A_SLOT32 + w * TM * 1024, offa, kina, (sh.kt0 + kt) * DK, sh.kend,
                                ka_bytes);
        };
        auto load_a64 = [&](int u, int half) {                    // half 0/1 of unit u (k = 64 u ..)
            const unsigned buf = lds_a + (u % NAW) * ST::A_SLOT64 + (w * 2 * TM + half * TM) * 1024;
            const int k0 = 64 * ((sh.kt0 >> 1) + u);
            if (half == 0) fetch_range<TM, 64>(ra, buf, offw0, kinw0, k0, sh.kend, 2u);
            else fetch_range<TM, 64>(ra, buf, offw1, kinw1, k0, sh.kend, 2u);
        };
        // prologue: everything the rings hold, except the second half of the last wide unit
        if (WIDE) {
            load_a64(0, 0); load_a64(0, 1); load_b(0);
            load_a64(1, 0); load_a64(1, 1); load_a64(2, 0);
#pragma unroll
            for (int s0 = 1; s0 < NB; ++s0) load_b(s0);
            wait_vmcnt<3 * TM + (NB - 1) * TN>();                 // unit 0 and B step 0 have landed
        } else {
            load_a32(0); load_b(0);
#pragma unroll
            for (int s0 = 1; s0 < NB; ++s0) { load_a32(s0); load_b(s0); }
            wait_vmcnt<(NB - 1) * LPS>();
        }
        __builtin_amdgcn_s_barrier();
        // Loads in flight allowed at the barrier of k-step kt (k-step kt+1 must have landed).  B step
        // kt+1 went out as the last loads of k-step kt+1-NB; the second half of a wide unit that starts
        // at kt+1 went out as the first loads of k-step kt-3.
        constexpr int W_B = (NB - 2) * LPS;
        constexpr int W_A = WIDE ? TN + 2 * LPS : TN + (NB - 2) * LPS;
        constexpr int W = W_A < W_B ? W_A : W_B;
        for (int kt = 0; kt < sh.nk; ++kt) {
            // The first two k-steps of a wide A come straight after the prologue, which ends with the
            // B steps: fewer loads follow the ones needed than in the steady state.
            if (WIDE && kt == 0) wait_vmcnt<(NB - 2) * TN>();                  // B step 1
            else if (WIDE && kt == 1) wait_vmcnt<(NB - 3) * TN + LPS>();       // unit 1, B step 2
            else wait_vmcnt<W>();
            __builtin_amdgcn_s_barrier();                         // k-step kt has been read by everyone
            if (WIDE) {
                // odd kt = 2u+1 frees unit u: first half of unit u+3; even kt = 2u+2: its second half
                if (kt & 1) load_a64((kt >> 1) + 3, 0);
                else load_a64((kt >> 1) + 2, 1);
            } else {
                load_a32(kt + NB);
            }
            load_b(kt + NB);
        }
        wait_vmcnt<0>();                                          // nothing lands in LDS during the epilogue
        __builtin_amdgcn_s_barrier();
        epilogue_helper<ST>(p, smem, wave, lane, m0, n0, sh.partial);   // shares the rows of math wavefront wave - 4
        return;
    }

    // ---------------- math wavefronts ----------------
    const int wm = wave >> 1, wn = wave & 1;
    constexpr int NM = TM * TN;
    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;
    // Registers: the accumulators take 3/4 of a wavefront's budget (two wavefronts per SIMD), so only
    // the B fragments and the last A fragment are double buffered; A fragment i < TM-1 of the next
    // k-substep is read into the registers of the current one once row i's matrix instructions are issued.
    bf16x8 fa[TM - 1], fal[2], fb[2][TN];
    auto rd_a = [&](bf16x8& dst, int kt, int ks, int i) {         // k-substep ks (16 k) of k-step kt
        if (WIDE) dst = wide_frag(smem + ((kt >> 1) % NAW) * ST::A_SLOT64, (wm * TM + i) * 32, (kt & 1) * 2 + ks, lane);
        else dst = dma_frag<A_KMAJ, BM>(smem + (kt % NB) * ST::A_SLOT32, (wm * TM + i) * 32, ks, lane);
    };
    auto rd_b = [&](bf16x8& dst, int kt, int ks, int j) {
        dst = dma_frag<B_KMAJ, BN>(smem + A_BYTES + (kt % NB) * ST::B_SLOT, (wn * TN + j) * 32, ks, lane);
    };
    auto mhalf = [&](auto curc, int rkt, int rks) {
        constexpr int CUR = decltype(curc)::value, NXT = CUR ^ 1;
        int free_rd = 0;                                          // next of: B fragments 0..TN-1, last A fragment
#pragma unroll
        for (int m = 0; m < NM; ++m) {
            const int i = m / TN, j = m % TN;
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(i < TM - 1 ? fa[i] : fal[CUR], fb[CUR][j], acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            if (j == TN - 1 && i < TM - 1) {
                rd_a(fa[i], rkt, rks, i);                         // row i is done: refill in place
                __builtin_amdgcn_sched_barrier(0);
            } else if (free_rd <= TN) {
                if (free_rd < TN) rd_b(fb[NXT][free_rd], rkt, rks, free_rd);
                else rd_a(fal[NXT], rkt, rks, TM - 1);
                ++free_rd;
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };
    using C0 = std::integral_constant<int, 0>;
    using C1 = std::integral_constant<int, 1>;
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int i = 0; i < TM - 1; ++i) rd_a(fa[i], 0, 0, i);
    rd_a(fal[0], 0, 0, TM - 1);
#pragma unroll
    for (int j = 0; j < TN; ++j) rd_b(fb[0][j], 0, 0, j);
    __builtin_amdgcn_sched_barrier(0);
    for (int kt = 0; kt < sh.nk; ++kt) {
        mhalf(C0{}, kt, 1);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        mhalf(C1{}, kt + 1, 0);
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    epilogue_shared<ST>(p, acc, smem, wave, lane, m0, n0, sh.partial);
}

// Sum of the K shares in share order, then the epilogue; 8 columns per thread, every access 16 or 32 bytes.
__global__ __launch_bounds__(256) void gemm_sum_shares_kernel(GemmParams p, int shares) {
    const int64_t chunk = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t idx = chunk * 8;
    const int64_t mn = (int64_t)p.M * p.N;
    if (idx >= mn) return;
    float v8[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int s = 0; s < shares; ++s) {
        const float4* src = reinterpret_cast<const float4*>(p.partial + s * mn + idx);
        const float4 x0 = src[0], x1 = src[1];
        v8[0] += x0.x; v8[1] += x0.y; v8[2] += x0.z; v8[3] += x0.w;
        v8[4] += x1.x; v8[5] += x1.y; v8[6] += x1.z; v8[7] += x1.w;
    }
    if (p.bias) {
        float b8[8];
        unpack8(*reinterpret_cast<const uint4*>(p.bias + idx % p.N), b8);
#pragma unroll
        for (int e = 0; e < 8; ++e) v8[e] += b8[e];
    }
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


// =================================================================================================
// Fetch and math wavefronts on the 16x16x32 matrix instruction (K-major A only): the tile, the rings and the
// fetching wavefronts of the kernel above, the matrix instruction of the 8-wavefront kernel.  A math wavefront
// owns 128 x 96 = 8 x 6 blocks: 192 accumulator registers of the 256 a wavefront has at two per SIMD, so
// fragments cannot be double buffered.  The 6 B fragments of a k-step stay in registers; the 8 A fragments
// (one per row of blocks, used for 6 consecutive instructions) rotate through four register sets, each refilled
// two rows ahead of its use.  A B fragment is refilled with the next k-step's as soon as it is dead: the last
// two rows are walked column by column, so B fragment j is dead after two instructions, and the next k-step
// starts with two rows walked the same way, which gives every B fragment ten instructions (160 cycles) to
// arrive.  Because the last fragment reads of k-step kt+1 are still in flight when k-step kt ends, the slot of
// k-step kt is handed back to the fetching wavefronts one barrier later than above (at barrier kt+1), and the
// fetch schedule is one k-step shorter: after barrier j, B k-step j+4 and (j even) the whole A unit j/2+2.
// =================================================================================================
__device__ __forceinline__ bf16x8 wide_frag16(const char* tile, int mn_base, int k32, int lane) {
    int row = mn_base + (lane & 15);
    int c = 4 * k32 + (lane >> 4);
    return *reinterpret_cast<const bf16x8*>(tile + row * 128 + ((c ^ swz_k64(row)) << 4));
}
__device__ __forceinline__ void mfma16_v(f32x4& acc, const bf16x8& a, const bf16x8& b) {
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "v"(b));
}

template <typename ST, bool B_KMAJ>
__global__ __launch_bounds__(512) void gemm_bf16_spec16_kernel(GemmParams p) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    constexpr int TM = ST::TM, TN = ST::TN, BM = ST::BM, BN = ST::BN, NB = ST::NB, NAW = ST::NA_WIDE;
    constexpr int A_BYTES = ST::template a_bytes<true>();
    constexpr int LA = 2 * TM, LBW = TN;                          // loads per fetching wavefront: A unit, B k-step
    static_assert(NB == 5 && NAW == 3, "the fetch schedule below is written for these ring depths");
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const KShare sh = k_share(p, share_of_block(blockIdx.x, gridDim.x));   // sh.kt0 is even (host)
    int tm, tn;
    tile_coords(sh.tile, p.tiles_m, p.tiles_n, p.band, tm, tn);
    const int m0 = tm * BM, n0 = tn * BN;

    if (wave >= 4) {
        // ---------------- fetching wavefronts ----------------
        const int w = __builtin_amdgcn_readfirstlane(wave) & 3;
        const i32x4 ra = make_rsrc(p.A, (unsigned)((int64_t)p.M * p.lda * 2));
        const i32x4 rb = make_rsrc(p.B, (unsigned)((int64_t)(B_KMAJ ? p.N : p.K) * p.ldb * 2));
        const unsigned lds_a = (unsigned)(uintptr_t)(lds_void_ptr)smem, lds_b = lds_a + A_BYTES;
        // lane offsets of this wavefront's loads (see fetch_range)
        unsigned offb[TN], offw[LA];
        int kinb[TN], kinw[LA];
        {
            bool okb[TN];
            int kc;
            dma_offsets<B_KMAJ, TN, true, true>(offb, okb, kc, p.ldb, n0, p.N, w, lane);
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                if (!B_KMAJ) offb[j] = okb[j] ? offb[j] : OOB_HALF;
                kinb[j] = B_KMAJ ? kc : mn_krow<TN>(w, j, lane);
            }
        }
#pragma unroll
        for (int q = 0; q < LA; ++q) {
            const int row = (w * LA + q) * 8 + (lane >> 3);
            const int c = (lane & 7) ^ swz_k64(row);
            kinw[q] = c * 8;
            offw[q] = m0 + row < p.M ? (unsigned)(((int64_t)(m0 + row) * p.lda + c * 8) * 2) : OOB_HALF;
        }
        const unsigned kb_bytes = B_KMAJ ? 2u : (unsigned)p.ldb * 2u;
        auto load_b = [&](int kt) {                               // k-step kt (of this K share) of B into its slot
            fetch_range<TN, DK>(rb, lds_b + (kt % NB) * ST::B_SLOT + w * TN * 1024, offb, kinb, (sh.kt0 + kt) * DK, sh.kend,
                                kb_bytes);
        };
        auto load_a = [&](int u) {                                // unit u (k-steps 2u, 2u+1 of this K share) of A
            fetch_range<LA, 64>(ra, lds_a + (u % NAW) * ST::A_SLOT64 + w * LA * 1024, offw, kinw, 64 * ((sh.kt0 >> 1) + u),
                                sh.kend, 2u);
        };
        load_a(0); load_b(0); load_b(1); load_a(1); load_b(2); load_b(3);
        wait_vmcnt<LA + 3 * LBW>();                               // unit 0 and B k-step 0 have landed
        __builtin_amdgcn_s_barrier();
        // At barrier kt k-step kt+1 must have landed.  Loads go out in batches after each barrier (the A unit,
        // then the B k-step); the two newest batches, LA + 2 LBW loads, may still be in flight.
        for (int kt = 0; kt < sh.nk; ++kt) {
            wait_vmcnt<LA + 2 * LBW>();
            __builtin_amdgcn_s_barrier();                         // k-step kt-1 has been read by everyone
            if ((kt & 1) == 0) load_a((kt >> 1) + 2);
            load_b(kt + NB - 1);
        }
        wait_vmcnt<0>();                                          // nothing lands in LDS during the epilogue
        __builtin_amdgcn_s_barrier();
        epilogue_helper<ST>(p, smem, wave, lane, m0, n0, sh.partial);   // shares the rows of math wavefront wave - 4
        return;
    }

    // ---------------- math wavefronts ----------------
    const int wm = wave >> 1, wn = wave & 1;
    constexpr int FM = 2 * TM, FN = 2 * TN;
    static_assert(FM >= 4, "head and tail pairs need four rows of blocks");
    f32x4 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[i][j][v] = 0.0f;
    static_assert(FM == 8, "the row schedule below is written for 8 rows of blocks");
    bf16x8 fa[4], fb[FN];                                         // A fragments rotate through four registers sets
    auto rd_a = [&](int kt, int row, int r) {                     // row `row` of k-step kt into set r
        fa[r] = wide_frag16(smem + ((kt >> 1) % NAW) * ST::A_SLOT64, (wm * FM + row) * 16, kt & 1, lane);
        __builtin_amdgcn_sched_barrier(0);
    };
    // MN-major B (rows of BN values per k, chunk c of row k at position c ^ xor16(k)): fragment f = wn FN + j of
    // the tile is chunks 2f, 2f+1; a lane reads rows k = 8 (lane/16) + 4 h + (lane%16)/4, h = 0, 1, whose xor16
    // does not depend on h, so fragment f sits at bpos[(f ^ x) & 3] + 128 (f / 4) + 1536 h with x fixed per lane:
    // four base registers, everything else immediates and scalars.
    unsigned bpos[4];
    int bq[FN], bs[FN];                                           // per fragment: which base, scalar byte offset
    if (!B_KMAJ) {
        const int k0 = 8 * (lane >> 4) + ((lane & 15) >> 2);
        const int x = ((lane >> 3) & 1) | (((lane >> 4) & 1) << 1);
        const unsigned base = (unsigned)(k0 * (BN * 2) + 8 * (lane & 1) + 16 * ((lane & 3) >> 1));
#pragma unroll
        for (int q = 0; q < 4; ++q) bpos[q] = base + 32u * (unsigned)((q + 2 * wn) & 3 ^ x);
#pragma unroll
        for (int j = 0; j < FN; ++j) { bq[j] = j & 3; bs[j] = 128 * ((wn * FN + j) >> 2); }
    }
    auto rd_b = [&](int kt, int j) {
        const char* slot = smem + A_BYTES + (kt % NB) * ST::B_SLOT;
        if (B_KMAJ) {
            fb[j] = dma_frag16<true, BN>(slot, (wn * FN + j) * 16, lane);
        } else {
            const char* src = slot + __builtin_amdgcn_readfirstlane(bs[j]) + bpos[bq[j]];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(src + h * 4 * (BN * 2)));
                bf16x4 b4 = __builtin_bit_cast(bf16x4, v);
                fb[j][4 * h + 0] = b4[0]; fb[j][4 * h + 1] = b4[1]; fb[j][4 * h + 2] = b4[2]; fb[j][4 * h + 3] = b4[3];
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    auto mm = [&](int i, int r, int j) {                          // block (i, j) with the A fragment in set r
        mfma16_v(acc[i][j], fa[r], fb[j]);
        __builtin_amdgcn_sched_barrier(0);
    };
    // reads still in flight at the end of a k-step: the FN B fragments and 2 A fragments of its last lines
    constexpr int TAIL_READS = (B_KMAJ ? FN : 2 * FN) + 2;
    static_assert(TAIL_READS <= 15, "lgkmcnt is a 4-bit counter");
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int r = 0; r < 4; ++r) rd_a(0, r, r);
#pragma unroll
    for (int j = 0; j < FN; ++j) rd_b(0, j);
    // Row schedule of a k-step (sets 0..3 hold rows 0..3 at its start):
    //   rows 0,1 column by column | read rows 4,5 -> sets 0,1 | row 2, read row 6 -> set 2 | row 3, read row 7 -> set 3
    //   | row 4, read next row 0 -> set 0 | row 5, read next row 1 -> set 1
    //   | rows 6,7 column by column, each B fragment refilled once both have used it | read next rows 2,3 -> sets 2,3
    for (int kt = 0; kt < sh.nk; ++kt) {
        asm volatile("s_waitcnt lgkmcnt(%0)" :: "n"(TAIL_READS) : "memory");   // every read of k-step kt-1's slots is done
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < FN; ++j) { mm(0, 0, j); mm(1, 1, j); }
        rd_a(kt, 4, 0);
        rd_a(kt, 5, 1);
#pragma unroll
        for (int j = 0; j < FN; ++j) mm(2, 2, j);
        rd_a(kt, 6, 2);
#pragma unroll
        for (int j = 0; j < FN; ++j) mm(3, 3, j);
        rd_a(kt, 7, 3);
#pragma unroll
        for (int j = 0; j < FN; ++j) mm(4, 0, j);
        rd_a(kt + 1, 0, 0);
#pragma unroll
        for (int j = 0; j < FN; ++j) mm(5, 1, j);
        rd_a(kt + 1, 1, 1);
#pragma unroll
        for (int j = 0; j < FN; ++j) {
            mm(6, 2, j); mm(7, 3, j);
            rd_b(kt + 1, j);
        }
        rd_a(kt + 1, 2, 2);
        rd_a(kt + 1, 3, 3);
    }
    mfma16_drain();
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    epilogue16_shared<ST>(p, acc, smem, wave, lane, m0, n0, sh.partial);
}

// =================================================================================================
// 192 x 192, two workgroups per compute unit, on the 16x16x32 matrix instruction: the tile of the weight
// gradients (short K, where co-resident workgroups hide each other's start and end) at the lower energy per flop
// of this instruction.  Four wavefronts that fetch and compute; each owns 96 x 96 = 6 x 6 blocks, 144
// accumulator registers, and since two workgroups share a SIMD's registers fragments are single buffered as in
// the kernel above: six B fragments refilled in a column-wise tail, A fragments rotating through four register
// sets.  The sets hold rows 0..3 at the start of a k-step and rows 2,3,0,1 of the next at its end, so two k-steps
// (ROT = 0, 2) are unrolled.  One barrier per k-step, placed after the third row: by then every read of the
// current stage has been issued (rows 4, 5 are fetched right after the first two rows), so the barrier frees this
// stage's slot for stage kt+3 and makes stage kt+1 visible for the reads that follow it.
// =================================================================================================
template <typename TL, bool A_KMAJ, bool B_KMAJ, bool COLSUM = false>
__global__ __launch_bounds__(256, 2) void gemm_bf16_x16s_kernel(GemmParams p) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    constexpr int TM = TL::TM, TN = TL::TN, BM = TL::BM, BN = TL::BN, DSTAGES = TL::STAGES;
    constexpr int FM = 2 * TM, FN = 2 * TN, L = TL::LOADS, LH = L / 2;
    static_assert(FM == 6 && DSTAGES == 3 && L % 2 == 0, "row schedule and ring accounting are written for this tile");
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const KShare sh = k_share(p, share_of_block(blockIdx.x, gridDim.x));
    const i32x4 ra = make_rsrc(p.A, (unsigned)((int64_t)(A_KMAJ ? p.M : p.K) * p.lda * 2));
    const i32x4 rb = make_rsrc(p.B, (unsigned)((int64_t)(B_KMAJ ? p.N : p.K) * p.ldb * 2));
    const unsigned lds0 = (unsigned)(uintptr_t)(lds_void_ptr)smem;
    int tm, tn;
    tile_coords(sh.tile, p.tiles_m, p.tiles_n, p.band, tm, tn);
    const int m0 = tm * BM, n0 = tn * BN;

    f32x4 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[i][j][v] = 0.0f;

    unsigned offa[TM], offb[TN];
    bool oka[TM], okb[TN];
    int kca, kcb;
    dma_offsets<A_KMAJ, TM, true, true>(offa, oka, kca, p.lda, m0, p.M, wave, lane);
    dma_offsets<B_KMAJ, TN, true, true>(offb, okb, kcb, p.ldb, n0, p.N, wave, lane);
    // MN-major operands: the lane's offset is loop invariant (columns outside the matrix folded in), the k position
    // is the load's scalar offset, and a stage past the end of the K share reads through a descriptor of zero
    // records (everything out of bounds), so such a load costs no vector arithmetic at all.
#pragma unroll
    for (int d = 0; d < TM; ++d) if (!A_KMAJ) offa[d] = oka[d] ? offa[d] : OOB_HALF;
#pragma unroll
    for (int e = 0; e < TN; ++e) if (!B_KMAJ) offb[e] = okb[e] ? offb[e] : OOB_HALF;
    auto dma_one = [&](int slot_off, int s, int d) {              // load d of stage s (of this K share) into its slot
        const unsigned buf = lds0 + (unsigned)slot_off;
        const int k0 = (sh.kt0 + s) * DK;
        if (d < TM) {
            const unsigned dst = buf + (wave_u * TM + d) * 1024;
            if (A_KMAJ) {
                buffer_load_lds_b128(ra, dst, k0 + kca < sh.kend ? offa[d] + (unsigned)k0 * 2u : OOB_OFFSET);
            } else {
                i32x4 r = ra;
                r[2] = k0 < sh.kend ? ra[2] : 0;
                buffer_load_lds_b128_s(r, dst, offa[d], (unsigned)k0 * (unsigned)p.lda * 2u);
            }
        } else {
            const int e = d - TM;
            const unsigned dst = buf + TL::A_BYTES + (wave_u * TN + e) * 1024;
            if (B_KMAJ) {
                buffer_load_lds_b128(rb, dst, k0 + kcb < sh.kend ? offb[e] + (unsigned)k0 * 2u : OOB_OFFSET);
            } else {
                i32x4 r = rb;
                r[2] = k0 < sh.kend ? rb[2] : 0;
                buffer_load_lds_b128_s(r, dst, offb[e], (unsigned)k0 * (unsigned)p.ldb * 2u);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    bf16x8 fa[4], fb[FN];
    // MN-major operands use the xor16 chunk positions and four per-lane base registers (see the kernel above)
    unsigned apos[4], bpos[4];
    {
        const int k0 = 8 * (lane >> 4) + ((lane & 15) >> 2);
        const int x = ((lane >> 3) & 1) | (((lane >> 4) & 1) << 1);
        const unsigned lane_off = (unsigned)(8 * (lane & 1) + 16 * ((lane & 3) >> 1));
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            apos[q] = (unsigned)(k0 * (BM * 2)) + lane_off + 32u * (unsigned)(((q + 2 * wm) & 3) ^ x);
            bpos[q] = (unsigned)(k0 * (BN * 2)) + lane_off + 32u * (unsigned)(((q + 2 * wn) & 3) ^ x);
        }
    }
    auto rd_mn = [&](bf16x8& dst, const char* tile, const unsigned (&pos)[4], int w, int f, int R) {
        const char* src = tile + __builtin_amdgcn_readfirstlane(128 * ((w * 6 + f) >> 2)) + pos[f & 3];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(src + h * 4 * (R * 2)));
            bf16x4 b4 = __builtin_bit_cast(bf16x4, v);
            dst[4 * h + 0] = b4[0]; dst[4 * h + 1] = b4[1]; dst[4 * h + 2] = b4[2]; dst[4 * h + 3] = b4[3];
        }
    };
    auto rd_a = [&](int slot_off, int row, int r) {
        const char* tile = smem + slot_off;
        if (A_KMAJ) fa[r] = dma_frag16<true, BM>(tile, (wm * FM + row) * 16, lane);
        else rd_mn(fa[r], tile, apos, wm, row, BM);
        __builtin_amdgcn_sched_barrier(0);
    };
    auto rd_b = [&](int slot_off, int j) {
        const char* tile = smem + slot_off + TL::A_BYTES;
        if (B_KMAJ) fb[j] = dma_frag16<true, BN>(tile, (wn * FN + j) * 16, lane);
        else rd_mn(fb[j], tile, bpos, wn, j, BN);
        __builtin_amdgcn_sched_barrier(0);
    };
    auto mm = [&](int i, int r, int j) {
        mfma16_v(acc[i][j], fa[r], fb[j]);
        __builtin_amdgcn_sched_barrier(0);
    };
    // k-step kt with the A sets rotated by ROT (0 or 2): logical set q is register set (q + ROT) & 3.
    // o0, o1, o2: byte offsets of the ring slots of stages kt, kt+1, kt+2 (stage kt+3 reuses o0).
    // COLSUM: the column sums of B over k (a bias gradient: B = dY, k = tokens) ride along as one more output row.
    // A fragment of ones in place of A makes every row of a 16 x 16 block the sum over the k-step of B's columns, in
    // float on the matrix cores and in k order; only the wavefronts that hold the first rows of tile row 0 do it
    // (six more matrix instructions per k-step for them), and they run their own copy of the loop, so the others
    // pay nothing.
    f32x4 cs[COLSUM ? FN : 1];
    bf16x8 ones;
#pragma unroll
    for (int e = 0; e < 8; ++e) ones[e] = (bf16_t)1.0f;
#pragma unroll
    for (int j = 0; j < (COLSUM ? FN : 1); ++j)
#pragma unroll
        for (int v = 0; v < 4; ++v) cs[j][v] = 0.0f;
    auto stage = [&](int kt, int o0, int o1, int o2, auto rotc, auto csc) __attribute__((always_inline)) {
        constexpr int ROT = decltype(rotc)::value;
        constexpr bool CS = decltype(csc)::value;
        constexpr int S0 = ROT & 3, S1 = (1 + ROT) & 3, S2 = (2 + ROT) & 3, S3 = (3 + ROT) & 3;
#pragma unroll
        for (int j = 0; j < FN; ++j) {                            // rows 0, 1 column by column
            mm(0, S0, j); mm(1, S1, j);
            if constexpr (CS) { mfma16_v(cs[j], ones, fb[j]); __builtin_amdgcn_sched_barrier(0); }
            if (j == 1) dma_one(o2, kt + 2, LH);                  // second half of stage kt+2's loads
            if (j == 3) dma_one(o2, kt + 2, LH + 1);
        }
        rd_a(o0, 4, S0);
        rd_a(o0, 5, S1);
#pragma unroll
        for (int j = 0; j < FN; ++j) {
            mm(2, S2, j);
            if (j == 1) dma_one(o2, kt + 2, LH + 2);
        }
        // every read of stage kt has been issued; stage kt+1 has landed once only stage kt+2's loads are in flight
        wait_vmcnt<L>();
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        rd_a(o1, 0, S2);
#pragma unroll
        for (int j = 0; j < FN; ++j) {
            mm(3, S3, j);
            if (j == 2) dma_one(o0, kt + 3, 0);                   // first half of stage kt+3's loads: slot of stage kt
        }
        rd_a(o1, 1, S3);
#pragma unroll
        for (int j = 0; j < FN; ++j) {                            // rows 4, 5 column by column; B refilled when dead
            mm(4, S0, j); mm(5, S1, j);
            rd_b(o1, j);
            if (j == 1) dma_one(o0, kt + 3, 1);
            if (j == 4) dma_one(o0, kt + 3, 2);
        }
        rd_a(o1, 2, S0);
        rd_a(o1, 3, S1);
    };
    static_assert(LH == 3, "three loads before and three after the barrier of a k-step");
    using R0 = std::integral_constant<int, 0>;
    using R2 = std::integral_constant<int, 2>;
    constexpr int SB = TL::STAGE_BYTES;

#pragma unroll
    for (int d = 0; d < L; ++d) dma_one(0, 0, d);
#pragma unroll
    for (int d = 0; d < L; ++d) dma_one(SB, 1, d);
#pragma unroll
    for (int d = 0; d < LH; ++d) dma_one(2 * SB, 2, d);
    wait_vmcnt<L + LH>();                                        // stage 0 has landed
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int r = 0; r < 4; ++r) rd_a(0, r, r);
#pragma unroll
    for (int j = 0; j < FN; ++j) rd_b(0, j);
    auto run = [&](auto csc) __attribute__((always_inline)) {
        int kt = 0, o0 = 0, o1 = SB, o2 = 2 * SB;                 // slots of stages kt, kt+1, kt+2 (scalars)
        for (; kt + 1 < sh.nk; kt += 2) {
            stage(kt, o0, o1, o2, R0{}, csc);
            stage(kt + 1, o1, o2, o0, R2{}, csc);
            const int t0 = o0; o0 = o2; o2 = o1; o1 = t0;         // two stages on: (o2, o0, o1)
        }
        if (kt < sh.nk) stage(kt, o0, o1, o2, R0{}, csc);
    };
    const bool cs_on = COLSUM && tm == 0 && __builtin_amdgcn_readfirstlane(wm) == 0;    // uniform over the wavefront
    if constexpr (COLSUM) {
        if (cs_on) run(std::true_type{});                         // both copies have one barrier per k-step
        else run(std::false_type{});
    } else {
        run(std::false_type{});
    }
    mfma16_drain();
    if (cs_on && lane < 16) {                                     // lanes 0..15 hold row 0 of each block: columns 0..15
#pragma unroll
        for (int j = 0; j < (COLSUM ? FN : 1); ++j) {
            const int col = n0 + (wn * FN + j) * 16 + lane;
            if (col < p.N) p.colsum[col] = (bf16_t)cs[j][0];
        }
    }
    wait_vmcnt<0>();
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    epilogue16<TL>(p, acc, smem, wave, lane, m0, n0, sh.partial);
}



bool gemm_bf16_supported(const GemmArgs& a) {
    if (a.dtype != BF16) return false;
    if (a.M % 8 || a.N % 8 || a.K % 8) return false;
    // 32-bit buffer offsets: operands below 2 GiB
    if (a.M * a.K * 2 >= 0x7FFFFFFFll || a.N * a.K * 2 >= 0x7FFFFFFFll) return false;
    int64_t tiles = ((a.M + 127) / 128) * ((a.N + 127) / 128);
    return tiles < (1 << 24) && a.K < (1 << 24);
}

// Band height of the tile order.  An XCD's L2 (4 MiB) holds no operand panel for long: what it saves is the reuse
// among the tiles in flight on the XCD at one time, which walk K together: `inflight` consecutive tiles of the list =
// h rows x inflight / h columns of the tile grid, needing h A slices and inflight / h B slices per k-step.  The band
// height minimises h * bm + (inflight / h) * bn.  The option gemm_band = h forces a height.
static int choose_band(int R, int bm, int bn, int lds_bytes) {
    if (const int v = options().gemm_band; v > 0) return v;
    // 32 compute units per XCD; the kernels with two workgroups per unit were also measured fastest with the band of
    // 32 tiles in flight (4 rows, 0.6 % of the step ahead of 8), so the count is not doubled for them
    (void)lds_bytes;
    const int inflight = 32;
    int best = 1;
    double best_cost = 1e300;
    for (int h = 1; h <= inflight; h *= 2) {
        const int hh = h < R ? h : R;
        const double cost = (double)hh * bm + (double)inflight / hh * bn;
        if (cost < best_cost) { best_cost = cost; best = hh; }
        if (h >= R) break;
    }
    return best;
}

template <typename TL, bool AK, bool BK_>
static hipError_t launch(GemmParams p, const GemmArgs& a, int shares) {
    static bool attr_set = false;   // raising the dynamic LDS limit is a per-function, one-off call
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_bf16_kernel<TL, AK, BK_>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, TL::LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    p.tiles_m = (int)((a.M + TL::BM - 1) / TL::BM);
    p.tiles_n = (int)((a.N + TL::BN - 1) / TL::BN);
    p.band = choose_band(p.tiles_m, TL::BM, TL::BN, TL::LDS_BYTES);
    hipLaunchKernelGGL((gemm_bf16_kernel<TL, AK, BK_>), dim3(p.tiles_m * p.tiles_n * shares), dim3(256),
                       TL::LDS_BYTES, a.stream, p);
    return hipGetLastError();
}

template <typename TL>
static hipError_t launch_layout(const GemmParams& p, const GemmArgs& a, int shares) {
    const bool a_kmaj = !a.trans_a, b_kmaj = a.trans_b;
    if (a_kmaj && b_kmaj) return launch<TL, true, true>(p, a, shares);
    if (a_kmaj && !b_kmaj) return launch<TL, true, false>(p, a, shares);
    if (!a_kmaj && b_kmaj) return launch<TL, false, true>(p, a, shares);
    return launch<TL, false, false>(p, a, shares);
}

template <typename TL, bool AK, bool BK_, bool CS = false>
static hipError_t launch_x16s(GemmParams p, const GemmArgs& a, int shares) {
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_bf16_x16s_kernel<TL, AK, BK_, CS>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, TL::LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    p.tiles_m = (int)((a.M + TL::BM - 1) / TL::BM);
    p.tiles_n = (int)((a.N + TL::BN - 1) / TL::BN);
    p.band = choose_band(p.tiles_m, TL::BM, TL::BN, TL::LDS_BYTES);
    hipLaunchKernelGGL((gemm_bf16_x16s_kernel<TL, AK, BK_, CS>), dim3(p.tiles_m * p.tiles_n * shares), dim3(256),
                       TL::LDS_BYTES, a.stream, p);
    return hipGetLastError();
}
template <typename TL>
static hipError_t launch_x16s_layout(const GemmParams& p, const GemmArgs& a, int shares) {
    const bool a_kmaj = !a.trans_a, b_kmaj = a.trans_b;
    if (a_kmaj && b_kmaj) return launch_x16s<TL, true, true>(p, a, shares);
    if (a_kmaj && !b_kmaj) return launch_x16s<TL, true, false>(p, a, shares);
    if (!a_kmaj && b_kmaj) return launch_x16s<TL, false, true>(p, a, shares);
    if (p.colsum) return launch_x16s<TL, false, false, true>(p, a, shares);
    return launch_x16s<TL, false, false>(p, a, shares);
}

template <typename TL, bool AK, bool BK_>
static hipError_t launch_w8(GemmParams p, const GemmArgs& a, int shares) {
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_bf16_x16w8_kernel<TL, AK, BK_>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, TL::LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    p.tiles_m = (int)((a.M + TL::BM - 1) / TL::BM);
    p.tiles_n = (int)((a.N + TL::BN - 1) / TL::BN);
    p.band = choose_band(p.tiles_m, TL::BM, TL::BN, TL::LDS_BYTES);
    hipLaunchKernelGGL((gemm_bf16_x16w8_kernel<TL, AK, BK_>), dim3(p.tiles_m * p.tiles_n * shares), dim3(512),
                       TL::LDS_BYTES, a.stream, p);
    return hipGetLastError();
}
template <typename TL>
static hipError_t launch_w8_layout(const GemmParams& p, const GemmArgs& a, int shares) {
    const bool a_kmaj = !a.trans_a, b_kmaj = a.trans_b;
    if (a_kmaj && b_kmaj) return launch_w8<TL, true, true>(p, a, shares);
    if (a_kmaj && !b_kmaj) return launch_w8<TL, true, false>(p, a, shares);
    if (!a_kmaj && b_kmaj) return launch_w8<TL, false, true>(p, a, shares);
    return launch_w8<TL, false, false>(p, a, shares);
}

template <typename ST, bool AK, bool BK_>
static hipError_t launch_spec(GemmParams p, const GemmArgs& a, int shares) {
    constexpr int LDS = ST::template lds_bytes<AK>();
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_bf16_spec_kernel<ST, AK, BK_>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    p.tiles_m = (int)((a.M + ST::BM - 1) / ST::BM);
    p.tiles_n = (int)((a.N + ST::BN - 1) / ST::BN);
    p.band = choose_band(p.tiles_m, ST::BM, ST::BN, LDS);
    hipLaunchKernelGGL((gemm_bf16_spec_kernel<ST, AK, BK_>), dim3(p.tiles_m * p.tiles_n * shares), dim3(512), LDS, a.stream, p);
    return hipGetLastError();
}
template <typename ST, bool BK_>
static hipError_t launch_spec16(GemmParams p, const GemmArgs& a, int shares) {
    constexpr int LDS = ST::template lds_bytes<true>();
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_bf16_spec16_kernel<ST, BK_>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    p.tiles_m = (int)((a.M + ST::BM - 1) / ST::BM);
    p.tiles_n = (int)((a.N + ST::BN - 1) / ST::BN);
    p.band = choose_band(p.tiles_m, ST::BM, ST::BN, LDS);
    hipLaunchKernelGGL((gemm_bf16_spec16_kernel<ST, BK_>), dim3(p.tiles_m * p.tiles_n * shares), dim3(512), LDS, a.stream, p);
    return hipGetLastError();
}
template <typename ST>
static hipError_t launch_spec_layout(const GemmParams& p, const GemmArgs& a, int shares) {
    const bool a_kmaj = !a.trans_a, b_kmaj = a.trans_b;
    if (a_kmaj && b_kmaj) return launch_spec<ST, true, true>(p, a, shares);
    if (a_kmaj && !b_kmaj) return launch_spec<ST, true, false>(p, a, shares);
    if (!a_kmaj && b_kmaj) return launch_spec<ST, false, true>(p, a, shares);
    return launch_spec<ST, false, false>(p, a, shares);
}

// Tile variants.  The host launches the one with the least estimated time
//   (tiles per compute unit, rounded up) x (k-stages) x (time per stage) + (per-tile fixed cost),
// with per-stage times measured on 8192^3 GEMMs.  The fixed cost (pipeline fill, and an epilogue that
// is bandwidth-bound because a round's workgroups all reach it together) is paid per round by the
// variants that fit one workgroup per compute unit and once by those that fit two (192 x 192 and
// 128 x 128), whose co-resident workgroups overlap each other's fill and epilogue.  So long-K GEMMs
// with few tiles prefer the big tiles, short-K weight gradients the co-resident ones, and a GEMM
// whose 256 x 256 tile count fills the last round badly a shape that divides better.
static int compute_units() {
    static int cus = 0;
    if (cus == 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        cus = (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess)
                  ? prop.multiProcessorCount : 256;
    }
    return cus;
}

constexpr int NVARIANTS = 8;
constexpr int MAX_SHARES = 16;
struct Plan { int variant, shares, nk_share; };

// Splitting K.  A GEMM with few output tiles and a long K (the data gradient of a narrow projection: N = 1536,
// K = 12288 ... 49152) leaves compute units idle or gives each a very long serial K walk.  Its K range is then
// cut into `shares` equal runs of k-steps, one workgroup per (tile, share); every workgroup writes its float
// partial sums to the workspace and a second kernel adds the shares in share order and applies the epilogue,
// so the result does not depend on scheduling.  The estimate charges that second pass with its memory traffic.
static Plan make_plan(int64_t M, int64_t N, int64_t K, bool a_kmaj, bool b_kmaj) {
    // variant 5: 256 x 192 on 8 wavefronts and the 16x16x32 instruction; 6: fetch and math wavefronts on 16x16x32;
    // 7: 192 x 192, two workgroups per compute unit, on 16x16x32
    static const int bm[NVARIANTS] = {256, 256, 128, 192, 256, 256, 256, 192};
    static const int bn[NVARIANTS] = {256, 192, 128, 192, 192, 192, 192, 192};
    static const int wgs_per_cu[NVARIANTS] = {1, 1, 2, 2, 1, 1, 1, 2};
    static const double us_per_stage[NVARIANTS] = {0.92, 0.758, 0.348, 0.5576, 0.658, 0.70, 0.602, 0.509};
    static const double fixed_us[NVARIANTS] = {12.0, 12.0, 12.0, 12.0, 18.0, 12.5, 18.0, 12.0};
    // tuning / test overrides (Options): one variant for every GEMM, a K split, or plans of single shapes
    const Options& opt = options();
    int forced_v = (opt.gemm_tile >= 0 && opt.gemm_tile < NVARIANTS) ? opt.gemm_tile : -1;
    int forced_s = opt.gemm_shares;
    // gemm_force = "MxNxK@ab=v[:shares];..." (a, b = 1 if A, B is K-major) overrides the plan of single shapes (tuning inside a whole step)
    int forced_shape_v = -1;
    if (opt.gemm_force[0]) {
        const char* q = opt.gemm_force;
        while (*q) {
            long long m = 0, n = 0, k = 0; int ak = 0, bk = 0, v = -1, sh = 0, used = 0;
            if (sscanf(q, "%lldx%lldx%lld@%1d%1d=%d%n", &m, &n, &k, &ak, &bk, &v, &used) >= 6) {   // @ab: A, B K-major
                const char* r = q + used;
                if (*r == ':') sh = atoi(r + 1);
                if (m == M && n == N && k == K && (ak != 0) == a_kmaj && (bk != 0) == b_kmaj && v >= 0 && v < NVARIANTS) {
                    forced_shape_v = v;
                    if (sh > 0) forced_s = sh;
                }
            }
            while (*q && *q != ';') ++q;
            if (*q == ';') ++q;
        }
    }
    if (forced_shape_v >= 0) forced_v = forced_shape_v;
    // Shapes whose plan was measured inside a whole layer step (two chains) against the estimate's choice and came out
    // ahead by more than 1 % of the step: the short-K and square GEMMs of the 1024- and 4096-wide encoder shards,
    // where the estimate below (calibrated on long-K GEMMs under the power cap) overrates the 256-wide tiles.
    static const struct { int M, N, K; bool a_kmaj, b_kmaj; int variant; } measured[] = {
        {8192, 2048, 1024, true, false, 7}, {8192, 2048, 1024, true, true, 7},      // roberta-large, TP 2: up / down-dgrad
        {4096, 4096, 4096, true, false, 7}, {4096, 4096, 1024, true, false, 7},     // 10B encoder, TP 4: up / out
    };
    if (forced_v < 0 && forced_s <= 0)
        for (const auto& e : measured)
            if (e.M == M && e.N == N && e.K == K && e.a_kmaj == a_kmaj && e.b_kmaj == b_kmaj) { forced_v = e.variant; forced_s = 1; }
    const int cus = compute_units();
    const int nk = (int)((K + DK - 1) / DK);
    Plan best{0, 1, nk};
    double best_c = -1;
    for (int v = 0; v < NVARIANTS; ++v) {
        if (forced_v >= 0 && v != forced_v) continue;
        // the variant with fetch-only wavefronts is built for a K-major A (its MN-major A path spills)
        if (forced_v < 0 && v == 4 && !a_kmaj) continue;
        if (v == 6 && !a_kmaj) continue;              // written for a K-major A only
        // the two-per-CU 16x16x32 tile is the weight-gradient kernel (MN-major A); with a K-major A it pays when K is
        // short (co-resident workgroups hide each other's start and end: the out-projection, K = 1536, -30 us per
        // forward pass against the 8-wavefront variant) or when many rounds of tiles amortise its cold starts; on the
        // long-K forward and data-gradient GEMMs it is 2-5 % slower per step (all measured inside the layer step by
        // forcing single shapes with TPL_GEMM_FORCE, not in isolated loops); the same holds for its 32x32x16 sibling,
        // variant 3 (config 4's out-projection data gradient: -1.2 % of the step without it)
        if (forced_v < 0 && (v == 7 || v == 3) && a_kmaj && nk > 64 &&
            ((M + bm[v] - 1) / bm[v]) * ((N + bn[v] - 1) / bn[v]) < 4 * compute_units()) continue;
        // with an MN-major B its 20 fragment reads per k-step hold up the matrix instructions: no gain there
        if (forced_v < 0 && v == 6 && !b_kmaj) continue;
        // the 8-wavefront variant was measured against the others on K-major A only (forward, data gradients)
        if (forced_v < 0 && v == 5 && !a_kmaj) continue;
        const int64_t tiles = ((M + bm[v] - 1) / bm[v]) * ((N + bn[v] - 1) / bn[v]);
        for (int want = 1; want <= MAX_SHARES; ++want) {
            if (forced_s > 0 && want != (forced_s < MAX_SHARES ? forced_s : MAX_SHARES)) continue;
            if (forced_s <= 0 && want > 1 && (tiles * (want - 1) >= cus || nk / want < 48 || v == 5)) break;
            int per = (nk + want - 1) / want;
            if (v == 4 || v == 6) per = (per + 1) & ~1;          // its wide A slots hold two k-steps: shares start on even steps
            const int shares = (nk + per - 1) / per;
            if (forced_s <= 0 && shares != want) continue;   // the same plan as a smaller `want`
            const double per_cu = (double)((tiles * shares + cus - 1) / cus);
            double c = per_cu * per * us_per_stage[v] + fixed_us[v] * (wgs_per_cu[v] == 1 ? per_cu : 1.0);
            if (shares > 1) c += 6.0 + (double)M * N * (8.0 * shares + 2.0) / 3.0e6;   // second pass at ~3 TB/s
            // a split GEMM that takes (nearly) every compute unit leaves none to the kernels of the other chain:
            // measured inside the whole step, the out-projection data gradient is fastest with 3 shares (192
            // workgroups), 0.8 % of the step ahead of 4 (256 workgroups)
            if (shares > 1 && tiles * shares * 4 > (int64_t)cus * 3) c *= 1.10;
            if (best_c < 0 || c < best_c) { best = Plan{v, shares, per}; best_c = c; }
        }
    }
    return best;
}

// Plans are computed once per (shape, layout) and kept: a launch looks its plan up (a short scan under a mutex), it
// does not run the planner.  Entries carry the generation of the options they were planned under.
static Plan plan_for(int64_t M, int64_t N, int64_t K, bool a_kmaj, bool b_kmaj) {
    struct Entry { int64_t M, N, K; int layout; unsigned gen; Plan plan; };
    constexpr int CAP = 128;
    static Entry cache[CAP];
    static int used = 0, next = 0;
    static std::mutex mu;
    const int layout = (a_kmaj ? 1 : 0) | (b_kmaj ? 2 : 0);
    const unsigned gen = options().generation;
    std::lock_guard<std::mutex> lock(mu);
    for (int i = 0; i < used; ++i) {
        const Entry& e = cache[i];
        if (e.M == M && e.N == N && e.K == K && e.layout == layout && e.gen == gen) return e.plan;
    }
    const Plan pl = make_plan(M, N, K, a_kmaj, b_kmaj);
    const int slot = used < CAP ? used++ : (next++ % CAP);
    cache[slot] = Entry{M, N, K, layout, gen, pl};
    return pl;
}

size_t gemm_bf16_workspace_bytes(int64_t M, int64_t N, int64_t K) {
    size_t need = 0;
    for (int layout = 0; layout < 4; ++layout) {
        const Plan pl = plan_for(M, N, K, (layout & 1) != 0, (layout & 2) != 0);
        if (pl.shares > 1) need = std::max(need, (size_t)pl.shares * (size_t)M * (size_t)N * sizeof(float));
    }
    return need;
}

hipError_t gemm_bf16(const GemmArgs& a, bool* colsum_done) {
    if (colsum_done) *colsum_done = false;
    GemmParams p;
    p.A = (const bf16_t*)a.A; p.B = (const bf16_t*)a.B; p.C = (bf16_t*)a.C;
    p.bias = (const bf16_t*)a.bias; p.resid = (const bf16_t*)a.resid; p.aux = (bf16_t*)a.aux;
    p.M = (int)a.M; p.N = (int)a.N; p.K = (int)a.K;
    p.nt_store = a.c_streaming ? 1 : 0;
    p.lda = a.trans_a ? (int)a.M : (int)a.K;
    p.ldb = a.trans_b ? (int)a.K : (int)a.N;
    p.epi = a.epi;
    p.tiles_m = p.tiles_n = 0;
    p.band = 8;
    const Plan pl = plan_for(a.M, a.N, a.K, !a.trans_a, a.trans_b != 0);
    p.nk_total = (int)((a.K + DK - 1) / DK);
    p.nk = pl.nk_share;
    p.partial = nullptr;
    // the column sums of B ride along only on request (option fuse_colsum), in the weight-gradient kernel (both operands
    // MN-major) with K unsplit
    p.colsum = (a.colsum_b && options().fuse_colsum && pl.variant == 7 && pl.shares == 1 && a.trans_a && !a.trans_b)
                   ? (bf16_t*)a.colsum_b : nullptr;
    if (colsum_done) *colsum_done = p.colsum != nullptr;
    if (pl.shares > 1) {
        if (a.ws == nullptr || a.ws_bytes < (size_t)pl.shares * (size_t)a.M * (size_t)a.N * sizeof(float))
            return hipErrorInvalidValue;
        p.partial = (float*)a.ws;
    }
    hipError_t e;
    switch (pl.variant) {
        case 4: e = launch_spec_layout<SpecTile<4, 3>>(p, a, pl.shares); break;   // 256 x 192, fetch and math wavefronts
        case 1: e = launch_layout<Tile<4, 3, 4>>(p, a, pl.shares); break;    // 256 x 192
        case 2: e = launch_layout<Tile<2, 2, 4>>(p, a, pl.shares); break;    // 128 x 128, two workgroups per CU
        case 3: e = launch_layout<Tile<3, 3, 3>>(p, a, pl.shares); break;    // 192 x 192, two workgroups per CU
        case 5: e = launch_w8_layout<Tile8<2, 3, 5>>(p, a, pl.shares); break;      // 256 x 192, 8 wavefronts, 16x16x32
        case 7: e = launch_x16s_layout<Tile<3, 3, 3>>(p, a, pl.shares); break;     // 192 x 192, 2 workgroups/CU, 16x16x32
        case 6:                                                                    // 256 x 192, fetch + math, 16x16x32
            e = a.trans_b ? launch_spec16<SpecTile<4, 3>, true>(p, a, pl.shares)
                          : launch_spec16<SpecTile<4, 3>, false>(p, a, pl.shares);
            break;
        default: e = launch_layout<Tile<4, 4, 4>>(p, a, pl.shares); break;   // 256 x 256
    }
    if (e != hipSuccess || pl.shares == 1) return e;
    const int64_t chunks = a.M * a.N / 8;
    hipLaunchKernelGGL(gemm_sum_shares_kernel, dim3((unsigned)((chunks + 255) / 256)), dim3(256), 0, a.stream, p, pl.shares);
    return hipGetLastError();
}

}  // namespace tpl
