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
// Backward is a row-dot kernel (D = rowsum(dO * O)) and one launch whose workgroups are dK/dV workgroups (per key
// block) or dQ workgroups (per query block), each accumulating in registers in a fixed order: no atomics, results
// are run-to-run identical.
//
// Streaming.  K/V (or Q/dO) tiles of 64 rows go from global memory straight into a two-stage LDS ring (buffer
// loads with the LDS flag), the tile of step t+1 requested at the start of step t; fragments are read from LDS a
// phase ahead of the MFMAs that use them.  A tile step is bound by vector arithmetic (exp2, scaling, conversions),
// not by the matrix cores.
//
// Strips and chunks.  The tile steps of one (128-row block, head) form a strip; under the causal mask
// strips are triangular (2 to S/64 steps) and the longest one is the critical path of the launch.  When
// the caller supplies a workspace, strips longer than a chunk length are cut into chunks of equal length,
// each chunk is a workgroup of its own that writes float partials (forward: running max, sum and
// unnormalised O; backward: partial dQ or dK, dV), and a second kernel combines the chunks of a strip in
// chunk order.  Strips of one chunk write their result directly, as without a workspace.
#include <hip/hip_runtime.h>

#include <cstdlib>
#include <type_traits>

#include "device_math.h"
#include "kernels.h"
#include "lds_dma.h"

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
constexpr float RESCALE_LAG = 8.0f;  // forward: how far (log2) the row maximum may run ahead of the reference point

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

// ---- global -> LDS without passing through registers ---------------------------------------------
// A tile is TILE rows x DH bf16 = TILE*DH/8 chunks of 16 bytes; a buffer load with the LDS flag writes the 64
// chunks of a wavefront to 64 consecutive LDS positions.  Position p = t + NT*i (row p / NC, slot p % NC) must
// hold chunk (slot ^ swz(row)) of its row, so the swizzle is applied to the global offset each lane requests.
// Offsets are relative to row 0 of this (batch, head); the descriptor ends after the head's slice of row S-1,
// which makes rows >= S read as zero.
template <int DH, int NT>
__device__ __forceinline__ void dma_offsets(unsigned (&off)[(NCHUNKS<DH, NT>)], int64_t ld, int t) {
    constexpr int NC = DH / 8;
#pragma unroll
    for (int i = 0; i < NCHUNKS<DH, NT>; ++i) {
        const int p = t + NT * i, row = p / NC, c = (p % NC) ^ swz<DH>(row);
        off[i] = (unsigned)row * (unsigned)(ld * 2) + (unsigned)c * 16u;
    }
}
template <int DH>
__device__ __forceinline__ i32x4 head_rsrc(const bf16_t* base, int64_t ld, int S) {
    return make_rsrc(base, (unsigned)(((int64_t)(S - 1) * ld + DH) * 2));
}
// rows [row0, row0 + TILE) -> LDS tile at byte address lds_tile; wave = wavefront index (uniform)
template <int DH, int NT>
__device__ __forceinline__ void tile_dma(i32x4 rsrc, unsigned lds_tile, const unsigned (&off)[(NCHUNKS<DH, NT>)],
                                         unsigned row0_bytes, int wave) {
#pragma unroll
    for (int i = 0; i < NCHUNKS<DH, NT>; ++i)
        buffer_load_lds_b128(rsrc, lds_tile + (unsigned)(i * NT + wave * 64) * 16u, off[i] + row0_bytes);
}
// A use of v that the compiler must order after the load that produces v: placed before a streaming loop, it
// makes the compiler wait for prologue loads there, instead of inside the loop at their first use, where the
// wait (a count of all loads in flight) would also drain the tile requested for the next step.
template <typename T> __device__ __forceinline__ void settle(const T& v) { asm volatile("" ::"v"(v)); }
// The loads above are invisible to the compiler's own wait counting: wait for all of them before the barrier
// that hands the tile to the readers.
__device__ __forceinline__ void dma_wait() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

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
// Byte offsets of those two kinds of read inside a tile, for kernels that keep them in registers across the streaming
// loop (computed per read they are ~100 vector instructions per tile step, more than the softmax arithmetic itself;
// matrix and vector instructions do not overlap on a SIMD, so every one of them is matrix time lost).  Both are
// unchanged by adding a multiple of 16 to the row (the swizzle uses row bits 0..3 only): a second block of 16 rows is
// the same offset plus 16 rows.
template <int DH> __device__ __forceinline__ unsigned frag_k_off(int row_base, int ks, int lane) {
    int row = row_base + (lane & 31);
    int c = 2 * ks + (lane >> 5);
    return (unsigned)(row * (DH * 2) + ((c ^ swz<DH>(row)) << 4));
}
template <int DH> __device__ __forceinline__ unsigned frag_t_off(int d_base, int r_base, int h, int lane) {
    int l16 = lane & 15;
    int d = d_base + (lane & 16) + 4 * (l16 & 3);
    int row = r_base + 8 * h + 4 * (lane >> 5) + (l16 >> 2);
    return (unsigned)(row * (DH * 2) + ((((d >> 3) ^ swz<DH>(row))) << 4) + (d & 7) * 2);
}
typedef __attribute__((address_space(3))) const bf16x8* lds_bf16x8_cptr;
// The reads themselves from a 32-bit LDS address held in a register plus a compile-time byte offset (an immediate).
template <int IMM> __device__ __forceinline__ bf16x8 lds_frag_k(unsigned addr) {
    return *reinterpret_cast<lds_bf16x8_cptr>((uintptr_t)(addr + IMM));
}
template <int IMM> __device__ __forceinline__ bf16x8 lds_frag_t(unsigned addr0, unsigned addr1) {
    s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(uintptr_t)(addr0 + IMM));
    s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(uintptr_t)(addr1 + IMM));
    bf16x4 b0 = __builtin_bit_cast(bf16x4, v0), b1 = __builtin_bit_cast(bf16x4, v1);
    bf16x8 out;
    out[0] = b0[0]; out[1] = b0[1]; out[2] = b0[2]; out[3] = b0[3];
    out[4] = b1[0]; out[5] = b1[1]; out[6] = b1[2]; out[7] = b1[3];
    return out;
}
template <typename T> __device__ __forceinline__ void keep_in_register(T& v) { asm volatile("" : "+v"(v)); }
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
// max(v[l], v[l ^ 32]) in every lane by one lane-swap instruction (no trip through the LDS crossbar, whose latency would
// sit in the middle of the softmax chain): swapping the upper half of a with the lower half of b, for a = b = v, leaves
// (v.lo, v.lo) and (v.hi, v.hi).
__device__ __forceinline__ float cross_half_max(float v) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
// 2^x on the hardware transcendental unit (arguments here are <= ~0; results below 2^-126 flush to 0).
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
#define MFMA(a, b, c) __builtin_amdgcn_mfma_f32_32x32x16_bf16((a), (b), (c), 0, 0, 0)

// ---- strips and chunks (host and device agree through these) --------------------------------------
// Blocks are ranked heaviest first: query blocks from the last one down (forward, dQ), key blocks from the
// first one up (dK/dV).  Workgroup `slot` of a head is chunk c of the block of rank r, slots numbered
// rank-major, so that the heaviest chunks are dispatched first.
__host__ __device__ inline int strip_block(bool kv_side, int nblk, int rank) { return kv_side ? rank : nblk - 1 - rank; }
__host__ __device__ inline int strip_tiles(bool causal, bool kv_side, int S, int blk) {
    const int nt = (S + TILE - 1) / TILE;
    if (!causal) return nt;
    if (kv_side) return nt - (blk * BLK) / TILE;          // query tiles from the diagonal to the end
    const int end = (blk + 1) * BLK < S ? (blk + 1) * BLK : S;
    return (end + TILE - 1) / TILE;                       // key tiles from 0 to the diagonal
}
// Chunk length with the multiplier that replaces the division by it (the slot search runs in every workgroup):
// magic = floor(2^32 / ch) + 1 gives floor(n / ch) = (n * magic) >> 32 exactly for n * ch < 2^32 (here n, ch < 2^16).
struct ChunkLen { int ch; unsigned magic; };
inline ChunkLen make_chunk_len(int ch) {
    return ChunkLen{ch, ch > 1 && ch < (1 << 16) ? (unsigned)((1ull << 32) / (unsigned)ch) + 1u : 0u};
}
__host__ __device__ inline int strip_chunks(int tiles, ChunkLen ch) {
    if (tiles <= ch.ch) return 1;
    if (ch.ch == 1) return tiles;
    return (int)(((unsigned long long)(unsigned)(tiles + ch.ch - 1) * ch.magic) >> 32);
}
__host__ __device__ inline int strip_slots(bool causal, bool kv_side, int S, ChunkLen ch) {
    const int nblk = (S + BLK - 1) / BLK;
    int n = 0;
    for (int r = 0; r < nblk; ++r) n += strip_chunks(strip_tiles(causal, kv_side, S, strip_block(kv_side, nblk, r)), ch);
    return n;
}
struct Chunk {
    int blk;        // query block (forward, dQ) or key block (dK/dV)
    int nch;        // chunks of this block's strip
    int slot0;      // slot of the strip's chunk 0
    int t0, t1;     // tile steps [t0, t1) of this chunk
};
// Chunk of workgroup `slot`; with slot < 0: the strip of block `want_blk` (t0, t1 = whole strip).
__device__ inline Chunk find_chunk(bool causal, bool kv_side, int S, ChunkLen ch, int slot, int want_blk) {
    const int nblk = (S + BLK - 1) / BLK;
    const int nt = (S + TILE - 1) / TILE;
    Chunk k{0, 1, 0, 0, 0};
    int acc = 0;
    for (int r = 0; r < nblk; ++r) {
        const int blk = strip_block(kv_side, nblk, r);
        const int tiles = strip_tiles(causal, kv_side, S, blk);
        const int nch = strip_chunks(tiles, ch);
        const bool hit = slot >= 0 ? slot < acc + nch : blk == want_blk;
        if (hit) {
            const int first = kv_side ? nt - tiles : 0;
            k.blk = blk; k.nch = nch; k.slot0 = acc;
            if (slot >= 0) {
                const int c = slot - acc, len = (tiles + nch - 1) / nch;
                k.t0 = first + c * len;
                k.t1 = first + ((c + 1) * len < tiles ? (c + 1) * len : tiles);
            } else {
                k.t0 = first; k.t1 = first + tiles;
            }
            return k;
        }
        acc += nch;
    }
    return k;
}
__device__ __forceinline__ void store_f4(float* p, float a, float b, float c, float d) {
    *reinterpret_cast<float4*>(p) = make_float4(a, b, c, d);
}

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
__global__ __launch_bounds__(FTHREADS, DH == 64 ? 4 : 2) void attn_fwd_kernel(const bf16_t* __restrict__ qkv,
                                                            bf16_t* __restrict__ o,
                                                            float* __restrict__ lse, int S, int nl, int BH,
                                                            float* __restrict__ part, ChunkLen ch) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    constexpr int TB = tile_bytes<DH>();
    constexpr int NCH = NCHUNKS<DH, FTHREADS>;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6, half = lane >> 5;
    const int qs = wave & 3, kvh = wave >> 2;
    const int bh = blockIdx.x % BH, slot = blockIdx.x / BH;      // head fastest: heaviest chunks of all heads first
    const Chunk ck = find_chunk(CAUSAL, false, S, ch, slot, 0);
    const int qb = ck.blk;
    const int b = bh / nl, h = bh % nl;
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
    const int tile0 = ck.t0, ntiles = ck.t1;
    const unsigned lds0 = (unsigned)(uintptr_t)(lds_void_ptr)smem;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const i32x4 desc_k = head_rsrc<DH>(kbase, ld, S), desc_v = head_rsrc<DH>(vbase, ld, S);
    unsigned off[NCH];
    dma_offsets<DH, FTHREADS>(off, ld, t);
    auto fetch_tile = [&](int kt, unsigned stage) {       // K and V rows of tile kt -> LDS stage
        const unsigned r0 = (unsigned)kt * TILE * (unsigned)(ld * 2);
        tile_dma<DH, FTHREADS>(desc_k, stage, off, r0, wave_u);
        tile_dma<DH, FTHREADS>(desc_v, stage + TB, off, r0, wave_u);
    };
    // LDS addresses of this lane's fragment reads in stage 0 (K tile at lds0, V tile one tile further), kept in registers
    unsigned ka[DH / 16], va[DH / 32][2];
#pragma unroll
    for (int ks = 0; ks < DH / 16; ++ks) { ka[ks] = lds0 + frag_k_off<DH>(kvh * 32, ks, lane); keep_in_register(ka[ks]); }
#pragma unroll
    for (int dt = 0; dt < DH / 32; ++dt)
#pragma unroll
        for (int h = 0; h < 2; ++h) { va[dt][h] = lds0 + TB + frag_t_off<DH>(dt * 32, kvh * 32, h, lane); keep_in_register(va[dt][h]); }
    fetch_tile(tile0, lds0);
#pragma unroll
    for (int ks = 0; ks < DH / 16; ++ks) settle(qf[ks]);
    dma_wait();
    __syncthreads();
    // one tile step on ring stage STG (a compile-time constant, so that the stage is an immediate of every fragment read)
    auto step = [&](int kt, auto stg) __attribute__((always_inline)) {
        constexpr int STG = decltype(stg)::value;
        constexpr int SOFF = STG * 2 * TB;
        // the other stage was last read before the barrier that ended the previous step
        if (kt + 1 < ntiles) fetch_tile(kt + 1, lds0 + (1 - STG) * 2 * TB);
        const int kv0 = kt * TILE + kvh * 32;
        if (kv0 < kv_end && !(CAUSAL && kv0 > q0 + 31)) {                 // wavefront-uniform
            // All K fragments are requested before the first MFMA and all V fragments before the softmax arithmetic,
            // so that LDS latency is paid once per phase instead of once per MFMA (the fences keep that order).
            f32x16 s = zero16();
            bf16x8 fr[DH / 16];
#pragma unroll
            for (int ks = 0; ks < DH / 16; ++ks) fr[ks] = lds_frag_k<SOFF>(ka[ks]);
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_s_setprio(1);
#pragma unroll
            for (int ks = 0; ks < DH / 16; ++ks) s = MFMA(fr[ks], qf[ks], s);
            __builtin_amdgcn_s_setprio(0);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int dt = 0; dt < DH / 32; ++dt) {
                fr[2 * dt] = lds_frag_t<SOFF>(va[dt][0], va[dt][1]);
                fr[2 * dt + 1] = lds_frag_t<SOFF + 16 * DH * 2>(va[dt][0], va[dt][1]);
            }
            __builtin_amdgcn_sched_barrier(0);
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
            mb = cross_half_max(mb) * c2;                     // c2 > 0: scaling commutes with max
            // The reference point m of the running sums moves only when the maximum has grown by more than
            // RESCALE_LAG (log2 units): probabilities then reach 2^RESCALE_LAG at most, which float sums and
            // bf16 operands hold without loss, and the accumulators are rescaled in a few early tiles only
            // instead of in most of them.  Any reference point gives the same O and LSE up to rounding.
            const float mn = (mb - m > RESCALE_LAG) ? mb : m;   // false for NaN (-inf - -inf): m stays
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
            __builtin_amdgcn_s_setprio(1);
#pragma unroll
            for (int dt = 0; dt < DH / 32; ++dt) {
                oacc[dt] = MFMA(fr[2 * dt], pb0, oacc[dt]);
                oacc[dt] = MFMA(fr[2 * dt + 1], pb1, oacc[dt]);
            }
            __builtin_amdgcn_s_setprio(0);
        }
        dma_wait();
        __syncthreads();
    };
    {
        int kt = tile0;
        for (; kt + 1 < ntiles; kt += 2) {
            step(kt, std::integral_constant<int, 0>{});
            step(kt + 1, std::integral_constant<int, 1>{});
        }
        if (kt < ntiles) step(kt, std::integral_constant<int, 0>{});
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
        if (ck.nch > 1) {
            // one chunk of a longer strip: (max, sum, unnormalised O) of this chunk's keys, float, [query][dh]
            float* pp = part + ((int64_t)slot * BH + bh) * (BLK * (DH + 2));
            const int ql = qs * 32 + (lane & 31);
#pragma unroll
            for (int dt = 0; dt < DH / 32; ++dt)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    float r[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        r[j] = oacc[dt][4 * i + j] * f0 + mg[(2 + dt * 16 + 4 * i + j) * 64] * f1;
                    store_f4(pp + ql * DH + dt * 32 + 8 * i + 4 * half, r[0], r[1], r[2], r[3]);
                }
            if (half == 0) { pp[BLK * DH + ql] = mn; pp[BLK * DH + BLK + ql] = ltot; }
        } else if (q < S) {
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

// Forward, second kernel: merges the chunks of every strip that was cut (max, rescale, add, in chunk order),
// normalises and writes O and LSE.  Workgroup = (256 / (DH/4) query rows of a block, batch*head); DH/4 threads per row.
template <int DH, bool CAUSAL>
__global__ __launch_bounds__(256) void attn_fwd_combine_kernel(const float* __restrict__ part, bf16_t* __restrict__ o,
                                                               float* __restrict__ lse, int S, int nl, int BH, ChunkLen ch,
                                                               int blk0) {
    constexpr int TPR = DH / 4, PSZ = BLK * (DH + 2), RPW = 256 / TPR, WPB = BLK / RPW;
    const Chunk ck = find_chunk(CAUSAL, false, S, ch, -1, blk0 + (int)blockIdx.x / WPB);
    if (ck.nch == 1) return;
    const int bh = blockIdx.y, b = bh / nl, h = bh % nl;
    const int tc = threadIdx.x % TPR;
    {
        const int ql = ((int)blockIdx.x % WPB) * RPW + threadIdx.x / TPR;
        const int q = ck.blk * BLK + ql;
        if (q >= S) return;
        const float* p0 = part + ((int64_t)ck.slot0 * BH + bh) * PSZ;
        float mtot = -INFINITY;
        for (int c = 0; c < ck.nch; ++c) mtot = fmaxf(mtot, p0[(int64_t)c * BH * PSZ + BLK * DH + ql]);
        const float mu = mtot == -INFINITY ? 0.0f : mtot;
        float ltot = 0.0f, a0 = 0.0f, a1 = 0.0f, a2 = 0.0f, a3 = 0.0f;
        for (int c = 0; c < ck.nch; ++c) {
            const float* pc = p0 + (int64_t)c * BH * PSZ;
            const float f = fast_exp2(pc[BLK * DH + ql] - mu);
            ltot = fmaf(pc[BLK * DH + BLK + ql], f, ltot);
            const float4 v = *reinterpret_cast<const float4*>(pc + ql * DH + 4 * tc);
            a0 = fmaf(v.x, f, a0); a1 = fmaf(v.y, f, a1); a2 = fmaf(v.z, f, a2); a3 = fmaf(v.w, f, a3);
        }
        const float inv = ltot > 0.0f ? 1.0f / ltot : 0.0f;
        store4(o + ((int64_t)b * S + q) * ((int64_t)nl * DH) + (int64_t)h * DH + 4 * tc, a0 * inv, a1 * inv, a2 * inv,
               a3 * inv);
        if (tc == 0) lse[((int64_t)b * nl + h) * S + q] = (mtot + log2f(ltot)) * LN2;
    }
}

// Backward, last kernel: dQ, dK, dV of every strip that was cut = sum of its chunks' partials in chunk order.
// blockIdx.z = 0: dQ (query-block strips), 1: dK, 2: dV (key-block strips; a slot holds [dK | dV]); workgroup =
// (256 / (DH/4) rows of a block, batch*head), DH/4 threads per row.
template <int DH, bool CAUSAL>
__global__ __launch_bounds__(256) void attn_bwd_combine_kernel(const float* __restrict__ part_q,
                                                               const float* __restrict__ part_kv,
                                                               bf16_t* __restrict__ dqkv, int S, int nl, int BH,
                                                               ChunkLen ch_q, ChunkLen ch_kv,
                                                               int blk0_q, int ncut_q, int blk0_kv, int ncut_kv) {
    constexpr int TPR = DH / 4, RPW = 256 / TPR, WPB = BLK / RPW;
    const int which = blockIdx.z;
    if ((int)blockIdx.x / WPB >= (which == 0 ? ncut_q : ncut_kv)) return;
    const Chunk ck = find_chunk(CAUSAL, which != 0, S, which == 0 ? ch_q : ch_kv, -1,
                                (which == 0 ? blk0_q : blk0_kv) + (int)blockIdx.x / WPB);
    if (ck.nch == 1) return;
    const int bh = blockIdx.y, b = bh / nl, h = bh % nl;
    const int psz = which == 0 ? BLK * DH : 2 * BLK * DH;
    const float* p0 = (which == 0 ? part_q : part_kv) + ((int64_t)ck.slot0 * BH + bh) * psz + (which == 2 ? BLK * DH : 0);
    const float f = which == 2 ? 1.0f : 1.0f / sqrtf((float)DH);
    const int64_t ld = 3LL * nl * DH;
    const int tc = threadIdx.x % TPR;
    {
        const int rl = ((int)blockIdx.x % WPB) * RPW + threadIdx.x / TPR;
        const int row = ck.blk * BLK + rl;
        if (row >= S) return;
        float a0 = 0.0f, a1 = 0.0f, a2 = 0.0f, a3 = 0.0f;
        for (int c = 0; c < ck.nch; ++c) {
            const float4 v = *reinterpret_cast<const float4*>(p0 + (int64_t)c * BH * psz + rl * DH + 4 * tc);
            a0 += v.x; a1 += v.y; a2 += v.z; a3 += v.w;
        }
        store4(dqkv + ((int64_t)b * S + row) * ld + (int64_t)which * nl * DH + (int64_t)h * DH + 4 * tc, a0 * f, a1 * f,
               a2 * f, a3 * f);
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
                                              int S, int nl, int bh, const Chunk& ck, float* __restrict__ pslot) {
    constexpr int TB = tile_bytes<DH>();
    constexpr int NCH = NCHUNKS<DH, FTHREADS>;
    constexpr int STAGE = 2 * TB + 2 * TILE * 4;          // Q tile, dO tile, LSE*log2e, D
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6, half = lane >> 5;
    const int kb = ck.blk;
    const int b = bh / nl, h = bh % nl;
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

    const int qt0 = ck.t0, ntiles = ck.t1;                // query tiles of this chunk (the strip starts at the diagonal)
    const unsigned lds0 = (unsigned)(uintptr_t)(lds_void_ptr)smem;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const i32x4 desc_q = head_rsrc<DH>(qbase, ld, S), desc_do = head_rsrc<DH>(dobase, ldo, S);
    unsigned off_q[NCH], off_do[NCH];
    dma_offsets<DH, FTHREADS>(off_q, ld, t);
    dma_offsets<DH, FTHREADS>(off_do, ldo, t);
    float rl = 0.0f, rd = 0.0f;
    // Q and dO rows of tile qt straight into LDS; LSE and D of its rows through registers (r2s stores them)
    auto g2r = [&](int qt, unsigned stage) {
        tile_dma<DH, FTHREADS>(desc_q, stage, off_q, (unsigned)qt * TILE * (unsigned)(ld * 2), wave_u);
        tile_dma<DH, FTHREADS>(desc_do, stage + TB, off_do, (unsigned)qt * TILE * (unsigned)(ldo * 2), wave_u);
        if (t < TILE) {
            int qi = qt * TILE + t;
            rl = qi < S ? lrow[qi] * LOG2E : 0.0f;
            rd = qi < S ? drow[qi] : 0.0f;
        }
    };
    auto r2s = [&](char* st) {
        if (t < TILE) {
            reinterpret_cast<float*>(st + 2 * TB)[t] = rl;
            reinterpret_cast<float*>(st + 2 * TB)[TILE + t] = rd;
        }
    };
    if (qt0 < ntiles) { g2r(qt0, lds0); r2s(smem); }
#pragma unroll
    for (int ks = 0; ks < DH / 16; ++ks) {
        settle(kf[ks]);
        if (DK_ROLE) settle(vf[ks]);
    }
    dma_wait();
    __syncthreads();
    for (int qt = qt0; qt < ntiles; ++qt) {
        const char* st = smem + ((qt - qt0) & 1) * STAGE;
        char* nxt = smem + ((qt - qt0 + 1) & 1) * STAGE;
        const char* qs = st;
        const char* dos = st + TB;
        const float* ls = reinterpret_cast<const float*>(st + 2 * TB);
        const float* ds_ = ls + TILE;
        const bool more = qt + 1 < ntiles;
        if (more) g2r(qt + 1, lds0 + ((qt - qt0 + 1) & 1) * STAGE);
#pragma unroll
        for (int sb = 0; sb < 2; ++sb) {
            const int qs0 = qt * TILE + sb * 32;
            if (qs0 >= S || (CAUSAL && qs0 + 31 < k0)) continue;          // wavefront-uniform
            // Fragments of all MFMA phases (Q for S, dO for dP in the dK role, then Q or dO transposed) through a
            // rolling window of W registers, as in the dQ kernel.
            f32x16 s = zero16(), dp = zero16();
            constexpr int NF = DH / 16, W = DH == 64 ? NF : NF / 2, NP = DK_ROLE ? 2 * NF : NF;
            bf16x8 fr[W];
            const char* src = DK_ROLE ? qs : dos;                          // dK += dS^T Q ; dV += P^T dO
            auto fetch = [&](int i) {
                if (i < NF) return frag_k<DH>(qs, sb * 32, i, lane);
                if (i < NP) return frag_k<DH>(dos, sb * 32, i - NF, lane);
                const int k = i - NP;
                return frag_t<DH>(src, (k >> 1) * 32, sb * 32 + (k & 1) * 16, lane);
            };
#pragma unroll
            for (int i = 0; i < W; ++i) fr[i] = fetch(i);
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_s_setprio(1);
#pragma unroll
            for (int i = 0; i < NP; ++i) {
                if (i < NF) s = MFMA(fr[i % W], kf[i], s);
                else dp = MFMA(fr[i % W], vf[DK_ROLE ? i - NF : 0], dp);
                fr[i % W] = fetch(i + W);
                __builtin_amdgcn_sched_barrier(0);
            }
            __builtin_amdgcn_s_setprio(0);
            const bool need_mask = qs0 + 31 >= S || k0 + 31 >= S || (CAUSAL && k0 + 31 > qs0);
            if (need_mask) {                          // wave-uniform: only tiles on the diagonal or at the end of S
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    int qi = qs0 + 8 * (v >> 2) + 4 * half + (v & 3);
                    bool ok = qi < S && kv < S && (!CAUSAL || kv <= qi);
                    s[v] = ok ? s[v] : -INFINITY;         // exp2(-inf) = 0
                }
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float4 l4 = *reinterpret_cast<const float4*>(ls + sb * 32 + 8 * i + 4 * half);
                float4 d4 = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
                if (DK_ROLE) d4 = *reinterpret_cast<const float4*>(ds_ + sb * 32 + 8 * i + 4 * half);
                const float lv[4] = {l4.x, l4.y, l4.z, l4.w}, dvv[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    int v = 4 * i + j;
                    const float p = fast_exp2(fmaf(s[v], c2, -lv[j]));
                    s[v] = DK_ROLE ? p * (dp[v] - dvv[j]) : p;             // dS, or P
                }
            }
            bf16x8 g0 = pack_regs(s, 0), g1 = pack_regs(s, 8);
            __builtin_amdgcn_s_setprio(1);
#pragma unroll
            for (int k = 0; k < NF; ++k) {
                acc[k >> 1] = MFMA(fr[k % W], (k & 1) ? g1 : g0, acc[k >> 1]);
                if (k + W < NF) {
                    fr[k % W] = fetch(NP + k + W);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            __builtin_amdgcn_s_setprio(0);
        }
        if (more) r2s(nxt);
        dma_wait();
        __syncthreads();
    }
    if (ck.nch > 1) {
        // one chunk of a longer strip: unscaled float partial, [dK | dV][key][dh]
        float* pp = pslot + (DK_ROLE ? 0 : BLK * DH) + ((wave & 3) * 32 + (lane & 31)) * DH;
#pragma unroll
        for (int dt = 0; dt < DH / 32; ++dt)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                store_f4(pp + dt * 32 + 8 * i + 4 * half, acc[dt][4 * i], acc[dt][4 * i + 1], acc[dt][4 * i + 2],
                         acc[dt][4 * i + 3]);
    } else if (kv < S) {
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

// dK/dV workgroup number wg (head fastest, then slot)
template <int DH, bool CAUSAL>
__device__ __forceinline__ void attn_dkv_wg(char* smem, const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ d_o,
                                            const float* __restrict__ lse, const float* __restrict__ dsum,
                                            bf16_t* __restrict__ dqkv, int S, int nl, int BH,
                                            float* __restrict__ part, ChunkLen ch, int wg) {
    const int bh = wg % BH, slot = wg / BH;
    const Chunk ck = find_chunk(CAUSAL, true, S, ch, slot, 0);
    float* pslot = part + ((int64_t)slot * BH + bh) * (2 * BLK * DH);
    // the role is uniform per wavefront; both bodies run the same loop and the same barriers
    if ((threadIdx.x >> 6) < 4) attn_dkv_body<DH, CAUSAL, false>(smem, qkv, d_o, lse, dsum, dqkv, S, nl, bh, ck, pslot);
    else attn_dkv_body<DH, CAUSAL, true>(smem, qkv, d_o, lse, dsum, dqkv, S, nl, bh, ck, pslot);
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

// dQ workgroup number wg (head fastest, then slot)
template <int DH, bool CAUSAL>
__device__ __forceinline__ void attn_dq_wg(char* smem, const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ d_o,
                                           const float* __restrict__ lse, const float* __restrict__ dsum,
                                           bf16_t* __restrict__ dqkv, int S, int nl, int BH,
                                           float* __restrict__ part, ChunkLen ch, int wg) {
    constexpr int TB = tile_bytes<DH>();
    constexpr int NCH = NCHUNKS<DH, FTHREADS>;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6, half = lane >> 5;
    const int qs = wave & 3, kvh = wave >> 2;
    const int bh = wg % BH, slot = wg / BH;
    const Chunk ck = find_chunk(CAUSAL, false, S, ch, slot, 0);
    const int qb = ck.blk;
    const int b = bh / nl, h = bh % nl;
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
    const int tile0 = ck.t0, ntiles = ck.t1;
    const unsigned lds0 = (unsigned)(uintptr_t)(lds_void_ptr)smem;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const i32x4 desc_k = head_rsrc<DH>(kbase, ld, S), desc_v = head_rsrc<DH>(vbase, ld, S);
    unsigned off[NCH];
    dma_offsets<DH, FTHREADS>(off, ld, t);
    auto fetch_tile = [&](int kt, unsigned stage) {       // K and V rows of tile kt -> LDS stage
        const unsigned r0 = (unsigned)kt * TILE * (unsigned)(ld * 2);
        tile_dma<DH, FTHREADS>(desc_k, stage, off, r0, wave_u);
        tile_dma<DH, FTHREADS>(desc_v, stage + TB, off, r0, wave_u);
    };
    fetch_tile(tile0, lds0);
#pragma unroll
    for (int ks = 0; ks < DH / 16; ++ks) { settle(qf[ks]); settle(dof[ks]); }
    settle(l2);
    settle(dq_d);
    dma_wait();
    __syncthreads();
    for (int kt = tile0; kt < ntiles; ++kt) {
        const char* ks_ = smem + ((kt - tile0) & 1) * 2 * TB;
        const char* vs_ = ks_ + TB;
        // the other stage was last read before the barrier that ended the previous step
        if (kt + 1 < ntiles) fetch_tile(kt + 1, lds0 + ((kt - tile0 + 1) & 1) * 2 * TB);
        const int kv0 = kt * TILE + kvh * 32;
        if (kv0 < kv_end && !(CAUSAL && kv0 > q0 + 31)) {                 // wavefront-uniform
            // The fragments of the three MFMA phases (K for S, V for dP, K transposed for dQ) form one sequence that
            // is read through a rolling window of W registers: fragment i + W is requested right after the MFMA
            // that used fragment i, so LDS latency hides under W MFMAs instead of being paid before every one.
            f32x16 s = zero16(), dp = zero16();
            constexpr int NF = DH / 16, W = DH == 64 ? NF : NF / 2;
            bf16x8 fr[W];
            auto fetch = [&](int i) {                       // i is a compile-time constant after unrolling
                if (i < NF) return frag_k<DH>(ks_, kvh * 32, i, lane);
                if (i < 2 * NF) return frag_k<DH>(vs_, kvh * 32, i - NF, lane);
                const int k = i - 2 * NF;
                return frag_t<DH>(ks_, (k >> 1) * 32, kvh * 32 + (k & 1) * 16, lane);
            };
#pragma unroll
            for (int i = 0; i < W; ++i) fr[i] = fetch(i);
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_s_setprio(1);
#pragma unroll
            for (int i = 0; i < 2 * NF; ++i) {
                if (i < NF) s = MFMA(fr[i % W], qf[i], s);
                else dp = MFMA(fr[i % W], dof[i - NF], dp);
                fr[i % W] = fetch(i + W);
                __builtin_amdgcn_sched_barrier(0);
            }
            __builtin_amdgcn_s_setprio(0);
            const bool need_mask = q0 + 31 >= S || kv0 + 31 >= S || (CAUSAL && kv0 + 31 > q0);
            if (need_mask) {                          // wave-uniform: only tiles on the diagonal or at the end of S
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    int kv = kv0 + (v >> 2) * 8 + half * 4 + (v & 3);
                    bool ok = q < S && kv < S && (!CAUSAL || kv <= q);
                    s[v] = ok ? s[v] : -INFINITY;         // exp2(-inf) = 0
                }
            }
#pragma unroll
            for (int v = 0; v < 16; ++v) dp[v] = fast_exp2(fmaf(s[v], c2, -l2)) * (dp[v] - dq_d);
            bf16x8 g0 = pack_regs(dp, 0), g1 = pack_regs(dp, 8);
            __builtin_amdgcn_s_setprio(1);
#pragma unroll
            for (int k = 0; k < NF; ++k) {
                dq[k >> 1] = MFMA(fr[k % W], (k & 1) ? g1 : g0, dq[k >> 1]);
                if (k + W < NF) {
                    fr[k % W] = fetch(2 * NF + k + W);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            __builtin_amdgcn_s_setprio(0);
        }
        dma_wait();
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
    if (kvh == 0 && ck.nch > 1) {
        // one chunk of a longer strip: unscaled float partial, [query][dh]
        float* pp = part + ((int64_t)slot * BH + bh) * (BLK * DH) + (qs * 32 + (lane & 31)) * DH;
#pragma unroll
        for (int dt = 0; dt < DH / 32; ++dt)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float r[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) r[j] = dq[dt][4 * i + j] + mg[(dt * 16 + 4 * i + j) * 64];
                store_f4(pp + dt * 32 + 8 * i + 4 * half, r[0], r[1], r[2], r[3]);
            }
    } else if (kvh == 0 && q < S) {
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

// =================================================================================================
// Backward in one launch: workgroups [0, wgs_kv) compute dK/dV chunks, the rest dQ chunks.  The two are independent,
// both are bound by their longest strip rather than by the amount of work, and a compute unit holds one such
// workgroup at a time: in one launch the units that finish the short chunks of one kind pick up chunks of the other
// instead of idling until the launch ends.  dK/dV first: its steps are the longer ones.
// =================================================================================================
template <int DH, bool CAUSAL>
__global__ __launch_bounds__(FTHREADS, 2) void attn_bwd_kernel(const bf16_t* __restrict__ qkv,
                                                               const bf16_t* __restrict__ d_o,
                                                               const float* __restrict__ lse,
                                                               const float* __restrict__ dsum,
                                                               bf16_t* __restrict__ dqkv, int S, int nl, int BH,
                                                               float* __restrict__ part_kv, float* __restrict__ part_q,
                                                               ChunkLen ch_kv, ChunkLen ch_q, int wgs_kv) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int wg = blockIdx.x;                               // uniform: one kind per workgroup, its own barriers
    if (wg < wgs_kv) attn_dkv_wg<DH, CAUSAL>(smem, qkv, d_o, lse, dsum, dqkv, S, nl, BH, part_kv, ch_kv, wg);
    else attn_dq_wg<DH, CAUSAL>(smem, qkv, d_o, lse, dsum, dqkv, S, nl, BH, part_q, ch_q, wg - wgs_kv);
}

// ---- host side ----------------------------------------------------------------------------------
bool attn_bf16_supported(const AttnArgs& a) {
    // tile loads address a (batch, head) slice with 32-bit byte offsets
    return a.dtype == BF16 && (a.dh == 64 || a.dh == 128) && a.S >= 1 && (int64_t)a.B * a.nl <= 65535 &&
           (int64_t)a.S * 3 * a.nl * a.dh * 2 < (1LL << 31);
}

template <typename K>
static hipError_t set_lds(K kernel, int bytes) {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
}

// Chunk length in tile steps.  No workspace: strips are never cut.  The option attn_chunk = n forces n (0: never cut).
// Every workgroup costs a few steps' worth of start-up and merge and every cut strip its partials, so strips are
// cut only where the longest one would otherwise set the duration, and never into chunks of fewer than 8 steps.
constexpr int NEVER_CUT = 1 << 30;
static bool forced_chunk(const AttnArgs& a, int* ch) {
    if (!a.ws) { *ch = NEVER_CUT; return true; }
    if (const int v = options().attn_chunk; v >= 0) {
        *ch = v > 0 && v < (1 << 16) ? v : NEVER_CUT;
        return true;
    }
    // Inside a layer pass the attention kernels share the chip with the GEMMs of the other chain, which take the
    // compute units that short strips free early: cutting strips there measured 1.2 % slower per step (more
    // workgroups holding units, plus the combine kernel), so the layer leaves the strips whole.
    if (!a.own_chunking) { *ch = NEVER_CUT; return true; }
    return false;
}
static int device_cus() {
    static int cus = 0;
    if (!cus) {
        int dev = 0;
        hipDeviceProp_t pr;
        if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&pr, dev) != hipSuccess) return 0;
        cus = pr.multiProcessorCount;
    }
    return cus;
}
// Forward (a launch of its own): only when there are fewer strips than compute units (with more, the units that
// finish their short strips early pick up the queued ones): the shortest chunk length for which the chunks of all
// heads still run in one round (one workgroup per compute unit, 5 % over allowed).
static int chunk_tiles_fwd(const AttnArgs& a) {
    int ch;
    if (forced_chunk(a, &ch)) return ch;
    const int cus = device_cus();
    const int64_t bh = (int64_t)a.B * a.nl, nblk = (a.S + BLK - 1) / BLK;
    if (!cus || nblk * bh >= cus) return NEVER_CUT;
    const int longest = (a.S + TILE - 1) / TILE;
    for (ch = 8; ch < longest; ++ch)
        if (strip_slots(a.causal, false, a.S, make_chunk_len(ch)) * bh * 100 <= 105LL * cus) return ch;
    return NEVER_CUT;
}
// Backward: dK/dV and dQ workgroups share one launch, so the units that finish short strips of one kind pick up
// strips of the other; with at least as many workgroups as compute units cutting measured no faster (the combine
// kernel costs what the shorter critical path gains).  With fewer, the same rule as forward over both kinds.
static int chunk_tiles_bwd(const AttnArgs& a, bool kv_side) {
    int ch;
    (void)kv_side;                              // one length for both kinds
    if (forced_chunk(a, &ch)) return ch;
    const int cus = device_cus();
    const int64_t bh = (int64_t)a.B * a.nl, nblk = (a.S + BLK - 1) / BLK;
    if (!cus || 2 * nblk * bh >= cus) return NEVER_CUT;
    const int longest = (a.S + TILE - 1) / TILE;
    for (ch = 8; ch < longest; ++ch) {
        const ChunkLen c = make_chunk_len(ch);
        if ((strip_slots(a.causal, false, a.S, c) + strip_slots(a.causal, true, a.S, c)) * bh * 100 <= 105LL * cus) return ch;
    }
    return NEVER_CUT;
}
static size_t part_bytes_fwd(const AttnArgs& a, ChunkLen ch) {
    return (size_t)strip_slots(a.causal, false, a.S, ch) * a.B * a.nl * BLK * (a.dh + 2) * sizeof(float);
}
static size_t part_bytes_dq(const AttnArgs& a, ChunkLen ch) {
    return (size_t)strip_slots(a.causal, false, a.S, ch) * a.B * a.nl * BLK * a.dh * sizeof(float);
}
static size_t part_bytes_dkv(const AttnArgs& a, ChunkLen ch) {
    return (size_t)strip_slots(a.causal, true, a.S, ch) * a.B * a.nl * BLK * 2 * a.dh * sizeof(float);
}
// Blocks whose strips are cut: a contiguous range (strip length is monotonic in the block index).
static void cut_range(const AttnArgs& a, bool kv_side, ChunkLen ch, int* blk0, int* n) {
    const int nblk = (a.S + BLK - 1) / BLK;
    int lo = nblk, hi = -1;
    for (int blk = 0; blk < nblk; ++blk)
        if (strip_tiles(a.causal, kv_side, a.S, blk) > ch.ch) { lo = blk < lo ? blk : lo; hi = blk; }
    *blk0 = hi < 0 ? 0 : lo;
    *n = hi < 0 ? 0 : hi - lo + 1;
}
static bool cuts(const AttnArgs& a, bool kv_side, ChunkLen ch) {
    return strip_slots(a.causal, kv_side, a.S, ch) != (a.S + BLK - 1) / BLK;
}
// Workspace that lets the strips be cut (0: they would not be cut anyway).  Sized with a stand-in non-null
// workspace pointer so that the same rule decides as at launch.
size_t attn_bf16_workspace_bytes(const AttnArgs& a0, bool bwd) {
    AttnArgs a = a0;
    a.ws = reinterpret_cast<void*>(16);
    if (!bwd) {
        const ChunkLen ch = make_chunk_len(chunk_tiles_fwd(a));
        return cuts(a, false, ch) ? part_bytes_fwd(a, ch) : 0;
    }
    const ChunkLen ch_q = make_chunk_len(chunk_tiles_bwd(a, false)), ch_kv = make_chunk_len(chunk_tiles_bwd(a, true));
    return (cuts(a, false, ch_q) ? part_bytes_dq(a, ch_q) : 0) + (cuts(a, true, ch_kv) ? part_bytes_dkv(a, ch_kv) : 0);
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
    const ChunkLen ch = make_chunk_len(chunk_tiles_fwd(a));
    if (a.ws && cuts(a, false, ch) && part_bytes_fwd(a, ch) > a.ws_bytes) return hipErrorInvalidValue;
    const int BH = a.B * a.nl;
    const int64_t wgs = (int64_t)strip_slots(CAUSAL, false, a.S, ch) * BH;
    if (wgs > 0x7fffffffLL) return hipErrorInvalidValue;
    float* part = static_cast<float*>(a.ws);
    hipLaunchKernelGGL((attn_fwd_kernel<DH, CAUSAL>), dim3((unsigned)wgs), dim3(FTHREADS), LDS, a.stream,
                       (const bf16_t*)a.qkv, (bf16_t*)a.o, a.lse, a.S, a.nl, BH, part, ch);
    int blk0 = 0, ncut = 0;
    cut_range(a, false, ch, &blk0, &ncut);
    if (ncut)
        hipLaunchKernelGGL((attn_fwd_combine_kernel<DH, CAUSAL>), dim3(ncut * (BLK * DH / 1024), BH), dim3(256), 0,
                           a.stream, part, (bf16_t*)a.o, a.lse, a.S, a.nl, BH, ch, blk0);
    return hipGetLastError();
}

template <int DH, bool CAUSAL>
static hipError_t bwd_t(const AttnArgs& a) {
    constexpr int LDS_KV = 2 * (2 * tile_bytes<DH>() + 2 * TILE * 4);
    constexpr int LDS_Q = dq_lds_bytes<DH>();
    constexpr int LDS = LDS_KV > LDS_Q ? LDS_KV : LDS_Q;
    static bool once = false;
    if (!once) {
        hipError_t e = set_lds(&attn_bwd_kernel<DH, CAUSAL>, LDS);
        if (e != hipSuccess) return e;
        once = true;
    }
    const ChunkLen ch_q = make_chunk_len(chunk_tiles_bwd(a, false)), ch_kv = make_chunk_len(chunk_tiles_bwd(a, true));
    const bool cut_q = cuts(a, false, ch_q), cut_kv = cuts(a, true, ch_kv);
    const size_t bytes_q = cut_q ? part_bytes_dq(a, ch_q) : 0, bytes_kv = cut_kv ? part_bytes_dkv(a, ch_kv) : 0;
    if (a.ws && bytes_q + bytes_kv > a.ws_bytes) return hipErrorInvalidValue;
    const int BH = a.B * a.nl;
    const int64_t wgs_q = (int64_t)strip_slots(CAUSAL, false, a.S, ch_q) * BH;
    const int64_t wgs_kv = (int64_t)strip_slots(CAUSAL, true, a.S, ch_kv) * BH;
    if (wgs_q + wgs_kv > 0x7fffffffLL) return hipErrorInvalidValue;
    float* part_q = static_cast<float*>(a.ws);
    float* part_kv = a.ws ? reinterpret_cast<float*>(static_cast<char*>(a.ws) + bytes_q) : nullptr;
    const int64_t rows = (int64_t)a.B * a.S;
    hipLaunchKernelGGL((attn_dsum_kernel<DH>), dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, a.stream,
                       (const bf16_t*)a.o, (const bf16_t*)a.d_o, a.dsum, a.B, a.S, a.nl);
    hipLaunchKernelGGL((attn_bwd_kernel<DH, CAUSAL>), dim3((unsigned)(wgs_kv + wgs_q)), dim3(FTHREADS), LDS, a.stream,
                       (const bf16_t*)a.qkv, (const bf16_t*)a.d_o, a.lse, a.dsum, (bf16_t*)a.dqkv, a.S, a.nl, BH,
                       part_kv, part_q, ch_kv, ch_q, (int)wgs_kv);
    int blk0_q = 0, ncut_q = 0, blk0_kv = 0, ncut_kv = 0;
    cut_range(a, false, ch_q, &blk0_q, &ncut_q);
    cut_range(a, true, ch_kv, &blk0_kv, &ncut_kv);
    if (ncut_q || ncut_kv)
        hipLaunchKernelGGL((attn_bwd_combine_kernel<DH, CAUSAL>),
                           dim3((ncut_q > ncut_kv ? ncut_q : ncut_kv) * (BLK * DH / 1024), BH, 3), dim3(256), 0, a.stream,
                           part_q, part_kv, (bf16_t*)a.dqkv, a.S, a.nl, BH, ch_q, ch_kv, blk0_q, ncut_q, blk0_kv,
                           ncut_kv);
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
