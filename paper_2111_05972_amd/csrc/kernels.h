// Internal launch interface between the C-ABI host code and the HIP kernels.
#pragma once
#include <hip/hip_runtime_api.h>
#include <stddef.h>
#include <stdint.h>

namespace tpl {

enum Dtype { F32 = 0, BF16 = 1 };

// Tuning overrides of the kernel choices (tests run every tile variant through them; tuning forces single plans).
// Read from the environment ONCE, when the library is first used (TPL_GEMM_TILE, TPL_GEMM_SHARES, TPL_GEMM_BAND,
// TPL_GEMM_FORCE, TPL_ATTN_CHUNK); afterwards only tp_layer_set_option changes them.  Nothing on a launch path
// reads the environment.  `generation` increases with every change: plans cached per shape carry it.
struct Options {
    int gemm_tile = -1;        // force one tile variant (0 .. number of variants - 1); -1: the planner chooses
    int gemm_shares = 0;       // force a K split; 0: the planner chooses
    int gemm_band = 0;         // force the band height of the tile order; 0: choose_band
    int attn_chunk = -1;       // force the chunk length of attention strips in 64-row tile steps (0: never cut); -1: unset
    int side_chains = 0;       // chains of a backward pass under TPL_SIDE_STREAM: 2, or 3 (dW_dn and dW_o on a stream of their
                               // own); 0: the library chooses by the size of the weight gradients
    int fuse_colsum = 0;       // 1: bias gradients as one more output row of the weight-gradient GEMM where its kernel can
    char gemm_force[1024] = "";   // "MxNxK@ab=v[:shares];..." plans of single shapes (a, b = 1: A, B K-major)
    unsigned generation = 0;
};
const Options& options();
// name: "gemm_tile", "gemm_shares", "gemm_band", "gemm_force", "attn_chunk", "fuse_colsum", "side_chains"; value null or "": back to unset.
// Returns false for an unknown name or a value that does not parse.
bool set_option(const char* name, const char* value);
enum Epi { EPI_NONE = 0, EPI_GELU = 1, EPI_DGELU = 2 };

// C[M,N] = epi(opA(A) opB(B)); see tp_layer_gemm in tp_layer.h for the meaning of each field.
struct GemmArgs {
    int dtype;
    int trans_a, trans_b;
    int64_t M, N, K;
    const void* A;
    const void* B;
    void* C;
    const void* bias;   // [N] or null
    const void* resid;  // [M,N] or null
    void* aux;          // [M,N]: written (EPI_GELU) or read (EPI_DGELU)
    int epi;
    void* ws;
    size_t ws_bytes;
    hipStream_t stream;
    bool c_streaming;   // C is not read again soon (weight gradients): store it with the non-temporal hint
    void* colsum_b;     // [N] or null: where the kernel may also leave sum_k B[k][n] (the bias gradient that goes with a
                        // weight gradient); whether it did is reported by gemm_bf16 / run through colsum_done
    bool colsum_done;
};

struct AttnArgs {
    int dtype;
    int B, S, nl, dh;
    int causal;
    const void* qkv;   // [B*S, 3*nl*dh]
    void* o;           // fwd: written; bwd: read
    float* lse;        // [B, nl, S]
    const void* d_o;   // bwd only
    void* dqkv;        // bwd only
    float* dsum;       // bwd only: [B, nl, S] scratch, rowsum(dO * O)
    void* ws;          // optional (bf16 kernels): float partials that let long strips be cut into chunks
    size_t ws_bytes;
    int own_chunking;  // 1: the kernels may cut strips by their own rule; 0: only when TPL_ATTN_CHUNK forces a length
    hipStream_t stream;
};

// Generic kernels (any shape; the only path for float).
hipError_t gemm_simple(const GemmArgs& a);
hipError_t attn_simple_fwd(const AttnArgs& a);
hipError_t attn_simple_bwd(const AttnArgs& a);
// out[n] = sum_m X[m,n]  (bias gradients), deterministic.
hipError_t colsum(int dtype, int64_t M, int64_t N, const void* X, void* out, float* scratch, hipStream_t s);
size_t colsum_scratch_bytes(int64_t M, int64_t N);
// The library's own scratch (a static device array, one copy per GPU) for entry points that may not allocate:
// *ptr = its address on the current device.  Calls that use it on one GPU share it.
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)4 << 20;
hipError_t static_scratch(void** ptr);
// out[n] = sum over slabs of part[slab * stride + n], in slab order.
hipError_t sum_partials_strided(int dtype, int64_t slabs, int64_t N, const float* part, int64_t stride,
                                void* out, hipStream_t s);

// LayerNorm over the hidden dimension of z = a (+ b): HBM-bound, one pass over each tensor.
struct LnArgs {
    int dtype;
    int64_t M, H;
    const void* a; const void* b;          // b may be null
    const void* gamma; const void* beta;
    float eps;
    void* z;                               // fwd: a + b written here if non-null; bwd: the normalised input
    void* y;
    float* mean; float* rstd;              // [M]
    const void* dy; void* dz; void* dgamma; void* dbeta;   // bwd
    float* partials;                       // bwd scratch: ln_scratch_bytes(M, H)
    hipStream_t stream;
};
bool ln_supported(int64_t H);
int64_t ln_partial_rows(int64_t M);
size_t ln_scratch_bytes(int64_t M, int64_t H);
hipError_t ln_fwd(const LnArgs& a);
hipError_t ln_bwd(const LnArgs& a);

// Distributed layer normalisation of a channel slice [M, Hs] (of H channels in all) and bias / residual / GeLU on a
// slice: the element-wise pieces of the memory-optimised distribution.  sums / totals are [M][2] floats.
hipError_t ln_dist_moments(int dtype, int64_t M, int64_t Hs, const void* x, float* sums, hipStream_t s);
hipError_t ln_dist_stats(int64_t M, int64_t H, float eps, const float* totals, float* mean, float* rstd,
                         hipStream_t s);
hipError_t ln_dist_apply(int dtype, int64_t M, int64_t Hs, const void* x, const float* mean, const float* rstd,
                         const void* gamma, const void* beta, void* y, hipStream_t s);
hipError_t ln_dist_bwd_sums(int dtype, int64_t M, int64_t Hs, const void* dy, const void* x, const float* mean,
                            const float* rstd, const void* gamma, float* sums, hipStream_t s);
hipError_t ln_dist_bwd_apply(int dtype, int64_t M, int64_t Hs, int64_t H, const void* dy, const void* x,
                             const float* mean, const float* rstd, const void* gamma, const float* totals,
                             const void* dx_add, void* dx, void* dgamma, void* dbeta, float* partials,
                             hipStream_t s);
size_t ln_dist_scratch_bytes(int64_t M, int64_t Hs);
hipError_t slice_epilogue_fwd(int dtype, bool gelu, int64_t M, int64_t N, const void* in, const void* bias,
                              const void* resid, void* u, void* out, hipStream_t s);
hipError_t gelu_bwd(int dtype, int64_t M, int64_t N, const void* dg, const void* u, void* du, hipStream_t s);

// bf16 MFMA kernels for gfx950.
bool gemm_bf16_supported(const GemmArgs& a);
size_t gemm_bf16_workspace_bytes(int64_t M, int64_t N, int64_t K);
hipError_t gemm_bf16(const GemmArgs& a, bool* colsum_done = nullptr);
bool attn_bf16_supported(const AttnArgs& a);
hipError_t attn_bf16_fwd(const AttnArgs& a);
hipError_t attn_bf16_bwd(const AttnArgs& a);
size_t attn_bf16_workspace_bytes(const AttnArgs& a, bool bwd);

}  // namespace tpl
