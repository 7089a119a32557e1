// Internal launch interface between the C-ABI host code and the HIP kernels.
#pragma once
#include <hip/hip_runtime_api.h>
#include <stddef.h>
#include <stdint.h>

namespace tpl {

enum Dtype { F32 = 0, BF16 = 1 };
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
    hipStream_t stream;
};

// Generic kernels (any shape; the only path for float).
hipError_t gemm_simple(const GemmArgs& a);
hipError_t attn_simple_fwd(const AttnArgs& a);
hipError_t attn_simple_bwd(const AttnArgs& a);
// out[n] = sum_m X[m,n]  (bias gradients), deterministic.
hipError_t colsum(int dtype, int64_t M, int64_t N, const void* X, void* out, float* scratch, hipStream_t s);
size_t colsum_scratch_bytes(int64_t M, int64_t N);

// bf16 MFMA kernels for gfx950.
bool gemm_bf16_supported(const GemmArgs& a);
size_t gemm_bf16_workspace_bytes(int64_t M, int64_t N, int64_t K);
hipError_t gemm_bf16(const GemmArgs& a);
bool attn_bf16_supported(const AttnArgs& a);
hipError_t attn_bf16_fwd(const AttnArgs& a);
hipError_t attn_bf16_bwd(const AttnArgs& a);

}  // namespace tpl
