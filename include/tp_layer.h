/*
 * tp_layer.h - C ABI of the tensor-parallel transformer-layer shard for MI355X (gfx950).
 *
 * One call computes what ONE tensor-parallel rank computes for ONE transformer layer under the
 * speed-optimised distribution of the paper (arXiv 2111.05972, App. F.1 "Speed-optimized
 * distribution"; Sec. 5.3): in the self-attention block and in the MLP block the first linear
 * layer is split across ranks over its output channels and the second over its input channels.
 * The activations between the two are sharded, everything else is replicated, and each block ends
 * in a partial sum that the ranks of the tensor-parallel group would all-reduce.  This library
 * stops before that all-reduce: partial sums are returned as they are (forward), and so are the
 * partial input gradients that `bwd_allreduce_for_tp` (App. I.5) would reduce (backward).
 *
 * Notation: H hidden size, nh heads, dh head size, I MLP width, T tensor-parallel degree,
 * r rank, S sequence length, B micro-batch, M = B*S tokens, nl = nh/T, Hl = nl*dh, Il = I/T.
 *
 * Layout.  Every tensor is dense row-major in DEVICE memory; a linear layer is y = x W + b with
 * W stored [in, out].  Rank r holds
 *   w_qkv [H, 3*Hl]  columns ordered (q | k | v), then local head, then dh;   b_qkv [3*Hl]
 *   w_o   [Hl, H]    rows r*Hl .. of the unsharded matrix;                      b_o   [H]
 *   w_up  [H, Il]    columns r*Il .. of the unsharded matrix;                   b_up  [Il]
 *   w_dn  [Il, H]    rows r*Il .. of the unsharded matrix;                      b_dn  [H]
 * Activations and their gradients are [M, H] (token m = b*S + s).  Element type is `dtype`
 * (float, or bfloat16 with float accumulation) for everything except LSE and the softmax
 * row terms, which are float.
 *
 * The bias of a row-split linear layer lives on one rank only ((W1 x1 + b) + W2 x2 = W x + b,
 * caption of Fig. 7).  TPL_ROW_EPILOGUE marks that rank: it adds b_o / b_dn and the residual
 * input to its partial sums, and in backward receives db_o, db_dn and adds dy to its partial dx.
 *
 * Ownership.  The caller owns every buffer, including `saved` and `ws`; the library allocates no
 * device memory, never synchronises with the host, and orders all work on `hip_stream` (a
 * hipStream_t passed as void*; NULL = the default stream): work enqueued on `hip_stream` before a
 * call happens before it, work enqueued after the call happens after it.  By default every kernel
 * of a call is enqueued on `hip_stream` itself.  With TPL_SIDE_STREAM in the descriptor's flags,
 * tp_layer_fwd / tp_layer_bwd / tp_layer_bwd_recompute enqueue the attention block and the MLP
 * block, which share no tensor, as two chains, the second on a stream the library creates once per
 * device (default priority) and forks from / joins to `hip_stream` with events (also when the call
 * fails half-way); for small layers the backward pass runs a third chain (the two weight gradients
 * that depend on nothing computed in the pass) on another such stream.  These streams and their
 * events are shared by all calls on a device: host
 * threads that make such calls on the same device at the same time must serialise them.
 * Pointers must be 16-byte aligned.  Outputs must not alias inputs.  Gradients are overwritten,
 * not accumulated.  `ws` contents need not be preserved between calls; calls that share a `ws`
 * must be stream-ordered.
 *
 * Environment.  Nothing on a launch path reads the environment.  The tuning overrides
 * TPL_GEMM_TILE, TPL_GEMM_SHARES, TPL_GEMM_BAND, TPL_GEMM_FORCE and TPL_ATTN_CHUNK are read once,
 * when the library is first used, as initial values of the options of tp_layer_set_option.
 *
 * Errors.  Every entry point returns a tpl_status and never aborts; arguments are validated
 * before anything is enqueued.
 */
#ifndef TP_LAYER_H
#define TP_LAYER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    TPL_OK = 0,
    TPL_EINVAL = 1,        /* NULL pointer, non-positive size, sizes that do not divide          */
    TPL_EUNSUPPORTED = 2,  /* valid layer, but a shape/dtype this build has no kernel for       */
    TPL_EWORKSPACE = 3,    /* ws_bytes smaller than tp_layer_workspace_bytes()                  */
    TPL_EALIGN = 4,        /* a device pointer is not 16-byte aligned                           */
    TPL_EHIP = 5           /* the HIP runtime refused a launch                                  */
} tpl_status;

typedef enum { TPL_F32 = 0, TPL_BF16 = 1 } tpl_dtype;

enum {
    TPL_CAUSAL = 1u,       /* query i attends keys j <= i (else no mask); Sec. I.4 `causal_mask_size` */
    TPL_ROW_EPILOGUE = 2u, /* this rank adds b_o, b_dn and the residual (tp_rank 0 by the Fig. 7 rule) */
    TPL_SIDE_STREAM = 4u   /* scheduling only: run the two blocks of a pass as two chains (see Ownership) */
};

/* The layer and this rank's place in it (App. F.1; constructor arguments of
 * DistributedTransformerLayer in Sec. I.4; tensor_parallel_degree in Sec. I.1). */
typedef struct {
    int32_t hidden;        /* H                                                    */
    int32_t heads;         /* nh, over all ranks                                   */
    int32_t head_dim;      /* dh; 0 means hidden / heads                           */
    int32_t intermediate;  /* I, over all ranks; 0 means 4 * hidden                */
    int32_t tp_degree;     /* T                                                    */
    int32_t tp_rank;       /* r, 0 <= r < T (identifies the shard; not used in arithmetic) */
    int32_t seq;           /* S                                                    */
    int32_t micro_batch;   /* B                                                    */
    int32_t dtype;         /* tpl_dtype                                            */
    uint32_t flags;        /* TPL_CAUSAL | TPL_ROW_EPILOGUE | TPL_SIDE_STREAM      */
} tp_layer_desc;

/* This rank's parameter shard (device pointers, read-only).  b_o and b_dn may be NULL unless
 * TPL_ROW_EPILOGUE is set. */
typedef struct {
    const void *w_qkv, *b_qkv, *w_o, *b_o, *w_up, *b_up, *w_dn, *b_dn;
} tp_layer_params;

/* Gradients of the shard (device pointers, written).  db_o and db_dn are written only with
 * TPL_ROW_EPILOGUE and may be NULL otherwise. */
typedef struct {
    void *dw_qkv, *db_qkv, *dw_o, *db_o, *dw_up, *db_up, *dw_dn, *db_dn;
} tp_layer_grads;

/* Byte offsets inside `saved` of what forward keeps for backward. */
typedef struct {
    size_t qkv;  /* [M, 3*Hl] dtype : fused projection output, columns (q|k|v, head, dh) */
    size_t o;    /* [M, Hl]   dtype : attention output, columns (head, dh)                */
    size_t lse;  /* [B, nl, S] float: log-sum-exp of each softmax row                    */
    size_t u;    /* [M, Il]   dtype : MLP pre-activation                                 */
    size_t g;    /* [M, Il]   dtype : gelu(u)                                            */
    size_t total;
} tp_layer_saved_layout;

/* Pure host check of a descriptor: sizes positive, heads*head_dim == hidden, heads and
 * intermediate divisible by tp_degree, 0 <= tp_rank < tp_degree, known dtype and flags.
 * TPL_EUNSUPPORTED if the layer is valid but not computable here (bf16 needs H, Hl, Il
 * multiples of 8 for 16-byte rows; head_dim <= 256).  Needs no GPU. */
int tp_layer_validate(const tp_layer_desc* desc);

/* Size and layout of the `saved` buffer.  Return 0 / TPL_EINVAL for an invalid descriptor. */
size_t tp_layer_saved_bytes(const tp_layer_desc* desc);
int tp_layer_saved_offsets(const tp_layer_desc* desc, tp_layer_saved_layout* out);

/* Scratch the forward (bwd == 0) or backward (bwd != 0) pass needs; 0 for an invalid descriptor. */
size_t tp_layer_workspace_bytes(const tp_layer_desc* desc, int bwd);

/* Forward of the shard (App. F.1):
 *   QKV = x_attn w_qkv + b_qkv;  per (b, local head): P = softmax(mask(Q K^T / sqrt(dh))), O = P V
 *   y_attn_partial = O w_o            (+ b_o  + x_attn with TPL_ROW_EPILOGUE)
 *   U = x_mlp w_up + b_up;  G = gelu(U) (exact erf form)
 *   y_mlp_partial  = G w_dn           (+ b_dn + x_mlp  with TPL_ROW_EPILOGUE)
 * x_attn, x_mlp: [M, H] inputs replicated over the tensor-parallel group (x_mlp would be the
 * all-reduced, normalised attention output in a full model; the caller supplies it).
 * y_*_partial: [M, H], the unreduced row-parallel partial sums.  `saved`: tp_layer_saved_bytes(). */
int tp_layer_fwd(const tp_layer_desc* desc, const tp_layer_params* params,
                 const void* x_attn, const void* x_mlp,
                 void* y_attn_partial, void* y_mlp_partial,
                 void* saved, void* ws, size_t ws_bytes, void* hip_stream);

/* Backward of the shard for upstream gradients dy_attn, dy_mlp [M, H] (replicated):
 *   dG = dy_mlp w_dn^T; dw_dn = G^T dy_mlp; dU = dG * gelu'(U); dw_up = x_mlp^T dU; db_up = sum_m dU
 *   dx_mlp_partial = dU w_up^T        (+ dy_mlp with TPL_ROW_EPILOGUE; then also db_dn = sum_m dy_mlp)
 *   dO = dy_attn w_o^T; dw_o = O^T dy_attn; softmax-attention backward gives dQKV
 *   dw_qkv = x_attn^T dQKV; db_qkv = sum_m dQKV
 *   dx_attn_partial = dQKV w_qkv^T    (+ dy_attn with TPL_ROW_EPILOGUE; then also db_o = sum_m dy_attn)
 * `saved` is what tp_layer_fwd wrote for the same inputs. */
int tp_layer_bwd(const tp_layer_desc* desc, const tp_layer_params* params,
                 const void* x_attn, const void* x_mlp,
                 const void* dy_attn, const void* dy_mlp,
                 const void* saved, const tp_layer_grads* grads,
                 void* dx_attn_partial, void* dx_mlp_partial,
                 void* ws, size_t ws_bytes, void* hip_stream);

/* Activation-checkpoint mode (App. H.2: activations are recomputed in backward instead of kept):
 * backward without `saved`.  QKV, O, LSE, U and G are recomputed from x_attn, x_mlp into the front of
 * `ws` (the two row-parallel forward GEMMs, whose outputs backward never reads, are not recomputed),
 * then the backward of tp_layer_bwd runs.  Results are bit-identical to tp_layer_fwd + tp_layer_bwd.
 * b_qkv and b_up must be set in `params`.  ws_bytes >= tp_layer_workspace_bytes_recompute(). */
size_t tp_layer_workspace_bytes_recompute(const tp_layer_desc* desc);
int tp_layer_bwd_recompute(const tp_layer_desc* desc, const tp_layer_params* params,
                           const void* x_attn, const void* x_mlp,
                           const void* dy_attn, const void* dy_mlp,
                           const tp_layer_grads* grads,
                           void* dx_attn_partial, void* dx_mlp_partial,
                           void* ws, size_t ws_bytes, void* hip_stream);

/* Replicated layer normalisation either side of the shard.  In the speed-optimised distribution
 * layer normalisation is not distributed (Sec. I.1): each rank normalises the whole [M, H] tensor.
 *   z = a + b (b may be NULL: z = a);  y = (z - mean_H(z)) / sqrt(var_H(z) + eps) * gamma + beta
 * (biased variance over the hidden dimension; eps is `layernorm_epsilon` of Sec. I.4).  Writes y, the
 * per-row mean and 1/sqrt(var + eps) (float [M]) and, if z != NULL, the residual sum z.
 * H must be a multiple of 8 and at most 16384.  a, b, z, y: [M, H] dtype; gamma, beta: [H] dtype. */
int tp_layer_ln_fwd(int dtype, int64_t M, int64_t H, const void* a, const void* b,
                    const void* gamma, const void* beta, float eps,
                    void* z, void* y, float* mean, float* rstd, void* hip_stream);
/* Backward: dz = rstd * (g - mean_H(g) - zh * mean_H(g * zh)), g = dy * gamma, zh = (z - mean) * rstd
 * (dz is the gradient of both a and b); dgamma = sum_m dy * zh; dbeta = sum_m dy (fixed summation
 * order).  z is the normalised input (what forward wrote to z, or a itself when b was NULL). */
size_t tp_layer_ln_workspace_bytes(int64_t M, int64_t H);
int tp_layer_ln_bwd(int dtype, int64_t M, int64_t H, const void* dy, const void* z,
                    const float* mean, const float* rstd, const void* gamma,
                    void* dz, void* dgamma, void* dbeta, void* ws, size_t ws_bytes, void* hip_stream);

/* Memory-optimised distribution, local compute of one rank (App. F.2): every linear layer is split
 * over its INPUT channels, its product is a full-width partial sum and a reduce-scatter over the
 * ranks replaces the all-reduce; layer normalisation is distributed too.  The collectives are the
 * caller's.  The linear layers themselves are tp_layer_gemm calls on the rank's operands:
 *   forward  partial[M, N] = x_loc[M, Ks] w_rows[Ks, N]         (trans_a = 0, trans_b = 0, no epilogue)
 *   backward dx_loc = dy_full w_rows^T (trans_b = 1);  dw_rows = x_loc^T dy_full (trans_a = 1)
 * with dy_full the all-gathered output gradient; attention on the local heads is tp_layer_attn_*.
 * The entry points below are the pieces around them.  All tensors device memory, 16-byte aligned;
 * Hs and N multiples of 8, Hs <= 16384; sums / totals are float [M][2].
 *
 * Distributed layer normalisation of the channel slice x_loc [M, Hs] (H channels over all ranks):
 *   1. tp_layer_ln_moments : sums[m] = (sum_c x_loc[m,c], sum_c x_loc[m,c]^2)
 *      (the caller all-reduces `sums` over the ranks: two scalars per token)
 *   2. tp_layer_ln_stats   : mean = S1/H, rstd = 1/sqrt(S2/H - mean^2 + eps) from the totals
 *   3. tp_layer_ln_apply_fwd ("ApplyLayerNorm"): y = (x_loc - mean) * rstd * gamma_loc + beta_loc
 * and its backward, xh = (x_loc - mean) * rstd:
 *   4. tp_layer_ln_apply_bwd_sums : sums[m] = (sum_c dy*gamma_loc, sum_c dy*gamma_loc*xh)   (all-reduced by the caller)
 *   5. tp_layer_ln_apply_bwd      : dx = rstd * (dy*gamma_loc - C1/H - xh*C2/H) with the totals (C1, C2),
 *      plus dx_add if it is not NULL (the gradient that reaches x over the residual branch);
 *      dgamma_loc = sum_m dy*xh, dbeta_loc = sum_m dy (fixed summation order).
 *      ws_bytes >= tp_layer_ln_apply_workspace_bytes(M, Hs). */
int tp_layer_ln_moments(int dtype, int64_t M, int64_t Hs, const void* x_loc, float* sums, void* hip_stream);
int tp_layer_ln_stats(int64_t M, int64_t H, float eps, const float* totals, float* mean, float* rstd,
                      void* hip_stream);
int tp_layer_ln_apply_fwd(int dtype, int64_t M, int64_t Hs, const void* x_loc, const float* mean,
                          const float* rstd, const void* gamma_loc, const void* beta_loc, void* y,
                          void* hip_stream);
int tp_layer_ln_apply_bwd_sums(int dtype, int64_t M, int64_t Hs, const void* dy, const void* x_loc,
                               const float* mean, const float* rstd, const void* gamma_loc, float* sums,
                               void* hip_stream);
size_t tp_layer_ln_apply_workspace_bytes(int64_t M, int64_t Hs);
int tp_layer_ln_apply_bwd(int dtype, int64_t M, int64_t Hs, int64_t H, const void* dy, const void* x_loc,
                          const float* mean, const float* rstd, const void* gamma_loc, const float* totals,
                          const void* dx_add, void* dx, void* dgamma_loc, void* dbeta_loc, void* ws,
                          size_t ws_bytes, void* hip_stream);
/* What a rank does to the slice [M, N] it keeps after a reduce-scatter (the product of an input-split
 * linear is a partial sum, so bias, residual and activation cannot ride in the GEMM epilogue):
 *   forward : v = in + bias (+ resid if resid != NULL);
 *             TPL_ACT_NONE: out = v;   TPL_ACT_GELU: u = v (kept for backward), out = gelu(v)
 *   backward: TPL_ACT_GELU: din = dout * gelu'(u);  TPL_ACT_NONE: the gradient of `in` (and of `resid`) is
 *             dout itself and din is not written (may be NULL);  dbias = sum_m of that gradient (fixed order).
 * in, resid, u, out, dout, din: [M, N] dtype; bias, dbias: [N] dtype; out may alias in.
 * ws_bytes >= tp_layer_slice_epilogue_workspace_bytes(M, N). */
enum { TPL_ACT_NONE = 0, TPL_ACT_GELU = 1 };
int tp_layer_slice_epilogue_fwd(int dtype, int act, int64_t M, int64_t N, const void* in, const void* bias,
                                const void* resid, void* u, void* out, void* hip_stream);
size_t tp_layer_slice_epilogue_workspace_bytes(int64_t M, int64_t N);
int tp_layer_slice_epilogue_bwd(int dtype, int act, int64_t M, int64_t N, const void* dout, const void* u,
                                void* din, void* dbias, void* ws, size_t ws_bytes, void* hip_stream);

/* tp_layer_slice_epilogue_bwd for callers that cannot allocate or pass a workspace (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): the same kernels, with the column-sum partials in a
 * static device array of the library instead of `ws`.  The array is tp_layer_static_scratch_bytes() (4 MiB) per
 * GPU and is held until the process ends; a problem whose partials do not fit
 * (tp_layer_slice_epilogue_workspace_bytes(M, N) above that size, i.e. ceil(M / 64) * N floats) is refused with
 * TPL_EWORKSPACE.  The call allocates nothing and never synchronises.  All calls on one GPU share the array:
 * calls that overlap on one GPU (different streams without ordering) race on it; stream-ordered calls do not. */
size_t tp_layer_static_scratch_bytes(void);
int tp_layer_slice_epilogue_bwd_static(int dtype, int act, int64_t M, int64_t N, const void* dout, const void* u,
                                       void* din, void* dbias, void* hip_stream);

/* One GEMM of the path with its fused epilogue, exposed for per-kernel tests and timing:
 *   C[M,N] = epi( opA(A) opB(B) ),  element type `dtype`, float accumulation.
 * trans_a == 0: A is [M,K] row-major, else A is [K,M] row-major (used as its transpose).
 * trans_b == 0: B is [K,N] row-major, else B is [N,K] row-major (used as its transpose).
 * epi: v = acc (+ bias[n] if bias) (+ resid[m,n] if resid);
 *      TPL_EPI_GELU : aux[m,n] = v (pre-activation), C = gelu(v)
 *      TPL_EPI_DGELU: C = v * gelu'(aux[m,n])
 * bias, resid, aux may be NULL when unused.  ws as for tp_layer_fwd (tp_layer_gemm_workspace_bytes). */
enum { TPL_EPI_NONE = 0, TPL_EPI_GELU = 1, TPL_EPI_DGELU = 2 };
size_t tp_layer_gemm_workspace_bytes(int dtype, int64_t M, int64_t N, int64_t K);
int tp_layer_gemm(int dtype, int trans_a, int trans_b, int64_t M, int64_t N, int64_t K,
                  const void* A, const void* B, void* C,
                  const void* bias, const void* resid, void* aux, int epi,
                  void* ws, size_t ws_bytes, void* hip_stream);

/* Softmax attention over local heads, exposed for per-kernel tests and timing.
 * qkv [B*S, 3*nl*dh] (columns q|k|v, head, dh) -> o [B*S, nl*dh], lse [B, nl, S] float.
 * ws (device, 16-byte aligned, caller-owned, contents undefined afterwards) may be NULL.  With a
 * workspace of tp_layer_attn_workspace_bytes(..., bwd) bytes the bf16 kernels may cut the tile steps
 * of a (128-row block, head) into chunks that run as separate workgroups and are combined in chunk
 * order by a second kernel (float partials in ws): the causal mask makes those strips triangular
 * and the longest one would otherwise set the duration of the launch.  Results are deterministic
 * either way; they differ between the two ways by float rounding only.  A non-NULL ws that is too
 * small gives TPL_EWORKSPACE.  The option attn_chunk = n (tp_layer_set_option) forces chunks of n
 * 64-row tile steps (0: never cut); it must not change between the size query and the call. */
size_t tp_layer_attn_workspace_bytes(int dtype, int B, int S, int nl, int dh, int causal, int bwd);
int tp_layer_attn_fwd(int dtype, int B, int S, int nl, int dh, int causal,
                      const void* qkv, void* o, float* lse, void* ws, size_t ws_bytes, void* hip_stream);
/* d_scratch: [B, nl, S] float scratch (row sums of dO*O); dqkv [B*S, 3*nl*dh]. */
int tp_layer_attn_bwd(int dtype, int B, int S, int nl, int dh, int causal,
                      const void* qkv, const void* o, const float* lse, const void* d_o,
                      void* dqkv, float* d_scratch, void* ws, size_t ws_bytes, void* hip_stream);

/* Diagnostics for benchmarks (not thread-safe, off by default).  tp_layer_profile(1) makes every
 * GEMM launched by this library (inside tp_layer_fwd / tp_layer_bwd / tp_layer_gemm) be bracketed by
 * two HIP events on its launch stream and restarts the record; tp_layer_profile(0) stops.
 * tp_layer_profile_read waits for the recorded launches (at most 4096, in launch order), writes their
 * durations in milliseconds to ms_out[0..*count) and restarts the record.  ms_out is HOST memory. */
int tp_layer_profile(int enable);
int tp_layer_profile_read(float* ms_out, int capacity, int* count);

/* Tuning overrides, for tests (which run every kernel variant through them) and for tuning; process-wide, not
 * thread-safe, and they must not change between a workspace-size query and the call it sizes.  name:
 *   "gemm_tile"   force one GEMM tile variant (0..7) for every bf16 GEMM
 *   "gemm_shares" force the number of K shares of every bf16 GEMM
 *   "gemm_band"   force the band height of the GEMM tile order
 *   "gemm_force"  "MxNxK@ab=v[:shares];..." plans for single shapes (a, b = 1 where A, B has K contiguous)
 *   "attn_chunk"  chunk length of attention strips in 64-row tile steps (0: never cut)
 *   "side_chains" 2 or 3: chains of a backward pass under TPL_SIDE_STREAM (3: the two weight gradients that depend on
 *                 nothing computed in the pass, dW_dn and dW_o, on a second library stream); unset: chosen by size
 *   "fuse_colsum" 1: the bias gradients db_qkv, db_up are one more output row of the weight-gradient GEMM whenever
 *                 its kernel supports that; 0 (default): they come from the column-sum kernels (measured inside the
 *                 whole step the two are equal on one stream and the fused form is 0.4 % slower on two chains)
 * value: decimal text; NULL or "" returns the option to "let the library choose".  TPL_EINVAL for an unknown
 * name or a value that does not parse. */
int tp_layer_set_option(const char* name, const char* value);

/* Static description of a status code. */
const char* tp_layer_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* TP_LAYER_H */
