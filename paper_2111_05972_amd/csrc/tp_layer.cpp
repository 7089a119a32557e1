// C-ABI entry points: descriptor validation, buffer layouts, and the order in which the kernels of
// one tensor-parallel rank's forward and backward pass are enqueued (App. F.1 of the paper).
#include "../../include/tp_layer.h"

#include <algorithm>
#include <cstdlib>
#include <cstring>

#include "kernels.h"

using namespace tpl;

// ---- tuning overrides (see Options in kernels.h) -------------------------------------------------------------------
namespace tpl {
namespace {
bool parse_int(const char* v, int unset, int lo, int hi, int* out) {
    if (!v || !*v) { *out = unset; return true; }
    char* end = nullptr;
    const long x = strtol(v, &end, 10);
    if (end == v || *end != 0 || x < lo || x > hi) return false;
    *out = (int)x;
    return true;
}
Options& mutable_options() {
    static Options opt = [] {
        Options o;                                      // the environment is read here, once per process
        parse_int(getenv("TPL_GEMM_TILE"), -1, 0, 63, &o.gemm_tile);
        parse_int(getenv("TPL_GEMM_SHARES"), 0, 0, 64, &o.gemm_shares);
        parse_int(getenv("TPL_GEMM_BAND"), 0, 0, 1 << 20, &o.gemm_band);
        parse_int(getenv("TPL_ATTN_CHUNK"), -1, 0, 1 << 16, &o.attn_chunk);
        if (const char* f = getenv("TPL_GEMM_FORCE")) { strncpy(o.gemm_force, f, sizeof(o.gemm_force) - 1); }
        return o;
    }();
    return opt;
}
}  // namespace
const Options& options() { return mutable_options(); }
bool set_option(const char* name, const char* value) {
    if (!name) return false;
    Options& o = mutable_options();
    bool ok = false;
    if (!strcmp(name, "gemm_tile")) ok = parse_int(value, -1, 0, 63, &o.gemm_tile);
    else if (!strcmp(name, "gemm_shares")) ok = parse_int(value, 0, 0, 64, &o.gemm_shares);
    else if (!strcmp(name, "gemm_band")) ok = parse_int(value, 0, 0, 1 << 20, &o.gemm_band);
    else if (!strcmp(name, "attn_chunk")) ok = parse_int(value, -1, 0, 1 << 16, &o.attn_chunk);
    else if (!strcmp(name, "fuse_colsum")) ok = parse_int(value, 0, 0, 1, &o.fuse_colsum);
    else if (!strcmp(name, "side_chains")) ok = parse_int(value, 0, 2, 3, &o.side_chains);
    else if (!strcmp(name, "gemm_force")) {
        const char* v = value ? value : "";
        if (strlen(v) < sizeof(o.gemm_force)) { strcpy(o.gemm_force, v); ok = true; }
    }
    if (ok) ++o.generation;
    return ok;
}
}  // namespace tpl

namespace {

constexpr size_t ALIGN = 256;
inline size_t up(size_t x) { return (x + ALIGN - 1) / ALIGN * ALIGN; }

// Resolved sizes of a valid descriptor.
struct Dims {
    int64_t H, nh, dh, I, T, r, S, B, M, nl, Hl, Il;
    int dtype;
    size_t esz;
    bool causal, row_epi, side_stream;
};

int resolve(const tp_layer_desc* d, Dims* o) {
    if (!d) return TPL_EINVAL;
    if (d->hidden <= 0 || d->heads <= 0 || d->tp_degree <= 0 || d->seq <= 0 || d->micro_batch <= 0)
        return TPL_EINVAL;
    if (d->head_dim < 0 || d->intermediate < 0) return TPL_EINVAL;
    if (d->dtype != TPL_F32 && d->dtype != TPL_BF16) return TPL_EINVAL;
    if (d->flags & ~(uint32_t)(TPL_CAUSAL | TPL_ROW_EPILOGUE | TPL_SIDE_STREAM)) return TPL_EINVAL;
    if (d->tp_rank < 0 || d->tp_rank >= d->tp_degree) return TPL_EINVAL;
    Dims x;
    x.H = d->hidden; x.nh = d->heads; x.T = d->tp_degree; x.r = d->tp_rank;
    x.S = d->seq; x.B = d->micro_batch;
    if (x.H % x.nh) return TPL_EINVAL;
    x.dh = d->head_dim ? d->head_dim : x.H / x.nh;
    if (x.dh * x.nh != x.H) return TPL_EINVAL;
    x.I = d->intermediate ? d->intermediate : 4 * x.H;
    if (x.nh % x.T || x.I % x.T) return TPL_EINVAL;
    x.M = x.B * x.S; x.nl = x.nh / x.T; x.Hl = x.nl * x.dh; x.Il = x.I / x.T;
    x.dtype = d->dtype; x.esz = d->dtype == TPL_F32 ? 4 : 2;
    x.causal = d->flags & TPL_CAUSAL; x.row_epi = d->flags & TPL_ROW_EPILOGUE;
    x.side_stream = d->flags & TPL_SIDE_STREAM;
    if (x.M > (int64_t)1 << 24 || x.H > (int64_t)1 << 20 || x.I > (int64_t)1 << 24) return TPL_EUNSUPPORTED;
    if (x.dh > 256) return TPL_EUNSUPPORTED;
    // 16-byte rows for every matrix the kernels touch
    if (x.dtype == TPL_BF16 && (x.H % 8 || x.Hl % 8 || x.Il % 8)) return TPL_EUNSUPPORTED;
    if (x.dtype == TPL_F32 && (x.H % 4 || x.Hl % 4 || x.Il % 4)) return TPL_EUNSUPPORTED;
    if (o) *o = x;
    return TPL_OK;
}

void saved_layout(const Dims& x, tp_layer_saved_layout* L) {
    size_t off = 0;
    L->qkv = off; off += up((size_t)x.M * 3 * x.Hl * x.esz);
    L->o = off;   off += up((size_t)x.M * x.Hl * x.esz);
    L->lse = off; off += up((size_t)x.B * x.nl * x.S * sizeof(float));
    L->u = off;   off += up((size_t)x.M * x.Il * x.esz);
    L->g = off;   off += up((size_t)x.M * x.Il * x.esz);
    L->total = off;
}

size_t gemm_ws(int dtype, int64_t M, int64_t N, int64_t K) {
    return dtype == TPL_BF16 ? up(gemm_bf16_workspace_bytes(M, N, K)) : 0;
}

// Backward scratch: dU, dO, dQKV, D, and per chain (attention, MLP) column-sum partials and GEMM scratch.
struct BwdWs { size_t du, d_o, dqkv, dsum, colsum, colsum2, gemm, gemm2, gemm3, gemm_each, attn, attn_bytes, total; };

// Float partials of attention strips cut into chunks: inside a layer pass only when TPL_ATTN_CHUNK forces a chunk
// length (own_chunking stays 0: see attn_bf16.hip), so normally 0.
size_t attn_ws(const Dims& x, bool bwd) {
    AttnArgs a{};
    a.dtype = x.dtype; a.B = (int)x.B; a.S = (int)x.S; a.nl = (int)x.nl; a.dh = (int)x.dh; a.causal = x.causal;
    if (x.dtype != BF16 || !attn_bf16_supported(a)) return 0;
    return up(attn_bf16_workspace_bytes(a, bwd));
}

size_t fwd_gemm_ws(const Dims& x) {
    size_t g = 0;
    g = std::max(g, gemm_ws(x.dtype, x.M, 3 * x.Hl, x.H));
    g = std::max(g, gemm_ws(x.dtype, x.M, x.H, x.Hl));
    g = std::max(g, gemm_ws(x.dtype, x.M, x.Il, x.H));
    g = std::max(g, gemm_ws(x.dtype, x.M, x.H, x.Il));
    return std::max(g, ALIGN);
}
size_t fwd_ws_total(const Dims& x) { return 2 * fwd_gemm_ws(x) + attn_ws(x, false); }

void bwd_layout(const Dims& x, BwdWs* W) {
    size_t off = 0;
    W->du = off;   off += up((size_t)x.M * x.Il * x.esz);
    W->d_o = off;  off += up((size_t)x.M * x.Hl * x.esz);
    W->dqkv = off; off += up((size_t)x.M * 3 * x.Hl * x.esz);
    W->dsum = off; off += up((size_t)x.B * x.nl * x.S * sizeof(float));
    int64_t nmax = std::max(std::max(x.Il, 3 * x.Hl), x.H);
    W->colsum = off; off += up(colsum_scratch_bytes(x.M, nmax));
    W->colsum2 = off; off += up(colsum_scratch_bytes(x.M, nmax));
    size_t g = fwd_gemm_ws(x);   // dgrad shapes are the forward shapes with N and K swapped
    g = std::max(g, gemm_ws(x.dtype, x.M, x.Hl, x.H));
    g = std::max(g, gemm_ws(x.dtype, x.M, x.H, 3 * x.Hl));
    g = std::max(g, gemm_ws(x.dtype, x.Il, x.H, x.M));
    g = std::max(g, gemm_ws(x.dtype, x.H, x.Il, x.M));
    g = std::max(g, gemm_ws(x.dtype, x.Hl, x.H, x.M));
    g = std::max(g, gemm_ws(x.dtype, x.H, 3 * x.Hl, x.M));
    W->gemm_each = g;
    W->gemm = off; off += g;
    W->gemm2 = off; off += g;
    W->gemm3 = off; off += g;      // the two weight gradients that depend on nothing computed in the pass (third chain)
    W->attn_bytes = attn_ws(x, true);
    W->attn = off; off += W->attn_bytes;
    W->total = off;
}

inline bool misaligned(const void* p) { return ((uintptr_t)p & 15u) != 0; }

// Diagnostic timing of GEMM launches with HIP events on the launch stream (off by default).
struct GemmProfile {
    static constexpr int CAP = 4096;
    bool on = false;
    int n = 0;
    hipEvent_t start[CAP], stop[CAP];
    bool created[CAP] = {};
} g_prof;

// The attention block and the MLP block of one pass share no tensor (each has its own input, output and
// gradients).  By default both are enqueued on the caller's stream, in the order written.  With TPL_SIDE_STREAM in
// the descriptor's flags they are enqueued as two chains: the attention chain on the caller's stream and the MLP
// chain on a second stream that the library creates once per device (default priority, non-blocking).  The second
// stream is forked from the caller's stream and joined back to it with events, so the caller sees one pass on its
// stream and the host never waits.  What the overlap can buy: tiles of one chain fill the compute units the other
// leaves idle (a GEMM whose tile count is below the number of compute units, the attention kernels, the start and
// end of every kernel).  Per-GEMM timing (tp_layer_profile) keeps everything on the caller's stream.
struct SideStream {
    hipStream_t stream = nullptr;
    hipEvent_t fork = nullptr, join = nullptr;
    int state = 0;       // 0 = not tried, 1 = ready, -1 = unavailable
};
constexpr int MAX_DEVICES = 64;
constexpr int MAX_SIDE = 2;
SideStream g_side[MAX_DEVICES][MAX_SIDE];

// Returns the stream for the second chain, already waiting for everything enqueued on s so far; s itself when
// the second stream is not used.
hipStream_t side_fork(hipStream_t s, bool wanted, int which = 0) {
    if (!wanted || g_prof.on) return s;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return s;
    SideStream& ss = g_side[dev][which];
    if (ss.state == 0) {
        ss.state = (hipStreamCreateWithFlags(&ss.stream, hipStreamNonBlocking) == hipSuccess &&
                    hipEventCreateWithFlags(&ss.fork, hipEventDisableTiming) == hipSuccess &&
                    hipEventCreateWithFlags(&ss.join, hipEventDisableTiming) == hipSuccess) ? 1 : -1;
    }
    if (ss.state != 1) return s;
    if (hipEventRecord(ss.fork, s) != hipSuccess || hipStreamWaitEvent(ss.stream, ss.fork, 0) != hipSuccess) return s;
    return ss.stream;
}
// Makes s wait for everything enqueued on the second stream.
int side_join(hipStream_t s, hipStream_t s2, int which = 0) {
    if (s2 == s) return TPL_OK;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return TPL_EHIP;
    SideStream& ss = g_side[dev][which];
    if (hipEventRecord(ss.join, s2) != hipSuccess || hipStreamWaitEvent(s, ss.join, 0) != hipSuccess) return TPL_EHIP;
    return TPL_OK;
}
// A pass that fails after the fork still joins: the caller's stream must not run ahead of work already enqueued
// on the second stream that touches the caller's buffers.
struct SideJoin {
    hipStream_t s, s2;
    int which = 0;
    bool done = false;
    int finish() { done = true; return side_join(s, s2, which); }
    ~SideJoin() { if (!done) side_join(s, s2, which); }
};

int run_gemm(GemmArgs& g) {
    hipError_t e;
    int slot = -1;
    if (g_prof.on && g_prof.n < GemmProfile::CAP) {
        slot = g_prof.n++;
        if (!g_prof.created[slot]) {
            if (hipEventCreate(&g_prof.start[slot]) != hipSuccess || hipEventCreate(&g_prof.stop[slot]) != hipSuccess)
                return TPL_EHIP;
            g_prof.created[slot] = true;
        }
        if (hipEventRecord(g_prof.start[slot], g.stream) != hipSuccess) return TPL_EHIP;
    }
    g.colsum_done = false;
    if (g.dtype == BF16 && gemm_bf16_supported(g)) e = gemm_bf16(g, &g.colsum_done);
    else e = gemm_simple(g);
    if (slot >= 0 && hipEventRecord(g_prof.stop[slot], g.stream) != hipSuccess) return TPL_EHIP;
    return e == hipSuccess ? TPL_OK : TPL_EHIP;
}

int run_attn(AttnArgs& a, bool bwd) {
    hipError_t e;
    if (a.dtype == BF16 && attn_bf16_supported(a)) e = bwd ? attn_bf16_bwd(a) : attn_bf16_fwd(a);
    else e = bwd ? attn_simple_bwd(a) : attn_simple_fwd(a);
    return e == hipSuccess ? TPL_OK : TPL_EHIP;
}

// Scratch handed to every GEMM of one entry-point call.
struct GemmScratch { void* ws; size_t bytes; hipStream_t stream; };

GemmArgs mk(const Dims& x, int ta, int tb, int64_t M, int64_t N, int64_t K, const void* A,
            const void* B, void* C, GemmScratch& sc) {
    void* ws = sc.ws; size_t ws_bytes = sc.bytes; hipStream_t s = sc.stream;
    GemmArgs g{};
    g.dtype = x.dtype; g.trans_a = ta; g.trans_b = tb; g.M = M; g.N = N; g.K = K;
    g.A = A; g.B = B; g.C = C; g.epi = EPI_NONE; g.ws = ws; g.ws_bytes = ws_bytes; g.stream = s;
    return g;
}

// Forward kernels in order.  With row_parallel == false the two row-parallel GEMMs (whose outputs the
// backward pass never reads) are skipped: that is the recomputation done in checkpoint mode.
int fwd_impl(const Dims& x, const tp_layer_params* p, const void* x_attn, const void* x_mlp, void* y_attn,
             void* y_mlp, void* saved, void* ws, size_t ws_bytes, hipStream_t s, bool row_parallel) {
    int rc;
    tp_layer_saved_layout L;
    saved_layout(x, &L);
    char* sv = (char*)saved;
    void *qkv = sv + L.qkv, *o = sv + L.o, *u = sv + L.u, *g = sv + L.g;
    float* lse = (float*)(sv + L.lse);
    // each chain has its own half of the GEMM scratch
    const size_t half = fwd_gemm_ws(x);
    hipStream_t s2 = side_fork(s, x.side_stream);
    SideJoin sj{s, s2};
    GemmScratch sc{ws, half, s}, sc2{(char*)ws + half, half, s2};

    // MLP block (second chain): column-parallel up-projection + GeLU, row-parallel down-projection
    GemmArgs g4 = mk(x, 0, 0, x.M, x.Il, x.H, x_mlp, p->w_up, g, sc2);
    g4.bias = p->b_up; g4.aux = u; g4.epi = EPI_GELU;
    if ((rc = run_gemm(g4))) return rc;
    if (row_parallel) {
        GemmArgs g5 = mk(x, 0, 0, x.M, x.H, x.Il, g, p->w_dn, y_mlp, sc2);
        if (x.row_epi) { g5.bias = p->b_dn; g5.resid = x_mlp; }
        if ((rc = run_gemm(g5))) return rc;
    }
    // attention block: column-parallel fused QKV, attention on the local heads, row-parallel out-proj
    GemmArgs g1 = mk(x, 0, 0, x.M, 3 * x.Hl, x.H, x_attn, p->w_qkv, qkv, sc);
    g1.bias = p->b_qkv;
    if ((rc = run_gemm(g1))) return rc;
    AttnArgs at{};
    at.dtype = x.dtype; at.B = (int)x.B; at.S = (int)x.S; at.nl = (int)x.nl; at.dh = (int)x.dh;
    at.causal = x.causal; at.qkv = qkv; at.o = o; at.lse = lse; at.stream = s;
    at.ws_bytes = attn_ws(x, false);
    at.ws = at.ws_bytes ? (char*)ws + 2 * half : nullptr;
    if ((rc = run_attn(at, false))) return rc;
    if (row_parallel) {
        GemmArgs g3 = mk(x, 0, 0, x.M, x.H, x.Hl, o, p->w_o, y_attn, sc);
        if (x.row_epi) { g3.bias = p->b_o; g3.resid = x_attn; }
        if ((rc = run_gemm(g3))) return rc;
    }
    return sj.finish();
}

// Argument checks shared by the entry points: NULL pointers, then alignment.  `row_parallel`: the forward pass
// runs its two row-parallel GEMMs (they need b_o, b_dn on the epilogue rank); the recomputation of checkpoint
// mode does not.
int fwd_check(const Dims& x, const tp_layer_params* p, const void* x_attn, const void* x_mlp, const void* ws,
              bool row_parallel) {
    if (!p || !x_attn || !x_mlp || !ws) return TPL_EINVAL;
    if (!p->w_qkv || !p->b_qkv || !p->w_o || !p->w_up || !p->b_up || !p->w_dn) return TPL_EINVAL;
    if (row_parallel && x.row_epi && (!p->b_o || !p->b_dn)) return TPL_EINVAL;
    const void* ptrs[] = {x_attn, x_mlp, ws, p->w_qkv, p->b_qkv, p->w_o, p->b_o, p->w_up, p->b_up, p->w_dn, p->b_dn};
    for (const void* q : ptrs) if (misaligned(q)) return TPL_EALIGN;
    return TPL_OK;
}

int bwd_check(const Dims& x, const tp_layer_params* p, const void* x_attn, const void* x_mlp, const void* dy_attn,
              const void* dy_mlp, const tp_layer_grads* gr, const void* dx_attn, const void* dx_mlp, const void* ws) {
    if (!p || !gr || !x_attn || !x_mlp || !dy_attn || !dy_mlp || !dx_attn || !dx_mlp || !ws) return TPL_EINVAL;
    if (!p->w_qkv || !p->w_o || !p->w_up || !p->w_dn) return TPL_EINVAL;
    if (!gr->dw_qkv || !gr->db_qkv || !gr->dw_o || !gr->dw_up || !gr->db_up || !gr->dw_dn) return TPL_EINVAL;
    if (x.row_epi && (!gr->db_o || !gr->db_dn)) return TPL_EINVAL;
    const void* ptrs[] = {x_attn, x_mlp, dy_attn, dy_mlp, dx_attn, dx_mlp, ws, p->w_qkv, p->w_o,
                          p->w_up, p->w_dn, gr->dw_qkv, gr->db_qkv, gr->dw_o, gr->db_o, gr->dw_up,
                          gr->db_up, gr->dw_dn, gr->db_dn};
    for (const void* q : ptrs) if (misaligned(q)) return TPL_EALIGN;
    return TPL_OK;
}

// Backward kernels in order (arguments already checked, ws large enough).
int bwd_impl(const Dims& x, const tp_layer_params* p, const void* x_attn, const void* x_mlp, const void* dy_attn,
             const void* dy_mlp, const void* saved, const tp_layer_grads* gr, void* dx_attn, void* dx_mlp, void* ws,
             hipStream_t s) {
    int rc;
    BwdWs W;
    bwd_layout(x, &W);
    tp_layer_saved_layout L;
    saved_layout(x, &L);
    const char* sv = (const char*)saved;
    const void *qkv = sv + L.qkv, *o = sv + L.o, *u = sv + L.u, *g = sv + L.g;
    const float* lse = (const float*)(sv + L.lse);
    char* w = (char*)ws;
    void *du = w + W.du, *d_o = w + W.d_o, *dqkv = w + W.dqkv;
    float *dsum = (float*)(w + W.dsum), *cs = (float*)(w + W.colsum), *cs2 = (float*)(w + W.colsum2);
    hipStream_t s2 = side_fork(s, x.side_stream);
    SideJoin sj{s, s2};
    // dW_dn and dW_o need only the pass's inputs and saved activations: they can form a third chain on a stream of
    // their own (option side_chains = 2 or 3 forces the number of chains)
    // (measured inside whole steps: -4 % at the RoBERTa-large shard and -2 % at the BERT-large one, whose GEMMs leave
    // compute units idle; +1 to +2 % at the 10B and GPT-3 shards, whose GEMMs fill the chip and only get in each other's
    // way; left to itself the library takes three chains below 45 GFLOP per weight gradient)
    const int chains = options().side_chains ? options().side_chains
                                             : (2.0 * (double)x.Il * (double)x.H * (double)x.M < 45.0e9 ? 3 : 2);
    hipStream_t s3 = chains >= 3 ? side_fork(s, x.side_stream, 1) : nullptr;
    SideJoin sj3{s, s3 ? s3 : s, 1};
    GemmScratch sc{w + W.gemm, W.gemm_each, s}, sc2{w + W.gemm2, W.gemm_each, s2};
    GemmScratch sc3a{w + W.gemm3, W.gemm_each, s3 ? s3 : s2}, sc3b{w + W.gemm3, W.gemm_each, s3 ? s3 : s};

    // MLP block (second chain).  dU = (dy_m W_dn^T) * gelu'(U) in one GEMM epilogue.
    GemmArgs b5 = mk(x, 0, 1, x.M, x.Il, x.H, dy_mlp, p->w_dn, du, sc2);
    b5.aux = const_cast<void*>(u); b5.epi = EPI_DGELU;
    if ((rc = run_gemm(b5))) return rc;
    GemmArgs w5 = mk(x, 1, 0, x.Il, x.H, x.M, g, dy_mlp, gr->dw_dn, s3 ? sc3a : sc2);
    w5.c_streaming = true;                   // the weight gradient is not read again in this pass
    if ((rc = run_gemm(w5))) return rc;
    GemmArgs w4 = mk(x, 1, 0, x.H, x.Il, x.M, x_mlp, du, gr->dw_up, sc2);
    w4.c_streaming = true;
    w4.colsum_b = gr->db_up;                 // db_up = column sums of dU: one more output row of this GEMM where it can
    if ((rc = run_gemm(w4))) return rc;
    if (!w4.colsum_done && colsum(x.dtype, x.M, x.Il, du, gr->db_up, cs2, s2) != hipSuccess) return TPL_EHIP;
    GemmArgs d4 = mk(x, 0, 1, x.M, x.H, x.Il, du, p->w_up, dx_mlp, sc2);
    if (x.row_epi) d4.resid = dy_mlp;
    if ((rc = run_gemm(d4))) return rc;
    if (x.row_epi && colsum(x.dtype, x.M, x.H, dy_mlp, gr->db_dn, cs2, s2) != hipSuccess) return TPL_EHIP;

    // attention block
    GemmArgs d3 = mk(x, 0, 1, x.M, x.Hl, x.H, dy_attn, p->w_o, d_o, sc);
    if ((rc = run_gemm(d3))) return rc;
    GemmArgs w3 = mk(x, 1, 0, x.Hl, x.H, x.M, o, dy_attn, gr->dw_o, s3 ? sc3b : sc);
    w3.c_streaming = true;
    if ((rc = run_gemm(w3))) return rc;
    if (x.row_epi && colsum(x.dtype, x.M, x.H, dy_attn, gr->db_o, cs, s) != hipSuccess) return TPL_EHIP;
    AttnArgs at{};
    at.dtype = x.dtype; at.B = (int)x.B; at.S = (int)x.S; at.nl = (int)x.nl; at.dh = (int)x.dh;
    at.causal = x.causal; at.qkv = qkv; at.o = const_cast<void*>(o); at.lse = const_cast<float*>(lse);
    at.d_o = d_o; at.dqkv = dqkv; at.dsum = dsum; at.stream = s;
    at.ws_bytes = W.attn_bytes;
    at.ws = W.attn_bytes ? w + W.attn : nullptr;
    if ((rc = run_attn(at, true))) return rc;
    GemmArgs w1 = mk(x, 1, 0, x.H, 3 * x.Hl, x.M, x_attn, dqkv, gr->dw_qkv, sc);
    w1.c_streaming = true;
    w1.colsum_b = gr->db_qkv;
    if ((rc = run_gemm(w1))) return rc;
    if (!w1.colsum_done && colsum(x.dtype, x.M, 3 * x.Hl, dqkv, gr->db_qkv, cs, s) != hipSuccess) return TPL_EHIP;
    GemmArgs d1 = mk(x, 0, 1, x.M, x.H, 3 * x.Hl, dqkv, p->w_qkv, dx_attn, sc);
    if (x.row_epi) d1.resid = dy_attn;
    if ((rc = run_gemm(d1))) return rc;
    if ((rc = sj3.finish())) { return rc; }
    return sj.finish();
}
}  // namespace

extern "C" {

int tp_layer_validate(const tp_layer_desc* desc) { return resolve(desc, nullptr); }

size_t tp_layer_saved_bytes(const tp_layer_desc* desc) {
    Dims x;
    if (resolve(desc, &x) != TPL_OK) return 0;
    tp_layer_saved_layout L;
    saved_layout(x, &L);
    return L.total;
}

int tp_layer_saved_offsets(const tp_layer_desc* desc, tp_layer_saved_layout* out) {
    Dims x;
    int rc = resolve(desc, &x);
    if (rc != TPL_OK) return rc;
    if (!out) return TPL_EINVAL;
    saved_layout(x, out);
    return TPL_OK;
}

size_t tp_layer_workspace_bytes(const tp_layer_desc* desc, int bwd) {
    Dims x;
    if (resolve(desc, &x) != TPL_OK) return 0;
    if (!bwd) return fwd_ws_total(x);
    BwdWs W;
    bwd_layout(x, &W);
    return W.total;
}

int tp_layer_fwd(const tp_layer_desc* desc, const tp_layer_params* p, const void* x_attn,
                 const void* x_mlp, void* y_attn, void* y_mlp, void* saved, void* ws,
                 size_t ws_bytes, void* hip_stream) {
    Dims x;
    int rc = resolve(desc, &x);
    if (rc != TPL_OK) return rc;
    if ((rc = fwd_check(x, p, x_attn, x_mlp, ws, true))) return rc;
    if (!y_attn || !y_mlp || !saved) return TPL_EINVAL;
    if (misaligned(y_attn) || misaligned(y_mlp) || misaligned(saved)) return TPL_EALIGN;
    if (ws_bytes < fwd_ws_total(x)) return TPL_EWORKSPACE;
    return fwd_impl(x, p, x_attn, x_mlp, y_attn, y_mlp, saved, ws, ws_bytes, (hipStream_t)hip_stream, true);
}

int tp_layer_bwd(const tp_layer_desc* desc, const tp_layer_params* p, const void* x_attn,
                 const void* x_mlp, const void* dy_attn, const void* dy_mlp, const void* saved,
                 const tp_layer_grads* gr, void* dx_attn, void* dx_mlp, void* ws, size_t ws_bytes,
                 void* hip_stream) {
    Dims x;
    int rc = resolve(desc, &x);
    if (rc != TPL_OK) return rc;
    if ((rc = bwd_check(x, p, x_attn, x_mlp, dy_attn, dy_mlp, gr, dx_attn, dx_mlp, ws))) return rc;
    if (!saved) return TPL_EINVAL;
    if (misaligned(saved)) return TPL_EALIGN;
    BwdWs W;
    bwd_layout(x, &W);
    if (ws_bytes < W.total) return TPL_EWORKSPACE;
    return bwd_impl(x, p, x_attn, x_mlp, dy_attn, dy_mlp, saved, gr, dx_attn, dx_mlp, ws, (hipStream_t)hip_stream);
}

size_t tp_layer_workspace_bytes_recompute(const tp_layer_desc* desc) {
    Dims x;
    if (resolve(desc, &x) != TPL_OK) return 0;
    tp_layer_saved_layout L;
    saved_layout(x, &L);
    BwdWs W;
    bwd_layout(x, &W);
    return up(L.total) + std::max(W.total, fwd_ws_total(x));
}

int tp_layer_bwd_recompute(const tp_layer_desc* desc, const tp_layer_params* p, const void* x_attn,
                           const void* x_mlp, const void* dy_attn, const void* dy_mlp,
                           const tp_layer_grads* gr, void* dx_attn, void* dx_mlp, void* ws, size_t ws_bytes,
                           void* hip_stream) {
    Dims x;
    int rc = resolve(desc, &x);
    if (rc != TPL_OK) return rc;
    // everything either pass needs is checked before the recomputed forward is enqueued
    if ((rc = fwd_check(x, p, x_attn, x_mlp, ws, false))) return rc;
    if ((rc = bwd_check(x, p, x_attn, x_mlp, dy_attn, dy_mlp, gr, dx_attn, dx_mlp, ws))) return rc;
    if (ws_bytes < tp_layer_workspace_bytes_recompute(desc)) return TPL_EWORKSPACE;
    tp_layer_saved_layout L;
    saved_layout(x, &L);
    char* saved = (char*)ws;
    char* rest = saved + up(L.total);
    const size_t rest_bytes = ws_bytes - up(L.total);
    // recompute QKV, O, LSE, U, G from the block inputs, then the ordinary backward
    rc = fwd_impl(x, p, x_attn, x_mlp, nullptr, nullptr, saved, rest, rest_bytes, (hipStream_t)hip_stream, false);
    if (rc != TPL_OK) return rc;
    return bwd_impl(x, p, x_attn, x_mlp, dy_attn, dy_mlp, saved, gr, dx_attn, dx_mlp, rest, (hipStream_t)hip_stream);
}

static int ln_check(int dtype, int64_t M, int64_t H) {
    if (dtype != TPL_F32 && dtype != TPL_BF16) return TPL_EINVAL;
    if (M <= 0 || H <= 0) return TPL_EINVAL;
    if (!ln_supported(H)) return TPL_EUNSUPPORTED;
    return TPL_OK;
}

size_t tp_layer_ln_workspace_bytes(int64_t M, int64_t H) {
    if (M <= 0 || H <= 0) return 0;
    return up(ln_scratch_bytes(M, H));
}

int tp_layer_ln_fwd(int dtype, int64_t M, int64_t H, const void* a, const void* b, const void* gamma,
                    const void* beta, float eps, void* z, void* y, float* mean, float* rstd, void* hip_stream) {
    int rc = ln_check(dtype, M, H);
    if (rc) return rc;
    if (!a || !gamma || !beta || !y || !mean || !rstd || !(eps >= 0.0f)) return TPL_EINVAL;
    const void* ptrs[] = {a, b, gamma, beta, z, y, mean, rstd};
    for (const void* q : ptrs) if (misaligned(q)) return TPL_EALIGN;
    LnArgs l{};
    l.dtype = dtype; l.M = M; l.H = H; l.a = a; l.b = b; l.gamma = gamma; l.beta = beta; l.eps = eps;
    l.z = z; l.y = y; l.mean = mean; l.rstd = rstd; l.stream = (hipStream_t)hip_stream;
    return ln_fwd(l) == hipSuccess ? TPL_OK : TPL_EHIP;
}

int tp_layer_ln_bwd(int dtype, int64_t M, int64_t H, const void* dy, const void* z, const float* mean,
                    const float* rstd, const void* gamma, void* dz, void* dgamma, void* dbeta, void* ws,
                    size_t ws_bytes, void* hip_stream) {
    int rc = ln_check(dtype, M, H);
    if (rc) return rc;
    if (!dy || !z || !mean || !rstd || !gamma || !dz || !dgamma || !dbeta || !ws) return TPL_EINVAL;
    const void* ptrs[] = {dy, z, mean, rstd, gamma, dz, dgamma, dbeta, ws};
    for (const void* q : ptrs) if (misaligned(q)) return TPL_EALIGN;
    if (ws_bytes < tp_layer_ln_workspace_bytes(M, H)) return TPL_EWORKSPACE;
    LnArgs l{};
    l.dtype = dtype; l.M = M; l.H = H; l.dy = dy; l.z = const_cast<void*>(z); l.mean = const_cast<float*>(mean);
    l.rstd = const_cast<float*>(rstd); l.gamma = gamma; l.dz = dz; l.dgamma = dgamma; l.dbeta = dbeta;
    l.partials = (float*)ws; l.stream = (hipStream_t)hip_stream;
    return ln_bwd(l) == hipSuccess ? TPL_OK : TPL_EHIP;
}

static int dist_check(int dtype, int64_t M, int64_t Hs) {
    if (dtype != TPL_F32 && dtype != TPL_BF16) return TPL_EINVAL;
    if (M <= 0 || Hs <= 0) return TPL_EINVAL;
    if (!ln_supported(Hs)) return TPL_EUNSUPPORTED;
    return TPL_OK;
}
static int hip_rc(hipError_t e) { return e == hipSuccess ? TPL_OK : TPL_EHIP; }

int tp_layer_ln_moments(int dtype, int64_t M, int64_t Hs, const void* x_loc, float* sums, void* hip_stream) {
    int rc = dist_check(dtype, M, Hs);
    if (rc) return rc;
    if (!x_loc || !sums) return TPL_EINVAL;
    if (misaligned(x_loc) || misaligned(sums)) return TPL_EALIGN;
    return hip_rc(ln_dist_moments(dtype, M, Hs, x_loc, sums, (hipStream_t)hip_stream));
}

int tp_layer_ln_stats(int64_t M, int64_t H, float eps, const float* totals, float* mean, float* rstd,
                      void* hip_stream) {
    if (M <= 0 || H <= 0 || !(eps >= 0.0f) || !totals || !mean || !rstd) return TPL_EINVAL;
    return hip_rc(ln_dist_stats(M, H, eps, totals, mean, rstd, (hipStream_t)hip_stream));
}

int tp_layer_ln_apply_fwd(int dtype, int64_t M, int64_t Hs, const void* x_loc, const float* mean,
                          const float* rstd, const void* gamma_loc, const void* beta_loc, void* y,
                          void* hip_stream) {
    int rc = dist_check(dtype, M, Hs);
    if (rc) return rc;
    if (!x_loc || !mean || !rstd || !gamma_loc || !beta_loc || !y) return TPL_EINVAL;
    const void* ptrs[] = {x_loc, gamma_loc, beta_loc, y};
    for (const void* q : ptrs) if (misaligned(q)) return TPL_EALIGN;
    return hip_rc(ln_dist_apply(dtype, M, Hs, x_loc, mean, rstd, gamma_loc, beta_loc, y, (hipStream_t)hip_stream));
}

int tp_layer_ln_apply_bwd_sums(int dtype, int64_t M, int64_t Hs, const void* dy, const void* x_loc,
                               const float* mean, const float* rstd, const void* gamma_loc, float* sums,
                               void* hip_stream) {
    int rc = dist_check(dtype, M, Hs);
    if (rc) return rc;
    if (!dy || !x_loc || !mean || !rstd || !gamma_loc || !sums) return TPL_EINVAL;
    const void* ptrs[] = {dy, x_loc, gamma_loc};
    for (const void* q : ptrs) if (misaligned(q)) return TPL_EALIGN;
    return hip_rc(ln_dist_bwd_sums(dtype, M, Hs, dy, x_loc, mean, rstd, gamma_loc, sums, (hipStream_t)hip_stream));
}

size_t tp_layer_ln_apply_workspace_bytes(int64_t M, int64_t Hs) {
    if (M <= 0 || Hs <= 0) return 0;
    return up(ln_dist_scratch_bytes(M, Hs));
}

int tp_layer_ln_apply_bwd(int dtype, int64_t M, int64_t Hs, int64_t H, const void* dy, const void* x_loc,
                          const float* mean, const float* rstd, const void* gamma_loc, const float* totals,
                          const void* dx_add, void* dx, void* dgamma_loc, void* dbeta_loc, void* ws,
                          size_t ws_bytes, void* hip_stream) {
    int rc = dist_check(dtype, M, Hs);
    if (rc) return rc;
    if (H < Hs) return TPL_EINVAL;
    if (!dy || !x_loc || !mean || !rstd || !gamma_loc || !totals || !dx || !dgamma_loc || !dbeta_loc || !ws)
        return TPL_EINVAL;
    const void* ptrs[] = {dy, x_loc, gamma_loc, dx_add, dx, dgamma_loc, dbeta_loc, ws};
    for (const void* q : ptrs) if (misaligned(q)) return TPL_EALIGN;
    if (ws_bytes < tp_layer_ln_apply_workspace_bytes(M, Hs)) return TPL_EWORKSPACE;
    return hip_rc(ln_dist_bwd_apply(dtype, M, Hs, H, dy, x_loc, mean, rstd, gamma_loc, totals, dx_add, dx,
                                    dgamma_loc, dbeta_loc, (float*)ws, (hipStream_t)hip_stream));
}

static int ew_check(int dtype, int64_t M, int64_t N) {
    if (dtype != TPL_F32 && dtype != TPL_BF16) return TPL_EINVAL;
    if (M <= 0 || N <= 0) return TPL_EINVAL;
    if (N % 8) return TPL_EUNSUPPORTED;
    return TPL_OK;
}

int tp_layer_slice_epilogue_fwd(int dtype, int act, int64_t M, int64_t N, const void* in, const void* bias,
                                const void* resid, void* u, void* out, void* hip_stream) {
    int rc = ew_check(dtype, M, N);
    if (rc) return rc;
    if (act != TPL_ACT_NONE && act != TPL_ACT_GELU) return TPL_EINVAL;
    if (!in || !bias || !out || (act == TPL_ACT_GELU && !u)) return TPL_EINVAL;
    const void* ptrs[] = {in, bias, resid, u, out};
    for (const void* q : ptrs) if (misaligned(q)) return TPL_EALIGN;
    return hip_rc(slice_epilogue_fwd(dtype, act == TPL_ACT_GELU, M, N, in, bias, resid, u, out,
                                     (hipStream_t)hip_stream));
}

size_t tp_layer_slice_epilogue_workspace_bytes(int64_t M, int64_t N) {
    if (M <= 0 || N <= 0) return 0;
    return up(colsum_scratch_bytes(M, N));
}

int tp_layer_slice_epilogue_bwd(int dtype, int act, int64_t M, int64_t N, const void* dout, const void* u,
                                void* din, void* dbias, void* ws, size_t ws_bytes, void* hip_stream) {
    int rc = ew_check(dtype, M, N);
    if (rc) return rc;
    if (act != TPL_ACT_NONE && act != TPL_ACT_GELU) return TPL_EINVAL;
    if (!dout || !dbias || !ws || (act == TPL_ACT_GELU && (!u || !din))) return TPL_EINVAL;
    const void* ptrs[] = {dout, u, din, dbias, ws};
    for (const void* q : ptrs) if (misaligned(q)) return TPL_EALIGN;
    if (ws_bytes < tp_layer_slice_epilogue_workspace_bytes(M, N)) return TPL_EWORKSPACE;
    hipStream_t s = (hipStream_t)hip_stream;
    const void* d = dout;
    if (act == TPL_ACT_GELU) {
        if (gelu_bwd(dtype, M, N, dout, u, din, s) != hipSuccess) return TPL_EHIP;
        d = din;
    }
    return hip_rc(colsum(dtype, M, N, d, dbias, (float*)ws, s));
}

size_t tp_layer_static_scratch_bytes(void) { return STATIC_SCRATCH_BYTES; }

int tp_layer_slice_epilogue_bwd_static(int dtype, int act, int64_t M, int64_t N, const void* dout, const void* u,
                                       void* din, void* dbias, void* hip_stream) {
    int rc = ew_check(dtype, M, N);
    if (rc) return rc;
    if (act != TPL_ACT_NONE && act != TPL_ACT_GELU) return TPL_EINVAL;
    if (!dout || !dbias || (act == TPL_ACT_GELU && (!u || !din))) return TPL_EINVAL;
    const void* ptrs[] = {dout, u, din, dbias};
    for (const void* q : ptrs) if (misaligned(q)) return TPL_EALIGN;
    // the column-sum partials must fit the static array: nothing is allocated here
    if (colsum_scratch_bytes(M, N) > STATIC_SCRATCH_BYTES) return TPL_EWORKSPACE;
    void* ws = nullptr;
    if (static_scratch(&ws) != hipSuccess) return TPL_EHIP;
    hipStream_t s = (hipStream_t)hip_stream;
    const void* d = dout;
    if (act == TPL_ACT_GELU) {
        if (gelu_bwd(dtype, M, N, dout, u, din, s) != hipSuccess) return TPL_EHIP;
        d = din;
    }
    // every partial the second stage reads is written by the first in the same call: nothing to clear
    return hip_rc(colsum(dtype, M, N, d, dbias, (float*)ws, s));
}

size_t tp_layer_gemm_workspace_bytes(int dtype, int64_t M, int64_t N, int64_t K) {
    if (M <= 0 || N <= 0 || K <= 0) return 0;
    return std::max(gemm_ws(dtype, M, N, K), ALIGN);
}

int tp_layer_gemm(int dtype, int trans_a, int trans_b, int64_t M, int64_t N, int64_t K,
                  const void* A, const void* B, void* C, const void* bias, const void* resid,
                  void* aux, int epi, void* ws, size_t ws_bytes, void* hip_stream) {
    if (dtype != TPL_F32 && dtype != TPL_BF16) return TPL_EINVAL;
    if (M <= 0 || N <= 0 || K <= 0 || !A || !B || !C || !ws) return TPL_EINVAL;
    if (epi != TPL_EPI_NONE && epi != TPL_EPI_GELU && epi != TPL_EPI_DGELU) return TPL_EINVAL;
    if (epi != TPL_EPI_NONE && !aux) return TPL_EINVAL;
    int64_t q = dtype == TPL_BF16 ? 8 : 4;
    if (M % q || N % q || K % q) return TPL_EUNSUPPORTED;
    const void* ptrs[] = {A, B, C, bias, resid, aux, ws};
    for (const void* pp : ptrs) if (misaligned(pp)) return TPL_EALIGN;
    if (ws_bytes < tp_layer_gemm_workspace_bytes(dtype, M, N, K)) return TPL_EWORKSPACE;
    GemmArgs g{};
    g.dtype = dtype; g.trans_a = trans_a != 0; g.trans_b = trans_b != 0; g.M = M; g.N = N; g.K = K;
    g.A = A; g.B = B; g.C = C; g.bias = bias; g.resid = resid; g.aux = aux; g.epi = epi;
    g.ws = ws; g.ws_bytes = ws_bytes; g.stream = (hipStream_t)hip_stream;
    return run_gemm(g);
}

static int attn_check(int dtype, int B, int S, int nl, int dh) {
    if (dtype != TPL_F32 && dtype != TPL_BF16) return TPL_EINVAL;
    if (B <= 0 || S <= 0 || nl <= 0 || dh <= 0) return TPL_EINVAL;
    if (dh > 256 || (int64_t)nl * dh % (dtype == TPL_BF16 ? 8 : 4)) return TPL_EUNSUPPORTED;
    return TPL_OK;
}

size_t tp_layer_attn_workspace_bytes(int dtype, int B, int S, int nl, int dh, int causal, int bwd) {
    if (attn_check(dtype, B, S, nl, dh)) return 0;
    AttnArgs a{};
    a.dtype = dtype; a.B = B; a.S = S; a.nl = nl; a.dh = dh; a.causal = causal != 0; a.own_chunking = 1;
    if (dtype != BF16 || !attn_bf16_supported(a)) return 0;
    return up(attn_bf16_workspace_bytes(a, bwd != 0));
}

int tp_layer_attn_fwd(int dtype, int B, int S, int nl, int dh, int causal, const void* qkv, void* o,
                      float* lse, void* ws, size_t ws_bytes, void* hip_stream) {
    int rc = attn_check(dtype, B, S, nl, dh);
    if (rc) return rc;
    if (!qkv || !o || !lse) return TPL_EINVAL;
    if (misaligned(qkv) || misaligned(o) || misaligned(lse) || misaligned(ws)) return TPL_EALIGN;
    if (ws && ws_bytes < tp_layer_attn_workspace_bytes(dtype, B, S, nl, dh, causal, 0)) return TPL_EWORKSPACE;
    AttnArgs a{};
    a.dtype = dtype; a.B = B; a.S = S; a.nl = nl; a.dh = dh; a.causal = causal != 0;
    a.qkv = qkv; a.o = o; a.lse = lse; a.ws = ws; a.ws_bytes = ws_bytes; a.own_chunking = 1;
    a.stream = (hipStream_t)hip_stream;
    return run_attn(a, false);
}

int tp_layer_attn_bwd(int dtype, int B, int S, int nl, int dh, int causal, const void* qkv,
                      const void* o, const float* lse, const void* d_o, void* dqkv,
                      float* d_scratch, void* ws, size_t ws_bytes, void* hip_stream) {
    int rc = attn_check(dtype, B, S, nl, dh);
    if (rc) return rc;
    if (!qkv || !o || !lse || !d_o || !dqkv || !d_scratch) return TPL_EINVAL;
    const void* ptrs[] = {qkv, o, lse, d_o, dqkv, d_scratch, ws};
    for (const void* pp : ptrs) if (misaligned(pp)) return TPL_EALIGN;
    if (ws && ws_bytes < tp_layer_attn_workspace_bytes(dtype, B, S, nl, dh, causal, 1)) return TPL_EWORKSPACE;
    AttnArgs a{};
    a.dtype = dtype; a.B = B; a.S = S; a.nl = nl; a.dh = dh; a.causal = causal != 0;
    a.qkv = qkv; a.o = const_cast<void*>(o); a.lse = const_cast<float*>(lse); a.d_o = d_o;
    a.dqkv = dqkv; a.dsum = d_scratch; a.ws = ws; a.ws_bytes = ws_bytes; a.own_chunking = 1;
    a.stream = (hipStream_t)hip_stream;
    return run_attn(a, true);
}

int tp_layer_set_option(const char* name, const char* value) {
    return set_option(name, value) ? TPL_OK : TPL_EINVAL;
}

int tp_layer_profile(int enable) {
    g_prof.on = enable != 0;
    g_prof.n = 0;
    return TPL_OK;
}

int tp_layer_profile_read(float* ms_out, int capacity, int* count) {
    if (!ms_out || !count || capacity < 0) return TPL_EINVAL;
    int n = g_prof.n < capacity ? g_prof.n : capacity;
    for (int i = 0; i < n; ++i) {
        if (hipEventSynchronize(g_prof.stop[i]) != hipSuccess) return TPL_EHIP;
        if (hipEventElapsedTime(&ms_out[i], g_prof.start[i], g_prof.stop[i]) != hipSuccess) return TPL_EHIP;
    }
    *count = n;
    g_prof.n = 0;
    return TPL_OK;
}

const char* tp_layer_strerror(int status) {
    switch (status) {
        case TPL_OK: return "ok";
        case TPL_EINVAL: return "invalid argument (null pointer, non-positive or non-dividing size)";
        case TPL_EUNSUPPORTED: return "valid layer but unsupported shape or dtype";
        case TPL_EWORKSPACE: return "workspace too small (for a *_static entry point: the problem needs more scratch than the library's static array holds)";
        case TPL_EALIGN: return "pointer not 16-byte aligned";
        case TPL_EHIP: return "HIP launch failed";
        default: return "unknown status";
    }
}

}  // extern "C"
