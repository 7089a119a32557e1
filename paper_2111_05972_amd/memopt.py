"""One rank's local compute in the memory-optimised distribution (App. F.2 of the paper), as the phases
between collectives.  Buffer management and call order only: every arithmetic step is a library call.

The layer is y1 = x + Attn(LN1(x)), y2 = y1 + MLP(LN2(y1)) with every linear split over its input channels.
A rank holds channel slice r of x, y1, y2 ([M, Hs], Hs = H / T), rows r of every weight matrix, and the
bias / LayerNorm slices of the outputs it keeps.  Each method below runs up to the next collective and
returns the tensor the caller must hand to it; the next method takes the collective's result:

    forward                                  collective on the returned tensor
    f0_moments(x)              -> sums       all-reduce
    f1_qkv_partial(tot)        -> [M, 3H]    reduce-scatter (slice r = heads of rank r)
    f2_attn_partial(qkv_in)    -> [M, H]     reduce-scatter
    f3_moments(o_in)           -> sums       all-reduce
    f4_up_partial(tot)         -> [M, I]     reduce-scatter
    f5_down_partial(u_in)      -> [M, H]     reduce-scatter
    f6_finish(d_in)            -> y2 slice
    backward
    b0_start(dy2)              -> dy2        all-gather
    b1_down(dy2_full)          -> dU slice   all-gather
    b2_up(dU_full)             -> sums       all-reduce
    b3_ln2(tot)                -> dy1        all-gather
    b4_attn(dy1_full)          -> dQKV slice all-gather
    b5_qkv(dqkv_full)          -> sums       all-reduce
    b6_ln1(tot)                -> dx slice
"""
import torch

from . import binding as B

_TORCH_DTYPE = {B.TPL_F32: torch.float32, B.TPL_BF16: torch.bfloat16}
PARAM_SHAPES = lambda H, Hs, Hl, I, Il: {  # noqa: E731
    "w_qkv": (Hs, 3 * H), "b_qkv": (3 * Hl,), "w_o": (Hl, H), "b_o": (Hs,), "w_up": (Hs, I), "b_up": (Il,),
    "w_dn": (Il, H), "b_dn": (Hs,), "g1": (Hs,), "b1": (Hs,), "g2": (Hs,), "b2": (Hs,)}


class MemOptRank:
    def __init__(self, hidden, heads, intermediate, tp_degree, seq, micro_batch, dtype, causal, eps=1e-5,
                 device="cuda"):
        T = tp_degree
        if hidden % heads or heads % T or hidden % T or intermediate % T:
            raise ValueError("hidden, heads and intermediate must divide by the tensor-parallel degree")
        self.H, self.I, self.T = hidden, intermediate, T
        self.dh, self.nl = hidden // heads, heads // T
        self.Hs, self.Hl, self.Il = hidden // T, (heads // T) * (hidden // heads), intermediate // T
        self.B, self.S, self.M = micro_batch, seq, seq * micro_batch
        self.dtype, self.td, self.causal, self.eps, self.dev = dtype, _TORCH_DTYPE[dtype], int(causal), eps, device
        M, H, I = self.M, hidden, intermediate
        e = lambda *s: torch.empty(*s, dtype=self.td, device=device)          # noqa: E731
        f = lambda *s: torch.empty(*s, dtype=torch.float32, device=device)     # noqa: E731
        self.sums = f(M, 2)
        self.mean1, self.rstd1, self.mean2, self.rstd2 = f(M), f(M), f(M), f(M)
        self.h1, self.h2, self.y1, self.y2 = e(M, self.Hs), e(M, self.Hs), e(M, self.Hs), e(M, self.Hs)
        self.part = e(M, max(3 * H, I))                                         # full-width partial products
        self.qkv, self.o = e(M, 3 * self.Hl), e(M, self.Hl)
        self.lse = f(self.B, self.nl, self.S)
        self.u, self.g = e(M, self.Il), e(M, self.Il)
        # backward
        self.dg, self.du, self.dhid = e(M, self.Il), e(M, self.Il), e(M, self.Hs)
        self.dy1, self.dx = e(M, self.Hs), e(M, self.Hs)
        self.d_o, self.dqkv, self.dsum = e(M, self.Hl), e(M, 3 * self.Hl), f(self.B, self.nl, self.S)
        Hs, Hl, Il = self.Hs, self.Hl, self.Il
        gemm_shapes = [(M, 3 * H, Hs), (M, H, Hl), (M, I, Hs), (M, H, Il),          # forward partial products
                       (M, Il, H), (Il, H, M), (M, Hs, I), (Hs, I, M),              # data and weight gradients
                       (M, Hl, H), (Hl, H, M), (M, Hs, 3 * H), (Hs, 3 * H, M)]
        nws = max(B.tp_layer_ln_apply_workspace_bytes(M, Hs),
                  B.tp_layer_slice_epilogue_workspace_bytes(M, max(3 * Hl, Il, Hs)),
                  max(B.tp_layer_gemm_workspace_bytes(dtype, *g) for g in gemm_shapes),
                  max(B.tp_layer_attn_workspace_bytes(dtype, self.B, self.S, self.nl, self.dh, self.causal, bwd)
                      for bwd in (False, True)), 256)
        self.ws = torch.empty(nws, dtype=torch.uint8, device=device)
        self.grads = {k: e(*s) for k, s in PARAM_SHAPES(H, self.Hs, self.Hl, I, self.Il).items()}

    # -- helpers ------------------------------------------------------------------------------------
    def _st(self):
        return torch.cuda.current_stream()

    def _part(self, n):
        return self.part.view(-1)[:self.M * n].view(self.M, n)

    def _gemm(self, ta, tb, M, N, K, A, Bm, C):
        B.tp_layer_gemm(self.dtype, ta, tb, M, N, K, A, Bm, C, ws=self.ws, stream=self._st())

    # -- forward --------------------------------------------------------------------------------------
    def f0_moments(self, p, x):
        self.p, self.x = p, x
        B.tp_layer_ln_moments(self.dtype, self.M, self.Hs, x, self.sums, stream=self._st())
        return self.sums

    def f1_qkv_partial(self, tot):
        st = self._st()
        B.tp_layer_ln_stats(self.M, self.H, self.eps, tot, self.mean1, self.rstd1, stream=st)
        B.tp_layer_ln_apply_fwd(self.dtype, self.M, self.Hs, self.x, self.mean1, self.rstd1, self.p["g1"],
                                self.p["b1"], self.h1, stream=st)
        out = self._part(3 * self.H)
        self._gemm(0, 0, self.M, 3 * self.H, self.Hs, self.h1, self.p["w_qkv"], out)
        return out

    def f2_attn_partial(self, qkv_in):
        st = self._st()
        B.tp_layer_slice_epilogue_fwd(self.dtype, B.TPL_ACT_NONE, self.M, 3 * self.Hl, qkv_in, self.p["b_qkv"], None,
                                      None, self.qkv, stream=st)
        B.tp_layer_attn_fwd(self.dtype, self.B, self.S, self.nl, self.dh, self.causal, self.qkv, self.o, self.lse,
                            ws=self.ws, stream=st)
        out = self._part(self.H)
        self._gemm(0, 0, self.M, self.H, self.Hl, self.o, self.p["w_o"], out)
        return out

    def f3_moments(self, o_in):
        st = self._st()
        B.tp_layer_slice_epilogue_fwd(self.dtype, B.TPL_ACT_NONE, self.M, self.Hs, o_in, self.p["b_o"], self.x, None,
                                      self.y1, stream=st)
        B.tp_layer_ln_moments(self.dtype, self.M, self.Hs, self.y1, self.sums, stream=st)
        return self.sums

    def f4_up_partial(self, tot):
        st = self._st()
        B.tp_layer_ln_stats(self.M, self.H, self.eps, tot, self.mean2, self.rstd2, stream=st)
        B.tp_layer_ln_apply_fwd(self.dtype, self.M, self.Hs, self.y1, self.mean2, self.rstd2, self.p["g2"],
                                self.p["b2"], self.h2, stream=st)
        out = self._part(self.I)
        self._gemm(0, 0, self.M, self.I, self.Hs, self.h2, self.p["w_up"], out)
        return out

    def f5_down_partial(self, u_in):
        B.tp_layer_slice_epilogue_fwd(self.dtype, B.TPL_ACT_GELU, self.M, self.Il, u_in, self.p["b_up"], None, self.u,
                                      self.g, stream=self._st())
        out = self._part(self.H)
        self._gemm(0, 0, self.M, self.H, self.Il, self.g, self.p["w_dn"], out)
        return out

    def f6_finish(self, d_in):
        B.tp_layer_slice_epilogue_fwd(self.dtype, B.TPL_ACT_NONE, self.M, self.Hs, d_in, self.p["b_dn"], self.y1, None,
                                      self.y2, stream=self._st())
        return self.y2

    # -- backward -------------------------------------------------------------------------------------
    def b0_start(self, dy2):
        self.dy2 = dy2
        B.tp_layer_slice_epilogue_bwd(self.dtype, B.TPL_ACT_NONE, self.M, self.Hs, dy2, None, None,
                                      self.grads["b_dn"], self.ws, stream=self._st())
        return dy2

    def b1_down(self, dy2_full):
        self._gemm(0, 1, self.M, self.Il, self.H, dy2_full, self.p["w_dn"], self.dg)
        self._gemm(1, 0, self.Il, self.H, self.M, self.g, dy2_full, self.grads["w_dn"])
        B.tp_layer_slice_epilogue_bwd(self.dtype, B.TPL_ACT_GELU, self.M, self.Il, self.dg, self.u, self.du,
                                      self.grads["b_up"], self.ws, stream=self._st())
        return self.du

    def b2_up(self, du_full):
        self._gemm(0, 1, self.M, self.Hs, self.I, du_full, self.p["w_up"], self.dhid)
        self._gemm(1, 0, self.Hs, self.I, self.M, self.h2, du_full, self.grads["w_up"])
        B.tp_layer_ln_apply_bwd_sums(self.dtype, self.M, self.Hs, self.dhid, self.y1, self.mean2, self.rstd2,
                                     self.p["g2"], self.sums, stream=self._st())
        return self.sums

    def b3_ln2(self, tot):
        st = self._st()
        B.tp_layer_ln_apply_bwd(self.dtype, self.M, self.Hs, self.H, self.dhid, self.y1, self.mean2, self.rstd2,
                                self.p["g2"], tot, self.dy2, self.dy1, self.grads["g2"], self.grads["b2"], self.ws,
                                stream=st)
        B.tp_layer_slice_epilogue_bwd(self.dtype, B.TPL_ACT_NONE, self.M, self.Hs, self.dy1, None, None,
                                      self.grads["b_o"], self.ws, stream=st)
        return self.dy1

    def b4_attn(self, dy1_full):
        st = self._st()
        self._gemm(0, 1, self.M, self.Hl, self.H, dy1_full, self.p["w_o"], self.d_o)
        self._gemm(1, 0, self.Hl, self.H, self.M, self.o, dy1_full, self.grads["w_o"])
        B.tp_layer_attn_bwd(self.dtype, self.B, self.S, self.nl, self.dh, self.causal, self.qkv, self.o, self.lse,
                            self.d_o, self.dqkv, self.dsum, ws=self.ws, stream=st)
        B.tp_layer_slice_epilogue_bwd(self.dtype, B.TPL_ACT_NONE, self.M, 3 * self.Hl, self.dqkv, None, None,
                                      self.grads["b_qkv"], self.ws, stream=st)
        return self.dqkv

    def b5_qkv(self, dqkv_full):
        self._gemm(0, 1, self.M, self.Hs, 3 * self.H, dqkv_full, self.p["w_qkv"], self.dhid)
        self._gemm(1, 0, self.Hs, 3 * self.H, self.M, self.h1, dqkv_full, self.grads["w_qkv"])
        B.tp_layer_ln_apply_bwd_sums(self.dtype, self.M, self.Hs, self.dhid, self.x, self.mean1, self.rstd1,
                                     self.p["g1"], self.sums, stream=self._st())
        return self.sums

    def b6_ln1(self, tot):
        B.tp_layer_ln_apply_bwd(self.dtype, self.M, self.Hs, self.H, self.dhid, self.x, self.mean1, self.rstd1,
                                self.p["g1"], tot, self.dy1, self.dx, self.grads["g1"], self.grads["b1"], self.ws,
                                stream=self._st())
        return self.dx
