"""Plain float64 definition of one tensor-parallel rank's share of a transformer layer.

TEST INFRASTRUCTURE ONLY: imported by tests, by the smoke check and by the
benchmark's cpu_baseline leg; never by the product path.

What is computed (speed-optimised distribution, App. F.1 of the paper; the same
split as Megatron-LM): in both the self-attention block and the MLP block the
first linear layer is split over its output channels and the second over its
input channels, so the activation between them is sharded and everything else is
replicated; each rank's second linear therefore yields a partial sum that the
ranks would all-reduce.  Here the partial sums are returned as they are.  The
bias of a row-split linear lives on one rank only ((W1 x1 + b) + W2 x2 = W x + b,
caption of Fig. 7); the same rank also adds the residual.  Attention is softmax
attention over the local heads, causal or not (Sec. I.4 constructor arguments);
the activation is the exact (erf) GeLU; dropout is 0.

Every function is the textbook definition written with numpy in float64:
matmul is the only library primitive used as a step, there is no tiling, no
online softmax, no fusion.  Inputs are whatever values the caller passes
(float32 or bfloat16-representable numbers widened to float64); nothing is
rounded in between.

Pins (tests/test_oracle_*.py): central finite differences for every gradient,
sum-over-ranks equals unsharded layer, explicit triple-loop evaluation on tiny
inputs, softmax/causality invariants, closed forms for attention and GeLU, and a
T=1 cross-check against PyTorch's CPU autograd.  No function here is unpinned.

Layout conventions (row-major, y = x W + b, W is [in, out]):
  unsharded: Wqkv [H,3,nh,dh], bqkv [3,nh,dh], Wo [nh*dh,H], bo [H], Wup [H,I], bup [I],
             Wdn [I,H], bdn [H]
  rank r of T: w_qkv [H, 3*nl*dh] with columns ordered (q|k|v, local head, dh),
               w_o [nl*dh, H], w_up [H, Il], w_dn [Il, H]; b_o, b_dn are the full
               vectors and are used only when `row_epilogue` is set.
"""
import numpy as np
from scipy.special import erf as _erf

_F = np.float64


def shard_params(g, T, r):
    """Rank r's share of the unsharded parameters `g` (App. F.1: first linears by output
    channel = by head / MLP column, second linears by input channel = by row)."""
    Wqkv = np.asarray(g["Wqkv"])
    H, three, nh, dh = Wqkv.shape
    assert three == 3 and nh % T == 0
    nl = nh // T
    I = np.asarray(g["Wup"]).shape[1]
    assert I % T == 0
    Il = I // T
    hs = slice(r * nl, (r + 1) * nl)
    return {
        "w_qkv": np.ascontiguousarray(Wqkv[:, :, hs, :]).reshape(H, 3 * nl * dh),
        "b_qkv": np.ascontiguousarray(np.asarray(g["bqkv"])[:, hs, :]).reshape(3 * nl * dh),
        "w_o": np.ascontiguousarray(np.asarray(g["Wo"])[r * nl * dh:(r + 1) * nl * dh, :]),
        "b_o": np.asarray(g["bo"]),
        "w_up": np.ascontiguousarray(np.asarray(g["Wup"])[:, r * Il:(r + 1) * Il]),
        "b_up": np.ascontiguousarray(np.asarray(g["bup"])[r * Il:(r + 1) * Il]),
        "w_dn": np.ascontiguousarray(np.asarray(g["Wdn"])[r * Il:(r + 1) * Il, :]),
        "b_dn": np.asarray(g["bdn"]),
    }


def gelu(u):
    """Exact GeLU: u * Phi(u), Phi the standard normal CDF."""
    u = np.asarray(u, _F)
    return 0.5 * u * (1.0 + _erf(u / np.sqrt(2.0)))


def gelu_grad(u):
    """d/du [u Phi(u)] = Phi(u) + u phi(u)."""
    u = np.asarray(u, _F)
    Phi = 0.5 * (1.0 + _erf(u / np.sqrt(2.0)))
    phi = np.exp(-0.5 * u * u) / np.sqrt(2.0 * np.pi)
    return Phi + u * phi


def _split_heads(qkv, B, S, nl, dh):
    """[B*S, 3*nl*dh] with columns (q|k|v, head, dh) -> three [B, nl, S, dh] arrays."""
    t = qkv.reshape(B, S, 3, nl, dh)
    return (t[:, :, 0].transpose(0, 2, 1, 3), t[:, :, 1].transpose(0, 2, 1, 3),
            t[:, :, 2].transpose(0, 2, 1, 3))


def _scores(Q, K, causal):
    """Scaled logits and the boolean 'may attend' mask (key j <= query i when causal)."""
    dh = Q.shape[-1]
    S = Q.shape[-2]
    sc = np.matmul(Q, K.transpose(0, 1, 3, 2)) / np.sqrt(_F(dh))
    allowed = np.ones((S, S), dtype=bool)
    if causal:
        allowed = np.tril(allowed)
    return sc, allowed


def attention_fwd(Q, K, V, causal):
    """Softmax attention per (batch, head). Q,K,V [B,nl,S,dh] -> O [B,nl,S,dh], P [B,nl,S,S], LSE [B,nl,S]."""
    Q, K, V = (np.asarray(a, _F) for a in (Q, K, V))
    sc, allowed = _scores(Q, K, causal)
    sc = np.where(allowed, sc, -np.inf)
    mx = sc.max(axis=-1, keepdims=True)
    ex = np.exp(sc - mx)                     # masked entries: exp(-inf) = 0
    den = ex.sum(axis=-1, keepdims=True)
    P = ex / den
    O = np.matmul(P, V)
    LSE = (mx + np.log(den))[..., 0]
    return O, P, LSE


def attention_bwd(Q, K, V, P, dO):
    """Gradients of O = P V, P = softmax(Q K^T / sqrt(dh)) w.r.t. Q, K, V (masked entries have P = 0)."""
    Q, K, V, P, dO = (np.asarray(a, _F) for a in (Q, K, V, P, dO))
    dh = Q.shape[-1]
    dV = np.matmul(P.transpose(0, 1, 3, 2), dO)
    dP = np.matmul(dO, V.transpose(0, 1, 3, 2))
    D = (dP * P).sum(axis=-1, keepdims=True)          # equals rowsum(dO * O)
    dS = P * (dP - D)
    dQ = np.matmul(dS, K) / np.sqrt(_F(dh))
    dK = np.matmul(dS.transpose(0, 1, 3, 2), Q) / np.sqrt(_F(dh))
    return dQ, dK, dV


def layer_fwd(x_a, x_m, p, B, S, nl, dh, causal, row_epilogue):
    """Forward of one rank's shard.

    x_a, x_m [B*S, H]: replicated inputs of the attention block and of the MLP block.
    Returns (y_a, y_m, saved): y_* [B*S, H] are the partial sums before the all-reduce;
    saved holds QKV, O, LSE, U, G (and P, for the oracle's own backward).
    """
    x_a = np.asarray(x_a, _F)
    x_m = np.asarray(x_m, _F)
    w = {k: np.asarray(v, _F) for k, v in p.items()}
    e = 1.0 if row_epilogue else 0.0
    M = B * S
    QKV = x_a @ w["w_qkv"] + w["b_qkv"]
    Q, K, V = _split_heads(QKV, B, S, nl, dh)
    Oh, P, LSE = attention_fwd(Q, K, V, causal)
    O = Oh.transpose(0, 2, 1, 3).reshape(M, nl * dh)
    y_a = O @ w["w_o"]
    if row_epilogue:
        y_a = y_a + e * (w["b_o"] + x_a)
    U = x_m @ w["w_up"] + w["b_up"]
    G = gelu(U)
    y_m = G @ w["w_dn"]
    if row_epilogue:
        y_m = y_m + e * (w["b_dn"] + x_m)
    saved = {"QKV": QKV, "O": O, "LSE": LSE, "U": U, "G": G, "P": P}
    return y_a, y_m, saved


def layer_bwd(x_a, x_m, p, dy_a, dy_m, saved, B, S, nl, dh, causal, row_epilogue):
    """Backward of one rank's shard for the scalar <y_a, dy_a> + <y_m, dy_m>.

    Returns a dict with dx_a, dx_m (partial input gradients before the backward
    all-reduce), dw_qkv, db_qkv, dw_o, dw_up, db_up, dw_dn and, when row_epilogue,
    db_o and db_dn.
    """
    x_a, x_m, dy_a, dy_m = (np.asarray(a, _F) for a in (x_a, x_m, dy_a, dy_m))
    w = {k: np.asarray(v, _F) for k, v in p.items()}
    M = B * S
    out = {}
    # MLP block: y_m = gelu(x_m W_up + b_up) W_dn (+ b_dn + x_m)
    dG = dy_m @ w["w_dn"].T
    out["dw_dn"] = saved["G"].T @ dy_m
    dU = dG * gelu_grad(saved["U"])
    out["dw_up"] = x_m.T @ dU
    out["db_up"] = dU.sum(axis=0)
    out["dx_m"] = dU @ w["w_up"].T
    # attention block: y_a = O W_o (+ b_o + x_a)
    dO = dy_a @ w["w_o"].T
    out["dw_o"] = saved["O"].T @ dy_a
    Q, K, V = _split_heads(saved["QKV"], B, S, nl, dh)
    dOh = dO.reshape(B, S, nl, dh).transpose(0, 2, 1, 3)
    dQ, dK, dV = attention_bwd(Q, K, V, saved["P"], dOh)
    dQKV = np.stack([a.transpose(0, 2, 1, 3) for a in (dQ, dK, dV)], axis=2).reshape(M, 3 * nl * dh)
    out["dQKV"] = dQKV
    out["dw_qkv"] = x_a.T @ dQKV
    out["db_qkv"] = dQKV.sum(axis=0)
    out["dx_a"] = dQKV @ w["w_qkv"].T
    if row_epilogue:
        out["db_dn"] = dy_m.sum(axis=0)
        out["db_o"] = dy_a.sum(axis=0)
        out["dx_m"] = out["dx_m"] + dy_m
        out["dx_a"] = out["dx_a"] + dy_a
    return out


def full_layer_fwd(x_a, x_m, g, B, S, causal):
    """The unsharded layer: the T = 1 case with biases and residual applied."""
    nh, dh = np.asarray(g["Wqkv"]).shape[2:]
    return layer_fwd(x_a, x_m, shard_params(g, 1, 0), B, S, nh, dh, causal, True)


def full_layer_bwd(x_a, x_m, g, dy_a, dy_m, saved, B, S, causal):
    nh, dh = np.asarray(g["Wqkv"]).shape[2:]
    return layer_bwd(x_a, x_m, shard_params(g, 1, 0), dy_a, dy_m, saved, B, S, nh, dh, causal, True)


def max_rel_err(got, ref):
    """max|got - ref| / max|ref| over a tensor (the parity metric)."""
    got = np.asarray(got, _F)
    ref = np.asarray(ref, _F)
    den = np.abs(ref).max()
    num = np.abs(got - ref).max() if got.size else 0.0
    return float(num / den) if den > 0 else float(num)


# ------------------------------------------------------------------------------------------------
# Replicated LayerNorm around the shard (speed-optimised mode keeps layer normalisation undistributed,
# Sec. I.1; epsilon and the pre/post placement are constructor arguments in Sec. I.4).  The normalised
# tensor is the residual sum z = a + b (b optional); statistics are over the hidden dimension with the
# biased variance, as in the usual definition of layer normalisation.
# Pins: finite differences, zero-mean/unit-variance rows, shift invariance, PyTorch's F.layer_norm.
# ------------------------------------------------------------------------------------------------
def layernorm_fwd(a, b, gamma, beta, eps):
    """z = a (+ b); y = (z - mean) / sqrt(var + eps) * gamma + beta.  Returns y, z, mean [M], rstd [M]."""
    z = np.asarray(a, _F) + (0.0 if b is None else np.asarray(b, _F))
    mean = z.mean(axis=1)
    var = ((z - mean[:, None]) ** 2).mean(axis=1)
    rstd = 1.0 / np.sqrt(var + _F(eps))
    zh = (z - mean[:, None]) * rstd[:, None]
    y = zh * np.asarray(gamma, _F) + np.asarray(beta, _F)
    return y, z, mean, rstd


def layernorm_bwd(dy, z, mean, rstd, gamma):
    """Gradients of y w.r.t. z (the same for a and b), gamma and beta."""
    dy, z, gamma = np.asarray(dy, _F), np.asarray(z, _F), np.asarray(gamma, _F)
    zh = (z - np.asarray(mean, _F)[:, None]) * np.asarray(rstd, _F)[:, None]
    g = dy * gamma
    dz = (g - g.mean(axis=1, keepdims=True) - zh * (g * zh).mean(axis=1, keepdims=True)) * np.asarray(rstd, _F)[:, None]
    return dz, (dy * zh).sum(axis=0), dy.sum(axis=0)
