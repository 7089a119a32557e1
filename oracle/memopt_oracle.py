"""Plain float64 definition of one rank's local compute in the memory-optimised distribution.

TEST INFRASTRUCTURE ONLY: imported by tests, by the smoke check and by the
benchmark's cpu_baseline leg; never by the product path.

What is computed (memory-optimised distribution, App. F.2 of the paper): every
linear layer of the transformer layer is split over its INPUT channels, so rank r
holds the channel slice x[:, r] of each replicated-in-speed-mode activation and the
matching rows of every weight matrix; its product is a full-width partial sum, and
a reduce-scatter (sum over ranks, rank i keeps output slice i) stands where the
speed-optimised mode has an all-reduce.  Layer normalisation is distributed as
well: each rank forms the first and second moments (sum x, sum x^2) of its channel
slice per token, the moments are all-reduced (two scalars per token), and every
rank then normalises its own slice with the global mean and variance
("ApplyLayerNorm").  The backward pass of that decomposition needs two more
per-token scalars (sum dy*gamma, sum dy*gamma*xhat) summed over ranks.  The
collectives themselves are the caller's; `reduce_scatter` and `all_reduce` below
are their definitions, used by the tests to put T simulated ranks together.

Each function is the definition written out with numpy in float64; matmul is the
only library primitive used as a step.

The paper's figures of this mode are missing from its text, so the order of the
pieces inside a block is a reading: pre-normalised
blocks, y = x + Block(LN(x)), with the bias of an input-split linear (and the
residual) added once, after the reduce-scatter, by the rank that keeps that slice.

Pins (tests/test_oracle_memopt.py): moments + ApplyLayerNorm on T slices equals the
textbook layer normalisation of the full rows (np.mean / np.var) and PyTorch's
F.layer_norm; the sliced backward equals central finite differences of the full-row
normalisation; T simulated ranks joined by the collectives equal the unsharded
reference layer, forward and backward (finite differences on the unsharded one);
bias+GeLU closed forms; this module's own attention (`_attention`, `_attention_bwd`)
against the scalar definition by plain loops, a hand-computed two-key case that fixes
the 1/sqrt(dh) scale and the mask diagonal, PyTorch's CPU scaled_dot_product_attention
with autograd, and the speed-optimised oracle's attention; `reference_layer_fwd` against
the pre-normalised layer written with PyTorch's CPU operators; planted mistakes (no
scale, mask without the diagonal, a wrong dK, a post-normalised reference) each make a
pin fail.  No function here is unpinned.
"""
import numpy as np
from scipy.special import erf as _erf

_F = np.float64


# ---- distributed layer normalisation (App. F.2, second paragraph) --------------------------------
def ln_local_moments(x_loc):
    """Per-token first and second moments of this rank's channel slice: [M, 2] = (sum x, sum x^2)."""
    x = np.asarray(x_loc, _F)
    return np.stack([x.sum(axis=1), (x * x).sum(axis=1)], axis=1)


def ln_stats(total_moments, H, eps):
    """Global mean and 1/sqrt(var + eps) per token from the all-reduced moments over all H channels."""
    t = np.asarray(total_moments, _F)
    mean = t[:, 0] / H
    var = t[:, 1] / H - mean * mean
    return mean, 1.0 / np.sqrt(var + _F(eps))


def ln_apply_fwd(x_loc, mean, rstd, gamma_loc, beta_loc):
    """ApplyLayerNorm: element-wise normalisation of the local slice with the global statistics."""
    xh = (np.asarray(x_loc, _F) - np.asarray(mean, _F)[:, None]) * np.asarray(rstd, _F)[:, None]
    return xh * np.asarray(gamma_loc, _F) + np.asarray(beta_loc, _F)


def ln_apply_bwd_sums(dy_loc, x_loc, mean, rstd, gamma_loc):
    """Per-token local sums the backward needs from every rank: [M, 2] = (sum dy*gamma, sum dy*gamma*xhat)."""
    dy, g = np.asarray(dy_loc, _F), np.asarray(gamma_loc, _F)
    xh = (np.asarray(x_loc, _F) - np.asarray(mean, _F)[:, None]) * np.asarray(rstd, _F)[:, None]
    return np.stack([(dy * g).sum(axis=1), (dy * g * xh).sum(axis=1)], axis=1)


def ln_apply_bwd(dy_loc, x_loc, mean, rstd, gamma_loc, total_sums, H):
    """dx for the local slice given the all-reduced sums; dgamma, dbeta of the local channels."""
    dy, g = np.asarray(dy_loc, _F), np.asarray(gamma_loc, _F)
    rs = np.asarray(rstd, _F)[:, None]
    xh = (np.asarray(x_loc, _F) - np.asarray(mean, _F)[:, None]) * rs
    t = np.asarray(total_sums, _F)
    dx = (dy * g - t[:, 0:1] / H - xh * t[:, 1:2] / H) * rs
    return dx, (dy * xh).sum(axis=0), dy.sum(axis=0)


# ---- input-split linear (App. F.2, first paragraph) -----------------------------------------------
def linear_part_fwd(x_loc, w_rows):
    """Full-width partial product of the local input slice [M, Ks] with the matching weight rows [Ks, N]."""
    return np.asarray(x_loc, _F) @ np.asarray(w_rows, _F)


def linear_part_bwd(x_loc, w_rows, dy_full):
    """Given the all-gathered output gradient [M, N]: dx for the local slice, dW for the local rows."""
    dy = np.asarray(dy_full, _F)
    return dy @ np.asarray(w_rows, _F).T, np.asarray(x_loc, _F).T @ dy


# ---- bias + GeLU on the reduce-scattered slice ---------------------------------------------------
def gelu(u):
    u = np.asarray(u, _F)
    return 0.5 * u * (1.0 + _erf(u / np.sqrt(2.0)))


def gelu_grad(u):
    u = np.asarray(u, _F)
    return 0.5 * (1.0 + _erf(u / np.sqrt(2.0))) + u * np.exp(-0.5 * u * u) / np.sqrt(2.0 * np.pi)


def slice_epilogue_fwd(part_slice, bias, resid=None, act="none"):
    """What a rank does to the slice it keeps after a reduce-scatter: v = slice + bias (+ residual);
    returns (v, gelu(v)) for act == "gelu" (v is kept for the backward) and (None, v) otherwise."""
    v = np.asarray(part_slice, _F) + np.asarray(bias, _F)
    if resid is not None:
        v = v + np.asarray(resid, _F)
    return (v, gelu(v)) if act == "gelu" else (None, v)


def slice_epilogue_bwd(dout, u=None, act="none"):
    """Gradient of the slice (and of the residual, when act is "none") and of the bias (column sums)."""
    d = np.asarray(dout, _F) * gelu_grad(u) if act == "gelu" else np.asarray(dout, _F)
    return d, d.sum(axis=0)


def bias_gelu_fwd(u_in, bias):
    """U = u_in + bias (kept for the backward), G = gelu(U)."""
    return slice_epilogue_fwd(u_in, bias, None, "gelu")


def bias_gelu_bwd(dg, u):
    """dU = dG * gelu'(U); dbias = column sums of dU."""
    return slice_epilogue_bwd(dg, u, "gelu")


# ---- the collectives (definitions; performed by the caller in a real run) -------------------------
def all_reduce(parts):
    return sum(np.asarray(p, _F) for p in parts)


def reduce_scatter(parts, r, T):
    """Sum over ranks, rank r keeps column slice r of T equal slices."""
    s = all_reduce(parts)
    w = s.shape[1] // T
    return s[:, r * w:(r + 1) * w]


# ---- attention on the local heads (softmax attention, as in the speed-optimised mode) -------------
def _attention(qkv_loc, B, S, nl, dh, causal):
    """qkv_loc [B*S, 3*nl*dh] with columns (q|k|v, head, dh) -> O [B*S, nl*dh], P [B,nl,S,S]."""
    t = np.asarray(qkv_loc, _F).reshape(B, S, 3, nl, dh).transpose(2, 0, 3, 1, 4)
    Q, K, V = t[0], t[1], t[2]
    sc = np.einsum("bhid,bhjd->bhij", Q, K) / np.sqrt(dh)
    if causal:
        sc = np.where(np.tril(np.ones((S, S), bool)), sc, -np.inf)
    sc = sc - sc.max(axis=-1, keepdims=True)
    P = np.exp(sc)
    P = P / P.sum(axis=-1, keepdims=True)
    O = np.einsum("bhij,bhjd->bhid", P, V)
    return O.transpose(0, 2, 1, 3).reshape(B * S, nl * dh), (Q, K, V, P)


def _attention_bwd(dO_loc, saved, B, S, nl, dh):
    Q, K, V, P = saved
    dO = np.asarray(dO_loc, _F).reshape(B, S, nl, dh).transpose(0, 2, 1, 3)
    dV = np.einsum("bhij,bhid->bhjd", P, dO)
    dP = np.einsum("bhid,bhjd->bhij", dO, V)
    dS = P * (dP - (dP * P).sum(axis=-1, keepdims=True))
    dQ = np.einsum("bhij,bhjd->bhid", dS, K) / np.sqrt(dh)
    dK = np.einsum("bhij,bhid->bhjd", dS, Q) / np.sqrt(dh)
    return np.stack([dQ, dK, dV]).transpose(1, 3, 0, 2, 4).reshape(B * S, 3 * nl * dh)


# ---- unsharded reference layer (pre-normalised blocks) -------------------------------------------
def reference_layer_fwd(x, g, B, S, causal, eps):
    """y1 = x + Attn(LN1(x)) ; y2 = y1 + MLP(LN2(y1)).  g: Wqkv [H, 3*nh*dh] with columns ordered
    (rank-independent) (q|k|v, head, dh), bqkv, Wo, bo, Wup, bup, Wdn, bdn, g1, b1, g2, b2, nh."""
    x = np.asarray(x, _F)
    H = x.shape[1]
    nh = g["nh"]
    dh = H // nh

    def ln(v, gamma, beta):
        mean = v.mean(axis=1, keepdims=True)
        var = ((v - mean) ** 2).mean(axis=1, keepdims=True)
        return (v - mean) / np.sqrt(var + eps) * gamma + beta

    h1 = ln(x, np.asarray(g["g1"], _F), np.asarray(g["b1"], _F))
    qkv = h1 @ np.asarray(g["Wqkv"], _F) + np.asarray(g["bqkv"], _F)
    o, _ = _attention(qkv, B, S, nh, dh, causal)
    y1 = x + o @ np.asarray(g["Wo"], _F) + np.asarray(g["bo"], _F)
    h2 = ln(y1, np.asarray(g["g2"], _F), np.asarray(g["b2"], _F))
    u = h2 @ np.asarray(g["Wup"], _F) + np.asarray(g["bup"], _F)
    y2 = y1 + gelu(u) @ np.asarray(g["Wdn"], _F) + np.asarray(g["bdn"], _F)
    return y2


def shard_reference_params(g, T, r):
    """Rank r's share in the memory-optimised mode: rows r of every weight matrix (input split), and the
    slices of biases and LayerNorm parameters that belong to the output slice the rank keeps after each
    reduce-scatter.  The QKV output columns are regrouped so that slice r holds the heads of rank r."""
    H = np.asarray(g["Wo"]).shape[1]
    nh = g["nh"]
    dh = H // nh
    nl = nh // T
    I = np.asarray(g["Wup"]).shape[1]
    Hs, Il = H // T, I // T
    rows = slice(r * Hs, (r + 1) * Hs)
    # full-width QKV columns ordered (rank, q|k|v, local head, dh)
    perm = np.arange(3 * nh * dh).reshape(3, T, nl, dh).transpose(1, 0, 2, 3).reshape(-1)
    qs = slice(r * 3 * nl * dh, (r + 1) * 3 * nl * dh)
    return {
        "w_qkv": np.asarray(g["Wqkv"], _F)[rows][:, perm], "b_qkv": np.asarray(g["bqkv"], _F)[perm][qs],
        "w_o": np.asarray(g["Wo"], _F)[r * nl * dh:(r + 1) * nl * dh], "b_o": np.asarray(g["bo"], _F)[rows],
        "w_up": np.asarray(g["Wup"], _F)[rows], "b_up": np.asarray(g["bup"], _F)[r * Il:(r + 1) * Il],
        "w_dn": np.asarray(g["Wdn"], _F)[r * Il:(r + 1) * Il], "b_dn": np.asarray(g["bdn"], _F)[rows],
        "g1": np.asarray(g["g1"], _F)[rows], "b1": np.asarray(g["b1"], _F)[rows],
        "g2": np.asarray(g["g2"], _F)[rows], "b2": np.asarray(g["b2"], _F)[rows],
    }


def memopt_layer_fwd(x_slices, shards, B, S, nl, dh, causal, eps):
    """T simulated ranks.  x_slices[r] = x[:, slice r]; returns the output slices and what backward needs."""
    T = len(shards)
    H = sum(np.asarray(v).shape[1] for v in x_slices)
    sv = {"x": [np.asarray(v, _F) for v in x_slices]}

    def dist_ln(xs, gk, bk, tag):
        tot = all_reduce([ln_local_moments(v) for v in xs])
        mean, rstd = ln_stats(tot, H, eps)
        sv[tag] = (mean, rstd)
        return [ln_apply_fwd(xs[r], mean, rstd, shards[r][gk], shards[r][bk]) for r in range(T)]

    h1 = dist_ln(sv["x"], "g1", "b1", "ln1")
    part = [linear_part_fwd(h1[r], shards[r]["w_qkv"]) for r in range(T)]
    qkv = [slice_epilogue_fwd(reduce_scatter(part, r, T), shards[r]["b_qkv"])[1] for r in range(T)]
    att = [_attention(qkv[r], B, S, nl, dh, causal) for r in range(T)]
    part = [linear_part_fwd(att[r][0], shards[r]["w_o"]) for r in range(T)]
    y1 = [slice_epilogue_fwd(reduce_scatter(part, r, T), shards[r]["b_o"], sv["x"][r])[1] for r in range(T)]
    h2 = dist_ln(y1, "g2", "b2", "ln2")
    part = [linear_part_fwd(h2[r], shards[r]["w_up"]) for r in range(T)]
    ug = [bias_gelu_fwd(reduce_scatter(part, r, T), shards[r]["b_up"]) for r in range(T)]
    part = [linear_part_fwd(ug[r][1], shards[r]["w_dn"]) for r in range(T)]
    y2 = [slice_epilogue_fwd(reduce_scatter(part, r, T), shards[r]["b_dn"], y1[r])[1] for r in range(T)]
    sv.update(h1=h1, att=att, y1=y1, h2=h2, ug=ug)
    return y2, sv


def memopt_layer_bwd(dy_slices, shards, sv, B, S, nl, dh):
    """Backward of memopt_layer_fwd.  A reduce-scatter becomes an all-gather of the slice gradients.
    Returns dx slices and, per rank, the gradients of its parameter shard."""
    T = len(shards)
    H = sum(v.shape[1] for v in sv["x"])
    gr = [dict() for _ in range(T)]

    def dist_ln_bwd(dh_, xs, tag, gk, gname, bname):
        mean, rstd = sv[tag]
        tot = all_reduce([ln_apply_bwd_sums(dh_[r], xs[r], mean, rstd, shards[r][gk]) for r in range(T)])
        out = []
        for r in range(T):
            dx, dgam, dbet = ln_apply_bwd(dh_[r], xs[r], mean, rstd, shards[r][gk], tot, H)
            gr[r][gname], gr[r][bname] = dgam, dbet
            out.append(dx)
        return out

    dy2 = [np.asarray(v, _F) for v in dy_slices]
    # MLP block
    full = np.concatenate(dy2, axis=1)                             # all-gather
    dg, dhid = [], []
    for r in range(T):
        _, gr[r]["b_dn"] = slice_epilogue_bwd(dy2[r])
        d_in, gr[r]["w_dn"] = linear_part_bwd(sv["ug"][r][1], shards[r]["w_dn"], full)
        dg.append(d_in)
    du = []
    for r in range(T):
        d, gr[r]["b_up"] = bias_gelu_bwd(dg[r], sv["ug"][r][0])
        du.append(d)
    full = np.concatenate(du, axis=1)
    for r in range(T):
        d_in, gr[r]["w_up"] = linear_part_bwd(sv["h2"][r], shards[r]["w_up"], full)
        dhid.append(d_in)
    dy1 = [dy2[r] + v for r, v in enumerate(dist_ln_bwd(dhid, sv["y1"], "ln2", "g2", "g2", "b2"))]
    # attention block
    full = np.concatenate(dy1, axis=1)
    d_o = []
    for r in range(T):
        _, gr[r]["b_o"] = slice_epilogue_bwd(dy1[r])
        d_in, gr[r]["w_o"] = linear_part_bwd(sv["att"][r][0], shards[r]["w_o"], full)
        d_o.append(d_in)
    dqkv = [_attention_bwd(d_o[r], sv["att"][r][1], B, S, nl, dh) for r in range(T)]
    full = np.concatenate(dqkv, axis=1)
    dh1 = []
    for r in range(T):
        _, gr[r]["b_qkv"] = slice_epilogue_bwd(dqkv[r])
        d_in, gr[r]["w_qkv"] = linear_part_bwd(sv["h1"][r], shards[r]["w_qkv"], full)
        dh1.append(d_in)
    dx = [dy1[r] + v for r, v in enumerate(dist_ln_bwd(dh1, sv["x"], "ln1", "g1", "g1", "b1"))]
    return dx, gr
