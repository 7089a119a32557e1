"""Pins for the CPU oracle: each test checks it against something other than itself.

Finite differences (every gradient), sum over ranks = unsharded layer (Fig. 7 caption and
App. F.1 of the paper), explicit loop evaluation of the definitions on tiny inputs,
softmax/causality invariants, closed forms, and PyTorch's CPU autograd for T = 1.
"""
import math

import numpy as np
import pytest

import oracle
from oracle import tp_layer_oracle as O


def tiny_problem(seed=0, H=16, nh=4, dh=4, I=24, S=5, B=2, scale=0.5):
    rng = np.random.default_rng(seed)
    g = {
        "Wqkv": rng.normal(0, scale, (H, 3, nh, dh)), "bqkv": rng.normal(0, scale, (3, nh, dh)),
        "Wo": rng.normal(0, scale, (nh * dh, H)), "bo": rng.normal(0, scale, (H,)),
        "Wup": rng.normal(0, scale, (H, I)), "bup": rng.normal(0, scale, (I,)),
        "Wdn": rng.normal(0, scale, (I, H)), "bdn": rng.normal(0, scale, (H,)),
    }
    M = B * S
    x = {k: rng.normal(0, 1.0, (M, H)) for k in ("x_a", "x_m", "dy_a", "dy_m")}
    return g, x, dict(H=H, nh=nh, dh=dh, I=I, S=S, B=B)


# ---------------------------------------------------------------- finite differences
@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("row_epilogue", [True, False])
def test_gradients_match_central_differences(causal, row_epilogue):
    g, x, d = tiny_problem(1)
    T, r = 2, 1
    nl = d["nh"] // T
    p = oracle.shard_params(g, T, r)

    def loss(xa, xm, pp):
        ya, ym, _ = oracle.layer_fwd(xa, xm, pp, d["B"], d["S"], nl, d["dh"], causal, row_epilogue)
        return float((ya * x["dy_a"]).sum() + (ym * x["dy_m"]).sum())

    _, _, saved = oracle.layer_fwd(x["x_a"], x["x_m"], p, d["B"], d["S"], nl, d["dh"], causal, row_epilogue)
    grads = oracle.layer_bwd(x["x_a"], x["x_m"], p, x["dy_a"], x["dy_m"], saved,
                             d["B"], d["S"], nl, d["dh"], causal, row_epilogue)
    h = 1e-5
    rng = np.random.default_rng(7)

    def check(name, arr, rebuild, n_samples=40):
        ana = grads[name]
        assert ana.shape == arr.shape
        flat = arr.reshape(-1)
        idxs = range(flat.size) if flat.size <= n_samples else rng.choice(flat.size, n_samples, replace=False)
        scale = np.abs(ana).max() + 1e-30
        for i in idxs:
            old = flat[i]
            flat[i] = old + h
            lp = loss(*rebuild())
            flat[i] = old - h
            lm = loss(*rebuild())
            flat[i] = old
            num = (lp - lm) / (2 * h)
            assert abs(num - ana.reshape(-1)[i]) <= 1e-6 * scale + 1e-8, (name, i, num, ana.reshape(-1)[i])

    xa, xm = x["x_a"].copy(), x["x_m"].copy()
    pp = {k: np.array(v, dtype=np.float64) for k, v in p.items()}
    rb = lambda: (xa, xm, pp)  # noqa: E731
    check("dx_a", xa, rb)
    check("dx_m", xm, rb)
    for gname, pname in [("dw_qkv", "w_qkv"), ("db_qkv", "b_qkv"), ("dw_o", "w_o"), ("dw_up", "w_up"),
                         ("db_up", "b_up"), ("dw_dn", "w_dn")]:
        check(gname, pp[pname], rb)
    if row_epilogue:
        check("db_o", pp["b_o"], rb)
        check("db_dn", pp["b_dn"], rb)
    else:
        assert "db_o" not in grads and "db_dn" not in grads
        # without the epilogue the row-parallel biases must not influence the output at all
        base = loss(xa, xm, pp)
        pp["b_o"] = pp["b_o"] + 3.0
        pp["b_dn"] = pp["b_dn"] - 2.0
        assert loss(xa, xm, pp) == base


# ---------------------------------------------------------------- rank-sum invariants
@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("T", [1, 2, 4])
def test_partials_sum_to_unsharded_layer(causal, T):
    g, x, d = tiny_problem(2)
    B, S, nh, dh = d["B"], d["S"], d["nh"], d["dh"]
    ya_f, ym_f, sv_f = oracle.full_layer_fwd(x["x_a"], x["x_m"], g, B, S, causal)
    gr_f = oracle.full_layer_bwd(x["x_a"], x["x_m"], g, x["dy_a"], x["dy_m"], sv_f, B, S, causal)
    full_shards = None
    ya = ym = dxa = dxm = 0.0
    for r in range(T):
        p = oracle.shard_params(g, T, r)
        e = (r == 0)           # bias of a row-split linear resides on tp_rank 0 only
        a, m, sv = oracle.layer_fwd(x["x_a"], x["x_m"], p, B, S, nh // T, dh, causal, e)
        gr = oracle.layer_bwd(x["x_a"], x["x_m"], p, x["dy_a"], x["dy_m"], sv, B, S, nh // T, dh, causal, e)
        ya, ym, dxa, dxm = ya + a, ym + m, dxa + gr["dx_a"], dxm + gr["dx_m"]
        # weight gradients of a shard are the shard of the unsharded weight gradients
        gfull = {"Wqkv": gr_f["dw_qkv"].reshape(d["H"], 3, nh, dh), "bqkv": gr_f["db_qkv"].reshape(3, nh, dh),
                 "Wo": gr_f["dw_o"], "bo": gr_f["db_o"], "Wup": gr_f["dw_up"], "bup": gr_f["db_up"],
                 "Wdn": gr_f["dw_dn"], "bdn": gr_f["db_dn"]}
        full_shards = oracle.shard_params(gfull, T, r)
        for k_sh, k_gr in [("w_qkv", "dw_qkv"), ("b_qkv", "db_qkv"), ("w_o", "dw_o"), ("w_up", "dw_up"),
                           ("b_up", "db_up"), ("w_dn", "dw_dn")]:
            np.testing.assert_allclose(gr[k_gr], full_shards[k_sh], rtol=1e-11, atol=1e-11)
        if e:
            np.testing.assert_allclose(gr["db_o"], gr_f["db_o"], rtol=1e-12, atol=1e-12)
            np.testing.assert_allclose(gr["db_dn"], gr_f["db_dn"], rtol=1e-12, atol=1e-12)
    for got, ref in [(ya, ya_f), (ym, ym_f), (dxa, gr_f["dx_a"]), (dxm, gr_f["dx_m"])]:
        np.testing.assert_allclose(got, ref, rtol=1e-11, atol=1e-11)


def test_shard_shapes_and_column_order():
    g, x, d = tiny_problem(3)
    T, r = 2, 1
    H, nh, dh, I = d["H"], d["nh"], d["dh"], d["I"]
    nl = nh // T
    p = oracle.shard_params(g, T, r)
    assert p["w_qkv"].shape == (H, 3 * nl * dh) and p["w_o"].shape == (nl * dh, H)
    assert p["w_up"].shape == (H, I // T) and p["w_dn"].shape == (I // T, H)
    # column c = (which, local head, d): q block first, then k, then v; heads r*nl.. of the global
    for which in range(3):
        for hl in range(nl):
            for dd in range(dh):
                c = which * nl * dh + hl * dh + dd
                assert np.array_equal(p["w_qkv"][:, c], g["Wqkv"][:, which, r * nl + hl, dd])
                assert p["b_qkv"][c] == g["bqkv"][which, r * nl + hl, dd]


# ---------------------------------------------------------------- explicit-loop definition
@pytest.mark.parametrize("causal", [True, False])
def test_forward_matches_scalar_loops(causal):
    """Evaluate the layer with Python scalar loops straight from the definitions."""
    g, x, d = tiny_problem(4, H=8, nh=2, dh=4, I=12, S=4, B=2)
    T, r = 2, 1
    B, S, H, nh, dh, I = d["B"], d["S"], d["H"], d["nh"], d["dh"], d["I"]
    nl, Il = nh // T, I // T
    for e in (False, True):
        p = oracle.shard_params(g, T, r)
        ya, ym, sv = oracle.layer_fwd(x["x_a"], x["x_m"], p, B, S, nl, dh, causal, e)
        ya2 = np.zeros((B * S, H))
        ym2 = np.zeros((B * S, H))
        for b in range(B):
            for hl in range(nl):
                hg = r * nl + hl
                q = [[sum(x["x_a"][b * S + s, k] * g["Wqkv"][k, 0, hg, dd] for k in range(H)) + g["bqkv"][0, hg, dd]
                      for dd in range(dh)] for s in range(S)]
                kk = [[sum(x["x_a"][b * S + s, k] * g["Wqkv"][k, 1, hg, dd] for k in range(H)) + g["bqkv"][1, hg, dd]
                       for dd in range(dh)] for s in range(S)]
                v = [[sum(x["x_a"][b * S + s, k] * g["Wqkv"][k, 2, hg, dd] for k in range(H)) + g["bqkv"][2, hg, dd]
                      for dd in range(dh)] for s in range(S)]
                for i in range(S):
                    js = [j for j in range(S) if (j <= i or not causal)]
                    logits = [sum(q[i][dd] * kk[j][dd] for dd in range(dh)) / math.sqrt(dh) for j in js]
                    mx = max(logits)
                    ex = [math.exp(l - mx) for l in logits]
                    den = sum(ex)
                    assert abs(sv["LSE"][b, hl, i] - (mx + math.log(den))) < 1e-12
                    for dd in range(dh):
                        o = sum(ex[t] / den * v[j][dd] for t, j in enumerate(js))
                        assert abs(sv["O"][b * S + i, hl * dh + dd] - o) < 1e-12
                        for n in range(H):
                            ya2[b * S + i, n] += o * g["Wo"][hg * dh + dd, n]
        for m in range(B * S):
            for c in range(Il):
                u = sum(x["x_m"][m, k] * g["Wup"][k, r * Il + c] for k in range(H)) + g["bup"][r * Il + c]
                ge = 0.5 * u * (1.0 + math.erf(u / math.sqrt(2.0)))
                assert abs(sv["U"][m, c] - u) < 1e-12 and abs(sv["G"][m, c] - ge) < 1e-12
                for n in range(H):
                    ym2[m, n] += ge * g["Wdn"][r * Il + c, n]
        if e:
            ya2 += g["bo"] + x["x_a"]
            ym2 += g["bdn"] + x["x_m"]
        np.testing.assert_allclose(ya, ya2, rtol=0, atol=1e-11)
        np.testing.assert_allclose(ym, ym2, rtol=0, atol=1e-11)


def test_attention_backward_matches_scalar_loops():
    rng = np.random.default_rng(5)
    B, nl, S, dh = 1, 2, 4, 3
    Q, K, V, dO = (rng.normal(size=(B, nl, S, dh)) for _ in range(4))
    for causal in (True, False):
        Oo, P, _ = oracle.attention_fwd(Q, K, V, causal)
        dQ, dK, dV = oracle.attention_bwd(Q, K, V, P, dO)
        for h in range(nl):
            dq = np.zeros((S, dh)); dk = np.zeros((S, dh)); dv = np.zeros((S, dh))
            for i in range(S):
                Di = sum(dO[0, h, i, d] * Oo[0, h, i, d] for d in range(dh))
                for j in range(S):
                    if causal and j > i:
                        assert P[0, h, i, j] == 0.0
                        continue
                    dp = sum(dO[0, h, i, d] * V[0, h, j, d] for d in range(dh))
                    ds = P[0, h, i, j] * (dp - Di)
                    for d in range(dh):
                        dq[i, d] += ds * K[0, h, j, d] / math.sqrt(dh)
                        dk[j, d] += ds * Q[0, h, i, d] / math.sqrt(dh)
                        dv[j, d] += P[0, h, i, j] * dO[0, h, i, d]
            np.testing.assert_allclose(dQ[0, h], dq, atol=1e-12)
            np.testing.assert_allclose(dK[0, h], dk, atol=1e-12)
            np.testing.assert_allclose(dV[0, h], dv, atol=1e-12)


# ---------------------------------------------------------------- softmax / causality invariants
@pytest.mark.parametrize("causal", [True, False])
def test_softmax_rows_and_mask(causal):
    rng = np.random.default_rng(6)
    Q, K, V = (rng.normal(size=(2, 3, 7, 8)) * 3 for _ in range(3))
    Oo, P, LSE = oracle.attention_fwd(Q, K, V, causal)
    np.testing.assert_allclose(P.sum(-1), 1.0, atol=1e-13)
    assert (P >= 0).all() and np.isfinite(LSE).all()
    if causal:
        iu = np.triu_indices(7, 1)
        assert (P[..., iu[0], iu[1]] == 0).all()
        np.testing.assert_allclose(Oo[:, :, 0], V[:, :, 0], atol=1e-14)   # first row sees only itself
    # LSE is the log of the sum of exp of the (allowed) logits
    sc = np.einsum("bhid,bhjd->bhij", Q, K) / math.sqrt(8)
    if causal:
        sc = np.where(np.tril(np.ones((7, 7), bool)), sc, -np.inf)
    np.testing.assert_allclose(LSE, np.log(np.exp(sc).sum(-1)), atol=1e-12)
    # adding a constant to every logit of a row (q -> q + c*u with K u = 1 impossible in general;
    # use K shifted by a common vector instead: changes each row's logits by q_i . delta) leaves P unchanged
    delta = rng.normal(size=(8,))
    _, P2, _ = oracle.attention_fwd(Q, K + delta, V, causal)
    np.testing.assert_allclose(P2, P, atol=1e-12)


def test_causality_of_whole_shard():
    g, x, d = tiny_problem(8, S=6)
    p = oracle.shard_params(g, 2, 0)
    B, S = d["B"], d["S"]
    ya, _, _ = oracle.layer_fwd(x["x_a"], x["x_m"], p, B, S, d["nh"] // 2, d["dh"], True, True)
    j = 3
    xa2 = x["x_a"].copy()
    xa2[0 * S + j] += 1.0
    ya2, _, _ = oracle.layer_fwd(xa2, x["x_m"], p, B, S, d["nh"] // 2, d["dh"], True, True)
    assert np.array_equal(ya2[:j], ya[:j])                  # earlier tokens of batch 0 untouched
    assert np.array_equal(ya2[S:], ya[S:])                  # other batch element untouched
    assert not np.allclose(ya2[j:S], ya[j:S])
    yb, _, _ = oracle.layer_fwd(xa2, x["x_m"], p, B, S, d["nh"] // 2, d["dh"], False, True)
    yb0, _, _ = oracle.layer_fwd(x["x_a"], x["x_m"], p, B, S, d["nh"] // 2, d["dh"], False, True)
    assert not np.allclose(yb[:j], yb0[:j])                 # bidirectional: earlier tokens do change


def test_attention_closed_forms():
    rng = np.random.default_rng(9)
    B, nl, S, dh = 2, 2, 6, 4
    K, V = rng.normal(size=(B, nl, S, dh)), rng.normal(size=(B, nl, S, dh))
    # one token: O = V
    O1, _, L1 = oracle.attention_fwd(K[:, :, :1], K[:, :, :1], V[:, :, :1], True)
    np.testing.assert_allclose(O1, V[:, :, :1], atol=1e-15)
    # zero queries: uniform weights -> mean (bidirectional) / prefix mean (causal), LSE = log(count)
    Z = np.zeros_like(K)
    Ob, _, Lb = oracle.attention_fwd(Z, K, V, False)
    np.testing.assert_allclose(Ob, np.broadcast_to(V.mean(2, keepdims=True), V.shape), atol=1e-14)
    np.testing.assert_allclose(Lb, math.log(S), atol=1e-14)
    Oc, _, Lc = oracle.attention_fwd(Z, K, V, True)
    pref = np.cumsum(V, axis=2) / np.arange(1, S + 1)[None, None, :, None]
    np.testing.assert_allclose(Oc, pref, atol=1e-14)
    np.testing.assert_allclose(Lc, np.broadcast_to(np.log(np.arange(1, S + 1)), Lc.shape), atol=1e-14)
    # bidirectional attention is equivariant to permuting the sequence
    Q = rng.normal(size=(B, nl, S, dh))
    perm = rng.permutation(S)
    Oa, _, _ = oracle.attention_fwd(Q, K, V, False)
    Op, _, _ = oracle.attention_fwd(Q[:, :, perm], K[:, :, perm], V[:, :, perm], False)
    np.testing.assert_allclose(Op, Oa[:, :, perm], atol=1e-13)


def test_scale_is_inverse_sqrt_head_dim():
    # two keys, logits differ by exactly sqrt(dh)*ln(3) before scaling -> weights 3/4, 1/4
    dh = 16
    q = np.zeros((1, 1, 1, dh)); q[..., 0] = 1.0
    K = np.zeros((1, 1, 2, dh)); K[0, 0, 0, 0] = math.sqrt(dh) * math.log(3.0)
    V = np.zeros((1, 1, 2, dh)); V[0, 0, 0, 0] = 1.0
    # non-causal with 1 query: build by hand through the softmax definition
    sc = (q @ K.transpose(0, 1, 3, 2)) / math.sqrt(dh)
    Q2 = np.concatenate([q, q], axis=2)
    O2, P2, _ = oracle.attention_fwd(Q2, K, V, False)
    np.testing.assert_allclose(P2[0, 0, 0], [0.75, 0.25], atol=1e-14)
    np.testing.assert_allclose(sc[0, 0, 0], [math.log(3.0), 0.0], atol=1e-14)


# ---------------------------------------------------------------- GeLU
def test_gelu_closed_forms():
    assert oracle.gelu(0.0) == 0.0
    assert oracle.gelu_grad(0.0) == 0.5
    u = np.linspace(-6, 6, 101)
    np.testing.assert_allclose(oracle.gelu(u) - oracle.gelu(-u), u, atol=1e-14)
    np.testing.assert_allclose(oracle.gelu(np.array([12.0, -12.0])), [12.0, 0.0], atol=1e-12)
    np.testing.assert_allclose(oracle.gelu_grad(np.array([12.0, -12.0])), [1.0, 0.0], atol=1e-12)
    ref = np.array([0.5 * t * (1 + math.erf(t / math.sqrt(2))) for t in u])
    np.testing.assert_allclose(oracle.gelu(u), ref, atol=1e-15)
    # Phi(1) from tables
    assert abs(oracle.gelu(1.0) - 0.8413447460685429) < 1e-15
    h = 1e-6
    num = (oracle.gelu(u + h) - oracle.gelu(u - h)) / (2 * h)
    np.testing.assert_allclose(oracle.gelu_grad(u), num, atol=1e-9)


# ---------------------------------------------------------------- library special case: T = 1 against PyTorch CPU autograd
@pytest.mark.parametrize("causal", [True, False])
def test_unsharded_layer_matches_pytorch_autograd(causal):
    import torch
    import torch.nn.functional as F
    g, x, d = tiny_problem(10, H=32, nh=4, dh=8, I=48, S=9, B=3)
    B, S, H, nh, dh = d["B"], d["S"], d["H"], d["nh"], d["dh"]
    ya, ym, sv = oracle.full_layer_fwd(x["x_a"], x["x_m"], g, B, S, causal)
    gr = oracle.full_layer_bwd(x["x_a"], x["x_m"], g, x["dy_a"], x["dy_m"], sv, B, S, causal)
    t = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in {**g, **x}.items()}
    # nn.Linear convention is weight [out, in]; ours is [in, out]
    qkv = F.linear(t["x_a"], t["Wqkv"].reshape(H, 3 * nh * dh).T, t["bqkv"].reshape(-1))
    qkv = qkv.reshape(B, S, 3, nh, dh).permute(2, 0, 3, 1, 4)
    o = F.scaled_dot_product_attention(qkv[0], qkv[1], qkv[2], is_causal=causal)
    o = o.permute(0, 2, 1, 3).reshape(B * S, nh * dh)
    y_a = F.linear(o, t["Wo"].T, t["bo"]) + t["x_a"]
    y_m = F.linear(F.gelu(F.linear(t["x_m"], t["Wup"].T, t["bup"])), t["Wdn"].T, t["bdn"]) + t["x_m"]
    ((y_a * t["dy_a"]).sum() + (y_m * t["dy_m"]).sum()).backward()
    np.testing.assert_allclose(ya, y_a.detach().numpy(), atol=1e-11)
    np.testing.assert_allclose(ym, y_m.detach().numpy(), atol=1e-11)
    pairs = [("dx_a", "x_a"), ("dx_m", "x_m"), ("dw_qkv", "Wqkv"), ("db_qkv", "bqkv"), ("dw_o", "Wo"),
             ("db_o", "bo"), ("dw_up", "Wup"), ("db_up", "bup"), ("dw_dn", "Wdn"), ("db_dn", "bdn")]
    for gk, tk in pairs:
        np.testing.assert_allclose(gr[gk].reshape(-1), t[tk].grad.numpy().reshape(-1), atol=1e-10, err_msg=gk)


def test_parity_metric():
    ref = np.array([0.0, 1.0, -4.0])
    assert oracle.max_rel_err(ref, ref) == 0.0
    assert abs(oracle.max_rel_err(ref + np.array([0.04, 0, 0]), ref) - 0.01) < 1e-15


# ---------------------------------------------------------------- the pins do catch planted mistakes
@pytest.mark.parametrize("mutation", ["gelu_grad_drops_term", "no_softmax_scale", "mask_excludes_diagonal",
                                      "dk_uses_k", "bias_on_every_rank"])
def test_pins_fail_on_planted_mistakes(monkeypatch, mutation):
    """Each mistake is planted in the oracle (CPU only) and at least one pin must fail."""
    if mutation == "gelu_grad_drops_term":
        monkeypatch.setattr(O, "gelu_grad", lambda u: 0.5 * (1.0 + O._erf(np.asarray(u) / np.sqrt(2.0))))
        victims = [lambda: test_gradients_match_central_differences(True, True)]
    elif mutation == "no_softmax_scale":
        orig = O._scores
        monkeypatch.setattr(O, "_scores", lambda Q, K, c: (orig(Q, K, c)[0] * np.sqrt(Q.shape[-1]), orig(Q, K, c)[1]))
        victims = [lambda: test_forward_matches_scalar_loops(True), test_scale_is_inverse_sqrt_head_dim]
    elif mutation == "mask_excludes_diagonal":
        orig = O._scores

        def bad(Q, K, c):
            sc, al = orig(Q, K, c)
            if c:
                al = np.tril(al, -1) | np.eye(al.shape[0], dtype=bool) * (np.arange(al.shape[0]) == 0)[:, None]
            return sc, al
        monkeypatch.setattr(O, "_scores", bad)
        victims = [lambda: test_forward_matches_scalar_loops(True)]
    elif mutation == "dk_uses_k":
        orig = O.attention_bwd

        def bad(Q, K, V, P, dO):
            dQ, dK, dV = orig(Q, K, V, P, dO)
            _, dK2, _ = orig(K, K, V, P, dO)
            return dQ, dK2, dV
        monkeypatch.setattr(O, "attention_bwd", bad)
        victims = [lambda: test_gradients_match_central_differences(False, False)]
    else:
        orig = O.layer_fwd
        monkeypatch.setattr(O, "layer_fwd", lambda xa, xm, p, B, S, nl, dh, c, e: orig(xa, xm, p, B, S, nl, dh, c, True))
        monkeypatch.setattr(oracle, "layer_fwd", O.layer_fwd)
        victims = [lambda: test_partials_sum_to_unsharded_layer(True, 2)]
    for v in victims:
        with pytest.raises(AssertionError):
            v()
