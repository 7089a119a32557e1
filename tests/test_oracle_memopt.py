"""Pins for the oracle of the memory-optimised distribution's local compute (App. F.2 of the paper)."""
import numpy as np
import pytest

from oracle import memopt_oracle as mo


def _slices(a, T):
    w = a.shape[1] // T
    return [a[:, r * w:(r + 1) * w] for r in range(T)]


def test_moments_and_apply_equal_textbook_layer_norm():
    rng = np.random.default_rng(0)
    M, H, T, eps = 7, 24, 4, 1e-5
    x = rng.normal(0.7, 1.9, (M, H))
    gamma, beta = rng.normal(1, 0.3, H), rng.normal(0, 0.3, H)
    xs, gs, bs = _slices(x, T), _slices(gamma[None], T), _slices(beta[None], T)
    tot = mo.all_reduce([mo.ln_local_moments(v) for v in xs])
    np.testing.assert_allclose(tot[:, 0], x.sum(1))
    np.testing.assert_allclose(tot[:, 1], (x * x).sum(1))
    mean, rstd = mo.ln_stats(tot, H, eps)
    np.testing.assert_allclose(mean, x.mean(1), rtol=1e-13)
    np.testing.assert_allclose(rstd, 1 / np.sqrt(x.var(1) + eps), rtol=1e-12)      # biased variance
    y = np.concatenate([mo.ln_apply_fwd(xs[r], mean, rstd, gs[r][0], bs[r][0]) for r in range(T)], axis=1)
    ref = (x - x.mean(1, keepdims=True)) / np.sqrt(x.var(1, keepdims=True) + eps) * gamma + beta
    np.testing.assert_allclose(y, ref, atol=1e-12)
    import torch
    import torch.nn.functional as F
    yt = F.layer_norm(torch.tensor(x), (H,), torch.tensor(gamma), torch.tensor(beta), eps).numpy()
    np.testing.assert_allclose(y, yt, atol=1e-12)


def test_sliced_backward_equals_finite_differences_of_full_row_normalisation():
    rng = np.random.default_rng(1)
    M, H, T, eps, h = 3, 12, 3, 1e-3, 1e-6
    x = rng.normal(0.2, 1.3, (M, H))
    gamma, beta = rng.normal(1, 0.3, H), rng.normal(0, 0.3, H)
    dy = rng.normal(0, 1, (M, H))

    def loss(x_, g_, b_):
        y = (x_ - x_.mean(1, keepdims=True)) / np.sqrt(x_.var(1, keepdims=True) + eps) * g_ + b_
        return (y * dy).sum()

    def fd(arr, f):
        out = np.zeros_like(arr)
        for idx in np.ndindex(arr.shape):
            p, m = arr.copy(), arr.copy()
            p[idx] += h
            m[idx] -= h
            out[idx] = (f(p) - f(m)) / (2 * h)
        return out

    tot_m = mo.all_reduce([mo.ln_local_moments(v) for v in _slices(x, T)])
    mean, rstd = mo.ln_stats(tot_m, H, eps)
    xs, dys, gs = _slices(x, T), _slices(dy, T), _slices(gamma[None], T)
    sums = [mo.ln_apply_bwd_sums(dys[r], xs[r], mean, rstd, gs[r][0]) for r in range(T)]
    tot = mo.all_reduce(sums)
    res = [mo.ln_apply_bwd(dys[r], xs[r], mean, rstd, gs[r][0], tot, H) for r in range(T)]
    dx = np.concatenate([v[0] for v in res], axis=1)
    dgam = np.concatenate([v[1] for v in res])
    dbet = np.concatenate([v[2] for v in res])
    np.testing.assert_allclose(dx, fd(x, lambda v: loss(v, gamma, beta)), rtol=1e-6, atol=1e-8)
    np.testing.assert_allclose(dgam, fd(gamma, lambda v: loss(x, v, beta)), rtol=1e-6, atol=1e-8)
    np.testing.assert_allclose(dbet, fd(beta, lambda v: loss(x, gamma, v)), rtol=1e-6, atol=1e-8)
    # a rank that forgets the other ranks' share of the sums gets a different dx
    wrong, _, _ = mo.ln_apply_bwd(dys[0], xs[0], mean, rstd, gs[0][0], sums[0], H)
    assert np.abs(wrong - dx[:, :H // T]).max() > 1e-3


def test_bias_gelu_closed_forms_and_derivative():
    u = np.linspace(-4, 4, 41)
    _, g = mo.bias_gelu_fwd(u[None], np.zeros(41))
    _, gm = mo.bias_gelu_fwd(-u[None], np.zeros(41))
    np.testing.assert_allclose(g - gm, u[None], atol=1e-14)                 # gelu(u) - gelu(-u) = u
    assert mo.gelu(0.0) == 0.0 and mo.gelu_grad(0.0) == 0.5
    np.testing.assert_allclose(mo.gelu(np.array([8.0, -8.0])), [8.0, 0.0], atol=1e-13)
    h = 1e-6
    np.testing.assert_allclose(mo.gelu_grad(u), (mo.gelu(u + h) - mo.gelu(u - h)) / (2 * h), atol=1e-8)
    uu, gg = mo.bias_gelu_fwd(np.array([[1.0, 2.0]]), np.array([0.5, -2.0]))
    np.testing.assert_allclose(uu, [[1.5, 0.0]])
    du, db = mo.bias_gelu_bwd(np.array([[2.0, 3.0], [1.0, 1.0]]), np.array([[0.0, 0.0], [0.0, 0.0]]))
    np.testing.assert_allclose(du, [[1.0, 1.5], [0.5, 0.5]])
    np.testing.assert_allclose(db, [1.5, 2.0])


def test_input_split_linear_partials_add_up():
    rng = np.random.default_rng(2)
    M, K, N, T = 5, 12, 8, 3
    x, w, dy = rng.normal(size=(M, K)), rng.normal(size=(K, N)), rng.normal(size=(M, N))
    xs = _slices(x, T)
    ws = [w[r * (K // T):(r + 1) * (K // T)] for r in range(T)]
    parts = [mo.linear_part_fwd(xs[r], ws[r]) for r in range(T)]
    full = x @ w
    np.testing.assert_allclose(mo.all_reduce(parts), full, atol=1e-12)
    for r in range(2):                                             # any number of equal output slices
        np.testing.assert_allclose(mo.reduce_scatter(parts, r, 2), full[:, r * 4:(r + 1) * 4], atol=1e-12)
    for r in range(T):
        dx, dw = mo.linear_part_bwd(xs[r], ws[r], dy)
        np.testing.assert_allclose(dx, (dy @ w.T)[:, r * (K // T):(r + 1) * (K // T)], atol=1e-12)
        np.testing.assert_allclose(dw, (x.T @ dy)[r * (K // T):(r + 1) * (K // T)], atol=1e-12)


def _tiny(seed, H=16, nh=4, I=32, B=2, S=3):
    rng = np.random.default_rng(seed)
    g = {"nh": nh,
         "Wqkv": rng.normal(0, 0.3, (H, 3 * H)), "bqkv": rng.normal(0, 0.3, 3 * H),
         "Wo": rng.normal(0, 0.3, (H, H)), "bo": rng.normal(0, 0.3, H),
         "Wup": rng.normal(0, 0.3, (H, I)), "bup": rng.normal(0, 0.3, I),
         "Wdn": rng.normal(0, 0.3, (I, H)), "bdn": rng.normal(0, 0.3, H),
         "g1": rng.normal(1, 0.2, H), "b1": rng.normal(0, 0.2, H),
         "g2": rng.normal(1, 0.2, H), "b2": rng.normal(0, 0.2, H)}
    x = rng.normal(0, 1, (B * S, H))
    dy = rng.normal(0, 1, (B * S, H))
    return g, x, dy


@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("T", [1, 2, 4])
def test_simulated_ranks_equal_unsharded_layer(T, causal):
    g, x, _ = _tiny(3)
    B, S, eps = 2, 3, 1e-5
    H, nh = x.shape[1], g["nh"]
    shards = [mo.shard_reference_params(g, T, r) for r in range(T)]
    y, _ = mo.memopt_layer_fwd(_slices(x, T), shards, B, S, nh // T, H // nh, causal, eps)
    ref = mo.reference_layer_fwd(x, g, B, S, causal, eps)
    np.testing.assert_allclose(np.concatenate(y, axis=1), ref, atol=1e-12)


@pytest.mark.parametrize("causal", [True, False])
def test_simulated_ranks_backward_equals_finite_differences_of_unsharded_layer(causal):
    g, x, dy = _tiny(4)
    B, S, eps, T, h = 2, 3, 1e-5, 2, 1e-6
    H, nh = x.shape[1], g["nh"]
    dh, nl = H // nh, nh // T
    shards = [mo.shard_reference_params(g, T, r) for r in range(T)]
    y, sv = mo.memopt_layer_fwd(_slices(x, T), shards, B, S, nl, dh, causal, eps)
    dx, gr = mo.memopt_layer_bwd(_slices(dy, T), shards, sv, B, S, nl, dh)

    def loss(**kw):
        gg = dict(g)
        xx = kw.pop("x", x)
        gg.update(kw)
        return (mo.reference_layer_fwd(xx, gg, B, S, causal, eps) * dy).sum()

    def fd(name, arr):
        out = np.zeros_like(arr)
        for idx in np.ndindex(arr.shape):
            p, m = arr.copy(), arr.copy()
            p[idx] += h
            m[idx] -= h
            out[idx] = (loss(**{name: p}) - loss(**{name: m})) / (2 * h)
        return out

    np.testing.assert_allclose(np.concatenate(dx, axis=1), fd("x", x), rtol=2e-5, atol=1e-7)
    Hs, Il = H // T, g["Wup"].shape[1] // T
    perm = np.arange(3 * H).reshape(3, T, nl, dh).transpose(1, 0, 2, 3).reshape(-1)
    ref = {k: fd(k, g[k]) for k in ("Wqkv", "bqkv", "Wo", "bo", "Wup", "bup", "Wdn", "bdn", "g1", "b1", "g2", "b2")}
    for r in range(T):
        rows = slice(r * Hs, (r + 1) * Hs)
        tol = dict(rtol=2e-5, atol=1e-7)
        np.testing.assert_allclose(gr[r]["w_qkv"], ref["Wqkv"][rows][:, perm], **tol)
        np.testing.assert_allclose(gr[r]["b_qkv"], ref["bqkv"][perm][r * 3 * nl * dh:(r + 1) * 3 * nl * dh], **tol)
        np.testing.assert_allclose(gr[r]["w_o"], ref["Wo"][r * nl * dh:(r + 1) * nl * dh], **tol)
        np.testing.assert_allclose(gr[r]["b_o"], ref["bo"][rows], **tol)
        np.testing.assert_allclose(gr[r]["w_up"], ref["Wup"][rows], **tol)
        np.testing.assert_allclose(gr[r]["b_up"], ref["bup"][r * Il:(r + 1) * Il], **tol)
        np.testing.assert_allclose(gr[r]["w_dn"], ref["Wdn"][r * Il:(r + 1) * Il], **tol)
        np.testing.assert_allclose(gr[r]["b_dn"], ref["bdn"][rows], **tol)
        for k in ("g1", "b1", "g2", "b2"):
            np.testing.assert_allclose(gr[r][k], ref[k][rows], **tol)


# ---------------------------------------------------------------- pins of this module's own attention and
# unsharded reference layer against things outside it: the scalar definition, a hand-computed two-key case, the
# speed-optimised oracle's attention, and PyTorch's CPU operators with autograd.
def _qkv_case(seed, B=2, S=5, nl=3, dh=4):
    rng = np.random.default_rng(seed)
    return rng.normal(0, 1.0, (B * S, 3 * nl * dh)), rng.normal(0, 1.0, (B * S, nl * dh)), (B, S, nl, dh)


@pytest.mark.parametrize("causal", [True, False])
def test_attention_matches_scalar_definition(causal):
    """O[b,i,h,:] = sum_j softmax_j(q_i . k_j / sqrt(dh)) v_j with j <= i when causal, by plain loops."""
    import math
    qkv, _, (B, S, nl, dh) = _qkv_case(20)
    o, _ = mo._attention(qkv, B, S, nl, dh, causal)
    t = qkv.reshape(B, S, 3, nl, dh)
    for b in range(B):
        for h in range(nl):
            for i in range(S):
                js = range(i + 1) if causal else range(S)
                logit = [sum(t[b, i, 0, h, c] * t[b, j, 1, h, c] for c in range(dh)) / math.sqrt(dh) for j in js]
                mx = max(logit)
                w = [math.exp(v - mx) for v in logit]
                den = sum(w)
                for c in range(dh):
                    ref = sum(w[n] / den * t[b, j, 2, h, c] for n, j in enumerate(js))
                    assert abs(o[b * S + i, h * dh + c] - ref) < 1e-12


def test_attention_two_key_case_fixes_the_scale():
    """One head of size 4, two keys with q.k = 2 ln 3 and 0: the weights are (0.75, 0.25) only with 1/sqrt(dh)."""
    dh, S = 4, 2
    q = np.zeros((S, dh)); k = np.zeros((S, dh)); v = np.zeros((S, dh))
    q[:, 0] = 1.0
    k[0, 0] = 2.0 * np.log(3.0)                      # logits (ln 3, 0) after the division by sqrt(4) = 2
    v[0, 0], v[1, 0] = 1.0, 5.0
    qkv = np.concatenate([q, k, v], axis=1)
    o, (_, _, _, P) = mo._attention(qkv, 1, S, 1, dh, False)
    np.testing.assert_allclose(P[0, 0], [[0.75, 0.25], [0.75, 0.25]], atol=1e-14)
    np.testing.assert_allclose(o[:, 0], [2.0, 2.0], atol=1e-14)
    oc, (_, _, _, Pc) = mo._attention(qkv, 1, S, 1, dh, True)
    np.testing.assert_allclose(Pc[0, 0], [[1.0, 0.0], [0.75, 0.25]], atol=1e-14)     # key 1 hidden from query 0


@pytest.mark.parametrize("causal", [True, False])
def test_attention_and_its_backward_match_pytorch_and_the_other_oracle(causal):
    import torch
    import torch.nn.functional as F
    from oracle import tp_layer_oracle as so
    qkv, d_o, (B, S, nl, dh) = _qkv_case(21)
    o, saved = mo._attention(qkv, B, S, nl, dh, causal)
    dqkv = mo._attention_bwd(d_o, saved, B, S, nl, dh)
    tq = torch.tensor(qkv, dtype=torch.float64, requires_grad=True)
    t = tq.reshape(B, S, 3, nl, dh).permute(2, 0, 3, 1, 4)
    to = F.scaled_dot_product_attention(t[0], t[1], t[2], is_causal=causal).permute(0, 2, 1, 3).reshape(B * S, nl * dh)
    (to * torch.tensor(d_o)).sum().backward()
    np.testing.assert_allclose(o, to.detach().numpy(), atol=1e-12)
    np.testing.assert_allclose(dqkv, tq.grad.numpy(), atol=1e-12)
    Q, K, V = so._split_heads(qkv, B, S, nl, dh)
    O2, P2, _ = so.attention_fwd(Q, K, V, causal)
    np.testing.assert_allclose(o, O2.transpose(0, 2, 1, 3).reshape(B * S, nl * dh), atol=1e-13)
    np.testing.assert_allclose(saved[3], P2, atol=1e-14)


@pytest.mark.parametrize("causal", [True, False])
def test_reference_layer_matches_pytorch_pre_normalised_blocks(causal):
    """y1 = x + Attn(LN1(x)), y2 = y1 + MLP(LN2(y1)) written with PyTorch's CPU operators."""
    import torch
    import torch.nn.functional as F
    g, x, _ = _tiny(5, H=24, nh=4, I=40, B=2, S=6)
    B, S, eps = 2, 6, 1e-5
    H, nh = x.shape[1], g["nh"]
    dh = H // nh
    T_ = lambda a: torch.tensor(np.asarray(a), dtype=torch.float64)   # noqa: E731
    tx = T_(x)
    h1 = F.layer_norm(tx, (H,), T_(g["g1"]), T_(g["b1"]), eps)
    qkv = F.linear(h1, T_(g["Wqkv"]).T, T_(g["bqkv"])).reshape(B, S, 3, nh, dh).permute(2, 0, 3, 1, 4)
    o = F.scaled_dot_product_attention(qkv[0], qkv[1], qkv[2], is_causal=causal).permute(0, 2, 1, 3).reshape(B * S, H)
    y1 = tx + F.linear(o, T_(g["Wo"]).T, T_(g["bo"]))
    h2 = F.layer_norm(y1, (H,), T_(g["g2"]), T_(g["b2"]), eps)
    y2 = y1 + F.linear(F.gelu(F.linear(h2, T_(g["Wup"]).T, T_(g["bup"]))), T_(g["Wdn"]).T, T_(g["bdn"]))
    np.testing.assert_allclose(mo.reference_layer_fwd(x, g, B, S, causal, eps), y2.numpy(), atol=1e-11)


@pytest.mark.parametrize("mutation", ["no_softmax_scale", "mask_excludes_diagonal", "dk_uses_k", "post_norm_layer"])
def test_memopt_pins_fail_on_planted_mistakes(monkeypatch, mutation):
    """Each mistake is planted in this oracle (CPU only); at least one of the pins above must fail."""
    if mutation == "no_softmax_scale":
        orig = mo._attention
        monkeypatch.setattr(mo, "_attention", lambda q, B, S, nl, dh, c: orig(
            np.concatenate([q[:, :nl * dh] * np.sqrt(dh), q[:, nl * dh:]], axis=1), B, S, nl, dh, c))
        victims = [lambda: test_attention_matches_scalar_definition(True), test_attention_two_key_case_fixes_the_scale,
                   lambda: test_attention_and_its_backward_match_pytorch_and_the_other_oracle(False),
                   lambda: test_reference_layer_matches_pytorch_pre_normalised_blocks(True)]
    elif mutation == "mask_excludes_diagonal":
        real_tril = np.tril
        monkeypatch.setattr(mo.np, "tril", lambda a, k=0: real_tril(a, k - 1) | (real_tril(a, 0) & ~real_tril(a, -1) & (np.arange(a.shape[0]) == 0)[:, None]))
        victims = [lambda: test_attention_matches_scalar_definition(True), test_attention_two_key_case_fixes_the_scale]
    elif mutation == "dk_uses_k":
        orig = mo._attention_bwd

        def bad(dO, saved, B, S, nl, dh):
            Q, K, V, P = saved
            good = orig(dO, saved, B, S, nl, dh).reshape(B * S, 3, nl * dh)
            wrong = orig(dO, (K, K, V, P), B, S, nl, dh).reshape(B * S, 3, nl * dh)
            good[:, 1] = wrong[:, 1]
            return good.reshape(B * S, 3 * nl * dh)
        monkeypatch.setattr(mo, "_attention_bwd", bad)
        victims = [lambda: test_attention_and_its_backward_match_pytorch_and_the_other_oracle(True),
                   lambda: test_simulated_ranks_backward_equals_finite_differences_of_unsharded_layer(False)]
    else:
        orig = mo.reference_layer_fwd

        def post_norm(x, g, B, S, causal, eps):          # normalises after the residual sum instead of before the block
            gg = dict(g)
            H = np.asarray(x).shape[1]
            gg["g1"], gg["b1"] = np.ones(H), np.zeros(H)
            return orig(x, gg, B, S, causal, eps)
        monkeypatch.setattr(mo, "reference_layer_fwd", post_norm)
        victims = [lambda: test_reference_layer_matches_pytorch_pre_normalised_blocks(False),
                   lambda: test_simulated_ranks_equal_unsharded_layer(2, True)]
    for v in victims:
        with pytest.raises(AssertionError):
            v()
