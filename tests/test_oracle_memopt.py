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
