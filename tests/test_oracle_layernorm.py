"""Pins for the oracle's LayerNorm (the replicated normalisation either side of the shard)."""
import numpy as np
import pytest

import oracle


def _data(seed=0, M=5, H=12):
    rng = np.random.default_rng(seed)
    return (rng.normal(1.0, 2.0, (M, H)), rng.normal(0, 1, (M, H)), rng.normal(1, 0.3, H), rng.normal(0, 0.3, H),
            rng.normal(0, 1, (M, H)))


def test_rows_are_standardised_and_shift_invariant():
    a, b, gamma, beta, _ = _data()
    eps = 1e-5
    y, z, mean, rstd = oracle.layernorm_fwd(a, b, np.ones(12), np.zeros(12), eps)
    np.testing.assert_allclose(z, a + b)
    np.testing.assert_allclose(y.mean(1), 0.0, atol=1e-14)
    var = (a + b).var(axis=1)                       # biased variance
    np.testing.assert_allclose(y.var(axis=1), var / (var + eps), rtol=1e-12)
    np.testing.assert_allclose(mean, (a + b).mean(1))
    np.testing.assert_allclose(rstd, 1 / np.sqrt(var + eps))
    y2, *_ = oracle.layernorm_fwd(a + 7.5, b, np.ones(12), np.zeros(12), eps)   # adding a constant to a row
    np.testing.assert_allclose(y2, y, atol=1e-12)
    y3, *_ = oracle.layernorm_fwd(a, b, gamma, beta, eps)
    np.testing.assert_allclose(y3, y * gamma + beta, atol=1e-14)
    y4, z4, _, _ = oracle.layernorm_fwd(a, None, gamma, beta, eps)
    np.testing.assert_allclose(z4, a)


def test_two_element_closed_form():
    # a row (u, v): mean (u+v)/2, deviation +-d with d=(u-v)/2, var d^2 -> y = +-d / sqrt(d^2 + eps)
    y, *_ = oracle.layernorm_fwd(np.array([[3.0, 1.0]]), None, np.ones(2), np.zeros(2), 0.25)
    np.testing.assert_allclose(y, [[1 / np.sqrt(1.25), -1 / np.sqrt(1.25)]], atol=1e-15)


def test_matches_pytorch_layer_norm_and_autograd():
    import torch
    import torch.nn.functional as F
    a, b, gamma, beta, dy = _data(3, M=7, H=20)
    y, z, mean, rstd = oracle.layernorm_fwd(a, b, gamma, beta, 1e-5)
    dz, dg, db = oracle.layernorm_bwd(dy, z, mean, rstd, gamma)
    t = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in
         dict(a=a, b=b, gamma=gamma, beta=beta).items()}
    yt = F.layer_norm(t["a"] + t["b"], (20,), t["gamma"], t["beta"], 1e-5)
    (yt * torch.tensor(dy)).sum().backward()
    np.testing.assert_allclose(y, yt.detach().numpy(), atol=1e-12)
    np.testing.assert_allclose(dz, t["a"].grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(dz, t["b"].grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(dg, t["gamma"].grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(db, t["beta"].grad.numpy(), atol=1e-12)


def test_gradients_match_central_differences():
    a, b, gamma, beta, dy = _data(5, M=3, H=6)
    eps = 1e-3
    y, z, mean, rstd = oracle.layernorm_fwd(a, b, gamma, beta, eps)
    dz, dg, db = oracle.layernorm_bwd(dy, z, mean, rstd, gamma)
    loss = lambda aa, gg, bb: float((oracle.layernorm_fwd(aa, b, gg, bb, eps)[0] * dy).sum())  # noqa: E731
    h = 1e-6
    for (arr, grad, which) in [(a, dz, 0), (gamma, dg, 1), (beta, db, 2)]:
        flat = arr.reshape(-1)
        for i in range(flat.size):
            old = flat[i]
            flat[i] = old + h
            lp = loss(a, gamma, beta)
            flat[i] = old - h
            lm = loss(a, gamma, beta)
            flat[i] = old
            assert abs((lp - lm) / (2 * h) - grad.reshape(-1)[i]) < 1e-6, (which, i)


def test_planted_mistake_unbiased_variance_is_caught(monkeypatch):
    from oracle import tp_layer_oracle as O
    orig = O.layernorm_fwd

    def bad(a, b, gamma, beta, eps):
        y, z, mean, rstd = orig(a, b, gamma, beta, eps)
        H = z.shape[1]
        var = ((z - mean[:, None]) ** 2).sum(axis=1) / (H - 1)
        rstd = 1 / np.sqrt(var + eps)
        return (z - mean[:, None]) * rstd[:, None] * gamma + beta, z, mean, rstd
    monkeypatch.setattr(oracle, "layernorm_fwd", bad)
    with pytest.raises(AssertionError):
        test_matches_pytorch_layer_norm_and_autograd()


# ---------------------------------------------------------------- the LayerNorm + shard composition used by the GPU test
@pytest.mark.parametrize("pre_ln", [False, True])
def test_composed_layer_backward_matches_finite_differences(pre_ln):
    """tests/test_gpu_ln_compose.py chains LayerNorm and the shard's two blocks by hand (two shard calls per pass);
    here the same chain, run on the oracle, is checked against central differences of its own forward."""
    import synthetic
    from synthetic.configs import small_variant
    from test_gpu_ln_compose import OracleBackend, compose
    cfg = small_variant(synthetic.CONFIGS[1], name="ln-compose-tiny", hidden=16, heads=2, head_dim=8, intermediate=32,
                        tp_degree=2, tp_rank=0, seq=4, micro_batch=2, causal=True, sigma_w=0.3, sigma_x=1.0)
    g = {k: v.astype(np.float64) for k, v in synthetic.make_inputs(cfg).items()}
    rng = np.random.default_rng(5)
    H = cfg.hidden
    ln = {f"{n}{i}": rng.normal(1.0 if n == "g" else 0.0, 0.3, H) for n in "gb" for i in (1, 2, 3)}
    h, dout = g["x_a"], g["dy_a"]

    def loss(h_=h, ln_=ln, g_=g):
        return float((compose(OracleBackend(cfg, g_), cfg, pre_ln, h_, dout, ln_)["out"] * dout).sum())

    res = compose(OracleBackend(cfg, g), cfg, pre_ln, h, dout, ln)
    eps = 1e-6

    def fd(arr, setter):
        out = np.zeros_like(arr)
        for idx in np.ndindex(arr.shape):
            p, m = arr.copy(), arr.copy()
            p[idx] += eps
            m[idx] -= eps
            out[idx] = (setter(p) - setter(m)) / (2 * eps)
        return out

    np.testing.assert_allclose(res["dh"], fd(h, lambda v: loss(h_=v)), rtol=2e-5, atol=1e-7)
    for k in ("g1", "b1", "g2", "b2"):
        np.testing.assert_allclose(res["d" + k], fd(ln[k], lambda v: loss(ln_={**ln, k: v})), rtol=2e-5, atol=1e-7)
    # a weight gradient of each block, rank 1's shard: rows / columns r of the unsharded matrices
    nl, dh, Il = cfg.local_heads, cfg.head_dim, cfg.local_mlp
    gWo = fd(g["Wo"], lambda v: loss(g_={**g, "Wo": v}))
    np.testing.assert_allclose(res["r1.dw_o"], gWo[nl * dh:2 * nl * dh], rtol=2e-5, atol=1e-7)
    gWup = fd(g["Wup"], lambda v: loss(g_={**g, "Wup": v}))
    np.testing.assert_allclose(res["r1.dw_up"], gWup[:, Il:2 * Il], rtol=2e-5, atol=1e-7)
