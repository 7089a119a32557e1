"""The bf16 parity bound (2e-2 of a tensor's max) does its job: CPU emulations of the rounding the HIP path is
allowed to do pass it, and emulations of wrong variants fail it.

Everything here runs on the CPU with numpy.  "Got" tensors are produced by pushing the oracle's own definitions
through the rounding points of the bf16 path (stored tensors rounded to bf16, float accumulation), or through a
deliberately wrong variant of them; `gpu_util.compare` is the same function the GPU parity tests use.
"""
import numpy as np
import pytest

import oracle
import synthetic
from synthetic.configs import small_variant
from synthetic.gen import quantize

from gpu_util import compare, oracle_outputs, rms_rel_err, shard_inputs

# 2048 tokens as in the headline configuration: the weight gradients then sum over K = 2048 terms
CFG = small_variant(synthetic.CONFIGS[2], hidden=128, heads=2, intermediate=512, tp_degree=2, tp_rank=0,
                    seq=1024, micro_batch=2, causal=True, row_epilogue=True)


def _r(x):
    """One bf16 store."""
    return quantize(np.asarray(x, np.float32), "bf16").astype(np.float64)


def _gemm_f32(a, b):
    """bf16 operands, float accumulation, one rounding when stored."""
    return _r(np.asarray(a, np.float32) @ np.asarray(b, np.float32))


def _gemm_bf16_accumulate(a, b):
    """The wrong variant: a bf16 accumulator (the running sum is rounded to bf16 after every term)."""
    a, b = np.asarray(a, np.float32), np.asarray(b, np.float32)
    acc = np.zeros((a.shape[0], b.shape[1]), np.float32)
    for k in range(a.shape[1]):
        acc = quantize(acc + a[:, k:k + 1] * b[k:k + 1, :], "bf16")
    return acc.astype(np.float64)


def _emulate(cfg, d, sh, gemm=_gemm_f32, scale=None):
    """The shard with the rounding points of the bf16 path; `gemm` and the softmax `scale` can be made wrong."""
    B, S, nl, dh = cfg.micro_batch, cfg.seq, cfg.local_heads, cfg.head_dim
    M = B * S
    scale = 1.0 / np.sqrt(dh) if scale is None else scale
    x_a, x_m, dy_a, dy_m = (d[k].astype(np.float64) for k in ("x_a", "x_m", "dy_a", "dy_m"))
    w = {k: np.asarray(v, np.float64) for k, v in sh.items()}
    e = 1.0 if cfg.row_epilogue else 0.0
    out = {}
    qkv = _r(gemm(x_a, w["w_qkv"]) + w["b_qkv"]) if gemm is not _gemm_f32 else _r(x_a @ w["w_qkv"] + w["b_qkv"])
    Q, K, V = oracle.tp_layer_oracle._split_heads(qkv, B, S, nl, dh)
    sc = np.matmul(Q, K.transpose(0, 1, 3, 2)) * scale
    if cfg.causal:
        sc = np.where(np.tril(np.ones((S, S), bool)), sc, -np.inf)
    mx = sc.max(-1, keepdims=True)
    ex = np.exp(sc - mx)
    den = ex.sum(-1, keepdims=True)
    P = ex / den
    Oh = np.matmul(_r(P), V)                                        # probabilities are bf16 operands
    out["LSE"] = (mx + np.log(den))[..., 0]
    o = _r(Oh.transpose(0, 2, 1, 3).reshape(M, nl * dh))
    out["QKV"], out["O"] = qkv, o
    out["y_a"] = _r(gemm(o, w["w_o"]) + e * (w["b_o"] + x_a))
    u = _r(x_m @ w["w_up"] + w["b_up"])
    g = _r(oracle.gelu(u))
    out["U"], out["G"] = u, g
    out["y_m"] = _r(gemm(g, w["w_dn"]) + e * (w["b_dn"] + x_m))
    # backward from the stored (rounded) tensors
    du = _r((dy_m @ w["w_dn"].T) * oracle.gelu_grad(u))
    out["dw_dn"], out["dw_up"] = _r(gemm(g.T, dy_m)), _r(gemm(x_m.T, du))
    out["db_up"] = _r(du.sum(0))
    out["dx_m"] = _r(gemm(du, w["w_up"].T) + e * dy_m)
    d_o = _r(dy_a @ w["w_o"].T)
    out["dw_o"] = _r(gemm(o.T, dy_a))
    dOh = d_o.reshape(B, S, nl, dh).transpose(0, 2, 1, 3)
    dV = np.matmul(_r(P).transpose(0, 1, 3, 2), dOh)
    dP = np.matmul(dOh, V.transpose(0, 1, 3, 2))
    D = (dOh * Oh).sum(-1, keepdims=True)
    dS = _r(P * (dP - D))
    dQ, dK = np.matmul(dS, K) * scale, np.matmul(dS.transpose(0, 1, 3, 2), Q) * scale
    dqkv = _r(np.stack([a.transpose(0, 2, 1, 3) for a in (dQ, dK, dV)], axis=2).reshape(M, 3 * nl * dh))
    out["dw_qkv"], out["db_qkv"] = _r(gemm(x_a.T, dqkv)), _r(dqkv.sum(0))
    out["dx_a"] = _r(gemm(dqkv, w["w_qkv"].T) + e * dy_a)
    if cfg.row_epilogue:
        out["db_o"], out["db_dn"] = _r(dy_a.sum(0)), _r(dy_m.sum(0))
    return {k: np.asarray(v, np.float32) for k, v in out.items()}


@pytest.fixture(scope="module")
def problem():
    d, sh = shard_inputs(CFG)
    return d, sh, oracle_outputs(CFG, d, sh)


def test_faithful_bf16_rounding_is_inside_the_bound(problem):
    d, sh, ref = problem
    errs = compare(CFG, _emulate(CFG, d, sh), ref)
    assert max(errs.values()) < 1e-2            # the allowed roundings sit well inside 2e-2


def test_bf16_accumulation_fails_the_bound(problem):
    """Rounding the running sums of the GEMMs to bf16 (instead of float accumulation) must be caught."""
    d, sh, ref = problem
    with pytest.raises(AssertionError, match="over tolerance"):
        compare(CFG, _emulate(CFG, d, sh, gemm=_gemm_bf16_accumulate), ref)


def test_missing_softmax_scale_fails_the_bound(problem):
    d, sh, ref = problem
    with pytest.raises(AssertionError, match="over tolerance"):
        compare(CFG, _emulate(CFG, d, sh, scale=1.0), ref)


def test_rms_relative_error():
    ref = np.array([3.0, -4.0])
    assert rms_rel_err(ref, ref) == 0.0
    assert abs(rms_rel_err(ref + np.array([0.5, 0.5]), ref) - 0.5 / np.sqrt(12.5)) < 1e-15
