"""The replicated LayerNorm composed with the shard (Sec. I.1: layer normalisation is not distributed in the
speed-optimised mode; Sec. I.4: `pre_layernorm` / `post_layernorm`): x_attn and x_mlp of the shard come from real
LayerNorm outputs and the backward pass runs through both normalisations.

One composition function drives two backends in the same order: the HIP path (tp_layer_ln_fwd / tp_layer_fwd /
tp_layer_bwd / tp_layer_ln_bwd, all T ranks on the one GPU) and the oracle (float64, nothing rounded).  What the
tensor-parallel group would all-reduce is summed over the ranks by the test (float sum, one rounding to the
storage type on the GPU side).  Because the boundary takes the MLP block's input from the caller, a pass over a
layer calls the shard twice (attention block first, then again once x_mlp is known; the second call recomputes the
attention block, whose outputs are simply not used again).

post-LN (the paper's default): x_a = h;           Ya = sum_r y_a;  x_m = LN1(Ya);      Ym = sum_r y_m;  out = LN2(Ym)
                               (rank 0 adds b_o + x_a and b_dn + x_m: TPL_ROW_EPILOGUE)
pre-LN:                        x_a = LN1(h);      z2 = h + sum_r y_a;  x_m = LN2(z2);  z3 = z2 + sum_r y_m;  out = LN3(z3)
                               (the residual stream is the un-normalised input, added by the next normalisation's
                               fused a + b; the flagged epilogue adds the block's own input, so it stays off and the
                               row-parallel biases are not part of this composition)
"""
import numpy as np
import pytest

import oracle
import synthetic
from synthetic.configs import small_variant

from gpu_util import TOL, rms_rel_err

pytestmark = pytest.mark.gpu
EPS = 1e-5


def _draw(seed, shape, sigma, dtype, mean=0.0):
    n = int(np.prod(shape))
    return synthetic.quantize(synthetic.normal(seed, n, sigma) + np.float32(mean), dtype).reshape(shape)


def compose(be, cfg, pre_ln, h, dout, ln):
    """Forward and backward of one layer through backend `be`; returns a dict of outputs and gradients."""
    T = cfg.tp_degree
    R = range(T)
    flag = [(not pre_ln) and r == 0 for r in R]
    res = {}
    if not pre_ln:
        ya = be.allreduce([be.shard_fwd(r, flag[r], h, None)[0] for r in R])
        x_m, n1 = be.ln_fwd(ya, None, ln["g1"], ln["b1"])
        ym = be.allreduce([be.shard_fwd(r, flag[r], h, x_m)[1] for r in R])
        out, n2 = be.ln_fwd(ym, None, ln["g2"], ln["b2"])
        res["out"] = out
        dym, res["dg2"], res["db2"] = be.ln_bwd(dout, n2, ln["g2"])
        part = [be.shard_bwd(r, flag[r], h, x_m, None, dym) for r in R]
        dxm = be.allreduce([p["dx_m"] for p in part])
        dya, res["dg1"], res["db1"] = be.ln_bwd(dxm, n1, ln["g1"])
        part = [be.shard_bwd(r, flag[r], h, x_m, dya, dym) for r in R]
        res["dh"] = be.allreduce([p["dx_a"] for p in part])
    else:
        x_a, n1 = be.ln_fwd(h, None, ln["g1"], ln["b1"])
        ya = be.allreduce([be.shard_fwd(r, False, x_a, None)[0] for r in R])
        x_m, n2 = be.ln_fwd(ya, h, ln["g2"], ln["b2"])                     # z2 = h + Ya inside
        ym = be.allreduce([be.shard_fwd(r, False, x_a, x_m)[1] for r in R])
        out, n3 = be.ln_fwd(ym, n2["z"], ln["g3"], ln["b3"])               # z3 = z2 + Ym inside
        res["out"], res["z3"] = out, n3["z"]
        dz3, res["dg3"], res["db3"] = be.ln_bwd(dout, n3, ln["g3"])
        part = [be.shard_bwd(r, False, x_a, x_m, None, dz3) for r in R]
        dxm = be.allreduce([p["dx_m"] for p in part])
        dz2_ln, res["dg2"], res["db2"] = be.ln_bwd(dxm, n2, ln["g2"])
        dz2 = be.allreduce([dz3, dz2_ln])                                  # both branches into z2
        part = [be.shard_bwd(r, False, x_a, x_m, dz2, dz3) for r in R]
        dxa = be.allreduce([p["dx_a"] for p in part])
        dh_ln, res["dg1"], res["db1"] = be.ln_bwd(dxa, n1, ln["g1"])
        res["dh"] = be.allreduce([dz2, dh_ln])
    for r in R:
        for k, v in part[r].items():
            if k.startswith("dw_") or k in ("db_qkv", "db_up") or (flag[r] and k in ("db_o", "db_dn")):
                res[f"r{r}.{k}"] = v
    return res


class OracleBackend:
    def __init__(self, cfg, g):
        self.cfg, self.g = cfg, g
        self.sh = [oracle.shard_params(g, cfg.tp_degree, r) for r in range(cfg.tp_degree)]
        self.saved = [None] * cfg.tp_degree

    def _a(self, flag):
        c = self.cfg
        return (c.micro_batch, c.seq, c.local_heads, c.head_dim, c.causal, flag)

    def allreduce(self, parts):
        return sum(np.asarray(p, np.float64) for p in parts)

    def ln_fwd(self, a, b, gamma, beta):
        y, z, mean, rstd = oracle.layernorm_fwd(a, b, gamma, beta, EPS)
        return y, {"z": z, "mean": mean, "rstd": rstd}

    def ln_bwd(self, dy, n, gamma):
        return oracle.layernorm_bwd(dy, n["z"], n["mean"], n["rstd"], gamma)

    def shard_fwd(self, r, flag, x_a, x_m):
        x_m = np.zeros_like(x_a) if x_m is None else x_m
        ya, ym, self.saved[r] = oracle.layer_fwd(x_a, x_m, self.sh[r], *self._a(flag))
        return ya, ym

    def shard_bwd(self, r, flag, x_a, x_m, dy_a, dy_m):
        dy_a = np.zeros_like(x_a) if dy_a is None else dy_a
        return oracle.layer_bwd(x_a, x_m, self.sh[r], dy_a, dy_m, self.saved[r], *self._a(flag))


class GpuBackend:
    def __init__(self, cfg, g, pkg, torch):
        self.cfg, self.pkg, self.torch = cfg, pkg, torch
        self.dt = pkg.TPL_F32 if cfg.dtype == "f32" else pkg.TPL_BF16
        T = cfg.tp_degree
        self.p = [{k: pkg.to_device(np.ascontiguousarray(v), self.dt) for k, v in pkg.shard_params(g, T, r).items()}
                  for r in range(T)]
        self.layers = {}
        self.st = torch.cuda.current_stream()
        self.ws = torch.empty(pkg.tp_layer_ln_workspace_bytes(cfg.tokens, cfg.hidden), dtype=torch.uint8, device="cuda")

    def dev(self, v):
        return self.pkg.to_device(v, self.dt)

    def _layer(self, r, flag):
        c, pkg = self.cfg, self.pkg
        if (r, flag) not in self.layers:
            self.layers[(r, flag)] = pkg.TpLayer(c.hidden, c.heads, c.tp_degree, r, c.seq, c.micro_batch, self.dt,
                                                 c.causal, flag, c.head_dim, c.intermediate)
        return self.layers[(r, flag)]

    def allreduce(self, parts):
        tot = self.torch.stack([p.float() for p in parts]).sum(0)
        return tot.to(parts[0].dtype)

    def ln_fwd(self, a, b, gamma, beta):
        torch, pkg, c = self.torch, self.pkg, self.cfg
        M, H = c.tokens, c.hidden
        y = torch.empty_like(a)
        z = torch.empty_like(a) if b is not None else None
        mean = torch.empty(M, dtype=torch.float32, device="cuda")
        rstd = torch.empty_like(mean)
        pkg.tp_layer_ln_fwd(self.dt, M, H, a, b, gamma, beta, EPS, z, y, mean, rstd, stream=self.st)
        return y, {"z": z if b is not None else a, "mean": mean, "rstd": rstd}

    def ln_bwd(self, dy, n, gamma):
        torch, pkg, c = self.torch, self.pkg, self.cfg
        dz = torch.empty_like(dy)
        dg, db = torch.empty_like(gamma), torch.empty_like(gamma)
        pkg.tp_layer_ln_bwd(self.dt, c.tokens, c.hidden, dy, n["z"], n["mean"], n["rstd"], gamma, dz, dg, db, self.ws,
                            stream=self.st)
        return dz, dg, db

    def shard_fwd(self, r, flag, x_a, x_m):
        x_m = self.torch.zeros_like(x_a) if x_m is None else x_m
        return self._layer(r, flag).forward(self.p[r], x_a, x_m, stream=self.st)

    def shard_bwd(self, r, flag, x_a, x_m, dy_a, dy_m):
        dy_a = self.torch.zeros_like(x_a) if dy_a is None else dy_a
        grads, dx_a, dx_m = self._layer(r, flag).backward(self.p[r], x_a, x_m, dy_a, dy_m, stream=self.st)
        return {"dx_a": dx_a, "dx_m": dx_m, **grads}


CASES = [
    ("post-bf16-T2", small_variant(synthetic.CONFIGS[3], name="ln-post-bf16", hidden=512, heads=8, intermediate=2048,
                                   tp_degree=2, tp_rank=0, seq=192, micro_batch=2, causal=True), False),
    ("pre-bf16-T2", small_variant(synthetic.CONFIGS[3], name="ln-pre-bf16", hidden=512, heads=8, intermediate=2048,
                                  tp_degree=2, tp_rank=0, seq=192, micro_batch=2, causal=True), True),
    ("post-bf16-T1-dh128", small_variant(synthetic.CONFIGS[3], name="ln-post-T1", hidden=1024, heads=8, head_dim=128,
                                         intermediate=4096, tp_degree=1, tp_rank=0, seq=320, micro_batch=1,
                                         causal=False), False),
    ("post-f32-T2", small_variant(synthetic.CONFIGS[1], name="ln-post-f32", hidden=256, heads=4, intermediate=1024,
                                  tp_degree=2, tp_rank=0, seq=96, micro_batch=2, causal=True), False),
    ("pre-f32-T2", small_variant(synthetic.CONFIGS[1], name="ln-pre-f32", hidden=256, heads=4, intermediate=1024,
                                 tp_degree=2, tp_rank=0, seq=96, micro_batch=2, causal=True, sigma_x=1.0), True),
]


@pytest.mark.parametrize("name,cfg,pre_ln", CASES, ids=[c[0] for c in CASES])
def test_layernorm_composed_with_the_shard(name, cfg, pre_ln):
    import torch
    import paper_2111_05972_amd as pkg
    print(f"\n[ln-compose] {name} pre_ln={pre_ln}", flush=True)
    g = synthetic.make_inputs(cfg)                       # unsharded parameters; x_a is the layer input h
    M, H, dtype = cfg.tokens, cfg.hidden, cfg.dtype
    h, dout = g["x_a"], g["dy_a"]
    ln = {}
    for i in (1, 2, 3):
        ln[f"g{i}"] = _draw(700 + i, (H,), 0.2, dtype, mean=1.0)
        ln[f"b{i}"] = _draw(710 + i, (H,), 0.2, dtype)
    ref = compose(OracleBackend(cfg, g), cfg, pre_ln, h, dout, ln)
    be = GpuBackend(cfg, g, pkg, torch)
    got = compose(be, cfg, pre_ln, be.dev(h), be.dev(dout), {k: be.dev(v) for k, v in ln.items()})
    torch.cuda.synchronize()
    assert set(got) == set(ref)
    tol = TOL[dtype]
    errs = {k: oracle.max_rel_err(got[k].float().cpu().numpy(), ref[k]) for k in ref}
    print("[ln-compose] max-normalised / rms-relative: " + " ".join(
        f"{k}={errs[k]:.1e}/{rms_rel_err(got[k].float().cpu().numpy(), ref[k]):.1e}" for k in ref), flush=True)
    bad = {k: e for k, e in errs.items() if not e <= tol}
    assert not bad, f"{name}: over tolerance {tol}: {bad}"
