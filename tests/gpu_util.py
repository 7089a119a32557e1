"""Helpers for the GPU parity tests: run the HIP path on a config's seeded inputs, run the oracle."""
import numpy as np

import oracle
import synthetic

TOL = {"f32": 1e-4, "bf16": 2e-2}     # max|gpu - ref| / max|ref| per tensor (spec bounds)
OUT_KEYS = ("y_a", "y_m", "dx_a", "dx_m", "dw_qkv", "db_qkv", "dw_o", "db_o", "dw_up", "db_up", "dw_dn",
            "db_dn", "QKV", "O", "LSE", "U", "G")


def shard_inputs(cfg):
    """Seeded inputs and the ORACLE's shard of the parameters (the GPU side shards with the product's own rule)."""
    d = synthetic.make_inputs(cfg)
    if cfg.global_params:
        sh = oracle.shard_params(d, cfg.tp_degree, cfg.tp_rank)
    else:   # parameters were generated at shard shape: T=1 slicing only flattens them
        sh = oracle.shard_params(d, 1, 0)
    return d, sh


def product_shard(cfg, d):
    """The same shard cut by the product's sharding rule (paper_2111_05972_amd.shard_params)."""
    import paper_2111_05972_amd as pkg
    T, r = (cfg.tp_degree, cfg.tp_rank) if cfg.global_params else (1, 0)
    return {k: np.ascontiguousarray(v) for k, v in pkg.shard_params(d, T, r).items()}


def oracle_outputs(cfg, d, sh):
    a = (cfg.micro_batch, cfg.seq, cfg.local_heads, cfg.head_dim, cfg.causal, cfg.row_epilogue)
    ya, ym, sv = oracle.layer_fwd(d["x_a"], d["x_m"], sh, *a)
    ref = oracle.layer_bwd(d["x_a"], d["x_m"], sh, d["dy_a"], d["dy_m"], sv, *a)
    ref.update(y_a=ya, y_m=ym, QKV=sv["QKV"], O=sv["O"], LSE=sv["LSE"], U=sv["U"], G=sv["G"])
    return ref


def gpu_outputs(cfg, d, sh=None, repeat=1, side_stream=False):
    """Runs the HIP path.  The parameters are sharded by the product's own rule; `sh` (the oracle's shard) is
    accepted for the callers' convenience and not used on this side.  side_stream: the two-chain schedule
    (TPL_SIDE_STREAM), which is what bench.py times."""
    import torch
    import paper_2111_05972_amd as pkg
    sh = product_shard(cfg, d)
    dt = pkg.TPL_F32 if cfg.dtype == "f32" else pkg.TPL_BF16
    layer = pkg.TpLayer(cfg.hidden, cfg.heads, cfg.tp_degree, cfg.tp_rank, cfg.seq, cfg.micro_batch, dt,
                        cfg.causal, cfg.row_epilogue, cfg.head_dim, cfg.intermediate, side_stream=side_stream)
    p = {k: pkg.to_device(v, dt) for k, v in sh.items()}
    x = {k: pkg.to_device(d[k], dt) for k in ("x_a", "x_m", "dy_a", "dy_m")}
    runs = []
    for _ in range(repeat):
        y_a, y_m = layer.forward(p, x["x_a"], x["x_m"])
        grads, dx_a, dx_m = layer.backward(p, x["x_a"], x["x_m"], x["dy_a"], x["dy_m"])
        torch.cuda.synchronize()
        got = {"y_a": y_a, "y_m": y_m, "dx_a": dx_a, "dx_m": dx_m, **grads, **layer.saved_tensors()}
        if not cfg.row_epilogue:
            got.pop("db_o"), got.pop("db_dn")
        runs.append({k: v.float().cpu().numpy() for k, v in got.items()})
    return runs if repeat > 1 else runs[0]


def rms_rel_err(got, ref):
    """Root-mean-square error relative to the root-mean-square of the reference (reported beside the bound)."""
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    den = np.sqrt(np.mean(ref * ref))
    num = np.sqrt(np.mean((got - ref) ** 2)) if got.size else 0.0
    return float(num / den) if den > 0 else float(num)


def compare(cfg, got, ref, tol=None, report=True):
    tol = TOL[cfg.dtype] if tol is None else tol
    errs = {}
    for k in OUT_KEYS:
        if k not in got:
            assert k in ("db_o", "db_dn") and not cfg.row_epilogue, k
            continue
        assert got[k].shape == np.shape(ref[k]), (k, got[k].shape, np.shape(ref[k]))
        assert np.isfinite(got[k]).all(), k
        errs[k] = oracle.max_rel_err(got[k], ref[k])
    if report:      # max-normalised (the bound) and RMS-relative error per tensor
        print(f"[parity] {cfg.name}: " + " ".join(
            f"{k}={errs[k]:.1e}/{rms_rel_err(got[k], ref[k]):.1e}" for k in errs), flush=True)
    bad = {k: e for k, e in errs.items() if not e <= tol}
    assert not bad, f"{cfg.name}: over tolerance {tol}: {bad} (all: {errs})"
    return errs
