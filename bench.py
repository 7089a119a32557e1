#!/usr/bin/env python3
"""Benchmark: forward+backward of one tensor-parallel rank's layer shard on one MI355X.

A step is one tp_layer_fwd followed by one tp_layer_bwd on seeded synthetic tensors already resident
in HBM.  The default workload is the GPT-3-175B-shaped TP=8 shard (config 5).  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1..5|name] [--no-cpu-baseline]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

BF16_PEAK_TFLOPS = 2500.0     # MI355X dense bf16 MFMA (vendor figure, no sparsity)
F32_PEAK_TFLOPS = 157.3       # fp32 vector


def gemm_list(cfg):
    """The 12 GEMMs of a step: (name, trans_a, trans_b, M, N, K, operand keys) in launch order."""
    M, H, Hl, Il = cfg.tokens, cfg.hidden, cfg.local_attn, cfg.local_mlp
    return [
        ("qkv_fwd", 0, 0, M, 3 * Hl, H), ("out_fwd", 0, 0, M, H, Hl), ("up_fwd", 0, 0, M, Il, H),
        ("down_fwd", 0, 0, M, H, Il),
        ("down_dgrad", 0, 1, M, Il, H), ("down_wgrad", 1, 0, Il, H, M), ("up_wgrad", 1, 0, H, Il, M),
        ("up_dgrad", 0, 1, M, H, Il), ("out_dgrad", 0, 1, M, Hl, H), ("out_wgrad", 1, 0, Hl, H, M),
        ("qkv_wgrad", 1, 0, H, 3 * Hl, M), ("qkv_dgrad", 0, 1, M, H, 3 * Hl),
    ]


def bench_layernorm(args, cfg, dt, pkg, torch, synthetic):
    """Replicated LayerNorm (forward with residual add, then backward) on the config's [M, H] activation."""
    M, H = cfg.tokens, cfg.hidden
    es = 4 if cfg.dtype == "f32" else 2
    tdt = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
    mk = lambda seed, shape, sigma, mean=0.0: pkg.to_device(  # noqa: E731
        synthetic.quantize(synthetic.normal(seed, int(__import__("numpy").prod(shape)), sigma) + mean, cfg.dtype).reshape(shape), dt)
    a, b, dy = mk(1, (M, H), 1.0), mk(2, (M, H), 1.0), mk(3, (M, H), 1.0)
    gamma, beta = mk(4, (H,), 0.1, 1.0), mk(5, (H,), 0.1)
    z, y, dz = (torch.empty(M, H, dtype=tdt, device="cuda") for _ in range(3))
    dg, db = torch.empty_like(gamma), torch.empty_like(gamma)
    mean = torch.empty(M, dtype=torch.float32, device="cuda")
    rstd = torch.empty_like(mean)
    ws = torch.empty(pkg.tp_layer_ln_workspace_bytes(M, H), dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream()

    def fwd():
        pkg.tp_layer_ln_fwd(dt, M, H, a, b, gamma, beta, 1e-5, z, y, mean, rstd, stream=stream)

    def bwd():
        pkg.tp_layer_ln_bwd(dt, M, H, dy, z, mean, rstd, gamma, dz, dg, db, ws, stream=stream)

    def timed(fn, n):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(n):
            fn()
        e1.record(stream)
        e1.synchronize()
        return e0.elapsed_time(e1) / n
    for _ in range(args.warmup):
        fwd(); bwd()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(args.steps):
        fwd(); bwd()
    torch.cuda.synchronize()
    ms = 1e3 * (time.perf_counter() - t1) / args.steps
    fwd_ms, bwd_ms = timed(fwd, args.steps), timed(bwd, args.steps)
    fwd_bytes, bwd_bytes = 4.0 * M * H * es, 3.0 * M * H * es        # a, b -> z, y ; dy, z -> dz
    import oracle
    import numpy as np
    c0 = time.perf_counter()
    an, bn, gn, ben, dyn = (v.float().cpu().numpy() for v in (a, b, gamma, beta, dy))
    yr, zr, mr, rr = oracle.layernorm_fwd(an, bn, gn, ben, 1e-5)
    dzr, dgr, dbr = oracle.layernorm_bwd(dyn, zr, mr, rr, gn)
    cpu_s = time.perf_counter() - c0
    err = max(oracle.max_rel_err(y.float().cpu().numpy(), yr), oracle.max_rel_err(dz.float().cpu().numpy(), dzr),
              oracle.max_rel_err(dg.float().cpu().numpy(), dgr), oracle.max_rel_err(db.float().cpu().numpy(), dbr))
    gbs = (fwd_bytes + bwd_bytes) / (ms * 1e-3) / 1e9
    print(json.dumps({
        "metric": "GB/s of algorithmic HBM bytes, replicated LayerNorm fwd+bwd", "value": round(gbs, 1), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"LayerNorm on [M={M}, H={H}] of config {cfg.cfg_id}: {cfg.name}"},
        "roofline": {"kernel": "ln_fwd_kernel + ln_bwd_kernel", "bound": "hbm",
                     "achieved": round(gbs, 1), "peak": 8000.0, "unit": "GB/s", "frac": round(gbs / 8000.0, 4),
                     "traffic": None, "fwd": {"ms": round(fwd_ms, 4), "GBps": round(fwd_bytes / fwd_ms / 1e6, 1)},
                     "bwd": {"ms": round(bwd_ms, 4), "GBps": round(bwd_bytes / bwd_ms / 1e6, 1)}},
        "cpu_baseline": {"value": round((fwd_bytes + bwd_bytes) / cpu_s / 1e9, 2), "unit": "GB/s", "cores": os.cpu_count(),
                         "kind": "oracle", "sample": "full workload, one fwd+bwd pass", "seconds": round(cpu_s, 2)},
        "max_rel_err_vs_oracle": err}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="5")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-timing", action="store_true")
    ap.add_argument("--workload", default="layer", choices=["layer", "layer-checkpoint", "ln"],
                    help="layer: tp_layer_fwd + tp_layer_bwd (the headline metric); layer-checkpoint: tp_layer_fwd + "
                         "tp_layer_bwd_recompute; ln: replicated LayerNorm forward + backward on the config's [M, H]")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain 1 GiB device copy (reference point for rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs one tensor-parallel rank's shard on ONE GPU; "
              "--gpus above 1 is not supported (no collectives in this path)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import synthetic
    import paper_2111_05972_amd as pkg

    pkg.load_library()   # raises if the HIP library is missing: there is no fallback
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes": 1 << 30, "copies": 3}))
        return
    key = int(args.config) if args.config.isdigit() else args.config
    cfg = synthetic.get_config(key)
    dt = pkg.TPL_F32 if cfg.dtype == "f32" else pkg.TPL_BF16
    peak = F32_PEAK_TFLOPS if cfg.dtype == "f32" else BF16_PEAK_TFLOPS
    if args.workload == "ln":
        return bench_layernorm(args, cfg, dt, pkg, torch, synthetic)

    t0 = time.time()
    d = synthetic.make_inputs(cfg)
    host_sh = pkg.shard_params(d, cfg.tp_degree if cfg.global_params else 1,
                               cfg.tp_rank if cfg.global_params else 0)
    layer = pkg.TpLayer(cfg.hidden, cfg.heads, cfg.tp_degree, cfg.tp_rank, cfg.seq, cfg.micro_batch, dt,
                        cfg.causal, cfg.row_epilogue, cfg.head_dim, cfg.intermediate)
    p = {k: pkg.to_device(v, dt) for k, v in host_sh.items()}
    x = {k: pkg.to_device(d[k], dt) for k in ("x_a", "x_m", "dy_a", "dy_m")}
    y_a, y_m = layer.empty_outputs()
    dx_a, dx_m = layer.empty_outputs()
    grads = layer.empty_grads()
    stream = torch.cuda.current_stream()
    gen_s = time.time() - t0

    ckpt = args.workload == "layer-checkpoint"
    ws_ckpt = torch.empty(pkg.tp_layer_workspace_bytes_recompute(layer.desc), dtype=torch.uint8,
                          device="cuda") if ckpt else None

    def step():
        layer.forward(p, x["x_a"], x["x_m"], y_a, y_m, stream=stream)
        if ckpt:    # backward recomputes QKV, O, LSE, U, G from the block inputs instead of reading `saved`
            pkg.tp_layer_bwd_recompute(layer.desc, p, x["x_a"], x["x_m"], x["dy_a"], x["dy_m"], grads, dx_a, dx_m,
                                       ws_ckpt, stream=stream)
        else:
            layer.backward(p, x["x_a"], x["x_m"], x["dy_a"], x["dy_m"], grads, dx_a, dx_m, stream=stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t1
    ms_per_step = 1e3 * elapsed / args.steps
    f_fwd, f_bwd = cfg.flops()
    tflops = (f_fwd + f_bwd) / (ms_per_step * 1e-3) / 1e12

    # fwd / bwd split with events on the launch stream
    def timed(fn, n):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(n):
            fn()
        e1.record(stream)
        e1.synchronize()
        return e0.elapsed_time(e1) / n
    n_split = max(3, min(args.steps, 10))
    fwd_ms = timed(lambda: layer.forward(p, x["x_a"], x["x_m"], y_a, y_m, stream=stream), n_split)
    bwd_ms = timed(lambda: layer.backward(p, x["x_a"], x["x_m"], x["dy_a"], x["dy_m"], grads, dx_a, dx_m,
                                          stream=stream), n_split)

    # dominant kernel: the GEMM kernel.  Its 12 launches per step are timed inside real steps: the
    # library brackets each GEMM launch with HIP events on the launch stream (tp_layer_profile).
    roofline = None
    if not args.no_kernel_timing:
        names = [g[0] for g in gemm_list(cfg)]
        flops = {g[0]: 2.0 * g[3] * g[4] * g[5] for g in gemm_list(cfg)}
        shapes = {g[0]: {"M": g[3], "N": g[4], "K": g[5]} for g in gemm_list(cfg)}
        reps = max(3, min(args.steps, 10))
        pkg.tp_layer_profile(1)
        for _ in range(reps):
            step()
        torch.cuda.synchronize()
        ms = pkg.tp_layer_profile_read()
        pkg.tp_layer_profile(0)
        per_step = len(ms) // reps          # 12, or 14 with the recomputed QKV and up-projection GEMMs
        assert len(ms) == per_step * reps and per_step in (12, 14), len(ms)
        if per_step == 14:                  # launch order: 4 fwd, then recomputed qkv_fwd and up_fwd, then 8 bwd
            order = names[:4] + ["qkv_fwd", "up_fwd"] + names[4:]
        else:
            order = names
        per = {n: sum(ms[i] for i in range(len(ms)) if order[i % per_step] == n) / reps for n in names}
        if per_step == 14:
            for n in ("qkv_fwd", "up_fwd"):
                flops[n] *= 2
        tot_ms, tot_fl = sum(per.values()), sum(flops.values())
        achieved = tot_fl / (tot_ms * 1e-3) / 1e12
        traffic = None
        tpath = os.path.join(ROOT, "profiles", "traffic.json")
        if os.path.exists(tpath):
            try:
                traffic = json.load(open(tpath)).get(cfg.name, {}).get("bytes_per_launch")
            except Exception:
                traffic = None
        launches = {n: {**shapes[n], "ms": round(per[n], 4), "tflops": round(flops[n] / per[n] / 1e9, 1)} for n in names}
        roofline = {"kernel": "gemm_bf16_kernel (12 launches per step)" if cfg.dtype == "bf16" else "gemm_simple_kernel",
                    "bound": "mfma" if cfg.dtype == "bf16" else "alu",
                    "achieved": round(achieved, 2), "peak": peak, "unit": "TFLOP/s",
                    "frac": round(achieved / peak, 4), "traffic": traffic,
                    "flops_per_launch": tot_fl / 12, "avg_launch_ms": round(tot_ms / 12, 4),
                    "gemm_ms_per_step": round(tot_ms, 4), "launches": launches}

    cpu_baseline = None
    max_err = None
    if not args.no_cpu_baseline:
        import oracle
        try:
            from threadpoolctl import threadpool_info
            cores = max([i.get("num_threads", 1) for i in threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count()
        # bounded sample: the full workload if it is small enough, else the same widths on fewer tokens
        from synthetic.configs import small_variant
        scfg, sample = cfg, "full workload, one fwd+bwd pass"
        if sum(cfg.flops()) > 3.0e12:
            scfg = small_variant(cfg, seq=max(1, cfg.seq // 4))
            sample = f"same widths, seq {scfg.seq} (1/4 of the tokens), one fwd+bwd pass"
        if scfg is cfg:
            sd, ssh = d, host_sh
        else:
            sd = {k: (v[:scfg.tokens] if k in ("x_a", "x_m", "dy_a", "dy_m") else v) for k, v in d.items()}
            ssh = host_sh
        a = (scfg.micro_batch, scfg.seq, scfg.local_heads, scfg.head_dim, scfg.causal, scfg.row_epilogue)
        c0 = time.perf_counter()
        ya, ym, osv = oracle.layer_fwd(sd["x_a"], sd["x_m"], ssh, *a)
        ref = oracle.layer_bwd(sd["x_a"], sd["x_m"], ssh, sd["dy_a"], sd["dy_m"], osv, *a)
        cpu_s = time.perf_counter() - c0
        cpu_baseline = {"value": round(sum(scfg.flops()) / cpu_s / 1e12, 4), "unit": "TFLOP/s", "cores": int(cores),
                        "kind": "oracle", "sample": sample, "seconds": round(cpu_s, 2)}
        if scfg is cfg:
            ref.update(y_a=ya, y_m=ym)
            got = {"y_a": y_a, "y_m": y_m, "dx_a": dx_a, "dx_m": dx_m, **grads}
            step()
            torch.cuda.synchronize()
            max_err = max(oracle.max_rel_err(v.float().cpu().numpy(), ref[k]) for k, v in got.items() if k in ref)

    out = {
        "metric": "TFLOP/s (fwd+bwd) per TP-rank layer shard on 1 MI355X; % bf16 MFMA peak",
        "value": round(tflops, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "pct_of_peak": round(100.0 * tflops / peak, 2), "peak_tflops": peak,
        "fwd_ms": round(fwd_ms, 4), "bwd_ms": round(bwd_ms, 4),
        "config": {"workload": f"config {cfg.cfg_id}: {cfg.name}" + (" (activation-checkpoint backward)" if ckpt else ""), "hidden": cfg.hidden, "heads": cfg.heads,
                   "head_dim": cfg.head_dim, "tp_degree": cfg.tp_degree, "tp_rank": cfg.tp_rank, "seq": cfg.seq,
                   "micro_batch": cfg.micro_batch, "causal": cfg.causal, "row_epilogue": cfg.row_epilogue,
                   "model_tflop_per_step": round((f_fwd + f_bwd) / 1e12, 4),
                   "params": "shard generated directly" if not cfg.global_params else "sliced from unsharded"},
        "roofline": roofline, "cpu_baseline": cpu_baseline, "max_rel_err_vs_oracle": max_err,
        "input_gen_s": round(gen_s, 1),
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
